"""Reference oracle for K-TanH: test infrastructure, never imported by the GPU library."""
