"""K-TanH (arXiv:1909.07729) for AMD MI355X: hand-written HIP kernels behind a C ABI.

``binding`` holds the Python front-end of the C-ABI library ``libktanh.so``;
``workloads`` holds the seeded synthetic inputs.  Importing the package loads
nothing native; the first call into ``binding`` does, and raises if the library
has not been built.
"""
