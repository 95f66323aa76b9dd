// Internal to libktanh: the order in which the blocks of a streaming launch take their tiles.
// Plain C++ (no device headers) so that host tests can check it.
#pragma once

#ifdef __HIPCC__
#define KT_HOST_DEVICE __host__ __device__
#else
#define KT_HOST_DEVICE
#endif

namespace ktanh_device {

// Which tile a block takes.  Blocks are dispatched in index order, round-robin over the eight XCDs,
// so the tiles in flight at any moment form one window that moves through the tensor.  On large
// tensors two windows 128 or 256 MiB apart keep the memory busier than one: measured 0.8-2 % faster
// from 256 MiB of output upwards (windows closer than 64 MiB are slower by up to 9 %, and below
// 256 MiB nothing beats the plain order).  So a tensor is cut into segments of `1 << lg_seg` tiles
// (256 MiB; 512 MiB from 512 MiB of output on); inside each whole segment the blocks alternate, in
// groups of eight (one per XCD), between its two halves; what follows the last whole segment, and
// every tensor smaller than one segment, keeps the plain order.  A bijection on [0, tiles).
struct TileOrder {
    unsigned whole;   // tiles covered by whole segments (0 = plain order everywhere)
    unsigned lg_seg;  // log2 of the segment length in tiles
};

inline TileOrder tile_order_for(unsigned long long tiles)
{
    const unsigned lg = tiles >= (1ull << 19) ? 19u : 18u;
    return TileOrder{(unsigned)((tiles >> lg) << lg), lg};
}

KT_HOST_DEVICE inline unsigned tile_of_block(unsigned b, unsigned whole, unsigned lg_seg)
{
    if (b >= whole) return b;
    const unsigned mask = (1u << lg_seg) - 1u;
    const unsigned w = b & mask;
    return (b & ~mask) + (((w >> 3) & 1u) << (lg_seg - 1u)) + (((w >> 4) << 3) | (w & 7u));
}

}  // namespace ktanh_device
