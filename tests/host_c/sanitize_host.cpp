// Host-only sources of the library (table, validation, packing, fit) under AddressSanitizer and
// UndefinedBehaviorSanitizer: built and run by tests/test_boundary_host.py with g++, no GPU involved.
#include <cstdio>
#include <cstring>

#include <vector>

#include "ktanh_order.h"
#include "ktanh_pack.h"

int main()
{
    ktanh_lut_t fitted;
    ktanh_lut64_t fitted64;
    if (ktanh_fit_lut(&fitted) != KT_OK) return 1;
    if (std::memcmp(&fitted, ktanh_default_lut(), sizeof fitted) != 0) return 2;
    if (ktanh_fit_lut64(&fitted64) != KT_OK || ktanh_lut64_validate(&fitted64) != KT_OK) return 3;
    KtLutPack pack;
    if (kt_pack_lut_bf16(nullptr, &pack) != KT_OK || kt_pack_lut_f32(&fitted, &pack) != KT_OK) return 4;
    if (kt_pack_lut64_bf16(nullptr, &pack) != KT_OK || kt_pack_lut64_f32(&fitted64, &pack) != KT_OK) return 5;
    // every extreme a validated table may hold
    for (int t = 0; t < KTANH_INTERVALS; ++t) { fitted.E[t] = 254; fitted.r[t] = 7; fitted.b[t] = 127; }
    if (ktanh_lut_validate(&fitted) != KT_OK || kt_pack_lut_bf16(&fitted, &pack) != KT_OK) return 6;
    for (int t = 0; t < KTANH_INTERVALS; ++t) { fitted.E[t] = 1; fitted.r[t] = 0; fitted.b[t] = (int8_t)(-((t & 7) << 4)); }
    if (ktanh_lut_validate(&fitted) != KT_OK || kt_pack_lut_bf16(&fitted, &pack) != KT_OK) return 7;
    fitted.b[5] = -128;
    if (ktanh_lut_validate(&fitted) != KT_ERR_LUT) return 8;
    // the tile order is a bijection on [0, tiles) for sizes below, at and between whole segments
    for (unsigned long long tiles : {1ull, 7ull, 51200ull, (1ull << 18) - 1, 1ull << 18, (1ull << 18) + 5,
                                     307200ull, (1ull << 19) - 8, 1ull << 19, (1ull << 19) + 12345, 3ull << 18,
                                     1ull << 20, (1ull << 20) + (1ull << 18) + 3}) {
        const ktanh_device::TileOrder order = ktanh_device::tile_order_for(tiles);
        if (order.whole > tiles || (tiles >= (1ull << 18)) != (order.whole != 0)) return 9;
        std::vector<unsigned char> seen(tiles, 0);
        for (unsigned b = 0; b < tiles; ++b) {
            const unsigned t = ktanh_device::tile_of_block(b, order.whole, order.lg_seg);
            if (t >= tiles || seen[t]) return 10;
            seen[t] = 1;
        }
        if (ktanh_device::tile_of_block(0, order.whole, order.lg_seg) != 0) return 11;  // block 0 keeps the short first tile
    }
    std::puts("host sources clean");
    return 0;
}
