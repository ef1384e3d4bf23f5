// Internal declarations shared by the host dispatch code and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>

namespace convfwd {

// Everything a kernel needs; passed by value. All offsets are in floats and fit 32 bits
// (the host rejects tensors of 2^31 or more elements).
struct KernelArgs {
    const float* x;
    const float* w;
    float* y;
    int N, C, H, W, K, R, S, pad_h, pad_w;
    int P, Q, PQ, HW, CRS;
    int Hp;          // H + 2*pad_h: rows of one zero-padded image
    int total_pix;   // N*P*Q, output pixels in flattened (n,p,q) order
    // tiling (tap and pointwise families)
    int tile_pix;    // output pixels per work-group
    int ktiles;      // work-groups along K
    int ptiles;      // work-groups along the flattened pixels
    int chunk_c;     // channels per LDS round (multiple of 4)
    int nchunks;
    // LDS halo tile of the tap family
    int lds_rows, lds_pitch, lds_plane;
    int col_shift;   // LDS column of padded column 0 (keeps vector stores aligned)
    int w_pitch;     // floats per output channel in the LDS filter block
    int x_items;     // vector loads per chunk for the halo tile
    int w_items;     // vector loads per chunk for the filter block
};

// Tile shapes of the tap family. A work-group holds WK x WP x WC waves; a wave owns MT x NT MFMA
// tiles of 16 output channels x 16 pixels. The WC waves that share a tile position split the channel
// groups of every chunk between them and add their partial tiles through LDS at the end.
struct TapVariant {
    int MT, NT, WK, WP, WC;
    int occ;     // waves per SIMD the kernel is compiled for (bounds its registers)
    int xslots;  // halo-tile vector loads a thread may hold in flight
    int wslots;  // filter-block vector loads a thread may hold in flight
    bool dbuf;   // two copies of the LDS staging area (one barrier per chunk, stores hidden in the MAC loop)
    constexpr int tile_k() const { return 16 * MT * WK; }
    constexpr int max_pix() const { return 16 * NT * WP; }
    constexpr int block() const { return 64 * WK * WP * WC; }
    // LDS floats the cross-wave reduction needs (first round of the tree is the widest)
    constexpr int reduce_floats() const { return WC > 1 ? (WC / 2) * WK * WP * MT * NT * 256 : 0; }
    // LDS bytes a work-group may take so that as many work-groups as the registers allow share a CU
    constexpr int lds_limit() const { return 160 * 1024 / (occ * 256 / block() > 0 ? occ * 256 / block() : 1); }
};

constexpr TapVariant kTapVariants[] = {
    {1, 13, 4, 1, 1, 1, 8, 12, false},  // 0: 64 ch x 208 px, waves split K
    {1, 7, 4, 1, 1, 1, 8, 12, false},   // 1: 64 ch x 112 px, waves split K
    {1, 1, 1, 4, 1, 2, 6, 8, false},    // 2: 16 ch x  64 px, one MFMA tile per wave
    {2, 4, 2, 2, 1, 1, 8, 12, false},   // 3: 64 ch x 128 px, 2x4 tiles per wave
    {1, 2, 2, 2, 1, 2, 6, 8, false},    // 4: 32 ch x  64 px
    {1, 7, 4, 1, 1, 2, 6, 8, false},    // 5: 64 ch x 112 px, two work-groups per CU
    {4, 13, 1, 1, 4, 1, 7, 9, false},   // 6: 64 ch x 208 px (a 14x14 image), every wave owns the whole tile for 1/4 of the channels
    {4, 7, 1, 1, 4, 1, 8, 12, false},   // 7: 64 ch x 112 px, same scheme
    {2, 2, 1, 1, 4, 2, 4, 6, false},    // 8: 32 ch x  32 px, same scheme, for layers with few outputs
    {2, 13, 2, 1, 4, 2, 4, 5, true},    // 9: 64 ch x 208 px, 8 waves: 2 along K x 4 channel shares, two per SIMD
    {2, 7, 2, 1, 4, 2, 4, 6, true},     // 10: 64 ch x 112 px, same scheme
    {1, 13, 4, 1, 1, 1, 8, 12, true},   // 11: as 0 with double-buffered staging
    {1, 13, 4, 1, 2, 2, 4, 5, true},    // 12: 64 ch x 208 px, 8 waves: 4 along K x 2 channel shares, two per SIMD
    {1, 7, 4, 1, 2, 2, 4, 6, true},     // 13: 64 ch x 112 px, same scheme
};
constexpr int kNumTapVariants = sizeof(kTapVariants) / sizeof(kTapVariants[0]);
#define TAP_VARIANT_LIST(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13)

// rs_index: 0 -> 1x1, 1 -> 3x3, 2 -> 5x5. Returns hipSuccess or the launch error.
hipError_t launch_tap(int rs_index, int variant, int x_vec, int w_vec, int grid, int lds_bytes,
                      hipStream_t stream, const KernelArgs& a);
hipError_t launch_generic(int grid, int block, hipStream_t stream, const KernelArgs& a);

}  // namespace convfwd
