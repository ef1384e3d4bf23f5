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

// Tile shapes of the tap family. A work-group holds WK x WP waves; a wave owns
// MT x NT MFMA tiles of 16 output channels x 16 pixels.
struct TapVariant {
    int MT, NT, WK, WP;
    constexpr int tile_k() const { return 16 * MT * WK; }
    constexpr int max_pix() const { return 16 * NT * WP; }
    constexpr int block() const { return 64 * WK * WP; }
};

constexpr int kTapXSlots = 8;   // halo-tile vector loads a thread may hold in flight
constexpr int kTapWSlots = 12;  // filter-block vector loads a thread may hold in flight

constexpr TapVariant kTapVariants[] = {
    {1, 13, 4, 1},  // 0: 64 ch x 208 px  - one 14x14 image (196 px) per work-group
    {1, 7, 4, 1},   // 1: 64 ch x 112 px
    {1, 1, 1, 4},   // 2: 16 ch x  64 px  - small layers: one MFMA tile per wave
    {2, 4, 2, 2},   // 3: 64 ch x 128 px  - 2x4 tiles per wave, fewest LDS reads per MFMA
    {1, 2, 2, 2},   // 4: 32 ch x  64 px
};
constexpr int kNumTapVariants = sizeof(kTapVariants) / sizeof(kTapVariants[0]);

// rs_index: 0 -> 1x1, 1 -> 3x3, 2 -> 5x5. Returns hipSuccess or the launch error.
hipError_t launch_tap(int rs_index, int variant, int x_vec, int w_vec, int grid, int lds_bytes,
                      hipStream_t stream, const KernelArgs& a);
hipError_t launch_generic(int grid, int block, hipStream_t stream, const KernelArgs& a);

}  // namespace convfwd
