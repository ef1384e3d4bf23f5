// Internal declarations shared by the host dispatch code and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>

namespace convfwd {

constexpr int kMaxDevices = 16;  // per-device launch state is kept for this many GPUs of one process

// Division by a launch-time constant as multiply-high, subtract, shift (round-up method of Granlund and
// Montgomery: exact for every 32-bit unsigned dividend). The host fills it, the kernels only use div().
struct FastDiv {
    unsigned mul, sh1, sh2;
#if defined(__HIPCC__)
    __device__ __forceinline__ unsigned div(unsigned n) const
    {
        const unsigned t = __umulhi(mul, n);
        return (t + ((n - t) >> sh1)) >> sh2;
    }
#endif
};
inline FastDiv make_fastdiv(unsigned d)
{
    unsigned l = 0;
    while ((1ull << l) < d) ++l;  // ceil(log2 d)
    FastDiv f;
    f.mul = (unsigned)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l > 0 ? l - 1 : 0;
    return f;
}

#if defined(__HIPCC__)
// Fused epilogue (Section 2.1: the weighted sums of a layer are usually passed through a non-linear function
// such as ReLU): bias of the output channel, then the optional clamp at zero.
__device__ __forceinline__ float finish_output(float v, float b, int relu) { v += b; return relu ? fmaxf(v, 0.f) : v; }
#endif

// Everything a kernel needs; passed by value. All offsets are in floats and fit 32 bits
// (the host rejects tensors of 2^31 or more elements).
struct KernelArgs {
    const float* x;
    const float* w;
    float* y;
    const float* bias;  // K floats added to every output of a channel before the optional ReLU; null: none
    int relu;           // nonzero: outputs are max(., 0)
    int N, C, H, W, K, R, S, pad_h, pad_w;
    int P, Q, PQ, HW, CRS;
    int Hp;          // H + 2*pad_h: rows of one zero-padded image
    int total_pix;   // N*P*Q, output pixels in flattened (n,p,q) order
    // tiling (tap and pointwise families)
    int tile_pix;    // output pixels per work-group
    int ktiles;      // work-groups along K
    int ptiles;      // work-groups along the flattened pixels
    int nchunks;     // channel chunks (the chunk size is a property of the tile shape) of one work-group
    int split_c;     // tap family: channels one work-group reduces (a multiple of the chunk, or >= C: no splitting);
                     // work-group index = ((share * ptiles) + pixel tile) * ktiles + channel tile
    int k_group;     // tap family: channel tiles per group in the work-group numbering,
                     // index = ((group * pt_all) + (share * ptiles + pixel tile)) * k_group + channel tile within the group:
                     // ktiles = the channel tile is the fast index, 1 = work-group index = channel tile * pt_all + (share * ptiles + pixel tile),
                     // so that the run of work-groups one XCD receives shares few channel tiles (filters) and many pixel
                     // tiles; the host picks the order that makes the eight L2s fetch fewer bytes in total
    int pt_all;      // ptiles * shares
    // LDS halo tile of the tap family
    int lds_rows, lds_pitch, lds_plane;
    int col_shift;   // LDS column of padded column 0 (keeps vector stores aligned)
    int x_items;     // vector loads per chunk for the halo tile
    int direct;      // tap family: nonzero = the loader that moves global memory straight into LDS (2: issued by loader waves
                     // of their own; 3: with deep_copies() staging copies instead of two). Then x_items counts the
                     // vectors of the LDS halo tile of a chunk, padding included (chunk_c * lds_plane / x_vec), and
                     // div_slot_c / div_row_vecs divide by lds_plane / x_vec and lds_pitch / x_vec
    // dividers for the index arithmetic of the prologue
    FastDiv div_ktiles, div_ptiles, div_pt_all, div_k_group, div_PQ, div_Q, div_Hp, div_row_vecs, div_slot_c;
    // tap family: correctly rounded float reciprocals of the divisors of the per-lane index arithmetic (the divisors of
    // div_slot_c and div_row_vecs, Hp, Q, P, P*Q); the dividends there are small, see small_div in the kernel
    float inv_slot_c, inv_row_vecs, inv_Hp, inv_Q, inv_P, inv_PQ;
};

// Taps per software-pipeline unit of the tap kernel: the shortest of {1, S, R*S} that keeps enough matrix
// instructions between an LDS read and its use - 24 for the large tiles at one or two waves per SIMD, 3 where a wave
// holds one or two MFMA tiles, 7 at three waves per SIMD and a single tap at four, whose other waves cover the latency
// -, stepped down again if two operand sets would not fit ~96 registers (~64 with two or more waves per SIMD). Short
// units also spread the staging slots over more places in a chunk. Measured per tile shape over the shape grid: the
// 32 x 224 shape at three waves 3 % faster with units of one tap than of three; the four-wave shapes 2-9 % and the
// 16- and 32-channel shapes with channel shares 3-5 % faster with units of a tap or a filter row than of a whole
// filter; but 64 x 112 at two waves 2 % slower with one tap than with three, and 64 x 208 2-4 % slower with three
// than with one.
constexpr int tap_unit_taps(int S, int RS, int MT, int NT, int occ)
{
    const int cand[3] = {1, S, RS};
    int pick = 2;
    for (int i = 2; i >= 0; --i)
        if (cand[i] * MT * NT >= (occ >= 4 ? 1 : occ >= 3 ? 7 : MT * NT <= 2 ? 3 : 24)) pick = i;
    while (pick > 0 && 2 * cand[pick] * (MT + NT) > (occ > 1 ? 64 : 96)) --pick;
    return cand[pick];
}

// Tile shapes of the tap family. A work-group holds WK x WP x WC waves; a wave owns MT x NT MFMA
// tiles of 16 output channels x 16 pixels. A chunk is 4*WC*GPC input channels: the WC waves that share
// a tile position take the chunk's 4-channel groups in turn (GPC each) and add their partial tiles
// through LDS at the end.
#ifndef CONV_DEEP_COPIES
#define CONV_DEEP_COPIES 4
#endif
constexpr int kDeepCopies = CONV_DEEP_COPIES;
struct TapVariant {
    int MT, NT, WK, WP, WC, GPC;
    int occ;     // waves per SIMD the kernel is compiled for (bounds its registers)
    int xslots;  // dwordx4 halo-tile loads a thread keeps in flight (x2 as many when rows force dwordx2)
    int xslots1; // the same for rows that force single dwords (maps of odd width are small: fewer than 4 * xslots do)
    // Nonzero: the wave's last pixel tile holds at most four pixels and is multiplied by the 4x4x1 matrix instruction (16
    // blocks of 4 channels x 4 pixels, a quarter of the cycles of a 16 x 16 tile) instead of a 16 x 16 x 4 one that would
    // be three quarters padding: a 14 x 14 map (196 = 12 * 16 + 4 pixels) then costs 12.25 tiles instead of 13.
    int tail = 0;
    constexpr int xs(int x_vec) const { return x_vec == 1 ? xslots1 : xslots * 4 / x_vec; }
    // Direct loads (global memory -> LDS without passing the registers) also fetch the padding cells of the halo tile,
    // and a slot costs half the registers: half as many slots again.
    constexpr int xs_direct(int x_vec) const { return xs(x_vec) + (xs(x_vec) + 1) / 2; }
    constexpr int wslots_direct(int RS) const { return (tile_k() * (chunk_c() * RS / 4 + 1) + block() - 1) / block(); }
    // LDS floats of one staging copy with direct loads: both regions are whole runs of 64 dwordx4
    constexpr int staging_floats_direct(int RS, int plane) const
    {
        return (chunk_c() * plane + 255) / 256 * 256 + (tile_k() * (chunk_c() * RS + 4) + 255) / 256 * 256;
    }
    constexpr int tile_k() const { return 16 * MT * WK; }
    constexpr int max_pix() const { return 16 * NT * WP - (tail ? 12 : 0); }
    // matrix-pipeline cycles of one tap of one 4-channel group of a wave
    constexpr int tap_cycles() const { return MT * (32 * (NT - (tail ? 1 : 0)) + (tail ? 8 : 0)); }
    constexpr int block() const { return 64 * WK * WP * WC; }
    constexpr int chunk_c() const { return 4 * WC * GPC; }
    // filter-block loads per thread and chunk, and whether that many registers are reasonable
    constexpr int wslots(int RS, int w_vec) const { return (tile_k() * chunk_c() * RS / w_vec + block() - 1) / block(); }
    // (eight or more channel shares never paid off on 5x5 filters in the sweeps: the filter block per chunk gets too large)
    constexpr bool supports(int RS) const
    {
        return tile_k() * chunk_c() * RS <= (occ > 2 ? 20 : occ > 1 ? 40 : 64) * block() && (WC < 8 || RS <= 9);
    }
    // Filters whose rows dwordx4 cannot walk (C not a multiple of 4) are staged dword by dword, with inputs
    // as dwordx4 (maps whose width is a multiple of 4: first layers) or dwords: a table entry per dword
    // staged, so small filter blocks only.
    constexpr bool supports_scalar(int RS, int x_vec = 1) const
    {
        return supports(RS) && xs(x_vec) + tile_k() * chunk_c() * RS / block() <= (occ > 2 ? 24 : 48);
    }
    // LDS floats of one staging copy for a halo plane of `plane` floats (with the 256-float dump)
    constexpr int staging_floats(int RS, int plane) const
    {
        return ((chunk_c() * plane + tile_k() * (chunk_c() * RS + 4) + 3) & ~3) + 256;
    }
    // LDS floats the cross-wave reduction needs (the first round of the tree is the widest)
    constexpr int reduce_floats() const { return WC > 1 ? (WC / 2) * WK * WP * MT * NT * 256 : 0; }
    // Loader waves a build of this shape with dedicated loading waves adds (0: no such build). Built for the shapes of
    // eight waves at two per SIMD: a ninth to twelfth wave then fits the register file at three per SIMD.
    constexpr int loader_waves() const { return block() == 512 && occ == 2 ? 4 : 0; }
    // Staging copies of the deep direct loader (0: no such build): built for the shapes whose waves hold one or two MFMA
    // tiles - the shapes of batch-1 and other small layers, whose chunks are short against the time a load takes.
    constexpr int deep_copies() const { return MT * NT <= 2 ? kDeepCopies : 0; }
    // LDS bytes a work-group may take so that as many work-groups as the registers allow share a CU
    constexpr int lds_limit() const { return 160 * 1024 / (occ * 256 / block() > 0 ? occ * 256 / block() : 1); }
};

constexpr TapVariant kTapVariants[] = {
    {1, 13, 4, 1, 1, 4, 1, 8, 32},  //  0: 64 ch x 208 px, waves split K, 16-channel chunks
    {1, 7, 4, 1, 1, 4, 1, 8, 32},   //  1: 64 ch x 112 px
    {1, 1, 1, 4, 1, 2, 2, 4, 16},   //  2: 16 ch x  64 px, one MFMA tile per wave, 8-channel chunks
    {2, 4, 2, 2, 1, 4, 1, 8, 32},   //  3: 64 ch x 128 px, 2x4 tiles per wave
    {1, 2, 2, 2, 1, 2, 2, 4, 16},   //  4: 32 ch x  64 px, 8-channel chunks
    {2, 2, 1, 1, 4, 1, 2, 4, 16},   //  5: 32 ch x  32 px, 4 channel shares, for layers with few outputs
    {1, 13, 4, 1, 2, 2, 2, 2, 8},  //  6: 64 ch x 208 px (a 14x14 image), 8 waves (4 along K x 2 channel shares), two per SIMD
    {1, 7, 4, 1, 2, 2, 2, 2, 8},   //  7: 64 ch x 112 px, same scheme
    {1, 7, 4, 1, 1, 2, 1, 8, 32},   //  8: 64 ch x 112 px, 8-channel chunks (large filters)
    {2, 7, 2, 1, 2, 1, 1, 8, 32},   //  9: 64 ch x 112 px, 2 channel shares, 8-channel chunks (large filters)
    {1, 1, 1, 1, 4, 1, 2, 4, 16},   // 10: 16 ch x  16 px, 4 channel shares: many small work-groups for tiny layers
    {1, 2, 1, 1, 4, 1, 2, 4, 16},   // 11: 16 ch x  32 px, 4 channel shares
    {1, 7, 2, 1, 4, 1, 2, 8, 12},   // 12: 32 ch x 112 px, 8 waves (2 along K x 4 channel shares)
    {1, 2, 1, 1, 4, 1, 4, 4, 8},   // 13: as 11 with four waves per SIMD: the latency of short chunks is hidden by occupancy
    {1, 7, 1, 4, 1, 2, 2, 8, 16},   // 14: 16 ch x 448 px: layers with 16 or fewer filters on large maps
    {1, 4, 1, 4, 1, 4, 2, 8, 16},   // 15: 16 ch x 256 px, 16-channel chunks
    {1, 7, 1, 4, 1, 1, 2, 8, 16},   // 16: 16 ch x 448 px, 4-channel chunks: first layers (3 input channels)
    {1, 1, 1, 1, 16, 1, 4, 2, 8},   // 17: 16 ch x  16 px, 16 channel shares (64-channel chunks): deep N=1 layers on tiny maps
    {1, 2, 1, 1, 8, 1, 2, 4, 16},   // 18: 16 ch x  32 px, 8 channel shares (32-channel chunks)
    {1, 7, 2, 1, 4, 2, 2, 8, 12},   // 19: as 12 with 32-channel chunks: half as many barriers per layer
    {1, 2, 1, 1, 4, 2, 2, 4, 16},   // 20: as 11 with 32-channel chunks
    {1, 11, 4, 1, 2, 2, 2, 4, 12},  // 21: 64 ch x 176 px: a whole 13x13 image per work-group
    {1, 7, 1, 4, 1, 1, 3, 4, 8},    // 22: as 16 with three waves per SIMD: first layers are all prologue and stores, occupancy hides them
    {1, 7, 2, 2, 1, 1, 3, 4, 8},    // 23: 32 ch x 224 px, 4-channel chunks, three waves per SIMD
    {1, 1, 1, 4, 1, 2, 4, 4, 8},    // 24: as 2 with four waves per SIMD
    {1, 2, 2, 2, 1, 2, 4, 4, 8},    // 25: as 4 with four waves per SIMD
    {1, 13, 4, 1, 2, 2, 2, 2, 8, 1},  // 26: as 6 for tiles of 196 pixels (a 14x14 image, four 7x7 images): the 13th tile is a four-pixel tail
    {1, 7, 4, 1, 2, 2, 2, 3, 8, 1},   // 27: as 7 for tiles of up to 100 pixels (six tiles and a tail): 98 pixels put 8 x 56 x 56 outputs on 256 work-groups
    {1, 7, 2, 1, 4, 1, 2, 8, 12, 1},  // 28: as 12 with a tail: 32 ch x 100 px, half a 14x14 image per tile
    {1, 7, 2, 1, 4, 2, 2, 8, 12, 1},  // 29: as 19 with a tail
    {1, 7, 1, 4, 1, 1, 1, 16, 32},    // 30: as 16 with twice the staging slots and the whole LDS (one work-group per CU): maps 600 to ~1200 pixels wide, which no other shape's halo tile takes
};
constexpr int kNumTapVariants = sizeof(kTapVariants) / sizeof(kTapVariants[0]);

// Every staging slot a kernel instance is compiled with runs in every chunk, needed or not (a slot without data loads
// element 0 and stores to a dump row). A tile shape's slot count is sized for the largest halo tile it accepts, so the
// loaders for filter rows of whole dwordx4 are also built with half of it and - for input rows that move as single
// dwords, where the capacity is 4x the vector one - a quarter: the launcher takes the smallest build that covers the layer (on 7x7 maps that is
// 2 slots instead of 8, and a quarter less time for the deep batch-1 layers). Returns the divisor 1, 2 or 4.
constexpr int tap_x_slot_divisor(const TapVariant& tv, int x_vec, int w_vec, int x_items, bool direct = false)
{
    if (w_vec != 4) return 1;
    const int need = (x_items + tv.block() - 1) / tv.block();
    const int full = direct ? tv.xs_direct(x_vec) : tv.xs(x_vec);
    if (x_vec == 1 && (full + 3) / 4 >= need) return 4;
    return (full + 1) / 2 >= need ? 2 : 1;
}
#define TAP_VARIANT_LIST(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15) X(16) X(17) X(18) X(19) X(20) X(21) X(22) X(23) X(24) X(25) X(26) X(27) X(28) X(29) X(30)

// Filter sizes the tap kernel is instantiated for. The three the paper evaluates (Section 4: 1x1, 3x3, 5x5) get every
// tile shape; the others (filter rows and columns, even and 7x7 filters, as the factorised layers of later CNNs use)
// a small set that covers tiny, deep batch-1, medium and wide-map layers. Any other size runs the generic kernel.
#define TAP_EXTRA_VARIANTS(X, r, s) X(r, s, 2) X(r, s, 5) X(r, s, 7) X(r, s, 14) X(r, s, 16) X(r, s, 20) X(r, s, 22)
#define TAP_EXTRA_SIZES(X)                                                                                         \
    TAP_EXTRA_VARIANTS(X, 1, 3) TAP_EXTRA_VARIANTS(X, 3, 1) TAP_EXTRA_VARIANTS(X, 1, 5) TAP_EXTRA_VARIANTS(X, 5, 1) \
    TAP_EXTRA_VARIANTS(X, 1, 7) TAP_EXTRA_VARIANTS(X, 7, 1) TAP_EXTRA_VARIANTS(X, 2, 2) TAP_EXTRA_VARIANTS(X, 4, 4) \
    TAP_EXTRA_VARIANTS(X, 7, 7)
struct TapSize {
    int R, S;
};
constexpr TapSize kTapSizes[] = {{1, 1}, {3, 3}, {5, 5}, {1, 3}, {3, 1}, {1, 5}, {5, 1}, {1, 7}, {7, 1}, {2, 2}, {4, 4}, {7, 7}};
constexpr int kNumTapSizes = sizeof(kTapSizes) / sizeof(kTapSizes[0]);
constexpr int kNumFullTapSizes = 3;  // the leading entries of kTapSizes that have every tile shape
constexpr int tap_size_index(int R, int S)
{
    for (int i = 0; i < kNumTapSizes; ++i)
        if (kTapSizes[i].R == R && kTapSizes[i].S == S) return i;
    return -1;
}

// Tile shapes of the pointwise (1x1, no padding) family: a work-group is WC x WP waves on 16*MT output
// channels x WP*64 contiguous pixels of one image; the WC shares split the input channels.
struct PointwiseVariant {
    int MT, WC, WP;
    int PD;  // 16-channel steps of loads a wave keeps in flight (every wave runs a multiple of PD steps)
    constexpr int tile_k() const { return 16 * MT; }
    constexpr int tile_pix() const { return 64 * WP; }
    constexpr int block() const { return 64 * WC * WP; }
    constexpr int lds_bytes() const { return WC > 1 ? (WC / 2) * WP * MT * 4 * 1024 : 0; }
    constexpr int depth() const { return PD; }
};
constexpr PointwiseVariant kPointwiseVariants[] = {
    {1, 4, 1, 2}, {1, 8, 1, 2}, {2, 4, 1, 2}, {2, 8, 1, 2}, {4, 4, 1, 2}, {4, 8, 1, 2}, {1, 16, 1, 4}, {2, 16, 1, 2},  // 0-7: channel shares only
    {1, 1, 4, 2}, {2, 1, 4, 2}, {4, 1, 4, 2}, {2, 1, 2, 2}, {2, 2, 2, 2}, {4, 2, 2, 2},                            // 8-13: streaming shapes
    {1, 8, 1, 4}, {1, 4, 1, 4},  // 14-15: four steps in flight: deep N=1 layers, where a wave's chain of dependent loads sets the time
};
constexpr int kNumPointwiseVariants = sizeof(kPointwiseVariants) / sizeof(kPointwiseVariants[0]);
#define POINTWISE_VARIANT_LIST(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15)
hipError_t launch_pointwise(int variant, int x_vec, int grid, int lds_bytes, hipStream_t stream, const KernelArgs& a);

// Panel shapes of the pointwise family (batched 1x1 layers): a work-group of NW waves keeps the filters
// of 16*MT output channels in LDS and every wave streams 64-pixel tiles past them with PD 16-channel
// steps of input loads in flight. KernelArgs carry: ktiles, ptiles = work-groups per channel tile,
// nchunks = steps (C rounded up to 16*PD, over 16), x_items = 64-pixel tiles in all, lds_pitch = floats per
// panel row, div_ktiles, div_PQ, div_row_vecs (by 4 * nchunks); col_shift = pixel mode (launch_panel's pix); with
// tiles per image: tile_pix = tiles per image and div_ptiles divides by it.
struct PanelVariant {
    int MT, NW, PD;
    constexpr int tile_k() const { return 16 * MT; }
    constexpr int block() const { return 64 * NW; }
};
constexpr PanelVariant kPanelVariants[] = {
    {4, 8, 2}, {2, 8, 4}, {1, 8, 4}, {4, 4, 4}, {2, 4, 4}, {1, 4, 4},
    {4, 4, 2}, {2, 4, 2}, {2, 8, 2},  // two steps in flight: layers with 32 (mod 64) or fewer channels
};
constexpr int kNumPanelVariants = sizeof(kPanelVariants) / sizeof(kPanelVariants[0]);
#define PANEL_VARIANT_LIST(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8)
hipError_t launch_panel(int variant, int pix, int grid, int lds_bytes, hipStream_t stream, const KernelArgs& a);

// rs_index: index into kTapSizes. Returns hipSuccess, the launch error, or hipErrorInvalidValue for a (size, tile shape)
// pair that is not built (tap_is_built tells).
bool tap_is_built(int rs_index, int variant);
hipError_t launch_tap(int rs_index, int variant, int x_vec, int w_vec, int grid, int lds_bytes,
                      hipStream_t stream, const KernelArgs& a);
hipError_t launch_generic(int grid, int block, hipStream_t stream, const KernelArgs& a);
// *ptr = the current device's copy of the library's static scratch array (kStaticScratchBytes bytes, 256-byte aligned),
// looked up once per device
constexpr long long kStaticScratchBytes = 16ll << 20;
hipError_t static_scratch(float** ptr);
// buffer: 16-byte aligned device memory of at least `bytes` bytes; contents are overwritten
hipError_t launch_scratch_fill(void* buffer, long long bytes, hipStream_t stream);
// micro-probes: 8192 waves x iters x 16 fp32 MFMAs (2048 flops each); a dwordx4 copy of `bytes` (16-byte aligned pointers)
hipError_t launch_probe_mfma(int iters, float* sink, hipStream_t stream);
hipError_t launch_probe_copy(const void* src, void* dst, long long bytes, hipStream_t stream);
// y[i] = act(sum over shares of parts[share * total + i] + bias[channel of i]), shares added in index order;
// total = N*K*P*Q floats per share
hipError_t launch_split_reduce(const float* parts, float* y, const float* bias, int relu, int splits, int total, int PQ,
                               int K, hipStream_t stream);
// temp: R*S*N*K*P*Q floats (unused for 1x1 filters)
hipError_t launch_two_stage(hipStream_t stream, const KernelArgs& a, float* temp);

}  // namespace convfwd
