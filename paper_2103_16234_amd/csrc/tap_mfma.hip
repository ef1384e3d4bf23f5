// Tap-family kernel: direct convolution with the input halo tile and a filter block in LDS,
// reduced over (channel, tap) with full-precision fp32 MFMA (v_mfma_f32_16x16x4_f32).
//
// One work-group owns TK output channels x tile_pix output pixels, the pixels counted in
// flattened (n, p, q) order, and walks the input channels in chunks of CC = 4*WC*GPC:
//   a1  halo tile: the rows of the zero-padded, vertically stacked images that the pixel range
//       touches go HBM -> registers -> LDS with dwordx4 loads (dwordx2 / dword when the row length
//       forbids); padding cells are zeroed once and never written again;
//   a2  filter block: w[k0..k0+TK, c0..c0+CC, :, :] is CC*R*S contiguous floats per output channel
//       and takes the same path;
//   a3  for every (4-channel group, r, s): A = filters [16 k x 4 c], B = inputs [4 c x 16 px] read from
//       the halo tile at the tap's offset, acc += A*B on the matrix cores. Each input element in LDS
//       is reused by the R*S taps and by all TK channels, each filter element by all pixels (the two
//       reuse levels of Section 3);
//   a4  accumulators -> y in NCHW: no second pass and no workspace (the per-tap partial matrices of
//       the two-stage scheme of Section 3 never leave the registers).
//
// What shapes the code (measured on gfx950): a wave's matrix instructions issue back to back only if
// little else sits between them. One or two independent LDS reads / address adds per MFMA are free;
// bursts of scalar arithmetic, of global loads (the CU's address path takes 64 B/clk and the issuing
// wave stalls) or of LDS stores are not. Hence
//   * the MAC loop of one chunk is fully unrolled with every tap offset a compile-time immediate, and
//     the LDS reads of unit u+1 are interleaved with the MFMAs of unit u (software pipeline);
//   * the staging area exists twice. While chunk ch is read from copy ch&1, each thread drips its
//     staging slots through the chunk: slot k is written (data of chunk ch+1, loaded one chunk ago,
//     so HBM latency is long gone) to the other copy and at once reloaded with chunk ch+2. No
//     bursts, one barrier per chunk;
//   * waves can split the channels of a chunk (WC) and each own a larger tile, which cuts the LDS
//     reads per MFMA; their partial tiles are added through LDS in a fixed order at the end.
//
//   * the second loader (template flag DMA) skips the registers: a buffer load with the lds modifier moves 64
//     consecutive dwordx4 (or dwords) per wave instruction from 64 arbitrary offsets straight into LDS. A slot is then
//     a run of 64 vectors of a staging copy, padding cells included (those lanes carry an offset past the buffer's end
//     and receive zeros, so nothing is ever zero-filled or masked), one constant offset per slot instead of a table
//     entry and a data register, no LDS store instructions, no address arithmetic per chunk, and chunk ch+1 is fetched
//     while chunk ch is multiplied (one chunk of look-ahead: long layers gain, short latency-bound ones prefer the
//     register loader's two).
//
// Compiled once per (filter size, tile shape): TAP_R, TAP_S, TAP_VARIANT come from the build.
#include "conv_internal.h"

#include <atomic>
#include <utility>

namespace convfwd {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

template <int V> struct Vec;
template <> struct Vec<4> {
    f32x4 v;
    __device__ void load(const float* p) { v = *reinterpret_cast<const f32x4*>(p); }
    __device__ void keep_if(bool c) { v = c ? v : f32x4{0.f, 0.f, 0.f, 0.f}; }
    __device__ void store16(float* p) const { *reinterpret_cast<f32x4*>(p) = v; }
    __device__ void store8(float* p) const
    {
        *reinterpret_cast<f32x2*>(p) = f32x2{v.x, v.y};
        *reinterpret_cast<f32x2*>(p + 2) = f32x2{v.z, v.w};
    }
};
template <> struct Vec<2> {
    f32x2 v;
    __device__ void load(const float* p) { v = *reinterpret_cast<const f32x2*>(p); }
    __device__ void keep_if(bool c) { v = c ? v : f32x2{0.f, 0.f}; }
    __device__ void store16(float* p) const { *reinterpret_cast<f32x2*>(p) = v; }
    __device__ void store8(float* p) const { *reinterpret_cast<f32x2*>(p) = v; }
};
template <> struct Vec<1> {
    float v;
    __device__ void load(const float* p) { v = *p; }
    __device__ void keep_if(bool c) { v = c ? v : 0.f; }
    __device__ void store16(float* p) const { *p = v; }
    __device__ void store8(float* p) const { *p = v; }
};

template <int N> using IntC = std::integral_constant<int, N>;
// f(IntC<Lo>{}), ..., f(IntC<Hi - 1>{})
template <int Lo, int Hi, class F> __device__ __forceinline__ void for_range(F&& f)
{
    if constexpr (Lo < Hi) {
        f(IntC<Lo>{});
        for_range<Lo + 1, Hi>(f);
    }
}

// x / d for a small non-negative x (below 2^22) and a launch-time divisor d whose correctly rounded float reciprocal
// the host supplies: (x + 1/2) / d is at least 1/(2d) away from every integer, and the two roundings (the reciprocal, the
// fused multiply-add) move it by less than (x + 1/2) * 2^-23 / d, so truncation gives the exact quotient. Three full-rate
// vector instructions, where the multiply-high method takes a quarter-rate multiply and four more; the prologue's
// per-lane index arithmetic (slot tables, pixel table) and the epilogue's are made of these.
__device__ __forceinline__ int small_div(int x, float inv) { return static_cast<int>(fmaf(static_cast<float>(x), inv, 0.5f * inv)); }

// Scheduling directive for the straight-line code since the previous fence: issue the matrix
// instructions in order and slip in front of each a few address adds, up to two LDS reads, one LDS
// store and one global load; then fence so nothing moves across.
template <int N_MFMA> __device__ __forceinline__ void interleave_with_mfma()
{
#pragma unroll
    for (int i = 0; i < N_MFMA; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);  // VALU
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // DS read
        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // DS write
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // VMEM read
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
    }
    __builtin_amdgcn_sched_barrier(0);
}

// LW > 0: the work-group has LW more waves, the loader waves, which do nothing but the direct loads of the staging copies
// (all slots are theirs, XS and WS count slots per loader thread); the other waves then contain no memory instruction
// between the prologue and the stores. OCC counts all waves of a SIMD.
// DEPTH: staging copies in LDS. Two everywhere but in the deep direct loader (DMA, LW == 0), which keeps DEPTH - 1 chunks
// on their way while one is multiplied: a chunk's loads then have DEPTH - 1 chunk times to arrive instead of one, for
// layers whose chunk is shorter than the ~0.5-1 us a load takes from the L2 or beyond.
// TAIL: the wave's last pixel tile (index NT - 1) covers at most four pixels and is multiplied with v_mfma_f32_4x4x1 (16 blocks,
// 8 cycles instead of 32). Block b of that instruction takes lanes 4b .. 4b+3: with block = (channel lane >> 4, output-channel
// quad (lane >> 2) & 3) the A operand is the very register the 16 x 16 x 4 tiles use (lane holds w[k = lane & 15][c = lane >> 4]),
// and the B operand is read like any other tile's, only with pixel lane & 3 instead of lane & 15. Each block sums one channel:
// the four channels of a quad are added across lanes once, before the stores.
template <int R, int S, int MT, int NT, int WK, int WP, int WC, int GPC, int OCC, int XS, int WS, int VX, int VW, bool DMA = false, int LW = 0,
          int DEPTH = 2, bool TAIL = false>
__global__ void __launch_bounds__(64 * (WK * WP * WC + LW), OCC) conv_tap_mfma(const KernelArgs a)
{
#if defined(__HIP_DEVICE_COMPILE__)  // (the buffer-descriptor type below exists for the GPU only; the host needs just the kernel's symbol)
    static_assert(DEPTH == 2 || (DMA && LW == 0 && DEPTH > 2 && DEPTH <= 8), "only the direct loader of the multiplying waves runs deeper");
    static_assert((DEPTH - 2) * (XS + WS) <= 63, "the in-order load counter holds 63");
    static_assert(WC >= 1 && WC <= 16 && (WC & (WC - 1)) == 0, "the cross-wave reduction is a binary tree");
    static_assert(LW == 0 || DMA, "loader waves move data with direct loads");
    static_assert(!TAIL || (WP == 1 && NT >= 2), "the four-pixel tail is the last tile of the work-group's pixel range");
    constexpr int BLOCK = 64 * WK * WP * WC;  // threads of the waves that multiply
    constexpr int NWC = WK * WP * WC;
    constexpr int LB = LW > 0 ? 64 * LW : BLOCK;  // threads that own staging slots
    constexpr int RS = R * S;
    constexpr int TK = 16 * MT * WK;
    constexpr int CC = 4 * WC * GPC;     // channels per chunk
    constexpr int WPITCH = CC * RS + 4;  // floats per output channel in the LDS filter block (rows stay 16-byte aligned)
    // (With loader waves a unit is one tap: the multiplying waves then hold nothing but LDS reads and matrix instructions, and
    // the seven-tile shapes measured 2.5-5 % faster on 3x3 layers of 37..125 us than with units of a filter row.)
    constexpr int UT = LW > 0 ? 1 : tap_unit_taps(S, RS, MT, NT, OCC);
    constexpr int UNITS = RS / UT;       // pipeline units per 4-channel group
    constexpr int U = GPC * UNITS;       // pipeline units per chunk (per wave)
    constexpr int TS = XS + WS;          // staging slots per thread
    // Pipeline units of a chunk over which a thread's staging slots are spread: all of them, or - direct dwordx4 loads of
    // tile shapes whose chunk is short (64 matrix instructions per wave or fewer) - the first third, so that the data of
    // the next chunk is not still on its way when this one ends. Measured on the 3x3 / 5x5 layers of the shape grid that
    // run such shapes: batch-1 layers on 28..56-pixel maps 2-14 % faster (1 x 64 x 56 x 56 -> 64: 8.9 -> 7.7 us), layers of
    // 100 us and more unchanged; with single-dword rows (odd map widths: four times the slots) it loses 1-4 % instead.
    constexpr int UI = (DMA && LW == 0 && VX == 4 && MT * NT * GPC * RS <= 64) ? (U + 2) / 3 : U;

    extern __shared__ f32x4 smem4[];
    float* const lds = reinterpret_cast<float*>(smem4);
    // One staging copy: halo tile [CC][plane], filter block [TK][WPITCH], then a 64 x 16 B dump that
    // absorbs the stores of slots a thread does not own.
    // With direct loads (DMA) a wave instruction fills 64 consecutive vectors of LDS, so both regions are rounded
    // up to whole runs of 64 dwordx4 and there is no dump.
    constexpr int WREG = DMA ? (TK * WPITCH + 255) / 256 * 256 : TK * WPITCH;
    const int xs_floats = DMA ? (CC * a.lds_plane + 255) & ~255 : CC * a.lds_plane;
    const int dump_off = (xs_floats + TK * WPITCH + 3) & ~3;
    const int buf_floats = DMA ? xs_floats + WREG : dump_off + 256;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: wk, wp, wc live in SGPRs
    const int j = lane & 15;   // pixel column of B / D, output-channel row of A
    const int kq = lane >> 4;  // channel within the 4-channel group (A, B); row group of D
    const int wk = wave % WK;
    const int wp = (wave / WK) % WP;
    const int wc = wave / (WK * WP);  // this wave reduces the chunk's channel groups wc + WC*gi
    const bool is_loader = LW > 0 && wave >= NWC;      // wave-uniform
    const int lwave = LW > 0 ? wave - NWC : wave;       // position among the waves that own staging slots

    // Work-groups are dealt round-robin to the 8 XCDs; renumber them so that each XCD (one L2)
    // gets a contiguous run of tiles: neighbours share the pixel tile and walk a group of a.k_group channel tiles, then
    // the next pixel tile, and after the last one the next group (all channel tiles in one group: each L2 fetches few
    // inputs and every filter; groups of one: the reverse, for layers whose filters outweigh their inputs).
    int L;
    {
        const int nb = gridDim.x, b = blockIdx.x;
        const int per = nb >> 3, rem = nb & 7, xcd = b & 7;
        L = xcd * per + (xcd < rem ? xcd : rem) + (b >> 3);
    }
    const int pair = a.div_k_group.div(L);          // (group, pixel tile)
    const int group = a.div_pt_all.div(pair);
    const int pt_all = pair - group * a.pt_all;
    const int ktile = group * a.k_group + (L - pair * a.k_group);
    // Channel splitting across work-groups: share `split` reduces channels cb .. cb+C_l-1 and writes a whole
    // partial output tensor of its own (a.y then points at the workspace; a second kernel adds the shares).
    // Without splitting there is one share, all of C.
    const int split = a.div_ptiles.div(pt_all);
    const int ptile = pt_all - split * a.ptiles;
    const int cb = split * a.split_c;
    const int C_l = min(a.C - cb, a.split_c);
    const int nchunks = (C_l + CC - 1) / CC;
    const float* const x_share = a.x + static_cast<size_t>(cb) * a.HW;
    const float* const w_share = a.w + cb * RS;
    float* const y_share = a.y + static_cast<size_t>(split) * a.K * a.total_pix;
    const int k0 = ktile * TK;
    const int g0 = ptile * a.tile_pix;
    const int g_end = min(g0 + a.tile_pix, a.total_pix);
    // the tile's first pixel (n0, p0, q0): wave-uniform, kept in scalar registers. Every per-lane position below is this
    // plus a small offset, so the per-lane divisions only ever see small numbers.
    const int n0 = a.div_PQ.div(g0);
    const int pq0 = g0 - n0 * a.PQ;
    const int p0 = a.div_Q.div(pq0);
    const int q0 = pq0 - p0 * a.Q;
    // (the first stacked padded row held in LDS is V0 = n0 * Hp + p0)
    // row `row` of the LDS halo tile (stacked padded row V0 + row) -> image and input row of that image
    auto image_row = [&](int row, int& n, int& h) {
        int t = p0 + row;  // padded row counted from the top of image n0; runs on into the following images
        int dn = 0;
        const int r = t - a.Hp;
        if (r >= 0) {
            const int m = small_div(r, a.inv_Hp);
            dn = 1 + m;
            t = r - __mul24(m, a.Hp);  // (m > 0 only where an image has fewer rows than the halo tile)
        }
        n = n0 + dn;
        h = t - a.pad_h;
    };

    // Staging slots. xg / wg: offset in floats from the chunk's first channel in x / w; xl / wl: float
    // offset inside a staging copy in the low 16 bits, the slot's channel (x) or element offset in the
    // chunk's filter slice (w) above. Slots the thread does not own read element 0 and write the dump.
    constexpr int XR = DMA ? 1 : XS, WR = DMA ? 1 : WS;
    unsigned xg[XR], xl[XR], wg[WR], wl[WR];
    // Direct loads: slot i of a wave fills the vectors start .. start+63 of a region (start = x_position(i) /
    // w_position(i), wave-uniform), lane l the l-th of them. They are buffer loads: the address is a base held in scalar
    // registers - the first channel of the chunk being fetched, in the tile's first image (x) or first output channel (w) -
    // plus the slot's byte offset xo / wo, which never changes; moving on to the next chunk is scalar arithmetic on the two
    // bases, no vector instruction per slot (a 64-bit add per slot and chunk cost the 5x5 benchmark layer 4 % and the
    // others 1-2 %). Vectors that hold padding, rows outside the images, output channels past K, channels past a ragged
    // last chunk or nothing at all carry an offset beyond the buffer's size, for which the hardware returns zeros without
    // touching memory; past the last chunk the size is zero and every lane gets them. Runs that would reach past the
    // region start earlier and repeat part of the previous run.
    constexpr unsigned kNoData = 0xfffffff0u;  // (also the buffers' size: the host keeps real offsets 64 bytes below)
    unsigned xo[DMA ? XS : 1], wo[DMA ? WS : 1];
    const float* const x_tile = x_share + static_cast<size_t>(n0) * a.C * a.HW;
    const float* const w_tile = w_share + static_cast<size_t>(k0) * a.CRS;
    auto chunk_buffer = [&](const float* base, bool live) {
        // (stride 0: a raw buffer, offsets in bytes; the fourth word is the data format field every gfx9 descriptor carries)
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base), static_cast<short>(0), live ? kNoData : 0u, 0x00020000);
    };
    __amdgpu_buffer_rsrc_t x_buffer = chunk_buffer(x_tile, true), w_buffer = chunk_buffer(w_tile, true);
    constexpr int WPV = WPITCH / 4;  // vectors per output channel of the LDS filter block, the last one padding
    auto x_position = [&](int i) { return min(i * LB + lwave * 64, xs_floats / VX - 64); };  // wave-uniform
    auto w_position = [&](int i) { return min(i * LB + lwave * 64, WREG / 4 - 64); };
    // Direct loads: fetch the slot's vectors of the chunk the buffers stand at into the staging copy at dst_floats.
    auto slot_fetch = [&](auto kc, int dst_floats) {
        constexpr int k = decltype(kc)::value;
        if constexpr (k < XS) {
            float* const dst = lds + dst_floats + x_position(k) * VX;  // (uniform)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(x_buffer, LDS_PTR(dst), VX == 4 ? 16 : 4, xo[k], 0, 0, 0);
        } else {
            float* const dst = lds + dst_floats + xs_floats + w_position(k - XS) * 4;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(w_buffer, LDS_PTR(dst), 16, wo[k - XS], 0, 0, 0);
        }
    };
    // Building the slot offsets (and fetching chunk 0 into copy 0 with them; a slot whose channel lies past a share of less
    // than one chunk gets no data from the start).
    // The slot tables are a launch's fixed cost and pure vector arithmetic (one loader wave per SIMD builds some thirty slots
    // before the first byte moves), so what all channels of a chunk share is worked out once: a table in LDS - in the last
    // staging copy, which nothing fills before the chunk loop - maps a vector position of the halo plane to the offset of
    // its cell in channel 0 of the share (all ones: padding, a row outside the images, the plane's spare cells). A
    // slot then takes a division, a table look-up and a multiply-add per lane instead of decoding row, column and image
    // again for every channel (the 512-channel benchmark layer: 6.1 us until the last slot's load went out).
    // A direct load writes LDS, so no table look-up may move across one, and a wave that builds and fetches slot by slot
    // runs one short dependent chain after the other (measured: ~400 cycles per slot either way). Hence groups of eight:
    // eight pointers are worked out side by side, branch-free, then their eight loads go out.
    constexpr unsigned kNoCell = 0xffffffffu;
    [[maybe_unused]] unsigned* const cell_table = reinterpret_cast<unsigned*>(lds + (DEPTH - 1) * buf_floats);
    static_assert(!DMA || VW == 4, "filters move as dwordx4");
    constexpr int G = 8, XN = DMA ? XS : 0, WN = DMA ? WS : 0;
    auto build_x_slots = [&]() {
        const int plane_v = a.lds_plane / VX;
        auto point_x = [&](auto ic) {
            constexpr int i = decltype(ic)::value;
            const int e = x_position(i) + lane;
            const int c_l = small_div(e, a.inv_slot_c);
            const unsigned off = cell_table[e - __mul24(c_l, plane_v)];  // (e stays inside the CC planes and their round-up: the index is below plane_v)
            const bool cell = e < a.x_items && off != kNoCell && c_l < C_l;
            xo[i] = cell ? 4u * (off + static_cast<unsigned>(c_l) * a.HW) : kNoData;
        };
        for_range<0, (XN + G - 1) / G>([&](auto gc) {
            constexpr int lo = decltype(gc)::value * G, hi = lo + G < XN ? lo + G : XN;
            for_range<lo, hi>(point_x);
            for_range<lo, hi>([&](auto ic) { slot_fetch(ic, 0); });
        });
    };
    // (The filter slots need no table: their part of chunk 0 goes out first, before the table's barrier.)
    auto build_w_slots = [&]() {
        auto point_w = [&](auto ic) {
            constexpr int i = decltype(ic)::value;
            const int e = w_position(i) + lane;  // (below 2^16: small_div is exact)
            const int kl = small_div(e, 1.0f / WPV);
            const int ev = e - kl * WPV;
            const bool cell = kl < TK && ev < WPV - 1 && k0 + kl < a.K && ev * 4 < C_l * RS;
            // (the host checked that the filters of a channel tile span less than 2^32 bytes)
            wo[i] = cell ? 4u * (static_cast<unsigned>(kl) * a.CRS + ev * 4) : kNoData;
        };
        for_range<0, (WN + G - 1) / G>([&](auto gc) {
            constexpr int lo = decltype(gc)::value * G, hi = lo + G < WN ? lo + G : WN;
            for_range<lo, hi>(point_w);
            for_range<lo, hi>([&](auto ic) { slot_fetch(IntC<XS + decltype(ic)::value>{}, 0); });
        });
    };
    if constexpr (DMA) {
        if (LW == 0 || is_loader) build_w_slots();
        const int plane_v = a.lds_plane / VX, pitch_v = a.lds_pitch / VX;
        for (int v = tid; v < plane_v; v += 64 * (NWC + LW)) {
            const int row = small_div(v, a.inv_row_vecs);
            const int col = (v - __mul24(row, pitch_v)) * VX - a.col_shift - a.pad_w;
            int n, h;
            image_row(row, n, h);
            const bool cell = row < a.lds_rows && col >= 0 && col < a.W && n < a.N && h >= 0 && h < a.H;
            // (the host checked that the images a tile touches span less than 2^32 bytes)
            cell_table[v] = cell ? (static_cast<unsigned>(n - n0) * a.C * a.H + h) * a.W + col : kNoCell;  // (from x_tile)
        }
        // (a bare barrier: __syncthreads() carries a fence, before which the compiler would wait for the filter loads just issued)
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }
    if constexpr (DMA) {
        if constexpr (LW == 0) build_x_slots();  // chunk 0 goes out here too (with loader waves: theirs, where their role starts)
    } else {
        const int XV = a.W / VX;
        const int per_c = a.lds_rows * XV;
#pragma unroll
        for (int i = 0; i < XS; ++i) {
            const int e = tid + i * BLOCK;
            xg[i] = 0;
            xl[i] = dump_off + lane * 4;
            if (e < a.x_items) {
                const int c_l = small_div(e, a.inv_slot_c);
                const int rem = e - __mul24(c_l, per_c);
                const int row = small_div(rem, a.inv_row_vecs);
                const int cv = rem - __mul24(row, XV);
                int n, h;
                image_row(row, n, h);
                if (n < a.N && h >= 0 && h < a.H) {
                    // unsigned: a padding channel of the last image may lie past 2^31 elements before the ragged
                    // chunk is retargeted
                    xg[i] = (static_cast<unsigned>(n * a.C + c_l) * a.H + h) * a.W + cv * VX;
                    xl[i] = (c_l * a.lds_plane + row * a.lds_pitch + a.col_shift + a.pad_w + cv * VX) | (c_l << 16);
                }
            }
        }
        constexpr int WV = CC * RS / VW;
#pragma unroll
        for (int i = 0; i < WS; ++i) {
            const int e = tid + i * BLOCK;
            wg[i] = 0;
            wl[i] = dump_off + lane * 4;
            if (e < TK * WV) {
                const int kl = e / WV;
                const int ev = (e - kl * WV) * VW;
                if (k0 + kl < a.K) {
                    wg[i] = kl * a.CRS + ev;
                    wl[i] = (xs_floats + kl * WPITCH + ev) | (ev << 16);
                }
            }
        }
    }

    Vec<VX> xv[XR];
    Vec<VW> wv[WR];

    // One slot of the staging pipeline: slot k < XS is a halo-tile slot, the others filter slots.
    auto slot_load = [&](auto kc, int c0) {
        constexpr int k = decltype(kc)::value;
        if constexpr (k < XS) xv[k].load(x_share + c0 * a.HW + xg[k]);
        else wv[k - XS].load(w_share + k0 * a.CRS + c0 * RS + wg[k - XS]);
    };
    // When the share is not a multiple of the chunk, the last chunk's slots past its last channel would read past
    // the tensors. Before the first load of the last chunk (no other chunk is loaded after it) their table
    // entries are moved back to the last valid channel (x) or the last VW floats of the filter row (w);
    // what they fetch is replaced by zeros at the store anyway.
    const int last_c0 = (nchunks - 1) * CC;
    const bool ragged = C_l % CC != 0;
    auto retarget_last_chunk = [&]() {
        if constexpr (!DMA) {
#pragma unroll
            for (int i = 0; i < XS; ++i) {
                const int over = last_c0 + static_cast<int>(xl[i] >> 16) - (C_l - 1);
                if (over > 0) xg[i] -= over * a.HW;
            }
#pragma unroll
            for (int i = 0; i < WS; ++i) {
                const int over = last_c0 * RS + static_cast<int>(wl[i] >> 16) - (C_l * RS - VW);
                if (over > 0) wg[i] -= over;
            }
        }
    };
    // c0: first channel of the chunk the slot's data belongs to; channels past C are stored as zeros.
    auto slot_store = [&](auto kc, int c0, int dst_floats) {
        constexpr int k = decltype(kc)::value;
        if constexpr (k < XS) {
            Vec<VX> t = xv[k];
            t.keep_if(c0 + static_cast<int>(xl[k] >> 16) < C_l);
            t.store16(lds + dst_floats + (xl[k] & 0xffff));
        } else {
            Vec<VW> t = wv[k - XS];
            t.keep_if(static_cast<int>(wl[k - XS] >> 16) < (C_l - c0) * RS);
            t.store16(lds + dst_floats + (wl[k - XS] & 0xffff));
        }
    };
    // The buffers are about to stand at the last chunk of a share that is not a multiple of the chunk: vectors of
    // channels past the share get no data from here on.
    auto zero_past_share = [&]() {
        if constexpr (DMA) {
#pragma unroll
            for (int i = 0; i < XS; ++i) {
                const int e = x_position(i) + lane;
                if (e < a.x_items && last_c0 + small_div(e, a.inv_slot_c) >= C_l) xo[i] = kNoData;
            }
#pragma unroll
            for (int i = 0; i < WS; ++i) {
                const int ev = (w_position(i) + lane) % WPV;
                if (ev * 4 >= (C_l - last_c0) * RS) wo[i] = kNoData;
            }
        }
    };
    // Direct loads: the next fetches are those of chunk f. Past the last chunk the slots still run once (the loop is
    // branch-free): the buffers then have size zero, and nothing is read.
    auto before_fetch = [&](int f) {
        if constexpr (DMA) {
            if (ragged && f == nchunks - 1) zero_past_share();
            const int fc = min(f, nchunks - 1);
            x_buffer = chunk_buffer(x_tile + static_cast<size_t>(fc) * CC * a.HW, f < nchunks);
            w_buffer = chunk_buffer(w_tile + fc * (CC * RS), f < nchunks);
        }
    };
    // s_waitcnt vmcnt(n), n a constant below 64: bits 3:0 and 15:14 hold the count, the other counters are left alone
    auto wait_loads = [](auto nc) {
        constexpr int n = decltype(nc)::value;
        __builtin_amdgcn_s_waitcnt(0x0F70 | (n & 15) | ((n >> 4) << 14));
    };
    auto for_each_slot = [&](auto&& f) {
        [&]<int... Ks>(std::integer_sequence<int, Ks...>) { (f(IntC<Ks>{}), ...); }
        (std::make_integer_sequence<int, TS>{});
    };

    // Loader waves: chunk 0 into copy 0, then always one chunk ahead of the arithmetic - chunk ch+1 is fetched into the
    // other copy while the multiplying waves work on chunk ch, and the barrier at the end of a chunk is passed once the
    // fetched data has landed. They take part in every barrier of the work-group (those of the cross-wave reduction
    // too) and leave.
    if constexpr (LW > 0) {
        if (is_loader) {
            __builtin_amdgcn_s_setprio(3);  // their few instructions go ahead of the matrix work that shares the SIMD
            build_x_slots();  // (and chunk 0 is on its way)
            before_fetch(1);
            __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
            __syncthreads();
            for (int ch = 0; ch < nchunks; ++ch) {
                if (ch + 1 < nchunks) {
                    const int nxt_floats = ((ch + 1) & 1) * buf_floats;
                    for_each_slot([&](auto kc) { slot_fetch(kc, nxt_floats); });
                    before_fetch(ch + 2);
                    __builtin_amdgcn_s_waitcnt(0x0F70);
                }
                __syncthreads();
            }
            if constexpr (WC > 1) {
#pragma unroll
                for (int stride = WC / 2; stride >= 1; stride /= 2) {
                    if (stride != WC / 2) __syncthreads();
                    __syncthreads();
                }
            }
            return;
        }
    }

    f32x4 acc[MT][NT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[m][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Prologue: chunk 0 goes straight into copy 0, chunk 1 waits in the registers. While the first
    // loads are in flight, zero both staging copies (padding cells, rows past the batch and output
    // channels past K then stay zero for the whole kernel) and build the per-lane pixel table.
    // With direct loads chunk 0 is on its way to copy 0 at once and nothing has to be zeroed: every cell of a copy is
    // written by every chunk, padding included.
    if constexpr (LW > 0) {
        // (the loader waves fetch)
    } else if constexpr (DMA) {
        before_fetch(1);  // (chunk 0 went out with the slot tables)
#pragma unroll
        for (int d = 1; d < DEPTH - 1; ++d) {  // chunk d into copy d
            for_each_slot([&](auto kc) { slot_fetch(kc, d * buf_floats); });
            before_fetch(d + 1);
        }
    } else {
        if (ragged && nchunks == 1) retarget_last_chunk();
        for_each_slot([&](auto kc) { slot_load(kc, 0); });
        for (int i = tid; i < (2 * buf_floats) >> 2; i += BLOCK) smem4[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // Per-lane pixel table: byte offset inside a staging copy of the origin of the pixel's window, for
    // this lane's channel of this wave's first group (lanes past the end of the tile read the tile's
    // last pixel and are masked at the store).
    int xb[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int d = min((wp * NT + t) * 16 + ((TAIL && t == NT - 1) ? (j & 3) : j), g_end - 1 - g0);  // pixel g0 + d
        int q = q0 + d;  // below Q + the tile: small
        const int dp = small_div(q, a.inv_Q);
        q -= __mul24(dp, a.Q);
        int p = p0 + dp, dn = 0;  // output row counted from the top of image n0; may run on into the following images
        const int r = p - a.P;
        if (r >= 0) {
            const int m = small_div(r, a.inv_P);
            dn = 1 + m;
            p = r - __mul24(m, a.P);  // (m > 0 only on maps smaller than the tile)
        }
        // rows of LDS between this pixel's window and the tile's first: (n0 + dn) * Hp + p - V0
        xb[t] = 4 * ((4 * wc + kq) * a.lds_plane + __mul24(dn * a.Hp + p - p0, a.lds_pitch) + q + a.col_shift);
    }
    const int arow = 4 * (xs_floats + (wk * MT * 16 + j) * WPITCH + (4 * wc + kq) * RS);

    if constexpr (LW > 0) {
    } else if constexpr (DMA) {
        wait_loads(IntC<(DEPTH - 2) * TS>{});  // this wave's part of chunk 0 is in LDS (later chunks may still be on their way)
    } else {
        __syncthreads();  // zero fill complete before any data lands
        for_each_slot([&](auto kc) { slot_store(kc, 0, 0); });
        if (ragged && nchunks == 2) retarget_last_chunk();
        for_each_slot([&](auto kc) { slot_load(kc, min(CC, last_c0)); });
    }
    // The barrier between chunks. __syncthreads() carries a fence, and before a fence the compiler waits for every direct
    // load still in flight (they write LDS): the deep ring, whose later chunks must stay in flight across the barrier,
    // waits for its own loads by count (above and in the loop) and for its LDS reads here, and then takes the bare barrier.
    auto chunk_barrier = [] {
        if constexpr (DEPTH > 2) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        else __syncthreads();
    };
    chunk_barrier();

    struct Operands {
        float a[UT][MT];
        float b[UT][NT];
    };
    const char* const lds_bytes = reinterpret_cast<const char*>(lds);

    // Where work-groups share a CU, waves in the chunk loop go ahead of waves in a prologue, reduction or epilogue
    // (measured: +0.4-0.8 % on layers of 60 us and more, nothing elsewhere).
    __builtin_amdgcn_s_setprio(1);
    int ring_cur = 0, ring_fill = DEPTH - 1;  // ch % DEPTH and (ch + DEPTH - 1) % DEPTH
    for (int ch = 0; ch < nchunks; ++ch) {
        const int cur_copy = DEPTH == 2 ? (ch & 1) : ring_cur;
        const int fill_copy = DEPTH == 2 ? ((ch + 1) & 1) : ring_fill;
        const int cur_bytes = cur_copy * buf_floats * 4;
        const int nxt_floats = fill_copy * buf_floats;  // the copy the staging slots fill: chunk ch + DEPTH - 1
        const int c0_regs = min((ch + 1) * CC, last_c0);  // chunk whose data the staging registers hold
        const int c0_load = min((ch + 2) * CC, last_c0);  // chunk to fetch next (the last one again at the end)
        if constexpr (!DMA) {
            if (ragged && ch + 3 == nchunks) retarget_last_chunk();
        }

        const char* const a_base = lds_bytes + cur_bytes + arow;
        int xa[NT];  // B addresses of the filter row being read
        Operands o0, o1;

        // Operands of unit ui: taps tap0 .. tap0+UT-1 of this wave's group gi of the chunk.
        auto load_unit = [&](Operands& o, auto uic) {
            constexpr int ui = decltype(uic)::value;
            constexpr int gi = ui / UNITS;
            constexpr int tap0 = (ui % UNITS) * UT;
            constexpr int r0 = tap0 / S, s0 = tap0 % S;
            if constexpr (s0 == 0) {
                const int row_off = cur_bytes + 16 * gi * WC * a.lds_plane + 4 * r0 * a.lds_pitch;
#pragma unroll
                for (int t = 0; t < NT; ++t) xa[t] = xb[t] + row_off;
            }
#pragma unroll
            for (int i = 0; i < UT; ++i) {
                const int rr = i / S, s = s0 + i - rr * S;
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    o.a[i][m] = *reinterpret_cast<const float*>(
                        a_base + 4 * (gi * WC * 4 * RS + tap0 + i + m * 16 * WPITCH));
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    o.b[i][t] = *reinterpret_cast<const float*>(lds_bytes + (xa[t] + 4 * (rr * a.lds_pitch + s)));
            }
        };
        auto mfma_unit = [&](const Operands& o) {
#pragma unroll
            for (int i = 0; i < UT; ++i)
#pragma unroll
                for (int m = 0; m < MT; ++m)
#pragma unroll
                    for (int t = 0; t < NT; ++t)
                        if (TAIL && t == NT - 1) acc[m][t] = __builtin_amdgcn_mfma_f32_4x4x1f32(o.a[i][m], o.b[i][t], acc[m][t], 0, 0, 0);
                        else acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(o.a[i][m], o.b[i][t], acc[m][t], 0, 0, 0);
        };
        // Unit ui: read the operands of unit ui+1, move this unit's share of the staging slots
        // (write chunk ch+1 to the other copy, refill with chunk ch+2), multiply.
        auto unit = [&](auto uic) {
            constexpr int ui = decltype(uic)::value;
            Operands& cur = (ui & 1) ? o1 : o0;
            Operands& nxt = (ui & 1) ? o0 : o1;
            if constexpr (ui + 1 < U) load_unit(nxt, IntC<ui + 1>{});
            if constexpr (LW == 0) for_each_slot([&](auto kc) {
                if constexpr (decltype(kc)::value * UI / TS == ui) {
                    if constexpr (DMA) {
                        slot_fetch(kc, nxt_floats);  // chunk ch + DEPTH - 1 (past the last chunk: zeros, unused)
                    } else {
                        slot_store(kc, c0_regs, nxt_floats);
                        slot_load(kc, c0_load);
                    }
                }
            });
            mfma_unit(cur);
            interleave_with_mfma<UT * MT * NT>();
        };

        load_unit(o0, IntC<0>{});
        [&]<int... UIs>(std::integer_sequence<int, UIs...>) { (unit(IntC<UIs>{}), ...); }
        (std::make_integer_sequence<int, U>{});

        if constexpr (DMA && LW == 0) {
            before_fetch(ch + DEPTH);
            // this wave's part of chunk ch+1 is in LDS; after the last chunk nothing may still be on its way (the reduction
            // reuses the copies, and LDS that a load still writes must not be handed to another work-group)
            if (DEPTH == 2 || ch + 1 == nchunks) wait_loads(IntC<0>{});
            else wait_loads(IntC<(DEPTH - 2) * TS>{});
        }
        chunk_barrier();  // every wave is done reading this copy and writing the next one to fill
        ring_fill = ring_cur;
        ring_cur = ring_cur + 1 == DEPTH ? 0 : ring_cur + 1;
    }

    __builtin_amdgcn_s_setprio(0);

    // Waves that split the channels add their partial tiles through LDS, as a binary tree in a fixed
    // order (so results stay bitwise reproducible); the wc == 0 waves end up with the full sums.
    if constexpr (WC > 1) {
#pragma unroll
        for (int stride = WC / 2; stride >= 1; stride /= 2) {
            if (stride != WC / 2) __syncthreads();  // the previous round's partials are dead
            const int slot = ((wc - stride) * WP + wp) * WK + wk;
            f32x4* const part = smem4 + slot * (MT * NT * 64) + lane;
            if (wc >= stride && wc < 2 * stride) {
#pragma unroll
                for (int m = 0; m < MT; ++m)
#pragma unroll
                    for (int t = 0; t < NT; ++t) part[(m * NT + t) * 64] = acc[m][t];
            }
            __syncthreads();
            if (wc < stride) {
                const f32x4* const other = part + stride * (WP * WK * MT * NT * 64);
#pragma unroll
                for (int m = 0; m < MT; ++m)
#pragma unroll
                    for (int t = 0; t < NT; ++t) acc[m][t] += other[(m * NT + t) * 64];
            }
        }
        if (wc != 0) return;
    }

    // a4: lane (j, kq) holds output channels 4*kq..4*kq+3 of each tile for pixel j. The epilogue's
    // per-channel constants are fetched first and waited for once, so that no store has to wait for a load
    // that sits behind earlier stores in the in-order memory counter.
    float bk[MT][4];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            bk[m][v] = a.bias ? a.bias[min(k0 + (wk * MT + m) * 16 + 4 * kq + v, a.K - 1)] : 0.f;
    // Four-pixel tail: lane (c, quad, pixel) holds the sum over its one channel c of every 4-channel group, for output
    // channels 4*quad .. 4*quad+3 and the tail's pixel lane & 3. Adding the lanes 16 and 32 apart completes the sums (in
    // every lane; the c = 0 lanes store them).
    const int quad = (lane >> 2) & 3;
    float bt[TAIL ? MT : 1][4];
    if constexpr (TAIL) {
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float s = acc[m][NT - 1][v];
                s += __shfl_xor(s, 16, 64);
                s += __shfl_xor(s, 32, 64);
                acc[m][NT - 1][v] = s;
                bt[m][v] = a.bias ? a.bias[min(k0 + (wk * MT + m) * 16 + 4 * quad + v, a.K - 1)] : 0.f;
            }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    // Offsets in y of the lane's pixels (image n0 + dn, pixel pq of it); lanes past the end of the tile get -1.
    const int kpq = a.K * a.PQ;
    float* const y_tile = y_share + static_cast<size_t>(n0) * kpq;
    int yb[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const bool tail = TAIL && t == NT - 1;
        const int d = (wp * NT + t) * 16 + (tail ? (j & 3) : j);
        int pq = pq0 + d, dn = 0;
        const int r = pq - a.PQ;
        if (r >= 0) {
            const int m = small_div(r, a.inv_PQ);
            dn = 1 + m;
            pq = r - __mul24(m, a.PQ);  // (m > 0 only on maps smaller than the tile)
        }
        yb[t] = g0 + d < g_end && !(tail && lane >= 16) ? dn * kpq + pq : -1;
    }
    // Work-groups whose channel tile lies inside K (all but the last one along K) store without a test per channel.
    const bool whole_k = k0 + TK <= a.K;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (yb[t] < 0) continue;
            const bool tail = TAIL && t == NT - 1;
            const int kbase = k0 + (wk * MT + m) * 16 + 4 * (tail ? quad : kq);
            float* const yp = y_tile + static_cast<size_t>(kbase) * a.PQ + yb[t];
            if (whole_k) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    yp[static_cast<size_t>(v) * a.PQ] = finish_output(acc[m][t][v], tail ? bt[TAIL ? m : 0][v] : bk[m][v], a.relu);
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (kbase + v < a.K)
                        yp[static_cast<size_t>(v) * a.PQ] = finish_output(acc[m][t][v], tail ? bt[TAIL ? m : 0][v] : bk[m][v], a.relu);
            }
        }
    }
#endif
}

#ifndef TAP_R
#error "TAP_R, TAP_S and TAP_VARIANT must be defined by the build"
#endif

using KernFn = void (*)(const KernelArgs);

template <int VX, int VW, int DIV = 1, bool DMA = false, bool LOADER_WAVES = false, bool DEEP = false> static KernFn instance()
{
    constexpr TapVariant tv = kTapVariants[TAP_VARIANT];
    if constexpr (!tv.supports(TAP_R * TAP_S) || (VW == 1 && !tv.supports_scalar(TAP_R * TAP_S, VX))) {
        return nullptr;  // the filter block of this filter size does not fit the variant's registers
    } else if constexpr (DEEP) {
        constexpr int XS = (tv.xs_direct(VX) + DIV - 1) / DIV, WS = tv.wslots_direct(TAP_R * TAP_S);
        if constexpr (tv.deep_copies() == 0 || (tv.deep_copies() - 2) * (XS + WS) > 63) {
            return nullptr;
        } else {
            return conv_tap_mfma<TAP_R, TAP_S, tv.MT, tv.NT, tv.WK, tv.WP, tv.WC, tv.GPC, tv.occ, XS, WS, VX, VW, true, 0, tv.deep_copies(), tv.tail != 0>;
        }
    } else if constexpr (LOADER_WAVES) {
        constexpr int LW = tv.loader_waves();
        if constexpr (LW == 0) {
            return nullptr;
        } else {
            // the slots of the whole work-group, dealt to the loader threads
            constexpr int XS_ALL = (tv.xs_direct(VX) + DIV - 1) / DIV * tv.block();
            constexpr int WS_ALL = tv.wslots_direct(TAP_R * TAP_S) * tv.block();
            return conv_tap_mfma<TAP_R, TAP_S, tv.MT, tv.NT, tv.WK, tv.WP, tv.WC, tv.GPC, (tv.block() / 64 + LW + 3) / 4,
                                 (XS_ALL + 64 * LW - 1) / (64 * LW), (WS_ALL + 64 * LW - 1) / (64 * LW), VX, VW, true, LW, 2, tv.tail != 0>;
        }
    } else if constexpr (DMA) {
        return conv_tap_mfma<TAP_R, TAP_S, tv.MT, tv.NT, tv.WK, tv.WP, tv.WC, tv.GPC, tv.occ, (tv.xs_direct(VX) + DIV - 1) / DIV,
                             tv.wslots_direct(TAP_R * TAP_S), VX, VW, true, 0, 2, tv.tail != 0>;
    } else {
        return conv_tap_mfma<TAP_R, TAP_S, tv.MT, tv.NT, tv.WK, tv.WP, tv.WC, tv.GPC, tv.occ, (tv.xs(VX) + DIV - 1) / DIV,
                             tv.wslots(TAP_R * TAP_S, VW), VX, VW, false, 0, 2, tv.tail != 0>;
    }
}

// One exported launcher per translation unit, named by filter size and tile shape.
#define TAP_CAT2(a, b, c) launch_tap_##a##x##b##_v##c
#define TAP_CAT(a, b, c) TAP_CAT2(a, b, c)
hipError_t TAP_CAT(TAP_R, TAP_S, TAP_VARIANT)(int x_vec, int w_vec, int grid, int lds_bytes, hipStream_t stream,
                                              const KernelArgs& a)
{
    constexpr TapVariant tv = kTapVariants[TAP_VARIANT];
    const int div = tap_x_slot_divisor(tv, x_vec, w_vec, a.x_items, a.direct);
    KernFn fn = nullptr;
    int mode = -1;
    int block = tv.block();
    if (a.direct == 3 && w_vec == 4 && x_vec == 4) {
        fn = div == 2 ? instance<4, 4, 2, true, false, true>() : instance<4, 4, 1, true, false, true>();
        mode = div == 2 ? 20 : 19;
    } else if (a.direct == 3 && w_vec == 4 && x_vec == 1) {
        fn = div == 4   ? instance<1, 4, 4, true, false, true>()
             : div == 2 ? instance<1, 4, 2, true, false, true>()
                        : instance<1, 4, 1, true, false, true>();
        mode = div == 4 ? 23 : div == 2 ? 22 : 21;
    } else if (a.direct == 3) {
        return hipErrorInvalidValue;
    } else if (a.direct == 2 && w_vec == 4 && x_vec == 4) {
        fn = div == 2 ? instance<4, 4, 2, true, true>() : instance<4, 4, 1, true, true>();
        mode = div == 2 ? 15 : 14;
        block += 64 * tv.loader_waves();
    } else if (a.direct == 2 && w_vec == 4 && x_vec == 1) {
        fn = div == 4 ? instance<1, 4, 4, true, true>() : div == 2 ? instance<1, 4, 2, true, true>() : instance<1, 4, 1, true, true>();
        mode = div == 4 ? 18 : div == 2 ? 17 : 16;
        block += 64 * tv.loader_waves();
    } else if (a.direct == 2) {
        return hipErrorInvalidValue;
    } else if (a.direct && w_vec == 4 && x_vec == 4) {
        fn = div == 2 ? instance<4, 4, 2, true>() : instance<4, 4, 1, true>();
        mode = div == 2 ? 10 : 9;
    } else if (a.direct && w_vec == 4 && x_vec == 1) {
        fn = div == 4 ? instance<1, 4, 4, true>() : div == 2 ? instance<1, 4, 2, true>() : instance<1, 4, 1, true>();
        mode = div == 4 ? 13 : div == 2 ? 12 : 11;
    } else if (a.direct) {
        return hipErrorInvalidValue;
    } else if (w_vec == 4 && x_vec == 4) {
        fn = div == 2 ? instance<4, 4, 2>() : instance<4, 4>();
        mode = div == 2 ? 5 : 0;
    } else if (w_vec == 4 && x_vec == 2) {
        fn = div == 2 ? instance<2, 4, 2>() : instance<2, 4>();
        mode = div == 2 ? 8 : 1;
    } else if (w_vec == 4 && x_vec == 1) {
        fn = div == 4 ? instance<1, 4, 4>() : div == 2 ? instance<1, 4, 2>() : instance<1, 4>();
        mode = div == 4 ? 7 : div == 2 ? 6 : 2;
    } else if (w_vec == 1 && x_vec == 1) {
        fn = instance<1, 1>();
        mode = 3;
    } else if (w_vec == 1 && x_vec == 4) {
        fn = instance<4, 1>();
        mode = 4;
    }
    if (!fn) return hipErrorInvalidValue;
    // Kernels may use all 160 KB of a CU's LDS; the runtime wants to be told once per kernel (and device).
    static std::atomic<int> lds_allowed[24][kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) dev = 0;
    if (lds_bytes > 48 * 1024 && lds_allowed[mode][dev].load(std::memory_order_acquire) < lds_bytes) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        lds_allowed[mode][dev].store(160 * 1024, std::memory_order_release);
    }
    hipLaunchKernelGGL(fn, dim3(grid), dim3(block), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace convfwd
