// Tap-family kernel: direct convolution with the input halo tile and a filter block in LDS,
// reduced over (channel, tap) with full-precision fp32 MFMA (v_mfma_f32_16x16x4_f32).
//
// One work-group owns TK output channels x tile_pix output pixels, the pixels counted in
// flattened (n, p, q) order, and loops over the input channels in chunks:
//   a1  halo tile: the rows of the zero-padded, vertically stacked images that the pixel range
//       touches are copied HBM -> registers -> LDS with dwordx4 (dwordx2 / dword when the row
//       length forbids) loads; padding cells are zeroed once and never written again;
//   a2  filter block: w[k0..k0+TK, c0..c0+chunk_c, :, :] is chunk_c*R*S contiguous floats per
//       output channel and is copied the same way;
//   a3  for every (4-channel group, r, s): A = filters [16 k x 4 c], B = inputs [4 c x 16 px] read
//       from the halo tile at the tap's offset, acc += A*B on the matrix cores; each input element
//       in LDS is reused by the R*S taps and by all TK channels, each filter element by all pixels
//       (the two reuse levels of Section 3);
//   a4  accumulators -> y in NCHW, no second pass and no workspace (the per-tap partial matrices
//       of the two-stage scheme of Section 3 never leave the registers).
// The next chunk's global loads are issued before the current chunk's MFMA loop and written to
// LDS after it, so HBM/L2 latency overlaps the arithmetic.
//
// Compiled once per (filter size, tile shape): TAP_R, TAP_S, TAP_VARIANT come from the build.
#include "conv_internal.h"

namespace convfwd {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

template <int V> struct Vec;
template <> struct Vec<4> {
    f32x4 v;
    __device__ void load(const float* p) { v = *reinterpret_cast<const f32x4*>(p); }
    __device__ void zero() { v = f32x4{0.f, 0.f, 0.f, 0.f}; }
    __device__ void store16(float* p) const { *reinterpret_cast<f32x4*>(p) = v; }
    __device__ void store8(float* p) const {
        *reinterpret_cast<f32x2*>(p) = f32x2{v.x, v.y};
        *reinterpret_cast<f32x2*>(p + 2) = f32x2{v.z, v.w};
    }
};
template <> struct Vec<2> {
    f32x2 v;
    __device__ void load(const float* p) { v = *reinterpret_cast<const f32x2*>(p); }
    __device__ void zero() { v = f32x2{0.f, 0.f}; }
    __device__ void store16(float* p) const { *reinterpret_cast<f32x2*>(p) = v; }
    __device__ void store8(float* p) const { *reinterpret_cast<f32x2*>(p) = v; }
};
template <> struct Vec<1> {
    float v;
    __device__ void load(const float* p) { v = *p; }
    __device__ void zero() { v = 0.f; }
    __device__ void store16(float* p) const { *p = v; }
    __device__ void store8(float* p) const { *p = v; }
};

// Taps per pipeline unit: the shortest of {1, S, R*S} that keeps at least 24 matrix instructions
// between a read and its use, stepped down again if two operand sets would not fit ~96 registers (~64 with two waves per SIMD).
constexpr int unit_taps(int S, int RS, int MT, int NT, int OCC)
{
    const int cand[3] = {1, S, RS};
    int pick = 2;
    for (int i = 2; i >= 0; --i)
        if (cand[i] * MT * NT >= 24) pick = i;
    while (pick > 0 && 2 * cand[pick] * (MT + NT) > (OCC > 1 ? 64 : 96)) --pick;
    return cand[pick];
}

// Scheduling directive for the code since the previous barrier: issue the matrix instructions in
// order and slip (up to) two address computations and two LDS reads in front of each, then fence so nothing moves across.
template <int N_MFMA> __device__ __forceinline__ void interleave_reads_with_mfma()
{
#pragma unroll
    for (int i = 0; i < N_MFMA; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);  // VALU (addresses of the reads)
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // DS read
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
    }
    __builtin_amdgcn_sched_barrier(0);
}

template <int R, int S, int MT, int NT, int WK, int WP, int WC, int OCC, int XS, int WS, bool DB, int VX, int VW>
__global__ void __launch_bounds__(64 * WK * WP * WC, OCC) conv_tap_mfma(const KernelArgs a)
{
    static_assert(WC == 1 || WC == 2 || WC == 4, "the cross-wave reduction is a binary tree");
    constexpr int BLOCK = 64 * WK * WP * WC;
    constexpr int RS = R * S;
    constexpr int TK = 16 * MT * WK;

    extern __shared__ f32x4 smem4[];
    float* const xs = reinterpret_cast<float*>(smem4);
    const int xs_floats = a.chunk_c * a.lds_plane;
    float* const ws = xs + xs_floats;
    const int ws_floats = TK * a.w_pitch;
    // With DB the staging area exists twice: chunk ch is read from copy ch&1 while chunk ch+1 is
    // written to the other copy in the middle of the MAC loop, and one barrier per chunk suffices.
    const int buf_floats = (xs_floats + ws_floats + 3) & ~3;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps wk/wp/wc in SGPRs
    const int j = lane & 15;   // pixel column of B / D, output-channel row of A
    const int kq = lane >> 4;  // channel within the 4-channel group (A, B); row group of D
    const int wk = wave % WK;
    const int wp = (wave / WK) % WP;
    const int wc = wave / (WK * WP);  // which share of the channel groups this wave reduces

    // Work-groups are dealt round-robin to the 8 XCDs; renumber them so that each XCD (one L2)
    // gets a contiguous run of tiles: neighbours share the pixel tile and walk the K tiles.
    int L;
    {
        const int nb = gridDim.x, b = blockIdx.x;
        const int per = nb >> 3, rem = nb & 7, xcd = b & 7;
        L = xcd * per + (xcd < rem ? xcd : rem) + (b >> 3);
    }
    const int ptile = L / a.ktiles;
    const int ktile = L - ptile * a.ktiles;
    const int k0 = ktile * TK;
    const int g0 = ptile * a.tile_pix;
    const int g_end = min(g0 + a.tile_pix, a.total_pix);
    const int n0 = g0 / a.PQ;
    const int V0 = n0 * a.Hp + (g0 - n0 * a.PQ) / a.Q;  // first stacked padded row held in LDS

    // Zero the whole LDS allocation once: padding cells, rows past the batch and output
    // channels past K then stay zero for the whole kernel.
    {
        const int n4 = (DB ? 2 : 1) * (buf_floats >> 2);
        for (int i = tid; i < n4; i += BLOCK) smem4[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // Per-lane pixel table: byte offset in LDS of the origin of the pixel's window (lanes past the
    // end of the tile read the tile's last pixel and are masked at the store).
    int xb[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int gc = min(g0 + (wp * NT + t) * 16 + j, g_end - 1);
        const int n = gc / a.PQ;
        const int pq = gc - n * a.PQ;
        const int p = pq / a.Q;
        const int q = pq - p * a.Q;
        xb[t] = 4 * (kq * a.lds_plane + (n * a.Hp + p - V0) * a.lds_pitch + q + a.col_shift);
    }

    // Halo-tile load slots: global offset (channel 0 of the chunk) and packed LDS offset | channel<<20.
    int xg[XS], xl[XS];
    {
        const int XV = a.W / VX;
        const int per_c = a.lds_rows * XV;
#pragma unroll
        for (int i = 0; i < XS; ++i) {
            const int e = tid + i * BLOCK;
            xg[i] = 0;
            xl[i] = -1;
            if (e < a.x_items) {
                const int c_l = e / per_c;
                const int rem = e - c_l * per_c;
                const int row = rem / XV;
                const int cv = rem - row * XV;
                const int v = V0 + row;
                const int n = v / a.Hp;
                const int h = v - n * a.Hp - a.pad_h;
                if (n < a.N && h >= 0 && h < a.H) {
                    xg[i] = ((n * a.C + c_l) * a.H + h) * a.W + cv * VX;
                    xl[i] = (c_l * a.lds_plane + row * a.lds_pitch + a.col_shift + a.pad_w + cv * VX) | (c_l << 20);
                }
            }
        }
    }
    // Filter-block load slots: (local output channel << 16) | element offset inside the chunk's slice.
    int wpk[WS];
    {
        const int WV = a.chunk_c * RS / VW;
#pragma unroll
        for (int i = 0; i < WS; ++i) {
            const int e = tid + i * BLOCK;
            wpk[i] = -1;
            if (e < a.w_items) {
                const int kl = e / WV;
                const int ev = (e - kl * WV) * VW;
                if (k0 + kl < a.K) wpk[i] = (kl << 16) | ev;
            }
        }
    }

    Vec<VX> xv[XS];
    Vec<VW> wv[WS];

    auto load_chunk = [&](int c0) {
        const float* xc = a.x + c0 * a.HW;
#pragma unroll
        for (int i = 0; i < XS; ++i) {
            xv[i].zero();
            if (xl[i] >= 0 && c0 + (xl[i] >> 20) < a.C) xv[i].load(xc + static_cast<unsigned>(xg[i]));
        }
        const int valid_len = min(a.chunk_c, a.C - c0) * RS;
        const float* wc = a.w + k0 * a.CRS + c0 * RS;
#pragma unroll
        for (int i = 0; i < WS; ++i) {
            wv[i].zero();
            if (wpk[i] >= 0) {
                const int kl = wpk[i] >> 16, ev = wpk[i] & 0xffff;
                if (ev < valid_len) wv[i].load(wc + static_cast<unsigned>(kl * a.CRS + ev));
            }
        }
    };
    auto store_chunk = [&](int buf_off) {
#pragma unroll
        for (int i = 0; i < XS; ++i)
            if (xl[i] >= 0) xv[i].store16(xs + buf_off + (xl[i] & 0xfffff));
#pragma unroll
        for (int i = 0; i < WS; ++i)
            if (wpk[i] >= 0) {
                const int kl = wpk[i] >> 16, ev = wpk[i] & 0xffff;
                wv[i].store8(ws + buf_off + kl * a.w_pitch + ev);  // rows are 8-byte aligned (pitch = 2 mod 4)
            }
    };

    f32x4 acc[MT][NT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[m][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int arow = 4 * (xs_floats + (wk * MT * 16 + j) * a.w_pitch + kq * RS);  // bytes from the LDS base

    // A pipeline unit is UT consecutive taps of one 4-channel group (UT*MT*NT matrix instructions):
    // one tap when the wave owns many tiles, a filter row, or the whole filter when it owns few.
    constexpr int UT = unit_taps(S, RS, MT, NT, OCC);
    constexpr int UNITS = RS / UT;
    struct Operands {
        float a[UT][MT];
        float b[UT][NT];
    };
    int cur_bytes = 0;  // byte offset of the staging copy being read
    auto load_unit = [&](Operands& o, int u) {
        const int gi = u / UNITS;
        const int cs = wc + WC * gi;  // waves with different wc take the channel groups round-robin
        const int tap0 = (u - gi * UNITS) * UT;
        const int r0 = tap0 / S, s0 = tap0 - r0 * S;  // s0 is 0 unless the unit is a single tap
        const char* base = reinterpret_cast<const char*>(xs) + cur_bytes;
        const int woff = 4 * (cs * 4 * RS + tap0);  // wave-uniform byte offsets
        const int xoff = 4 * (cs * 4 * a.lds_plane + r0 * a.lds_pitch + s0);
#pragma unroll
        for (int i = 0; i < UT; ++i) {
            const int rr = i / S, s = i - rr * S;
#pragma unroll
            for (int m = 0; m < MT; ++m)
                o.a[i][m] = *reinterpret_cast<const float*>(base + (arow + woff + 4 * (m * 16 * a.w_pitch + i)));
#pragma unroll
            for (int t = 0; t < NT; ++t)
                o.b[i][t] = *reinterpret_cast<const float*>(base + (xb[t] + xoff + 4 * (rr * a.lds_pitch + s)));
        }
    };
    auto mfma_unit = [&](const Operands& o) {
#pragma unroll
        for (int i = 0; i < UT; ++i)
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(o.a[i][m], o.b[i][t], acc[m][t], 0, 0, 0);
    };

    load_chunk(0);
    __syncthreads();  // zero fill complete before any data lands
    store_chunk(0);
    __syncthreads();

    // A wave stalls while it issues its burst of global loads (the CU's address path takes them at
    // 64 B/clk) or LDS stores, and its own matrix instructions do not overlap that. Waves that share
    // a SIMD therefore do both at different points of their MAC loops: one of the two always has
    // matrix work to issue.
    const int stagger = (wave >> 2) & 1;

    for (int ch = 0; ch < a.nchunks; ++ch) {
        const int c0 = ch * a.chunk_c;
#ifdef EXP_NO_RELOAD
        const bool more = false;
#else
        const bool more = ch + 1 < a.nchunks;
#endif
        const int next_off = DB ? ((ch + 1) & 1) * buf_floats : 0;
        cur_bytes = DB ? (ch & 1) * buf_floats * 4 : 0;
        // a3, software pipelined: the LDS reads of unit u+1 are issued before the MFMAs of unit u. A
        // wave's own loads and address arithmetic do not overlap its matrix instructions, a second wave
        // on the SIMD does; hence few reads per MFMA and, where registers allow, two waves per SIMD.
        const int groups = (min(a.chunk_c, a.C - c0) + 3) >> 2;
        const int units = groups > wc ? (groups - wc + WC - 1) / WC * UNITS : 0;
        const int store_at = DB && more ? ((units * (2 + stagger)) >> 2) & ~1 : -1;
        const int load_at = DB && units >= 8 ? 2 * stagger : 0;
        bool stored = false;
        if (more && load_at == 0) load_chunk(c0 + a.chunk_c);
        Operands o0, o1;
        load_unit(o0, 0);  // in bounds even when this wave has no group in a ragged last chunk
        int u = 0;
        for (; u + 2 <= units; u += 2) {
            if (more && load_at != 0 && u == load_at) load_chunk(c0 + a.chunk_c);
            if (u == store_at) {
                store_chunk(next_off);
                stored = true;
            }
#ifdef EXP_NO_LDS_READ
            if (u == 0) load_unit(o1, u + 1);
            mfma_unit(o0);
            __builtin_amdgcn_sched_barrier(0);
            mfma_unit(o1);
            __builtin_amdgcn_sched_barrier(0);
#else
            load_unit(o1, u + 1);
            mfma_unit(o0);
            interleave_reads_with_mfma<UT * MT * NT>();
            load_unit(o0, min(u + 2, units - 1));
            mfma_unit(o1);
            interleave_reads_with_mfma<UT * MT * NT>();
#endif
        }
        if (u < units) mfma_unit(o0);

        if (more) {
            if (DB) {
                if (!stored) store_chunk(next_off);
                __syncthreads();  // all waves are done reading this copy and writing the other
            } else {
                __syncthreads();  // every wave has finished reading this chunk
                store_chunk(0);
                __syncthreads();
            }
        }
    }

    // Waves that split the channels add their partial tiles through LDS, as a binary tree in a fixed
    // order (so results stay bitwise reproducible); the wc == 0 waves end up with the full sums.
    if constexpr (WC > 1) {
#pragma unroll
        for (int stride = WC / 2; stride >= 1; stride /= 2) {
            __syncthreads();  // the staging buffers (first pass) or the previous round's partials are dead
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

    // a4: lane (j, kq) holds output channels 4*kq..4*kq+3 of each tile for pixel j.
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int kbase = k0 + (wk * MT + m) * 16 + 4 * kq;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int g = g0 + (wp * NT + t) * 16 + j;
            if (g >= g_end) continue;
            const int n = g / a.PQ;
            const int yb = n * a.K * a.PQ + (g - n * a.PQ);
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (kbase + v < a.K) a.y[yb + (kbase + v) * a.PQ] = acc[m][t][v];
        }
    }
}

#ifndef TAP_R
#error "TAP_R, TAP_S and TAP_VARIANT must be defined by the build"
#endif

using KernFn = void (*)(const KernelArgs);

template <int VX, int VW> static KernFn instance()
{
    constexpr TapVariant tv = kTapVariants[TAP_VARIANT];
    return conv_tap_mfma<TAP_R, TAP_S, tv.MT, tv.NT, tv.WK, tv.WP, tv.WC, tv.occ, tv.xslots, tv.wslots, tv.dbuf, VX, VW>;
}

// One exported launcher per translation unit, named by filter size and tile shape.
#define TAP_CAT2(a, b, c) launch_tap_##a##x##b##_v##c
#define TAP_CAT(a, b, c) TAP_CAT2(a, b, c)
hipError_t TAP_CAT(TAP_R, TAP_S, TAP_VARIANT)(int x_vec, int w_vec, int grid, int lds_bytes, hipStream_t stream,
                                              const KernelArgs& a)
{
    KernFn fn = nullptr;
    if (w_vec == 4) {
        fn = x_vec == 4 ? instance<4, 4>() : x_vec == 2 ? instance<2, 4>() : x_vec == 1 ? instance<1, 4>() : nullptr;
    } else if (w_vec == 1 && x_vec == 1) {
        fn = instance<1, 1>();
    }
    if (!fn) return hipErrorInvalidValue;
    if (lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
    }
    constexpr TapVariant tv = kTapVariants[TAP_VARIANT];
    hipLaunchKernelGGL(fn, dim3(grid), dim3(tv.block()), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace convfwd
