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

template <int R, int S, int MT, int NT, int WK, int WP, int VX, int VW>
__global__ void __launch_bounds__(64 * WK * WP) conv_tap_mfma(const KernelArgs a)
{
    constexpr int BLOCK = 64 * WK * WP;
    constexpr int RS = R * S;
    constexpr int TK = 16 * MT * WK;
    constexpr int XS = kTapXSlots;
    constexpr int WS = kTapWSlots;

    extern __shared__ f32x4 smem4[];
    float* const xs = reinterpret_cast<float*>(smem4);
    const int xs_floats = a.chunk_c * a.lds_plane;
    float* const ws = xs + xs_floats;
    const int ws_floats = TK * a.w_pitch;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int j = lane & 15;   // pixel column of B / D, output-channel row of A
    const int kq = lane >> 4;  // channel within the 4-channel group (A, B); row group of D
    const int wk = wave % WK;
    const int wp = wave / WK;

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
        const int n4 = (xs_floats + ws_floats + 3) >> 2;
        for (int i = tid; i < n4; i += BLOCK) smem4[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // Per-lane pixel tables: LDS offset of the pixel's window origin, and offset of the pixel in y.
    int xb[NT], yb[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int g = g0 + (wp * NT + t) * 16 + j;
        const bool valid = g < g_end;
        const int gc = valid ? g : g_end - 1;
        const int n = gc / a.PQ;
        const int pq = gc - n * a.PQ;
        const int p = pq / a.Q;
        const int q = pq - p * a.Q;
        xb[t] = 4 * (kq * a.lds_plane + (n * a.Hp + p - V0) * a.lds_pitch + q + a.col_shift);  // bytes
        yb[t] = valid ? n * a.K * a.PQ + pq : -1;
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
            if (xl[i] >= 0 && c0 + (xl[i] >> 20) < a.C) xv[i].load(xc + xg[i]);
        }
        const int valid_len = min(a.chunk_c, a.C - c0) * RS;
        const float* wc = a.w + k0 * a.CRS + c0 * RS;
#pragma unroll
        for (int i = 0; i < WS; ++i) {
            wv[i].zero();
            if (wpk[i] >= 0) {
                const int kl = wpk[i] >> 16, ev = wpk[i] & 0xffff;
                if (ev < valid_len) wv[i].load(wc + kl * a.CRS + ev);
            }
        }
    };
    auto store_chunk = [&]() {
#pragma unroll
        for (int i = 0; i < XS; ++i)
            if (xl[i] >= 0) xv[i].store16(xs + (xl[i] & 0xfffff));
#pragma unroll
        for (int i = 0; i < WS; ++i)
            if (wpk[i] >= 0) {
                const int kl = wpk[i] >> 16, ev = wpk[i] & 0xffff;
                wv[i].store8(ws + kl * a.w_pitch + ev);  // rows are 8-byte aligned (pitch = 2 mod 4)
            }
    };

    f32x4 acc[MT][NT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[m][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int arow = 4 * (xs_floats + (wk * MT * 16 + j) * a.w_pitch + kq * RS);  // bytes from the LDS base

    // A pipeline unit is RU filter rows of one 4-channel group: UT taps, UT*MT*NT matrix instructions.
    constexpr int RU = (MT * NT >= 6) ? 1 : R;
    constexpr int UNITS = R / RU;
    constexpr int UT = RU * S;
    struct Operands {
        float a[UT][MT];
        float b[UT][NT];
    };
    auto load_unit = [&](Operands& o, int u) {
        const int cs = u / UNITS;
        const int r0 = (u - cs * UNITS) * RU;
        const char* base = reinterpret_cast<const char*>(xs);
        const int woff = 4 * (cs * 4 * RS + r0 * S);                         // wave-uniform byte offsets
        const int xoff = 4 * (cs * 4 * a.lds_plane + r0 * a.lds_pitch);
#pragma unroll
        for (int rr = 0; rr < RU; ++rr)
#pragma unroll
            for (int s = 0; s < S; ++s) {
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    o.a[rr * S + s][m] = *reinterpret_cast<const float*>(
                        base + (arow + woff + 4 * (m * 16 * a.w_pitch + rr * S + s)));
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    o.b[rr * S + s][t] = *reinterpret_cast<const float*>(
                        base + (xb[t] + xoff + 4 * (rr * a.lds_pitch + s)));
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
    store_chunk();
    __syncthreads();

    for (int ch = 0; ch < a.nchunks; ++ch) {
        const int c0 = ch * a.chunk_c;
        const bool more = ch + 1 < a.nchunks;
        if (more) load_chunk(c0 + a.chunk_c);

        // a3, software pipelined: the LDS reads of unit u+1 are issued before the MFMAs of unit u, so
        // a wave that has its SIMD to itself never waits on LDS latency between matrix instructions.
        const int groups = (min(a.chunk_c, a.C - c0) + 3) >> 2;
        const int units = groups * UNITS;
        Operands o0, o1;
        load_unit(o0, 0);
        int u = 0;
        for (; u + 2 <= units; u += 2) {
            load_unit(o1, u + 1);
            mfma_unit(o0);
            interleave_reads_with_mfma<UT * MT * NT>();
            load_unit(o0, min(u + 2, units - 1));
            mfma_unit(o1);
            interleave_reads_with_mfma<UT * MT * NT>();
        }
        if (u < units) mfma_unit(o0);

        if (more) {
            __syncthreads();  // every wave has finished reading this chunk
            store_chunk();
            __syncthreads();
        }
    }

    // a4: lane (j, kq) holds output channels 4*kq..4*kq+3 of each tile for pixel j.
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int kbase = k0 + (wk * MT + m) * 16 + 4 * kq;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (yb[t] < 0) continue;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (kbase + v < a.K) a.y[yb[t] + (kbase + v) * a.PQ] = acc[m][t][v];
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
    return conv_tap_mfma<TAP_R, TAP_S, tv.MT, tv.NT, tv.WK, tv.WP, VX, VW>;
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
