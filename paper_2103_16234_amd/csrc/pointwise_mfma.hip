// Pointwise-family kernel: 1x1 filters without padding. For one image the layer is the matrix
// product y[K x HW] = w[K x C] * x[C x HW] (Section 3, last paragraph: with a 1x1 filter the first
// stage already yields the output), so nothing is reused across taps and the input is streamed
//   HBM -> registers -> fp32 MFMA
// without touching LDS: a lane's dwordx4 load of four consecutive pixels of one channel is, element by
// element, the B operand of four 16-pixel MFMA tiles (tile t holds pixels 4j+t), and a lane's dwordx4
// load of four consecutive input channels of one filter is the A operand of four successive MFMA steps
// (the channel <-> step assignment is a free permutation of the reduction as long as A and B agree).
// Outputs leave as dwordx4 stores of four consecutive pixels. Both tensors are read exactly once per
// work-group column; all loads of a wave are in flight together (one HBM round trip for small layers).
//
// A work-group is WC waves that share 16*MT output channels x 64 pixels of one image and split the
// input channels in steps of 16; their partial tiles are added through LDS in a fixed tree order.
#include "conv_internal.h"

namespace convfwd {

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int MT, int WC, int PD>
__global__ void __launch_bounds__(64 * WC) conv_pointwise_mfma(const KernelArgs a)
{
    static_assert((WC & (WC - 1)) == 0, "the cross-wave reduction is a binary tree");
    extern __shared__ f32x4 smem4[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wc = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15;
    const int kq = lane >> 4;

    // XCD-aware renumbering (see the tap kernel): neighbours on one L2 share the pixel tile.
    int L;
    {
        const int nb = gridDim.x, b = blockIdx.x;
        const int per = nb >> 3, rem = nb & 7, xcd = b & 7;
        L = xcd * per + (xcd < rem ? xcd : rem) + (b >> 3);
    }
    const int rest = a.div_ktiles.div(L);
    const int ktile = L - rest * a.ktiles;
    const int n = a.div_ptiles.div(rest);
    const int pt = rest - n * a.ptiles;
    const int k0 = ktile * (16 * MT);
    const int px = pt * 64 + 4 * j;
    const bool pvalid = px < a.HW;  // HW is a multiple of 4: the lane's four pixels are valid together

    const float* const xlane = a.x + n * a.C * a.HW + px;
    const float* wlane[MT];
    bool kvalid[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int k = k0 + 16 * m + j;
        kvalid[m] = k < a.K;
        wlane[m] = a.w + (kvalid[m] ? k : 0) * a.C + 4 * kq;
    }

    const int nsteps = (a.C + 15) >> 4;                         // steps of 16 input channels
    const int mine = nsteps > wc ? (nsteps - wc + WC - 1) / WC : 0;  // this wave takes steps wc, wc+WC, ...

    f32x4 xr[PD][4];
    f32x4 wr[PD][MT];
    auto load_step = [&](int slot, int i) {
        const int c = 16 * (wc + WC * i) + 4 * kq;  // this lane's four channels of the step: c .. c+3
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            xr[slot][e] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (pvalid && c + e < a.C) xr[slot][e] = *reinterpret_cast<const f32x4*>(xlane + (c + e) * a.HW);
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            wr[slot][m] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (kvalid[m] && c < a.C) wr[slot][m] = *reinterpret_cast<const f32x4*>(wlane[m] + (c - 4 * kq));
        }
    };

    f32x4 acc[MT][4];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[m][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto mfma_step = [&](int slot) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wr[slot][m][e], xr[slot][e][t], acc[m][t], 0, 0, 0);
    };

#pragma unroll
    for (int s = 0; s < PD; ++s)
        if (s < mine) load_step(s, s);
    for (int i = 0; i < mine; i += PD) {
#pragma unroll
        for (int s = 0; s < PD; ++s) {
            if (i + s < mine) {
                mfma_step(s);
                if (i + s + PD < mine) load_step(s, i + s + PD);
            }
        }
    }

    if constexpr (WC > 1) {
#pragma unroll
        for (int stride = WC / 2; stride >= 1; stride /= 2) {
            if (stride != WC / 2) __syncthreads();
            f32x4* const part = smem4 + (wc - stride) * (MT * 4 * 64) + lane;
            if (wc >= stride && wc < 2 * stride) {
#pragma unroll
                for (int m = 0; m < MT; ++m)
#pragma unroll
                    for (int t = 0; t < 4; ++t) part[(m * 4 + t) * 64] = acc[m][t];
            }
            __syncthreads();
            if (wc < stride) {
                const f32x4* const other = part + stride * (MT * 4 * 64);
#pragma unroll
                for (int m = 0; m < MT; ++m)
#pragma unroll
                    for (int t = 0; t < 4; ++t) acc[m][t] += other[(m * 4 + t) * 64];
            }
        }
        if (wc != 0) return;
    }

    // lane (j, kq) holds output channels 4*kq + v of tile m for pixels 4j .. 4j+3 (one per pixel tile)
    if (!pvalid) return;
    float* const ylane = a.y + n * a.K * a.HW + px;
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int k = k0 + 16 * m + 4 * kq + v;
            if (k < a.K)
                *reinterpret_cast<f32x4*>(ylane + k * a.HW) = f32x4{acc[m][0][v], acc[m][1][v], acc[m][2][v], acc[m][3][v]};
        }
}

using KernFn = void (*)(const KernelArgs);

template <int V> static KernFn pointwise_instance()
{
    constexpr PointwiseVariant pv = kPointwiseVariants[V];
    return conv_pointwise_mfma<pv.MT, pv.WC, (pv.WC * pv.MT >= 32 ? 2 : 4)>;  // 1024 threads leave 128 registers
}

hipError_t launch_pointwise(int variant, int grid, int lds_bytes, hipStream_t stream, const KernelArgs& a)
{
    static_assert(kNumPointwiseVariants == 8, "update the table below");
    static const KernFn table[kNumPointwiseVariants] = {
        pointwise_instance<0>(), pointwise_instance<1>(), pointwise_instance<2>(), pointwise_instance<3>(),
        pointwise_instance<4>(), pointwise_instance<5>(), pointwise_instance<6>(), pointwise_instance<7>()};
    if (variant < 0 || variant >= kNumPointwiseVariants) return hipErrorInvalidValue;
    hipLaunchKernelGGL(table[variant], dim3(grid), dim3(kPointwiseVariants[variant].block()), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace convfwd
