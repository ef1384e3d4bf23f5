// Pointwise-family kernel: 1x1 filters without padding. For one image the layer is the matrix
// product y[K x HW] = w[K x C] * x[C x HW] (Section 3, last paragraph: with a 1x1 filter the first
// stage already yields the output), so nothing is reused across taps and the input is streamed
//   HBM -> registers -> fp32 MFMA
// without touching LDS: a lane's dwordx4 load of four consecutive pixels of one channel is, element by
// element, the B operand of four 16-pixel MFMA tiles (tile t holds pixels 4j+t), and a lane's dwordx4
// load of four consecutive input channels of one filter is the A operand of four successive MFMA steps
// (the channel <-> step assignment is a free permutation of the reduction as long as A and B agree).
// Outputs leave as dwordx4 stores of four consecutive pixels. Both tensors are read exactly once per
// work-group column; two or four 16-channel steps of loads per wave are in flight at any time.
//
// A work-group is WC x WP waves on 16*MT output channels x WP*64 contiguous pixels of one image: the WP
// waves of a channel share take neighbouring 64-pixel runs (longer contiguous reads per channel row),
// the WC shares split the input channels in steps of 16 and add their partial tiles through LDS in a
// fixed tree order.
#include "conv_internal.h"

#include <utility>

namespace convfwd {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// MASK: some (wave, step) pair needs its filters zeroed: C is not a multiple of 16, or the steps do
// not divide evenly into pairs per wave. Loads are never predicated (addresses are clamped to valid
// elements instead), so the compiler keeps all of them in flight; masking happens just before the MFMAs.
// VEC = 4: H*W is a multiple of 4 and x, y are 16-byte aligned, a lane moves its four pixels as one
// dwordx4. VEC = 1: any H*W and alignment (7x7, 13x13, 27x27 maps), the four pixels move as four dwords.
// PD: 16-channel steps a wave keeps in flight (every wave runs a multiple of PD steps).
template <int MT, int WC, int WP, int PD, bool MASK, int VEC>
__global__ void __launch_bounds__(64 * WC * WP) conv_pointwise_mfma(const KernelArgs a)
{
    static_assert((WC & (WC - 1)) == 0, "the cross-wave reduction is a binary tree");
    extern __shared__ f32x4 smem4[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wp = wave % WP;  // which 64-pixel run of the work-group's WP*64 contiguous pixels
    const int wc = wave / WP;  // which share of the input channels
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
    // The lane's pixel of MFMA tile t: 4j + t when pixels move as dwordx4 (the lane owns four consecutive
    // pixels), 16t + j when they move as dwords (each load then reads 16 consecutive pixels per channel).
    const int px = (pt * WP + wp) * 64 + (VEC == 4 ? 4 * j : j);
    constexpr int PSTEP = VEC == 4 ? 1 : 16;
    const bool pvalid = px < a.HW;  // with VEC = 4 the lane's four pixels are valid together

    const float* const ximg = a.x + n * a.C * a.HW;
    const float* const xlane = ximg + (VEC == 4 ? min(px, a.HW - 4) : 0);
    int pxe[4];  // VEC = 1: the lane's pixels, clamped into the image
#pragma unroll
    for (int t = 0; t < 4; ++t) pxe[t] = min(px + PSTEP * t, a.HW - 1);
    const float* wlane[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) wlane[m] = a.w + min(k0 + 16 * m + j, a.K - 1) * a.C;

    // Steps of 16 input channels; wave wc takes steps wc, wc+WC, ...; every wave runs the same
    // multiple of PD steps (steps past the end are dummies with zeroed filters).
    const int nsteps = (a.C + 15) >> 4;
    const int mine = (((nsteps + WC - 1) / WC) + PD - 1) / PD * PD;

    f32x4 xr[PD][4];
    f32x4 wr[PD][MT];
    bool keep[PD];
    auto load_step = [&](auto slotc, int i) {
        constexpr int slot = decltype(slotc)::value;
        const int c_true = 16 * (wc + WC * i) + 4 * kq;  // this lane's four channels of the step
        const int c = MASK ? min(c_true, a.C - 4) : c_true;
        keep[slot] = c_true < a.C;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if constexpr (VEC == 4) {
                xr[slot][e] = *reinterpret_cast<const f32x4*>(xlane + (c + e) * a.HW);
            } else {
                const float* const row = xlane + (c + e) * a.HW;
                xr[slot][e] = f32x4{row[pxe[0]], row[pxe[1]], row[pxe[2]], row[pxe[3]]};
            }
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) wr[slot][m] = *reinterpret_cast<const f32x4*>(wlane[m] + c);
    };

    f32x4 acc[MT][4];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[m][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto mfma_step = [&](auto slotc) {
        constexpr int slot = decltype(slotc)::value;
        f32x4 wv[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) wv[m] = (!MASK || keep[slot]) ? wr[slot][m] : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[m][e], xr[slot][e][t], acc[m][t], 0, 0, 0);
    };

    auto for_each_slot = [&](auto&& f) {
        [&]<int... Ss>(std::integer_sequence<int, Ss...>) { (f(std::integral_constant<int, Ss>{}), ...); }
        (std::make_integer_sequence<int, PD>{});
    };
    for_each_slot([&](auto sc) { load_step(sc, decltype(sc)::value); });
    for (int i = 0; i < mine; i += PD) {
        const bool more = i + PD < mine;
        for_each_slot([&](auto sc) {
            mfma_step(sc);
            if (more) load_step(sc, i + PD + decltype(sc)::value);
        });
    }

    if constexpr (WC > 1) {
#pragma unroll
        for (int stride = WC / 2; stride >= 1; stride /= 2) {
            if (stride != WC / 2) __syncthreads();
            f32x4* const part = smem4 + ((wc - stride) * WP + wp) * (MT * 4 * 64) + lane;
            if (wc >= stride && wc < 2 * stride) {
#pragma unroll
                for (int m = 0; m < MT; ++m)
#pragma unroll
                    for (int t = 0; t < 4; ++t) part[(m * 4 + t) * 64] = acc[m][t];
            }
            __syncthreads();
            if (wc < stride) {
                const f32x4* const other = part + stride * (WP * MT * 4 * 64);
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
    // the epilogue's per-channel constants are fetched first and waited for once: a load between the stores
    // would make every later store wait for the earlier ones (one in-order counter for loads and stores)
    float bias_k[MT][4];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int v = 0; v < 4; ++v) bias_k[m][v] = a.bias ? a.bias[min(k0 + 16 * m + 4 * kq + v, a.K - 1)] : 0.f;
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    float* const ylane = a.y + n * a.K * a.HW + px;
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int k = k0 + 16 * m + 4 * kq + v;
            if (k >= a.K) continue;
            const float bk = bias_k[m][v];
            if constexpr (VEC == 4) {
                // whole 16-byte pieces of lines nothing here reads back: streaming stores (5-15 % on the large maps)
                __builtin_nontemporal_store(
                    f32x4{finish_output(acc[m][0][v], bk, a.relu), finish_output(acc[m][1][v], bk, a.relu),
                          finish_output(acc[m][2][v], bk, a.relu), finish_output(acc[m][3][v], bk, a.relu)},
                    reinterpret_cast<f32x4*>(ylane + k * a.HW));
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    if (px + PSTEP * t < a.HW) ylane[k * a.HW + PSTEP * t] = finish_output(acc[m][t][v], bk, a.relu);
            }
        }
}

using KernFn = void (*)(const KernelArgs);

template <int V, bool MASK, int VEC> static KernFn pointwise_instance()
{
    constexpr PointwiseVariant pv = kPointwiseVariants[V];
    return conv_pointwise_mfma<pv.MT, pv.WC, pv.WP, pv.depth(), MASK, VEC>;
}

hipError_t launch_pointwise(int variant, int x_vec, int grid, int lds_bytes, hipStream_t stream, const KernelArgs& a)
{
#define PW_PLAIN4(v) pointwise_instance<v, false, 4>(),
#define PW_MASKED4(v) pointwise_instance<v, true, 4>(),
#define PW_PLAIN1(v) pointwise_instance<v, false, 1>(),
#define PW_MASKED1(v) pointwise_instance<v, true, 1>(),
    static const KernFn plain4[kNumPointwiseVariants] = {POINTWISE_VARIANT_LIST(PW_PLAIN4)};
    static const KernFn masked4[kNumPointwiseVariants] = {POINTWISE_VARIANT_LIST(PW_MASKED4)};
    static const KernFn plain1[kNumPointwiseVariants] = {POINTWISE_VARIANT_LIST(PW_PLAIN1)};
    static const KernFn masked1[kNumPointwiseVariants] = {POINTWISE_VARIANT_LIST(PW_MASKED1)};
    if (variant < 0 || variant >= kNumPointwiseVariants) return hipErrorInvalidValue;
    // no masking needed when every wave gets an even number of whole 16-channel steps
    const bool mask = a.C % (16 * kPointwiseVariants[variant].depth() * kPointwiseVariants[variant].WC) != 0;
    const KernFn* const table = x_vec == 4 ? (mask ? masked4 : plain4) : (mask ? masked1 : plain1);
    hipLaunchKernelGGL(table[variant], dim3(grid), dim3(kPointwiseVariants[variant].block()), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace convfwd
