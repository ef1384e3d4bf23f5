// The paper's own scheme (Section 3), kept as an opt-in variant with an explicit workspace so it can be
// measured against the fused kernels on this GPU. It is prior art, not the hot path:
//   stage 1 ("scalar products"): a work-group owns one filter row - the C weights w[k, :, r, s] - brings it
//       into LDS and every thread computes, for its output positions, the C-long dot product of that row
//       with the input column that meets it: T[r,s][n,k,p,q] = sum_c w[k,c,r,s] * xpad[n,c,p+r,q+s].
//       Lanes walk q, so the input reads are coalesced along X without any layout change. A row is split
//       over several work-groups when it has more positions than one work-group's threads cover. With a
//       1x1 filter the result is the output itself and is written to y.
//   stage 2 ("sum"): y = sum over the R*S temporary matrices of each (input, filter) pair, in tap order.
// Plain fp32 FMA, one dot product per thread: no register-level reuse, which is the limit the paper
// reports for it.
#include "conv_internal.h"

#include <algorithm>

namespace convfwd {

constexpr int kTwoStageThreads = 256;
constexpr int kTwoStagePositionsPerThread = 2;

__global__ void __launch_bounds__(kTwoStageThreads) conv_scalar_prods(const KernelArgs a, float* __restrict__ temp, int splits)
{
    extern __shared__ float wrow[];
    const int RS = a.R * a.S;
    const int row = blockIdx.x / splits;  // filter row: (k, r, s)
    const int split = blockIdx.x - row * splits;
    const int k = row / RS;
    const int rs = row - k * RS;
    const int r = rs / a.S, s = rs - r * a.S;

    for (int c = threadIdx.x; c < a.C; c += kTwoStageThreads) wrow[c] = a.w[(k * a.C + c) * RS + rs];
    __syncthreads();

    float* const out = RS == 1 ? a.y : temp + (long long)rs * a.total_pix * a.K;
    const int first = split * (kTwoStageThreads * kTwoStagePositionsPerThread) + threadIdx.x;
#pragma unroll
    for (int i = 0; i < kTwoStagePositionsPerThread; ++i) {
        const int g = first + i * kTwoStageThreads;  // position in flattened (n, p, q) order
        if (g >= a.total_pix) break;
        const int n = g / a.PQ;
        const int pq = g - n * a.PQ;
        const int p = pq / a.Q, q = pq - p * a.Q;
        const int h = p + r - a.pad_h, v = q + s - a.pad_w;
        float acc = 0.f;
        if (h >= 0 && h < a.H && v >= 0 && v < a.W) {
            const float* xc = a.x + (n * a.C * a.H + h) * a.W + v;
            for (int c = 0; c < a.C; ++c) acc = fmaf(wrow[c], xc[c * a.HW], acc);
        }
        out[(n * a.K + k) * a.PQ + pq] = acc;
    }
}

__global__ void __launch_bounds__(256) conv_sum_taps(const KernelArgs a, const float* __restrict__ temp)
{
    const long long total = (long long)a.total_pix * a.K;
    const int RS = a.R * a.S;
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        float acc = temp[i];
        for (int rs = 1; rs < RS; ++rs) acc += temp[rs * total + i];
        a.y[i] = acc;
    }
}

hipError_t launch_two_stage(hipStream_t stream, const KernelArgs& a, float* temp)
{
    const int per_block = kTwoStageThreads * kTwoStagePositionsPerThread;
    const int splits = (a.total_pix + per_block - 1) / per_block;
    const long long blocks = (long long)a.K * a.R * a.S * splits;
    if (blocks >= (1ll << 31) || (long long)a.C * 4 > 64 * 1024) return hipErrorInvalidValue;
    hipLaunchKernelGGL(conv_scalar_prods, dim3((unsigned)blocks), dim3(kTwoStageThreads), a.C * sizeof(float), stream, a, temp,
                       splits);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.R * a.S == 1) return e;
    const long long total = (long long)a.total_pix * a.K;
    const int grid = (int)std::min<long long>((total + 255) / 256, 256 * 64);
    hipLaunchKernelGGL(conv_sum_taps, dim3(grid), dim3(256), 0, stream, a, temp);
    return hipGetLastError();
}

}  // namespace convfwd
