// Generic-family kernel: one output element per thread, plain fp32 FMA, any filter size and padding.
// It is the fallback for shapes outside the specialised families and follows the definition of the
// layer directly (Section 2.1): the dot product of one filter with one input sub-volume, padding
// taps skipped. Lanes of a wave hold consecutive q, so input reads are coalesced along X (Section 3).
#include "conv_internal.h"

#include <atomic>

#include <algorithm>

namespace convfwd {

__global__ void __launch_bounds__(256) conv_generic(const KernelArgs a)
{
    const long long total = (long long)a.total_pix * a.K;
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const int q = (int)(idx % a.Q);
        long long t = idx / a.Q;
        const int p = (int)(t % a.P);
        t /= a.P;
        const int k = (int)(t % a.K);
        const int n = (int)(t / a.K);
        const float* wk = a.w + k * a.CRS;
        const float* xn = a.x + n * a.C * a.HW;
        float acc = 0.f;
        for (int c = 0; c < a.C; ++c) {
            for (int r = 0; r < a.R; ++r) {
                const int h = p + r - a.pad_h;
                if (h < 0 || h >= a.H) continue;
                for (int s = 0; s < a.S; ++s) {
                    const int v = q + s - a.pad_w;
                    if (v < 0 || v >= a.W) continue;
                    acc = fmaf(xn[(c * a.H + h) * a.W + v], wk[(c * a.R + r) * a.S + s], acc);
                }
            }
        }
        a.y[idx] = finish_output(acc, a.bias ? a.bias[k] : 0.f, a.relu);
    }
}

// Streams zeros through a caller-provided scratch buffer: conv_fwd_find uses it to push the layer's tensors out of
// the L2s and the Infinity Cache between timed launches.
__global__ void __launch_bounds__(256) scratch_fill(float4* p, long long n16)
{
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = float4{0.f, 0.f, 0.f, 0.f};
}

// Scratch of conv_fwd_split_c_static, the entry point for callers that cannot allocate: the partial output tensors
// of the channel shares live here instead of in a caller's workspace. Every GPU the library runs on holds its own copy
// until the process ends. The name stands for the array in host code only as a symbol: its device address is looked up
// once per device (below) and everything - kernel arguments included - uses that address.
static __device__ __align__(256) float scratch[kStaticScratchBytes / 4];

hipError_t static_scratch(float** ptr)
{
    static std::atomic<float*> known[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    float* p = known[dev].load(std::memory_order_acquire);
    if (!p) {
        void* q = nullptr;
        e = hipGetSymbolAddress(&q, HIP_SYMBOL(scratch));  // the current device's copy of the array
        if (e != hipSuccess) return e;
        if (!q) return hipErrorInvalidSymbol;
        p = static_cast<float*>(q);
        known[dev].store(p, std::memory_order_release);
    }
    *ptr = p;
    return hipSuccess;
}

hipError_t launch_scratch_fill(void* buffer, long long bytes, hipStream_t stream)
{
    const long long n16 = bytes / 16;
    if (n16 <= 0) return hipSuccess;
    const int grid = (int)std::min<long long>((n16 + 255) / 256, 256 * 16);
    hipLaunchKernelGGL(scratch_fill, dim3(grid), dim3(256), 0, stream, reinterpret_cast<float4*>(buffer), n16);
    return hipGetLastError();
}

// Two micro-probes of what this GPU attains, for the benchmark's "fraction of measured peak" figures:
// a register-resident fp32 MFMA loop (16 independent accumulator tiles per wave, nothing else in the loop) and a
// dwordx4 stream copy.
typedef float probe_f32x4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256) probe_mfma(int iters, float* sink)
{
    probe_f32x4 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = probe_f32x4{0.f, 0.f, 0.f, 0.f};
    const float a = 1.0f + threadIdx.x * 1e-6f, b = 1.0f - threadIdx.x * 1e-6f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[i], 0, 0, 0);
    }
    probe_f32x4 sum = acc[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) sum += acc[i];
    if (sum.x + sum.y + sum.z + sum.w == 12345.678f) *sink = sum.x;  // keeps the loop alive, never true in practice
}

__global__ void __launch_bounds__(256) probe_copy(const float4* __restrict__ src, float4* __restrict__ dst, long long n16)
{
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// 256 CUs x 8 work-groups of 4 waves: 8192 waves x iters x 16 MFMAs of 2048 flops
hipError_t launch_probe_mfma(int iters, float* sink, hipStream_t stream)
{
    hipLaunchKernelGGL(probe_mfma, dim3(256 * 8), dim3(256), 0, stream, iters, sink);
    return hipGetLastError();
}

hipError_t launch_probe_copy(const void* src, void* dst, long long bytes, hipStream_t stream)
{
    const long long n16 = bytes / 16;
    if (n16 <= 0) return hipSuccess;
    const int grid = (int)std::min<long long>((n16 + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(probe_copy, dim3(grid), dim3(256), 0, stream, reinterpret_cast<const float4*>(src),
                       reinterpret_cast<float4*>(dst), n16);
    return hipGetLastError();
}

// Second pass of the channel-splitting mode: adds the partial output tensors the work-groups of each channel share
// wrote, always in share order (bitwise reproducible), then the epilogue. V floats per thread; V = 4 needs P*Q to be a
// multiple of 4 (a vector then lies inside one channel) and 16-byte aligned pointers.
template <int V>
__global__ void __launch_bounds__(256) conv_split_reduce(const float* __restrict__ parts, float* __restrict__ y,
                                                         const float* __restrict__ bias, int relu, int splits, int total,
                                                         int K, FastDiv div_PQ, FastDiv div_K)
{
    const long long i64 = (static_cast<long long>(blockIdx.x) * 256 + threadIdx.x) * V;  // may pass 2^31 in the last work-group
    if (i64 >= total) return;
    const int i = static_cast<int>(i64);
    const unsigned nk = div_PQ.div(i);
    const unsigned k = nk - div_K.div(nk) * K;
    const float b = bias ? bias[k] : 0.f;
    // four shares' loads in flight at a time; the additions keep the share order
    const float* p = parts + i;
    const size_t stride = static_cast<size_t>(total);
    if constexpr (V == 4) {
        float4 acc = *reinterpret_cast<const float4*>(p);
        int s = 1;
        for (; s + 4 <= splits; s += 4) {
            float4 t[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) t[u] = *reinterpret_cast<const float4*>(p + (s + u) * stride);
#pragma unroll
            for (int u = 0; u < 4; ++u) { acc.x += t[u].x; acc.y += t[u].y; acc.z += t[u].z; acc.w += t[u].w; }
        }
        for (; s < splits; ++s) {
            const float4 t = *reinterpret_cast<const float4*>(p + s * stride);
            acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
        }
        acc.x = finish_output(acc.x, b, relu); acc.y = finish_output(acc.y, b, relu);
        acc.z = finish_output(acc.z, b, relu); acc.w = finish_output(acc.w, b, relu);
        *reinterpret_cast<float4*>(y + i) = acc;
    } else {
        float acc = *p;
        int s = 1;
        for (; s + 4 <= splits; s += 4) {
            float t[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) t[u] = p[(s + u) * stride];
#pragma unroll
            for (int u = 0; u < 4; ++u) acc += t[u];
        }
        for (; s < splits; ++s) acc += p[s * stride];
        y[i] = finish_output(acc, b, relu);
    }
}

hipError_t launch_split_reduce(const float* parts, float* y, const float* bias, int relu, int splits, int total, int PQ,
                               int K, hipStream_t stream)
{
    // vectors only once single floats would already give every CU four work-groups
    const bool vec = PQ % 4 == 0 && total >= 256 * 256 * 4 && reinterpret_cast<uintptr_t>(parts) % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(y) % 16 == 0;
    const FastDiv div_PQ = make_fastdiv(PQ), div_K = make_fastdiv(K);
    if (vec) {
        hipLaunchKernelGGL(conv_split_reduce<4>, dim3((total / 4 + 255) / 256), dim3(256), 0, stream, parts, y, bias, relu,
                           splits, total, K, div_PQ, div_K);
    } else {
        hipLaunchKernelGGL(conv_split_reduce<1>, dim3((total + 255) / 256), dim3(256), 0, stream, parts, y, bias, relu,
                           splits, total, K, div_PQ, div_K);
    }
    return hipGetLastError();
}

hipError_t launch_generic(int grid, int block, hipStream_t stream, const KernelArgs& a)
{
    hipLaunchKernelGGL(conv_generic, dim3(grid), dim3(block), 0, stream, a);
    return hipGetLastError();
}

}  // namespace convfwd
