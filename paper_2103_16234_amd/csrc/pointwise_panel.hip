// Panel kernel of the pointwise family: 1x1 filters without padding on batched layers. For such a layer
// the whole batch is one matrix product y[K x N*HW] = w[K x C] * x[C x N*HW] per image block (Section 3, last
// paragraph: with a 1x1 filter the first stage already yields the output). A work-group keeps the filters
// of its 16*MT output channels - a panel of 16*MT x C floats - in LDS for its whole life and its waves
// stream 64-pixel tiles of the flattened (n, pixel) axis past it:
//   x: HBM -> registers (dwordx4 of four consecutive pixels = B operands of four MFMA tiles), PD steps of
//      16 channels in flight per wave, the stream of loads running on across tile boundaries;
//   w: LDS -> registers (one 16-byte read per 16 x 16 filter tile and step = A operands of four MFMAs);
//   y: registers -> HBM as dwordx4 of four consecutive pixels.
// Filter rows reach LDS through fully coalesced loads once per work-group instead of once per wave and
// step, which is what bounds the register-streaming kernel on deep layers (sixteen 64-byte row pieces per
// load instruction keep the vector cache busy four times longer than the same bytes read contiguously).
// Channels beyond C are zero in the panel, so the steps that pad C to a multiple of 16*PD need no masking:
// their inputs are read from clamped (valid) addresses and multiplied by zero.
#include "conv_internal.h"

#include <atomic>
#include <utility>

namespace convfwd {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// How the 64 pixels of a tile map to memory (PIX):
//   kFlatVec    H*W is a multiple of 4 and x, y are 16-byte aligned: tiles cut the flattened (n, pixel) axis, a
//               lane's four pixels 4j..4j+3 lie in one image and move as one aligned dwordx4;
//   kFlatDword  any H*W: same tiles, pixel t of lane j is 16t + j and moves as a dword (tiny maps, where tiles
//               per image would waste too much);
//   kImageVec   H*W not a multiple of 4 (13x13, 27x27 maps) or pointers only dword-aligned: tiles cut each
//               image on its own, the lane's four pixels move as one dwordx4 at a dword-aligned address (the
//               hardware runs in unaligned-access mode; the vector type below tells the compiler), and the
//               lanes past an image's last pixel are moved back onto its last four pixels.
// CLAMP: C is not a multiple of 16*PD, channel indices of the padding steps are clamped per lane.
enum { kFlatVec = 0, kFlatDword = 1, kImageVec = 2 };
typedef f32x4 f32x4_u __attribute__((aligned(4)));
template <int MT, int NW, int PD, int PIX, bool CLAMP>
__global__ void __launch_bounds__(64 * NW) conv_pointwise_panel(const KernelArgs a)
{
    extern __shared__ f32x4 smem4[];
    float* const panel = reinterpret_cast<float*>(smem4);
    constexpr int NTHREADS = 64 * NW;
    constexpr int NP = PIX == kFlatDword ? 4 : 1;  // pixel base pointers per lane

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15;
    const int kq = lane >> 4;

    // XCD-aware renumbering: work-groups that stream the same pixel tiles past different filter panels
    // sit on one L2.
    int L;
    {
        const int nb = gridDim.x, b = blockIdx.x;
        const int per = nb >> 3, rem = nb & 7, xcd = b & 7;
        L = xcd * per + (xcd < rem ? xcd : rem) + (b >> 3);
    }
    const int g = a.div_ktiles.div(L);
    const int k0 = (L - g * a.ktiles) * (16 * MT);

    const int nsteps = a.nchunks;   // 16-channel steps, a multiple of PD
    const int T = a.x_items;        // 64-pixel tiles of the flattened (n, pixel) axis
    const int stride = a.ptiles * NW;
    // Wave numbering along the tile axis: waves w and w + 4 of a work-group share a SIMD, and low numbers
    // get the extra tile when the tiles do not divide evenly, so the second half of an 8-wave work-group
    // counts down from the top: every SIMD then carries one "long" and one "short" wave.
    const int t0 = NW == 8 ? (wave < 4 ? g * 4 + wave : stride - 1 - (g * 4 + wave - 4)) : g * NW + wave;
    const int pitch = a.lds_pitch;

    // Addresses of the input loads are a uniform 64-bit base per tile (channel 0 of the image that holds
    // the tile's first pixel) plus 32-bit byte offsets per lane: the lane's pixels relative to that image
    // (a tile of small maps spans several images) and a running channel offset that is the same for all lanes.
    struct TileAddr {
        const char* base;
        unsigned voff[NP];
    };
    const unsigned hw4 = 4u * (unsigned)a.HW;
    // first pixel of the lane's i-th pixel group of tile t, as (image, pixel in the image)
    auto lane_pixel = [&](int t, int i, int& n, int& p) {
        if constexpr (PIX == kImageVec) {
            n = a.div_ptiles.div(t);  // a.tile_pix = tiles per image
            p = min((t - n * a.tile_pix) * 64 + 4 * j, a.HW - 4);
        } else {
            const int px = PIX == kFlatVec ? min(t * 64 + 4 * j, a.total_pix - 4) : min(t * 64 + 16 * i + j, a.total_pix - 1);
            n = a.div_PQ.div(px);
            p = px - n * a.HW;
        }
    };
    auto tile_addr = [&](int t, TileAddr& ta) {
        const int tt = min(t, T - 1);
        const int n0 = PIX == kImageVec ? a.div_ptiles.div(tt) : a.div_PQ.div(tt * 64);
        ta.base = reinterpret_cast<const char*>(a.x) + (size_t)n0 * a.C * a.HW * 4;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            int n, p;
            lane_pixel(tt, i, n, p);
            ta.voff[i] = 4u * (unsigned)((n - n0) * a.C * a.HW + p + (CLAMP ? 0 : 4 * kq * a.HW));
        }
    };

    f32x4 xr[PD][4];
    // one of the four input loads of a step: channel 16s + 4kq + e for the lane's four pixels;
    // soff = 4 * (16s + e) * HW bytes
    auto load_one = [&](auto slotc, auto ec, const TileAddr& ta, int s, unsigned soff) {
        constexpr int slot = decltype(slotc)::value;
        constexpr int e = decltype(ec)::value;
        const unsigned coff = CLAMP ? (unsigned)min(16 * s + 4 * kq + e, a.C - 1) * hw4 : soff;
        if constexpr (PIX == kFlatVec) {
            xr[slot][e] = *reinterpret_cast<const f32x4*>(ta.base + (ta.voff[0] + coff));
        } else if constexpr (PIX == kImageVec) {
            xr[slot][e] = *reinterpret_cast<const f32x4_u*>(ta.base + (ta.voff[0] + coff));
        } else {
            xr[slot][e] = f32x4{*reinterpret_cast<const float*>(ta.base + (ta.voff[0] + coff)),
                                *reinterpret_cast<const float*>(ta.base + (ta.voff[1] + coff)),
                                *reinterpret_cast<const float*>(ta.base + (ta.voff[2] + coff)),
                                *reinterpret_cast<const float*>(ta.base + (ta.voff[3] + coff))};
        }
    };
    auto for_each_e = [&](auto&& f) {
        [&]<int... Es>(std::integer_sequence<int, Es...>) { (f(std::integral_constant<int, Es>{}), ...); }
        (std::make_integer_sequence<int, 4>{});
    };
    auto for_each_slot = [&](auto&& f) {
        [&]<int... Ss>(std::integer_sequence<int, Ss...>) { (f(std::integral_constant<int, Ss>{}), ...); }
        (std::make_integer_sequence<int, PD>{});
    };

    TileAddr cur, nxt;
    tile_addr(t0, cur);
    // The first input steps are requested before the panel is fetched, so both latencies overlap. They are
    // issued in the order the loop issues and consumes them (the counter of outstanding loads is in order).
    for_each_slot([&](auto sc) {
        for_each_e([&](auto ec) {
            load_one(sc, ec, cur, decltype(sc)::value, (16u * decltype(sc)::value + decltype(ec)::value) * hw4);
            __builtin_amdgcn_sched_barrier(0);
        });
    });

    {
        const int rowv = nsteps * 4;  // dwordx4 per panel row
        const int total = 16 * MT * rowv;
        for (int base = 0; base < total; base += 8 * NTHREADS) {
            f32x4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * NTHREADS + tid;
                const int r = a.div_row_vecs.div(idx);
                const int c = 4 * (idx - r * rowv);
                const bool real = idx < total && c < a.C;
                v[u] = *reinterpret_cast<const f32x4*>(a.w + (real ? min(k0 + r, a.K - 1) * a.C + c : 0));
                if (!real) v[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * NTHREADS + tid;
                const int r = a.div_row_vecs.div(idx);
                const int c = 4 * (idx - r * rowv);
                if (idx < total) *reinterpret_cast<f32x4*>(panel + r * pitch + c) = v[u];
            }
        }
    }
    // The epilogue's per-channel constants live in registers for the kernel's whole life: a load inside the
    // tile loop would sit behind the prefetched inputs in the in-order counter and drain them at every tile.
    float bk[MT][4];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int v = 0; v < 4; ++v) bk[m][v] = a.bias ? a.bias[min(k0 + 16 * m + 4 * kq + v, a.K - 1)] : 0.f;

    // Every load so far is complete on every path before the main loop starts: the loop's own waits then
    // only have to track the loop's loads (vmcnt = 0, other counters untouched).
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();

    f32x4 acc[MT][4];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[m][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // lane (j, kq) reads channels 16s + 4kq .. +3 of filter 16m + j: the A operands of the four MFMAs
    // that consume the lane's four input loads of step s
    const float* const arow = panel + j * pitch + 4 * kq;
    f32x4 wv[2][MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) wv[0][m] = *reinterpret_cast<const f32x4*>(arow + 16 * m * pitch);

    // One round = PD steps: matrix instructions on the registers loaded PD steps ago, each register
    // reloaded (for step ls + slot of the load cursor's tile) right after its last use.
    auto round = [&](int it) {
        const bool last = it + PD >= nsteps;  // the loads issued in this round belong to the next tile
        const int ls = last ? 0 : it + PD;
        if (last) cur = nxt;
        for_each_slot([&](auto sc) {
            constexpr int slot = decltype(sc)::value;
            constexpr int wb = slot & 1;
            int sn = it + slot + 1;
            if (sn == nsteps) sn = 0;
#pragma unroll
            for (int m = 0; m < MT; ++m)
                wv[wb ^ 1][m] = *reinterpret_cast<const f32x4*>(arow + 16 * m * pitch + 16 * sn);
            const unsigned soff = 16u * (unsigned)(ls + slot) * hw4;
            // nothing moves across the barriers: every load keeps PD - 1 steps of distance to its use
            for_each_e([&](auto ec) {
                constexpr int e = decltype(ec)::value;
#pragma unroll
                for (int m = 0; m < MT; ++m)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[wb][m][e], xr[slot][e][t], acc[m][t], 0, 0, 0);
                load_one(sc, ec, cur, ls + slot, soff + e * hw4);
                __builtin_amdgcn_sched_barrier(0);
            });
        });
    };

    for (int ct = t0; ct < T; ct += stride) {
        tile_addr(ct + stride, nxt);
        // The first round of a tile is a copy of its own: it runs right after the previous tile's stores,
        // which share the in-order counter of outstanding memory operations with the loads, and its waits
        // can allow for them instead of draining the load stream.
        round(0);
        for (int it = PD; it < nsteps; it += PD) round(it);

        // Lane (j, kq) holds output channels 16m + 4kq + v for its four pixels of tile ct. Stores are
        // unconditional: lanes past the last pixel and rows past the last channel were computed from
        // clamped (duplicated) inputs and filters, so they rewrite the owner's value bit for bit.
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            int n, p;
            lane_pixel(ct, i, n, p);
            float* const yl = a.y + (size_t)n * a.K * a.HW + p;
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float* const dst = yl + (size_t)min(k0 + 16 * m + 4 * kq + v, a.K - 1) * a.HW;
                    const float b = bk[m][v];
                    if constexpr (PIX != kFlatDword) {
                        const f32x4 out{finish_output(acc[m][0][v], b, a.relu), finish_output(acc[m][1][v], b, a.relu),
                                        finish_output(acc[m][2][v], b, a.relu), finish_output(acc[m][3][v], b, a.relu)};
                        // Aligned tiles leave as streaming (nontemporal) stores: every store instruction fills whole
                        // cache lines that nothing in the kernel reads back, and keeping them from displacing inputs
                        // and filters is worth 7-30 % on write-heavy layers (128 x 64 x 56 x 56 -> 64 and -> 256
                        // filters). Stores that fill lines piecewise (the other two pixel modes) lose up to 25 % with
                        // the same hint, and so do the input loads wherever two channel tiles read the same pixels.
                        if constexpr (PIX == kFlatVec) __builtin_nontemporal_store(out, reinterpret_cast<f32x4*>(dst));
                        else *reinterpret_cast<f32x4_u*>(dst) = out;
                    } else {
                        *dst = finish_output(acc[m][i][v], b, a.relu);
                    }
                }
        }
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[m][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
}

using KernFn = void (*)(const KernelArgs);

template <int V, int PIX, bool CLAMP> static KernFn panel_instance()
{
    constexpr PanelVariant pv = kPanelVariants[V];
    return conv_pointwise_panel<pv.MT, pv.NW, pv.PD, PIX, CLAMP>;
}

// pix: 0 flattened tiles / aligned dwordx4, 1 flattened tiles / dwords, 2 tiles per image / dword-aligned dwordx4
hipError_t launch_panel(int variant, int pix, int grid, int lds_bytes, hipStream_t stream, const KernelArgs& a)
{
#define PANEL_ROW(v)                                                                                        \
    {panel_instance<v, kFlatVec, false>(),   panel_instance<v, kFlatVec, true>(),                           \
     panel_instance<v, kFlatDword, false>(), panel_instance<v, kFlatDword, true>(),                         \
     panel_instance<v, kImageVec, false>(),  panel_instance<v, kImageVec, true>()},
    static const KernFn table[kNumPanelVariants][6] = {PANEL_VARIANT_LIST(PANEL_ROW)};
    static std::atomic<int> lds_ready[kNumPanelVariants][6][kMaxDevices] = {};
    if (pix < 0 || pix > 2) return hipErrorInvalidValue;
    if (variant < 0 || variant >= kNumPanelVariants) return hipErrorInvalidValue;
    const PanelVariant pv = kPanelVariants[variant];
    const bool clamp = a.C % (16 * pv.PD) != 0;
    const int mode = 2 * pix + (clamp ? 1 : 0);
    const KernFn fn = table[variant][mode];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!lds_ready[variant][mode][dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        lds_ready[variant][mode][dev].store(1, std::memory_order_release);
    }
    hipLaunchKernelGGL(fn, dim3(grid), dim3(pv.block()), lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace convfwd
