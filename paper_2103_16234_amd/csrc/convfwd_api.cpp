// C-ABI entry points, argument validation and the per-shape tile planner (host only).
#include "../../include/convfwd.h"
#include "conv_internal.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <numeric>
#include <string>
#include <vector>

namespace convfwd {

using TapLauncher = hipError_t (*)(int, int, int, int, hipStream_t, const KernelArgs&);
#define DECLARE_TAP1(v) hipError_t launch_tap_1x1_v##v(int, int, int, int, hipStream_t, const KernelArgs&);
#define DECLARE_TAP3(v) hipError_t launch_tap_3x3_v##v(int, int, int, int, hipStream_t, const KernelArgs&);
#define DECLARE_TAP5(v) hipError_t launch_tap_5x5_v##v(int, int, int, int, hipStream_t, const KernelArgs&);
#define DECLARE_TAP_EXTRA(r, s, v) hipError_t launch_tap_##r##x##s##_v##v(int, int, int, int, hipStream_t, const KernelArgs&);
TAP_VARIANT_LIST(DECLARE_TAP1)
TAP_VARIANT_LIST(DECLARE_TAP3)
TAP_VARIANT_LIST(DECLARE_TAP5)
TAP_EXTRA_SIZES(DECLARE_TAP_EXTRA)

// [filter size][tile shape]; null where the pair is not built
struct TapLauncherTable {
    TapLauncher fn[kNumTapSizes][kNumTapVariants] = {};
    TapLauncherTable()
    {
#define ENTRY_TAP1(v) fn[0][v] = launch_tap_1x1_v##v;
#define ENTRY_TAP3(v) fn[1][v] = launch_tap_3x3_v##v;
#define ENTRY_TAP5(v) fn[2][v] = launch_tap_5x5_v##v;
#define ENTRY_TAP_EXTRA(r, s, v)                                                                                      \
    static_assert(tap_size_index(r, s) >= kNumFullTapSizes && v < kNumTapVariants, "size or tile shape missing from the tables"); \
    fn[tap_size_index(r, s)][v] = launch_tap_##r##x##s##_v##v;
        TAP_VARIANT_LIST(ENTRY_TAP1)
        TAP_VARIANT_LIST(ENTRY_TAP3)
        TAP_VARIANT_LIST(ENTRY_TAP5)
        TAP_EXTRA_SIZES(ENTRY_TAP_EXTRA)
    }
};
static const TapLauncherTable kTapLaunchers;

bool tap_is_built(int rs_index, int variant)
{
    return rs_index >= 0 && rs_index < kNumTapSizes && variant >= 0 && variant < kNumTapVariants &&
           kTapLaunchers.fn[rs_index][variant] != nullptr;
}

hipError_t launch_tap(int rs_index, int variant, int x_vec, int w_vec, int grid, int lds_bytes,
                      hipStream_t stream, const KernelArgs& a)
{
    if (!tap_is_built(rs_index, variant)) return hipErrorInvalidValue;
    return kTapLaunchers.fn[rs_index][variant](x_vec, w_vec, grid, lds_bytes, stream, a);
}

namespace {

constexpr int kNumCU = 256;              // MI355X: 8 XCDs x 32 CUs
constexpr int kLdsMax = 160 * 1024;      // LDS of one CU

thread_local hipStream_t g_stream = nullptr;  // per host thread: selecting a stream and launching on it cannot be split by another thread
thread_local std::string g_hip_error = "no HIP error recorded";

struct Shape {
    int N, C, H, W, K, R, S, pad_h, pad_w, P, Q;
};

int validate(int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w, Shape* s)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 || pad_h < 0 || pad_w < 0)
        return CONV_E_DIM;
    const int64_t P = (int64_t)H + 2 * (int64_t)pad_h - R + 1;
    const int64_t Q = (int64_t)W + 2 * (int64_t)pad_w - S + 1;
    if (P <= 0 || Q <= 0) return CONV_E_EMPTY;
    const int64_t lim = (int64_t)1 << 31;
    const int64_t nx = (int64_t)N * C * H * W;
    const int64_t nw = (int64_t)K * C * R * S;
    // guard the products step by step: the factors themselves can be near 2^31
    if ((int64_t)N * C >= lim || (int64_t)H * W >= lim || nx >= lim || nx / ((int64_t)H * W) != (int64_t)N * C)
        return CONV_E_OVERFLOW;
    if ((int64_t)K * C >= lim || (int64_t)R * S >= lim || nw >= lim) return CONV_E_OVERFLOW;
    if (P >= lim || Q >= lim || P * Q >= lim || (int64_t)N * K >= lim) return CONV_E_OVERFLOW;
    const int64_t ny = (int64_t)N * K * (P * Q);
    if (ny >= lim || ny / (P * Q) != (int64_t)N * K) return CONV_E_OVERFLOW;
    if (((int64_t)H + 2 * (int64_t)pad_h) * N >= lim || (int64_t)W + 2 * (int64_t)pad_w >= lim) return CONV_E_OVERFLOW;
    *s = Shape{N, C, H, W, K, R, S, pad_h, pad_w, (int)P, (int)Q};
    return CONV_OK;
}

// (in 64 bits: a dimension may be close to 2^31)
inline int ceil_div(int a, int b) { return (int)(((int64_t)a + b - 1) / b); }
inline int round_up(int v, int m) { return (int)std::min<int64_t>(((int64_t)v + m - 1) / m * m, INT32_MAX); }

int tap_rs_index(const Shape& s) { return tap_size_index(s.R, s.S); }

void base_args(const Shape& s, KernelArgs* a)
{
    std::memset(a, 0, sizeof(*a));
    a->N = s.N; a->C = s.C; a->H = s.H; a->W = s.W; a->K = s.K; a->R = s.R; a->S = s.S;
    a->pad_h = s.pad_h; a->pad_w = s.pad_w;
    a->P = s.P; a->Q = s.Q; a->PQ = s.P * s.Q; a->HW = s.H * s.W; a->CRS = s.C * s.R * s.S;
    a->Hp = s.H + 2 * s.pad_h;
    a->total_pix = s.N * s.P * s.Q;
    a->split_c = s.C;
}

void fill_common(const Shape& s, conv_plan_t* p)
{
    p->P = s.P; p->Q = s.Q;
    p->workspace_bytes = 0;
    p->c_splits = 1;
    p->flops = 2LL * s.N * s.K * s.P * s.Q * s.C * s.R * s.S;
    p->bytes = 4LL * ((int64_t)s.N * s.C * s.H * s.W + (int64_t)s.K * s.C * s.R * s.S + (int64_t)s.N * s.K * s.P * s.Q);
}

// Rows of the stacked zero-padded images (image n occupies rows n*Hp .. n*Hp+Hp-1) that the widest
// pixel tile touches. The tile phase repeats every PQ / gcd(PQ, tile_pix) tiles.
int max_halo_rows(const Shape& s, int tile_pix)
{
    const int64_t total = (int64_t)s.N * s.P * s.Q;
    const int PQ = s.P * s.Q, Hp = s.H + 2 * s.pad_h;
    const int64_t period = PQ / std::gcd(PQ, tile_pix);
    if (period > 4096) {
        // Too many phases to walk (maps of millions of pixels): an upper bound instead - the rows a run of tile_pix
        // pixels can touch at the worst phase, the filter's R-1 more, and the padding rows between images it crosses.
        const int64_t bound = ((int64_t)tile_pix + s.Q - 2) / s.Q + 1 + (s.R - 1) +
                              (((int64_t)tile_pix + PQ - 2) / PQ) * (Hp - s.P);
        return (int)std::min<int64_t>(bound, INT32_MAX / 2);
    }
    int rows = 0;
    int64_t g0 = 0;
    for (int64_t i = 0; i <= period && g0 < total; ++i, g0 += tile_pix) {
        const int64_t g1 = std::min<int64_t>(g0 + tile_pix, total) - 1;
        const int64_t v0 = (g0 / PQ) * Hp + (g0 % PQ) / s.Q;
        const int64_t v1 = (g1 / PQ) * Hp + (g1 % PQ) / s.Q + s.R - 1;
        rows = std::max<int>(rows, (int)(v1 - v0 + 1));
    }
    return rows;
}

// Resolve a tap-family mapping. tile_pix / chunk_c of 0 mean "choose". c_splits > 1 asks for that many channel
// shares, each reduced by work-groups of its own into a partial output tensor (fewer if C has fewer chunks).
// The eight XCDs (one L2 each) receive contiguous runs of the work-group numbering, which walks a group of g channel tiles,
// then the pixel tiles, then the groups. With g = all channel tiles a run holds every channel tile of a few pixel tiles,
// so each L2 fetches all the filters and an eighth of the inputs; with g = 1 it is the other way round; a divisor of the
// channel tiles in between shares both. Bytes all eight L2s fetch under a group size: a run of `per` work-groups touches
// ceil(per / g) (+1 where runs straddle) (group, pixel tile) pairs, so that many pixel indices (at most all) of
// ceil(pairs / pixel indices) groups; with channel shares (splits) a pixel index is a (share, pixel tile) pair and reads
// 1/splits of the channels.
double fetched_bytes(const Shape& s, int ktiles, int ptiles, int splits, int g)
{
    const double pt_all = (double)ptiles * splits;
    const double per = std::max(1.0, std::ceil(ktiles * pt_all / 8.0));
    const double w_unit = 4.0 * s.K * s.C * s.R * s.S / ((double)ktiles * splits);  // one channel tile, one share
    const double x_unit = 4.0 * s.N * s.C * s.H * s.W / pt_all;                      // one pixel tile, one share
    const double groups = (double)ktiles / g;
    const double pairs = std::min(groups * pt_all, std::ceil(per / g) + ((per > g && std::fmod(per, (double)g) != 0.0) ? 1.0 : 0.0));
    const double pix = std::min(pt_all, pairs);
    const double grp = std::min(groups, std::ceil(pairs / pt_all) + ((pairs > pt_all && std::fmod(pairs, pt_all) != 0.0) ? 1.0 : 0.0));
    const double kt = std::min<double>(std::min<double>(ktiles, per), grp * g);
    return 8.0 * (pix * x_unit + kt * std::min<double>(splits, std::ceil(pix / ptiles)) * w_unit);
}
// Group size of the work-group numbering: all channel tiles (the channel tile is the fast index) unless another divisor
// of their number fetches at least a fifth less; then the one that fetches least (ties: the larger group).
int pick_k_group(const Shape& s, int ktiles, int ptiles, int splits, bool groups_only = false)
{
    int best = groups_only ? 0 : ktiles;
    double best_bytes = groups_only ? 0.0 : 0.8 * fetched_bytes(s, ktiles, ptiles, splits, ktiles);
    for (int g = ktiles - 1; g >= 1; --g) {
        if (ktiles % g != 0 || (groups_only && g == 1)) continue;
        const double b = fetched_bytes(s, ktiles, ptiles, splits, g);
        if (best == 0 || b < best_bytes) { best = g; best_bytes = b; }
    }
    return best;
}

// Returns false if it cannot run.
// loader: 0 = by rule, else CONV_LOADER_REGISTERS / CONV_LOADER_DIRECT. order: 0 = by rule, else CONV_ORDER_*.
bool resolve_tap(const Shape& s, int variant, int tile_pix, int chunk_c, int x_cap, int w_cap,
                 conv_plan_t* p, KernelArgs* a, int c_splits = 1, int loader = 0, int order = 0, int k_group = 0)
{
    if (loader < 0 || loader > CONV_LOADER_DIRECT_DEEP) return false;
    if (order < 0 || order > CONV_ORDER_CHANNEL_GROUPS || k_group < 0) return false;
    const int rs_index = tap_rs_index(s);
    if (!tap_is_built(rs_index, variant)) return false;
    const TapVariant tv = kTapVariants[variant];
    // Rule for the loader waves, from timings of the same mapping with each loader on the layers of the shape grid that
    // run the eight-wave tile shapes: where the rule below would leave a deep layer (12 chunks or more) to the register
    // loader - rows of dwordx2 on 14-wide maps, 7 x 7 maps - the shapes with two channel shares run 1-4 % faster with
    // four loader waves (32 x 256 x 14 x 14 -> 256: 76.7 -> 73.7 us; 128 x 512 x 7 x 7 -> 512: 258 -> 248 us); the shapes
    // with four shares, short layers and layers whose rows already move as direct dwordx4 lose 1-10 %.
    // (Four shares on rows of dwordx2, eight chunks or more: timed on 8 x 512 x 14 x 14 -> 512 and 16 x 256 x 14 x 14 -> 256, where
    // the 32 x 112 shapes and their tail twins run 11-13 % faster with loader waves than with the register loader; against
    // the direct loader of the multiplying waves they keep 3-5 % on these and on 7 x 7 maps: 8 x 512 x 7 x 7 -> 2048 70.9 -> 67.3 us.)
    if (loader == 0 && tv.loader_waves() > 0 && s.C % 4 == 0 && w_cap >= 4 &&
        ((tv.WC == 2 && s.C >= 12 * tv.chunk_c() && (s.W % 4 == 2 || s.W < 13)) ||
         (tv.WC == 4 && s.C >= 8 * tv.chunk_c() && (s.W % 4 == 2 || s.W < 13))) &&
        resolve_tap(s, variant, tile_pix, chunk_c, x_cap, w_cap, p, a, c_splits, CONV_LOADER_DIRECT_WAVES, order, k_group))
        return true;
    // (rows of dwordx2 are not for the direct loader: by rule it takes them as dwords where that fits)
    if (loader == 0 && s.C % 4 == 0 && w_cap >= 4 && std::min(s.W % 4 == 0 ? 4 : s.W % 2 == 0 ? 2 : 1, x_cap) == 2 &&
        resolve_tap(s, variant, tile_pix, chunk_c, x_cap, w_cap, p, a, c_splits, CONV_LOADER_DIRECT, order, k_group))
        return true;
    const int RS = s.R * s.S, TK = tv.tile_k(), BLOCK = tv.block();
    const int64_t total64 = (int64_t)s.N * s.P * s.Q;
    if (tile_pix == 0) tile_pix = (int)std::min<int64_t>(tv.max_pix(), total64);
    if (tile_pix < 1 || tile_pix > tv.max_pix()) return false;
    if (total64 > (int64_t)INT32_MAX - 4096) return false;  // pixel indices of the last, partly empty tile stay inside 32 bits
    const int total = (int)total64;

    int w_vec = (s.C % 4 == 0 && w_cap >= 4) ? 4 : 1;
    int x_vec = s.W % 4 == 0 ? 4 : s.W % 2 == 0 ? 2 : 1;
    x_vec = std::min(x_vec, x_cap);
    if (w_vec == 1 && x_vec != 4) x_vec = 1;  // the loaders built: (4, 4), (2, 4), (1, 4), (4, 1), (1, 1)
    // Loader waves only know direct loads, which move dwordx4 or single dwords: rows of dwordx2 go dword by dword.
    const bool loader_waves = loader == CONV_LOADER_DIRECT_WAVES;
    if (loader_waves && (tv.loader_waves() == 0 || w_vec != 4)) return false;
    if (loader_waves && x_vec == 2) x_vec = 1;
    if (loader == CONV_LOADER_DIRECT && x_vec == 2) x_vec = 1;  // (on request only: the rule below never picks it)
    // The deep direct loader: the same loads, into a ring of tv.deep_copies() staging copies.
    const bool deep = loader == CONV_LOADER_DIRECT_DEEP;
    if (deep && (tv.deep_copies() == 0 || w_vec != 4)) return false;
    if (deep && x_vec == 2) x_vec = 1;

    const int col_shift = (x_vec - s.pad_w % x_vec) % x_vec;
    // Sizes of the halo tile in 64 bits first: a padded row, R of them, or a plane that cannot fit LDS ends the attempt
    // here, before any product of them is narrowed to int (a copy holds fewer than 2^16 floats, checked below).
    const int64_t pitch64 = ((int64_t)s.W + 2 * (int64_t)s.pad_w + col_shift + x_vec - 1) / x_vec * x_vec;
    if (pitch64 * s.R * 4 > kLdsMax) return false;
    const int pitch = (int)pitch64;
    const int rows = max_halo_rows(s, tile_pix);
    // channel planes start 16 banks apart (mod 32): the four channels one B operand spans do not collide
    const int64_t plane64 = (std::max<int64_t>((int64_t)rows * pitch - 16, 0) + 31) / 32 * 32 + 16;
    if (plane64 * tv.chunk_c() * 4 > kLdsMax) return false;
    const int plane = (int)plane64;
    const int row_vecs = s.W / x_vec;
    // The direct loader moves dwordx4 or single dwords; its slots also cover the padding cells of the halo tile.
    const bool direct_fits = w_vec == 4 && (x_vec == 4 || x_vec == 1) &&
                             (int64_t)tv.chunk_c() * plane / x_vec <= (int64_t)tv.xs_direct(x_vec) * BLOCK &&
                             // a slot's byte offset from the first channel of its chunk in the tile's first image (x), from the
                             // chunk's first element of the tile's first output channel (w), is kept in 32 bits
                             ((int64_t)(rows / (s.H + 2 * s.pad_h) + 2) * s.C + tv.chunk_c()) * s.H * s.W * 4 < ((int64_t)1 << 32) - 64 &&
                             (int64_t)TK * s.C * RS * 4 < ((int64_t)1 << 32) - 64;
    if ((loader == CONV_LOADER_DIRECT || loader_waves || deep) && !direct_fits) return false;
    // Rule: direct loads wherever they fit. (With a pointer and a 64-bit add per slot and chunk they lost to the register
    // loader on short layers with rows of single dwords and on 7x7 maps; as buffer loads with a constant offset per slot
    // they win almost everywhere - the cost model's best mapping under each loader, timed on the 188 3x3 / 5x5 layers of
    // the shape grid and 113 random layers off it: where the old rule chose the register loader (84 layers) the direct
    // loader is 11.5 % faster in the geometric mean, 10 % slower at worst (1 x 512 x 7 x 7 -> 512); rows of dwordx2 go dword
    // by dword.)
    const bool direct = loader == CONV_LOADER_DIRECT || loader_waves || deep || (loader == 0 && direct_fits);

    // The chunk is a property of the tile shape; a caller may only name that size.
    const int cc = tv.chunk_c();
    if (chunk_c != 0 && chunk_c != cc) return false;
    chunk_c = cc;
    if (!tv.supports(RS) || (w_vec == 1 && !tv.supports_scalar(RS, x_vec))) return false;  // staging would not fit the registers
    const int64_t x_floats = (int64_t)cc * rows * s.W;
    if (!direct && x_floats > (int64_t)tv.xs(x_vec) * x_vec * BLOCK) return false;
    const int64_t copy_floats = direct ? tv.staging_floats_direct(RS, plane) : tv.staging_floats(RS, plane);
    const int64_t lds = 4 * std::max<int64_t>((deep ? tv.deep_copies() : 2) * copy_floats, tv.reduce_floats());
    // (the deep ring is for launches of about one work-group per CU: it may take the whole LDS)
    if (lds > (deep ? kLdsMax : tv.lds_limit()) || lds > kLdsMax || copy_floats >= (1 << 16)) return false;
    if (deep) {
        // loads that stay in flight across the wait at the end of a chunk: the counter that orders them holds 63
        const int div = tap_x_slot_divisor(tv, x_vec, w_vec, cc * plane / x_vec, true);
        const int slots = (tv.xs_direct(x_vec) + div - 1) / div + tv.wslots_direct(RS);
        if ((tv.deep_copies() - 2) * slots > 63) return false;
    }

    base_args(s, a);
    a->tile_pix = tile_pix;
    a->ktiles = ceil_div(s.K, TK);
    a->ptiles = ceil_div(total, tile_pix);
    // shares hold whole chunks, all but the last the same number
    const int chunks_all = ceil_div(s.C, cc);
    const int chunks_share = ceil_div(chunks_all, std::max(1, std::min(c_splits, chunks_all)));
    const int splits = ceil_div(chunks_all, chunks_share);
    if ((int64_t)a->ktiles * a->ptiles * splits >= ((int64_t)1 << 31)) return false;
    a->nchunks = chunks_share;
    if (splits > 1) a->split_c = chunks_share * cc;
    a->lds_rows = rows; a->lds_pitch = pitch; a->lds_plane = plane; a->col_shift = col_shift;
    a->x_items = direct ? cc * plane / x_vec : cc * rows * row_vecs;
    a->direct = deep ? 3 : loader_waves ? 2 : direct ? 1 : 0;
    a->div_ktiles = make_fastdiv(a->ktiles); a->div_ptiles = make_fastdiv(a->ptiles);
    a->pt_all = a->ptiles * splits; a->div_pt_all = make_fastdiv(a->pt_all);
    if (order == CONV_ORDER_CHANNEL_FAST) a->k_group = a->ktiles;
    else if (order == CONV_ORDER_PIXEL_FAST) a->k_group = 1;
    else if (order == CONV_ORDER_CHANNEL_GROUPS && k_group > 0) a->k_group = k_group;
    else a->k_group = pick_k_group(s, a->ktiles, a->ptiles, splits, order == CONV_ORDER_CHANNEL_GROUPS);
    // (a group must divide the channel tiles and lie strictly between the two plain orders)
    if (order == CONV_ORDER_CHANNEL_GROUPS && (a->k_group <= 1 || a->k_group >= a->ktiles || a->ktiles % a->k_group != 0)) return false;
    a->div_k_group = make_fastdiv(a->k_group);
    a->div_PQ = make_fastdiv(a->PQ); a->div_Q = make_fastdiv(s.Q); a->div_Hp = make_fastdiv(a->Hp);
    a->div_row_vecs = make_fastdiv(direct ? pitch / x_vec : row_vecs);
    a->div_slot_c = make_fastdiv(direct ? plane / x_vec : rows * row_vecs);
    a->inv_row_vecs = 1.0f / static_cast<float>(direct ? pitch / x_vec : row_vecs);
    a->inv_slot_c = 1.0f / static_cast<float>(direct ? plane / x_vec : rows * row_vecs);
    a->inv_Hp = 1.0f / static_cast<float>(a->Hp); a->inv_Q = 1.0f / static_cast<float>(s.Q);
    a->inv_P = 1.0f / static_cast<float>(s.P); a->inv_PQ = 1.0f / static_cast<float>(a->PQ);

    std::memset(p, 0, sizeof(*p));
    p->kernel = CONV_KERNEL_TAP; p->variant = variant;
    p->tile_k = TK; p->tile_pix = tile_pix; p->chunk_c = cc;
    p->x_vec = x_vec; p->w_vec = w_vec;
    p->lds_rows = rows; p->lds_pitch = pitch; p->lds_plane = plane;
    p->grid = a->ktiles * a->ptiles * splits; p->block = BLOCK + (loader_waves ? 64 * tv.loader_waves() : 0);
    p->lds_bytes = (int)lds;
    fill_common(s, p);
    p->c_splits = splits;
    p->loader = deep ? CONV_LOADER_DIRECT_DEEP : loader_waves ? CONV_LOADER_DIRECT_WAVES : direct ? CONV_LOADER_DIRECT : CONV_LOADER_REGISTERS;
    p->order = a->k_group == a->ktiles ? CONV_ORDER_CHANNEL_FAST : a->k_group == 1 ? CONV_ORDER_PIXEL_FAST : CONV_ORDER_CHANNEL_GROUPS;
    p->k_group = a->k_group;
    if (splits > 1) p->workspace_bytes = 4LL * splits * s.K * total;
    return true;
}

// Pointwise family: 1x1 filters, no padding, filter rows that dwordx4 can walk. Pixels move as dwordx4
// when H*W is a multiple of 4 and x, y are 16-byte aligned, as single dwords otherwise.
bool pointwise_ok(const Shape& s, int x_cap, int w_cap, int y_cap)
{
    (void)x_cap; (void)y_cap;
    return s.R == 1 && s.S == 1 && s.pad_h == 0 && s.pad_w == 0 && s.C % 4 == 0 && w_cap >= 4;
}
int pointwise_x_vec(const Shape& s, int x_cap, int y_cap)
{
    return ((s.H * s.W) % 4 == 0 && x_cap >= 4 && y_cap >= 4) ? 4 : 1;
}

bool resolve_pointwise(const Shape& s, int variant, int x_cap, int w_cap, int y_cap, conv_plan_t* p, KernelArgs* a)
{
    if (!pointwise_ok(s, x_cap, w_cap, y_cap) || variant < 0 || variant >= kNumPointwiseVariants) return false;
    const PointwiseVariant pv = kPointwiseVariants[variant];
    base_args(s, a);
    a->tile_pix = pv.tile_pix();
    a->ktiles = ceil_div(s.K, pv.tile_k());
    a->ptiles = ceil_div(s.H * s.W, pv.tile_pix());  // per image
    const int64_t grid = (int64_t)a->ktiles * a->ptiles * s.N;
    if (grid >= ((int64_t)1 << 31)) return false;
    a->nchunks = ceil_div(s.C, 16);
    a->div_ktiles = make_fastdiv(a->ktiles); a->div_ptiles = make_fastdiv(a->ptiles);
    std::memset(p, 0, sizeof(*p));
    p->kernel = CONV_KERNEL_POINTWISE; p->variant = variant;
    p->tile_k = pv.tile_k(); p->tile_pix = pv.tile_pix(); p->chunk_c = 16 * pv.WC;
    p->x_vec = pointwise_x_vec(s, x_cap, y_cap); p->w_vec = 4;
    p->grid = (int)grid; p->block = pv.block(); p->lds_bytes = pv.lds_bytes();
    fill_common(s, p);
    return true;
}

// Pixel mode of the panel kernel: 0 = aligned dwordx4 over flattened tiles when H*W is a multiple of 4 and x, y are
// 16-byte aligned; otherwise 2 = dword-aligned dwordx4 over tiles cut per image if that wastes at most 6 % of the
// tiles' pixels (27x27: 729 of 768; measured 5-11 % faster than dwords there, but 25 % slower on 13x13 maps, which
// fill 169 of 192), else 1 = single dwords over flattened tiles.
int panel_pixel_mode(const Shape& s, int x_cap, int y_cap)
{
    if (pointwise_x_vec(s, x_cap, y_cap) == 4) return 0;
    const int hw = s.H * s.W;
    return (hw >= 4 && ceil_div(hw, 64) * 64 * 100 <= hw * 106) ? 2 : 1;
}

// Panel kernel of the pointwise family: the filters of a channel tile must fit LDS whole. tile_pix > 0
// requests that many work-groups per channel tile (0 = choose).
// With groups chosen here, *modelled (if given) receives the chosen grid's cost in cycles of the busiest SIMD.
bool resolve_panel(const Shape& s, int variant, int groups_req, int x_cap, int w_cap, int y_cap, conv_plan_t* p, KernelArgs* a,
                   double* modelled = nullptr)
{
    if (!pointwise_ok(s, x_cap, w_cap, y_cap) || variant < 0 || variant >= kNumPanelVariants) return false;
    const PanelVariant pv = kPanelVariants[variant];
    const int steps = round_up(s.C, 16 * pv.PD) / 16;
    const int pitch = 16 * steps + 4;
    const int64_t lds = (int64_t)pv.tile_k() * pitch * 4;
    if (lds > kLdsMax) return false;
    base_args(s, a);
    if (a->total_pix < 4 || a->total_pix > (1 << 30)) return false;  // tile * 64 + lane offsets stay far inside 32 bits
    const int per_image = ceil_div(a->HW, 64);
    const int pix = panel_pixel_mode(s, x_cap, y_cap);
    const int tiles = pix == 2 ? s.N * per_image : ceil_div(a->total_pix, 64);
    if ((int64_t)s.N * per_image >= (1 << 30)) return false;
    // the kernel addresses inputs as a 64-bit tile base plus 32-bit byte offsets that cover every image a
    // 64-pixel tile touches and all (padded) channels
    if ((int64_t)(64 / a->HW + 3) * (s.C + 64) * a->HW * 4 >= ((int64_t)1 << 32)) return false;
    a->ktiles = ceil_div(s.K, pv.tile_k());
    int groups = groups_req;
    const int most = ceil_div(tiles, pv.NW);  // one tile per wave
    if (groups <= 0) {
        // Work-groups are dealt round-robin to the 256 CUs and the longest CU decides. Candidates: grids of
        // 1..8 work-groups per CU (measured: 400 work-groups of 3.9 tiles per wave take 130 us where 512 of
        // 3.06 take 118 - the 144 CUs that get a second work-group finish last), and one tile per wave.
        // Cost of a candidate, in units of one tile of one wave: the busiest CU's tiles per SIMD (over 0.85
        // if a SIMD only ever holds one wave) plus its panel loads (~32 B/clk).
        const int per_cu = std::max(1, std::min((int)(kLdsMax / lds), 8 / pv.NW));
        const double tile_cycles = steps * 16.0 * pv.MT * 32.0;
        // Layers near or below the machine balance (~20 flop per byte) stream: there one work-group per CU is fastest
        // (measured on 128 x 64 x 56 x 56 -> 64: 40.7 us with 256 work-groups, 45.0 with 512; 128 x 64 x 27 x 27 -> 64:
        // 11.6 against 14.4), a second wave per SIMD buys nothing and every further work-group per CU costs ~8 %.
        // That holds for long layers only (six or more tiles per wave at one work-group per CU); short ones gain more
        // from the extra waves that hide their start-up latencies.
        // On maps whose pixels do not move as aligned dwordx4 the same holds further out: up to ~55 flop per byte and
        // from 2.5 tiles per wave, grids of two work-groups per CU ran 10-20 % behind grids of one on 13 x 13 and
        // 35 x 35 maps (128 x 64 x 13 x 13 -> 256: 20.3 us against 17.2; 64 x 192 x 35 x 35 -> 256: 79.4 against 69.9).
        const double flop_per_byte = 2.0 * s.C * s.K / (4.0 * (s.C + s.K));
        const bool streaming = pix != 0 ? flop_per_byte < 60.0 && 2 * (int64_t)tiles * a->ktiles >= (int64_t)5 * kNumCU * pv.NW
                                        : flop_per_byte < 32.0 && (int64_t)tiles * a->ktiles >= (int64_t)6 * kNumCU * pv.NW;
        double best = 0;
        auto consider = [&](int g) {
            g = std::max(1, std::min(g, most));
            const int64_t wgs = (int64_t)g * a->ktiles;
            if (wgs >= ((int64_t)1 << 20)) return;  // (the loop below is per work-group)
            const int stride = g * pv.NW;
            std::vector<int> load(kNumCU, 0), count(kNumCU, 0);
            for (int64_t L = 0; L < wgs; ++L) {
                const int first_wave = (int)(L / a->ktiles) * pv.NW;
                const int per_wave = first_wave < tiles ? ceil_div(tiles - first_wave, stride) : 0;
                load[L % kNumCU] += per_wave * (pv.NW / 4);
                count[L % kNumCU] += 1;
            }
            const int busiest = *std::max_element(load.begin(), load.end());
            const int most_wgs = *std::max_element(count.begin(), count.end());
            const double waves_per_simd = std::min<double>(per_cu, most_wgs) * pv.NW / 4.0;
            const double resident = std::min<double>(per_cu, most_wgs);
            const double cost = (streaming ? busiest * (1.0 + 0.08 * (resident - 1.0)) : busiest / (waves_per_simd >= 2 ? 1.0 : 0.85)) +
                                most_wgs * (lds / 32.0) / tile_cycles;
            if (groups <= 0 || cost < best * 0.999) { groups = g; best = cost; }
        };
        for (int m = 1; m <= 8; ++m) {
            const int g = std::max(1, std::min(ceil_div(kNumCU * m, a->ktiles), most));
            // first the fewest work-groups that need no more tiles per wave than g does (ties keep the first)
            // (not for streaming layers: they want every CU's memory pipeline busy)
            if (!streaming) consider(ceil_div(tiles, ceil_div(tiles, g * pv.NW) * pv.NW));
            consider(kNumCU * m / a->ktiles);
            consider(g);
        }
        consider(most);
        if (modelled) *modelled = best * tile_cycles;
    }
    groups = std::min(groups, most);
    if ((int64_t)groups * a->ktiles >= ((int64_t)1 << 31)) return false;
    a->ptiles = groups;
    a->tile_pix = pix == 2 ? per_image : 64;
    a->div_ptiles = make_fastdiv(per_image);
    a->col_shift = pix;
    a->nchunks = steps;
    a->x_items = tiles;
    a->lds_pitch = pitch;
    a->div_ktiles = make_fastdiv(a->ktiles);
    a->div_PQ = make_fastdiv(a->HW);
    a->div_row_vecs = make_fastdiv(4 * steps);
    std::memset(p, 0, sizeof(*p));
    p->kernel = CONV_KERNEL_PANEL; p->variant = variant;
    p->tile_k = pv.tile_k(); p->tile_pix = groups; p->chunk_c = 16 * pv.PD;
    p->x_vec = pix == 1 ? 1 : 4; p->w_vec = 4;
    p->lds_pitch = pitch;
    p->grid = groups * a->ktiles; p->block = pv.block(); p->lds_bytes = (int)lds;
    fill_common(s, p);
    return true;
}

// Choice of the pointwise tile shape, from sweeps: with plenty of work, 32 channels x 64 pixels per
// work-group and four channel shares (inputs are re-read through L2 by the second channel tile, which
// costs less than fewer, longer-lived waves); for small layers 16 channels per work-group and as many
// channel shares (4 or 8) as it takes to put ~4 waves on every SIMD's queue.
int pick_pointwise(const Shape& s)
{
    const int64_t pix_tiles = (int64_t)s.N * ceil_div(s.H * s.W, 64);
    const int64_t waves_v2 = pix_tiles * ceil_div(s.K, 32) * 4;
    if (waves_v2 >= 4096) return 2;  // {MT 2, WC 4}
    const int64_t groups = pix_tiles * ceil_div(s.K, 16);
    const int steps = ceil_div(s.C, 16);
    // about one 32-channel work-group per CU and 256 or more channels: eight shares of them (measured 4-18 % over the
    // 16-channel shapes on 32 x 832 x 7 x 7 -> 256, 4 x 512 x 14 x 14 -> 512, 16 x 320 x 7 x 7 -> 512)
    const int64_t groups32 = pix_tiles * ceil_div(s.K, 32);
    // (and about two per CU: 4-25 % over the other shapes on 1 x 256 x 56 x 56 -> 320, 2 x 512 x 40 x 40 -> 320)
    if (((groups32 >= 224 && groups32 <= 288) || (groups32 >= 448 && groups32 <= 576)) && steps >= 16) return 3;  // {MT 2, WC 8}
    // {1, 4} or {1, 8} shares (16 shares, 1024 threads, measured 25 % slower even on 512..832 channels); with three or
    // more steps per wave the twin that keeps four steps of loads in flight (3-7 % on 512..1024-channel N=1 layers)
    const int pick = (groups * 4 >= 1024 || steps <= 8) ? (steps >= 12 ? 15 : 0) : (steps >= 24 ? 14 : 1);
    // Every wave runs the same multiple of (channel shares x steps in flight) steps: where that rounds the layer's steps up
    // by more than 40 % (640 channels = 40 steps on the shape of 8 shares x 4 in flight: 64), the shape among these four
    // that pads least runs 12-25 % faster (timed on batch 1..4 layers with 320 and 640 channels)
    auto padded = [&](int v) { return round_up(steps, kPointwiseVariants[v].WC * kPointwiseVariants[v].PD); };
    if (padded(pick) * 10 > steps * 14) {
        int best = pick;
        for (int v : {14, 1, 15, 0})
            if (padded(v) < padded(best)) best = v;
        return best;
    }
    return pick;
}

// Panel kernel or not, from sweeps over batched 1x1 layers: it wins once there are about 700 units of
// (64-pixel tile) x (32 output channels) - roughly one per SIMD with some to spare - and loses below, where
// splitting the channels over the waves of a work-group fills the chip better. 32 channels per panel and two
// steps in flight is the best or within 3 % of it almost everywhere on maps whose pixels move as aligned dwordx4;
// on the others the four shapes are ranked by the grid each would get.
int pick_panel(const Shape& s, int x_cap, int w_cap, int y_cap)
{
    const int64_t tiles = ((int64_t)s.N * s.H * s.W + 63) / 64;
    const int pix = panel_pixel_mode(s, x_cap, y_cap);
    // Maps whose pixels do not move as aligned dwordx4 (7 x 7, 13 x 13, 27 x 27, ...): the grid model of resolve_panel
    // ranks the four shapes once each is weighted for what that model leaves out - a wave's input loads per output fall
    // with the channels of its panel, and eight waves hide more of a work-group's start than four. Weights fitted on
    // timings of the four shapes over 63 layers (batch 16..128, 256..512 channels, 64..384 filters): the pick is
    // 0.9 % (single dwords) and 1.5 % (tiles cut per image) behind the measured best in the geometric mean, 6 % and 13 %
    // at worst, where fixed thresholds on the work were 7 % and 3 % behind, 35 % and 26 % at worst (a grid of
    // 64-channel panels two work-groups over a multiple of the CU count runs a whole extra round).
    auto ranked = [&]() {
        static constexpr int kShapes[4] = {5, 7, 6, 8};
        static constexpr double kWeight[2][4] = {{1.2, 1.0, 0.75, 0.9}, {1.5, 1.0, 0.92, 1.08}};
        int pick = -1;
        double least = 0;
        for (int i = 0; i < 4; ++i) {
            conv_plan_t tp;
            KernelArgs ta;
            double cycles = 0;
            if (!resolve_panel(s, kShapes[i], 0, x_cap, w_cap, y_cap, &tp, &ta, &cycles)) continue;
            cycles *= kWeight[pix - 1][i];
            if (pick < 0 || cycles < least) { pick = kShapes[i]; least = cycles; }
        }
        return pick;
    };
    if (tiles * ceil_div(s.K, 32) < 704) {
        // fewer 32-channel units than that, but 512 or more 16-channel ones: 16 channels per panel still beat the
        // channel-splitting kernel by 5-25 % in the sweeps (deep layers on 7..14-pixel maps at batch 8..32)
        // (at batch 1 only with 256 or more input channels: with fewer the resident filters save too little to pay for
        // the panel's start-up)
        if ((s.N > 1 || s.C >= 256) && tiles * ceil_div(s.K, 16) >= 512 && 16 * (round_up(s.C, 64) + 4) * 4 <= kLdsMax) {
            // ... unless one tile per wave makes a few work-groups more than the chip has CUs: the CUs that get two of them
            // take twice as long (260 work-groups on 1 x 256 x 56 x 56 -> 320 and 2 x 512 x 40 x 40 -> 320: 12.4 and 20.4 us,
            // where eight channel shares of the pointwise kernel take 9.1 and 14.8)
            const int64_t one_tile_each = (int64_t)ceil_div(s.K, 16) * ((tiles + 3) / 4);
            if (pix == 0 && one_tile_each > kNumCU && one_tile_each <= kNumCU + kNumCU / 8) return -1;
            return pix != 0 ? ranked() : 5;  // {1, 4, 4}
        }
        return -1;
    }
    if (pix != 0) return ranked();
    const int c64 = round_up(s.C, 32);
    // Aligned dwordx4 pixels: timings of every panel shape on 27 such layers with 256 or more filters put the 32-channel
    // panel ahead of the 64-channel one on all of them (8.5 % in the geometric mean, up to 32 %).
    // A 32-channel panel of more than half the LDS leaves one work-group per CU: eight waves then (two per SIMD)
    // when every CU still gets a work-group whose waves all have a tile
    if (32 * (c64 + 4) * 4 > kLdsMax / 2 && 32 * (c64 + 4) * 4 <= kLdsMax &&
        static_cast<long long>(ceil_div(s.K, 32)) * ceil_div(tiles, 8) >= kNumCU) return 8;                    // {2, 8, 2}
    if (32 * (c64 + 4) * 4 <= kLdsMax) return 7;                                                                // {2, 4, 2}
    if (16 * (round_up(s.C, 64) + 4) * 4 <= kLdsMax) return 5;                                                  // {1, 4, 4}
    return -1;
}

void resolve_generic(const Shape& s, conv_plan_t* p, KernelArgs* a)
{
    base_args(s, a);
    std::memset(p, 0, sizeof(*p));
    p->kernel = CONV_KERNEL_GENERIC;
    p->block = 256;
    const int64_t outputs = (int64_t)a->total_pix * s.K;
    p->grid = (int)std::min<int64_t>((outputs + 255) / 256, (int64_t)kNumCU * 64);
    p->tile_k = 1; p->tile_pix = 256; p->x_vec = 1; p->w_vec = 1;
    fill_common(s, p);
}

// Estimated cycles of a tap mapping on 256 CUs, fitted to timings of every tile shape x pixel tile over the 3x3
// and 5x5 layers of the shape grid (batch 1..128, maps 7..224) and over ~80 random layers off it: the mapping it
// picks is on average within 2 % of the best one measured (worst case 1.22x). Work-groups are dealt round-robin,
// so the busiest CU runs cu = ceil(grid / 256) of them, wpc at a time (registers, LDS). Per chunk that CU takes the
// longest of
//   all its matrix work          (cu x per-SIMD cycles: 32 per MFMA plus ~110 per staging slot of a thread - the
//                                 load, the LDS store and their address arithmetic take issue slots from the
//                                 matrix instructions - or ~25 per slot of the direct loader, which has no LDS
//                                 store, no masking and no address arithmetic (40 with loader waves: their traffic
//                                 into LDS is still the multiplying waves' business); issue efficiency 0.88 with
//                                 two or more waves per SIMD, 0.64 with one),
//   its latency chains           (one per batch of co-resident work-groups: ~750 cycles from a staging load's
//                                 issue to its data sitting in LDS behind the barrier - 1500 for the direct loader,
//                                 whose loads run one chunk ahead instead of two - plus the chunk's own work), and
//   its staging traffic          (halo rows + filter block into LDS, ~16 B/clk per CU);
// every batch of co-resident work-groups adds ~12000 cycles of prologue and epilogue (first loads, LDS fill; 17000
// with the direct loader, which cannot start chunk 1 before chunk 0 has landed), every work-group its reduction tree
// and stores (~32 B/clk), the launch ~5000 and the dispatcher ~8 per work-group. Constants fitted to timings of every
// tile shape x candidate pixel tile x loader on the 3x3 / 5x5 layers of the shape grid and on 84 random layers off it;
// the direct loader's (once 50 and 80 per slot, 20000 per batch) were lowered by hand when its loads became buffer loads
// with constant offsets, and checked against the mappings conv_fwd_find measures on the same layers (default / found
// 1.03 in the geometric mean before and after).
double tap_cost(const conv_plan_t& p, const KernelArgs& a, const TapVariant& tv, int RS)
{
    const int by_regs = std::max(1, tv.occ * 256 / tv.block());
    const int by_lds = std::max(1, kLdsMax / std::max(p.lds_bytes, 1));
    const int wpc = std::min(std::min(by_regs, by_lds), 8);  // work-groups sharing a CU
    const int cu = ceil_div(p.grid, kNumCU);                 // work-groups of the busiest CU
    const int batches = ceil_div(cu, wpc);
    const double waves_per_simd = tv.block() / 256.0;
    const double eff = std::min(wpc, cu) * waves_per_simd >= 2 ? 0.88 : 0.64;
    // staging slots that run per chunk: the loader build the launcher will take, not just the slots with data
    const int x_slots = ceil_div(a.direct ? tv.xs_direct(p.x_vec) : tv.xs(p.x_vec), tap_x_slot_divisor(tv, p.x_vec, p.w_vec, a.x_items, a.direct != 0));
    const int slots = x_slots + (a.direct ? tv.wslots_direct(RS) : ceil_div(tv.tile_k() * tv.chunk_c() * RS / p.w_vec, tv.block()));
    // (with loader waves the slots are not the multiplying waves' business, but their traffic into LDS still is: measured
    // 2-4 % under the register loader on deep layers)
    const double work = waves_per_simd * ((double)tv.tap_cycles() * tv.GPC * RS + (a.direct == 2 ? 40.0 : a.direct ? 25.0 : 110.0) * slots);  // per SIMD, chunk, work-group
    const double staged = 4.0 * ((double)tv.chunk_c() * a.lds_rows * a.W + (double)tv.tile_k() * tv.chunk_c() * RS);
    const double chunk = std::max(std::max(cu * work / eff, batches * ((a.direct ? 1500.0 : 750.0) + work)), cu * staged / 16.0);
    // cross-wave reduction: per round of the tree every tile goes through LDS once each way (~8 cycles per 64 B with
    // the waves of a round writing at once, then reading), plus ~1000 cycles of barriers
    const double tree = tv.WC > 1 ? tv.MT * tv.NT * 128.0 * tv.WK * tv.WP * std::log2((double)tv.WC) + 1000.0 : 0.0;
    const double cycles = a.nchunks * chunk + batches * (a.direct ? 17000.0 : 12000.0) + cu * (4.0 * tv.tile_k() * p.tile_pix / 32.0 + tree) + 5000.0 +
                          8.0 * p.grid;
    // Tile shapes compiled for three or four waves per SIMD measure 3-5 % faster per step of occupancy than their
    // two-wave twins even where the model sees no difference (all work-groups co-resident either way).
    // (between pixel tiles that cost the same otherwise, the one whose halo tile has fewer rows: a tile of 98 pixels of a
    // 14 x 14 map against one of 100 - 8 x 512 x 14 x 14 -> 512 runs 5 % faster on it)
    const double tie_break = 1.0 + 1e-3 * a.lds_rows / std::max(1, p.tile_pix);
    return cycles * (1.0 - 0.05 * std::max(0, tv.occ - 2)) * tie_break;
}

// The deep direct loader (a ring of four staging copies) pays where a launch is one or two rounds of work-groups whose
// chunks are shorter than a load takes: every mapping of the 3x3 / 5x5 layers of the shape grid with batch <= 16 and of
// 18 layers off it was timed with each loader, and against the model's choice these substitutions did not lose:
//  - the 16 x 64 shapes (2 and its four-wave twin 24), four chunks or more, at most 400 work-groups (256 where rows move
//    as dwordx4: two layers of 300 work-groups lost 8 %; 512 with 256 channels or more): shape 2 with the deep ring,
//    0.5-22 % faster (1 x 64 x 56 x 56 -> 64: 8.9 -> 7.7 us; 8 x 256 x 14 x 14 -> 256: 35.4 -> 30.9 us; 2 x 320 x 17 x 17
//    -> 768: 45.3 -> 37.1 us);
//  - the 16 x 32 shapes with eight channel shares (18 and 20), at most 256 work-groups, 256 channels or more, rows that
//    do not move as dwordx4: shape 18 with the deep ring, 3-10 % faster (1 x 512 x 14 x 14 -> 512: 23.4 -> 20.8 us; with
//    dwordx4 rows the plain direct loader is already the choice and the ring lost 4 % on 1 x 320 x 20 x 20 -> 256);
//    where four copies of its 32-channel chunks do not fit LDS (maps wider than ~30), shape 13 (16-channel chunks) with
//    the ring instead (1 x 448 x 35 x 35 -> 48: 29.2 -> 25.1 us). Batch 1 and 2 only: every such layer timed had one of
//    them but 16 x 320 x 7 x 7 -> 160, which lost 10 %.
// Elsewhere (more rounds of work-groups, short reductions, the four-share shapes as the model's own choice) it lost as
// often as it won, by up to 2x where the ring's LDS keeps a second work-group off the CU.
void prefer_deep_ring(const Shape& s, int x_cap, int w_cap, conv_plan_t* p, KernelArgs* a)
{
    int variant = -1, fallback = -1;
    const bool wide_rows = s.W % 4 == 0;
    if ((p->variant == 2 || p->variant == 24) && s.C >= 4 * kTapVariants[2].chunk_c() &&
        p->grid <= (wide_rows ? 256 : s.C >= 256 ? 512 : 400))
        variant = 2;
    if ((p->variant == 18 || p->variant == 20) && p->grid <= 256 && s.C >= 256 && !wide_rows && s.N <= 2) {
        variant = 18; fallback = 13;
    }
    if (variant < 0 || p->c_splits > 1) return;
    conv_plan_t dp;
    KernelArgs da;
    for (int v : {variant, fallback})
        if (v >= 0 && resolve_tap(s, v, p->tile_pix, 0, x_cap, w_cap, &dp, &da, 1, CONV_LOADER_DIRECT_DEEP) && dp.grid == p->grid) {
            *p = dp; *a = da;
            return;
        }
}

// conv_fwd plans on every call; remember recent shapes so a launch costs a table lookup.
struct CacheEntry {
    Shape s;
    int x_cap, w_cap, y_cap;
    conv_plan_t p;
    KernelArgs a;
};
std::mutex g_cache_mutex;
std::vector<CacheEntry> g_cache;
constexpr size_t kCacheEntries = 64;

bool same_shape(const Shape& a, const Shape& b) { return std::memcmp(&a, &b, sizeof(Shape)) == 0; }

int plan_shape_uncached(const Shape& s, int x_cap, int w_cap, int y_cap, conv_plan_t* p, KernelArgs* a);

int plan_shape(const Shape& s, int x_cap, int w_cap, int y_cap, conv_plan_t* p, KernelArgs* a)
{
    {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        for (const CacheEntry& e : g_cache)
            if (same_shape(e.s, s) && e.x_cap == x_cap && e.w_cap == w_cap && e.y_cap == y_cap) {
                *p = e.p; *a = e.a;
                return CONV_OK;
            }
    }
    const int rc = plan_shape_uncached(s, x_cap, w_cap, y_cap, p, a);
    if (rc == CONV_OK) {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        if (g_cache.size() >= kCacheEntries) g_cache.erase(g_cache.begin());
        g_cache.push_back(CacheEntry{s, x_cap, w_cap, y_cap, *p, *a});
    }
    return rc;
}

// Candidate pixel tiles of a tap tile shape: full capacity, an even split, whole images, whole rows (or the largest part that
// divides a row longer than the tile), halves, quarters.
int tap_tile_candidates(const Shape& s, const TapVariant& tv, int (&cands)[10])
{
    const int PQ = s.P * s.Q;
    const int64_t total = (int64_t)s.N * PQ;
    const int cap = tv.max_pix();
    int nc = 0;
    cands[nc++] = (int)std::min<int64_t>(cap, total);
    cands[nc++] = (int)((total + (total + cap - 1) / cap - 1) / ((total + cap - 1) / cap));
    if (PQ <= cap) cands[nc++] = cap / PQ * PQ;
    if (PQ > cap) {
        const int parts = ceil_div(PQ, cap);
        if (PQ % parts == 0) cands[nc++] = PQ / parts;
        for (int d = parts; d <= std::min(PQ, parts + 8); ++d)
            if (PQ % d == 0) { cands[nc++] = PQ / d; break; }
    }
    if (s.Q <= cap) cands[nc++] = cap / s.Q * s.Q;
    else {
        // rows longer than a tile: the largest part of a row that divides it (tiles then never straddle two rows, which would
        // cost a fourth halo row - on maps a thousand pixels wide the difference between fitting LDS and not)
        const int parts = ceil_div(s.Q, cap);
        for (int d = parts; d <= std::min(s.Q, parts + 16); ++d)
            if (s.Q % d == 0) { cands[nc++] = s.Q / d; break; }
    }
    if (cap >= 32) cands[nc++] = cap / 2;
    if (cap >= 64) cands[nc++] = cap / 4;
    return nc;
}

int plan_shape_uncached(const Shape& s, int x_cap, int w_cap, int y_cap, conv_plan_t* p, KernelArgs* a)
{
    if (pointwise_ok(s, x_cap, w_cap, y_cap)) {
        const int pv = pick_panel(s, x_cap, w_cap, y_cap);
        // Small layers with few input channels (under ~150 MFLOP, C <= 80, pixels that move as dwordx4) have nothing
        // to share between waves: the register-streaming shape whose four waves each take 64 pixels and all channels
        // beats the panel kernel by 10-20 % there (measured on 64 x 48 x 14 x 14 -> 64, 4 x 16 x 80 x 80 -> 48,
        // 1 x 32 x 112 x 112 -> 64, ...).
        // (with 32 channels or fewer it also wins on maps whose pixels move as dwords, up to ~300 MFLOP, as long as its
        // 256-pixel tiles waste less than 30 % of an image: 64 x 24 x 35 x 35 -> 48: 12.7 -> 9.6 us)
        const int64_t hw = (int64_t)s.H * s.W;
        const double pw_flops = 2.0 * s.N * s.H * s.W * s.C * s.K;
        // (and up to ~120 MFLOP whatever its tiles waste: on 7 x 7 ... 17 x 17 maps at batch 1..8 it matches the other shapes
        // where all of them sit at the launch floor and is 10-25 % faster from ~300 work-groups of theirs on,
        // 8 x 16 x 13 x 13 -> 768: 6.2 -> 4.8 us, 2 x 32 x 17 x 17 -> 768: 5.1 -> 3.7 us)
        const bool small_thin = (s.C <= 80 && hw % 4 == 0 && pw_flops <= 1.5e8) ||
                                (s.C <= 32 && pw_flops <= 3e8 && (hw + 255) / 256 * 256 * 10 <= hw * 13) ||
                                (s.C <= 32 && pw_flops <= 1.2e8);
        if (small_thin && resolve_pointwise(s, 8, x_cap, w_cap, y_cap, p, a)) return CONV_OK;
        if (pv >= 0 && resolve_panel(s, pv, 0, x_cap, w_cap, y_cap, p, a)) return CONV_OK;
        if (resolve_pointwise(s, pick_pointwise(s), x_cap, w_cap, y_cap, p, a)) return CONV_OK;
    }
    if (tap_rs_index(s) >= 0) {
        bool found = false;
        double best = 0;
        for (int v = 0; v < kNumTapVariants; ++v) {
            const TapVariant tv = kTapVariants[v];
            // The shapes with eight and sixteen channel shares are for deep layers: on layers of less than two of their
            // chunks (24..80 channels on the 64-channel chunks of shape 17) most of their waves multiply padding, which the
            // model does not see - five of the six largest misses on random layers off the grid (1.20-1.36x).
            if (tv.WC >= 8 && s.C < 2 * tv.chunk_c()) continue;
            int cands[10];
            const int nc = tap_tile_candidates(s, tv, cands);
            for (int i = 0; i < nc; ++i) {
                conv_plan_t cp;
                KernelArgs ca;
                if (cands[i] < 1 || !resolve_tap(s, v, cands[i], 0, x_cap, w_cap, &cp, &ca)) continue;
                const double c = tap_cost(cp, ca, tv, s.R * s.S);
                if (!found || c < best * 0.999) {
                    found = true; best = c; *p = cp; *a = ca;
                }
            }
        }
        if (found) {
            prefer_deep_ring(s, x_cap, w_cap, p, a);
            return CONV_OK;
        }
    }
    resolve_generic(s, p, a);
    return CONV_OK;
}

// Channel-splitting mode: as the tap branch of plan_shape_uncached, with the number of channel shares as a third
// search dimension. The model sees a share as a layer with fewer chunks and more work-groups; the second pass costs
// a dependent launch (~6000 cycles; 10000 until the direct loader's buffer loads made the unsplit kernels faster than
// the model's picture of a split one), ~500 per share and the traffic of the partial outputs (fitted to timings of
// every tile shape x pixel tile x share count on the batch-1 layers of the shape grid; shares that would put more
// than two work-groups on a CU never won there and are not considered).
constexpr double kSplitPassCycles = 6000.0;
constexpr double kSplitShareCycles = 500.0;
constexpr int kSplitCandidates[] = {1, 2, 3, 4, 6, 8, 12, 16};
void search_split_plans(const Shape& s, int x_cap, int w_cap, conv_plan_t* p, KernelArgs* a);
double split_pass_cycles(int splits, int K, int total_pix)
{
    // (the partial outputs are written, read back and the sum written: at ~8 B/clk per CU, the rate a streaming kernel
    // sustains on this GPU; half of that was assumed at first and made two-share splits of 30-50 us layers look 5 % better
    // than they measured)
    return kSplitPassCycles + kSplitShareCycles * splits + 4.0 * (splits + 1) * K * total_pix / (kNumCU * 8.0);
}
std::vector<CacheEntry> g_split_cache;  // under g_cache_mutex, like g_cache

int plan_split_shape(const Shape& s, int x_cap, int w_cap, int y_cap, conv_plan_t* p, KernelArgs* a)
{
    {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        for (const CacheEntry& e : g_split_cache)
            if (same_shape(e.s, s) && e.x_cap == x_cap && e.w_cap == w_cap && e.y_cap == y_cap) {
                *p = e.p; *a = e.a;
                return CONV_OK;
            }
    }
    if (int rc = plan_shape(s, x_cap, w_cap, y_cap, p, a)) return rc;
    // Where the single-kernel default already runs the deep ring on rows that move as dwordx2 or dwordx4, shares stopped
    // paying once it existed (8 x 256 x 14 x 14 -> 256: 1.14x before, 0.99x after; 1 x 512 x 14 x 14 -> 512: 1.08x -> 0.96x);
    // on odd widths, where the single kernel's dword loads are bound by the address path, they still gain 12-18 %.
    const bool ring_suffices = p->kernel == CONV_KERNEL_TAP && p->loader == CONV_LOADER_DIRECT_DEEP && s.W % 2 == 0;
    if (p->kernel == CONV_KERNEL_TAP && !ring_suffices) search_split_plans(s, x_cap, w_cap, p, a);
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    if (g_split_cache.size() >= kCacheEntries) g_split_cache.erase(g_split_cache.begin());
    g_split_cache.push_back(CacheEntry{s, x_cap, w_cap, y_cap, *p, *a});
    return CONV_OK;
}

void search_split_plans(const Shape& s, int x_cap, int w_cap, conv_plan_t* p, KernelArgs* a)
{
    // the default plan stays unless a mapping with shares is modelled at least 4 % faster than every mapping without
    double best_whole = 0, best_split = 0;
    bool have_whole = false, have_split = false;
    conv_plan_t sp;
    KernelArgs sa;
    for (int v = 0; v < kNumTapVariants; ++v) {
        const TapVariant tv = kTapVariants[v];
        int cands[10];
        const int nc = tap_tile_candidates(s, tv, cands);
        for (int i = 0; i < nc; ++i) {
            for (int splits : kSplitCandidates) {
                conv_plan_t cp;
                KernelArgs ca;
                if (cands[i] < 1 || !resolve_tap(s, v, cands[i], 0, x_cap, w_cap, &cp, &ca, splits)) continue;
                if (cp.c_splits != splits) continue;  // fewer chunks than shares: same as a smaller candidate
                double c = tap_cost(cp, ca, tv, s.R * s.S);
                if (splits == 1) {
                    if (!have_whole || c < best_whole) { have_whole = true; best_whole = c; }
                    continue;
                }
                if (cp.grid > 2 * kNumCU) continue;
                c += split_pass_cycles(splits, s.K, ca.total_pix);
                // (two shares gain least and miss most: three 5x5 layers of 30-50 us measured 4-9 % slower split in two
                // where the model saw 4-6 % gain)
                if (splits == 2) c *= 1.04;
                if (!have_split || c < best_split * 0.999) {
                    have_split = true; best_split = c; sp = cp; sa = ca;
                }
            }
        }
    }
    if (have_split && (!have_whole || best_split < 0.96 * best_whole)) {
        *p = sp; *a = sa;
    }
}

int record_hip(hipError_t e)
{
    if (e == hipSuccess) return CONV_OK;
    g_hip_error = std::string(hipGetErrorName(e)) + ": " + hipGetErrorString(e);
    return CONV_E_HIP;
}

int launch(const conv_plan_t& p, KernelArgs& a, const Shape& s, const float* x, const float* w, float* y,
           const float* bias = nullptr, int relu = 0)
{
    a.x = x; a.w = w; a.y = y; a.bias = bias; a.relu = relu;
    hipStream_t stream = g_stream;
    if (p.kernel == CONV_KERNEL_TAP)
        return record_hip(launch_tap(tap_rs_index(s), p.variant, p.x_vec, p.w_vec, p.grid, p.lds_bytes, stream, a));
    if (p.kernel == CONV_KERNEL_POINTWISE) return record_hip(launch_pointwise(p.variant, p.x_vec, p.grid, p.lds_bytes, stream, a));
    if (p.kernel == CONV_KERNEL_PANEL) return record_hip(launch_panel(p.variant, a.col_shift, p.grid, p.lds_bytes, stream, a));
    if (p.kernel == CONV_KERNEL_GENERIC) return record_hip(launch_generic(p.grid, p.block, stream, a));
    return CONV_E_PLAN;
}

void pointer_caps(const float* x, const float* w, const float* y, int* x_cap, int* w_cap, int* y_cap)
{
    const uintptr_t xa = reinterpret_cast<uintptr_t>(x), wa = reinterpret_cast<uintptr_t>(w);
    *x_cap = xa % 16 == 0 ? 4 : xa % 8 == 0 ? 2 : 1;
    *w_cap = wa % 16 == 0 ? 4 : 1;
    *y_cap = reinterpret_cast<uintptr_t>(y) % 16 == 0 ? 4 : 1;
}

}  // namespace
}  // namespace convfwd

using namespace convfwd;

extern "C" int conv_fwd_plan(int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w, conv_plan_t* out)
{
    if (!out) return CONV_E_NULL;
    Shape s;
    if (int rc = validate(N, C, H, W, K, R, S, pad_h, pad_w, &s)) return rc;
    KernelArgs a;
    return plan_shape(s, 4, 4, 4, out, &a);
}

extern "C" int conv_fwd(const float* x, const float* w, float* y, int N, int C, int H, int W, int K, int R, int S,
                        int pad_h, int pad_w)
{
    if (!x || !w || !y) return CONV_E_NULL;
    Shape s;
    if (int rc = validate(N, C, H, W, K, R, S, pad_h, pad_w, &s)) return rc;
    int x_cap, w_cap, y_cap;
    pointer_caps(x, w, y, &x_cap, &w_cap, &y_cap);
    conv_plan_t p;
    KernelArgs a;
    if (int rc = plan_shape(s, x_cap, w_cap, y_cap, &p, &a)) return rc;
    return launch(p, a, s, x, w, y);
}

// Shared by conv_fwd_planned and conv_fwd_bias_relu: resolve the requested mapping (or plan, when none is
// requested) and enqueue the kernel.
// A caller's request (family, tile shape, pixel tile or work-groups per channel tile, shares) resolved into a launch;
// remembered per shape and request, so that repeated planned calls cost a table lookup like conv_fwd's.
struct RequestEntry {
    Shape s;
    int x_cap, w_cap, y_cap;
    int kernel, variant, tile_pix, chunk_c, c_splits, loader, order, k_group;
    conv_plan_t p;
    KernelArgs a;
};
static std::vector<RequestEntry> g_request_cache;  // under g_cache_mutex

static int resolve_request(const Shape& s, int x_cap, int w_cap, int y_cap, const conv_plan_t& req, bool may_split,
                           conv_plan_t* p, KernelArgs* a)
{
    if (req.c_splits > 1 && (!may_split || req.kernel != CONV_KERNEL_TAP))
        return CONV_E_PLAN;  // only the tap family splits channels across work-groups, and only with a workspace
    {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        for (const RequestEntry& e : g_request_cache)
            if (same_shape(e.s, s) && e.x_cap == x_cap && e.w_cap == w_cap && e.y_cap == y_cap && e.kernel == req.kernel &&
                e.variant == req.variant && e.tile_pix == req.tile_pix && e.chunk_c == req.chunk_c && e.c_splits == req.c_splits &&
                e.loader == req.loader && e.order == req.order && e.k_group == req.k_group) {
                *p = e.p; *a = e.a;
                return CONV_OK;
            }
    }
    if (req.kernel == CONV_KERNEL_POINTWISE) {
        if (!resolve_pointwise(s, req.variant, x_cap, w_cap, y_cap, p, a)) return CONV_E_PLAN;
    } else if (req.kernel == CONV_KERNEL_PANEL) {
        if (req.tile_pix < 0 || !resolve_panel(s, req.variant, req.tile_pix, x_cap, w_cap, y_cap, p, a)) return CONV_E_PLAN;
    } else if (req.kernel == CONV_KERNEL_GENERIC) {
        resolve_generic(s, p, a);
    } else if (req.kernel == CONV_KERNEL_TAP) {
        if (req.tile_pix < 0 || req.chunk_c < 0 || req.c_splits < 0) return CONV_E_PLAN;
        if (!resolve_tap(s, req.variant, req.tile_pix, req.chunk_c, x_cap, w_cap, p, a, std::max(1, req.c_splits), req.loader, req.order, req.k_group))
            return CONV_E_PLAN;
    } else {
        return CONV_E_PLAN;
    }
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    if (g_request_cache.size() >= kCacheEntries) g_request_cache.erase(g_request_cache.begin());
    g_request_cache.push_back(RequestEntry{s, x_cap, w_cap, y_cap, req.kernel, req.variant, req.tile_pix, req.chunk_c,
                                           req.c_splits, req.loader, req.order, req.k_group, *p, *a});
    return CONV_OK;
}

static int run_planned(const float* x, const float* w, const float* bias, float* y, int N, int C, int H, int W, int K,
                       int R, int S, int pad_h, int pad_w, int relu, const conv_plan_t* plan, conv_plan_t* resolved,
                       bool may_split = false, float* workspace = nullptr, long long workspace_bytes = 0,
                       bool static_workspace = false)
{
    if (!x || !w || !y) return CONV_E_NULL;
    Shape s;
    if (int rc = validate(N, C, H, W, K, R, S, pad_h, pad_w, &s)) return rc;
    int x_cap, w_cap, y_cap;
    pointer_caps(x, w, y, &x_cap, &w_cap, &y_cap);
    conv_plan_t p;
    KernelArgs a;
    if (!plan) {
        if (int rc = may_split ? plan_split_shape(s, x_cap, w_cap, y_cap, &p, &a) : plan_shape(s, x_cap, w_cap, y_cap, &p, &a))
            return rc;
    } else {
        if (int rc = resolve_request(s, x_cap, w_cap, y_cap, *plan, may_split, &p, &a)) return rc;
    }
    if (resolved) *resolved = p;
    if (p.c_splits <= 1) return launch(p, a, s, x, w, y, bias, relu);
    // channel shares: the tap kernel writes c_splits partial outputs into the workspace, a second kernel adds them
    if (static_workspace) {
        // the library's own static array takes the caller's place; larger layers are refused, never allocated for
        if (p.workspace_bytes > kStaticScratchBytes) return CONV_E_WORKSPACE;
        if (int rc = record_hip(static_scratch(&workspace))) return rc;
        workspace_bytes = kStaticScratchBytes;
    }
    if (!workspace) return CONV_E_NULL;
    if (workspace_bytes < p.workspace_bytes) return CONV_E_WORKSPACE;
    if (int rc = launch(p, a, s, x, w, workspace)) return rc;
    return record_hip(launch_split_reduce(workspace, y, bias, relu, p.c_splits, s.K * a.total_pix, a.PQ, s.K, g_stream));
}

extern "C" int conv_fwd_plan_request(int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w,
                                     const conv_plan_t* request, conv_plan_t* resolved, double* model_cycles)
{
    if (!request || !resolved) return CONV_E_NULL;
    Shape s;
    if (int rc = validate(N, C, H, W, K, R, S, pad_h, pad_w, &s)) return rc;
    KernelArgs a;
    if (int rc = resolve_request(s, 4, 4, 4, *request, true, resolved, &a)) return rc;
    if (model_cycles) {
        *model_cycles = 0.0;
        if (resolved->kernel == CONV_KERNEL_TAP) {
            *model_cycles = tap_cost(*resolved, a, kTapVariants[resolved->variant], s.R * s.S);
            if (resolved->c_splits > 1) *model_cycles += split_pass_cycles(resolved->c_splits, s.K, a.total_pix);
        }
    }
    return CONV_OK;
}

extern "C" int conv_fwd_plan_split_c(int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w, conv_plan_t* out)
{
    if (!out) return CONV_E_NULL;
    Shape s;
    if (int rc = validate(N, C, H, W, K, R, S, pad_h, pad_w, &s)) return rc;
    KernelArgs a;
    return plan_split_shape(s, 4, 4, 4, out, &a);
}

extern "C" int conv_fwd_split_c(const float* x, const float* w, const float* bias, float* y, float* workspace,
                                long long workspace_bytes, int N, int C, int H, int W, int K, int R, int S, int pad_h,
                                int pad_w, int relu, const conv_plan_t* plan, conv_plan_t* resolved)
{
    return run_planned(x, w, bias, y, N, C, H, W, K, R, S, pad_h, pad_w, relu != 0, plan, resolved, true, workspace,
                       workspace_bytes);
}

static_assert(kStaticScratchBytes == CONV_STATIC_SCRATCH_BYTES, "header and library disagree on the static scratch size");
extern "C" int conv_fwd_split_c_static(const float* x, const float* w, const float* bias, float* y, int N, int C, int H, int W,
                                       int K, int R, int S, int pad_h, int pad_w, int relu, const conv_plan_t* plan,
                                       conv_plan_t* resolved)
{
    return run_planned(x, w, bias, y, N, C, H, W, K, R, S, pad_h, pad_w, relu != 0, plan, resolved, true, nullptr, 0, true);
}

extern "C" int conv_fwd_planned(const float* x, const float* w, float* y, int N, int C, int H, int W, int K, int R,
                                int S, int pad_h, int pad_w, const conv_plan_t* plan, conv_plan_t* resolved)
{
    if (!plan) return CONV_E_NULL;
    return run_planned(x, w, nullptr, y, N, C, H, W, K, R, S, pad_h, pad_w, 0, plan, resolved);
}

extern "C" int conv_fwd_bias_relu(const float* x, const float* w, const float* bias, float* y, int N, int C, int H, int W,
                                  int K, int R, int S, int pad_h, int pad_w, int relu, const conv_plan_t* plan,
                                  conv_plan_t* resolved)
{
    return run_planned(x, w, bias, y, N, C, H, W, K, R, S, pad_h, pad_w, relu != 0, plan, resolved);
}

// Every mapping worth timing for a layer: all pointwise and panel shapes (panel: with the planner's grid and with one
// and two work-groups per CU), every tap shape x candidate pixel tile whose modelled cost is within 2.5x of the best
// modelled one, or the generic kernel.
struct Candidate {
    conv_plan_t p;
    KernelArgs a;
    double model;  // tap family: modelled cycles; 0 elsewhere
};

static void enumerate_candidates(const Shape& s, int x_cap, int w_cap, int y_cap, std::vector<Candidate>* out)
{
    Candidate c;
    c.model = 0;
    if (pointwise_ok(s, x_cap, w_cap, y_cap)) {
        for (int v = 0; v < kNumPointwiseVariants; ++v)
            if (resolve_pointwise(s, v, x_cap, w_cap, y_cap, &c.p, &c.a)) out->push_back(c);
        for (int v = 0; v < kNumPanelVariants; ++v) {
            if (!resolve_panel(s, v, 0, x_cap, w_cap, y_cap, &c.p, &c.a)) continue;
            out->push_back(c);
            // besides the planner's grid: one and two work-groups per CU
            const int planned = c.p.tile_pix, ktiles = c.a.ktiles;
            for (int per_cu = 1; per_cu <= 2; ++per_cu) {
                const int groups = std::max(1, ceil_div(kNumCU * per_cu, ktiles));
                if (groups != planned && resolve_panel(s, v, groups, x_cap, w_cap, y_cap, &c.p, &c.a) && c.p.tile_pix != planned)
                    out->push_back(c);
            }
        }
    }
    if (tap_rs_index(s) >= 0) {
        std::vector<Candidate> taps;
        double best = 0;
        for (int v = 0; v < kNumTapVariants; ++v) {
            const TapVariant tv = kTapVariants[v];
            int cands[10];
            const int nc = tap_tile_candidates(s, tv, cands);
            for (int i = 0; i < nc; ++i) {
                bool seen = false;
                for (int k = 0; k < i; ++k) seen = seen || cands[k] == cands[i];
                if (seen || cands[i] < 1) continue;
                for (int loader = CONV_LOADER_REGISTERS; loader <= CONV_LOADER_DIRECT_DEEP; ++loader) {  // each one that can run
                    if (!resolve_tap(s, v, cands[i], 0, x_cap, w_cap, &c.p, &c.a, 1, loader)) continue;
                    c.model = tap_cost(c.p, c.a, tv, s.R * s.S);
                    if (taps.empty() || c.model < best) best = c.model;
                    taps.push_back(c);
                }
            }
        }
        for (const Candidate& t : taps)
            if (t.model <= 2.5 * best) out->push_back(t);
    }
    if (out->empty()) {
        resolve_generic(s, &c.p, &c.a);
        c.model = 0;
        out->push_back(c);
    }
}

extern "C" int conv_fwd_find(const float* x, const float* w, float* y, int N, int C, int H, int W, int K, int R, int S,
                             int pad_h, int pad_w, void* flush, long long flush_bytes, conv_plan_t* best_plan,
                             float* best_us)
{
    if (!x || !w || !y) return CONV_E_NULL;
    Shape s;
    if (int rc = validate(N, C, H, W, K, R, S, pad_h, pad_w, &s)) return rc;
    int x_cap, w_cap, y_cap;
    pointer_caps(x, w, y, &x_cap, &w_cap, &y_cap);
    const bool cold = flush && flush_bytes >= (1 << 20) && reinterpret_cast<uintptr_t>(flush) % 16 == 0;
    std::vector<Candidate> cands;
    enumerate_candidates(s, x_cap, w_cap, y_cap, &cands);

    hipStream_t stream = g_stream;
    hipEvent_t t0, t1;
    if (int rc = record_hip(hipEventCreate(&t0))) return rc;
    if (int rc = record_hip(hipEventCreate(&t1))) { (void)hipEventDestroy(t0); return rc; }
    int best = -1, rc_last = CONV_E_PLAN;
    float best_ms = 0.f;
    for (size_t i = 0; i < cands.size(); ++i) {
        Candidate& c = cands[i];
        int rc = launch(c.p, c.a, s, x, w, y);  // warm-up: kernel attributes, instruction caches
        float ms = 0.f;
        if (cold) {
            // three single launches, each after the scratch buffer has been streamed through the caches; the fastest counts
            for (int rep = 0; rep < 3 && rc == CONV_OK; ++rep) {
                float one = 0.f;
                rc = record_hip(launch_scratch_fill(flush, flush_bytes, stream));
                if (rc == CONV_OK) rc = record_hip(hipEventRecord(t0, stream));
                if (rc == CONV_OK) rc = launch(c.p, c.a, s, x, w, y);
                if (rc == CONV_OK) rc = record_hip(hipEventRecord(t1, stream));
                if (rc == CONV_OK) rc = record_hip(hipEventSynchronize(t1));
                if (rc == CONV_OK) rc = record_hip(hipEventElapsedTime(&one, t0, t1));
                ms = rep == 0 ? one : std::min(ms, one);
            }
        } else {
            // one launch timed alone to size the batch, then a batch of 2..16
            for (int pass = 0; pass < 2 && rc == CONV_OK; ++pass) {
                const int reps = pass == 0 ? 1 : std::max(2, std::min(16, (int)(0.1f / std::max(ms, 1e-4f))));
                rc = record_hip(hipEventRecord(t0, stream));
                for (int r = 0; r < reps && rc == CONV_OK; ++r) rc = launch(c.p, c.a, s, x, w, y);
                if (rc == CONV_OK) rc = record_hip(hipEventRecord(t1, stream));
                if (rc == CONV_OK) rc = record_hip(hipEventSynchronize(t1));
                if (rc == CONV_OK) rc = record_hip(hipEventElapsedTime(&ms, t0, t1));
                ms /= reps;
            }
        }
        if (rc != CONV_OK) { rc_last = rc; continue; }
        if (best < 0 || ms < best_ms) { best = (int)i; best_ms = ms; }
    }
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    if (best < 0) return rc_last;
    {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        bool replaced = false;
        for (CacheEntry& e : g_cache)
            if (same_shape(e.s, s) && e.x_cap == x_cap && e.w_cap == w_cap && e.y_cap == y_cap) {
                e.p = cands[best].p; e.a = cands[best].a;
                replaced = true;
            }
        if (!replaced) {
            if (g_cache.size() >= kCacheEntries) g_cache.erase(g_cache.begin());
            g_cache.push_back(CacheEntry{s, x_cap, w_cap, y_cap, cands[best].p, cands[best].a});
        }
    }
    // leave y holding the result of the mapping that won
    if (int rc = launch(cands[best].p, cands[best].a, s, x, w, y)) return rc;
    if (best_plan) *best_plan = cands[best].p;
    if (best_us) *best_us = best_ms * 1000.f;
    return CONV_OK;
}

extern "C" long long conv_two_stage_workspace_bytes(int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w)
{
    Shape s;
    if (int rc = validate(N, C, H, W, K, R, S, pad_h, pad_w, &s)) return rc;
    if (R * S == 1) return 0;
    return 4LL * R * S * N * K * s.P * s.Q;
}

extern "C" int conv_fwd_two_stage(const float* x, const float* w, float* y, float* workspace, long long workspace_bytes,
                                  int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w)
{
    if (!x || !w || !y) return CONV_E_NULL;
    Shape s;
    if (int rc = validate(N, C, H, W, K, R, S, pad_h, pad_w, &s)) return rc;
    const long long need = conv_two_stage_workspace_bytes(N, C, H, W, K, R, S, pad_h, pad_w);
    if (need / 4 >= (1LL << 31) || C > 16384) return CONV_E_PLAN;
    if (need > 0 && !workspace) return CONV_E_NULL;
    if (workspace_bytes < need) return CONV_E_WORKSPACE;
    KernelArgs a;
    base_args(s, &a);
    a.x = x; a.w = w; a.y = y;
    return record_hip(launch_two_stage(g_stream, a, workspace));
}

extern "C" long long conv_probe_mfma(int iters, float* sink)
{
    if (!sink) return CONV_E_NULL;
    if (iters < 1 || iters > (1 << 24)) return CONV_E_DIM;
    if (int rc = record_hip(launch_probe_mfma(iters, sink, g_stream))) return rc;
    return 8192LL * iters * 16 * 2048;
}

extern "C" int conv_probe_copy(const void* src, void* dst, long long bytes)
{
    if (!src || !dst) return CONV_E_NULL;
    if (bytes < 16 || reinterpret_cast<uintptr_t>(src) % 16 || reinterpret_cast<uintptr_t>(dst) % 16) return CONV_E_DIM;
    return record_hip(launch_probe_copy(src, dst, bytes, g_stream));
}

extern "C" int conv_variant_count(int kernel)
{
    if (kernel == CONV_KERNEL_GENERIC) return 1;
    if (kernel == CONV_KERNEL_TAP) return kNumTapVariants;
    if (kernel == CONV_KERNEL_POINTWISE) return kNumPointwiseVariants;
    if (kernel == CONV_KERNEL_PANEL) return kNumPanelVariants;
    return 0;
}

extern "C" int conv_variant_info(int kernel, int variant, int* tile_k, int* max_tile_pix, int* block)
{
    if (variant < 0 || variant >= conv_variant_count(kernel)) return CONV_E_PLAN;
    int tk = 1, mp = 256, bl = 256;
    if (kernel == CONV_KERNEL_TAP) {
        tk = kTapVariants[variant].tile_k(); mp = kTapVariants[variant].max_pix(); bl = kTapVariants[variant].block();
    }
    if (kernel == CONV_KERNEL_POINTWISE) {
        tk = kPointwiseVariants[variant].tile_k(); mp = kPointwiseVariants[variant].tile_pix(); bl = kPointwiseVariants[variant].block();
    }
    if (kernel == CONV_KERNEL_PANEL) {
        tk = kPanelVariants[variant].tile_k(); mp = 64 * kPanelVariants[variant].NW; bl = kPanelVariants[variant].block();
    }
    if (tile_k) *tile_k = tk;
    if (max_tile_pix) *max_tile_pix = mp;
    if (block) *block = bl;
    return CONV_OK;
}

extern "C" int conv_set_stream(void* hip_stream)
{
    g_stream = reinterpret_cast<hipStream_t>(hip_stream);
    return CONV_OK;
}

extern "C" const char* conv_strerror(int code)
{
    switch (code) {
        case CONV_OK: return "ok";
        case CONV_E_NULL: return "null pointer";
        case CONV_E_DIM: return "dimension not positive or padding negative";
        case CONV_E_EMPTY: return "empty output (P <= 0 or Q <= 0)";
        case CONV_E_OVERFLOW: return "tensor has 2^31 or more elements";
        case CONV_E_HIP: return g_hip_error.c_str();
        case CONV_E_PLAN: return "plan does not fit the shape or the kernels";
        case CONV_E_WORKSPACE: return "workspace too small";
        default: return "unknown error code";
    }
}
