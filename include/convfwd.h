/*
 * convfwd: stride-1 forward convolution of a CNN layer on one MI355X (gfx950),
 * computed directly on NCHW fp32 activations and KCRS fp32 filters.
 *
 * The operation (Section 2.1 of the paper: every output element is the dot
 * product of one filter with a C x R x S sub-volume of the input, the
 * sub-volume translated over X and Y; padding adds rows and columns around the
 * input; Section 3: NCHW layout, X contiguous; Section 4: stride 1, fp32):
 *
 *   y[n,k,p,q] = sum_{c<C, r<R, s<S} xpad[n, c, p+r-pad_h, q+s-pad_w] * w[k,c,r,s]
 *   xpad = x inside [0,H) x [0,W) and 0 outside
 *   P = H + 2*pad_h - R + 1,   Q = W + 2*pad_w - S + 1
 *
 * The filter is not flipped, there is no scaling, y is overwritten, and bias and
 * activation exist only as the optional fused epilogue of conv_fwd_bias_relu /
 * conv_fwd_split_c. All arithmetic is fp32 (fp32 FMA or full-precision fp32 MFMA,
 * fp32 accumulation); no reduced-precision type is used anywhere.
 *
 * Layout: x is [N][C][H][W], w is [K][C][R][S], y is [N][K][P][Q], all dense
 * and contiguous, W / S / Q fastest. Stride, dilation and groups are fixed to 1.
 *
 * Ownership: x, w and y are DEVICE pointers owned by the caller; the library
 * never allocates, frees or keeps them, and needs no workspace except in the two
 * opt-in entry points that take one from the caller (conv_fwd_split_c,
 * conv_fwd_two_stage). Its only device memory is static: a 16-byte block of zeros
 * (read by the tap family's direct loader) and the scratch array of
 * conv_fwd_split_c_static; their addresses are looked up at the first use on a
 * device. x and w must not overlap y. Calls are asynchronous on
 * the stream given to conv_set_stream (default: the null stream); the caller
 * synchronises.
 *
 * Errors: every entry point returns 0 on success or a negative CONV_E_* code;
 * nothing throws or aborts. Results are bitwise reproducible for equal inputs
 * and equal plans (no atomics).
 */
#ifndef CONVFWD_H
#define CONVFWD_H

#ifdef __cplusplus
extern "C" {
#endif

#define CONV_OK 0
#define CONV_E_NULL (-1)      /* a required pointer is null */
#define CONV_E_DIM (-2)       /* a dimension is not positive or a padding is negative */
#define CONV_E_EMPTY (-3)     /* P <= 0 or Q <= 0 */
#define CONV_E_OVERFLOW (-4)  /* a tensor has 2^31 or more elements (kernels index with 32 bits) */
#define CONV_E_HIP (-5)       /* a HIP runtime call failed; conv_strerror gives its text */
#define CONV_E_PLAN (-6)      /* a caller-supplied plan does not fit the shape or the kernels */
#define CONV_E_WORKSPACE (-7) /* the workspace given to conv_fwd_two_stage / conv_fwd_split_c is too small */

/* Kernel families a plan can name. */
#define CONV_KERNEL_GENERIC 0 /* one output per thread, fp32 FMA; any R, S, padding (also what maps too wide for a halo tile of
                                 whole padded rows run: wider than ~1500 pixels for 3x3 filters on rows of whole dwordx4,
                                 about half of that for odd widths or 5x5 filters) */
#define CONV_KERNEL_TAP 1     /* LDS halo tile + filter block, fp32 MFMA over (channel, tap). Built for 1x1 and 3x3 with all
                                 31 tile shapes; for 5x5 with the 15 whose filter block fits the staging registers (2, 4,
                                 8-12, 14-16, 22-24, 28, 30); for 1x3, 3x1, 1x5, 5x1, 1x7, 7x1, 2x2, 4x4 with shapes 2, 5, 7, 14, 16,
                                 20, 22 and for 7x7 with 2, 14, 16, 22. conv_fwd_plan_request tells whether a pair exists */
#define CONV_KERNEL_POINTWISE 2 /* 1x1, pad 0: inputs and filters streamed HBM -> registers -> fp32 MFMA, waves split C */
#define CONV_KERNEL_PANEL 3   /* 1x1, pad 0, batched: filters of a channel tile resident in LDS, waves stream pixel tiles */

/* Loaders of the tap family (conv_plan_t.loader): through the registers (global load, then LDS store, two chunks
 * ahead of the arithmetic), or straight from global memory into LDS (one chunk ahead, no register staging; it also
 * fetches the padding cells of the halo tile, from a block of zeros). */
#define CONV_LOADER_REGISTERS 1
#define CONV_LOADER_DIRECT 2
/* Direct loads issued by four loader waves of their own (tile shapes of eight waves only): the waves that multiply
 * then issue no memory instruction between prologue and stores; conv_plan_t.block counts the loader waves too. */
#define CONV_LOADER_DIRECT_WAVES 3
/* Direct loads into a ring of four staging copies instead of two (tile shapes whose waves hold one or two MFMA tiles):
 * three chunks are on their way while one is multiplied, for layers whose chunks are shorter than a load takes. */
#define CONV_LOADER_DIRECT_DEEP 4

/* Work-group numbering of the tap family (conv_plan_t.order). */
#define CONV_ORDER_CHANNEL_FAST 1
#define CONV_ORDER_PIXEL_FAST 2
#define CONV_ORDER_CHANNEL_GROUPS 3 /* in between: the channel tiles in groups of conv_plan_t.k_group, the pixel tiles of a group
                                       next, then the groups - an XCD's work-groups then share some channel tiles and some pixel
                                       tiles, and the eight L2s fetch fewer bytes in all than under either plain order */

/*
 * How one layer is mapped onto the GPU. Filled by conv_fwd_plan; plain data.
 * In conv_fwd_plan's mappings the reduction over (c, r, s) stays inside one
 * work-group, so they need no workspace (unlike the two-stage scheme of
 * Section 3, whose first stage writes R*S partial matrices per input/filter
 * pair). Only the channel-splitting mode (conv_fwd_plan_split_c) has
 * c_splits > 1 and a workspace.
 */
typedef struct conv_plan {
    int kernel;          /* CONV_KERNEL_* */
    int variant;         /* tile shape index inside the family (see conv_variant_info) */
    int tile_k;          /* output channels per work-group */
    int tile_pix;        /* output pixels per work-group, counted in flattened (n,p,q) order
                            (CONV_KERNEL_PANEL: work-groups per channel tile, each wave streaming 64-pixel tiles) */
    int chunk_c;         /* input channels staged in LDS per round */
    int x_vec, w_vec;    /* dwords per global load of input rows / filter slices: 4, 2 or 1 */
    int lds_rows;        /* input rows (of the zero-padded, vertically stacked images) held per channel */
    int lds_pitch;       /* floats between consecutive rows of the LDS halo tile */
    int lds_plane;       /* floats between consecutive channels of the LDS halo tile */
    int grid;            /* work-groups */
    int block;           /* threads per work-group */
    int lds_bytes;       /* dynamic LDS per work-group */
    int P, Q;            /* output height and width */
    int c_splits;        /* work-groups that share the channels of one output tile; 1: the whole reduction in one */
    int loader;          /* CONV_KERNEL_TAP: how a chunk reaches LDS, CONV_LOADER_REGISTERS or CONV_LOADER_DIRECT
                            (as a request: 0 = the planner's rule); 0 for the other families */
    int order;           /* CONV_KERNEL_TAP: which tile index runs fastest in the work-group numbering, and so what the
                            work-groups of one XCD (one L2) share: CONV_ORDER_CHANNEL_FAST (a few pixel tiles, every
                            channel tile: the inputs are fetched once, the filters by every L2) or CONV_ORDER_PIXEL_FAST
                            (the reverse, for layers whose filters outweigh their inputs) or CONV_ORDER_CHANNEL_GROUPS;
                            as a request: 0 = the planner's rule; 0 for the other families */
    int k_group;         /* CONV_KERNEL_TAP: channel tiles that are neighbours in the work-group numbering: all of them
                            (CHANNEL_FAST), 1 (PIXEL_FAST) or a divisor of their number in between (CHANNEL_GROUPS; as a
                            request with that order: 0 = the group that fetches least); 0 for the other families */
    long long workspace_bytes; /* 0 unless c_splits > 1: then 4 * c_splits * N*K*P*Q */
    long long flops;     /* 2*N*K*P*Q*C*R*S */
    long long bytes;     /* 4*(N*C*H*W + K*C*R*S + N*K*P*Q): compulsory HBM traffic */
} conv_plan_t;

/*
 * y = conv(x, w). Plans the launch (as conv_fwd_plan does, then narrows the
 * vector widths if x or w is not 16-byte aligned) and enqueues one kernel.
 * x, w, y: device pointers (see the header comment). Returns CONV_OK or
 * CONV_E_NULL / _DIM / _EMPTY / _OVERFLOW / _HIP.
 */
int conv_fwd(const float* x, const float* w, float* y,
             int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w);

/*
 * Host-only: choose kernel family, tile shape, channel chunk, grid and LDS size
 * for a shape (Section 3 discusses this choice as the number of thread blocks
 * per filter row; Section 4.2 shows both too many and too few blocks lose).
 * Touches no device. out: host pointer, fully written on success.
 */
int conv_fwd_plan(int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w,
                  conv_plan_t* out);

/*
 * As conv_fwd, with the mapping requested by the caller. Only plan->kernel,
 * plan->variant, plan->tile_pix and plan->chunk_c are read as requests (0 in
 * tile_pix means "the variant's capacity"; chunk_c is fixed by the variant and
 * may be left 0); every derived field is recomputed and checked, and
 * CONV_E_PLAN is returned if the request cannot be honoured (family does not
 * support R x S, tile exceeds the variant's capacity, staging does not fit
 * the variant's registers or LDS). plan->loader may also name the tap family's loader (0: the planner's rule;
 * CONV_LOADER_DIRECT needs filter slices of whole dwordx4 - C a multiple of 4 - and input rows that move as
 * dwordx4 or single dwords). If resolved is not null it receives the plan actually used.
 */
int conv_fwd_planned(const float* x, const float* w, float* y,
                     int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w,
                     const conv_plan_t* plan, conv_plan_t* resolved);

/*
 * Host-only "what if": resolves a request exactly as conv_fwd_planned / conv_fwd_split_c would for 16-byte aligned
 * tensors (request fields as in conv_fwd_planned, plus c_splits), without touching a device. resolved receives
 * the launch; model_cycles (may be null) the planner's cost estimate of it in GPU cycles - tap family only
 * (0 for the others), second pass included when c_splits > 1. The planner of Section 3's "number of thread
 * blocks" question is this estimate minimised over the tile shapes and pixel tiles. Returns CONV_OK,
 * CONV_E_NULL / _DIM / _EMPTY / _OVERFLOW, or CONV_E_PLAN if the request cannot be honoured.
 */
int conv_fwd_plan_request(int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w,
                          const conv_plan_t* request, conv_plan_t* resolved, double* model_cycles);

/*
 * Measured choice of the mapping, for callers who run a layer many times (what "the best algorithm of the
 * library" means in the comparisons of Section 4): runs every mapping the kernels accept for this layer on
 * the caller's tensors - all tile shapes of the matching families with the planner's candidate pixel tiles
 * (panel kernel: the planner's grid and one and two work-groups per CU; tap shapes with either loader, and only
 * while their modelled cost is within 2.5x of the best) - times each with events on the
 * library's stream, and keeps the fastest: it is stored in the plan cache, so conv_fwd and
 * conv_fwd_bias_relu use it from then on for this shape and pointer alignment, and returned in *best_plan
 * with its time per launch in *best_us (either may be null). Without a flush buffer each mapping is timed
 * over a batch of 2..16 back-to-back launches on cache-warm tensors. With one (flush: 16-byte aligned device
 * memory of flush_bytes >= 1 MiB owned by the caller, contents overwritten; 512 MiB clears the 256 MiB
 * Infinity Cache) every timed launch runs alone after the buffer has been streamed through the caches,
 * three times, and the fastest counts: the ranking a layer sees whose inputs come from HBM.
 * y is overwritten repeatedly and finally holds conv(x, w). Synchronous (waits for the stream, so it cannot
 * be captured into a graph); allocates no device memory. Returns CONV_OK or the error codes of conv_fwd.
 */
int conv_fwd_find(const float* x, const float* w, float* y,
                  int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w,
                  void* flush, long long flush_bytes, conv_plan_t* best_plan, float* best_us);

/*
 * The layer with its fused epilogue: y = act(conv(x, w) + bias[k]). Section 2.1: the weighted sums of a
 * convolutional layer are usually passed through a non-linear function such as ReLU; the per-filter
 * constant is what CNN layers add before it (the paper does not mention one: pass null to leave it out).
 * bias: device pointer to K floats, or null. relu: nonzero applies max(., 0) to every output. The epilogue
 * runs in the store path of the same single kernel (after the cross-wave reduction where waves split C);
 * no second pass over y and no workspace. plan: null plans as conv_fwd does, otherwise a request as in
 * conv_fwd_planned. resolved (may be null) receives the plan used. x, w, y as for conv_fwd; y is overwritten.
 * Returns CONV_OK or the error codes of conv_fwd / conv_fwd_planned.
 */
int conv_fwd_bias_relu(const float* x, const float* w, const float* bias, float* y,
                       int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w,
                       int relu, const conv_plan_t* plan, conv_plan_t* resolved);

/*
 * Channel splitting across work-groups, for layers with too few output tiles to fill 256 CUs (batch 1, small
 * maps, many channels: the layers Section 4.2 singles out, where the number of thread blocks decides the
 * time; Section 5 names fusing and redistributing the work as future work). The C channels are cut into
 * c_splits shares of whole chunks; each (output tile, share) is one work-group of the tap kernel, which
 * writes its partial sums into share-th slice of the workspace; a second kernel adds the slices in share
 * order (results stay bitwise reproducible) and applies the epilogue of conv_fwd_bias_relu.
 * conv_fwd_plan_split_c: host-only; as conv_fwd_plan, but tap-family layers may get c_splits > 1 and then
 * workspace_bytes = 4 * c_splits * N*K*P*Q. Layers conv_fwd_plan maps to other families keep that mapping.
 * conv_fwd_split_c: plan null -> conv_fwd_plan_split_c's choice for these pointers; otherwise a request as in
 * conv_fwd_planned, where c_splits (0 or 1: none) is honoured up to the number of chunks C holds and needs
 * kernel = CONV_KERNEL_TAP. workspace: device pointer owned by the caller, 16-byte aligned for the fastest second
 * pass, at least resolved->workspace_bytes long (may be null when that is 0), not overlapping x, w or y;
 * contents undefined afterwards. Returns CONV_OK, the error codes of conv_fwd_planned, CONV_E_NULL for a
 * missing workspace or CONV_E_WORKSPACE for a short one.
 */
int conv_fwd_plan_split_c(int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w, conv_plan_t* out);
int conv_fwd_split_c(const float* x, const float* w, const float* bias, float* y, float* workspace,
                     long long workspace_bytes, int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w,
                     int relu, const conv_plan_t* plan, conv_plan_t* resolved);

/*
 * conv_fwd_split_c for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. The partial outputs of the channel shares go
 * into a static device array of CONV_STATIC_SCRATCH_BYTES bytes that the library's code object carries (every
 * GPU the library runs on holds its own copy until the process ends; its address is looked up once per device,
 * at the first call on that device). Arguments, results (bit for bit) and errors are those of conv_fwd_split_c
 * without workspace / workspace_bytes; a layer whose mapping needs more than CONV_STATIC_SCRATCH_BYTES
 * (resolved->workspace_bytes = 4 * c_splits * N*K*P*Q) is refused with CONV_E_WORKSPACE and nothing is launched.
 * The call allocates and frees nothing on the device and enqueues the same two kernels on the calling thread's
 * stream. All calls on one GPU share the array: it keeps the last call's partial sums (nothing needs clearing -
 * every element the second kernel reads was written by the first), and calls that overlap on one GPU (two streams,
 * two threads) race on it - serialise them. Mappings without channel shares (c_splits == 1) do not touch it.
 */
#define CONV_STATIC_SCRATCH_BYTES (16ll << 20)
int conv_fwd_split_c_static(const float* x, const float* w, const float* bias, float* y,
                            int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w,
                            int relu, const conv_plan_t* plan, conv_plan_t* resolved);

/*
 * The paper's own two-stage scheme (Section 3), opt-in and outside the planner, for comparison with the
 * fused kernels: stage 1 computes, per filter tap (r,s), the channel-reduced matrix
 * T[r,s][n,k,p,q] = sum_c w[k,c,r,s] * xpad[n,c,p+r-pad_h,q+s-pad_w] into the workspace (one work-group
 * per filter row staged in LDS, one dot product per thread), stage 2 adds the R*S matrices into y; a 1x1
 * filter needs no second stage and no workspace. workspace: device pointer to at least
 * conv_two_stage_workspace_bytes(...) bytes, owned by the caller, contents undefined afterwards (may be
 * null when that size is 0). Two kernels are enqueued on the library's stream. Returns CONV_OK,
 * CONV_E_NULL / _DIM / _EMPTY / _OVERFLOW / _HIP, CONV_E_WORKSPACE if workspace_bytes is too small, or
 * CONV_E_PLAN if C exceeds 16384 (a filter row must fit LDS) or the workspace would pass 2^31 elements.
 */
long long conv_two_stage_workspace_bytes(int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w);
int conv_fwd_two_stage(const float* x, const float* w, float* y, float* workspace, long long workspace_bytes,
                       int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w);

/*
 * Measurement aids, not part of the convolution: two micro-probes of what the GPU attains, so that the
 * benchmark can quote fractions of measured peaks beside the datasheet ones. conv_probe_mfma enqueues a
 * register-resident fp32 MFMA loop (8192 waves x iters x 16 v_mfma_f32_16x16x4_f32) and returns the
 * number of floating-point operations it performs (or a negative CONV_E_*); sink: device pointer to one
 * float, never written in practice. conv_probe_copy enqueues a dwordx4 copy of `bytes` bytes (rounded down to
 * a multiple of 16) between two 16-byte aligned device buffers. Both run on the library's stream; the caller times them.
 */
long long conv_probe_mfma(int iters, float* sink);
int conv_probe_copy(const void* src, void* dst, long long bytes);

/*
 * Number of tile shapes of a kernel family (0 for an unknown family), and the
 * capacity of one: output channels and output pixels per work-group and
 * threads per work-group. Host-only. Returns CONV_E_PLAN for bad indices.
 */
int conv_variant_count(int kernel);
int conv_variant_info(int kernel, int variant, int* tile_k, int* max_tile_pix, int* block);

/*
 * Stream used by later launching calls (conv_fwd, conv_fwd_planned, conv_fwd_bias_relu, conv_fwd_split_c,
 * conv_fwd_two_stage, conv_fwd_find, the probes) OF THE CALLING HOST THREAD: a hipStream_t passed as void*,
 * NULL = null stream. The setting is per thread (a thread that never called it launches on the null stream), so
 * two threads driving different streams do not disturb each other.
 */
int conv_set_stream(void* hip_stream);

/* Text for a CONV_E_* code; for CONV_E_HIP the text of the last HIP error seen. Never null. */
const char* conv_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CONVFWD_H */
