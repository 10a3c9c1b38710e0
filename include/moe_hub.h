/*
 * moe_hub.h - C ABI of the MI355X (gfx950) MoE-layer hot path.
 *
 * One GPU's share of an expert-parallel MoE layer, following the five steps of
 * the paper's Section II-A (routing, dispatch, expert computation, combine,
 * scaling).  The dispatch step is split the way Section III-A describes the
 * software "mediation" that precedes any transfer: first the destination
 * address of every routed row is resolved (moe_dispatch_layout), then rows are
 * moved into dense, send-ready regions (moe_permute).
 *
 * Conventions shared by every call
 *  - All data pointers are DEVICE pointers owned by the caller.  The library
 *    never allocates, frees or copies to the host, and never synchronises: a
 *    call enqueues kernels on `stream` (a hipStream_t passed as void*; NULL is
 *    the default stream) and returns.  Segment offsets and counts stay on the
 *    device between calls; no step needs them on the host.
 *  - Matrices are row-major and dense.  A row is one token (Section IV-A);
 *    rows must be 16-byte aligned: base pointers 16-byte aligned and
 *    H * sizeof(element) (and F * sizeof(element)) a multiple of 16.
 *  - dtype is the storage type of activations and expert weights: MOE_BF16
 *    (fp32 accumulation) or MOE_F32.  Router weights and logits are fp32.
 *  - Return value: MOE_OK, or a negative error; moe_last_error() describes it.
 *    Every argument error (MOE_ERR_ARG, MOE_ERR_UNSUPPORTED, MOE_ERR_WORKSPACE)
 *    is found before the first launch: nothing was enqueued and no output was
 *    touched.  MOE_ERR_LAUNCH means the HIP runtime refused one of the call's
 *    launches; earlier launches of the same call may already be enqueued.  A
 *    HIP error that the caller's own earlier work left pending is cleared at
 *    entry and never reported as this library's.
 *  - N == 0 (or M == 0) is a successful no-op.  Inputs must be finite.
 *  - The only state the library keeps between calls is a per-device cache of
 *    device properties (compute-unit count, raised LDS limit), filled on first
 *    use and safe to fill from several threads; calls on different streams or
 *    threads are independent as long as their buffers are.
 */
#ifndef MOE_HUB_H
#define MOE_HUB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MOE_OK = 0,
    MOE_ERR_ARG = -1,         /* null pointer, size out of range, misaligned row */
    MOE_ERR_UNSUPPORTED = -2, /* valid but not built (dtype, E too large, ...)    */
    MOE_ERR_WORKSPACE = -3,   /* workspace missing or smaller than required       */
    MOE_ERR_LAUNCH = -4,      /* the HIP runtime refused a launch                 */
    MOE_ERR_STATE = -5        /* moe_ffn_status: a GEMM step ran without a schedule or gave up a wait */
};

enum { MOE_BF16 = 0, MOE_F32 = 1 };

enum {
    MOE_SCORE_SOFTMAX_TOPK = 0, /* softmax over the K selected logits               */
    MOE_SCORE_SIGMOID_TOPK = 1  /* sigmoid of each selected logit, divided by their sum */
};

enum { MOE_OP_ROUTE = 0, MOE_OP_DISPATCH_LAYOUT = 1, MOE_OP_GROUPED_FFN = 2 };

enum { MOE_MAX_EXPERTS = 1024, MOE_MAX_TOPK = 32 };

/* Size of the histogram array built into the library for moe_dispatch_layout_static. */
#define MOE_LAYOUT_STATIC_MAX_BYTES (4u << 20)

/* Text of the last error raised on the calling thread ("" if none). */
const char *moe_last_error(void);

/* Bytes of device workspace `op` needs for these sizes (arguments an op does not
 * use are ignored).  ROUTE: N*E fp32 logits (only when logits_opt is NULL).
 * DISPATCH_LAYOUT: per-chunk expert histograms.  GROUPED_FFN: the activation
 * a[M,F] between the two GEMMs plus the tile schedule.  Returns 0 on bad sizes. */
size_t moe_workspace_bytes(int op, int64_t N, int64_t H, int E, int K, int G, int64_t F, int dtype);

/*
 * Routing (Section II-A, step 1): gating scores, top-K selection, normalisation.
 *
 *   logit[n,e] = sum_h x[n,h] * W_r[h,e]  (+ bias[e] when bias != NULL)
 * in fp32, in one fixed order so that the selection is reproducible bit for
 * bit: 64 partial sums, partial l accumulates h = l, l+64, ... ascending with
 * fused multiply-adds; the partials are then folded in six pairwise rounds
 * s = 32,16,8,4,2,1 (p[l] += p[l^s]); the bias is added last.
 * Selection is on the logits: the K largest per token, equal logits to the
 * lower expert index; topk_idx[n,0..K) in descending preference.
 * topk_w[n,k]: per score_mode, normalised over the K selected (sums to 1).
 *
 *   x        [N,H] dtype          W_r  [H,E] fp32        bias [E] fp32 or NULL
 *   topk_idx [N,K] int32 (out)    topk_w [N,K] fp32 (out)
 *   logits_opt [N,E] fp32 (out) or NULL; when NULL, ws must hold N*E floats.
 * Requires 1 <= K <= min(E, MOE_MAX_TOPK), E <= MOE_MAX_EXPERTS.
 */
int moe_route(const void *x, int dtype, int64_t N, int64_t H,
              const float *W_r, const float *bias, int E, int K, int score_mode,
              int32_t *topk_idx, float *topk_w, float *logits_opt,
              void *ws, size_t ws_bytes, void *stream);

/*
 * Address resolution (the mediation of Section III-A, kept on the GPU): how
 * many rows each expert and each logical destination receives, where each
 * region starts, and the slot of every routed row.  Regions are dense, sized
 * by the counts, and laid out back to back in expert order; nothing is dropped
 * or padded (Section IV-A: conservative regions, dense packing; the byte
 * address of slot s is base + s * RowSize).  Expert e belongs to destination
 * e / (E/G).  Inside a region rows keep ascending flat order r = n*K + k, so
 * the result is the stable counting sort of topk_idx by expert and is unique.
 *
 *   topk_idx       [N*K] int32, values in [0,E)
 *   expert_counts  [E]    expert_offsets [E+1]  (exclusive scan, [E] = N*K)
 *   dest_counts    [G]    dest_offsets   [G+1]  (dest_offsets[g] = expert_offsets[g*E/G])
 *   slot_of_row    [N*K]  slot of flat row r
 *   row_of_slot    [N*K]  inverse map
 * Requires E % G == 0, N*K < 2^31.  ws: moe_workspace_bytes(MOE_OP_DISPATCH_LAYOUT, ...).
 * Out-of-range expert indices are a precondition violation (rows are then ignored).
 */
int moe_dispatch_layout(const int32_t *topk_idx, int64_t N, int K, int E, int G,
                        int32_t *expert_counts, int32_t *expert_offsets,
                        int32_t *dest_counts, int32_t *dest_offsets,
                        int32_t *slot_of_row, int32_t *row_of_slot,
                        void *ws, size_t ws_bytes, void *stream);

/*
 * moe_dispatch_layout for callers that cannot allocate device memory or pass a
 * workspace they allocated: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments (without ws), same kernels and
 * bit for bit the same outputs; the per-unit histograms go into an array of
 * MOE_LAYOUT_STATIC_MAX_BYTES (4 MiB) that is part of the library's device image.
 * The call allocates nothing and frees nothing.  Limit: moe_workspace_bytes(
 * MOE_OP_DISPATCH_LAYOUT, N, 0, E, K, G, 0, 0) <= MOE_LAYOUT_STATIC_MAX_BYTES, i.e.
 * ceil(N*K / 512) * E <= 2^20 (N*K = 131072 rows with E = 1024 experts fit four
 * times over); beyond it MOE_ERR_UNSUPPORTED.  Each GPU holds its own copy of the
 * array from the library's first use there until the process ends, and every call
 * on that GPU uses it: calls that overlap on one GPU (two streams, two threads)
 * race; calls in stream order on one stream do not.  The first call on a device
 * looks the array's address up (hipGetSymbolAddress) with that device current.
 */
int moe_dispatch_layout_static(const int32_t *topk_idx, int64_t N, int K, int E, int G,
                               int32_t *expert_counts, int32_t *expert_offsets,
                               int32_t *dest_counts, int32_t *dest_offsets,
                               int32_t *slot_of_row, int32_t *row_of_slot, void *stream);

/*
 * Address resolution in arrival order (the allocation unit of Section IV-A3: a row
 * pointer per region, read and incremented atomically by each arriving row, which
 * packs rows densely whatever order they come in; the flat row number kept in
 * row_of_slot is the source information of Section IV-A4 that the combine needs).
 * Counts, offsets and the per-destination view are exactly those of
 * moe_dispatch_layout; slot_of_row / row_of_slot are again inverse bijections and
 * every row lands inside its expert's region, but the order of rows inside a
 * region is the order in which their atomics were served: it is not unique and may
 * differ from call to call.  Every later step accepts either layout, and the
 * layer's output does not depend on the choice: an expert row's result does not
 * depend on its slot, and moe_combine sums in ascending k.
 * Arguments as in moe_dispatch_layout; no workspace.
 */
int moe_dispatch_layout_arrival(const int32_t *topk_idx, int64_t N, int K, int E, int G,
                                int32_t *expert_counts, int32_t *expert_offsets,
                                int32_t *dest_counts, int32_t *dest_offsets,
                                int32_t *slot_of_row, int32_t *row_of_slot, void *stream);

/*
 * Routing and arrival-order address resolution in one call, the row pointer taken
 * as the row is produced (Section IV-A3: a routed row draws its local row id from its
 * region's row pointer at the moment it arrives): the top-K kernel of moe_route draws
 * it for each of a token's K rows right after selecting their experts, so the separate
 * rank pass of moe_dispatch_layout_arrival (and its re-read of topk_idx) is gone.
 * Outputs are those of moe_route followed by moe_dispatch_layout_arrival: topk_idx
 * and topk_w as moe_route gives them (bit for bit); counts, offsets and the
 * per-destination view exact; slot_of_row / row_of_slot a valid dense packing in the
 * order the atomics were served.  Arguments as in the two calls; ws as in moe_route
 * (N*E*4 bytes when logits_opt is NULL).  Three launches beside the logits kernel:
 * clear of the E row pointers, top-K with the draw, placement.  The draw is one
 * atomic per routed row, N*K of them on E addresses; moe_dispatch_layout_arrival
 * aggregates 1024 rows per workgroup first and is the faster form on this chip
 * (this call exists for the comparison).
 */
int moe_route_resolve_arrival(const void *x, int dtype, int64_t N, int64_t H, const float *W_r,
                              const float *bias, int E, int K, int G, int score_mode,
                              int32_t *topk_idx, float *topk_w, float *logits_opt,
                              int32_t *expert_counts, int32_t *expert_offsets,
                              int32_t *dest_counts, int32_t *dest_offsets,
                              int32_t *slot_of_row, int32_t *row_of_slot,
                              void *ws, size_t ws_bytes, void *stream);

/*
 * Dispatch, local half (Section II-A, step 2): xp[slot_of_row[n*K+k], :] = x[n, :],
 * a bitwise copy of each token row into each of its K slots.  The result is
 * expert-contiguous and therefore destination-contiguous: segment
 * [dest_offsets[g], dest_offsets[g+1]) is what would be sent to destination g.
 *   x [N,H] dtype     xp [N*K,H] dtype (out)
 * Requires K <= 64 (MOE_ERR_UNSUPPORTED otherwise).  row_of_slot is accepted for
 * symmetry with the layout's outputs and is not read.
 */
int moe_permute(const void *x, int dtype, int64_t N, int64_t H, int K,
                const int32_t *slot_of_row, const int32_t *row_of_slot,
                void *xp, void *stream);

/*
 * Expert computation (Section II-A, step 3: two GEMMs with an activation in
 * between), gated form, for E_local experts over the rows of xp:
 *   rows [seg_offsets[e], seg_offsets[e+1]) belong to local expert e
 *   g = xp_row W_gate[e]^T, u = xp_row W_up[e]^T, a = g/(1+exp(-g)) * u,
 *   y_row = a W_down[e]^T
 * Weights are stored "out x in" (the reduction index is contiguous):
 *   W_gate, W_up [E_local,F,H]    W_down [E_local,H,F]    (dtype)
 *   xp [M,H]   y [M,H] (out)   seg_offsets [E_local+1] int32 ON THE DEVICE,
 *   non-decreasing, within [0,M].  Rows outside every segment are not written.
 * bf16: fp32 accumulation, `a` and `y` rounded to bf16 (nearest even).
 * ws: moe_workspace_bytes(MOE_OP_GROUPED_FFN, M, H, E_local, 0, 0, F, dtype).
 * For an expert-parallel rank pass seg_offsets = expert_offsets + g*E/G and the
 * weights of that destination's experts.
 */
int moe_grouped_ffn(const void *xp, int dtype, int64_t M, int64_t H, int64_t F,
                    int E_local, const int32_t *seg_offsets,
                    const void *W_gate, const void *W_up, const void *W_down,
                    void *y, void *ws, size_t ws_bytes, void *stream);

/*
 * The same computation in its three parts, for callers that want to time or
 * overlap the two GEMMs of Section II-A step 3 separately ("GEMM1" = gate and up
 * projection with the activation fused, "GEMM2" = down projection).  Arguments
 * as in moe_grouped_ffn; all three share one workspace of
 * moe_workspace_bytes(MOE_OP_GROUPED_FFN, ...) bytes, and
 *   moe_ffn_schedule -> moe_ffn_gate_up -> moe_ffn_down   (in stream order)
 * is exactly moe_grouped_ffn.  moe_ffn_schedule turns seg_offsets into the
 * device-side tile tables both GEMMs read; moe_ffn_gate_up leaves the activation
 * a[M,F] in the workspace; moe_ffn_down reads it and writes y.  The GEMM steps
 * may be launched again over the same schedule.  On a workspace that
 * moe_ffn_schedule has not filled for the same M (bf16) they find no tile table,
 * leave their outputs untouched and set an error word in the workspace; the
 * call itself still returns MOE_OK (it never waits for the device).
 * moe_ffn_status reports that word.
 */
int moe_ffn_schedule(int dtype, int64_t M, int64_t H, int64_t F, int E_local,
                     const int32_t *seg_offsets, void *ws, size_t ws_bytes, void *stream);
int moe_ffn_gate_up(const void *xp, int dtype, int64_t M, int64_t H, int64_t F,
                    int E_local, const int32_t *seg_offsets,
                    const void *W_gate, const void *W_up,
                    void *ws, size_t ws_bytes, void *stream);
/*
 * Both GEMMs of the expert computation in ONE launch, the second consuming the first's
 * output as it becomes available: the software counterpart of the paper's data
 * availability manager (Section IV-C: what each group of thread blocks depends on is
 * known in advance, arrivals are counted, and a block is released as soon as its own
 * data are complete instead of after a global barrier).  A workgroup works through the
 * tiles of the gate/up projection and then goes on to tiles of the down projection; a
 * down-projection tile needs the rows [m0, m0 + rows) of the activation a, complete over
 * all F columns, and nothing else: every wavefront of a gate/up tile bumps that row
 * tile's arrival counter (in the workspace) once its stores are acknowledged, and the
 * down-projection tile starts when the counter is full.  The tail of the first GEMM and
 * the head of the second overlap, and one launch replaces two.
 *   moe_ffn_schedule -> moe_ffn_gate_up_down   (in stream order)
 * gives bit for bit the y of moe_ffn_schedule -> moe_ffn_gate_up -> moe_ffn_down.  It may
 * be launched again over the same schedule.  (moe_grouped_ffn runs the two separate
 * launches, which are the faster form on this chip: the XCDs' L2 caches do not see each
 * other's lines, so the gate/up projection has to store its result through to memory.)
 * Arguments as in moe_grouped_ffn.  wait_limit: how many polls (about a microsecond
 * each) a down-projection tile spends on its rows before its workgroup gives up; 0 = the
 * default (seconds).  Every gate/up tile is drawn by a workgroup that waits for nothing
 * before any down-projection tile is drawn, so a wait always ends; the limit turns a
 * broken schedule into an exit instead of a hang: the workgroup leaves, sets the
 * workspace's error word (moe_ffn_status then returns MOE_ERR_STATE) and y stays
 * incomplete.  The call itself still returns MOE_OK.  MOE_BF16 needs a 128-byte aligned
 * ws (with F % 64 == 0, as for every bf16 FFN, each row of the activation then is a whole
 * number of cache lines, so no line holds rows of two row tiles, one complete and one
 * still being written); otherwise MOE_ERR_UNSUPPORTED, and the two separate calls serve.  MOE_F32: runs the two
 * simple kernels one after the other.
 */
int moe_ffn_gate_up_down(const void *xp, int dtype, int64_t M, int64_t H, int64_t F,
                         int E_local, const int32_t *seg_offsets,
                         const void *W_gate, const void *W_up, const void *W_down,
                         void *y, void *ws, size_t ws_bytes, int64_t wait_limit, void *stream);

/*
 * Did every GEMM step launched over this workspace since the last moe_ffn_schedule
 * find its schedule?  The one call of the library that waits: it synchronises
 * `stream`, copies the workspace's two error words to the host and returns MOE_OK
 * or MOE_ERR_STATE (a bf16 GEMM step ran over a workspace that moe_ffn_schedule had
 * not filled for the same M, and wrote nothing; or a tile of moe_ffn_gate_up_down ran
 * into its wait_limit).  For tests and debugging; the
 * hot path does not need it.  fp32 workspaces have no schedule: always MOE_OK.
 */
int moe_ffn_status(int dtype, int64_t M, int64_t H, int64_t F, int E_local,
                   const void *ws, size_t ws_bytes, void *stream);
/*
 * GEMM1 with the dispatch's row move folded into its operand loads: the paper's
 * ideal MoE layer (Section II-C) runs routing, expert computation and scaling with
 * no additional step in between; the extra handling of data that Section II-C
 * counts among the scheduling overheads, and the shuffling of rows whose cost
 * Section VI-B says grows with the sequence length, are what this variant removes
 * on the dispatch side.  Row
 * m of the virtual xp is x[row_of_slot[m] / K, :], fetched where moe_ffn_gate_up
 * would fetch xp[m, :]; xp is neither written nor read.  The result, a[N*K,F] in
 * the workspace, is bit for bit that of moe_permute followed by moe_ffn_gate_up,
 * and moe_ffn_schedule (with M = N*K) / moe_ffn_down go before / after it as
 * they do there.  For a single device that computes all experts itself; an
 * expert-parallel rank still needs the materialised send buffer.
 *   x [N,H] dtype    row_of_slot [N*K] int32 (of moe_dispatch_layout)
 * bf16 needs N*H*2 bytes of x to stay below 4 GiB (MOE_ERR_UNSUPPORTED otherwise).
 */
int moe_ffn_gate_up_gather(const void *x, int dtype, int64_t N, int K, int64_t H, int64_t F,
                           int E_local, const int32_t *seg_offsets, const int32_t *row_of_slot,
                           const void *W_gate, const void *W_up,
                           void *ws, size_t ws_bytes, void *stream);
int moe_ffn_down(int dtype, int64_t M, int64_t H, int64_t F,
                 int E_local, const int32_t *seg_offsets, const void *W_down,
                 void *y, void *ws, size_t ws_bytes, void *stream);

/*
 * GEMM2 with the combine folded into its epilogue: the other half of a layer without data-
 * shuffling steps (the ideal layer of Section II-C), for a single device that computes all experts.
 * y is neither written nor read.  For every slot m with flat row r = row_of_slot[m] = n*K + k,
 *   sums[n, :] += topk_w[n, k] * (a[m, :] W_down[e(m)]^T)
 * is added with fp32 atomic adds to `sums` [N,H] fp32 (caller's scratch, cleared by the call), and
 * out[n, :] is sums[n, :] rounded once to dtype.  moe_ffn_schedule (with M = N*K) and a GEMM1 go
 * before it as they go before moe_ffn_down.  The K additions of an element happen in the order
 * the workgroups reach them, so, unlike moe_ffn_down + moe_combine (ascending k), the result is
 * not bit-reproducible from run to run (fp32 addition order; the products are not rounded to
 * bf16 first, so it is the closer of the two to the exact sum).
 * MOE_BF16 only.  sums and out 16-byte aligned; H a multiple of 8.
 */
int moe_ffn_down_combine(int dtype, int64_t N, int K, int64_t H, int64_t F, int E_local,
                         const int32_t *seg_offsets, const void *W_down,
                         const int32_t *row_of_slot, const float *topk_w, float *sums,
                         void *out, void *ws, size_t ws_bytes, void *stream);

/*
 * Combine and scaling (Section II-A, steps 4-5): rows return to their tokens
 * and are summed with the routing weights,
 *   out[n,:] = sum_{k=0..K-1} topk_w[n,k] * y[slot_of_row[n*K+k], :]
 * accumulated in fp32 in ascending k, rounded once to dtype.
 *   y [N*K,H] dtype    topk_w [N,K] fp32    out [N,H] dtype (out)
 */
int moe_combine(const void *y, int dtype, int64_t N, int64_t H, int K,
                const int32_t *slot_of_row, const float *topk_w,
                void *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_HUB_H */
