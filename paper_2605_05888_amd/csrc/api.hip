// C ABI of the MoE-layer hot path: argument checks, then one launcher per step.
// Every check happens before the first launch, so an error leaves all outputs
// untouched.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "common.h"

namespace moe {

static thread_local char g_err[256] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

// Entry of every call: forget the last message, and a HIP error that the caller's own earlier work
// left pending (it would otherwise be reported as a failed launch of ours).
void clear_error()
{
    g_err[0] = 0;
    (void)hipGetLastError();
}

int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail(MOE_ERR_LAUNCH, "%s: %s", what, hipGetErrorString(e));
    return MOE_OK;
}

static int elt_bytes(int dtype) { return dtype == MOE_BF16 ? 2 : 4; }

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int check_dtype(int dtype)
{
    if (dtype != MOE_BF16 && dtype != MOE_F32)
        return fail(MOE_ERR_UNSUPPORTED, "dtype %d is neither MOE_BF16 nor MOE_F32", dtype);
    return MOE_OK;
}

static int check_rows(const char *name, int64_t cols, int dtype)
{
    if (cols < 1)
        return fail(MOE_ERR_ARG, "%s must be >= 1 (got %lld)", name, (long long)cols);
    if ((cols * elt_bytes(dtype)) % 16 != 0)
        return fail(MOE_ERR_ARG, "%s * element size must be a multiple of 16 bytes (got %lld)",
                    name, (long long)(cols * elt_bytes(dtype)));
    return MOE_OK;
}

static int check_routing_sizes(int64_t N, int K, int E)
{
    if (N < 0)
        return fail(MOE_ERR_ARG, "N must be >= 0 (got %lld)", (long long)N);
    if (E < 1 || K < 1 || K > E)
        return fail(MOE_ERR_ARG, "need 1 <= K <= E (got K=%d, E=%d)", K, E);
    if (E > MOE_MAX_EXPERTS)
        return fail(MOE_ERR_UNSUPPORTED, "E=%d exceeds MOE_MAX_EXPERTS=%d", E, MOE_MAX_EXPERTS);
    if (N * (int64_t)K >= ((int64_t)1 << 31))
        return fail(MOE_ERR_ARG, "N*K must be below 2^31 (got %lld)", (long long)(N * K));
    return MOE_OK;
}

#define MOE_TRY(expr)          \
    do {                       \
        int rc_ = (expr);      \
        if (rc_ != MOE_OK)     \
            return rc_;        \
    } while (0)

#define MOE_NEED(ptr)                                              \
    do {                                                           \
        if ((ptr) == nullptr)                                      \
            return fail(MOE_ERR_ARG, "%s must not be NULL", #ptr); \
        if (!aligned16(ptr))                                       \
            return fail(MOE_ERR_ARG, "%s must be 16-byte aligned", #ptr); \
    } while (0)

}  // namespace moe

using namespace moe;

extern "C" const char *moe_last_error(void) { return g_err; }

extern "C" size_t moe_workspace_bytes(int op, int64_t N, int64_t H, int E, int K, int G, int64_t F,
                                      int dtype)
{
    (void)G;
    switch (op) {
    case MOE_OP_ROUTE:
        if (N < 0 || E < 1)
            return 0;
        return (size_t)N * (size_t)E * sizeof(float);
    case MOE_OP_DISPATCH_LAYOUT:
        if (N < 0 || K < 1 || E < 1 || E > MOE_MAX_EXPERTS)
            return 0;
        return layout_workspace_bytes(N * (int64_t)K, E);
    case MOE_OP_GROUPED_FFN:
        if (N < 0 || H < 1 || F < 1 || E < 1 || (dtype != MOE_BF16 && dtype != MOE_F32))
            return 0;
        return ffn_workspace_bytes(N, H, F, E, dtype);
    default:
        return 0;
    }
}

extern "C" int moe_route(const void *x, int dtype, int64_t N, int64_t H, const float *W_r,
                         const float *bias, int E, int K, int score_mode, int32_t *topk_idx,
                         float *topk_w, float *logits_opt, void *ws, size_t ws_bytes, void *stream)
{
    clear_error();
    MOE_TRY(check_dtype(dtype));
    MOE_TRY(check_routing_sizes(N, K, E));
    MOE_TRY(check_rows("H", H, dtype));
    if (K > MOE_MAX_TOPK)
        return fail(MOE_ERR_UNSUPPORTED, "K=%d exceeds MOE_MAX_TOPK=%d", K, MOE_MAX_TOPK);
    if (score_mode != MOE_SCORE_SOFTMAX_TOPK && score_mode != MOE_SCORE_SIGMOID_TOPK)
        return fail(MOE_ERR_ARG, "unknown score_mode %d", score_mode);
    if (N == 0)
        return MOE_OK;
    MOE_NEED(x);
    MOE_NEED(W_r);
    MOE_NEED(topk_idx);
    MOE_NEED(topk_w);
    if (bias && !aligned16(bias))
        return fail(MOE_ERR_ARG, "bias must be 16-byte aligned");
    float *logits = logits_opt;
    if (!logits) {
        size_t need = (size_t)N * (size_t)E * sizeof(float);
        if (!ws || ws_bytes < need)
            return fail(MOE_ERR_WORKSPACE, "moe_route needs %zu workspace bytes when logits_opt is NULL (got %zu)",
                        need, ws ? ws_bytes : (size_t)0);
        logits = static_cast<float *>(ws);
    }
    if (!aligned16(logits))
        return fail(MOE_ERR_ARG, "logits buffer must be 16-byte aligned");
    return launch_route(x, dtype, N, H, W_r, bias, E, K, score_mode, topk_idx, topk_w, logits,
                        static_cast<hipStream_t>(stream));
}

extern "C" int moe_route_resolve_arrival(const void *x, int dtype, int64_t N, int64_t H, const float *W_r,
                                         const float *bias, int E, int K, int G, int score_mode,
                                         int32_t *topk_idx, float *topk_w, float *logits_opt,
                                         int32_t *expert_counts, int32_t *expert_offsets,
                                         int32_t *dest_counts, int32_t *dest_offsets, int32_t *slot_of_row,
                                         int32_t *row_of_slot, void *ws, size_t ws_bytes, void *stream)
{
    clear_error();
    MOE_TRY(check_dtype(dtype));
    MOE_TRY(check_routing_sizes(N, K, E));
    MOE_TRY(check_rows("H", H, dtype));
    if (K > MOE_MAX_TOPK)
        return fail(MOE_ERR_UNSUPPORTED, "K=%d exceeds MOE_MAX_TOPK=%d", K, MOE_MAX_TOPK);
    if (score_mode != MOE_SCORE_SOFTMAX_TOPK && score_mode != MOE_SCORE_SIGMOID_TOPK)
        return fail(MOE_ERR_ARG, "unknown score_mode %d", score_mode);
    if (G < 1 || E % G != 0)
        return fail(MOE_ERR_ARG, "G must divide E (got E=%d, G=%d)", E, G);
    if (!expert_counts || !expert_offsets || !dest_counts || !dest_offsets)
        return fail(MOE_ERR_ARG, "count and offset outputs must not be NULL");
    float *logits = logits_opt;
    if (N > 0) {
        MOE_NEED(x);
        MOE_NEED(W_r);
        MOE_NEED(topk_idx);
        MOE_NEED(topk_w);
        MOE_NEED(slot_of_row);
        MOE_NEED(row_of_slot);
        if (bias && !aligned16(bias))
            return fail(MOE_ERR_ARG, "bias must be 16-byte aligned");
        if (!logits) {
            size_t need = (size_t)N * (size_t)E * sizeof(float);
            if (!ws || ws_bytes < need)
                return fail(MOE_ERR_WORKSPACE,
                            "moe_route_resolve_arrival needs %zu workspace bytes when logits_opt is NULL (got %zu)", need,
                            ws ? ws_bytes : (size_t)0);
            logits = static_cast<float *>(ws);
        }
        if (!aligned16(logits))
            return fail(MOE_ERR_ARG, "logits buffer must be 16-byte aligned");
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    MOE_TRY(launch_arrival_clear(expert_counts, E, st));
    if (N > 0)
        MOE_TRY(launch_route(x, dtype, N, H, W_r, bias, E, K, score_mode, topk_idx, topk_w, logits, st, expert_counts,
                             slot_of_row));
    return launch_arrival_place(topk_idx, N * (int64_t)K, E, G, expert_counts, expert_offsets, dest_counts,
                                dest_offsets, slot_of_row, row_of_slot, st);
}

extern "C" int moe_dispatch_layout(const int32_t *topk_idx, int64_t N, int K, int E, int G,
                                   int32_t *expert_counts, int32_t *expert_offsets,
                                   int32_t *dest_counts, int32_t *dest_offsets,
                                   int32_t *slot_of_row, int32_t *row_of_slot, void *ws,
                                   size_t ws_bytes, void *stream)
{
    clear_error();
    MOE_TRY(check_routing_sizes(N, K, E));
    if (G < 1 || E % G != 0)
        return fail(MOE_ERR_ARG, "G must divide E (got E=%d, G=%d)", E, G);
    if (!expert_counts || !expert_offsets || !dest_counts || !dest_offsets)
        return fail(MOE_ERR_ARG, "count and offset outputs must not be NULL");
    int64_t R = N * (int64_t)K;
    if (R > 0) {
        if (!topk_idx || !slot_of_row || !row_of_slot)
            return fail(MOE_ERR_ARG, "topk_idx, slot_of_row and row_of_slot must not be NULL");
    }
    size_t need = layout_workspace_bytes(R, E);
    if (need && (!ws || ws_bytes < need))
        return fail(MOE_ERR_WORKSPACE, "moe_dispatch_layout needs %zu workspace bytes (got %zu)",
                    need, ws ? ws_bytes : (size_t)0);
    if (ws && !aligned16(ws))
        return fail(MOE_ERR_ARG, "ws must be 16-byte aligned");
    return launch_layout(topk_idx, R, E, G, expert_counts, expert_offsets, dest_counts,
                         dest_offsets, slot_of_row, row_of_slot, ws,
                         static_cast<hipStream_t>(stream));
}

extern "C" int moe_dispatch_layout_static(const int32_t *topk_idx, int64_t N, int K, int E, int G,
                                          int32_t *expert_counts, int32_t *expert_offsets,
                                          int32_t *dest_counts, int32_t *dest_offsets,
                                          int32_t *slot_of_row, int32_t *row_of_slot, void *stream)
{
    clear_error();
    MOE_TRY(check_routing_sizes(N, K, E));
    if (G < 1 || E % G != 0)
        return fail(MOE_ERR_ARG, "G must divide E (got E=%d, G=%d)", E, G);
    if (!expert_counts || !expert_offsets || !dest_counts || !dest_offsets)
        return fail(MOE_ERR_ARG, "count and offset outputs must not be NULL");
    int64_t R = N * (int64_t)K;
    if (R > 0 && (!topk_idx || !slot_of_row || !row_of_slot))
        return fail(MOE_ERR_ARG, "topk_idx, slot_of_row and row_of_slot must not be NULL");
    return launch_layout_static(topk_idx, R, E, G, expert_counts, expert_offsets, dest_counts,
                                dest_offsets, slot_of_row, row_of_slot, static_cast<hipStream_t>(stream));
}

extern "C" int moe_dispatch_layout_arrival(const int32_t *topk_idx, int64_t N, int K, int E, int G,
                                           int32_t *expert_counts, int32_t *expert_offsets,
                                           int32_t *dest_counts, int32_t *dest_offsets,
                                           int32_t *slot_of_row, int32_t *row_of_slot, void *stream)
{
    clear_error();
    MOE_TRY(check_routing_sizes(N, K, E));
    if (G < 1 || E % G != 0)
        return fail(MOE_ERR_ARG, "G must divide E (got E=%d, G=%d)", E, G);
    if (!expert_counts || !expert_offsets || !dest_counts || !dest_offsets)
        return fail(MOE_ERR_ARG, "count and offset outputs must not be NULL");
    int64_t R = N * (int64_t)K;
    if (R > 0 && (!topk_idx || !slot_of_row || !row_of_slot))
        return fail(MOE_ERR_ARG, "topk_idx, slot_of_row and row_of_slot must not be NULL");
    return launch_layout_arrival(topk_idx, R, E, G, expert_counts, expert_offsets, dest_counts,
                                 dest_offsets, slot_of_row, row_of_slot,
                                 static_cast<hipStream_t>(stream));
}

extern "C" int moe_permute(const void *x, int dtype, int64_t N, int64_t H, int K,
                           const int32_t *slot_of_row, const int32_t *row_of_slot, void *xp,
                           void *stream)
{
    clear_error();
    MOE_TRY(check_dtype(dtype));
    MOE_TRY(check_rows("H", H, dtype));
    if (N < 0 || K < 1 || N * (int64_t)K >= ((int64_t)1 << 31))
        return fail(MOE_ERR_ARG, "need N >= 0, K >= 1, N*K < 2^31 (got N=%lld, K=%d)", (long long)N, K);
    if (K > kWave)
        return fail(MOE_ERR_UNSUPPORTED, "moe_permute supports K <= %d (got %d)", kWave, K);
    if (N == 0)
        return MOE_OK;
    MOE_NEED(x);
    MOE_NEED(xp);
    if (!slot_of_row || !row_of_slot)
        return fail(MOE_ERR_ARG, "slot_of_row and row_of_slot must not be NULL");
    return launch_permute(x, H * elt_bytes(dtype), N, K, slot_of_row, xp,
                          static_cast<hipStream_t>(stream));
}

namespace moe {

static int check_ffn_common(int dtype, int64_t M, int64_t H, int64_t F, int E_local,
                            const int32_t *seg_offsets, void *ws, size_t ws_bytes)
{
    MOE_TRY(check_dtype(dtype));
    MOE_TRY(check_rows("H", H, dtype));
    MOE_TRY(check_rows("F", F, dtype));
    if (M < 0 || M >= ((int64_t)1 << 31))
        return fail(MOE_ERR_ARG, "M must be in [0, 2^31) (got %lld)", (long long)M);
    if (E_local < 1 || E_local > MOE_MAX_EXPERTS)
        return fail(MOE_ERR_ARG, "E_local must be in [1, %d] (got %d)", MOE_MAX_EXPERTS, E_local);
    MOE_TRY(check_ffn_shape(dtype, H, F));
    if (M == 0)
        return MOE_OK;
    if (!seg_offsets)
        return fail(MOE_ERR_ARG, "seg_offsets must not be NULL");
    size_t need = ffn_workspace_bytes(M, H, F, E_local, dtype);
    if (!ws || ws_bytes < need)
        return fail(MOE_ERR_WORKSPACE, "the grouped FFN needs %zu workspace bytes (got %zu)", need,
                    ws ? ws_bytes : (size_t)0);
    if (!aligned16(ws))
        return fail(MOE_ERR_ARG, "ws must be 16-byte aligned");
    return MOE_OK;
}

}  // namespace moe

extern "C" int moe_ffn_schedule(int dtype, int64_t M, int64_t H, int64_t F, int E_local,
                                const int32_t *seg_offsets, void *ws, size_t ws_bytes, void *stream)
{
    clear_error();
    MOE_TRY(check_ffn_common(dtype, M, H, F, E_local, seg_offsets, ws, ws_bytes));
    if (M == 0)
        return MOE_OK;
    return launch_ffn_schedule(dtype, M, H, F, E_local, seg_offsets, ws, static_cast<hipStream_t>(stream));
}

extern "C" int moe_ffn_status(int dtype, int64_t M, int64_t H, int64_t F, int E_local, const void *ws,
                              size_t ws_bytes, void *stream)
{
    clear_error();
    int32_t dummy_seg = 0; // check_ffn_common only tests seg_offsets for NULL
    MOE_TRY(check_ffn_common(dtype, M, H, F, E_local, &dummy_seg, const_cast<void *>(ws), ws_bytes));
    if (M == 0 || dtype == MOE_F32)
        return MOE_OK;
    return ffn_status(M, H, F, E_local, ws, static_cast<hipStream_t>(stream));
}

extern "C" int moe_ffn_gate_up(const void *xp, int dtype, int64_t M, int64_t H, int64_t F,
                               int E_local, const int32_t *seg_offsets, const void *W_gate,
                               const void *W_up, void *ws, size_t ws_bytes, void *stream)
{
    clear_error();
    MOE_TRY(check_ffn_common(dtype, M, H, F, E_local, seg_offsets, ws, ws_bytes));
    if (M == 0)
        return MOE_OK;
    MOE_NEED(xp);
    MOE_NEED(W_gate);
    MOE_NEED(W_up);
    return launch_ffn_gate_up(xp, dtype, M, H, F, E_local, seg_offsets, W_gate, W_up, ws,
                              static_cast<hipStream_t>(stream));
}

extern "C" int moe_ffn_gate_up_gather(const void *x, int dtype, int64_t N, int K, int64_t H, int64_t F,
                                      int E_local, const int32_t *seg_offsets,
                                      const int32_t *row_of_slot, const void *W_gate,
                                      const void *W_up, void *ws, size_t ws_bytes, void *stream)
{
    clear_error();
    if (N < 0 || K < 1 || N * (int64_t)K >= ((int64_t)1 << 31))
        return fail(MOE_ERR_ARG, "need N >= 0, K >= 1, N*K < 2^31 (got N=%lld, K=%d)", (long long)N, K);
    const int64_t M = N * K;
    MOE_TRY(check_ffn_common(dtype, M, H, F, E_local, seg_offsets, ws, ws_bytes));
    if (M == 0)
        return MOE_OK;
    // the gathered rows are addressed with 32-bit byte offsets from x
    if (dtype == MOE_BF16 && (N + 1) * H * 2 + 4096 >= ((int64_t)1 << 32))
        return fail(MOE_ERR_UNSUPPORTED, "moe_ffn_gate_up_gather needs x below 4 GiB (got N=%lld, H=%lld)",
                    (long long)N, (long long)H);
    MOE_NEED(x);
    MOE_NEED(W_gate);
    MOE_NEED(W_up);
    if (!row_of_slot)
        return fail(MOE_ERR_ARG, "row_of_slot must not be NULL");
    return launch_ffn_gate_up(x, dtype, M, H, F, E_local, seg_offsets, W_gate, W_up, ws,
                              static_cast<hipStream_t>(stream), row_of_slot, K, N);
}

extern "C" int moe_ffn_down(int dtype, int64_t M, int64_t H, int64_t F, int E_local,
                            const int32_t *seg_offsets, const void *W_down, void *y, void *ws,
                            size_t ws_bytes, void *stream)
{
    clear_error();
    MOE_TRY(check_ffn_common(dtype, M, H, F, E_local, seg_offsets, ws, ws_bytes));
    if (M == 0)
        return MOE_OK;
    MOE_NEED(W_down);
    MOE_NEED(y);
    return launch_ffn_down(dtype, M, H, F, E_local, seg_offsets, W_down, y, ws,
                           static_cast<hipStream_t>(stream));
}

extern "C" int moe_ffn_down_combine(int dtype, int64_t N, int K, int64_t H, int64_t F, int E_local,
                                    const int32_t *seg_offsets, const void *W_down,
                                    const int32_t *row_of_slot, const float *topk_w, float *sums,
                                    void *out, void *ws, size_t ws_bytes, void *stream)
{
    clear_error();
    if (N < 0 || K < 1 || K > MOE_MAX_TOPK || N * (int64_t)K >= ((int64_t)1 << 31))
        return fail(MOE_ERR_ARG, "N >= 0, 1 <= K <= %d and N*K < 2^31 are required (got N=%lld, K=%d)",
                    MOE_MAX_TOPK, (long long)N, K);
    const int64_t M = N * (int64_t)K;
    MOE_TRY(check_ffn_common(dtype, M, H, F, E_local, seg_offsets, ws, ws_bytes));
    if (dtype != MOE_BF16)
        return fail(MOE_ERR_UNSUPPORTED, "moe_ffn_down_combine is built for MOE_BF16 only");
    if (M == 0)
        return MOE_OK;
    MOE_NEED(W_down);
    MOE_NEED(row_of_slot);
    MOE_NEED(topk_w);
    MOE_NEED(sums);
    MOE_NEED(out);
    if (!aligned16(sums) || !aligned16(out))
        return fail(MOE_ERR_ARG, "sums and out must be 16-byte aligned");
    return launch_ffn_down_combine(N, K, H, F, E_local, W_down, row_of_slot, topk_w, sums, out, ws,
                                   static_cast<hipStream_t>(stream));
}

extern "C" int moe_grouped_ffn(const void *xp, int dtype, int64_t M, int64_t H, int64_t F,
                               int E_local, const int32_t *seg_offsets, const void *W_gate,
                               const void *W_up, const void *W_down, void *y, void *ws,
                               size_t ws_bytes, void *stream)
{
    clear_error();
    MOE_TRY(check_ffn_common(dtype, M, H, F, E_local, seg_offsets, ws, ws_bytes));
    if (M == 0)
        return MOE_OK;
    MOE_NEED(xp);
    MOE_NEED(W_gate);
    MOE_NEED(W_up);
    MOE_NEED(W_down);
    MOE_NEED(y);
    hipStream_t st = static_cast<hipStream_t>(stream);
    MOE_TRY(launch_ffn_schedule(dtype, M, H, F, E_local, seg_offsets, ws, st));
    MOE_TRY(launch_ffn_gate_up(xp, dtype, M, H, F, E_local, seg_offsets, W_gate, W_up, ws, st));
    return launch_ffn_down(dtype, M, H, F, E_local, seg_offsets, W_down, y, ws, st);
}

extern "C" int moe_ffn_gate_up_down(const void *xp, int dtype, int64_t M, int64_t H, int64_t F,
                                    int E_local, const int32_t *seg_offsets, const void *W_gate,
                                    const void *W_up, const void *W_down, void *y, void *ws,
                                    size_t ws_bytes, int64_t wait_limit, void *stream)
{
    clear_error();
    MOE_TRY(check_ffn_common(dtype, M, H, F, E_local, seg_offsets, ws, ws_bytes));
    if (wait_limit < 0)
        return fail(MOE_ERR_ARG, "wait_limit must be >= 0 (got %lld)", (long long)wait_limit);
    if (M == 0)
        return MOE_OK;
    MOE_NEED(xp);
    MOE_NEED(W_gate);
    MOE_NEED(W_up);
    MOE_NEED(W_down);
    MOE_NEED(y);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == MOE_BF16) {
        // A down-projection tile reads rows of `a` while other rows are still being written by other
        // XCDs.  A cache line that held rows of two row tiles could be fetched for the first and found,
        // stale, for the second; rows that are whole lines (F % 64 == 0 holds for every bf16 FFN, and
        // `a` starts the workspace) rule that out.
        if (reinterpret_cast<uintptr_t>(ws) % 128 != 0)
            return fail(MOE_ERR_UNSUPPORTED,
                        "moe_ffn_gate_up_down needs a 128-byte aligned ws (rows of the activation must be whole "
                        "cache lines); use moe_ffn_gate_up + moe_ffn_down");
        return launch_ffn_gate_up_down(xp, M, H, F, E_local, W_gate, W_up, W_down, y, ws, wait_limit, st);
    }
    // fp32 (correctness path): the two simple kernels, one after the other
    MOE_TRY(launch_ffn_gate_up(xp, dtype, M, H, F, E_local, seg_offsets, W_gate, W_up, ws, st));
    return launch_ffn_down(dtype, M, H, F, E_local, seg_offsets, W_down, y, ws, st);
}

extern "C" int moe_combine(const void *y, int dtype, int64_t N, int64_t H, int K,
                           const int32_t *slot_of_row, const float *topk_w, void *out,
                           void *stream)
{
    clear_error();
    MOE_TRY(check_dtype(dtype));
    MOE_TRY(check_rows("H", H, dtype));
    if (N < 0 || K < 1 || K > MOE_MAX_TOPK || N * (int64_t)K >= ((int64_t)1 << 31))
        return fail(MOE_ERR_ARG, "need N >= 0, 1 <= K <= %d, N*K < 2^31 (got N=%lld, K=%d)",
                    MOE_MAX_TOPK, (long long)N, K);
    if (N == 0)
        return MOE_OK;
    MOE_NEED(y);
    MOE_NEED(out);
    if (!slot_of_row || !topk_w)
        return fail(MOE_ERR_ARG, "slot_of_row and topk_w must not be NULL");
    return launch_combine(y, dtype, N, H, K, slot_of_row, topk_w, out,
                          static_cast<hipStream_t>(stream));
}
