/*
 * CPU oracle for one GPU's share of an expert-parallel MoE layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * HIP library is checked against.  It shares no code with the HIP path and
 * must never be called from it; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg load it.
 *
 * The layer is the five-step flow of the paper's Section II-A (routing,
 * dispatch, expert computation, combine, scaling) with the dispatch step
 * split into the software "address-resolution mediation" of Section III-A
 * (count, derive the memory layout, derive per-token offsets) and the row
 * move itself.  Every function below writes out the definition of its step:
 * no blocking, no fusion, no reordering.  The only parallelism is an OpenMP
 * loop over independent tokens or rows.
 *
 * Floating point: everything is accumulated in fp64 from the stored values,
 * except the router logits.  The logits decide integers (the top-K indices),
 * so they are computed in fp32 in one fixed summation order ("R64", below)
 * that the GPU reproduces operation by operation.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -mfma -fopenmp -shared -fPIC
 * (-ffp-contract=off: only the explicit fmaf calls are fused.)
 *
 * Pins (tests/test_oracle_*.py): exact-rational brute force for R64 on tiny
 * inputs and fp64 dot products; stable sort of (-logit, index) pairs for the
 * selection; library softmax; numpy bincount / cumsum / stable argsort and an
 * O(R^2) rank count for the layout (and, for its arrival-order form, a stable
 * argsort of the experts taken in arrival order); float64 library matmuls, linearity and
 * equivariance for the FFN; identity experts for the combine.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_BF16 = 0, ORACLE_F32 = 1, ORACLE_F64 = 2 };
enum { ORACLE_SOFTMAX_TOPK = 0, ORACLE_SIGMOID_TOPK = 1 };

static double load_elt(const void *p, int dtype, int64_t i)
{
    if (dtype == ORACLE_BF16) {
        uint32_t b = (uint32_t)((const uint16_t *)p)[i] << 16;
        float f;
        memcpy(&f, &b, 4);
        return (double)f;
    }
    if (dtype == ORACLE_F32)
        return (double)((const float *)p)[i];
    return ((const double *)p)[i];
}

static float load_elt_f32(const void *p, int dtype, int64_t i)
{
    /* bf16 -> fp32 is exact; fp32 is itself */
    return (float)load_elt(p, dtype, i);
}

/* ---------------------------------------------------------------------- *
 * Routing, step 1 of Section II-A: gating scores.
 *
 * logit[n,e] = sum_h x[n,h] * W_r[h,e]  (+ bias[e]),  fp32, order R64:
 *   64 partial sums; partial l takes h = l, l+64, l+128, ... in ascending
 *   order, each step one fused multiply-add (round once);
 *   then six pairwise rounds s = 32,16,8,4,2,1:  p[l] = p[l] + p[l ^ s];
 *   p[0] is the sum.  The bias is added last with one fp32 addition.
 * W_r is [H,E] row-major fp32.  x is [N,H] in `dtype` (bf16 or f32).
 * ---------------------------------------------------------------------- */
float oracle_logit_r64(const void *x, int dtype, int64_t H, int64_t n,
                       const float *W_r, int E, int e)
{
    float p[64], q[64];
    for (int l = 0; l < 64; ++l)
        p[l] = 0.0f;
    for (int64_t h = 0; h < H; ++h) {
        float a = load_elt_f32(x, dtype, n * H + h);
        float b = W_r[h * E + e];
        p[h & 63] = fmaf(a, b, p[h & 63]);
    }
    for (int s = 32; s >= 1; s >>= 1) {
        for (int l = 0; l < 64; ++l)
            q[l] = p[l] + p[l ^ s];
        memcpy(p, q, sizeof p);
    }
    return p[0];
}

void oracle_logits(const void *x, int dtype, int64_t N, int64_t H,
                   const float *W_r, const float *bias, int E, float *logits)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int e = 0; e < E; ++e) {
            float v = oracle_logit_r64(x, dtype, H, n, W_r, E, e);
            if (bias)
                v = v + bias[e];
            logits[n * E + e] = v;
        }
}

/* ---------------------------------------------------------------------- *
 * Routing, continued: selection of the top-K experts and normalisation.
 *
 * Selection is on the fp32 logits: K times, take the not yet taken expert
 * with the largest logit; equal logits go to the lower expert index.
 * topk_idx[n,k] is the k-th pick (descending preference).
 * Weights (fp64):
 *   SOFTMAX_TOPK: softmax over the K selected logits
 *   SIGMOID_TOPK: sigmoid of each selected logit, divided by their sum
 * ---------------------------------------------------------------------- */
void oracle_topk(const float *logits, int64_t N, int E, int K, int score_mode,
                 int32_t *topk_idx, double *topk_w)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const float *row = logits + n * E;
        char *taken = (char *)calloc((size_t)E, 1);
        double *s = (double *)malloc(sizeof(double) * (size_t)K);
        for (int k = 0; k < K; ++k) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e])
                    continue;
                if (best < 0 || row[e] > row[best])
                    best = e; /* strict >: a later equal logit never replaces */
            }
            taken[best] = 1;
            topk_idx[n * K + k] = best;
        }
        double top = (double)row[topk_idx[n * K]];
        double sum = 0.0;
        for (int k = 0; k < K; ++k) {
            double z = (double)row[topk_idx[n * K + k]];
            s[k] = (score_mode == ORACLE_SOFTMAX_TOPK) ? exp(z - top)
                                                       : 1.0 / (1.0 + exp(-z));
            sum += s[k];
        }
        for (int k = 0; k < K; ++k)
            topk_w[n * K + k] = s[k] / sum;
        free(s);
        free(taken);
    }
}

/* ---------------------------------------------------------------------- *
 * Mediation (Section III-A): per-expert and per-destination counts, the
 * exclusive scan that lays the expert regions out back to back, and the
 * slot of every routed row.  Regions are dense and nothing is dropped
 * (Section IV-A: conservative regions, dense packing; address of a slot is
 * base + slot * RowSize + RowOffset).  Order inside a region: by token, then
 * by k, i.e. ascending flat row r = n*K + k (a stable counting sort).
 * Experts are blocked onto destinations: dest(e) = e / (E/G).
 * Serial on purpose: it is the serial layout computation of the text.
 * ---------------------------------------------------------------------- */
void oracle_layout(const int32_t *topk_idx, int64_t N, int K, int E, int G,
                   int32_t *expert_counts, int32_t *expert_offsets,
                   int32_t *dest_counts, int32_t *dest_offsets,
                   int32_t *slot_of_row, int32_t *row_of_slot)
{
    int64_t R = N * K;
    int Eg = E / G;
    for (int e = 0; e < E; ++e)
        expert_counts[e] = 0;
    for (int64_t r = 0; r < R; ++r)
        expert_counts[topk_idx[r]] += 1;
    expert_offsets[0] = 0;
    for (int e = 0; e < E; ++e)
        expert_offsets[e + 1] = expert_offsets[e] + expert_counts[e];
    for (int g = 0; g < G; ++g) {
        int32_t c = 0;
        for (int j = 0; j < Eg; ++j)
            c += expert_counts[g * Eg + j];
        dest_counts[g] = c;
    }
    dest_offsets[0] = 0;
    for (int g = 0; g < G; ++g)
        dest_offsets[g + 1] = dest_offsets[g] + dest_counts[g];
    int32_t *cursor = (int32_t *)calloc((size_t)E, sizeof(int32_t));
    for (int64_t r = 0; r < R; ++r) {
        int e = topk_idx[r];
        int32_t slot = expert_offsets[e] + cursor[e];
        cursor[e] += 1;
        slot_of_row[r] = slot;
        row_of_slot[slot] = (int32_t)r;
    }
    free(cursor);
}

/* ---------------------------------------------------------------------- *
 * The same address resolution with the allocation unit of Section IV-A3 in
 * place of the stable order: each region has a row pointer; an arriving row
 * takes the pointer's value as its local row id and increments it, so rows
 * are packed densely in the order they arrive.  arrival[i] is the flat row
 * that arrives i-th (a permutation of 0..R-1).  Region bases are the same
 * exclusive scan of the counts as above (counts do not depend on the
 * order); slot = base[e] + local row id (the address formula of that
 * section with RowSize factored out).  row_of_slot is the source
 * information of Section IV-A4.
 * ---------------------------------------------------------------------- */
void oracle_layout_arrival(const int32_t *topk_idx, int64_t N, int K, int E, int G,
                           const int32_t *arrival,
                           int32_t *expert_counts, int32_t *expert_offsets,
                           int32_t *dest_counts, int32_t *dest_offsets,
                           int32_t *slot_of_row, int32_t *row_of_slot)
{
    int64_t R = N * K;
    int Eg = E / G;
    int32_t *row_pointer = (int32_t *)calloc((size_t)E, sizeof(int32_t));
    int32_t *local_id = (int32_t *)malloc((size_t)(R > 0 ? R : 1) * sizeof(int32_t));
    for (int64_t i = 0; i < R; ++i) {
        int32_t r = arrival[i];
        int e = topk_idx[r];
        local_id[r] = row_pointer[e];
        row_pointer[e] += 1;
    }
    expert_offsets[0] = 0;
    for (int e = 0; e < E; ++e) {
        expert_counts[e] = row_pointer[e];
        expert_offsets[e + 1] = expert_offsets[e] + row_pointer[e];
    }
    for (int g = 0; g <= G; ++g)
        dest_offsets[g] = expert_offsets[g * Eg];
    for (int g = 0; g < G; ++g)
        dest_counts[g] = dest_offsets[g + 1] - dest_offsets[g];
    for (int64_t r = 0; r < R; ++r) {
        int32_t slot = expert_offsets[topk_idx[r]] + local_id[r];
        slot_of_row[r] = slot;
        row_of_slot[slot] = (int32_t)r;
    }
    free(local_id);
    free(row_pointer);
}

/* ---------------------------------------------------------------------- *
 * Dispatch, step 2 of Section II-A, local half: the row of token n goes,
 * unchanged, to each of its K slots.  row_bytes = H * element size.
 * ---------------------------------------------------------------------- */
void oracle_permute(const void *x, int64_t row_bytes, int64_t N, int K,
                    const int32_t *slot_of_row, void *xp)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < N * K; ++r)
        memcpy((char *)xp + (int64_t)slot_of_row[r] * row_bytes,
               (const char *)x + (r / K) * row_bytes, (size_t)row_bytes);
}

/* ---------------------------------------------------------------------- *
 * Expert computation, step 3 of Section II-A: two GEMMs with an activation
 * between them, here the gated (SwiGLU) form:
 *   g = W_gate_e xp_row,  u = W_up_e xp_row            (length F)
 *   a = g / (1 + exp(-g)) * u
 *   y = W_down_e a                                      (length H)
 * for every row of expert e's segment [seg_offsets[e], seg_offsets[e+1]).
 * Weights are "out x in": W_gate, W_up [E,F,H]; W_down [E,H,F].
 * Computes the rows listed in `rows` (nrows of them; all M rows when rows is
 * NULL) into y_out[nrows,H], fp64, no intermediate rounding.
 * ---------------------------------------------------------------------- */
void oracle_ffn_rows(const void *xp, int dtype, int64_t M, int64_t H, int64_t F,
                     int E_local, const int32_t *seg_offsets,
                     const void *W_gate, const void *W_up, const void *W_down,
                     int wdtype, const int64_t *rows, int64_t nrows, double *y_out)
{
    if (!rows)
        nrows = M;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t m = rows ? rows[i] : i;
        int e = -1;
        for (int j = 0; j < E_local; ++j)
            if (m >= seg_offsets[j] && m < seg_offsets[j + 1])
                e = j;
        double *yrow = y_out + i * H;
        if (e < 0) { /* row outside every segment: not computed */
            for (int64_t c = 0; c < H; ++c)
                yrow[c] = 0.0;
            continue;
        }
        double *a = (double *)malloc(sizeof(double) * (size_t)F);
        for (int64_t f = 0; f < F; ++f) {
            double g = 0.0, u = 0.0;
            int64_t wbase = ((int64_t)e * F + f) * H;
            for (int64_t h = 0; h < H; ++h) {
                double xv = load_elt(xp, dtype, m * H + h);
                g += xv * load_elt(W_gate, wdtype, wbase + h);
                u += xv * load_elt(W_up, wdtype, wbase + h);
            }
            a[f] = g / (1.0 + exp(-g)) * u;
        }
        for (int64_t c = 0; c < H; ++c) {
            double acc = 0.0;
            int64_t wbase = ((int64_t)e * H + c) * F;
            for (int64_t f = 0; f < F; ++f)
                acc += a[f] * load_elt(W_down, wdtype, wbase + f);
            yrow[c] = acc;
        }
        free(a);
    }
}

/* ---------------------------------------------------------------------- *
 * Combine and scaling, steps 4-5 of Section II-A: every token gathers its K
 * expert outputs from their slots and sums them weighted by the routing
 * weights, k ascending.  Computes the tokens listed in `tokens` (all N when
 * NULL) into out[ntok,H], fp64.
 * ---------------------------------------------------------------------- */
void oracle_combine(const void *y, int dtype, int64_t N, int64_t H, int K,
                    const int32_t *slot_of_row, const double *topk_w,
                    const int64_t *tokens, int64_t ntok, double *out)
{
    if (!tokens)
        ntok = N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < ntok; ++i) {
        int64_t n = tokens ? tokens[i] : i;
        for (int64_t c = 0; c < H; ++c) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += topk_w[n * K + k] *
                       load_elt(y, dtype, (int64_t)slot_of_row[n * K + k] * H + c);
            out[i * H + c] = acc;
        }
    }
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
