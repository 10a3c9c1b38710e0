// Routing (Section II-A, step 1): gating logits in the fixed fp32 order that makes
// the top-K selection reproducible bit for bit, then selection and normalisation.
//
// Order of the logit sum ("R64"): 64 partial sums, partial l takes
// h = l, l+64, ... ascending with one fused multiply-add per term; the partials
// are folded in six pairwise rounds s = 32,...,1 (p[l] + p[l^s]); bias last.
// A wavefront maps onto it directly: lane l owns partial l.  Each wavefront
// carries a kTok x kExp register tile of (token, expert) pairs so that every
// x and W_r value fetched is used kExp resp. kTok times.  The six rounds are done
// as a halving exchange: in round s a lane keeps the half of its values chosen by
// its own bit s and receives the partner's copy of that half, so 63 exchanges
// fold all 64 values and lane i ends with value i - the same additions, pair by
// pair, as folding every value separately.
//
// This step runs on the plain vector ALUs: matrix-core accumulation order is not
// exposed, so it could not be matched on a CPU.
#include <math.h>

#include "common.h"

namespace moe {

constexpr int kTok = 8;
constexpr int kExp = 8;
constexpr int kRouteWaves = 4;

template <bool kBf16>
__device__ __forceinline__ float load_x(const void *x, int64_t i)
{
    if (kBf16)
        return bf16_bits_to_f32(static_cast<const uint16_t *>(x)[i]);
    return static_cast<const float *>(x)[i];
}

template <int kHalf>
__device__ __forceinline__ void fold_round(float *v, bool upper)
{
#pragma unroll
    for (int i = 0; i < kHalf; ++i) {
        float keep = upper ? v[i + kHalf] : v[i];
        float send = upper ? v[i] : v[i + kHalf];
        v[i] = keep + __shfl_xor(send, kHalf);
    }
}

template <bool kBf16>
__global__ __launch_bounds__(kWave *kRouteWaves) void router_logits(
    const void *__restrict__ x, int64_t N, int64_t H, const float *__restrict__ W_r,
    const float *__restrict__ bias, int E, float *__restrict__ logits)
{
    const int lane = threadIdx.x % kWave;
    const int64_t n0 = ((int64_t)blockIdx.x * kRouteWaves + threadIdx.x / kWave) * kTok;
    const int e0 = blockIdx.y * kExp;
    if (n0 >= N)
        return;

    int64_t xrow[kTok];
#pragma unroll
    for (int t = 0; t < kTok; ++t) {
        int64_t n = n0 + t;
        xrow[t] = (n < N ? n : N - 1) * H;
    }
    int ecol[kExp];
#pragma unroll
    for (int j = 0; j < kExp; ++j)
        ecol[j] = (e0 + j < E) ? e0 + j : E - 1;

    float acc[kTok * kExp];
#pragma unroll
    for (int i = 0; i < kTok * kExp; ++i)
        acc[i] = 0.0f;

    const bool full = (e0 + kExp <= E) && (E % 4 == 0);
    if (full) {
        for (int64_t h = lane; h < H; h += kWave) {
            const f32x4 *wp = reinterpret_cast<const f32x4 *>(W_r + h * E + e0);
            f32x4 w0 = wp[0], w1 = wp[1];
            float wv[kExp] = {w0[0], w0[1], w0[2], w0[3], w1[0], w1[1], w1[2], w1[3]};
            float xv[kTok];
#pragma unroll
            for (int t = 0; t < kTok; ++t)
                xv[t] = load_x<kBf16>(x, xrow[t] + h);
#pragma unroll
            for (int t = 0; t < kTok; ++t)
#pragma unroll
                for (int j = 0; j < kExp; ++j)
                    acc[t * kExp + j] = fmaf(xv[t], wv[j], acc[t * kExp + j]);
        }
    } else {
        for (int64_t h = lane; h < H; h += kWave) {
            float wv[kExp], xv[kTok];
#pragma unroll
            for (int j = 0; j < kExp; ++j)
                wv[j] = W_r[h * E + ecol[j]];
#pragma unroll
            for (int t = 0; t < kTok; ++t)
                xv[t] = load_x<kBf16>(x, xrow[t] + h);
#pragma unroll
            for (int t = 0; t < kTok; ++t)
#pragma unroll
                for (int j = 0; j < kExp; ++j)
                    acc[t * kExp + j] = fmaf(xv[t], wv[j], acc[t * kExp + j]);
        }
    }

    fold_round<32>(acc, lane & 32);
    fold_round<16>(acc, lane & 16);
    fold_round<8>(acc, lane & 8);
    fold_round<4>(acc, lane & 4);
    fold_round<2>(acc, lane & 2);
    fold_round<1>(acc, lane & 1);

    // lane i now holds pair i = t * kExp + j
    const int t = lane / kExp, j = lane % kExp;
    const int64_t n = n0 + t;
    const int e = e0 + j;
    if (n < N && e < E) {
        float v = acc[0];
        if (bias)
            v = v + bias[e];
        logits[n * E + e] = v;
    }
}

// (value, index) order of the selection: larger logit first, equal logits to the lower index.
__device__ __forceinline__ bool better(float va, int ia, float vb, int ib)
{
    return (va > vb) || (va == vb && ia < ib);
}

constexpr int kMaxPerLane = MOE_MAX_EXPERTS / kWave;

// One wavefront per token.  Lane l holds experts l, l+64, ...
__global__ __launch_bounds__(kWave *kRouteWaves) void router_topk(
    const float *__restrict__ logits, int64_t N, int E, int K, int score_mode,
    int32_t *__restrict__ topk_idx, float *__restrict__ topk_w)
{
    const int lane = threadIdx.x % kWave;
    const int64_t n = (int64_t)blockIdx.x * kRouteWaves + threadIdx.x / kWave;
    if (n >= N)
        return;
    const float *row = logits + n * E;
    const int per = (E + kWave - 1) / kWave;
    float val[kMaxPerLane];
#pragma unroll
    for (int i = 0; i < kMaxPerLane; ++i) {
        int e = i * kWave + lane;
        val[i] = (i < per && e < E) ? row[e] : 0.0f;
    }
    uint32_t taken = 0;
#pragma unroll
    for (int i = 0; i < kMaxPerLane; ++i)
        if (!(i < per && i * kWave + lane < E))
            taken |= 1u << i; // slots past E never compete

    float my_logit = 0.0f; // lane k keeps the k-th pick
    int my_pick = 0;
    for (int k = 0; k < K; ++k) {
        float bv = 0.0f;
        int bi = -1;
#pragma unroll
        for (int i = 0; i < kMaxPerLane; ++i) {
            if (i < per && !(taken & (1u << i))) {
                int e = i * kWave + lane;
                if (bi < 0 || better(val[i], e, bv, bi)) {
                    bv = val[i];
                    bi = e;
                }
            }
        }
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) {
            float ov = __shfl_xor(bv, s);
            int oi = __shfl_xor(bi, s);
            if (oi >= 0 && (bi < 0 || better(ov, oi, bv, bi))) {
                bv = ov;
                bi = oi;
            }
        }
        // every lane agrees on (bv, bi); its owner retires it
        if ((bi % kWave) == lane)
            taken |= 1u << (bi / kWave);
        if (lane == k) {
            my_logit = bv;
            my_pick = bi;
        }
    }

    const float top = __shfl(my_logit, 0);
    float s = 0.0f;
    if (lane < K)
        s = (score_mode == MOE_SCORE_SOFTMAX_TOPK) ? expf(my_logit - top)
                                                   : 1.0f / (1.0f + expf(-my_logit));
    float sum = s;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1)
        sum += __shfl_xor(sum, d);
    if (lane < K) {
        topk_idx[n * K + lane] = my_pick;
        topk_w[n * K + lane] = s / sum;
    }
}

int launch_route(const void *x, int dtype, int64_t N, int64_t H, const float *W_r,
                 const float *bias, int E, int K, int score_mode, int32_t *topk_idx,
                 float *topk_w, float *logits, hipStream_t st)
{
    const dim3 block(kWave * kRouteWaves);
    const dim3 grid1((unsigned)ceil_div(N, (int64_t)kTok * kRouteWaves), (unsigned)ceil_div(E, kExp));
    if (dtype == MOE_BF16)
        hipLaunchKernelGGL(router_logits<true>, grid1, block, 0, st, x, N, H, W_r, bias, E, logits);
    else
        hipLaunchKernelGGL(router_logits<false>, grid1, block, 0, st, x, N, H, W_r, bias, E, logits);
    const dim3 grid2((unsigned)ceil_div(N, kRouteWaves));
    hipLaunchKernelGGL(router_topk, grid2, block, 0, st, logits, N, E, K, score_mode, topk_idx,
                       topk_w);
    return check_launch("moe_route");
}

}  // namespace moe
