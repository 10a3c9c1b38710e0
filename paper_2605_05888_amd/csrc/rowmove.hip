// Row moves of the dispatch and combine steps (Section II-A, steps 2, 4, 5).
// Both are pure HBM traffic: 16-byte vector accesses, one wavefront per token,
// whole rows contiguous so every access is fully coalesced.
//
//   permute : x[n,:] is read once and written to its K slots.
//             algorithmic bytes = N*H*b (read) + N*K*H*b (write) + 4*N*K (slots)
//   combine : K rows are gathered per token, scaled, summed in fp32 (k ascending)
//             and rounded once.  bytes = N*K*H*b (read) + N*H*b (write) + 8*N*K
#include <type_traits>

#include "common.h"

namespace moe {

constexpr int kTokensPerBlock = 4; // one wavefront each
#ifndef MOE_COMBINE_U
#define MOE_COMBINE_U 4 // 16-byte chunks of a row a lane gathers at a time (per k), at most
#endif

// Value of lane k (k wave-uniform) whatever lanes are active: the chunk loops below run a different
// number of times per lane, and a cross-lane read that honours the execution mask (__shfl) returns 0
// for a lane that has already left the loop.
__device__ __forceinline__ int32_t lane_value(int32_t v, int k) { return __builtin_amdgcn_readlane(v, k); }
__device__ __forceinline__ float lane_value(float v, int k)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int32_t)__float_as_uint(v), k));
}

__global__ __launch_bounds__(kWave *kTokensPerBlock) void permute_rows(
    const u32x4 *__restrict__ x, int chunks, int64_t N, int K,
    const int32_t *__restrict__ slot_of_row, u32x4 *__restrict__ xp)
{
    const int lane = threadIdx.x % kWave;
    const int64_t n = (int64_t)blockIdx.x * kTokensPerBlock + threadIdx.x / kWave;
    if (n >= N)
        return;
    // lane k keeps slot k of this token
    int32_t my_slot = (lane < K) ? slot_of_row[n * K + lane] : 0;
    const u32x4 *src = x + n * chunks;
    int c = lane;
    for (; c + 3 * kWave < chunks; c += 4 * kWave) {
        u32x4 v0 = __builtin_nontemporal_load(src + c);
        u32x4 v1 = __builtin_nontemporal_load(src + c + kWave);
        u32x4 v2 = __builtin_nontemporal_load(src + c + 2 * kWave);
        u32x4 v3 = __builtin_nontemporal_load(src + c + 3 * kWave);
        for (int k = 0; k < K; ++k) {
            u32x4 *dst = xp + (int64_t)lane_value(my_slot, k) * chunks + c;
            dst[0] = v0;
            dst[kWave] = v1;
            dst[2 * kWave] = v2;
            dst[3 * kWave] = v3;
        }
    }
    for (; c < chunks; c += kWave) {
        u32x4 v = __builtin_nontemporal_load(src + c);
        for (int k = 0; k < K; ++k)
            xp[(int64_t)lane_value(my_slot, k) * chunks + c] = v;
    }
}

template <bool kBf16>
__global__ __launch_bounds__(kWave *kTokensPerBlock) void combine_rows(
    const u32x4 *__restrict__ y, int chunks, int64_t N, int K,
    const int32_t *__restrict__ slot_of_row, const float *__restrict__ topk_w,
    u32x4 *__restrict__ out)
{
    const int lane = threadIdx.x % kWave;
    const int64_t n = (int64_t)blockIdx.x * kTokensPerBlock + threadIdx.x / kWave;
    if (n >= N)
        return;
    int32_t my_slot = (lane < K) ? slot_of_row[n * K + lane] : 0;
    float my_w = (lane < K) ? topk_w[n * K + lane] : 0.0f;
    // kU chunks of a row at a time, so that kU gathers per lane are in flight (a single one leaves
    // the small workloads, with only a few thousand wavefronts, waiting on memory latency)
    auto rows_of = [&](auto u_tag, int c) {
        constexpr int kU = decltype(u_tag)::value;
        float acc[kU][8];
#pragma unroll
        for (int u = 0; u < kU; ++u)
#pragma unroll
            for (int i = 0; i < 8; ++i)
                acc[u][i] = 0.0f;
        for (int k = 0; k < K; ++k) { // ascending k: the order of the sum is part of the contract
            const float w = lane_value(my_w, k);
            const u32x4 *src = y + (int64_t)lane_value(my_slot, k) * chunks + c;
            u32x4 v[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u)
                v[u] = __builtin_nontemporal_load(&src[u * kWave]); // read once: no need to keep it cached
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                if (kBf16) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        acc[u][2 * i] = fmaf(w, bf16_bits_to_f32(v[u][i] & 0xFFFFu), acc[u][2 * i]);
                        acc[u][2 * i + 1] = fmaf(w, __uint_as_float(v[u][i] & 0xFFFF0000u), acc[u][2 * i + 1]);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        acc[u][i] = fmaf(w, __uint_as_float(v[u][i]), acc[u][i]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            u32x4 o;
            if (kBf16) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    o[i] = pack_bf16x2(acc[u][2 * i], acc[u][2 * i + 1]);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    o[i] = __float_as_uint(acc[u][i]);
            }
            __builtin_nontemporal_store(o, &out[n * chunks + c + u * kWave]);
        }
    };
    int c = lane;
#if MOE_COMBINE_U == 8
    for (; c + 7 * kWave < chunks; c += 8 * kWave)
        rows_of(std::integral_constant<int, 8>{}, c);
#endif
    for (; c + 3 * kWave < chunks; c += 4 * kWave)
        rows_of(std::integral_constant<int, 4>{}, c);
    for (; c + kWave < chunks; c += 2 * kWave)
        rows_of(std::integral_constant<int, 2>{}, c);
    for (; c < chunks; c += kWave)
        rows_of(std::integral_constant<int, 1>{}, c);
}

int launch_permute(const void *x, int64_t row_bytes, int64_t N, int K, const int32_t *slot_of_row,
                   void *xp, hipStream_t st)
{
    const int chunks = (int)(row_bytes / 16);
    const unsigned blocks = (unsigned)ceil_div(N, kTokensPerBlock);
    hipLaunchKernelGGL(permute_rows, dim3(blocks), dim3(kWave * kTokensPerBlock), 0, st,
                       static_cast<const u32x4 *>(x), chunks, N, K, slot_of_row,
                       static_cast<u32x4 *>(xp));
    return check_launch("moe_permute");
}

int launch_combine(const void *y, int dtype, int64_t N, int64_t H, int K,
                   const int32_t *slot_of_row, const float *topk_w, void *out, hipStream_t st)
{
    const unsigned blocks = (unsigned)ceil_div(N, kTokensPerBlock);
    const dim3 block(kWave * kTokensPerBlock);
    if (dtype == MOE_BF16) {
        hipLaunchKernelGGL(combine_rows<true>, dim3(blocks), block, 0, st,
                           static_cast<const u32x4 *>(y), (int)(H * 2 / 16), N, K, slot_of_row,
                           topk_w, static_cast<u32x4 *>(out));
    } else {
        hipLaunchKernelGGL(combine_rows<false>, dim3(blocks), block, 0, st,
                           static_cast<const u32x4 *>(y), (int)(H * 4 / 16), N, K, slot_of_row,
                           topk_w, static_cast<u32x4 *>(out));
    }
    return check_launch("moe_combine");
}

}  // namespace moe
