// Shared declarations of the HIP MoE-layer library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/moe_hub.h"

namespace moe {

// Records a message for moe_last_error() and returns `code`.
int fail(int code, const char *fmt, ...);
void clear_error();

// Launch check: turns a pending HIP launch error into MOE_ERR_LAUNCH.
int check_launch(const char *what);

constexpr int kWave = 64;

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16)
{
    return __uint_as_float(bits16 << 16);
}

// Round-to-nearest-even fp32 -> bf16 bit pattern (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t b = __float_as_uint(f);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

// Two fp32 -> one register of two bf16 (lo in the low half), round-to-nearest-even in hardware
// (v_cvt_pk_bf16_f32).
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- per-step launchers (each validates nothing: api.hip has done it) ----
// row_pointer != nullptr: the top-K kernel also draws every routed row's local row id from
// row_pointer[expert] (which must be zero on entry) into rank[n*K + k].
int launch_route(const void *x, int dtype, int64_t N, int64_t H, const float *W_r,
                 const float *bias, int E, int K, int score_mode, int32_t *topk_idx,
                 float *topk_w, float *logits, hipStream_t st, int32_t *row_pointer = nullptr,
                 int32_t *rank = nullptr);

size_t layout_workspace_bytes(int64_t R, int E);
int launch_layout(const int32_t *topk_idx, int64_t R, int E, int G, int32_t *expert_counts,
                  int32_t *expert_offsets, int32_t *dest_counts, int32_t *dest_offsets,
                  int32_t *slot_of_row, int32_t *row_of_slot, void *ws, hipStream_t st);
int launch_layout_static(const int32_t *topk_idx, int64_t R, int E, int G, int32_t *expert_counts,
                         int32_t *expert_offsets, int32_t *dest_counts, int32_t *dest_offsets,
                         int32_t *slot_of_row, int32_t *row_of_slot, hipStream_t st);
int launch_layout_arrival(const int32_t *topk_idx, int64_t R, int E, int G, int32_t *expert_counts,
                          int32_t *expert_offsets, int32_t *dest_counts, int32_t *dest_offsets,
                          int32_t *slot_of_row, int32_t *row_of_slot, hipStream_t st);
// The two halves of the above around a rank pass done elsewhere: clear the E row pointers; turn
// ranks (in slot_of_row) and final pointers (= counts) into offsets and slots.
int launch_arrival_clear(int32_t *expert_counts, int E, hipStream_t st);
int launch_arrival_place(const int32_t *topk_idx, int64_t R, int E, int G, int32_t *expert_counts,
                         int32_t *expert_offsets, int32_t *dest_counts, int32_t *dest_offsets,
                         int32_t *slot_of_row, int32_t *row_of_slot, hipStream_t st);

int launch_permute(const void *x, int64_t row_bytes, int64_t N, int K,
                   const int32_t *slot_of_row, void *xp, hipStream_t st);

int launch_combine(const void *y, int dtype, int64_t N, int64_t H, int K,
                   const int32_t *slot_of_row, const float *topk_w, void *out, hipStream_t st);

size_t ffn_workspace_bytes(int64_t M, int64_t H, int64_t F, int E_local, int dtype);
int check_ffn_shape(int dtype, int64_t H, int64_t F);
int launch_ffn_schedule(int dtype, int64_t M, int64_t H, int64_t F, int E_local,
                        const int32_t *seg_offsets, void *ws, hipStream_t st);
int launch_ffn_gate_up(const void *xp, int dtype, int64_t M, int64_t H, int64_t F, int E_local,
                       const int32_t *seg_offsets, const void *W_gate, const void *W_up, void *ws,
                       hipStream_t st, const int32_t *gather_rows = nullptr, int K = 1, int64_t N = 0);
int launch_ffn_down(int dtype, int64_t M, int64_t H, int64_t F, int E_local,
                    const int32_t *seg_offsets, const void *W_down, void *y, void *ws,
                    hipStream_t st);
int launch_ffn_gate_up_down(const void *xp, int64_t M, int64_t H, int64_t F, int E_local, const void *W_gate,
                            const void *W_up, const void *W_down, void *y, void *ws, int64_t wait_limit,
                            hipStream_t st);
int ffn_status(int64_t M, int64_t H, int64_t F, int E_local, const void *ws, hipStream_t st);
int launch_ffn_down_combine(int64_t N, int K, int64_t H, int64_t F, int E_local, const void *W_down,
                            const int32_t *row_of_slot, const float *topk_w, float *sums, void *out,
                            void *ws, hipStream_t st);

}  // namespace moe
