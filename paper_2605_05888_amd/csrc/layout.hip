// Address resolution on the GPU (the software mediation of Section III-A):
// per-expert / per-destination counts, exclusive scan to region offsets, and the
// stable slot of every routed row.  Integer only, deterministic, no atomics.
//
// The flat row list r = n*K + k is cut into units of kUnitRows consecutive rows;
// one wavefront owns one unit.
//   pass 1  unit_hist[e][u] = rows of unit u routed to expert e
//   pass 2  per expert: exclusive scan over units (in place) and the total count
//   pass 3  every wavefront rebuilds the region offsets from the counts, starts
//           its cursors at offset[e] + unit_base[e][u] and walks its unit 64 rows
//           at a time; inside a 64-row step the rank among equal experts comes
//           from wavefront ballots, so the order is ascending r everywhere.
#include "common.h"

namespace moe {

constexpr int kUnitSteps = 8;                 // 64-row steps per unit
constexpr int kUnitRows = kWave * kUnitSteps; // rows per unit (one wavefront)
constexpr int kWavesPerBlock = 4;

static inline int64_t num_units(int64_t R) { return ceil_div(R, kUnitRows); }

size_t layout_workspace_bytes(int64_t R, int E)
{
    size_t b = (size_t)num_units(R) * (size_t)E * sizeof(int32_t);
    return (b + 255) & ~(size_t)255;
}

// Lanes of the wavefront whose (valid) expert equals this lane's expert.
__device__ __forceinline__ uint64_t same_expert_lanes(int e, bool valid, int nbits)
{
    uint64_t m = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
        bool bit = (e >> b) & 1;
        uint64_t bal = __ballot(valid && bit);
        m &= bit ? bal : ~bal;
    }
    return m;
}

__device__ __forceinline__ uint64_t lanes_below(int lane)
{
    return (lane == 0) ? 0ull : (~0ull >> (64 - lane));
}

__global__ __launch_bounds__(kWave *kWavesPerBlock) void layout_unit_hist(
    const int32_t *__restrict__ idx, int64_t R, int E, int nbits, int U, int32_t *__restrict__ unit_hist)
{
    extern __shared__ int32_t lds[];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    int32_t *cnt = lds + wave * E;
    const int u = blockIdx.x * kWavesPerBlock + wave;
    if (u >= U)
        return;
    for (int e = lane; e < E; e += kWave)
        cnt[e] = 0;
    const int64_t r0 = (int64_t)u * kUnitRows;
    for (int s = 0; s < kUnitSteps; ++s) {
        int64_t r = r0 + s * kWave + lane;
        int e = (r < R) ? idx[r] : -1;
        bool valid = (e >= 0) && (e < E);
        uint64_t m = same_expert_lanes(e, valid, nbits);
        if (valid && (m & lanes_below(lane)) == 0) // lowest lane of its group
            cnt[e] += __popcll(m);
    }
    for (int e = lane; e < E; e += kWave)
        unit_hist[(int64_t)e * U + u] = cnt[e];
}

// One wavefront per expert: unit_hist[e][*] becomes its exclusive scan over units.
__global__ __launch_bounds__(kWave) void layout_scan_units(int32_t *__restrict__ unit_hist, int U,
                                                          int32_t *__restrict__ expert_counts)
{
    const int e = blockIdx.x, lane = threadIdx.x;
    int32_t *row = unit_hist + (int64_t)e * U;
    int32_t running = 0;
    for (int base = 0; base < U; base += kWave) {
        int u = base + lane;
        int32_t v = (u < U) ? row[u] : 0;
        int32_t inc = v;
        for (int d = 1; d < kWave; d <<= 1) {
            int32_t t = __shfl_up(inc, d);
            if (lane >= d)
                inc += t;
        }
        if (u < U)
            row[u] = running + inc - v;
        running += __shfl(inc, kWave - 1);
    }
    if (lane == 0)
        expert_counts[e] = running;
}

__global__ __launch_bounds__(kWave *kWavesPerBlock) void layout_assign_slots(
    const int32_t *__restrict__ idx, int64_t R, int E, int G, int nbits, int U,
    const int32_t *__restrict__ unit_base, const int32_t *__restrict__ expert_counts,
    int32_t *__restrict__ expert_offsets, int32_t *__restrict__ dest_counts,
    int32_t *__restrict__ dest_offsets, int32_t *__restrict__ slot_of_row,
    int32_t *__restrict__ row_of_slot)
{
    extern __shared__ int32_t lds[];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    int32_t *cursor = lds + wave * (E + 1);
    const int u = blockIdx.x * kWavesPerBlock + wave;
    const bool writer = (blockIdx.x == 0 && wave == 0);
    if (u >= U && !writer)
        return;

    // region offsets: exclusive scan of the counts; lane owns a contiguous run of experts
    const int per = (E + kWave - 1) / kWave;
    const int e_lo = lane * per;
    int32_t mine = 0;
    for (int j = 0; j < per; ++j)
        if (e_lo + j < E)
            mine += expert_counts[e_lo + j];
    int32_t inc = mine;
    for (int d = 1; d < kWave; d <<= 1) {
        int32_t t = __shfl_up(inc, d);
        if (lane >= d)
            inc += t;
    }
    int32_t run = inc - mine;
    for (int j = 0; j < per; ++j)
        if (e_lo + j < E) {
            cursor[e_lo + j] = run;
            run += expert_counts[e_lo + j];
        }
    if (lane == kWave - 1)
        cursor[E] = inc; // total = N*K

    if (writer) {
        for (int e = lane; e <= E; e += kWave)
            expert_offsets[e] = cursor[e];
        const int Eg = E / G;
        for (int g = lane; g <= G; g += kWave) {
            int32_t o = cursor[g * Eg];
            dest_offsets[g] = o;
            if (g < G)
                dest_counts[g] = cursor[(g + 1) * Eg] - o;
        }
    }
    if (u >= U)
        return;

    for (int e = lane; e < E; e += kWave)
        cursor[e] += unit_base[(int64_t)e * U + u];

    const int64_t r0 = (int64_t)u * kUnitRows;
    for (int s = 0; s < kUnitSteps; ++s) {
        int64_t r = r0 + s * kWave + lane;
        int e = (r < R) ? idx[r] : -1;
        bool valid = (e >= 0) && (e < E);
        uint64_t m = same_expert_lanes(e, valid, nbits);
        uint64_t below = m & lanes_below(lane);
        int32_t base = valid ? cursor[e] : 0;
        if (valid) {
            int32_t slot = base + __popcll(below);
            slot_of_row[r] = slot;
            row_of_slot[slot] = (int32_t)r;
        }
        if (valid && below == 0)
            cursor[e] = base + __popcll(m);
    }
}

int launch_layout(const int32_t *topk_idx, int64_t R, int E, int G, int32_t *expert_counts,
                  int32_t *expert_offsets, int32_t *dest_counts, int32_t *dest_offsets,
                  int32_t *slot_of_row, int32_t *row_of_slot, void *ws, hipStream_t st)
{
    const int U = (int)num_units(R);
    int nbits = 1;
    while ((1 << nbits) < E)
        ++nbits;
    int32_t *unit_hist = static_cast<int32_t *>(ws);
    const int blocks = (int)ceil_div(U, kWavesPerBlock);
    if (U > 0) {
        hipLaunchKernelGGL(layout_unit_hist, dim3(blocks), dim3(kWave * kWavesPerBlock),
                           kWavesPerBlock * E * sizeof(int32_t), st, topk_idx, R, E, nbits, U,
                           unit_hist);
    }
    hipLaunchKernelGGL(layout_scan_units, dim3(E), dim3(kWave), 0, st, unit_hist, U, expert_counts);
    hipLaunchKernelGGL(layout_assign_slots, dim3(blocks > 0 ? blocks : 1),
                       dim3(kWave * kWavesPerBlock), kWavesPerBlock * (E + 1) * sizeof(int32_t), st,
                       topk_idx, R, E, G, nbits, U, unit_hist, expert_counts, expert_offsets,
                       dest_counts, dest_offsets, slot_of_row, row_of_slot);
    return check_launch("moe_dispatch_layout");
}

}  // namespace moe
