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
#include <atomic>

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
    // the unit's rows are fetched up front: one memory round trip per unit instead of one per step
    int ev[kUnitSteps];
#pragma unroll
    for (int s = 0; s < kUnitSteps; ++s) {
        const int64_t r = r0 + s * kWave + lane;
        ev[s] = (r < R) ? idx[r] : -1;
    }
#pragma unroll
    for (int s = 0; s < kUnitSteps; ++s) {
        const int e = ev[s];
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

// One wavefront: off[0..E] = exclusive scan of expert_counts[0..E), off[E] = total.
// Each lane owns a contiguous run of experts.
__device__ __forceinline__ void region_offsets(const int32_t *__restrict__ expert_counts, int E,
                                               int lane, int32_t *off)
{
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
            off[e_lo + j] = run;
            run += expert_counts[e_lo + j];
        }
    if (lane == kWave - 1)
        off[E] = inc; // total = N*K
}

// Block 0's first wavefront publishes the offsets and the per-destination view.
__device__ __forceinline__ void write_region_tables(const int32_t *off, int E, int G, int lane,
                                                    int32_t *__restrict__ expert_offsets,
                                                    int32_t *__restrict__ dest_counts,
                                                    int32_t *__restrict__ dest_offsets)
{
    for (int e = lane; e <= E; e += kWave)
        expert_offsets[e] = off[e];
    const int Eg = E / G;
    for (int g = lane; g <= G; g += kWave) {
        int32_t o = off[g * Eg];
        dest_offsets[g] = o;
        if (g < G)
            dest_counts[g] = off[(g + 1) * Eg] - o;
    }
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

    // the unit's rows are fetched before the cursors are set up: their round trip runs under that
    const int64_t r0 = (int64_t)u * kUnitRows;
    int ev[kUnitSteps];
#pragma unroll
    for (int s = 0; s < kUnitSteps; ++s) {
        const int64_t r = r0 + s * kWave + lane;
        ev[s] = (r < R) ? idx[r] : -1;
    }

    region_offsets(expert_counts, E, lane, cursor);

    if (writer)
        write_region_tables(cursor, E, G, lane, expert_offsets, dest_counts, dest_offsets);
    if (u >= U)
        return;

    for (int e = lane; e < E; e += kWave)
        cursor[e] += unit_base[(int64_t)e * U + u];

#pragma unroll
    for (int s = 0; s < kUnitSteps; ++s) {
        const int64_t r = r0 + s * kWave + lane;
        const int e = ev[s];
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

// ---------------------------------------------------------------------------
// The same address resolution for callers that cannot hand over a workspace they allocated: the
// per-unit histograms live in a fixed array in the library's own device image.  Every GPU the
// library runs on holds one copy of the array (at its own address) until the process ends; all
// calls on a GPU share it, so calls that overlap there race.  Nothing in it has to start at zero:
// pass 1 writes every entry that passes 2 and 3 read.
// ---------------------------------------------------------------------------
constexpr size_t kLayoutScratchBytes = MOE_LAYOUT_STATIC_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[kLayoutScratchBytes];

// Device address of this GPU's copy of `scratch` (in host code the array's name is only a handle for
// the runtime, never an address a kernel may use).  Looked up once per device, with that device
// current; racing first calls all store the same value.
static int scratch_address(void **out)
{
    constexpr int kMaxDevices = 64;
    static std::atomic<void *> cached[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return fail(MOE_ERR_LAUNCH, "moe_dispatch_layout_static: no current device");
    void *p = cached[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr)
            return fail(MOE_ERR_LAUNCH, "moe_dispatch_layout_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        cached[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return MOE_OK;
}

int launch_layout_static(const int32_t *topk_idx, int64_t R, int E, int G, int32_t *expert_counts,
                         int32_t *expert_offsets, int32_t *dest_counts, int32_t *dest_offsets,
                         int32_t *slot_of_row, int32_t *row_of_slot, hipStream_t st)
{
    const size_t need = layout_workspace_bytes(R, E);
    if (need > kLayoutScratchBytes)
        return fail(MOE_ERR_UNSUPPORTED,
                    "moe_dispatch_layout_static: N*K=%lld rows over E=%d experts need %zu bytes of histograms, "
                    "the built-in array holds %zu; use moe_dispatch_layout with a workspace",
                    (long long)R, E, need, kLayoutScratchBytes);
    void *ws = nullptr;
    const int rc = scratch_address(&ws);
    if (rc != MOE_OK)
        return rc;
    return launch_layout(topk_idx, R, E, G, expert_counts, expert_offsets, dest_counts, dest_offsets,
                         slot_of_row, row_of_slot, ws, st);
}

// ---------------------------------------------------------------------------
// Arrival-order variant (Section IV-A3): every region has a row pointer that an
// arriving row reads and increments atomically, so rows are packed densely in
// whatever order they arrive.  Here the regions keep their scan-derived bases (the
// counts are the same whatever the order), a row "arrives" when its wavefront
// reaches its atomic, and the flat row number is the source information that
// Section IV-A4 carries with each row (row_of_slot).
//   pass 1  rank[r] = row pointer of expert idx[r] before the increment
//   pass 2  slot = offset[e] + rank; both maps written
// ---------------------------------------------------------------------------
constexpr int kArrivalThreads = 256;
constexpr int kArrivalRowsPerThread = 4;

__global__ void layout_clear_counts(int32_t *__restrict__ counts, int E)
{
    int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < E)
        counts[e] = 0;
}

__global__ __launch_bounds__(kArrivalThreads) void arrival_take_rank(
    const int32_t *__restrict__ idx, int64_t R, int E,
    int32_t *__restrict__ row_pointer, int32_t *__restrict__ rank)
{
    // Two levels of row pointers: the rows of a workgroup first draw from pointers in LDS, then
    // the workgroup draws one range per expert from the global pointer and rebases its rows.
    extern __shared__ int32_t group_pointer[]; // E
    for (int e = threadIdx.x; e < E; e += kArrivalThreads)
        group_pointer[e] = 0;
    __syncthreads();
    const int64_t r0 = (int64_t)blockIdx.x * (kArrivalThreads * kArrivalRowsPerThread);
    int expert[kArrivalRowsPerThread];
    int32_t local[kArrivalRowsPerThread];
#pragma unroll
    for (int j = 0; j < kArrivalRowsPerThread; ++j) {
        const int64_t r = r0 + j * kArrivalThreads + threadIdx.x;
        int e = (r < R) ? idx[r] : -1;
        expert[j] = (e >= 0 && e < E) ? e : -1;
        local[j] = (expert[j] >= 0) ? atomicAdd(&group_pointer[expert[j]], 1) : 0;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kArrivalThreads) {
        int32_t c = group_pointer[e];
        if (c > 0)
            group_pointer[e] = atomicAdd(&row_pointer[e], c);
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kArrivalRowsPerThread; ++j) {
        const int64_t r = r0 + j * kArrivalThreads + threadIdx.x;
        if (expert[j] >= 0)
            rank[r] = group_pointer[expert[j]] + local[j];
    }
}

__global__ __launch_bounds__(kArrivalThreads) void arrival_place_rows(
    const int32_t *__restrict__ idx, int64_t R, int E, int G,
    const int32_t *__restrict__ expert_counts, int32_t *__restrict__ expert_offsets,
    int32_t *__restrict__ dest_counts, int32_t *__restrict__ dest_offsets,
    int32_t *__restrict__ slot_of_row, int32_t *__restrict__ row_of_slot)
{
    extern __shared__ int32_t off[]; // E + 1
    if (threadIdx.x < kWave) {
        region_offsets(expert_counts, E, threadIdx.x, off);
        if (blockIdx.x == 0)
            write_region_tables(off, E, G, threadIdx.x, expert_offsets, dest_counts, dest_offsets);
    }
    __syncthreads();
    const int64_t r0 = (int64_t)blockIdx.x * (kArrivalThreads * kArrivalRowsPerThread);
#pragma unroll
    for (int j = 0; j < kArrivalRowsPerThread; ++j) {
        const int64_t r = r0 + j * kArrivalThreads + threadIdx.x;
        if (r >= R)
            continue;
        int e = idx[r];
        if (e < 0 || e >= E)
            continue;
        int32_t slot = off[e] + slot_of_row[r]; // slot_of_row holds the rank of pass 1
        slot_of_row[r] = slot;
        row_of_slot[slot] = (int32_t)r;
    }
}

int launch_layout_arrival(const int32_t *topk_idx, int64_t R, int E, int G, int32_t *expert_counts,
                          int32_t *expert_offsets, int32_t *dest_counts, int32_t *dest_offsets,
                          int32_t *slot_of_row, int32_t *row_of_slot, hipStream_t st)
{
    const int64_t per_block = kArrivalThreads * kArrivalRowsPerThread;
    const int blocks = (int)ceil_div(R, per_block);
    hipLaunchKernelGGL(layout_clear_counts, dim3((int)ceil_div(E, 256)), dim3(256), 0, st,
                       expert_counts, E);
    if (blocks > 0)
        hipLaunchKernelGGL(arrival_take_rank, dim3(blocks), dim3(kArrivalThreads),
                           E * sizeof(int32_t), st, topk_idx, R, E, expert_counts, slot_of_row);
    hipLaunchKernelGGL(arrival_place_rows, dim3(blocks > 0 ? blocks : 1), dim3(kArrivalThreads),
                       (E + 1) * sizeof(int32_t), st, topk_idx, R, E, G, expert_counts,
                       expert_offsets, dest_counts, dest_offsets, slot_of_row, row_of_slot);
    return check_launch("moe_dispatch_layout_arrival");
}

int launch_arrival_clear(int32_t *expert_counts, int E, hipStream_t st)
{
    hipLaunchKernelGGL(layout_clear_counts, dim3((int)ceil_div(E, 256)), dim3(256), 0, st, expert_counts, E);
    return check_launch("moe_route_resolve_arrival");
}

int launch_arrival_place(const int32_t *topk_idx, int64_t R, int E, int G, int32_t *expert_counts,
                         int32_t *expert_offsets, int32_t *dest_counts, int32_t *dest_offsets,
                         int32_t *slot_of_row, int32_t *row_of_slot, hipStream_t st)
{
    const int64_t per_block = kArrivalThreads * kArrivalRowsPerThread;
    const int blocks = (int)ceil_div(R, per_block);
    hipLaunchKernelGGL(arrival_place_rows, dim3(blocks > 0 ? blocks : 1), dim3(kArrivalThreads),
                       (E + 1) * sizeof(int32_t), st, topk_idx, R, E, G, expert_counts,
                       expert_offsets, dest_counts, dest_offsets, slot_of_row, row_of_slot);
    return check_launch("moe_route_resolve_arrival");
}

}  // namespace moe
