// bf16 matrix-core grouped GEMM for gfx950: C[m, n] = sum_k A[m, k] * B[e(m), n, k]
// over ragged row segments described by a device-side tile table.
//
// Both operands have k contiguous.  One workgroup = WM x WN wavefronts computes a
// BM x BN tile; every wavefront owns a (BM/WM) x (BN/WN) sub-tile as 32x32 blocks of
// v_mfma_f32_32x32x16_bf16.
//
// Pipeline (K tiles of BK = 64 elements; LDS is a ring of U units, a unit holding the A rows
// or the B rows of one K tile):
//   * global -> LDS goes through buffer_load_dwordx4 ... lds: no staging registers, no
//     ds_write.  A wavefront instruction fills 1 KiB of consecutive tile rows; the
//     16-byte chunk a lane fetches is chosen so that the LDS image is XOR swizzled
//     and the 16-byte operand reads are bank-conflict free.
//   * a K tile is BK/16 k-steps of 16 MFMAs (for a 128x128 wavefront tile).  The
//     operands of k-step ks+1 are read from LDS while the MFMAs of ks run.  Before
//     the last k-step of tile kt there is ONE barrier: by then every wavefront has
//     read all of tile kt, and tile kt+1 has landed (own loads: vmcnt, everyone's:
//     the barrier).  The barrier frees the two units of tile kt.
//   * loads are issued a few at a time under the MFMAs of every k-step, the B rows of
//     tile kt+U/2 into a unit just freed.  With an odd U (5 units of 32 KiB for the
//     256x256x64 tile: all 160 KiB) one unit is spare, so the A rows run one tile further
//     ahead than the B rows and the B loads can all go out right after the barrier: every
//     load then has two k-steps or more (about a microsecond) to land before the barrier
//     that waits for it, which is what a load from HBM needs here.
//   * The matrix-core operands are swapped (weights as the "A" operand), so a lane
//     ends up with 4 consecutive output columns of one row per accumulator
//     quadruple and stores them as one 8-byte vector.
//   * kSwiglu: the B tile holds BN/2 gate rows and the same BN/2 up rows, arranged
//     so that each wavefront has matching gate/up blocks; the epilogue writes
//     silu(g)*u, so g and u never reach memory.
//
// Scheduling: the grid is persistent, one workgroup per compute unit.  Workgroups draw tiles
// from per-XCD counters of the tile table (own XCD first), so the tiles an XCD holds at a
// time are neighbours in the table's order; while a workgroup multiplies the last K tiles of
// one output tile, its loads already fetch the first K tiles of its next one.  The table has
// two streams of tiles, served by two tile geometries inside the one kernel: 256x256 tiles, and
// 64x256 tiles four K tiles deep for experts with at most 64 rows, which do little arithmetic
// and live on how many bytes they keep in flight.  A 256-row tile can be "tall": the last full
// tile of an expert also computes a remainder of up to 64 rows, against the B tiles it has in LDS
// anyway, with the extra rows' operand and accumulators in vector registers (see GemmCfg).
#pragma once

#include <type_traits>

#include "common.h"

namespace moe {

struct TileEntry {
    int32_t expert; // local expert
    int32_t m0;     // first row of the tile
    int32_t m_end;  // end of the expert's segment (rows >= m_end are not written)
    int32_t n_tile; // column tile; bits 24..: rows beyond BM that this tile also computes (tall tile)
};
constexpr int kTileColBits = 24;

constexpr int kXcds = 8;
constexpr int kMaxGemmWorkgroups = 896; // workgroups of the persistent grid (ticket words of a table)

// Head of a tile table.  The table holds two streams of tiles, one after the other: stream 0 the
// tiles of experts with two row tiles or more (their weight tiles are shared by several
// workgroups and the matrix cores bound them), stream 1 the tiles of experts with one row tile
// (they stream their weights from memory once and mostly wait for them).
struct TileTableHeader {
    int32_t len[2];         // tiles in each stream; stream s starts at entry (s ? len[0] : 0)
    int32_t light_slots;    // of the 32 workgroup slots an XCD has, how many take stream 1 first
    int32_t done;           // workgroups that have left the kernel (the last one resets the counters)
    int32_t magic;          // kTableMagic once build_tile_table has filled the table ...
    int32_t rows;           // ... for this many rows
    int32_t error;          // kNoScheduleError / kDependencyTimeout, see below (cleared by the schedule)
    int32_t out_cols;       // output columns per tile the table was built for (a kernel of another geometry must not walk it)
    int32_t next[2][kXcds]; // per stream and XCD: tickets handed out so far
    // dependency-driven launches (both GEMMs in one kernel), kept in GEMM1's header:
    int32_t epoch;          // such launches completed over this schedule
    int32_t all_done;       // epoch + 1 once every GEMM1 tile of the running launch is stored
    int32_t pad2[6];
    int32_t ticket[kMaxGemmWorkgroups][8]; // per workgroup: tiles drawn by its first thread for all of it
};
constexpr size_t kTileTableHeaderBytes = 32768;
constexpr int32_t kTableMagic = 0x4D6F4554;
constexpr int32_t kNoScheduleError = 0x4E6F5363;   // a GEMM step found no tile table for its rows
constexpr int32_t kDependencyTimeout = 0x44657054; // a wait for rows of the first GEMM ran into its poll limit
constexpr int kReadyBit = 1 << 30;                 // in a drawn tile word: the tile's rows were complete when it was drawn
// How a producer tile makes its rows visible to consumers on other XCDs (whose L2 does not snoop this
// one's): 1 = device-scope stores, written through the L2 (the form that is used); 0 = ordinary stores
// and a device-scope release, i.e. a write-back of the whole L2, per wavefront and tile (measured: tens
// of microseconds each, the launch takes twice as long); 2 = ordinary stores and no write-back: NOT
// coherent, for timing experiments only.
#ifndef MOE_LIGHT_AUX
#define MOE_LIGHT_AUX 2 // cache policy of a shallow tile's weight loads: 2 = non-temporal
#endif
#ifndef MOE_DEP_STORE_THROUGH
#define MOE_DEP_STORE_THROUGH 1
#endif

// Ticket j of an XCD -> position in a stream: each XCD takes runs of `patch` consecutive tiles, so
// its L2 sees tiles that share weight and activation rows.
__device__ __forceinline__ int stream_position(int xcd, int j, int patch)
{
    return (j / patch) * (patch * kXcds) + xcd * patch + (j % patch);
}

// silu(g) * u with the hardware reciprocal (1 ulp): the result is rounded to bf16 right after
__device__ __forceinline__ float silu_mul(float g, float u)
{
    return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
}

// One accumulator out of the accumulation registers, at this point of the program and no earlier:
// left to itself the compiler copies a whole tile's accumulators into vector registers as soon as
// the K loop ends, and everything else that is live there has to make room.
__device__ __forceinline__ float acc_read(float a)
{
    float v;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
    return v;
}

// XOR key of a tile row with kChunks 16-byte chunks: equal logical chunks of any 8 and
// of any 16 consecutive rows land in different banks, whether the LDS serves 128 or 256
// bytes per clock.
template <int kChunks>
__device__ __forceinline__ int row_key(int r)
{
    if (kChunks == 8) // 128-byte rows
        return ((r ^ (r >> 3)) & 1) | (r & 6);
    return (((r >> 1) ^ (r >> 3)) & 1) | ((r >> 1) & 2); // 64-byte rows
}

// s_waitcnt with only vmcnt set (gfx9 encoding: vmcnt = [15:14][3:0], expcnt [6:4], lgkmcnt [11:8])
#define MOE_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
// s_waitcnt lgkmcnt(0) only
#define MOE_WAIT_LGKM0() __builtin_amdgcn_s_waitcnt(0xC07F)

// Workgroup barrier without the memory fence of __syncthreads (a fence would drain the
// outstanding global->LDS loads of the tiles still in flight).  The empty asm statements keep
// the compiler from moving LDS accesses across it.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Scheduling hint for one k-step: start with an MFMA, then alternate the kReads LDS reads
// (and, after the barrier, the kLoads global->LDS loads) with MFMAs so that they all issue
// early under the matrix pipe, and finish with the remaining MFMAs.
template <int kMfma, int kReads, int kLoads>
__device__ __forceinline__ void interleave_under_mfma()
{
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); // MFMA
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0); // VMEM read
    }
#pragma unroll
    for (int i = 0; i < kReads; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); // DS read
    }
    constexpr int kRest = kMfma - kReads - kLoads;
    if constexpr (kRest > 0)
        __builtin_amdgcn_sched_group_barrier(0x008, kRest, 0);
}

// Loads of position p of a window, from a hexadecimal digit string (most significant digit =
// position 0).
constexpr int part_loads(int dist, int parts, int p) { return (dist >> (4 * (parts - 1 - p))) & 15; }
constexpr int part_first(int dist, int parts, int p)
{
    int s = 0;
    for (int i = 0; i < p; ++i)
        s += part_loads(dist, parts, i);
    return s;
}
// Loads of a window that are issued after the last load the next barrier has to wait for.  Inside a
// position the loads of the "near" operand (the one the next barrier needs) go first, then those of
// the "far" operand; `far_needed` says whether the far loads of the window belong to the same K tile
// as its near loads (else they belong to a later one and nobody waits yet).
constexpr int window_tail(int dist_far, int dist_near, int parts, bool far_needed)
{
    int after = 0;
    for (int p = parts - 1; p >= 0; --p) {
        if (far_needed && part_loads(dist_far, parts, p) > 0)
            return after;
        after += part_loads(dist_far, parts, p);
        if (part_loads(dist_near, parts, p) > 0)
            return after;
    }
    return after;
}

// One tile geometry: BM x BN output tile, WM x WN wavefronts, K tiles of kBK, LDS ring of kUnits
// units, kDistA / kDistB the load schedule (see the kernel), kKind the tile stream it serves.
// kExtra_ > 0 ("tall"): a tile may carry up to kExtra_ rows beyond its BM, the short remainder of
// an expert's segment.  Those rows do not pass through LDS: every wavefront keeps one more 32-row
// block of accumulators and fetches that block's operand straight into registers.
// kFarB_ (odd rings only): which operand uses the spare unit to run one K tile further ahead: the A
// rows (false) or the B rows, i.e. the weights (true).  The operand that runs ahead has two K tiles
// and more to land, the other one about one: the one that runs ahead should be the one that comes
// from furthest away.
template <int BM_, int BN_, int WM_, int WN_, bool kSwiglu, int kBK_, int kUnits_, int kDistA_, int kDistB_, int kKind_,
          int kExtra_ = 0, bool kFarB_ = false>
struct GemmCfg {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, kBK = kBK_, kUnits = kUnits_;
    static constexpr int kDistA = kDistA_, kDistB = kDistB_, kKind = kKind_, kExtra = kExtra_;
    static constexpr bool kTall = kExtra_ > 0;
    static constexpr bool kFarB = kFarB_;
    static_assert(!kFarB_ || (kUnits_ % 2 == 1 && BM_ == BN_), "only an odd ring has a unit to spare");
    static_assert(kExtra_ == 0 || (kExtra_ == 32 * WM_ && WM_ == 2 && (BN_ / WN_ / 32) % 2 == 0),
                  "one extra 32-row block per wavefront row, two wavefront rows that can share one block");
    static constexpr int kWaves = WM * WN;
    static constexpr int kThreads = kWaves * kWave;
    static constexpr int kWaveM = BM / WM;    // rows per wavefront
    static constexpr int kWaveN = BN / WN;    // LDS B rows per wavefront
    static constexpr int kBlkM = kWaveM / 32; // 32x32 blocks per wavefront
    static constexpr int kBlkN = kWaveN / 32;
    static constexpr int kRowBytes = kBK * 2;
    static constexpr int kChunks = kRowBytes / 16;       // 16-byte chunks per tile row
    static constexpr int kGroupRows = 1024 / kRowBytes;  // rows one wavefront load instruction fills
    static constexpr int kAGroups = BM / kGroupRows / kWaves;
    static constexpr int kBGroups = BN / kGroupRows / kWaves;
    static constexpr int kLoadsPerTile = kAGroups + kBGroups; // per lane, per K tile
    static constexpr int kKSteps = kBK / 16;
    static constexpr int kOutCols = kSwiglu ? BN / 2 : BN;
    // LDS is a ring of kUnits units; a unit holds the A rows or the B rows of one K tile.  With
    // BM == BN all units have one size and the ring may be odd; otherwise the units come in
    // (A, B) pairs and the ring is even.
    static constexpr int kABytes = BM * kRowBytes, kBBytes = BN * kRowBytes;
    static constexpr int kDepth = kUnits / 2;  // K tiles whose B part fits besides the one in use
    static constexpr int kAhead = kUnits % 2;  // an odd ring lets one operand's loads run one tile further ahead
    static constexpr size_t kLdsBytes =
        BM == BN ? (size_t)kUnits * kABytes : (size_t)(kUnits / 2) * (kABytes + kBBytes);
    static constexpr int unit_base(int unit)
    {
        return BM == BN ? unit * kABytes : (unit >> 1) * (kABytes + kBBytes) + (unit & 1) * kABytes;
    }
    static_assert(kBK == 32 || kBK == 64, "K tile");
    static_assert(kUnits >= 4 && (BM == BN || kUnits % 2 == 0), "ring");
    static_assert(kWaveM % 32 == 0 && kWaveN % 32 == 0, "wave tile must be 32x32 blocks");
    static_assert(BM % (kGroupRows * kWaves) == 0 && BN % (kGroupRows * kWaves) == 0, "load groups");
    static_assert(!kSwiglu || kBlkN % 2 == 0, "gate and up halves");
    static_assert(kLoadsPerTile * (kDepth + kAhead) <= 63, "vmcnt budget");
};

// What one GEMM needs.  The last five members drive the dependency-driven form, in which both GEMMs of
// the expert computation run in one launch and a tile of the second starts as soon as the rows it reads
// have been stored by the first (the role the paper gives its data availability manager, Section IV-C:
// a table of what each group of thread blocks depends on, counters of what has arrived, and a ready
// signal to the scheduler - here a counter per row tile in global memory, bumped by the producing
// wavefronts and polled by the consuming workgroup's first thread).
struct GemmArgs {
    const uint16_t *A;
    int64_t M;
    int Kdim, Ndim;
    const uint16_t *B0, *B1;
    uint16_t *C;
    TileTableHeader *hdr;
    const TileEntry *table;
    int patch;
    const int32_t *gather_rows;
    int gather_div;
    uint32_t gather_bytes;
    const float *scatter_w;
    int32_t *ready;            // [M], indexed by a row tile's first row: wavefronts that have stored their part of it
    TileTableHeader *hdr_dep;  // the producing GEMM's header (epoch, all_done)
    int32_t ready_per_launch;  // what a row tile's counter gains per launch: wavefronts x column tiles of the producer
    int64_t wait_limit;        // polls a consumer spends on one row tile before it gives up
};

// Persistent grouped GEMM, as a function: a kernel runs one of them, or (the dependency-driven expert
// computation) the two GEMMs one after the other.  Main: the geometry of stream 0 (and of everything when there is no
// second geometry); Light: the geometry of stream 1, tiles of experts with at most Light::BM rows,
// or `void`.  Both geometries have the same workgroup size, BN and K tile.
// kGather: row m of the A operand is row gather_rows[m] / gather_div of `A` (the dispatch's row
// move done by the operand loads themselves) instead of row m.
// kScatter: the result is not stored as row m of C.  `C` is an fp32 matrix of Ndim columns, and row
// m of the result, times scatter_w[gather_rows[m]], is added (atomically) to its row
// gather_rows[m] / gather_div: the combine step done by the epilogue.
// kDep: 0 = plain; 1 = producer: results are stored through to memory and every wavefront bumps its
// row tile's counter once its stores are acknowledged; 2 = consumer: a tile whose rows were not
// complete when it was drawn is not prefetched, and its workgroup waits for the counter before loading.
#if defined(__HIP_DEVICE_COMPILE__) // the body uses device-only types (buffer resources); the host pass only needs the kernels' stubs
template <class Main, class Light, bool kSwiglu, bool kGather, bool kScatter, int kDep>
__device__ __forceinline__ void gemm_phase(const GemmArgs &g)
{
    const uint16_t *__restrict__ const A = g.A;
    const int64_t M = g.M;
    const int Kdim = g.Kdim, Ndim = g.Ndim;
    const uint16_t *__restrict__ const B0 = g.B0, *__restrict__ const B1 = g.B1;
    uint16_t *__restrict__ const C = g.C;
    TileTableHeader *__restrict__ const hdr = g.hdr;
    const TileEntry *__restrict__ const table = g.table;
    const int patch = g.patch;
    const int32_t *__restrict__ const gather_rows = g.gather_rows;
    const int gather_div = g.gather_div;
    const uint32_t gather_bytes = g.gather_bytes;
    const float *__restrict__ const scatter_w = g.scatter_w;
    static_assert(!(kGather && kScatter) && !(kScatter && kSwiglu), "kScatter belongs to the down projection");
    static_assert(kDep == 0 || (!kGather && !kScatter), "the dependency-driven form is built for the plain GEMMs");
    constexpr bool kTwo = !std::is_void<Light>::value;
    if constexpr (kTwo)
        static_assert(std::conditional_t<kTwo, Light, Main>::kBK == Main::kBK &&
                          std::conditional_t<kTwo, Light, Main>::BN == Main::BN &&
                          std::conditional_t<kTwo, Light, Main>::kThreads == Main::kThreads,
                      "the two geometries share K tile, BN and workgroup size");
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);

    // ---- tiles are handed out at run time.  The grid is persistent (one workgroup per
    //      workgroup slot of the chip); workgroup ids are dealt round-robin to the XCDs, and a
    //      workgroup takes tickets from its own XCD's counter of a stream, then from the others'.
    //      Of the 32 slots of an XCD, hdr->light_slots prefer the stream of memory-bound tiles, the
    //      rest the matrix-bound one, so both kinds run side by side from start to end.
    //      Thread 0 draws for the whole workgroup and passes the tile on through global memory
    //      (LDS is full and a register cannot cross wavefronts): {tile, sequence number}, stored
    //      and loaded as one 8-byte unit.  A reader that finds an older sequence number reads
    //      again, so nobody waits for the store to land and nobody acts on a stale tile.
    if (hdr->magic != kTableMagic || hdr->rows != (int32_t)M || hdr->out_cols != Main::kOutCols) {
        // no schedule for these rows in this workspace: nothing to go by.  The host is not waiting for
        // this kernel, so all it can do is leave a word that moe_ffn_status finds.
        if (blockIdx.x == 0 && threadIdx.x == 0)
            hdr->error = kNoScheduleError;
        return;
    }
    const int xcd = blockIdx.x % kXcds;
    int32_t *const my_ticket = hdr->ticket[blockIdx.x];
#ifdef MOE_TRACE_CLOCK
    // timing build only: shader-clock and 100 MHz stamps of the workgroup's life, left in its ticket words
    const uint64_t trace_c0 = __builtin_amdgcn_s_memtime(), trace_r0 = __builtin_amdgcn_s_memrealtime();
    uint32_t trace_ticks[4] = {0, 0, 0, 0}, trace_tiles[4] = {0, 0, 0, 0}; // full, tall, ragged, shallow
#endif
    const int len0 = hdr->len[0], len1 = hdr->len[1];
    const int slot = (blockIdx.x / kXcds) % 32, ls = hdr->light_slots;
    const bool light_first = ((slot + 1) * ls) / 32 > (slot * ls) / 32;
    auto fetch_tile = [&]() -> int { // thread 0 only
#pragma unroll 1
        for (int k = 0; k < 2; ++k) {
            const int s = light_first ? 1 - k : k;
            const int len = s ? len1 : len0;
#pragma unroll 1
            for (int i = 0; i < kXcds && len > 0; ++i) {
                const int x = (xcd + i) % kXcds;
                int32_t *ctr = &hdr->next[s][x];
                if (k + i > 0) { // (the first choice is taken without looking: it is rarely spent)
                    const int seen = __hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (stream_position(x, seen, patch) >= len)
                        continue; // positions grow with the ticket: this counter is spent
                }
                const int j = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const int p = stream_position(x, j, patch);
                if (p < len)
                    return (s ? len0 : 0) + p;
            }
        }
        return -1;
    };
    // a drawn tile travels as a word: -1 = none, else the table entry, plus (consumer) kReadyBit
    auto entry_of = [](int word) { return word & ~kReadyBit; };
    auto kind_of = [&](int word) { return kTwo && entry_of(word) >= len0 ? 1 : 0; };
    // consumer, thread 0 only: were the rows this tile reads complete at the time of the draw?
    const int32_t dep_epoch1 =
        kDep != 0 ? __hip_atomic_load(&(kDep == 1 ? hdr : g.hdr_dep)->epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1 : 0;
    const int64_t dep_target = (int64_t)dep_epoch1 * g.ready_per_launch;
    bool all_done_seen = false;
    auto rows_complete = [&](int m0) {
        return (int64_t)__hip_atomic_load(g.ready + m0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= dep_target;
    };
    auto with_ready_bit = [&](int tile) {
        if constexpr (kDep == 2) {
            if (tile < 0)
                return tile;
            if (!all_done_seen)
                all_done_seen = __hip_atomic_load(&g.hdr_dep->all_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == dep_epoch1;
            if (!all_done_seen && !rows_complete(table[tile].m0))
                return tile;
            return tile | kReadyBit;
        } else {
            return tile;
        }
    };
    // words 0, 1: the workgroup's first two tiles; words 2..5: two {tile, sequence number} pairs,
    // used in turn, so that a draw stays readable until the draw after the next one is published
    uint32_t seq = 0; // draws published so far
    auto slot_of = [&](uint32_t q) { return reinterpret_cast<uint64_t *>(my_ticket + 2 + 2 * (q & 1)); };
    auto publish = [&](int tile) { // thread 0 only
        __hip_atomic_store(slot_of(seq), ((uint64_t)seq << 32) | (uint32_t)tile, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    };
    auto read_slot = [&]() { return __hip_atomic_load(slot_of(seq), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };

    const int KT = Main::kBK > 0 ? Kdim / Main::kBK : 0;
    const int64_t b1_delta = kSwiglu ? B1 - B0 : 0;
    int cur_t, nxt_t;   // the tile being computed and the next one, as table entries (-1: none)
    int after_next = -1; // the tile after `nxt`, picked up from the ticket slot inside the K loop
    int drawn = -1;      // thread 0: the tile after that
    bool gave_up = false; // consumer: a wait ran into its poll limit

    // ---- everything that depends on the tile geometry.  One call works through the workgroup's
    //      tiles as long as they are of this geometry's kind.
    auto engine = [&](auto cfg_tag) {
    using Cfg = decltype(cfg_tag);
    constexpr int BM = Cfg::BM, WN = Cfg::WN, kBK = Cfg::kBK, kUnits = Cfg::kUnits;
    constexpr int kDistA = Cfg::kDistA, kDistB = Cfg::kDistB;
    constexpr int kChunks = Cfg::kChunks, kRowBytes = Cfg::kRowBytes, kKSteps = Cfg::kKSteps;
    constexpr int kDepth = Cfg::kDepth, kAhead = Cfg::kAhead;
    constexpr bool kTall = Cfg::kTall, kFarB = Cfg::kFarB;
    // loads of a window: how far ahead of the tile whose barrier opened it each operand is fetched
    constexpr int kAheadOfA = kDepth + (kFarB ? 0 : kAhead), kAheadOfB = kDepth + (kFarB ? kAhead : 0);
    const int wm = wave / WN, wn = wave % WN;

    // ---- global->LDS loads (buffer_load_dwordx4 ... lds): the lane at 16-byte position p of its
    //      row fetches chunk p ^ key(row).  Buffer addressing keeps the per-lane part of the address
    //      in one 32-bit register (row offset inside the tile, the same for every tile and the whole
    //      K loop); the tile base sits in the scalar resource and the K offset in a scalar register.
    // (kGather: the row part of the offset differs from tile to tile and is looked up, a_off holds
    // the chunk part; cur_row / nxt_row hold the row parts of `cur` and `nxt`)
    // B rows of one wavefront (kSwiglu): first half gate columns, second half the same up columns.
    // A load group never straddles the two halves, so its resource is wave-uniform.
    int a_off[Cfg::kAGroups], b_off[Cfg::kBGroups];
    int x_off = 0;                   // tall tiles: the lane's part of the extra rows' operand address
    int a_off0 = 0, b_off0 = 0;      // operand reads from LDS, see read_frags
    int ld_row = 0, fr_x = 0;        // the lane's row inside a load group / inside a 32-row block
    uint32_t cur_row[Cfg::kAGroups], nxt_row[Cfg::kAGroups];
#pragma unroll
    for (int g = 0; g < Cfg::kAGroups; ++g)
        cur_row[g] = nxt_row[g] = 0u;
    // The per-lane constants are worked out again for every output tile from a lane number the
    // optimiser cannot see through.  Computed once, they (and those of the other geometry) would
    // stay in registers of their own from the start of the kernel to its end, across epilogues
    // that need every register they can get.
    auto lane_setup = [&]() {
        int lane = tid % kWave;
        asm volatile("" : "+v"(lane));
        ld_row = lane / kChunks;
        const int ld_pc = lane % kChunks;
#pragma unroll
        for (int g = 0; g < Cfg::kAGroups; ++g) {
            const int r = (wave * Cfg::kAGroups + g) * Cfg::kGroupRows + ld_row;
            a_off[g] = ((kGather ? 0 : r * Kdim) + ((ld_pc ^ row_key<kChunks>(r)) * 8)) * 2;
        }
#pragma unroll
        for (int g = 0; g < Cfg::kBGroups; ++g) {
            const int r = (wave * Cfg::kBGroups + g) * Cfg::kGroupRows + ld_row;
            int col;
            if (kSwiglu) {
                const int w = r / Cfg::kWaveN, jj = r % Cfg::kWaveN, half = Cfg::kWaveN / 2;
                col = w * half + (jj % half);
            } else {
                col = r;
            }
            b_off[g] = (col * Kdim + ((ld_pc ^ row_key<kChunks>(r)) * 8)) * 2;
        }
        // operand reads: lane (i = lane%32, kg = lane/32) reads chunk (2*ks + kg) of row i of a block.
        // Block and wavefront offsets are multiples of 32 rows, so the key depends on i only, and
        // k-step ks is the k-step-0 offset with chunk bits flipped by 2*ks.
        const int fr = lane % 32, kg = lane / 32;
        const int key = row_key<kChunks>(fr);
        a_off0 = (wm * Cfg::kWaveM + fr) * kRowBytes + ((kg ^ key) << 4);
        b_off0 = (wn * Cfg::kWaveN + fr) * kRowBytes + ((kg ^ key) << 4);
        fr_x = fr;
        x_off = ((kGather ? 0 : (BM + wm * 32 + fr) * Kdim) + kg * 8) * 2;
    };
    // With kDepth + kAhead K tiles or more per output tile, the loads that would run past the
    // end of a tile's reduction fetch the first K tiles of the workgroup's next tile (if that is
    // of the same kind), so that tile starts with its operands in LDS.  (Shorter reductions
    // start every tile from scratch.)
    const bool warm = KT >= kDepth + kAhead;

    // What the loads of a tile need.  Rows past the end of the segment (and columns past Ndim) lie
    // beyond the byte counts: the bounds check returns zeros for them without touching memory; a
    // count of zero turns every load of a tile that does not exist into such a no-op, so the loop
    // issues the same number of loads in every iteration and the vmcnt arithmetic below holds
    // from the first K tile to the last.
    struct Operands {
        const uint16_t *a, *b; // b: the gate (or only) weight rows; the up rows lie b1_delta further
        uint32_t a_bytes, b_bytes;
        int32_t m0, m_end, n0;
        int32_t ext; // rows beyond BM (tall tiles)
    };
    auto operands_of = [&](int tile) {
        Operands o = {A, B0, 0u, 0u, 0, 0, 0, 0};
        if (tile >= 0) {
            const TileEntry te = table[entry_of(tile)];
            const int n0 = (te.n_tile & ((1 << kTileColBits) - 1)) * Cfg::kOutCols;
            o.ext = kTall ? te.n_tile >> kTileColBits : 0;
            const int64_t rows_left = (int64_t)te.m_end - te.m0; // >= 1
            const int cols_left = Ndim - n0;                      // >= 1
            if (kGather) { // any row of A may be needed; rows past the segment get an offset past the end
                o.a = A;
                o.a_bytes = gather_bytes;
            } else {
                o.a = A + (int64_t)te.m0 * Kdim;
                o.a_bytes = (uint32_t)((rows_left < BM ? rows_left : BM) * (int64_t)Kdim * 2);
            }
            o.b = B0 + ((int64_t)te.expert * Ndim + n0) * Kdim;
            o.b_bytes = (uint32_t)((cols_left < Cfg::kOutCols ? cols_left : Cfg::kOutCols) * (int64_t)Kdim * 2);
            o.m0 = te.m0;
            o.m_end = te.m_end;
            o.n0 = n0;
        }
        return o;
    };
    Operands cur, nxt; // the tile being computed; the one whose first K tiles are fetched behind it
    // kGather: the lane's rows of a tile -> their entries of gather_rows (rows past the segment: ~0) ...
    auto gather_lookup = [&](const Operands &o, uint32_t (&row)[Cfg::kAGroups]) {
#pragma unroll
        for (int g = 0; g < Cfg::kAGroups; ++g) {
            const int64_t m = (int64_t)o.m0 + (wave * Cfg::kAGroups + g) * Cfg::kGroupRows + ld_row;
            row[g] = m < o.m_end ? (uint32_t)gather_rows[m] : ~0u;
        }
    };
    // ... -> in place, byte offsets of those rows in A (rows past the segment: just past the last byte,
    // which the bounds check turns into zeros)
    auto gather_offsets = [&](uint32_t (&row)[Cfg::kAGroups]) {
#pragma unroll
        for (int g = 0; g < Cfg::kAGroups; ++g)
            row[g] = row[g] != ~0u ? row[g] / (uint32_t)gather_div * (uint32_t)(Kdim * 2) : gather_bytes;
    };
    // ---- tall tiles: the lane's operand of the extra 32-row block of its wavefront row.  Lane
    //      (i, kg) holds, for k-step ks, k = 16 ks + 8 kg .. + 8 of extra row 32 wm + i of the K tile
    //      being multiplied: xa[ks].  It comes straight from memory: right after k-step ks has used
    //      xa[ks], the load of the next K tile's xa[ks] goes out, one K tile ahead of its use.  The
    //      loads, the instructions that consume them and the waits in between (counted like those of
    //      the LDS loads) are written out by hand: the compiler would wait for the youngest load in
    //      flight at the top of every K tile.  It therefore does not know that xa[ks] is not valid
    //      until that wait, and must not copy these registers while a load is on its way.  It has no
    //      reason to inside the K loop of such a tile, which is one basic block; at the tile's start
    //      the operands of K tile 0 are loaded and waited for in one statement, and the loads behind
    //      the last K tile fetch nothing.
    constexpr int kXRegs = kTall ? kKSteps : 1;
    u32x4 xa[kXRegs];
#pragma unroll
    for (int ks = 0; ks < kXRegs; ++ks)
        xa[ks] = u32x4{0u, 0u, 0u, 0u};
    uint32_t cur_xrow = 0u; // kGather: row part of the offset, per tile
    // (kHalf: at most 32 extra rows, one block that both wavefront rows work on, see run_tile)
    auto gather_lookup_x = [&](const Operands &o, uint32_t &row, bool half) {
        const int64_t m = (int64_t)o.m0 + BM + (half ? 0 : wm * 32) + fr_x;
        row = m < o.m_end ? (uint32_t)gather_rows[m] : ~0u;
    };
    auto gather_offset_x = [&](uint32_t &row) {
        row = row != ~0u ? row / (uint32_t)gather_div * (uint32_t)(Kdim * 2) : gather_bytes;
    };
    using lds_ptr = __attribute__((address_space(3))) void *;
    auto x_resource = [&](bool real) {
        const uint64_t base = reinterpret_cast<uint64_t>(cur.a);
        const uint32_t bytes =
            real && cur.ext > 0 ? (kGather ? gather_bytes : (uint32_t)((BM + cur.ext) * Kdim * 2)) : 0u;
        return u32x4{(uint32_t)base, (uint32_t)(base >> 32) & 0xffffu, bytes, 0x00020000u};
    };
    auto x_voffset = [&](bool half) {
        return kGather ? (int)(cur_xrow + (uint32_t)x_off) : x_off - (half ? wm * 32 * Kdim * 2 : 0);
    };
    // xa[ks] <- K tile t of `cur`; past the last K tile a load of zero bytes, which keeps the number
    // of loads per K tile fixed and touches no memory
    auto load_x = [&](auto ks_tag, int t, bool half) {
        constexpr int ks = decltype(ks_tag)::value;
        const u32x4 rs = x_resource(t < KT);
        const int voff = x_voffset(half), soff = t * (kBK * 2) + ks * 32;
        u32x4 &dst = xa[ks < kXRegs ? ks : 0]; // (a generic lambda does not capture through an asm operand)
        asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen" : "+v"(dst) : "v"(voff), "s"(rs), "s"(soff));
    };
    // all of K tile 0, complete on return (this also waits for every older load of the wavefront)
    auto load_x_first = [&](bool half) {
        static_assert(!kTall || kXRegs == 4, "four k-steps per K tile");
        const u32x4 rs = x_resource(true);
        const int voff = x_voffset(half);
        u32x4 &d0 = xa[0], &d1 = xa[kXRegs > 1 ? 1 : 0], &d2 = xa[kXRegs > 2 ? 2 : 0], &d3 = xa[kXRegs > 3 ? 3 : 0];
        asm volatile("buffer_load_dwordx4 %0, %4, %5, 0 offen\n\t"
                     "buffer_load_dwordx4 %1, %4, %5, 0 offen offset:32\n\t"
                     "buffer_load_dwordx4 %2, %4, %5, 0 offen offset:64\n\t"
                     "buffer_load_dwordx4 %3, %4, %5, 0 offen offset:96\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(d0), "=&v"(d1), "=&v"(d2), "=&v"(d3)
                     : "v"(voff), "s"(rs));
    };
    // K tile t of `cur`; past its last K tile (kTail only): K tile t - KT of `nxt`
    auto load_a_group = [&](int t, int unit, int g, auto tail_tag) {
        constexpr bool kTail = decltype(tail_tag)::value;
        const bool here = !kTail || t < KT;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(here ? cur.a : nxt.a), 0, here ? cur.a_bytes : nxt.a_bytes, 0x00020000);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rs, (lds_ptr)(lds + Cfg::unit_base(unit) + (wave * Cfg::kAGroups + g) * 1024), 16,
            kGather ? (int)((here ? cur_row[g] : nxt_row[g]) + (uint32_t)a_off[g]) : a_off[g],
            (here ? t : t - KT) * (kBK * 2), 0, 0);
    };
    auto load_b_group = [&](int t, int unit, int g, auto tail_tag) {
        constexpr bool kTail = decltype(tail_tag)::value;
        const bool here = !kTail || t < KT;
        const int r0 = (wave * Cfg::kBGroups + g) * Cfg::kGroupRows; // uniform
        const bool up = kSwiglu && (r0 % Cfg::kWaveN) >= Cfg::kWaveN / 2;
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>((here ? cur.b : nxt.b) + (up ? b1_delta : 0)), 0,
            here ? cur.b_bytes : nxt.b_bytes, 0x00020000);
        // The weights of a light tile are read once by one workgroup: fetched with the non-temporal
        // hint (aux bit 1) they do not push the other tiles' shared operands out of the caches.
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rs, (lds_ptr)(lds + Cfg::unit_base(unit) + (wave * Cfg::kBGroups + g) * 1024), 16, b_off[g],
            (here ? t : t - KT) * (kBK * 2), 0, Cfg::kKind == 1 ? MOE_LIGHT_AUX : 0);
    };

    // ---- the ring.  K tile t keeps the rows of its "far" operand (the one whose loads run ahead in
    //      an odd ring: A, or B with kFarB) in unit (2t) % kUnits and those of the other in unit
    //      (2t+1) % kUnits, counting the K tiles of a workgroup's successive output tiles on (when
    //      `warm`).  `u` below is always the far operand's unit of the K tile being multiplied.
    auto wrap = [](int x) { return x >= kUnits ? x - kUnits : x; };
    auto unit_a = [&](int u, int ahead) { return wrap(u + (2 * ahead + (kFarB ? 1 : 0)) % kUnits); };
    auto unit_b = [&](int u, int ahead) { return wrap(u + (2 * ahead + (kFarB ? 0 : 1)) % kUnits); };

    // ---- load schedule.  The barrier that ends the reads of K tile t opens a "window": the units
    //      of tile t are free, and until the next barrier the loads of B(t + kAheadOfB) and of
    //      A(t + kAheadOfA) are issued, in kKSteps positions: position 0 under the last
    //      k-step of tile t, position p under k-step p-1 of tile t+1 (kDistB / kDistA say how many
    //      loads each position takes; inside a position the operand needed sooner goes first).
    //      Spreading them keeps the four wavefronts from pushing a whole tile into the memory
    //      pipeline in one burst; the loads of the operand the next barrier needs go early, which
    //      gives them two to three k-steps to land, and those of the operand that runs ahead in an
    //      odd ring, needed one tile later, fill the rest.
    static_assert(part_first(kDistA, kKSteps, kKSteps) == Cfg::kAGroups, "A loads of a window");
    static_assert(part_first(kDistB, kKSteps, kKSteps) == Cfg::kBGroups, "B loads of a window");
    auto issue_position = [&](int t, int u, auto pos_tag, auto tail_tag) { // window opened by the barrier of tile t
        constexpr int p = decltype(pos_tag)::value;
        if constexpr (!kFarB) {
#pragma unroll
            for (int g = part_first(kDistB, kKSteps, p); g < part_first(kDistB, kKSteps, p + 1); ++g)
                load_b_group(t + kAheadOfB, unit_b(u, kAheadOfB), g, tail_tag);
        }
#pragma unroll
        for (int g = part_first(kDistA, kKSteps, p); g < part_first(kDistA, kKSteps, p + 1); ++g)
            load_a_group(t + kAheadOfA, unit_a(u, kAheadOfA), g, tail_tag);
        if constexpr (kFarB) {
#pragma unroll
            for (int g = part_first(kDistB, kKSteps, p); g < part_first(kDistB, kKSteps, p + 1); ++g)
                load_b_group(t + kAheadOfB, unit_b(u, kAheadOfB), g, tail_tag);
        }
    };
    auto loads_at = [](int p) { return part_loads(kDistA, kKSteps, p) + part_loads(kDistB, kKSteps, p); };
    // loads that may still be in flight when a barrier needs the next tile complete
    constexpr int kInFlight = (kDepth - 2) * Cfg::kLoadsPerTile +
                              (kFarB ? window_tail(kDistB, kDistA, kKSteps, false) : window_tail(kDistA, kDistB, kKSteps, kAhead == 0));
    using tail_yes = std::integral_constant<bool, true>;
    using tail_no = std::integral_constant<bool, false>;

    bf16x8 fa[2][Cfg::kBlkM], fb[2][Cfg::kBlkN];
    // `act` = number of this wavefront's 32-row blocks that hold rows of the segment: blocks past
    // the end of a ragged segment are neither read nor multiplied.
    auto read_frags = [&](int u, int ks, int slot, auto act_tag) { // u = far operand's unit of the tile
        constexpr int kAct = decltype(act_tag)::value;
        const unsigned char *pa = lds + Cfg::unit_base(unit_a(u, 0)) + (a_off0 ^ (ks << 5));
        const unsigned char *pb = lds + Cfg::unit_base(unit_b(u, 0)) + (b_off0 ^ (ks << 5));
#pragma unroll
        for (int i = 0; i < kAct; ++i)
            fa[slot][i] = *reinterpret_cast<const bf16x8 *>(pa + i * 32 * kRowBytes);
        if constexpr (kAct > 0) {
#pragma unroll
            for (int j = 0; j < Cfg::kBlkN; ++j)
                fb[slot][j] = *reinterpret_cast<const bf16x8 *>(pb + j * 32 * kRowBytes);
        }
    };

    f32x16 acc[Cfg::kBlkM][Cfg::kBlkN];
    auto mfma_all = [&](int slot, auto act_tag) {
        constexpr int kAct = decltype(act_tag)::value;
#pragma unroll
        for (int i = 0; i < kAct; ++i)
#pragma unroll
            for (int j = 0; j < Cfg::kBlkN; ++j) // weights first: the result block is [n][m]
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[slot][j], fa[slot][i], acc[i][j], 0, 0, 0);
    };

    // Tall tiles: the extra block row of this wavefront.  The 256 accumulators above fill the
    // accumulation registers, so these live in ordinary vector registers and are multiplied by
    // instructions written out by hand (the two leading wait states cover a vector-ALU write of an
    // operand just before).
    f32x16 accx[kTall ? Cfg::kBlkN : 1];
    // loads issued between the load of xa[ks] and its use one K tile later: a K tile's worth but itself
    constexpr int kXWait = Cfg::kLoadsPerTile + kXRegs - 1;
    auto mfma_x = [&](int slot, auto ks_tag, int next_t, auto half_tag) {
        constexpr int ks = decltype(ks_tag)::value;
        constexpr bool kHalf = decltype(half_tag)::value;
        MOE_WAIT_VMCNT(kXWait);
        const u32x4 &x = xa[ks < kXRegs ? ks : 0];
        if constexpr (kHalf) {
            static_assert(!kSwiglu || Cfg::kBlkN % 4 == 0, "a gate block and its up block per wavefront row");
            // one extra block row for the whole workgroup: wavefront row wm takes column blocks
            // wm, wm + 2, ... of its wavefront column (for SwiGLU a gate block and its up block)
#pragma unroll
            for (int jj = 0; jj < Cfg::kBlkN / 2; ++jj) {
                f32x16 &c = accx[jj];
                const bf16x8 w = wm ? fb[slot][2 * jj + 1] : fb[slot][2 * jj];
                asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(w), "v"(x));
            }
        } else {
#pragma unroll
            for (int j = 0; j < Cfg::kBlkN; ++j) {
                f32x16 &c = accx[j];
                const bf16x8 &w = fb[slot][j];
                asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(w), "v"(x));
            }
        }
        load_x(ks_tag, next_t, kHalf);
    };

    int u = 0; // ring position: A unit of the K tile to multiply next

    // One output tile: K loop, then the epilogue.  On entry K tile 0 of `cur` is in LDS (everyone's
    // loads, behind a barrier) and the windows before it have issued what they should.
    auto run_tile = [&](auto act, auto ext_tag) {
        constexpr int kAct = decltype(act)::value;
        // 0: no extra rows; 1: up to 32, one block row shared by the two wavefront rows (each takes
        // half of its column blocks: 1/8 more MFMAs); 2: up to 64, a block row per wavefront row (1/4 more)
        constexpr int kExtMode = decltype(ext_tag)::value;
        constexpr bool kExt = kExtMode > 0, kHalf = kExtMode == 1;
        using half_tag = std::integral_constant<bool, kHalf>;
        constexpr int kMfma = kAct * Cfg::kBlkN, kReads = kAct ? kAct + Cfg::kBlkN : 0;
        if constexpr (kExt) {
#pragma unroll
            for (int j = 0; j < Cfg::kBlkN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    accx[j][r] = 0.0f;
            if constexpr (kGather) { // the extra rows of this tile: looked up here, a round trip per tall tile
                gather_lookup_x(cur, cur_xrow, kHalf);
                gather_offset_x(cur_xrow);
            }
            load_x_first(kHalf);
        }
#pragma unroll
        for (int i = 0; i < Cfg::kBlkM; ++i)
#pragma unroll
            for (int j = 0; j < Cfg::kBlkN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc[i][j][r] = 0.0f;
        read_frags(u, 0, 0, act);

        // k-step ks of K tile kt (not its last): position ks+1 of the window goes out, the operands
        // of k-step ks+1 are read, all under this step's MFMAs
        auto kstep = [&](int kt, auto ks_tag, auto tail_tag) {
            constexpr int ks = decltype(ks_tag)::value;
            issue_position(kt - 1, wrap(u + kUnits - 2), std::integral_constant<int, ks + 1>{}, tail_tag);
            read_frags(u, ks + 1, (ks + 1) & 1, act);
            mfma_all(ks & 1, act);
            if constexpr (kExt)
                mfma_x(ks & 1, ks_tag, kt + 1, half_tag{});
            interleave_under_mfma<kMfma, kReads, loads_at(ks + 1)>();
        };
        // The body is branch free (a branch around the LDS reads would make the compiler wait for
        // them before MFMAs that do not need them).
        auto ktile = [&](int kt, auto tail_tag) {
            kstep(kt, std::integral_constant<int, 0>{}, tail_tag);
            if constexpr (kKSteps > 2) {
                kstep(kt, std::integral_constant<int, 1>{}, tail_tag);
                kstep(kt, std::integral_constant<int, 2>{}, tail_tag);
            }
            __builtin_amdgcn_sched_barrier(0); // keep this k-step's MFMAs above the waits
            MOE_WAIT_LGKM0();                  // my reads of tile kt are complete
            MOE_WAIT_VMCNT(kInFlight + (kExt ? kXRegs - 1 : 0)); // my part of tile kt+1 has landed
            lds_barrier();                     // ... and everyone's; the units of tile kt are free
            issue_position(kt, u, std::integral_constant<int, 0>{}, tail_tag);
            read_frags(wrap(u + 2), 0, 0, act); // past the last K tile: the next output tile's, read again there
            mfma_all((kKSteps - 1) & 1, act);
            if constexpr (kExt)
                mfma_x((kKSteps - 1) & 1, std::integral_constant<int, kKSteps - 1>{}, kt + 1, half_tag{});
            interleave_under_mfma<kMfma, kReads, loads_at(0)>();
            u = wrap(u + 2);
        };
        // the last kDepth + kAhead K tiles look past the end of this tile's reduction
        uint64_t slot_v = 0; // (sequence number 0: never a published one)
        if constexpr (kExt) {
            // one loop and nothing else between its K tiles, see xa; the next tile is looked up below
            if constexpr (kGather)
                gather_offsets(nxt_row);
            for (int kt = 0; kt < KT; ++kt)
                ktile(kt, tail_yes{});
            // the (empty) loads behind the last K tile still write xa: they must have done so before
            // the compiler, for which these registers are free from here on, puts anything else there
            {
                u32x4 &d0 = xa[0], &d1 = xa[kXRegs > 1 ? 1 : 0], &d2 = xa[kXRegs > 2 ? 2 : 0], &d3 = xa[kXRegs > 3 ? 3 : 0];
                asm volatile("s_waitcnt vmcnt(0)" : "+v"(d0), "+v"(d1), "+v"(d2), "+v"(d3));
            }
        } else {
            const int k_split = KT - (kDepth + kAhead);
            if (k_split > 0)
                ktile(0, tail_no{});
            else
                ktile(0, tail_yes{});
            // The tile after `nxt`: thread 0 stored it before it reached the barrier of K tile 0.  The
            // load is left in flight and looked at after the K loop.
            slot_v = read_slot();
            if constexpr (kGather)
                gather_offsets(nxt_row); // looked up before K tile 0, long landed; needed from k_split on
            for (int kt = 1; kt < k_split; ++kt)
                ktile(kt, tail_no{});
            for (int kt = (k_split > 1 ? k_split : 1); kt < KT; ++kt)
                ktile(kt, tail_yes{});
        }
        // (if the store had not landed when the load ran, the sequence number is an older one)
        while ((uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(slot_v >> 32)) != seq)
            slot_v = read_slot();
        after_next = (int)__builtin_amdgcn_readfirstlane((uint32_t)slot_v);
        // Thread 0 draws the tile that will follow `after_next` now, so that the counter's round trip
        // runs under the epilogue; the tile is published after it.
        drawn = -1;
        if (tid == 0 && after_next >= 0)
            drawn = with_ready_bit(fetch_tile());

        // ---- epilogue.  Block (i, j), register r of lane l:
        //      output row    m = i*32 + l%32               (within the wavefront's rows)
        //      output column n = j*32 + 8*(r/4) + 4*(l/32) + r%4
        // (acc_read is opaque to the compiler's hazard handling: the matrix pipe's last result may be
        // read 18 wait states after its instruction at the earliest)
        asm volatile("s_nop 15\n\ts_nop 3");
        int m_lane = lane % 32, n_lane = (lane / 32) * 4;
        // opaque to the optimiser: otherwise every column offset derived from them is kept in a
        // register of its own across the whole persistent loop
        asm volatile("" : "+v"(m_lane), "+v"(n_lane));
        constexpr int kOutBlkN = kSwiglu ? Cfg::kBlkN / 2 : Cfg::kBlkN;
        // where row m of the result goes: row m of C, or (kScatter) its token's row of the fp32 sums
        struct RowDst {
            uint16_t *crow;
            float *sums;
            float w;
        };
        auto row_dst = [&](int64_t m) {
            RowDst d = {nullptr, nullptr, 0.0f};
            if constexpr (kScatter) {
                const int32_t r = gather_rows[m];
                d.w = scatter_w[r];
                d.sums = reinterpret_cast<float *>(C) + (int64_t)(r / gather_div) * Ndim;
            } else {
                d.crow = C + m * Ndim;
            }
            return d;
        };
        auto put4 = [&](const RowDst &d, int col, const float (&v)[4]) {
            if constexpr (kScatter) {
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    unsafeAtomicAdd(d.sums + col + t, d.w * v[t]);
            } else if constexpr (kDep == 1 && MOE_DEP_STORE_THROUGH == 1) {
                // device-scope store: written through this XCD's L2, which the other XCDs do not snoop
                const uint64_t o = (uint64_t)pack_bf16x2(v[0], v[1]) | ((uint64_t)pack_bf16x2(v[2], v[3]) << 32);
                __hip_atomic_store(reinterpret_cast<uint64_t *>(d.crow + col), o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                u32x2 o;
                o[0] = pack_bf16x2(v[0], v[1]);
                o[1] = pack_bf16x2(v[2], v[3]);
                *reinterpret_cast<u32x2 *>(d.crow + col) = o;
            }
        };
        // one 32-row block row of accumulators -> row m of the result
        auto store_row = [&](int64_t m, const auto &blk, auto in_acc_regs) {
            constexpr bool kAccRegs = decltype(in_acc_regs)::value;
            if (m >= cur.m_end)
                return;
            const RowDst dst = row_dst(m);
#pragma unroll
            for (int j = 0; j < kOutBlkN; ++j) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = cur.n0 + wn * (kOutBlkN * 32) + j * 32 + q * 8 + n_lane;
                    if (col >= Ndim)
                        continue;
                    float v[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const int r = q * 4 + t;
                        if constexpr (kSwiglu)
                            v[t] = kAccRegs ? silu_mul(acc_read(blk[j][r]), acc_read(blk[j + kOutBlkN][r]))
                                            : silu_mul(blk[j][r], blk[j + kOutBlkN][r]);
                        else
                            v[t] = kAccRegs ? acc_read(blk[j][r]) : blk[j][r];
                    }
                    put4(dst, col, v);
                }
                // one block at a time: left alone, the scheduler first copies the whole tile out of the
                // accumulation registers and needs some two hundred registers to hold it
                __builtin_amdgcn_sched_barrier(0);
            }
        };
#pragma unroll
        for (int i = 0; i < kAct; ++i)
            store_row((int64_t)cur.m0 + wm * Cfg::kWaveM + i * 32 + m_lane, acc[i], std::true_type{});
        if constexpr (kExt) {
            // the hand-written instructions are opaque to the compiler's hazard handling: a result of
            // the matrix pipe may be read by the vector ALU 18 wait states after the instruction at
            // the earliest; the last one was issued before the block rows above were stored
            asm volatile("s_nop 15\n\ts_nop 3" : "+v"(accx[0]), "+v"(accx[1]), "+v"(accx[Cfg::kBlkN - 2]), "+v"(accx[Cfg::kBlkN - 1]));
            if constexpr (!kHalf) {
                store_row((int64_t)cur.m0 + BM + wm * 32 + m_lane, accx, std::false_type{});
            } else {
                // accx[jj] is column block wm + 2 jj of this wavefront column
                const int64_t m = (int64_t)cur.m0 + BM + m_lane;
                if (m < cur.m_end) {
                    const RowDst dst = row_dst(m);
#pragma unroll
                    for (int jo = 0; jo < (kSwiglu ? 1 : Cfg::kBlkN / 2); ++jo) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int col = cur.n0 + wn * (kOutBlkN * 32) + (wm + 2 * jo) * 32 + q * 8 + n_lane;
                            if (col >= Ndim)
                                continue;
                            float v[4];
#pragma unroll
                            for (int t = 0; t < 4; ++t)
                                v[t] = kSwiglu ? silu_mul(accx[0][q * 4 + t], accx[1][q * 4 + t]) : accx[jo][q * 4 + t];
                            put4(dst, col, v);
                        }
                    }
                }
            }
        }
        if constexpr (kDep == 1 && MOE_DEP_STORE_THROUGH != 0) {
            // this wavefront's part of the row tile is in memory once its stores are acknowledged
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (lane == 0)
                __hip_atomic_fetch_add(g.ready + cur.m0, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else if constexpr (kDep == 1) {
            // The stores went into this XCD's L2, which the other XCDs do not snoop: a device-scope release
            // (wait for the stores, write the L2's dirty lines back) before the counter is bumped.
            __hip_atomic_fetch_add(g.ready + cur.m0, lane == 0 ? 1 : 0, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
    };

    bool primed = false; // K tile 0 of `cur` is in LDS already
    while (cur_t >= 0 && kind_of(cur_t) == Cfg::kKind) {
        lane_setup();
        // the next tile's first K tiles ride behind this one's last
        const bool chain = warm && nxt_t >= 0 && kind_of(nxt_t) == Cfg::kKind && (kDep != 2 || (nxt_t & kReadyBit));
        nxt = operands_of(chain ? nxt_t : -1);
        if constexpr (kGather)
            gather_lookup(nxt, nxt_row);
        if (!primed) {
            cur = operands_of(cur_t);
            if constexpr (kDep == 2) {
                // The rows were not complete when this tile was drawn: wait for them now.  Nothing of the
                // workgroup is in flight here and LDS is idle, so the first thread polls and tells the
                // others through LDS.  Every producer tile has been drawn by a workgroup that waits for
                // nothing, so the wait ends; the poll limit only guards against a broken schedule.
                if (!(cur_t & kReadyBit)) {
                    volatile int32_t *const outcome = reinterpret_cast<volatile int32_t *>(lds);
                    if (tid == 0) {
                        int64_t polls = 0;
                        bool ok = rows_complete(cur.m0);
                        while (!ok && polls++ < g.wait_limit) {
                            __builtin_amdgcn_s_sleep(32);
                            ok = rows_complete(cur.m0);
                        }
                        if (!ok)
                            __hip_atomic_store(&hdr->error, kDependencyTimeout, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        *outcome = ok ? 1 : 0;
                    }
                    __syncthreads();
                    const bool ok = __builtin_amdgcn_readfirstlane(*outcome) != 0;
                    __syncthreads();
                    if (!ok) { // give up: this workgroup's tiles stay undone, the error word says so
                        cur_t = nxt_t = -1;
                        gave_up = true;
                        break;
                    }
                }
            }
            if constexpr (kGather) {
                gather_lookup(cur, cur_row);
                gather_offsets(cur_row);
            }

            // everything the windows before K tile 0 would have issued, then position 0 of the
            // window before it; K tile 0 landed
            u = 0;
#pragma unroll
            for (int t = 0; t + 1 < kDepth + kAhead; ++t) {
                const bool both = t + 1 < kDepth; // else only the operand that runs ahead
                if (both || !kFarB) {
#pragma unroll
                    for (int g = 0; g < Cfg::kAGroups; ++g)
                        load_a_group(t, unit_a((2 * t) % kUnits, 0), g, tail_yes{});
                }
                if (both || kFarB) {
#pragma unroll
                    for (int g = 0; g < Cfg::kBGroups; ++g)
                        load_b_group(t, unit_b((2 * t) % kUnits, 0), g, tail_yes{});
                }
            }
            issue_position(-1, kUnits - 2, std::integral_constant<int, 0>{}, tail_yes{});
            // in flight after K tile 0: tiles 1 .. kDepth-2, the rows that run ahead, position 0
            MOE_WAIT_VMCNT((kDepth - 2) * Cfg::kLoadsPerTile + kAhead * (kFarB ? Cfg::kBGroups : Cfg::kAGroups) + loads_at(0));
            lds_barrier();
        }
        // rows of the segment inside this wavefront's part of the tile -> active 32-row blocks
        const int64_t rows = (int64_t)cur.m_end - ((int64_t)cur.m0 + wm * Cfg::kWaveM);
        const int active = rows <= 0 ? 0 : (rows >= Cfg::kWaveM ? Cfg::kBlkM : (int)((rows + 31) / 32));
#ifdef MOE_TRACE_CLOCK
        const uint64_t trace_t0 = __builtin_amdgcn_s_memrealtime();
        const int trace_kind = Cfg::kKind == 1 ? 3 : (cur.ext > 0 ? 1 : (cur.m_end - cur.m0 >= Cfg::BM ? 0 : 2));
#endif
        using ext_no = std::integral_constant<int, 0>;
        using ext_half = std::integral_constant<int, kTall ? 1 : 0>;
        using ext_full = std::integral_constant<int, kTall ? 2 : 0>;
        if (active == Cfg::kBlkM) {
            if (kTall && cur.ext > 32)
                run_tile(std::integral_constant<int, Cfg::kBlkM>{}, ext_full{});
            else if (kTall && cur.ext > 0)
                run_tile(std::integral_constant<int, Cfg::kBlkM>{}, ext_half{});
            else
                run_tile(std::integral_constant<int, Cfg::kBlkM>{}, ext_no{});
        } else if (active == 0)
            run_tile(std::integral_constant<int, 0>{}, ext_no{});
        else if (active == 1)
            run_tile(std::integral_constant<int, 1>{}, ext_no{});
        else if (Cfg::kBlkM > 2 && active == 2)
            run_tile(std::integral_constant<int, (Cfg::kBlkM > 2 ? 2 : 1)>{}, ext_no{});
        else
            run_tile(std::integral_constant<int, (Cfg::kBlkM > 3 ? 3 : 1)>{}, ext_no{});

#ifdef MOE_TRACE_CLOCK
        trace_ticks[trace_kind] += (uint32_t)(__builtin_amdgcn_s_memrealtime() - trace_t0);
        trace_tiles[trace_kind] += 1;
#endif
        // Thread 0 leaves the tile it drew before the epilogue in the other slot under the next
        // sequence number; the others look there after the next tile's first barrier.
        ++seq;
        if (tid == 0)
            publish(drawn);
        cur_t = nxt_t;
        nxt_t = after_next;
        if (chain) {
            cur = nxt; // its first K tiles are in LDS or on their way
            if constexpr (kGather) {
#pragma unroll
                for (int g = 0; g < Cfg::kAGroups; ++g)
                    cur_row[g] = nxt_row[g];
            }
            primed = true;
        } else {
            primed = false;
            MOE_WAIT_VMCNT(0); // the no-op loads past the last K tile still write LDS: let them finish
            lds_barrier();     // before anyone refills those units, in this layout or the other
        }
    }
    }; // engine

    // ---- the workgroup's first three tiles.  The words still hold what an earlier launch left
    //      there, so these stores have to be in memory before anyone looks.
    //      A launch with about one tile per workgroup draws one tile at a time instead: the first
    //      workgroups to start would otherwise take three tiles each and leave others without.  So
    //      does a consumer phase with only a few tiles per workgroup, whose workgroups arrive one
    //      by one as they run out of producer tiles.  Such a tile starts cold (no operands fetched
    //      behind its predecessor), which long or few tiles can afford.
    const int n_tiles_all = len0 + len1, n_groups = (int)gridDim.x;
    // Drawing ahead also means that the last tiles of a launch are held by workgroups that are still busy
    // while others have run out: with only a few tiles per workgroup, and tiles long enough that a cold
    // start is a small part of them, one at a time is the better deal as well (512 tiles of 224 K tiles on
    // 256 workgroups: some took three and some one).
#ifndef MOE_LEAN_ROUNDS
#define MOE_LEAN_ROUNDS 8  // fewer tiles than this per workgroup ...
#define MOE_LEAN_KTILES 64 // ... each at least this many K tiles long (a cold start costs about five)
#endif
    const bool one_at_a_time = n_tiles_all < n_groups + n_groups / 2 || (kDep == 2 && n_tiles_all < 4 * n_groups) ||
                               (n_tiles_all < MOE_LEAN_ROUNDS * n_groups && KT >= MOE_LEAN_KTILES);
    bool again;
    do {
        seq = 1;
        if (tid == 0) {
            int t = 0;
#pragma unroll 1
            for (int w = 0; w < 3; ++w) {
                t = t >= 0 && (w == 0 || !one_at_a_time) ? with_ready_bit(fetch_tile()) : -1;
                if (w < 2)
                    __hip_atomic_store(my_ticket + w, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                else
                    publish(t);
            }
        }
        MOE_WAIT_VMCNT(0);
        __syncthreads();
        cur_t = __builtin_amdgcn_readfirstlane(
            __hip_atomic_load(my_ticket + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        nxt_t = __builtin_amdgcn_readfirstlane(
            __hip_atomic_load(my_ticket + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        again = one_at_a_time && cur_t >= 0;
        while (cur_t >= 0) {
            if constexpr (kTwo) {
                if (kind_of(cur_t) == 1)
                    engine(std::conditional_t<kTwo, Light, Main>{});
                else
                    engine(Main{});
            } else {
                engine(Main{});
            }
        }
        MOE_WAIT_VMCNT(0);
    } while (again && !gave_up);
#ifdef MOE_TRACE_CLOCK
    if (tid == 0) {
        my_ticket[6] = (int32_t)(__builtin_amdgcn_s_memtime() - trace_c0);
        my_ticket[7] = (int32_t)(__builtin_amdgcn_s_memrealtime() - trace_r0);
        // per tile kind: 100 MHz ticks and tiles, behind the table's last entry (the table must have room)
        uint32_t *out = reinterpret_cast<uint32_t *>(const_cast<TileEntry *>(table) + len0 + len1) + blockIdx.x * 8;
        for (int k = 0; k < 4; ++k) {
            out[2 * k] = trace_ticks[k];
            out[2 * k + 1] = trace_tiles[k];
        }
    }
#endif
    if constexpr (kDep != 0)
        __syncthreads(); // every wavefront of the workgroup has stored (and signalled) what it had to
    // the last workgroup to leave resets the counters for the next launch over this table
    if (tid == 0) {
        if (__hip_atomic_fetch_add(&hdr->done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (int)gridDim.x - 1) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
                for (int x = 0; x < kXcds; ++x)
                    __hip_atomic_store(&hdr->next[s][x], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&hdr->done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if constexpr (kDep == 1) // all producer tiles are in memory: consumers need not look at counters any more
                __hip_atomic_store(&hdr->all_done, dep_epoch1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if constexpr (kDep == 2) // the launch is over: the next one counts from here
                __hip_atomic_store(&g.hdr_dep->epoch, dep_epoch1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}
#endif // __HIP_DEVICE_COMPILE__

// One GEMM per launch.
template <class Main, class Light, bool kSwiglu, bool kGather, bool kScatter = false>
__global__ __launch_bounds__(Main::kThreads, (Main::kLdsBytes <= 80 * 1024 ? 2 : 1)) void grouped_gemm_bf16(GemmArgs g)
{
    static_assert(!(kGather && kScatter) && !(kScatter && kSwiglu), "kScatter belongs to the down projection");
#if defined(__HIP_DEVICE_COMPILE__) // the body uses device-only types (buffer resources); the host pass only needs the stub
    gemm_phase<Main, Light, kSwiglu, kGather, kScatter, 0>(g);
#endif
}

// Both GEMMs of the expert computation in one launch: a workgroup works through the tiles of the first
// (gate/up projection with the activation) and, when none is left to draw, goes on to those of the
// second (down projection), each of which waits for its own rows only.  The tail of the first GEMM and
// the head of the second overlap, and there is one launch instead of two.
template <class Main1, class Light1, class Main2, class Light2>
__global__ __launch_bounds__(Main1::kThreads, 1) void grouped_ffn_bf16(GemmArgs g1, GemmArgs g2)
{
#if defined(__HIP_DEVICE_COMPILE__)
    gemm_phase<Main1, Light1, true, false, false, 1>(g1);
    __syncthreads(); // the ring is drained (every path out of a phase waits for its loads); LDS changes hands
    gemm_phase<Main2, Light2, false, false, false, 2>(g2);
#endif
}

}  // namespace moe
