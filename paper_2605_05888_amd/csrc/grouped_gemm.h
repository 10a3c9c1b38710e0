// bf16 matrix-core grouped GEMM for gfx950: C[m, n] = sum_k A[m, k] * B[e(m), n, k]
// over ragged row segments described by a device-side tile table.
//
// Both operands have k contiguous.  One workgroup = WM x WN wavefronts computes a
// BM x BN tile; every wavefront owns a (BM/WM) x (BN/WN) sub-tile as 32x32 blocks of
// v_mfma_f32_32x32x16_bf16.
//
// Pipeline (K tiles of BK = 32 or 64 elements; LDS is a ring of U units, a unit holding the A rows
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
#pragma once

#include <type_traits>

#include "common.h"

namespace moe {

struct TileEntry {
    int32_t expert; // local expert
    int32_t m0;     // first row of the tile
    int32_t m_end;  // end of the expert's segment (rows >= m_end are not written)
    int32_t n_tile; // column tile
};

struct TileTableHeader {
    int32_t num_tiles;
    int32_t pad[3];
};

constexpr int kXcds = 8;

// Workgroup id -> position in the tile order.  Ids are dealt round-robin to the
// 8 XCDs; each XCD takes runs of `patch` consecutive tiles so its L2 sees tiles
// that share weight and activation rows.
__device__ __forceinline__ int tile_of_workgroup(int id, int patch)
{
    const int xcd = id % kXcds, j = id / kXcds;
    return (j / patch) * (patch * kXcds) + xcd * patch + (j % patch);
}

__device__ __forceinline__ float silu_mul(float g, float u)
{
    return g / (1.0f + __expf(-g)) * u;
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

// Waits until at most `tiles` K tiles (kLoads loads each) of this lane are still in flight;
// `tiles` is clamped to [0, kMax].
template <int kLoads, int kMax>
__device__ __forceinline__ void wait_tiles_in_flight(int tiles)
{
    if constexpr (kMax <= 0) {
        MOE_WAIT_VMCNT(0);
    } else {
        if (tiles >= kMax)
            MOE_WAIT_VMCNT(kMax * kLoads);
        else
            wait_tiles_in_flight<kLoads, kMax - 1>(tiles);
    }
}

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
// position the B loads go first, then the A loads; `a_needed` says whether the A loads of the window
// belong to the same K tile as its B loads (else they belong to a later one and nobody waits yet).
constexpr int window_tail(int dist_a, int dist_b, int parts, bool a_needed)
{
    int after = 0;
    for (int p = parts - 1; p >= 0; --p) {
        if (a_needed && part_loads(dist_a, parts, p) > 0)
            return after;
        after += part_loads(dist_a, parts, p);
        if (part_loads(dist_b, parts, p) > 0)
            return after;
    }
    return after;
}

template <int BM, int BN, int WM, int WN, bool kSwiglu, int kBK, int kUnits>
struct GemmCfg {
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
    // LDS is a ring of kUnits units; a unit holds the A rows or the B rows of one K tile.
    static constexpr int kUnitBytes = (BM > BN ? BM : BN) * kRowBytes;
    static constexpr int kDepth = kUnits / 2;  // K tiles whose B part fits besides the one in use
    static constexpr int kAheadA = kUnits % 2; // an odd ring lets the A loads run one tile further ahead
    static constexpr size_t kLdsBytes = (size_t)kUnits * kUnitBytes;
    static_assert(kBK == 32 || kBK == 64, "K tile");
    static_assert(kUnits >= 4, "two K tiles at least");
    static_assert(kWaveM % 32 == 0 && kWaveN % 32 == 0, "wave tile must be 32x32 blocks");
    static_assert(BM % (kGroupRows * kWaves) == 0 && BN % (kGroupRows * kWaves) == 0, "load groups");
    static_assert(!kSwiglu || kBlkN % 2 == 0, "gate and up halves");
    static_assert(kLoadsPerTile * (kDepth + kAheadA) <= 63, "vmcnt budget");
};

template <int BM, int BN, int WM, int WN, bool kSwiglu, int kBK, int kUnits, int kDistA, int kDistB>
__global__ __launch_bounds__(WM *WN *kWave, (BM * BN <= 256 * 128 ? 2 : 1)) void grouped_gemm_bf16(
    const uint16_t *__restrict__ A, int64_t M, int Kdim, int Ndim,
    const uint16_t *__restrict__ B0, const uint16_t *__restrict__ B1,
    uint16_t *__restrict__ C, const TileTableHeader *__restrict__ hdr,
    const TileEntry *__restrict__ table, int patch)
{
#if defined(__HIP_DEVICE_COMPILE__) // the body uses device-only types (buffer resources); the host pass only needs the stub
    using Cfg = GemmCfg<BM, BN, WM, WN, kSwiglu, kBK, kUnits>;
    constexpr int kChunks = Cfg::kChunks, kRowBytes = Cfg::kRowBytes, kKSteps = Cfg::kKSteps;
    constexpr int kDepth = Cfg::kDepth, kAheadA = Cfg::kAheadA;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int L = tile_of_workgroup(blockIdx.x, patch);
    if (L >= hdr->num_tiles)
        return;
    const TileEntry te = table[L];
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int wm = wave / WN, wn = wave % WN;
    const int n0 = te.n_tile * Cfg::kOutCols;

    // ---- global->LDS loads (buffer_load_dwordx4 ... lds): the lane at 16-byte position p of its
    //      row fetches chunk p ^ key(row).  Buffer addressing keeps the per-lane part of the address
    //      in one 32-bit register (row offset inside the tile, fixed for the whole K loop); the tile
    //      base sits in the scalar resource and the K offset in a scalar register.
    const int ld_row = lane / kChunks, ld_pc = lane % kChunks;
    //      Rows past the end of the segment (and columns past Ndim) lie beyond the resource's byte
    //      count: the bounds check returns zeros for them without touching memory.
    const int64_t rows_left = (int64_t)te.m_end - te.m0; // >= 1
    const int64_t a_bytes = (rows_left < BM ? rows_left : BM) * (int64_t)Kdim * 2;
    const uint16_t *a_base = A + (int64_t)te.m0 * Kdim;
    int a_off[Cfg::kAGroups];
#pragma unroll
    for (int g = 0; g < Cfg::kAGroups; ++g) {
        const int r = (wave * Cfg::kAGroups + g) * Cfg::kGroupRows + ld_row;
        a_off[g] = (r * Kdim + ((ld_pc ^ row_key<kChunks>(r)) * 8)) * 2;
    }
    // B rows of one wavefront (kSwiglu): first half gate columns, second half the same up columns.
    // A load group never straddles the two halves, so its resource is wave-uniform.
    const int cols_left = Ndim - n0; // >= 1
    const int64_t b_bytes = (cols_left < Cfg::kOutCols ? cols_left : Cfg::kOutCols) * (int64_t)Kdim * 2;
    const uint16_t *b0_base = B0 + ((int64_t)te.expert * Ndim + n0) * Kdim;
    const uint16_t *b1_base = (kSwiglu ? B1 : B0) + ((int64_t)te.expert * Ndim + n0) * Kdim;
    int b_off[Cfg::kBGroups];
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
    const int KT = Kdim / kBK;
    // A K tile past the end of the reduction is "loaded" through a resource of zero bytes: every
    // lane is out of range, nothing is fetched and zeros land in a unit nobody reads.  So the
    // loop issues the same number of loads in every iteration and the vmcnt arithmetic below
    // holds from the first tile to the last.
    auto resource = [&](const uint16_t *base, int64_t bytes, int tile) {
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(base), 0,
                                                 tile < KT ? (unsigned)bytes : 0u, 0x00020000);
    };
    using lds_ptr = __attribute__((address_space(3))) void *;
    auto load_a_group = [&](int tile, int unit, int g) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            resource(a_base, a_bytes, tile),
            (lds_ptr)(lds + unit * Cfg::kUnitBytes + (wave * Cfg::kAGroups + g) * 1024), 16, a_off[g],
            tile * (kBK * 2), 0, 0);
    };
    auto load_b_group = [&](int tile, int unit, int g) {
        const int r0 = (wave * Cfg::kBGroups + g) * Cfg::kGroupRows; // uniform
        const bool up = kSwiglu && (r0 % Cfg::kWaveN) >= Cfg::kWaveN / 2;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            resource(up ? b1_base : b0_base, b_bytes, tile),
            (lds_ptr)(lds + unit * Cfg::kUnitBytes + (wave * Cfg::kBGroups + g) * 1024), 16, b_off[g],
            tile * (kBK * 2), 0, 0);
    };

    // ---- the ring.  K tile t keeps its A rows in unit (2t) % kUnits and its B rows in unit
    //      (2t+1) % kUnits.  `u` below is always the A unit of the tile being multiplied.
    auto wrap = [](int x) { return x >= kUnits ? x - kUnits : x; };
    auto unit_a = [&](int u, int ahead) { return wrap(u + (2 * ahead) % kUnits); };
    auto unit_b = [&](int u, int ahead) { return wrap(u + (2 * ahead + 1) % kUnits); };

    // ---- load schedule.  The barrier that ends the reads of tile t opens a "window": the units of
    //      tile t are free, and until the next barrier the loads of B(t + kDepth) and of
    //      A(t + kDepth + kAheadA) are issued, in kKSteps positions: position 0 under the last
    //      k-step of tile t, position p under k-step p-1 of tile t+1 (kDistB / kDistA say how many
    //      loads each position takes; B first, then A).  Spreading them keeps the four wavefronts
    //      from pushing a whole tile into the memory pipeline in one burst; putting the B loads
    //      early gives them two to three k-steps to land before the barrier that needs them, and
    //      the A loads, which are needed one tile later when the ring is odd, fill the rest.
    static_assert(part_first(kDistA, kKSteps, kKSteps) == Cfg::kAGroups, "A loads of a window");
    static_assert(part_first(kDistB, kKSteps, kKSteps) == Cfg::kBGroups, "B loads of a window");
    auto issue_position = [&](int t, int u, auto pos_tag) { // window opened by the barrier of tile t
        constexpr int p = decltype(pos_tag)::value;
#pragma unroll
        for (int g = part_first(kDistB, kKSteps, p); g < part_first(kDistB, kKSteps, p + 1); ++g)
            load_b_group(t + kDepth, unit_b(u, kDepth), g);
#pragma unroll
        for (int g = part_first(kDistA, kKSteps, p); g < part_first(kDistA, kKSteps, p + 1); ++g)
            load_a_group(t + kDepth + kAheadA, unit_a(u, kDepth + kAheadA), g);
    };
    auto loads_at = [](int p) { return part_loads(kDistA, kKSteps, p) + part_loads(kDistB, kKSteps, p); };
    // loads that may still be in flight when a barrier needs the next tile complete
    constexpr int kInFlight = (kDepth - 2) * Cfg::kLoadsPerTile + window_tail(kDistA, kDistB, kKSteps, kAheadA == 0);

    // ---- operand reads: lane (i = lane%32, kg = lane/32) reads chunk (2*ks + kg) of row i of a block.
    //      Block and wavefront offsets are multiples of 32 rows, so the key depends on i only, and
    //      k-step ks is the k-step-0 offset with chunk bits flipped by 2*ks.
    const int fr = lane % 32, kg = lane / 32;
    const int key = row_key<kChunks>(fr);
    const int a_off0 = (wm * Cfg::kWaveM + fr) * kRowBytes + ((kg ^ key) << 4);
    const int b_off0 = (wn * Cfg::kWaveN + fr) * kRowBytes + ((kg ^ key) << 4);

    bf16x8 fa[2][Cfg::kBlkM], fb[2][Cfg::kBlkN];
    // `act` = number of this wavefront's 32-row blocks that hold rows of the segment: blocks past
    // the end of a ragged segment are neither read nor multiplied.
    auto read_frags = [&](int u, int ks, int slot, auto act_tag) { // u = A unit of the tile
        constexpr int kAct = decltype(act_tag)::value;
        const unsigned char *pa = lds + u * Cfg::kUnitBytes + (a_off0 ^ (ks << 5));
        const unsigned char *pb = lds + wrap(u + 1) * Cfg::kUnitBytes + (b_off0 ^ (ks << 5));
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
#pragma unroll
    for (int i = 0; i < Cfg::kBlkM; ++i)
#pragma unroll
        for (int j = 0; j < Cfg::kBlkN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0.0f;

    auto mfma_all = [&](int slot, auto act_tag) {
        constexpr int kAct = decltype(act_tag)::value;
#pragma unroll
        for (int i = 0; i < kAct; ++i)
#pragma unroll
            for (int j = 0; j < Cfg::kBlkN; ++j) // weights first: the result block is [n][m]
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[slot][j], fa[slot][i], acc[i][j], 0, 0, 0);
    };

    auto pipeline = [&](auto act) {
        constexpr int kAct = decltype(act)::value;
        constexpr int kMfma = kAct * Cfg::kBlkN, kReads = kAct ? kAct + Cfg::kBlkN : 0;
        // ---- prologue: everything the windows before tile 0 would have issued, then position 0
        //      of the window before tile 0; tile 0 landed
#pragma unroll
        for (int t = 0; t + 1 < kDepth + kAheadA; ++t) {
#pragma unroll
            for (int g = 0; g < Cfg::kAGroups; ++g)
                load_a_group(t, (2 * t) % kUnits, g);
            if (t + 1 < kDepth) {
#pragma unroll
                for (int g = 0; g < Cfg::kBGroups; ++g)
                    load_b_group(t, (2 * t + 1) % kUnits, g);
            }
        }
        issue_position(-1, kUnits - 2, std::integral_constant<int, 0>{});
        // in flight after B(0): tiles 1 .. kDepth-2, the A rows that run ahead, position 0
        MOE_WAIT_VMCNT((kDepth - 2) * Cfg::kLoadsPerTile + kAheadA * Cfg::kAGroups + loads_at(0));
        lds_barrier();
        read_frags(0, 0, 0, act);

        // k-step ks of tile kt (not its last): position ks+1 of the window goes out, the operands
        // of k-step ks+1 are read, all under this step's MFMAs
        auto kstep = [&](int kt, int u, auto ks_tag) {
            constexpr int ks = decltype(ks_tag)::value;
            issue_position(kt - 1, wrap(u + kUnits - 2), std::integral_constant<int, ks + 1>{});
            read_frags(u, ks + 1, (ks + 1) & 1, act);
            mfma_all(ks & 1, act);
            interleave_under_mfma<kMfma, kReads, loads_at(ks + 1)>();
        };
        // The body is branch free (a branch around the LDS reads would make the compiler wait for
        // them before MFMAs that do not need them).
        int u = 0;
        for (int kt = 0; kt < KT; ++kt) {
            kstep(kt, u, std::integral_constant<int, 0>{});
            if constexpr (kKSteps > 2) {
                kstep(kt, u, std::integral_constant<int, 1>{});
                kstep(kt, u, std::integral_constant<int, 2>{});
            }
            __builtin_amdgcn_sched_barrier(0); // keep this k-step's MFMAs above the waits
            MOE_WAIT_LGKM0();                  // my reads of tile kt are complete
            MOE_WAIT_VMCNT(kInFlight);         // my part of tile kt+1 has landed
            lds_barrier();                     // ... and everyone's; the units of tile kt are free
            issue_position(kt, u, std::integral_constant<int, 0>{});
            read_frags(unit_a(u, 1), 0, 0, act); // after the last tile: a unit of zeros, unused
            mfma_all((kKSteps - 1) & 1, act);
            interleave_under_mfma<kMfma, kReads, loads_at(0)>();
            u = unit_a(u, 1);
        }
        MOE_WAIT_VMCNT(0); // the zero-byte loads past the last tile still write LDS: let them finish
    };
    // rows of the segment inside this wavefront's part of the tile -> active 32-row blocks
    {
        const int64_t rows = (int64_t)te.m_end - ((int64_t)te.m0 + wm * Cfg::kWaveM);
        const int active = rows <= 0 ? 0 : (rows >= Cfg::kWaveM ? Cfg::kBlkM : (int)((rows + 31) / 32));
        if (active == Cfg::kBlkM)
            pipeline(std::integral_constant<int, Cfg::kBlkM>{});
        else if (active == 0)
            pipeline(std::integral_constant<int, 0>{});
        else if (active == 1)
            pipeline(std::integral_constant<int, 1>{});
        else if (Cfg::kBlkM > 2 && active == 2)
            pipeline(std::integral_constant<int, (Cfg::kBlkM > 2 ? 2 : 1)>{});
        else
            pipeline(std::integral_constant<int, (Cfg::kBlkM > 3 ? 3 : 1)>{});
    }

    // ---- epilogue.  Block (i, j), register r of lane l:
    //      output row    m = i*32 + l%32               (within the wavefront's rows)
    //      output column n = j*32 + 8*(r/4) + 4*(l/32) + r%4
    const int m_lane = lane % 32, n_lane = (lane / 32) * 4;
    constexpr int kOutBlkN = kSwiglu ? Cfg::kBlkN / 2 : Cfg::kBlkN;
#pragma unroll
    for (int i = 0; i < Cfg::kBlkM; ++i) {
        const int64_t m = (int64_t)te.m0 + wm * Cfg::kWaveM + i * 32 + m_lane;
        if (m >= te.m_end)
            continue;
        uint16_t *crow = C + m * Ndim;
#pragma unroll
        for (int j = 0; j < kOutBlkN; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = n0 + wn * (kOutBlkN * 32) + j * 32 + q * 8 + n_lane;
                if (col >= Ndim)
                    continue;
                float v[4];
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    v[t] = kSwiglu ? silu_mul(acc[i][j][q * 4 + t], acc[i][j + kOutBlkN][q * 4 + t])
                                   : acc[i][j][q * 4 + t];
                u32x2 o;
                o[0] = pack_bf16x2(v[0], v[1]);
                o[1] = pack_bf16x2(v[2], v[3]);
                *reinterpret_cast<u32x2 *>(crow + col) = o;
            }
        }
    }
#endif
}

}  // namespace moe
