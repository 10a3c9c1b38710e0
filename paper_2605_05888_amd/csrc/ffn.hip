// Expert computation (Section II-A, step 3): grouped SwiGLU FFN over ragged,
// expert-contiguous row segments whose offsets live on the device.
//
//   GEMM1  a[m, f] = silu(xp[m,:] . W_gate[e,f,:]) * (xp[m,:] . W_up[e,f,:])
//   GEMM2  y[m, c] = a[m,:] . W_down[e,c,:]
//
// Both operands of both GEMMs have the reduction index contiguous, so every lane
// fetches its matrix-core operand (8 consecutive bf16 of one row) with a single
// 16-byte LDS read.  bf16 path: v_mfma_f32_32x32x16_bf16, fp32 accumulators,
// operand tiles brought global -> LDS without staging registers into a ring of
// XOR-swizzled units (grouped_gemm.h), one barrier per K tile.  GEMM1 keeps gate and up columns of the same f in one wavefront, so
// the activation is applied to the accumulators and `g`, `u` never reach memory.
//
// Scheduling is device side: a small kernel turns seg_offsets into a tile table
// (expert, first row, end row, column tile), ordered so that tiles that run
// together share weight tiles; workgroup ids are spread so that each XCD's L2
// sees a compact patch of that order.  Nothing about the routing result is read
// on the host.
#include <atomic>

#include "common.h"
#include "grouped_gemm.h"

namespace moe {

// ------------------------------------------------------------------------
// tile table
// ------------------------------------------------------------------------
constexpr int kSchedThreads = 256;
// relative cost of a tile of a one-row-tile expert and of a full tile, for sharing out the workgroup slots
constexpr int kLightCost = 3, kHeavyCost = 7;
#ifndef MOE_ORDER_ROWS
#define MOE_ORDER_ROWS 4
#define MOE_ORDER_COLS 8
#endif
#ifndef MOE_ORDER_LONG_FIRST
#define MOE_ORDER_LONG_FIRST 1
#endif
constexpr int kOrderRows = MOE_ORDER_ROWS, kOrderCols = MOE_ORDER_COLS; // block of the tile order inside an expert
// experts with at most this many rows go through the shallow tile geometry
constexpr int kLightRows = 64;

// Experts come in two classes: "light" ones with at most `light_rows` rows, whose one row tile
// streams its weights from memory once and mostly waits for them (the GEMM has a shallow, deeply
// prefetching tile geometry for those), and the rest.  Each class forms a stream of tiles (order:
// expert, then column tile, then row tile); the table holds stream 0 (the rest), then stream 1
// (light).  The GEMM's persistent workgroups draw from both.
// Row tiles of an expert with `rows` rows: a remainder of at most `extra` rows rides with the last
// full tile instead of forming a tile of its own.
__device__ __forceinline__ int row_tiles(int32_t rows, int BM, int extra)
{
    const int full = rows / BM, rest = rows - full * BM;
    return full > 0 && rest <= extra ? full : full + (rest > 0 ? 1 : 0);
}

__device__ __forceinline__ int32_t clamped_rows(const int32_t *seg_offsets, int e, int64_t M, int64_t &lo)
{
    int64_t hi = seg_offsets[e + 1];
    lo = seg_offsets[e];
    lo = lo < 0 ? 0 : (lo > M ? M : lo);
    hi = hi < lo ? lo : (hi > M ? M : hi);
    return (int32_t)(hi - lo);
}

// One launch builds the tables of both GEMMs: blockIdx.y picks the set of arguments.
struct TableArgs {
    int n_tiles, max_tiles, out_cols;
    TileTableHeader *hdr;
    TileEntry *table;
};

__global__ __launch_bounds__(kSchedThreads) void build_tile_table(
    const int32_t *__restrict__ seg_offsets, int E_local, int64_t M, int BM, int extra, int light_rows,
    TableArgs gemm1, TableArgs gemm2, int32_t *__restrict__ ready)
{
    const TableArgs &args = blockIdx.y == 0 ? gemm1 : gemm2;
    if (blockIdx.y == 0) // arrival counters of the row tiles start at zero with every schedule
        for (int64_t i = (int64_t)blockIdx.x * kSchedThreads + threadIdx.x; i < M; i += (int64_t)gridDim.x * kSchedThreads)
            ready[i] = 0;
    const int n_tiles = args.n_tiles, max_tiles = args.max_tiles;
    TileTableHeader *__restrict__ hdr = args.hdr;
    TileEntry *__restrict__ table = args.table;
    __shared__ int32_t start[2][MOE_MAX_EXPERTS + 1]; // first tile of each expert in the heavy [0] / light [1] stream
    __shared__ int32_t wave_tot[2][kSchedThreads / kWave];
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    // exclusive scans of tiles per expert; a thread owns a contiguous run of experts
    const int per = (E_local + kSchedThreads - 1) / kSchedThreads;
    const int e_lo = tid * per;
    int32_t mine[2] = {0, 0};
    for (int j = 0; j < per; ++j) {
        const int e = e_lo + j;
        if (e < E_local) {
            int64_t lo;
            const int32_t rows = clamped_rows(seg_offsets, e, M, lo);
            mine[rows <= light_rows ? 1 : 0] += row_tiles(rows, BM, extra) * n_tiles;
        }
    }
    int32_t inc[2] = {mine[0], mine[1]};
    for (int d = 1; d < kWave; d <<= 1) {
        const int32_t t0 = __shfl_up(inc[0], d), t1 = __shfl_up(inc[1], d);
        if (lane >= d) {
            inc[0] += t0;
            inc[1] += t1;
        }
    }
    if (lane == kWave - 1) {
        wave_tot[0][wave] = inc[0];
        wave_tot[1][wave] = inc[1];
    }
    __syncthreads();
    int32_t run[2] = {inc[0] - mine[0], inc[1] - mine[1]};
    for (int w = 0; w < wave; ++w) {
        run[0] += wave_tot[0][w];
        run[1] += wave_tot[1][w];
    }
    for (int j = 0; j < per; ++j) {
        const int e = e_lo + j;
        if (e < E_local) {
            int64_t lo;
            const int32_t rows = clamped_rows(seg_offsets, e, M, lo);
            start[0][e] = run[0];
            start[1][e] = run[1];
            run[rows <= light_rows ? 1 : 0] += row_tiles(rows, BM, extra) * n_tiles;
        }
    }
    if (tid == kSchedThreads - 1) { // the last thread's running sums are the totals
        start[0][E_local] = run[0];
        start[1][E_local] = run[1];
    }
    __syncthreads();
    int32_t len[2] = {start[0][E_local], start[1][E_local]};
    if (len[0] + len[1] > max_tiles) { // cannot happen for monotone offsets within [0, M]
        len[0] = len[0] < max_tiles ? len[0] : max_tiles;
        len[1] = max_tiles - len[0];
    }
    if (blockIdx.x == 0 && tid == 0) {
        hdr->len[0] = len[0];
        hdr->len[1] = len[1];
        // share of the workgroup slots that take the light stream first: the light tiles' share of
        // the work, a light tile counted as kLightCost/kHeavyCost of a heavy one
        const int64_t wl = (int64_t)len[1] * kLightCost, wh = (int64_t)len[0] * kHeavyCost;
        hdr->light_slots = wl + wh > 0 ? (int32_t)((32 * wl + (wl + wh) / 2) / (wl + wh)) : 0;
        hdr->done = 0;
        hdr->error = 0;
        hdr->epoch = 0;
        hdr->all_done = 0;
        hdr->magic = kTableMagic;
        hdr->rows = (int32_t)M;
        hdr->out_cols = args.out_cols;
        for (int s = 0; s < 2; ++s)
            for (int x = 0; x < kXcds; ++x)
                hdr->next[s][x] = 0;
    }
    const int32_t total = len[0] + len[1];
    for (int L = blockIdx.x * kSchedThreads + tid; L < total; L += gridDim.x * kSchedThreads) {
        const int c = L < len[0] ? 0 : 1;
        const int32_t pos = L - (c ? len[0] : 0); // position in the stream
        int lo_e = 0, hi_e = E_local;             // last e with start[c][e] <= pos: the expert that owns it
        while (hi_e - lo_e > 1) {
            const int mid = (lo_e + hi_e) >> 1;
            if (start[c][mid] <= pos)
                lo_e = mid;
            else
                hi_e = mid;
        }
        const int e = lo_e;
        int64_t lo;
        const int32_t n_rows_e = clamped_rows(seg_offsets, e, M, lo);
        const int m_tiles = row_tiles(n_rows_e, BM, extra);
        // Inside an expert the tiles go in blocks of kOrderRows x kOrderCols (row tiles x column
        // tiles): the 32 tiles an XCD takes together (one per compute unit) then share 8 weight tiles
        // and 4 activation tiles in its L2, instead of 32 and one.
        const int local = pos - start[c][e];
        const int band_tiles = kOrderRows * n_tiles; // tiles of a full band of kOrderRows row tiles
        int rb = local / band_tiles;
        const int last_band = (m_tiles - 1) / kOrderRows;
        rb = rb > last_band ? last_band : rb;
        const int h = m_tiles - rb * kOrderRows < kOrderRows ? m_tiles - rb * kOrderRows : kOrderRows;
        const int in_band = local - rb * band_tiles;
        const int cb = in_band / (kOrderCols * h);
        const int in_block = in_band - cb * kOrderCols * h;
        TileEntry t;
        t.expert = e;
        int row_in_band = in_block % h, col_in_block = in_block / h;
#if MOE_ORDER_LONG_FIRST
        // The expert's last row tile takes another time than the full ones: longer when a remainder rides
        // with it, shorter when it is ragged.  Inside a block the long tiles are handed out first and the
        // short ones last, so that the workgroups that finish their previous tile early take the long ones
        // (it is the same set of tiles per block either way).
        if (rb == last_band && h > 1 && n_rows_e != m_tiles * BM) {
            const int wb = n_tiles - cb * kOrderCols < kOrderCols ? n_tiles - cb * kOrderCols : kOrderCols;
            const bool tall = n_rows_e > m_tiles * BM;
            const int first = tall ? wb : 0;                  // tiles of the odd row handed out before the others
            if (tall && in_block < wb) {
                row_in_band = h - 1, col_in_block = in_block;
            } else if (!tall && in_block >= wb * (h - 1)) {
                row_in_band = h - 1, col_in_block = in_block - wb * (h - 1);
            } else {
                row_in_band = (in_block - first) % (h - 1), col_in_block = (in_block - first) / (h - 1);
            }
        }
#endif
        const int row_tile = rb * kOrderRows + row_in_band;
        // rows that the expert's last tile computes beyond its BM
        const int ext = row_tile == m_tiles - 1 && n_rows_e > m_tiles * BM ? n_rows_e - m_tiles * BM : 0;
        t.n_tile = (cb * kOrderCols + col_in_block) | (ext << kTileColBits);
        t.m0 = (int32_t)lo + row_tile * BM;
        t.m_end = (int32_t)lo + n_rows_e;
        table[L] = t;
    }
}

// ------------------------------------------------------------------------
// bf16 matrix-core grouped GEMM
// ------------------------------------------------------------------------
// ------------------------------------------------------------------------
// fp32 path (small, correctness-oriented): one thread per output element
// ------------------------------------------------------------------------
__device__ __forceinline__ int expert_of_row(const int32_t *seg, int E_local, int64_t m)
{
    int lo = 0, hi = E_local; // last e with seg[e] <= m
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (seg[mid] <= m)
            lo = mid;
        else
            hi = mid;
    }
    return (m >= seg[lo] && m < seg[lo + 1]) ? lo : -1;
}

// gather_rows != nullptr: row m of xp is row gather_rows[m] / gather_div of `xp`
__global__ __launch_bounds__(256) void ffn_f32_gate_up(const float *__restrict__ xp, int64_t M, int H,
                                                     int F, int E_local,
                                                     const int32_t *__restrict__ seg,
                                                     const float *__restrict__ Wg,
                                                     const float *__restrict__ Wu,
                                                     float *__restrict__ a,
                                                     const int32_t *__restrict__ gather_rows, int gather_div)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= M * F)
        return;
    const int64_t m = i / F;
    const int f = (int)(i % F);
    const int e = expert_of_row(seg, E_local, m);
    if (e < 0)
        return;
    const float *xr = xp + (gather_rows ? (int64_t)(gather_rows[m] / gather_div) : m) * H;
    const float *g = Wg + ((int64_t)e * F + f) * H;
    const float *u = Wu + ((int64_t)e * F + f) * H;
    float sg = 0.0f, su = 0.0f;
    for (int h = 0; h < H; ++h) {
        sg = fmaf(xr[h], g[h], sg);
        su = fmaf(xr[h], u[h], su);
    }
    a[i] = sg / (1.0f + expf(-sg)) * su;
}

__global__ __launch_bounds__(256) void ffn_f32_down(const float *__restrict__ a, int64_t M, int H, int F,
                                                  int E_local, const int32_t *__restrict__ seg,
                                                  const float *__restrict__ Wd, float *__restrict__ y)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= M * H)
        return;
    const int64_t m = i / H;
    const int c = (int)(i % H);
    const int e = expert_of_row(seg, E_local, m);
    if (e < 0)
        return;
    const float *ar = a + m * F;
    const float *w = Wd + ((int64_t)e * H + c) * F;
    float s = 0.0f;
    for (int f = 0; f < F; ++f)
        s = fmaf(ar[f], w[f], s);
    y[i] = s;
}

// ------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------
// Geometries.  Big: 256x256x64 tile, ring of 5 units (all 160 KiB of LDS); per window the 8 B loads
// of a wavefront go out under the first two k-steps after the barrier, the 8 A loads under the
// other two.  An expert's last full tile also takes a remainder of up to 64 rows ("tall" tile).  Shallow: 64x256x64 tile for experts with few rows, four (A, B) unit pairs, so that
// three K tiles of weights are in flight while one is multiplied. 
// MOE_WEIGHTS_AHEAD: the operand that uses the ring's spare unit to run one K tile further ahead is the
// weights (1) or the activations (0).
#ifndef MOE_WEIGHTS_AHEAD
#define MOE_WEIGHTS_AHEAD 1
#endif
template <bool kSwiglu>
using BigTile = GemmCfg<256, 256, 2, 2, kSwiglu, 64, 5, (MOE_WEIGHTS_AHEAD ? 0x4400 : 0x0044),
                        (MOE_WEIGHTS_AHEAD ? 0x0044 : 0x4400), 0, 64, (MOE_WEIGHTS_AHEAD != 0)>;
#ifndef MOE_SHALLOW_UNITS
#define MOE_SHALLOW_UNITS 8
#endif
template <bool kSwiglu> using ShallowTile = GemmCfg<64, 256, 1, 4, kSwiglu, 64, MOE_SHALLOW_UNITS, 0x1010, 0x2222, 1>;

// The down projection with 128-column tiles, for launches with fewer tiles than compute units (few
// tokens): every tile of such a launch streams its whole weight panel alone and the launch lasts as
// long as one tile, so half as wide a panel on twice as many compute units halves it.  Every output
// element is the same sum in the same order, so y has the same bits as with the 256-column tiles.
template <bool kSwiglu> using NarrowBig = GemmCfg<256, 128, 2, 2, kSwiglu, 64, 6, 0x2222, 0x1111, 0, 64>;
template <bool kSwiglu> using NarrowShallow = GemmCfg<64, 128, 1, 4, kSwiglu, 64, 8, 0x1010, 0x1111, 1>;
// upper bound of the down projection's 256-column tiles up to which the narrow form is used
#ifndef MOE_NARROW_TILE_BOUND
#define MOE_NARROW_TILE_BOUND 256
#endif
constexpr int kNarrowTileBound = MOE_NARROW_TILE_BOUND;

struct FfnPlan {
    bool narrow2; // the down projection runs with NarrowBig / NarrowShallow
    int BM, out_cols1, out_cols2;
    int n_tiles1, n_tiles2, max_m_tiles;
    size_t off_a, off_hdr1, off_tab1, off_hdr2, off_tab2, off_ready, total;
};

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static FfnPlan make_plan(int64_t M, int64_t H, int64_t F, int E_local)
{
    FfnPlan p;
    p.BM = BigTile<true>::BM;
    p.out_cols1 = BigTile<true>::kOutCols; // GEMM1 writes BN/2 columns of `a` per tile
    p.narrow2 = (M / BigTile<false>::BM + E_local) * ceil_div(H, BigTile<false>::kOutCols) <= kNarrowTileBound;
    p.out_cols2 = p.narrow2 ? NarrowBig<false>::kOutCols : BigTile<false>::kOutCols;
    p.n_tiles1 = (int)ceil_div(F, p.out_cols1);
    p.n_tiles2 = (int)ceil_div(H, p.out_cols2);
    p.max_m_tiles = (int)(M / p.BM) + E_local;
    size_t o = 0;
    p.off_a = o;
    o = align_up(o + (size_t)M * F * 2, 256);
    p.off_hdr1 = o;
    o += kTileTableHeaderBytes;
    p.off_tab1 = o;
    o = align_up(o + (size_t)p.max_m_tiles * p.n_tiles1 * sizeof(TileEntry), 256);
    p.off_hdr2 = o;
    o += kTileTableHeaderBytes;
    p.off_tab2 = o;
    o = align_up(o + (size_t)p.max_m_tiles * p.n_tiles2 * sizeof(TileEntry), 256);
    p.off_ready = o; // per row: arrival counter of the row tile that starts there (dependency-driven launches)
    o = align_up(o + (size_t)M * sizeof(int32_t), 256);
    p.total = o;
    return p;
}

size_t ffn_workspace_bytes(int64_t M, int64_t H, int64_t F, int E_local, int dtype)
{
    if (dtype == MOE_F32)
        return align_up((size_t)M * F * 4, 256);
    return make_plan(M, H, F, E_local).total;
}

// Per-device facts, cached on first use.  Entries are written with relaxed atomics and every writer
// stores the same value, so threads that race on the first call of a device do no harm.
constexpr int kMaxDevices = 64;
static int current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return -1;
    return dev;
}

static int compute_units()
{
    static std::atomic<int> cus[kMaxDevices];
    const int dev = current_device();
    int n = dev >= 0 ? cus[dev].load(std::memory_order_relaxed) : 0;
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev < 0 ? 0 : dev) != hipSuccess || n <= 0)
            return kXcds * 32;
        if (dev >= 0)
            cus[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// workgroup slots of the device: compute units times the workgroups of this kernel a unit holds
static int workgroup_slots(int per_cu)
{
    const int cus = compute_units();
    int g = cus * per_cu / kXcds * kXcds; // whole rounds over the XCDs
    if (g > kMaxGemmWorkgroups)
        g = kMaxGemmWorkgroups / kXcds * kXcds;
    return g < kXcds ? kXcds : g;
}

// Raises the kernel's dynamic LDS limit once per device (idempotent, so a race only repeats it).
template <class Kernel>
static void allow_lds(Kernel kern, size_t lds_bytes, std::atomic<uint64_t> &raised)
{
    const int dev = current_device();
    if (dev < 0 || !(raised.load(std::memory_order_relaxed) >> dev & 1)) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds_bytes);
        if (dev >= 0)
            raised.fetch_or(uint64_t(1) << dev, std::memory_order_relaxed);
    }
}

template <class Main, class Light>
static size_t lds_bytes_of()
{
    size_t b = Main::kLdsBytes;
    if constexpr (!std::is_void<Light>::value)
        b = b > Light::kLdsBytes ? b : Light::kLdsBytes;
    return b;
}

static GemmArgs gemm_args(const uint16_t *A, int64_t M, int Kdim, int Ndim, const uint16_t *B0, const uint16_t *B1,
                          uint16_t *C, TileTableHeader *hdr, const TileEntry *table, int patch)
{
    GemmArgs g = {};
    g.A = A, g.M = M, g.Kdim = Kdim, g.Ndim = Ndim, g.B0 = B0, g.B1 = B1, g.C = C, g.hdr = hdr, g.table = table;
    g.patch = patch, g.gather_div = 1;
    return g;
}

template <class Main, class Light, bool kSwiglu, bool kGather = false, bool kScatter = false>
static void launch_gemm(const uint16_t *A, int64_t M, int Kdim, int Ndim, const uint16_t *B0,
                        const uint16_t *B1, uint16_t *C, TileTableHeader *hdr,
                        const TileEntry *table, int patch, hipStream_t st,
                        const int32_t *gather_rows = nullptr, int gather_div = 1, uint32_t gather_bytes = 0,
                        const float *scatter_w = nullptr)
{
    auto kern = grouped_gemm_bf16<Main, Light, kSwiglu, kGather, kScatter>;
    const size_t lds_bytes = lds_bytes_of<Main, Light>();
    static std::atomic<uint64_t> raised{0};
    allow_lds(kern, lds_bytes, raised);
    GemmArgs g = gemm_args(A, M, Kdim, Ndim, B0, B1, C, hdr, table, patch);
    g.gather_rows = gather_rows, g.gather_div = gather_div, g.gather_bytes = gather_bytes, g.scatter_w = scatter_w;
    // persistent grid: the workgroups draw their tiles from the table's counters
    const int grid = workgroup_slots(Main::kLdsBytes <= 80 * 1024 ? 2 : 1);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(Main::kThreads), lds_bytes, st, g);
}

int check_ffn_shape(int dtype, int64_t H, int64_t F)
{
    if (dtype == MOE_BF16 && (H % 64 != 0 || F % 64 != 0))
        return fail(MOE_ERR_UNSUPPORTED,
                    "bf16 moe_grouped_ffn needs H and F to be multiples of 64 (got H=%lld, F=%lld)",
                    (long long)H, (long long)F);
    return MOE_OK;
}

// consecutive tiles each XCD takes at a time (see stream_position)
#ifndef MOE_PATCH
#define MOE_PATCH 32
#endif
constexpr int kPatch = MOE_PATCH;
// polls (about a microsecond each) a dependent tile spends on its rows before it gives up: seconds
constexpr int64_t kDefaultWaitLimit = (int64_t)1 << 22;

struct FfnWorkspace {
    uint16_t *a;
    TileTableHeader *hdr1, *hdr2;
    TileEntry *tab1, *tab2;
    int max1, max2;
    int32_t *ready;
};

static FfnWorkspace carve(const FfnPlan &p, void *ws)
{
    unsigned char *w = static_cast<unsigned char *>(ws);
    FfnWorkspace k;
    k.a = reinterpret_cast<uint16_t *>(w + p.off_a);
    k.hdr1 = reinterpret_cast<TileTableHeader *>(w + p.off_hdr1);
    k.tab1 = reinterpret_cast<TileEntry *>(w + p.off_tab1);
    k.hdr2 = reinterpret_cast<TileTableHeader *>(w + p.off_hdr2);
    k.tab2 = reinterpret_cast<TileEntry *>(w + p.off_tab2);
    k.max1 = p.max_m_tiles * p.n_tiles1;
    k.max2 = p.max_m_tiles * p.n_tiles2;
    k.ready = reinterpret_cast<int32_t *>(w + p.off_ready);
    return k;
}


int launch_ffn_schedule(int dtype, int64_t M, int64_t H, int64_t F, int E_local,
                        const int32_t *seg_offsets, void *ws, hipStream_t st)
{
    if (dtype == MOE_F32)
        return MOE_OK; // the fp32 kernels look their expert up per row
    const FfnPlan p = make_plan(M, H, F, E_local);
    const FfnWorkspace k = carve(p, ws);
    const int max_both = k.max1 > k.max2 ? k.max1 : k.max2;
    hipLaunchKernelGGL(build_tile_table, dim3((unsigned)ceil_div(max_both, kSchedThreads), 2),
                       dim3(kSchedThreads), 0, st, seg_offsets, E_local, M, p.BM, BigTile<true>::kExtra, kLightRows,
                       TableArgs{p.n_tiles1, k.max1, p.out_cols1, k.hdr1, k.tab1},
                       TableArgs{p.n_tiles2, k.max2, p.out_cols2, k.hdr2, k.tab2},
                       k.ready);
    return check_launch("moe_ffn_schedule");
}

// gather_rows == nullptr: xp holds the M rows.  Otherwise xp is x[N, H] and row m is x[gather_rows[m] / K].
int launch_ffn_gate_up(const void *xp, int dtype, int64_t M, int64_t H, int64_t F, int E_local,
                       const int32_t *seg_offsets, const void *W_gate, const void *W_up, void *ws,
                       hipStream_t st, const int32_t *gather_rows, int K, int64_t N)
{
    if (dtype == MOE_F32) {
        hipLaunchKernelGGL(ffn_f32_gate_up, dim3((unsigned)ceil_div(M * F, 256)), dim3(256), 0, st,
                           static_cast<const float *>(xp), M, (int)H, (int)F, E_local, seg_offsets,
                           static_cast<const float *>(W_gate), static_cast<const float *>(W_up),
                           static_cast<float *>(ws), gather_rows, K);
        return check_launch("moe_ffn_gate_up(f32)");
    }
    const FfnPlan p = make_plan(M, H, F, E_local);
    const FfnWorkspace k = carve(p, ws);
    const uint16_t *xpb = static_cast<const uint16_t *>(xp);
    const uint16_t *wg = static_cast<const uint16_t *>(W_gate), *wu = static_cast<const uint16_t *>(W_up);
    if (gather_rows)
        launch_gemm<BigTile<true>, ShallowTile<true>, true, true>(xpb, M, (int)H, (int)F, wg, wu, k.a, k.hdr1, k.tab1,
                                                                  kPatch, st, gather_rows, K, (uint32_t)(N * H * 2));
    else
        launch_gemm<BigTile<true>, ShallowTile<true>, true>(xpb, M, (int)H, (int)F, wg, wu, k.a, k.hdr1, k.tab1, kPatch, st);
    return check_launch("moe_ffn_gate_up");
}

int launch_ffn_down(int dtype, int64_t M, int64_t H, int64_t F, int E_local,
                    const int32_t *seg_offsets, const void *W_down, void *y, void *ws, hipStream_t st)
{
    if (dtype == MOE_F32) {
        hipLaunchKernelGGL(ffn_f32_down, dim3((unsigned)ceil_div(M * H, 256)), dim3(256), 0, st,
                           static_cast<const float *>(ws), M, (int)H, (int)F, E_local, seg_offsets,
                           static_cast<const float *>(W_down), static_cast<float *>(y));
        return check_launch("moe_ffn_down(f32)");
    }
    const FfnPlan p = make_plan(M, H, F, E_local);
    const FfnWorkspace k = carve(p, ws);
    const uint16_t *wd = static_cast<const uint16_t *>(W_down);
    uint16_t *yb = static_cast<uint16_t *>(y);
    if (p.narrow2)
        launch_gemm<NarrowBig<false>, NarrowShallow<false>, false>(k.a, M, (int)F, (int)H, wd, nullptr, yb, k.hdr2, k.tab2, kPatch, st);
    else
        launch_gemm<BigTile<false>, ShallowTile<false>, false>(k.a, M, (int)F, (int)H, wd, nullptr, yb, k.hdr2, k.tab2, kPatch, st);
    return check_launch("moe_ffn_down");
}

// Both GEMMs in one launch, the second consuming the first's rows tile by tile (after launch_ffn_schedule).
template <class Main2, class Light2>
static void launch_both(const FfnPlan &p, const FfnWorkspace &k, const void *xp, int64_t M, int64_t H, int64_t F,
                        const void *W_gate, const void *W_up, const void *W_down, void *y, int64_t wait_limit,
                        hipStream_t st)
{
    using Main1 = BigTile<true>;
    using Light1 = ShallowTile<true>;
    auto kern = grouped_ffn_bf16<Main1, Light1, Main2, Light2>;
    size_t lds_bytes = lds_bytes_of<Main1, Light1>();
    lds_bytes = lds_bytes > lds_bytes_of<Main2, Light2>() ? lds_bytes : lds_bytes_of<Main2, Light2>();
    static std::atomic<uint64_t> raised{0};
    allow_lds(kern, lds_bytes, raised);
    GemmArgs g1 = gemm_args(static_cast<const uint16_t *>(xp), M, (int)H, (int)F, static_cast<const uint16_t *>(W_gate),
                            static_cast<const uint16_t *>(W_up), k.a, k.hdr1, k.tab1, kPatch);
    GemmArgs g2 = gemm_args(k.a, M, (int)F, (int)H, static_cast<const uint16_t *>(W_down), nullptr,
                            static_cast<uint16_t *>(y), k.hdr2, k.tab2, kPatch);
    g1.ready = g2.ready = k.ready;
    g1.hdr_dep = g2.hdr_dep = k.hdr1;
    g1.ready_per_launch = g2.ready_per_launch = Main1::kWaves * p.n_tiles1;
    g1.wait_limit = g2.wait_limit = wait_limit > 0 ? wait_limit : kDefaultWaitLimit;
    hipLaunchKernelGGL(kern, dim3(workgroup_slots(1)), dim3(Main1::kThreads), lds_bytes, st, g1, g2);
}

int launch_ffn_gate_up_down(const void *xp, int64_t M, int64_t H, int64_t F, int E_local, const void *W_gate,
                            const void *W_up, const void *W_down, void *y, void *ws, int64_t wait_limit,
                            hipStream_t st)
{
    const FfnPlan p = make_plan(M, H, F, E_local);
    const FfnWorkspace k = carve(p, ws);
    if (p.narrow2)
        launch_both<NarrowBig<false>, NarrowShallow<false>>(p, k, xp, M, H, F, W_gate, W_up, W_down, y, wait_limit, st);
    else
        launch_both<BigTile<false>, ShallowTile<false>>(p, k, xp, M, H, F, W_gate, W_up, W_down, y, wait_limit, st);
    return check_launch("moe_ffn_gate_up_down");
}

// Waits for `st`, then reads the two tables' error words.
int ffn_status(int64_t M, int64_t H, int64_t F, int E_local, const void *ws, hipStream_t st)
{
    const FfnPlan p = make_plan(M, H, F, E_local);
    const FfnWorkspace k = carve(p, const_cast<void *>(ws));
    int32_t err[2] = {0, 0};
    if (hipMemcpyAsync(&err[0], &k.hdr1->error, sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipMemcpyAsync(&err[1], &k.hdr2->error, sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
        return check_launch("moe_ffn_status") != MOE_OK ? MOE_ERR_LAUNCH
                                                        : fail(MOE_ERR_LAUNCH, "moe_ffn_status: copy failed");
    for (int g = 0; g < 2; ++g) {
        if (err[g] == kNoScheduleError)
            return fail(MOE_ERR_STATE, "GEMM%d ran over a workspace that moe_ffn_schedule had not filled for M=%lld "
                                       "(and this H, F, E_local)", g + 1, (long long)M);
        if (err[g] == kDependencyTimeout)
            return fail(MOE_ERR_STATE, "GEMM%d gave up waiting for rows of the first GEMM (poll limit reached); "
                                       "its output is incomplete", g + 1);
    }
    return MOE_OK;
}

// ------------------------------------------------------------------------
// down projection with the combine in its epilogue
// ------------------------------------------------------------------------
__global__ void fill_zero_16B(u32x4 *__restrict__ p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        p[i] = u32x4{0u, 0u, 0u, 0u};
}

// sums[N*H] fp32 -> out[N*H] bf16, eight elements per thread
__global__ void round_sums_bf16(const f32x4 *__restrict__ sums, u32x4 *__restrict__ out, int64_t n8)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n8)
        return;
    const f32x4 a = __builtin_nontemporal_load(&sums[2 * i]), b = __builtin_nontemporal_load(&sums[2 * i + 1]);
    u32x4 o;
    o[0] = pack_bf16x2(a[0], a[1]);
    o[1] = pack_bf16x2(a[2], a[3]);
    o[2] = pack_bf16x2(b[0], b[1]);
    o[3] = pack_bf16x2(b[2], b[3]);
    out[i] = o;
}

int launch_ffn_down_combine(int64_t N, int K, int64_t H, int64_t F, int E_local, const void *W_down,
                            const int32_t *row_of_slot, const float *topk_w, float *sums, void *out,
                            void *ws, hipStream_t st)
{
    const int64_t M = N * K;
    const FfnPlan p = make_plan(M, H, F, E_local);
    const FfnWorkspace k = carve(p, ws);
    const int64_t n16 = N * H / 4, n8 = N * H / 8;
    hipLaunchKernelGGL(fill_zero_16B, dim3((unsigned)ceil_div(n16, 256)), dim3(256), 0, st,
                       reinterpret_cast<u32x4 *>(sums), n16);
    if (p.narrow2)
        launch_gemm<NarrowBig<false>, NarrowShallow<false>, false, false, true>(
            k.a, M, (int)F, (int)H, static_cast<const uint16_t *>(W_down), nullptr,
            reinterpret_cast<uint16_t *>(sums), k.hdr2, k.tab2, kPatch, st, row_of_slot, K, 0u, topk_w);
    else
        launch_gemm<BigTile<false>, ShallowTile<false>, false, false, true>(
            k.a, M, (int)F, (int)H, static_cast<const uint16_t *>(W_down), nullptr,
            reinterpret_cast<uint16_t *>(sums), k.hdr2, k.tab2, kPatch, st, row_of_slot, K, 0u, topk_w);
    hipLaunchKernelGGL(round_sums_bf16, dim3((unsigned)ceil_div(n8, 256)), dim3(256), 0, st,
                       reinterpret_cast<const f32x4 *>(sums), static_cast<u32x4 *>(out), n8);
    return check_launch("moe_ffn_down_combine");
}

}  // namespace moe
