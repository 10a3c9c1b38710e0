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

// ------------------------------------------------------------------------
// Tiled variant of the same sum for E % 4 == 0 (the benchmark shapes): a workgroup of four
// wavefronts computes 32 tokens x 16 experts.  Every wavefront owns 8 tokens and all 16
// experts (128 accumulators per lane, lane l = partial l of R64 as above).  K tiles of 128
// columns are staged in LDS by buffer_load ... lds: the W_r tile (128 rows x 16 experts, shared
// by the four wavefronts, 16-byte chunks XOR-swizzled so that the per-row reads are conflict
// free) and each wavefront's own 8 x 128 slice of x.  Two stages; the loads of tile kt+1 run
// under the multiply-adds of tile kt.  Rows past H and tokens past N come back as zeros from
// the buffer bounds check; adding a zero product never changes a partial sum (partials start
// at +0 and can never become -0), so the result is the R64 sum bit for bit.
// ------------------------------------------------------------------------
// MOE_ROUTER_MFMA: 1 = the tile is computed on the matrix cores (router_logits_mfma), 0 = on the vector
// ALUs (router_logits_tiled); same bits either way.
#ifndef MOE_ROUTER_MFMA
#define MOE_ROUTER_MFMA 1
#endif
constexpr int kRtTok = 8;        // tokens per wavefront
constexpr int kRtExp = 16;       // experts per workgroup
constexpr int kRtK = 128;        // K tile
#ifndef MOE_RT_WAVES
#define MOE_RT_WAVES 4
#endif
constexpr int kRtWaves = MOE_RT_WAVES;
// K tile of the matrix-core form: 128; 256 where a launch has one or two expert tiles only (E <= 32): few
// workgroups, each with a long reduction, and half as many barriers pay there (E = 8: -11 %), while with
// many expert tiles the larger LDS footprint costs more than that (E = 256: +7 %).
constexpr int kRtKShort = 128, kRtKLong = 256;
#ifndef MOE_RT_STAGES
#define MOE_RT_STAGES 2
#endif

__device__ __forceinline__ int rt_key(int r) { return (((r >> 1) ^ (r >> 3)) & 1) | ((r >> 1) & 2); }

template <bool kBf16>
__global__ __launch_bounds__(kWave *kRtWaves) void router_logits_tiled(
    const void *__restrict__ x, int64_t N, int H, const float *__restrict__ W_r,
    const float *__restrict__ bias, int E, float *__restrict__ logits)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int kXb = kBf16 ? 2 : 4;                  // bytes per x element
    constexpr int kXRow = kRtK * kXb;                   // bytes of one token row in a tile
    constexpr int kXTile = kRtTok * kXRow;              // per wavefront
    constexpr int kWTile = kRtK * kRtExp * 4;           // 8 KiB
    constexpr int kStage = kWTile + kRtWaves * kXTile;
    constexpr int kXLoads = kXTile / 1024;              // per wavefront per tile
    constexpr int kWLoads = kWTile / 1024 / kRtWaves;   // per wavefront per tile
    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * kStage];
    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int e0 = blockIdx.x * kRtExp;
    const int64_t n0 = ((int64_t)blockIdx.y * kRtWaves + wave) * kRtTok;

    // W_r tile rows are 64 bytes (16 experts); a load instruction fills 16 rows
    int w_off[kWLoads];
#pragma unroll
    for (int g = 0; g < kWLoads; ++g) {
        const int r = (wave * kWLoads + g) * 16 + lane / 4; // row inside the tile
        w_off[g] = (r * E + ((lane % 4) ^ rt_key(r)) * 4) * 4;
    }
    // x: this wavefront's 8 token rows; a load instruction fills 1024 / kXRow token rows
    const int64_t n_left = N - n0; // may be <= 0 for the last workgroup: then nothing is in range
    constexpr int kLanesPerRow = kXRow / 16;
    int x_off[kXLoads];
#pragma unroll
    for (int g = 0; g < kXLoads; ++g) {
        const int t = g * (kWave / kLanesPerRow) + lane / kLanesPerRow;
        x_off[g] = (t * H + (lane % kLanesPerRow) * (16 / kXb)) * kXb;
    }
    // The position of a K tile goes into the base address and the byte count of the buffer
    // resources, never into the loads' scalar offset: the range check covers the per-lane offset
    // only, and what has to come back as zeros (rows of W_r past H, tokens past N) is decided by
    // that check.  A column range [k0, k0 + 128) that crosses H makes the x loads of every token
    // but the last read the start of the next token's row: finite values that meet W_r rows of
    // zeros.
    auto clamp32 = [](int64_t b) { return (unsigned)(b < 0 ? 0 : (b > 0xFFFFFFFFll ? 0xFFFFFFFFll : b)); };
    auto issue = [&](int kt) {
        unsigned char *st = lds + (kt & 1) * kStage;
        const int k0 = kt * kRtK;
        const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float *>(W_r + (int64_t)k0 * E + e0), 0, clamp32(((int64_t)(H - k0) * E - e0) * 4),
            0x00020000);
        const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<unsigned char *>(static_cast<const unsigned char *>(x) + (n0 * H + k0) * kXb), 0,
            clamp32(n_left > 0 ? (n_left * H - k0) * kXb : 0), 0x00020000);
#pragma unroll
        for (int g = 0; g < kWLoads; ++g)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_w, (__attribute__((address_space(3))) void *)(st + (wave * kWLoads + g) * 1024), 16,
                w_off[g], 0, 0, 0);
#pragma unroll
        for (int g = 0; g < kXLoads; ++g)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_x, (__attribute__((address_space(3))) void *)(st + kWTile + wave * kXTile + g * 1024), 16,
                x_off[g], 0, 0, 0);
    };

    float acc[kRtTok * kRtExp];
#pragma unroll
    for (int i = 0; i < kRtTok * kRtExp; ++i)
        acc[i] = 0.0f;

    const int KT = (H + kRtK - 1) / kRtK;
    const int key = rt_key(lane); // rows lane and lane + 64 of a tile share the key bits
    issue(0);
    for (int kt = 0; kt < KT; ++kt) {
        __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0): tile kt has landed (own loads)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();       // ... and everyone's; tile kt-1 is no longer read
        asm volatile("" ::: "memory");
        if (kt + 1 < KT)
            issue(kt + 1);
        const unsigned char *st = lds + (kt & 1) * kStage;
        const unsigned char *xs = st + kWTile + wave * kXTile;
#pragma unroll
        for (int sub = 0; sub < kRtK / kWave; ++sub) {
            const int row = sub * kWave + lane; // tile row = column h of this lane
            float wv[kRtExp];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const f32x4 w4 = *reinterpret_cast<const f32x4 *>(st + row * 64 + ((c ^ key) << 4));
                wv[4 * c] = w4[0];
                wv[4 * c + 1] = w4[1];
                wv[4 * c + 2] = w4[2];
                wv[4 * c + 3] = w4[3];
            }
            float xv[kRtTok];
#pragma unroll
            for (int t = 0; t < kRtTok; ++t) {
                if (kBf16)
                    xv[t] = bf16_bits_to_f32(*reinterpret_cast<const uint16_t *>(xs + t * kXRow + row * 2));
                else
                    xv[t] = *reinterpret_cast<const float *>(xs + t * kXRow + row * 4);
            }
            // columns past H: W_r came back as zeros (x may hold the next row's values): the
            // products are +-0
#pragma unroll
            for (int t = 0; t < kRtTok; ++t)
#pragma unroll
                for (int j = 0; j < kRtExp; ++j)
                    acc[t * kRtExp + j] = fmaf(xv[t], wv[j], acc[t * kRtExp + j]);
        }
    }

    // fold the 64 partials of every (token, expert) pair: two groups of 64 pairs (experts 0-7, 8-15)
    float lo[64], hi[64];
#pragma unroll
    for (int t = 0; t < kRtTok; ++t)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            lo[t * 8 + j] = acc[t * kRtExp + j];
            hi[t * 8 + j] = acc[t * kRtExp + 8 + j];
        }
    fold_round<32>(lo, lane & 32);
    fold_round<32>(hi, lane & 32);
    fold_round<16>(lo, lane & 16);
    fold_round<16>(hi, lane & 16);
    fold_round<8>(lo, lane & 8);
    fold_round<8>(hi, lane & 8);
    fold_round<4>(lo, lane & 4);
    fold_round<4>(hi, lane & 4);
    fold_round<2>(lo, lane & 2);
    fold_round<2>(hi, lane & 2);
    fold_round<1>(lo, lane & 1);
    fold_round<1>(hi, lane & 1);
    const int t = lane / 8, j = lane % 8;
    const int64_t n = n0 + t;
    if (n < N) {
        const int ea = e0 + j, eb = e0 + 8 + j;
        if (ea < E) {
            float v = lo[0];
            if (bias)
                v = v + bias[ea];
            logits[n * E + ea] = v;
        }
        if (eb < E) {
            float v = hi[0];
            if (bias)
                v = v + bias[eb];
            logits[n * E + eb] = v;
        }
    }
#endif
}

// ------------------------------------------------------------------------
// The same tile on the matrix cores, without giving up the order of the sum.  v_mfma_f32_4x4x1_16B_f32
// multiplies sixteen independent 4x1 by 1x4 pairs: with a reduction length of ONE every output is
// exactly one fused multiply-add, d = fma(a, b, c) (checked bit for bit against fmaf, signed zeros and
// subnormal products included), so nothing about the summation order is left to the hardware - and
// the instruction retires 256 of them in 8 cycles, twice what the vector ALU does without packed
// arithmetic.  The sixteen blocks of an instruction are sixteen different partial sums of R64:
//   lane (blk = lane / 4, c = lane % 4), instruction (p, q, g):   partial l = 4 blk + g
//     a operand: x[token 4p + c, h]          h = 64 step + l
//     b operand: W_r[h, expert 4c + q]
//     result register r:  partial l of (token 4p + r, expert 4c + q)
// so a lane carries the same 128 accumulators as in the vector form, but now for all 8 tokens x 16
// experts x 4 partials (g), and every K step of 64 columns is 32 instructions instead of 128.
// LDS: the W_r tile keeps row h = 64 sub + 4 blk + g at row slot 64 sub + 16 g + blk (the loads
// gather it that way), so the 16-byte read of lane (blk, c) for a given g - experts 4c .. 4c + 3, the
// four q - is linear in the lane number; the x values of a lane for the four g are 4 consecutive
// elements of one token row.  The folding rounds s = 32, 16, 8, 4 run between lanes (blk bits), as a
// halving exchange; s = 2, 1 (g bits) inside the lane.
// ------------------------------------------------------------------------
template <int kHalf, int kXor>
__device__ __forceinline__ void fold_lanes(float *v, bool upper)
{
#pragma unroll
    for (int i = 0; i < kHalf; ++i) {
        float keep = upper ? v[i + kHalf] : v[i];
        float send = upper ? v[i] : v[i + kHalf];
        v[i] = keep + __shfl_xor(send, kXor);
    }
}

template <bool kBf16, int kRtKm>
__global__ __launch_bounds__(kWave *kRtWaves, 2) void router_logits_mfma(
    const void *__restrict__ x, int64_t N, int H, const float *__restrict__ W_r,
    const float *__restrict__ bias, int E, float *__restrict__ logits)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int kXb = kBf16 ? 2 : 4;                  // bytes per x element
    constexpr int kXRow = kRtKm * kXb;                   // bytes of one token row in a tile
    constexpr int kXTile = kRtTok * kXRow;              // per wavefront
    constexpr int kWTile = kRtKm * kRtExp * 4;           // 8 KiB
    constexpr int kStage = kWTile + kRtWaves * kXTile;
    constexpr int kXLoads = kXTile / 1024;              // per wavefront per tile
    constexpr int kWLoads = kWTile / 1024 / kRtWaves;   // per wavefront per tile
    static_assert(kRtTok == 8 && kRtExp == 16 && kRtKm % 64 == 0, "the index arithmetic below");
    constexpr int kStages = MOE_RT_STAGES;               // LDS ring: the loads run kStages - 1 tiles ahead
    __shared__ __attribute__((aligned(1024))) unsigned char lds[kStages * kStage];
    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int e0 = blockIdx.x * kRtExp;
    const int64_t n0 = ((int64_t)blockIdx.y * kRtWaves + wave) * kRtTok;
    const int blk = lane / 4, c = lane % 4;

    // W_r: load instruction k of a tile fills row slots 16k .. 16k + 15, i.e. (sub, g) = (k / 4, k % 4):
    // lane (blk', chunk) fetches chunk `chunk` of row 64 sub + 4 blk' + g
    int w_off[kWLoads];
#pragma unroll
    for (int gl = 0; gl < kWLoads; ++gl) {
        const int k = wave * kWLoads + gl;
        const int r = 64 * (k / 4) + 4 * blk + (k % 4);
        w_off[gl] = (r * E + c * 4) * 4;
    }
    const int64_t n_left = N - n0;
    constexpr int kLanesPerRow = kXRow / 16;
    int x_off[kXLoads];
#pragma unroll
    for (int gl = 0; gl < kXLoads; ++gl) {
        const int t = gl * (kWave / kLanesPerRow) + lane / kLanesPerRow;
        // 16-byte chunk j of token row t sits at chunk slot j ^ 4 (t % 4): the four rows a read below
        // touches then fall into different quarters of the banks
        x_off[gl] = (t * H + ((lane % kLanesPerRow) ^ ((t & 3) * 4)) * (16 / kXb)) * kXb;
    }
    // (the K tile's position goes into the resources, see router_logits_tiled)
    auto clamp32 = [](int64_t b) { return (unsigned)(b < 0 ? 0 : (b > 0xFFFFFFFFll ? 0xFFFFFFFFll : b)); };
    auto issue = [&](int kt) {
        unsigned char *st = lds + (kt % kStages) * kStage;
        const int k0 = kt * kRtKm;
        const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float *>(W_r + (int64_t)k0 * E + e0), 0, clamp32(k0 < H ? ((int64_t)(H - k0) * E - e0) * 4 : 0),
            0x00020000);
        const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<unsigned char *>(static_cast<const unsigned char *>(x) + (n0 * H + k0) * kXb), 0,
            clamp32(n_left > 0 && k0 < H ? (n_left * H - k0) * kXb : 0), 0x00020000);
#pragma unroll
        for (int gl = 0; gl < kWLoads; ++gl)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_w, (__attribute__((address_space(3))) void *)(st + (wave * kWLoads + gl) * 1024), 16,
                w_off[gl], 0, 0, 0);
#pragma unroll
        for (int gl = 0; gl < kXLoads; ++gl)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rs_x, (__attribute__((address_space(3))) void *)(st + kWTile + wave * kXTile + gl * 1024), 16,
                x_off[gl], 0, 0, 0);
    };

    // acc[((p * 4 + q) * 4 + g)][r]
    f32x4 acc[2 * 4 * 4];
#pragma unroll
    for (int i = 0; i < 32; ++i)
        acc[i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    const int KT = (H + kRtKm - 1) / kRtKm;
    // (tiles past the last one are issued too: their resources hold no bytes, so they fetch nothing and
    // the number of loads in flight stays what the wait below counts on)
#pragma unroll
    for (int t = 0; t + 1 < kStages; ++t)
        issue(t);
    for (int kt = 0; kt < KT; ++kt) {
        // all but the loads of the kStages - 2 tiles after kt have landed (own loads)
        __builtin_amdgcn_s_waitcnt(0x0F70 | (((kStages - 2) * (kWLoads + kXLoads)) & 15) |
                                   ((((kStages - 2) * (kWLoads + kXLoads)) >> 4) << 14));
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();       // ... and everyone's; tile kt-1 is no longer read
        asm volatile("" ::: "memory");
        issue(kt + kStages - 1);
        const unsigned char *st = lds + (kt % kStages) * kStage;
        const unsigned char *xs = st + kWTile + wave * kXTile;
#pragma unroll
        for (int sub = 0; sub < kRtKm / kWave; ++sub) {
            // b operands: for every g the four q of this lane's expert chunk
            f32x4 wv[4];
#pragma unroll
            for (int g = 0; g < 4; ++g)
                wv[g] = *reinterpret_cast<const f32x4 *>(st + (64 * sub + 16 * g + blk) * 64 + c * 16);
            // a operands: for p = 0, 1 the four g of token 4p + c
            float xv[2][4];
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const unsigned char *px = xs + (4 * p + c) * kXRow + (((64 * sub + 4 * blk) * kXb) ^ (c * 64));
                if (kBf16) {
                    const u32x2 raw = *reinterpret_cast<const u32x2 *>(px);
                    xv[p][0] = __uint_as_float(raw[0] << 16);
                    xv[p][1] = __uint_as_float(raw[0] & 0xFFFF0000u);
                    xv[p][2] = __uint_as_float(raw[1] << 16);
                    xv[p][3] = __uint_as_float(raw[1] & 0xFFFF0000u);
                } else {
                    const f32x4 raw = *reinterpret_cast<const f32x4 *>(px);
                    xv[p][0] = raw[0], xv[p][1] = raw[1], xv[p][2] = raw[2], xv[p][3] = raw[3];
                }
            }
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        acc[(p * 4 + q) * 4 + g] =
                            __builtin_amdgcn_mfma_f32_4x4x1f32(xv[p][g], wv[g][q], acc[(p * 4 + q) * 4 + g], 0, 0, 0);
        }
    }

    // Fold.  v index bits, most significant first: p, q (2), r (2), g (2).  The rounds s = 32, 16, 8, 4
    // of R64 pair partials that differ in a blk bit, i.e. lanes that differ in bit 5, 4, 3, 2; each
    // halves what a lane keeps (by p, q.hi, q.lo, r.hi).  Left: r.lo x g, and s = 2, 1 pair g.
    float v[128];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    v[((p * 4 + q) * 4 + r) * 4 + g] = acc[(p * 4 + q) * 4 + g][r];
    fold_lanes<64, 32>(v, lane & 32);
    fold_lanes<32, 16>(v, lane & 16);
    fold_lanes<16, 8>(v, lane & 8);
    fold_lanes<8, 4>(v, lane & 4);
    const int p_keep = (lane >> 5) & 1, q_keep = (lane >> 3) & 3, r_hi = (lane >> 2) & 1;
#pragma unroll
    for (int rl = 0; rl < 2; ++rl) {
        const float *u = v + rl * 4;
        const float w0 = u[0] + u[2], w1 = u[1] + u[3]; // s = 2
        float val = w0 + w1;                             // s = 1
        const int64_t n = n0 + 4 * p_keep + 2 * r_hi + rl;
        const int e = e0 + 4 * c + q_keep;
        if (n < N && e < E) {
            if (bias)
                val = val + bias[e];
            logits[n * E + e] = val;
        }
    }
#endif
}

// (value, index) order of the selection: larger logit first, equal logits to the lower index.
__device__ __forceinline__ bool better(float va, int ia, float vb, int ib)
{
    return (va > vb) || (va == vb && ia < ib);
}

constexpr int kMaxPerLane = MOE_MAX_EXPERTS / kWave;

// One wavefront per token.  Lane l holds experts l, l+64, ...
// kTakeRows: every routed row also takes its local row id from its expert's row pointer as it is
// produced (Section IV-A3: the allocation unit hands out the next free row of a region on arrival);
// rank[n*K + k] receives it, and the pointers end up as the experts' counts.
template <bool kTakeRows>
__global__ __launch_bounds__(kWave *kRouteWaves) void router_topk(
    const float *__restrict__ logits, int64_t N, int E, int K, int score_mode,
    int32_t *__restrict__ topk_idx, float *__restrict__ topk_w, int32_t *__restrict__ row_pointer,
    int32_t *__restrict__ rank)
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
        if constexpr (kTakeRows)
            rank[n * K + lane] = atomicAdd(&row_pointer[my_pick], 1);
    }
}

int launch_route(const void *x, int dtype, int64_t N, int64_t H, const float *W_r,
                 const float *bias, int E, int K, int score_mode, int32_t *topk_idx,
                 float *topk_w, float *logits, hipStream_t st, int32_t *row_pointer, int32_t *rank)
{
    const dim3 block(kWave * kRouteWaves);
    if (E % 4 == 0 && H * (int64_t)E * 4 < ((int64_t)1 << 31) && H * 8 * 4 < ((int64_t)1 << 31)) {
        const dim3 grid((unsigned)ceil_div(E, kRtExp), (unsigned)ceil_div(N, (int64_t)kRtTok * kRtWaves));
#if MOE_ROUTER_MFMA
        if (dtype == MOE_BF16 && E <= 2 * kRtExp)
            hipLaunchKernelGGL((router_logits_mfma<true, kRtKLong>), grid, dim3(kWave * kRtWaves), 0, st, x, N, (int)H,
                               W_r, bias, E, logits);
        else if (dtype == MOE_BF16)
            hipLaunchKernelGGL((router_logits_mfma<true, kRtKShort>), grid, dim3(kWave * kRtWaves), 0, st, x, N, (int)H,
                               W_r, bias, E, logits);
        else
            hipLaunchKernelGGL((router_logits_mfma<false, kRtKShort>), grid, dim3(kWave * kRtWaves), 0, st, x, N, (int)H,
                               W_r, bias, E, logits);
#else
        if (dtype == MOE_BF16)
            hipLaunchKernelGGL(router_logits_tiled<true>, grid, dim3(kWave * kRtWaves), 0, st, x, N, (int)H, W_r,
                               bias, E, logits);
        else
            hipLaunchKernelGGL(router_logits_tiled<false>, grid, dim3(kWave * kRtWaves), 0, st, x, N, (int)H, W_r,
                               bias, E, logits);
#endif
    } else {
        const dim3 grid1((unsigned)ceil_div(N, (int64_t)kTok * kRouteWaves), (unsigned)ceil_div(E, kExp));
        if (dtype == MOE_BF16)
            hipLaunchKernelGGL(router_logits<true>, grid1, block, 0, st, x, N, H, W_r, bias, E, logits);
        else
            hipLaunchKernelGGL(router_logits<false>, grid1, block, 0, st, x, N, H, W_r, bias, E, logits);
    }
    const dim3 grid2((unsigned)ceil_div(N, kRouteWaves));
    if (row_pointer)
        hipLaunchKernelGGL(router_topk<true>, grid2, block, 0, st, logits, N, E, K, score_mode, topk_idx, topk_w,
                           row_pointer, rank);
    else
        hipLaunchKernelGGL(router_topk<false>, grid2, block, 0, st, logits, N, E, K, score_mode, topk_idx, topk_w,
                           (int32_t *)nullptr, (int32_t *)nullptr);
    return check_launch("moe_route");
}

}  // namespace moe
