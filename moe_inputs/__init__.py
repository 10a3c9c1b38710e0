"""Seeded synthetic inputs for the MoE-layer hot path.

This module only *generates data*: activations, router weights, expert weights,
popularity biases and synthetic receive-buffer segment sizes.  It contains none
of the method's arithmetic (no gating, no layout, no FFN), so both the CPU
oracle's tests and the HIP path's tests may draw their inputs from it.

Every tensor element is a pure function of (seed, stream id, flat element
index): a counter-based generator.  The same function is implemented twice,
here with numpy (host) and in ``fill.hip`` (device), and the two agree bit for
bit because the recipe uses only 64-bit integer mixing, one int->float
conversion and one fp32 multiply.

Element recipe ("sum of twelve uniforms"):
    r_j   = mix64(key + (3*i + j + 1) * GOLDEN),  j = 0, 1, 2
    s     = sum of the twelve 16-bit fields of r_0, r_1, r_2
    value = float32(s - 6*65535) * float32(sigma / sqrt(65536**2 - 1))
which has mean 0, standard deviation sigma and an approximately normal shape
(support +-6 sigma).  bf16 tensors round that fp32 value to nearest-even.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

# stream ids: one per logical tensor of a configuration
STREAM_X = 1
STREAM_W_ROUTER = 2
STREAM_W_GATE = 3
STREAM_W_UP = 4
STREAM_W_DOWN = 5
STREAM_RANK_PERM = 6
STREAM_RECV_X = 7
STREAM_RECV_ASSIGN = 8

BF16 = "bf16"
F32 = "f32"

SCORE_SOFTMAX_TOPK = 0
SCORE_SIGMOID_TOPK = 1


@dataclasses.dataclass(frozen=True)
class MoEConfig:
    """One synthetic MoE-layer workload (shapes follow the paper's Table II and
    the larger public model shapes named by the benchmark definition)."""
    name: str
    N: int          # local tokens
    H: int          # hidden size
    E: int          # experts
    K: int          # top-K
    F: int          # expert FFN hidden size
    G: int          # logical destinations (E % G == 0)
    dtype: str      # BF16 or F32 (activations and expert weights)
    score_mode: int
    zipf_s: float   # 0 -> uniform routing, else Zipf exponent of expert popularity
    seed: int
    bias_gain: float = 0.0   # != 0 (with zipf_s == 0): router bias = bias_gain * a fixed seeded pattern (mild skew)

    @property
    def R(self) -> int:
        return self.N * self.K

    @property
    def elt_bytes(self) -> int:
        return 2 if self.dtype == BF16 else 4


CONFIGS = {
    "tiny": MoEConfig("tiny", 256, 128, 8, 2, 256, 1, F32, SCORE_SOFTMAX_TOPK, 0.0, 0),
    "mixtral": MoEConfig("mixtral", 4096, 4096, 8, 2, 14336, 1, BF16, SCORE_SOFTMAX_TOPK, 0.0, 1),
    "gptoss": MoEConfig("gptoss", 8192, 2880, 128, 4, 2880, 1, BF16, SCORE_SOFTMAX_TOPK, 1.0, 2),
    "dsv3": MoEConfig("dsv3", 16384, 7168, 256, 8, 2048, 1, BF16, SCORE_SIGMOID_TOPK, 0.0, 3),
    "dsv3_ep": MoEConfig("dsv3_ep", 8192, 7168, 256, 8, 2048, 32, BF16, SCORE_SIGMOID_TOPK, 1.2, 4),
    # the two other model shapes of the paper's Table II (Mixtral 8x7B is "mixtral" above)
    "qwen2moe": MoEConfig("qwen2moe", 8192, 2048, 64, 4, 1408, 1, BF16, SCORE_SOFTMAX_TOPK, 0.0, 5),
    "phi35moe": MoEConfig("phi35moe", 8192, 4096, 16, 2, 6400, 1, BF16, SCORE_SOFTMAX_TOPK, 0.0, 6),
}


def small_variant(cfg: MoEConfig, N: int, H: int, F: int, name: str | None = None) -> MoEConfig:
    """Same routing structure (E, K, G, skew, score mode, dtype), smaller tensors."""
    return dataclasses.replace(cfg, N=N, H=H, F=F, name=name or (cfg.name + "_small"))


# --------------------------------------------------------------------------
# counter-based generator (host side)
# --------------------------------------------------------------------------
def mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on a uint64 array (wrapping arithmetic)."""
    z = z ^ (z >> np.uint64(30))
    z = z * _M1
    z = z ^ (z >> np.uint64(27))
    z = z * _M2
    z = z ^ (z >> np.uint64(31))
    return z


def stream_key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        a = np.array([seed], dtype=np.uint64) * np.uint64(0xD1342543DE82EF95)
        b = np.array([stream], dtype=np.uint64) * GOLDEN
        return mix64(mix64(a + np.uint64(1)) ^ b)[0]


def scale_f32(sigma: float) -> np.float32:
    return np.float32(sigma / math.sqrt(65536.0 ** 2 - 1.0))


def raw_u64(seed: int, stream: int, start: int, count: int, lane: int = 0, lanes: int = 1) -> np.ndarray:
    """mix64(key + (lanes*i + lane + 1) * GOLDEN) for i in [start, start+count)."""
    key = stream_key(seed, stream)
    with np.errstate(over="ignore"):
        i = np.arange(start, start + count, dtype=np.uint64)
        return mix64(key + (np.uint64(lanes) * i + np.uint64(lane + 1)) * GOLDEN)


def normal_f32(seed: int, stream: int, start: int, count: int, sigma: float) -> np.ndarray:
    """fp32 values of flat elements [start, start+count) of a stream."""
    out = np.empty(count, dtype=np.float32)
    c = scale_f32(sigma)
    chunk = 1 << 22
    for lo in range(0, count, chunk):
        n = min(chunk, count - lo)
        s = np.zeros(n, dtype=np.int64)
        for j in range(3):
            r = raw_u64(seed, stream, start + lo, n, lane=j, lanes=3)
            for q in range(4):
                s += ((r >> np.uint64(16 * q)) & np.uint64(0xFFFF)).astype(np.int64)
        out[lo:lo + n] = (s - 6 * 65535).astype(np.float32) * c
    return out


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (finite inputs)."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def tensor_sigma(cfg: MoEConfig, stream: int) -> float:
    if stream in (STREAM_X, STREAM_RECV_X):
        return 1.0
    if stream in (STREAM_W_ROUTER, STREAM_W_GATE, STREAM_W_UP):
        return 1.0 / math.sqrt(cfg.H)       # N(0, 1/fan_in), fan_in = H
    if stream == STREAM_W_DOWN:
        return 1.0 / math.sqrt(cfg.F)       # fan_in = F
    raise ValueError(stream)


def tensor_shape(cfg: MoEConfig, stream: int) -> tuple:
    """Logical shapes.  Expert weights are stored "out x in" (reduction index
    contiguous): W_gate, W_up: [E, F, H];  W_down: [E, H, F].  Router: [H, E]."""
    if stream == STREAM_X:
        return (cfg.N, cfg.H)
    if stream == STREAM_W_ROUTER:
        return (cfg.H, cfg.E)
    if stream in (STREAM_W_GATE, STREAM_W_UP):
        return (cfg.E, cfg.F, cfg.H)
    if stream == STREAM_W_DOWN:
        return (cfg.E, cfg.H, cfg.F)
    raise ValueError(stream)


def tensor_dtype(cfg: MoEConfig, stream: int) -> str:
    return F32 if stream == STREAM_W_ROUTER else cfg.dtype


def host_tensor(cfg: MoEConfig, stream: int, first: int = 0, count: int | None = None) -> np.ndarray:
    """Slices [first, first+count) along the leading dimension of a tensor, as
    fp32 (dtype f32) or uint16 bf16 bit patterns (dtype bf16)."""
    shape = tensor_shape(cfg, stream)
    lead = shape[0]
    if count is None:
        count = lead - first
    inner = int(np.prod(shape[1:], dtype=np.int64))
    v = normal_f32(cfg.seed, stream, first * inner, count * inner, tensor_sigma(cfg, stream))
    if tensor_dtype(cfg, stream) == BF16:
        v = f32_to_bf16_bits(v)
    return v.reshape((count,) + shape[1:])


def popularity(cfg: MoEConfig) -> np.ndarray:
    """Target expert popularity p_e (sums to 1): uniform, or Zipf(s) over a
    seeded random ranking of the experts."""
    if cfg.zipf_s == 0.0:
        return np.full(cfg.E, 1.0 / cfg.E)
    order = np.argsort(raw_u64(cfg.seed, STREAM_RANK_PERM, 0, cfg.E), kind="stable")
    rank = np.empty(cfg.E, dtype=np.int64)
    rank[order] = np.arange(1, cfg.E + 1)
    p = rank.astype(np.float64) ** (-cfg.zipf_s)
    return p / p.sum()


def router_bias(cfg: MoEConfig) -> np.ndarray | None:
    """Per-expert logit bias that skews expert popularity: b_e = beta * ln(p_e / max p),
    beta = sqrt(6)/pi (the scale of a Gumbel whose variance matches the unit
    Gaussian logit noise).  None for uniform routing."""
    if cfg.zipf_s == 0.0 and cfg.bias_gain != 0.0:
        # a mild, graded skew: the experts' seeded ranks, centred and scaled to unit variance, times the
        # gain (imbalance sweeps search the gain that gives a wanted spread of the experts' token shares)
        order = np.argsort(raw_u64(cfg.seed, STREAM_RANK_PERM, 0, cfg.E), kind="stable")
        z = np.empty(cfg.E, dtype=np.float64)
        z[order] = np.arange(cfg.E, dtype=np.float64)
        z = (z - z.mean()) / (z.std() if cfg.E > 1 else 1.0)
        return (cfg.bias_gain * z).astype(np.float32)
    if cfg.zipf_s == 0.0:
        return None
    p = popularity(cfg)
    beta = math.sqrt(6.0) / math.pi
    return (beta * np.log(p / p.max())).astype(np.float32)


def recv_segment_counts(cfg: MoEConfig, M: int, g_local: int = 0) -> np.ndarray:
    """Row counts of the Eg local experts of destination g_local in a synthetic
    receive buffer of M rows: each row picks a local expert with probability
    proportional to the experts' popularity."""
    Eg = cfg.E // cfg.G
    p = popularity(cfg)[g_local * Eg:(g_local + 1) * Eg]
    cdf = np.cumsum(p / p.sum())
    u = (raw_u64(cfg.seed, STREAM_RECV_ASSIGN, 0, M) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))
    e = np.minimum(np.searchsorted(cdf, u, side="right"), Eg - 1)
    return np.bincount(e, minlength=Eg).astype(np.int32)
