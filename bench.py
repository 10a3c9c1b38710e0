#!/usr/bin/env python3
"""MoE-layer hot-path benchmark on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic tokens:
    moe_route -> moe_dispatch_layout -> moe_permute -> moe_ffn_schedule ->
    moe_ffn_gate_up -> moe_ffn_down -> moe_combine
all enqueued on one stream through the C ABI, inputs resident in HBM.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload dsv3] [--also a,b,c | --also none]
    python bench.py --sweep tokens      # Mixtral shape, 128 ... 32768 tokens
    python bench.py --sweep imbalance   # Mixtral shape, std of the experts' token shares 0 ... 0.05

Prints ONE JSON line.  Its top level is the main workload (by default the largest
single-GPU configuration, the DeepSeek-V3-shaped layer over all 256 experts): layer
tokens/s, the roofline of the dominant kernel (the gate/up grouped GEMM, timed live with
HIP events), the HBM rate of the permute and combine row moves, and the CPU oracle timed on
a bounded sample.  `also` holds the same measurements, in short, for the other workloads.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

WORKLOAD_TEXT = {
    "tiny": "Tiny MoE layer (fp32)",
    "mixtral": "Mixtral-8x7B-shaped layer",
    "gptoss": "gpt-oss-shaped layer, Zipf(1.0) expert popularity",
    "dsv3": "DeepSeek-V3-shaped routed layer, FFN over all 256 experts",
    "dsv3_ep": "one expert-parallel rank's share of a DeepSeek-V3-shaped layer (32 destinations, 8 local experts)",
    "qwen2moe": "Qwen2-MoE-2.7B-shaped layer (paper Table II)",
    "phi35moe": "Phi-3.5-MoE-shaped layer (paper Table II)",
}
DEFAULT_WORKLOAD = "dsv3"
DEFAULT_ALSO = "mixtral,gptoss,dsv3_ep,qwen2moe,phi35moe"
SWEEP_TOKENS = [128, 256, 512, 1024, 2048, 4096, 8192, 16384, 32768]
SWEEP_SHARE_STD = [0.0, 0.01, 0.02, 0.032, 0.04, 0.05]


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=list(WORKLOAD_TEXT))
    ap.add_argument("--also", default=None,
                    help="comma-separated workloads measured in short beside the main one ('none': no others; "
                         f"default: {DEFAULT_ALSO} when the main workload is {DEFAULT_WORKLOAD})")
    ap.add_argument("--sweep", default=None, choices=["tokens", "imbalance"],
                    help="emit a whole curve on the Mixtral shape under the key 'sweep' instead of 'also'")
    ap.add_argument("--tokens", type=int, default=0, help="override the workload's token count")
    ap.add_argument("--zipf", type=float, default=-1.0,
                    help="override the Zipf exponent of expert popularity (0 = uniform)")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip the HIP-graph replay of the step (one graph of all buffer sets' steps)")
    ap.add_argument("--ffn-split", action="store_true",
                    help="also time the two GEMMs over only the experts with more than 64 rows, and over only the "
                         "others (key 'ffn.split_by_expert_size')")
    ap.add_argument("--stream-probe", action="store_true",
                    help="also measure how fast 8 ... 256 workgroups, one per compute unit, stream a 4 GiB buffer from "
                         "memory into LDS (key 'stream_probe'): the per-compute-unit ceiling of weight streaming")
    ap.add_argument("--nbuf", type=int, default=0, help="activation buffer sets rotated per step (0 = auto)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target time of the oracle sample (0 = skip)")
    return ap.parse_args()


class Layer:
    """Device buffers of one workload and the step that walks the C ABI."""

    def __init__(self, cfg, nbuf):
        import torch
        import moe_inputs as mi
        import moe_inputs.device as mid
        import paper_2605_05888_amd as hub
        self.cfg, self.hub, self.torch = cfg, hub, torch
        dev = "cuda:0"
        dt = torch.bfloat16 if cfg.dtype == mi.BF16 else torch.float32
        self.code = hub.BF16 if cfg.dtype == mi.BF16 else hub.F32
        N, H, E, K, F, G = cfg.N, cfg.H, cfg.E, cfg.K, cfg.F, cfg.G
        R = N * K
        self.R = R
        self.ep = G > 1
        self.E_local = E // G
        # weights: router for all experts; expert weights for the experts this GPU computes
        self.W_r = mid.device_tensor(cfg, mi.STREAM_W_ROUTER)
        bias = mi.router_bias(cfg)
        self.bias = None if bias is None else mid.to_device(bias)
        self.W_gate = mid.device_tensor(cfg, mi.STREAM_W_GATE, 0, self.E_local)
        self.W_up = mid.device_tensor(cfg, mi.STREAM_W_UP, 0, self.E_local)
        self.W_down = mid.device_tensor(cfg, mi.STREAM_W_DOWN, 0, self.E_local)
        x0 = mid.device_tensor(cfg, mi.STREAM_X)
        self.sets = []
        i32 = dict(dtype=torch.int32, device=dev)
        ffn_ws = hub.workspace_bytes(hub.OP_GROUPED_FFN, N=R, H=H, E=self.E_local, F=F, dtype=self.code)
        for i in range(nbuf):
            s = dict(
                x=x0 if i == 0 else x0.clone(),
                idx=torch.empty((N, K), **i32), w=torch.empty((N, K), dtype=torch.float32, device=dev),
                cnt=torch.empty(E, **i32), off=torch.empty(E + 1, **i32),
                dcnt=torch.empty(G, **i32), doff=torch.empty(G + 1, **i32),
                slot=torch.empty(R, **i32), row=torch.empty(R, **i32),
                xp=torch.empty((R, H), dtype=dt, device=dev), y=torch.empty((R, H), dtype=dt, device=dev),
                out=torch.empty((N, H), dtype=dt, device=dev),
                ffn_ws=torch.empty(ffn_ws, dtype=torch.uint8, device=dev))
            self.sets.append(s)
        self.route_ws = torch.empty(hub.workspace_bytes(hub.OP_ROUTE, N=N, E=E), dtype=torch.uint8, device=dev)
        self.layout_ws = torch.empty(max(16, hub.workspace_bytes(hub.OP_DISPATCH_LAYOUT, N=N, E=E, K=K, G=G)),
                                     dtype=torch.uint8, device=dev)
        if self.ep:
            # what the peers would send: R rows for the local experts, split by their popularity
            self.recv = mid.fill_normal(torch.empty((R, H), dtype=dt, device=dev), cfg.seed, mi.STREAM_RECV_X, 0, 1.0)
            import numpy as np
            c = mi.recv_segment_counts(cfg, R, 0)
            seg = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
            self.recv_seg = mid.to_device(seg)
        self.sums = None
        self.names = ["route", "layout", "permute", "ffn_schedule", "ffn_gate_up", "ffn_down", "combine"]

    def set_bias(self, bias):
        import moe_inputs.device as mid
        self.bias = None if bias is None else mid.to_device(bias)

    def step(self, i, events=None, fused_gather=False, fused_combine=False, one_launch=False):
        """One pass of the layer.  one_launch: both GEMMs of the expert computation in one kernel, the second
        consuming the first's rows as they arrive (the `ffn_gate_up` event pair then brackets that kernel and
        `ffn_down` is empty).  fused_gather (single-device layers only): no permute; the gate/up GEMM
        fetches its rows from x through row_of_slot.  fused_combine: no y and no combine step; the down
        GEMM adds its gate-weighted rows into the tokens' fp32 sums."""
        hub, cfg = self.hub, self.cfg
        s = self.sets[i % len(self.sets)]
        rec = (lambda j: events[j].record()) if events is not None else (lambda j: None)
        rec(0)
        hub.moe_route(s["x"], self.W_r, self.bias, cfg.K, cfg.score_mode, s["idx"], s["w"], None, self.route_ws)
        rec(1)
        hub.moe_dispatch_layout(s["idx"], cfg.E, cfg.G, s["cnt"], s["off"], s["dcnt"], s["doff"], s["slot"],
                                s["row"], self.layout_ws)
        rec(2)
        if not fused_gather:
            hub.moe_permute(s["x"], cfg.K, s["slot"], s["row"], s["xp"])
        rec(3)
        if self.ep:
            ffn_in, seg = self.recv, self.recv_seg
        else:
            ffn_in, seg = s["xp"], s["off"]
        hub.moe_ffn_schedule(self.code, self.R, cfg.H, cfg.F, seg, s["ffn_ws"])
        rec(4)
        if one_launch:
            hub.moe_ffn_gate_up_down(ffn_in, seg, self.W_gate, self.W_up, self.W_down, s["y"], s["ffn_ws"])
        elif fused_gather:
            hub.moe_ffn_gate_up_gather(s["x"], cfg.K, seg, s["row"], self.W_gate, self.W_up, s["ffn_ws"])
        else:
            hub.moe_ffn_gate_up(ffn_in, seg, self.W_gate, self.W_up, s["ffn_ws"])
        rec(5)
        if one_launch:
            rec(6)
            hub.moe_combine(s["y"], cfg.K, s["slot"], s["w"], s["out"])
        elif fused_combine:
            if self.sums is None:
                self.sums = self.torch.empty((cfg.N, cfg.H), dtype=self.torch.float32, device="cuda:0")
            hub.moe_ffn_down_combine(cfg.K, seg, self.W_down, s["row"], s["w"], self.sums, s["out"], s["ffn_ws"])
            rec(6)
        else:
            hub.moe_ffn_down(seg, self.W_down, s["y"], s["ffn_ws"])
            rec(6)
            hub.moe_combine(s["y"], cfg.K, s["slot"], s["w"], s["out"])
        rec(7)


def cpu_baseline(cfg, layer, target_seconds):
    """The oracle, as it stands, on a bounded sample of the same workload: a mini-batch of S tokens
    through the whole layer (every expert the sample's rows reach, full H and F).  tokens/s = S / time
    spent inside the oracle.  Expert weights are copied back from HBM one expert at a time, outside the
    timed parts (the layer's weights need not fit host memory twice)."""
    import numpy as np
    import moe_inputs as mi
    import moe_inputs.device as mid
    import oracle
    Wr = mid.to_host(layer.W_r)
    bias = None if layer.bias is None else mid.to_host(layer.bias)
    E_run = layer.E_local if layer.ep else cfg.E
    x_all = mid.to_host(layer.sets[0]["x"])

    def run(S):
        x = x_all[:S]
        t0 = time.perf_counter()
        idx, w, _ = oracle.route(x, Wr, bias, cfg.K, cfg.score_mode)
        lay = oracle.layout(idx, cfg.E, cfg.G)
        xp = oracle.permute(x, cfg.K, lay["slot_of_row"])
        spent = time.perf_counter() - t0
        if layer.ep:   # the local experts see S*K received rows, split as in the GPU run
            c = mi.recv_segment_counts(cfg, S * cfg.K, 0)
            seg = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
        else:
            seg = lay["expert_offsets"]
        y = np.zeros((S * cfg.K, cfg.H), dtype=np.float64)
        for e in range(E_run):
            lo, hi = int(seg[e]), int(seg[e + 1])
            if hi == lo:
                continue
            We = [mid.to_host(W[e:e + 1]) for W in (layer.W_gate, layer.W_up, layer.W_down)]
            t0 = time.perf_counter()
            y[lo:hi] = oracle.ffn_rows(xp, np.array([lo, hi], np.int32), *We, rows=np.arange(lo, hi))
            spent += time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.combine(y, cfg.K, lay["slot_of_row"], w)
        return spent + time.perf_counter() - t0

    # first a sample large enough for every expert's rows to occupy the host's threads, then one scaled
    # to the target time
    S = int(min(cfg.N, max(16, 16 * E_run // cfg.K)))
    t = run(S)
    S2 = int(min(cfg.N, S * target_seconds / max(t, 1e-3)))
    if S2 > S * 1.5:
        S, t = S2, run(S2)
    return {"value": S / t, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{S} of {cfg.N} tokens through the whole layer (route, layout, permute, fp64 SwiGLU FFN "
                      f"over the {E_run} experts at full H and F, combine); {t:.1f} s of wall time inside the "
                      f"oracle on {oracle.num_threads()} threads"}


def profiled_traffic(workload, kernel):
    """HBM bytes per launch as read from rocprofv3 counters in an earlier, committed run
    (profiles/*_hbm_traffic.md); not measured by this run.  None if there is no such summary."""
    import glob
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*_hbm_traffic.md"))):
        for line in open(path):
            t = line.split()
            if len(t) == 4 and t[0] == "traffic_bytes" and t[1] == workload and t[2] == kernel:
                return float(t[3]), os.path.relpath(path, ROOT)
    return None, None


def time_layer(layer, steps, warmup, **variant):
    """ms per step from the host clock around `steps` steps, and the mean HIP-event time of every call."""
    import torch
    for i in range(warmup):
        layer.step(i, **variant)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(8)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        layer.step(i, ev[i], **variant)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    us = {n: sum(e[j].elapsed_time(e[j + 1]) for e in ev) * 1e3 / steps for j, n in enumerate(layer.names)}
    return ms, us


def summarise(cfg, layer, ms_per_step, us):
    """The figures every workload reports."""
    import moe_inputs as mi
    N, H, K, F = cfg.N, cfg.H, cfg.K, cfg.F
    R, b = N * K, cfg.elt_bytes
    flops_gu, flops_dn = 4.0 * R * H * F, 2.0 * R * H * F      # gate and up projections; down projection
    t_gu, t_dn = us["ffn_gate_up"] * 1e-6, us["ffn_down"] * 1e-6
    move_bytes = N * H * b + R * H * b          # permute: read x once, write xp; combine: the mirror image
    gbs_perm = (move_bytes + 4 * R) / (us["permute"] * 1e-6) / 1e9
    gbs_comb = (move_bytes + 8 * R) / (us["combine"] * 1e-6) / 1e9
    cnt = layer.sets[0]["cnt"].cpu().numpy().astype("float64")
    return {
        "ms_per_step": ms_per_step, "tokens_per_s": N / (ms_per_step * 1e-3),
        "gate_up_tflops": flops_gu / t_gu / 1e12, "gate_up_mfma_frac": flops_gu / t_gu / 1e12 / PEAK_BF16_TFLOPS,
        "down_tflops": flops_dn / t_dn / 1e12, "down_mfma_frac": flops_dn / t_dn / 1e12 / PEAK_BF16_TFLOPS,
        "ffn_mfma_frac": (flops_gu + flops_dn) / (t_gu + t_dn) / 1e12 / PEAK_BF16_TFLOPS,
        "permute_GBs": gbs_perm, "permute_hbm_frac": gbs_perm / PEAK_HBM_GBS,
        "combine_GBs": gbs_comb, "combine_hbm_frac": gbs_comb / PEAK_HBM_GBS,
        "step_breakdown_us": us,
        "routing": {"zipf_s": cfg.zipf_s, "rows_per_expert_min": int(cnt.min()), "rows_per_expert_max": int(cnt.max()),
                    "std_of_expert_share": float((cnt / max(cnt.sum(), 1.0)).std())},
        "dtype": "bf16" if cfg.dtype == mi.BF16 else "f32",
    }


def graph_replay(layer, steps):
    """The same steps captured once in a HIP graph and replayed: what a serving loop would do with a
    launch-bound layer.  Every replay is checked against the eager result (the kernels are deterministic, so
    bit for bit), with eager work and synchronisation between the replays."""
    import torch
    N = layer.cfg.N
    for i in range(len(layer.sets)):
        layer.step(i)
    eager_out = [st["out"].clone() for st in layer.sets]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        for i in range(len(layer.sets)):
            layer.step(i)                      # warm every buffer set on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            for i in range(len(layer.sets)):
                layer.step(i)
    torch.cuda.current_stream().wait_stream(side)
    reps = max(1, steps // len(layer.sets))
    same = True
    for rnd in range(3):
        for st in layer.sets:
            st["out"].zero_()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        same = same and all(torch.equal(st["out"], e) for st, e in zip(layer.sets, eager_out))
        layer.step(0)
    torch.cuda.synchronize()
    g_ms = (t1 - t0) * 1e3 / (reps * len(layer.sets))
    del graph
    return {"ms_per_step": g_ms, "tokens_per_s": N / (g_ms * 1e-3), "steps_per_graph": len(layer.sets),
            "replays_timed": reps, "matches_eager_bitwise": bool(same)}


def ffn_split(layer, cfg, light_rows=64, reps=20):
    """GEMM times (HIP events, mean of `reps` launches after 3 untimed ones) with the realised expert counts, with
    only the experts above `light_rows` rows, and with only the others; rows and weights are the layer's own."""
    import numpy as np
    import torch
    hub = layer.hub
    s0 = layer.sets[0]
    counts = s0["cnt"].cpu().numpy().astype(np.int64)
    H, F = cfg.H, cfg.F
    out = {"light_rows_max": light_rows}
    for tag, c in (("all", counts), ("heavy_only", np.where(counts > light_rows, counts, 0)),
                   ("light_only", np.where(counts <= light_rows, counts, 0))):
        M = int(c.sum())
        if M == 0:
            continue
        seg = torch.tensor(np.concatenate([[0], np.cumsum(c)]).astype(np.int32), device="cuda:0")
        hub.moe_ffn_schedule(layer.code, M, H, F, seg, s0["ffn_ws"])
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        for timed in (False, True):
            n = reps if timed else 3
            if timed:
                ev[0].record()
            for _ in range(n):
                hub.moe_ffn_gate_up(s0["xp"][:M], seg, layer.W_gate, layer.W_up, s0["ffn_ws"])
            if timed:
                ev[1].record()
            for _ in range(n):
                hub.moe_ffn_down(seg, layer.W_down, s0["y"][:M], s0["ffn_ws"])
        ev[2].record()
        torch.cuda.synchronize()
        t1, t2 = ev[0].elapsed_time(ev[1]) * 1e3 / reps, ev[1].elapsed_time(ev[2]) * 1e3 / reps
        n_exp = int((c > 0).sum())
        out[tag] = {"rows": M, "experts": n_exp, "gate_up_us": t1, "down_us": t2,
                    "gate_up_tflops": 4.0 * M * H * F / t1 / 1e6, "down_tflops": 2.0 * M * H * F / t2 / 1e6,
                    "gate_up_weight_GBs": n_exp * 2.0 * F * H * 2 / t1 / 1e3, "down_weight_GBs": n_exp * F * H * 2.0 / t2 / 1e3}
    # leave the layer's own schedule behind
    hub.moe_ffn_schedule(layer.code, layer.R, H, F, s0["off"], s0["ffn_ws"])
    return out


def pick_nbuf(cfg, nbuf_arg):
    N, H, K, F, b = cfg.N, cfg.H, cfg.K, cfg.F, cfg.elt_bytes
    act_bytes = (2 * N * H + 2 * N * K * H + N * K * F) * b
    return nbuf_arg or (4 if act_bytes < (1 << 30) else 1)   # rotate small working sets out of the 256 MB cache


def short_run(name, cfg, steps, warmup, nbuf_arg, graph=True):
    """One workload measured in short (the entries of `also` and of the sweeps)."""
    import torch
    nbuf = pick_nbuf(cfg, nbuf_arg)
    layer = Layer(cfg, nbuf)
    torch.cuda.synchronize()
    ms, us = time_layer(layer, steps, warmup)
    out = summarise(cfg, layer, ms, us)
    if out["dtype"] == "bf16":
        o_ms, o_us = time_layer(layer, steps, min(3, warmup), one_launch=True)
        out["ffn_one_launch"] = {"ms_per_step": o_ms, "ffn_us": o_us["ffn_gate_up"]}
    if graph:
        g = graph_replay(layer, steps)
        out["graph"] = {k: g[k] for k in ("ms_per_step", "tokens_per_s", "matches_eager_bitwise")}
    out["config"] = {"workload": f"{name}: {WORKLOAD_TEXT.get(name, name)}", "N": cfg.N, "H": cfg.H, "E": cfg.E,
                     "K": cfg.K, "F": cfg.F, "G": cfg.G, "activation_buffer_sets": nbuf}
    del layer
    torch.cuda.empty_cache()
    return out


def imbalance_point(base_cfg, target_std, steps, warmup, nbuf_arg):
    """Mixtral shape with the experts' logits biased along a fixed seeded pattern; the gain of the bias is
    searched (bisection over route + layout on the GPU) until the realised standard deviation of the
    experts' token shares is the target."""
    import torch
    import moe_inputs as mi
    nbuf = pick_nbuf(base_cfg, nbuf_arg)
    layer = Layer(base_cfg, nbuf)

    def realised(gain):
        cfg = dataclasses.replace(base_cfg, bias_gain=gain)
        layer.set_bias(mi.router_bias(cfg))
        layer.step(0)
        torch.cuda.synchronize()
        cnt = layer.sets[0]["cnt"].cpu().numpy().astype("float64")
        return float((cnt / cnt.sum()).std())

    lo, hi = 0.0, 4.0
    gain = 0.0
    if target_std > 0:
        for _ in range(24):
            gain = 0.5 * (lo + hi)
            if realised(gain) < target_std:
                lo = gain
            else:
                hi = gain
    got = realised(gain)
    cfg = dataclasses.replace(base_cfg, bias_gain=gain)
    ms, us = time_layer(layer, steps, warmup)
    out = summarise(cfg, layer, ms, us)
    out["target_std_of_expert_share"] = target_std
    out["bias_gain"] = gain
    assert abs(out["routing"]["std_of_expert_share"] - got) < 1e-9
    del layer
    torch.cuda.empty_cache()
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; there is no multi-GPU path to time "
              f"(--gpus {args.gpus} refused).", file=sys.stderr)
        sys.exit(2)
    import torch
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    import moe_inputs as mi
    import paper_2605_05888_amd as hub
    hub.load_library(build_if_missing=False)     # fail loudly if the HIP library is not built
    cfg = mi.CONFIGS[args.workload]
    if args.tokens > 0:
        cfg = dataclasses.replace(cfg, N=args.tokens)
    if args.zipf >= 0:
        cfg = dataclasses.replace(cfg, zipf_s=args.zipf)
    N, H, E, K, F, G = cfg.N, cfg.H, cfg.E, cfg.K, cfg.F, cfg.G
    R = N * K
    nbuf = pick_nbuf(cfg, args.nbuf)
    layer = Layer(cfg, nbuf)
    torch.cuda.synchronize()

    ms_per_step, us = time_layer(layer, args.steps, args.warmup)
    m = summarise(cfg, layer, ms_per_step, us)
    flops_gu = 4.0 * R * H * F
    t_gu = us["ffn_gate_up"] * 1e-6
    traffic, traffic_src = profiled_traffic(args.workload, "ffn_gate_up")
    result = {
        "metric": "moe_layer_tokens_per_s", "value": m["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": m["dtype"], "data": "synthetic",
        "config": {"workload": f"{args.workload}: {WORKLOAD_TEXT[args.workload]}", "N": N, "H": H, "E": E, "K": K,
                   "F": F, "G": G, "routed_rows": R, "activation_buffer_sets": nbuf, "routing": m["routing"]},
        "roofline": {"kernel": "grouped_gemm_bf16 (gate/up projection with fused SwiGLU)", "bound": "mfma",
                     "achieved": m["gate_up_tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": m["gate_up_mfma_frac"], "flops_per_launch": flops_gu,
                     "avg_launch_us": us["ffn_gate_up"],
                     # bytes per launch from rocprofv3 counters of an earlier run of this command (see the file)
                     "traffic": traffic, "traffic_from_committed_profile": traffic_src},
        "ffn": {"tflops_gate_up": m["gate_up_tflops"], "tflops_down": m["down_tflops"],
                "mfma_frac_gate_up": m["gate_up_mfma_frac"], "mfma_frac_down": m["down_mfma_frac"],
                "mfma_frac_both": m["ffn_mfma_frac"]},
        "dispatch_combine": {"permute_GBs": m["permute_GBs"], "combine_GBs": m["combine_GBs"],
                             "peak_GBs": PEAK_HBM_GBS, "permute_frac": m["permute_hbm_frac"],
                             "combine_frac": m["combine_hbm_frac"]},
        "step_breakdown_us": us,
    }
    # Address resolution alone, stable order against arrival order (atomic row pointers), same inputs.
    st0 = layer.sets[0]
    reps = 20
    la = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    for timed in (False, True):
        if timed:
            la[0].record()
        for _ in range(reps):
            hub.moe_dispatch_layout(st0["idx"], E, G, st0["cnt"], st0["off"], st0["dcnt"], st0["doff"], st0["slot"],
                                    st0["row"], layer.layout_ws)
        if timed:
            la[1].record()
        for _ in range(reps):
            hub.moe_dispatch_layout_arrival(st0["idx"], E, G, st0["cnt"], st0["off"], st0["dcnt"], st0["doff"],
                                            st0["slot"], st0["row"])
        if timed:
            la[2].record()
    # leave the stable layout in the buffers for what follows
    hub.moe_dispatch_layout(st0["idx"], E, G, st0["cnt"], st0["off"], st0["dcnt"], st0["doff"], st0["slot"],
                            st0["row"], layer.layout_ws)
    torch.cuda.synchronize()
    result["layout_order"] = {"stable_us": la[0].elapsed_time(la[1]) * 1e3 / reps,
                              "arrival_us": la[1].elapsed_time(la[2]) * 1e3 / reps}
    # Routing with the row pointers drawn in the top-K kernel, against routing followed by either layout.
    lr = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for timed in (False, True):
        if timed:
            lr[0].record()
        for _ in range(reps):
            hub.moe_route(st0["x"], layer.W_r, layer.bias, K, cfg.score_mode, st0["idx"], st0["w"], None, layer.route_ws)
            hub.moe_dispatch_layout(st0["idx"], E, G, st0["cnt"], st0["off"], st0["dcnt"], st0["doff"], st0["slot"],
                                    st0["row"], layer.layout_ws)
        if timed:
            lr[1].record()
        for _ in range(reps):
            hub.moe_route(st0["x"], layer.W_r, layer.bias, K, cfg.score_mode, st0["idx"], st0["w"], None, layer.route_ws)
            hub.moe_dispatch_layout_arrival(st0["idx"], E, G, st0["cnt"], st0["off"], st0["dcnt"], st0["doff"],
                                            st0["slot"], st0["row"])
        if timed:
            lr[2].record()
        for _ in range(reps):
            hub.moe_route_resolve_arrival(st0["x"], layer.W_r, layer.bias, K, G, cfg.score_mode, st0["idx"], st0["w"],
                                          st0["cnt"], st0["off"], st0["dcnt"], st0["doff"], st0["slot"], st0["row"],
                                          None, layer.route_ws)
    lr[3].record()
    hub.moe_dispatch_layout(st0["idx"], E, G, st0["cnt"], st0["off"], st0["dcnt"], st0["doff"], st0["slot"],
                            st0["row"], layer.layout_ws)
    torch.cuda.synchronize()
    result["layout_order"].update({"route_then_stable_us": lr[0].elapsed_time(lr[1]) * 1e3 / reps,
                                   "route_then_arrival_us": lr[1].elapsed_time(lr[2]) * 1e3 / reps,
                                   "route_resolve_arrival_us": lr[2].elapsed_time(lr[3]) * 1e3 / reps})
    # Both GEMMs in one launch, the down projection's tiles starting as their rows arrive (the dependency-driven
    # form): same bits; reported beside the layer, not as `value`.
    if cfg.dtype == mi.BF16:
        o_ms, o_us = time_layer(layer, args.steps, min(3, args.warmup), one_launch=True)
        result["ffn_one_launch"] = {"ms_per_step": o_ms, "tokens_per_s": N / (o_ms * 1e-3), "ffn_us": o_us["ffn_gate_up"],
                                    "ffn_us_two_launches": us["ffn_gate_up"] + us["ffn_down"],
                                    "mfma_frac_both": 6.0 * R * H * F / (o_us["ffn_gate_up"] * 1e-6) / 1e12 / PEAK_BF16_TFLOPS}
    if not layer.ep:
        # Variant without a dispatch row move (a single device that computes every expert needs no send
        # buffer): the gate/up GEMM gathers its rows from x.  Reported beside the layer, not as `value`.
        f_ms, f_us = time_layer(layer, args.steps, min(3, args.warmup), fused_gather=True)
        result["fused_gather"] = {"ms_per_step": f_ms, "tokens_per_s": N / (f_ms * 1e-3),
                                  "gate_up_us": f_us["ffn_gate_up"],
                                  "tflops_gate_up": flops_gu / (f_us["ffn_gate_up"] * 1e-6) / 1e12}
        # Both halves fused (no permute, no y, no combine step): the layer without data-shuffling steps.
        if cfg.dtype == mi.BF16:
            n_fc = max(2, args.steps // 5)          # (an atomic per element: several times slower)
            s_ms, s_us = time_layer(layer, n_fc, 1, fused_gather=True, fused_combine=True)
            result["fused_gather_and_combine"] = {
                "ms_per_step": s_ms, "tokens_per_s": N / (s_ms * 1e-3), "steps": n_fc,
                "down_and_combine_us": s_us["ffn_down"],
                "down_plus_combine_us_unfused": us["ffn_down"] + us["combine"]}
            layer.sums = None
    if not args.no_graph:
        result["graph"] = graph_replay(layer, args.steps)
    # achievable matrix rate of this box with this kernel: the gate/up GEMM over equal, tile-aligned segments
    M_even = (R // layer.E_local) // 256 * 256
    if M_even > 0 and cfg.dtype == mi.BF16:
        seg_even = (torch.arange(layer.E_local + 1, dtype=torch.int32, device="cuda:0") * M_even).contiguous()
        s0 = layer.sets[0]
        src = layer.recv if layer.ep else s0["xp"]
        rows = M_even * layer.E_local
        hub.moe_ffn_schedule(layer.code, rows, H, F, seg_even, s0["ffn_ws"])
        reps = max(3, min(20, int(30e-3 / max(t_gu, 1e-6))))      # about 30 ms of launches, untimed, then the same again
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for timed in (False, True):
            if timed:
                g0.record()
            for _ in range(reps):
                hub.moe_ffn_gate_up(src[:rows], seg_even, layer.W_gate, layer.W_up, s0["ffn_ws"])
        g1.record()
        torch.cuda.synchronize()
        result["ffn"]["tflops_gate_up_equal_segments"] = reps * 4.0 * rows * H * F / (g0.elapsed_time(g1) * 1e-3) / 1e12
    # Which experts cost what: the two GEMMs over all experts, over those with more than 64 rows only (tiles that
    # are bound by the matrix cores) and over the others only (tiles that stream their weights once for a few rows).
    if args.ffn_split and cfg.dtype == mi.BF16 and not layer.ep:
        result["ffn"]["split_by_expert_size"] = ffn_split(layer, cfg)
    # achievable copy bandwidth of this machine: plain 1 GiB device-to-device copy (read + write bytes)
    import moe_inputs.device as mid
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    mid.copy_bytes(dst, src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        mid.copy_bytes(dst, src)
    c1.record()
    torch.cuda.synchronize()
    result["dispatch_combine"]["plain_copy_GBs"] = 5 * 2 * (1 << 30) / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del src, dst
    if args.stream_probe:
        buf = torch.empty(4 << 30, dtype=torch.uint8, device="cuda:0")
        buf.fill_(1)
        pts = []
        for wgs in (8, 32, 64, 128, 256):
            best = None
            for _ in range(3):
                c0.record()
                nbytes = mid.stream_read(buf, wgs, row_bytes=2 * cfg.H)
                c1.record()
                torch.cuda.synchronize()
                t = c0.elapsed_time(c1) * 1e-3
                best = t if best is None or t < best else best
            pts.append({"workgroups": wgs, "GBs": nbytes / best / 1e9, "GBs_per_workgroup": nbytes / best / 1e9 / wgs})
        result["stream_probe"] = {"what": "buffer loads into LDS, rows of 2*H bytes, 32 KB in flight per workgroup, no reuse",
                                  "points": pts}
        del buf
    if args.cpu_seconds > 0:
        result["cpu_baseline"] = cpu_baseline(cfg, layer, args.cpu_seconds)
    del layer, st0
    torch.cuda.empty_cache()

    # ---- the other workloads, in short (same steps and warm-up, same measurements)
    if args.sweep is None:
        also = args.also
        if also is None:
            also = DEFAULT_ALSO if (args.workload == DEFAULT_WORKLOAD and args.tokens == 0 and args.zipf < 0) else "none"
        names = [n for n in also.split(",") if n and n != "none" and n != args.workload]
        if names:
            result["also"] = {n: short_run(n, mi.CONFIGS[n], args.steps, args.warmup, args.nbuf, not args.no_graph)
                              for n in names}
    elif args.sweep == "tokens":
        base = mi.CONFIGS["mixtral"]
        result["sweep"] = {"what": "token count on the Mixtral shape (the axis of the paper's Fig. 13)", "points": [
            dict(tokens=n, **short_run("mixtral", dataclasses.replace(base, N=n), args.steps, args.warmup, args.nbuf,
                                       not args.no_graph))
            for n in SWEEP_TOKENS]}
    else:
        base = mi.CONFIGS["mixtral"]
        result["sweep"] = {"what": "standard deviation of the experts' token shares on the Mixtral shape "
                                   "(the axis of the paper's Fig. 14)",
                           "points": [imbalance_point(base, s, args.steps, args.warmup, args.nbuf)
                                      for s in SWEEP_SHARE_STD]}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
