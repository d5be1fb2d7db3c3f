#!/usr/bin/env python3
"""Decode-step benchmark of the KVSwap hot path on one MI355X.

A "step" is one pass of the whole path (low-rank prediction over K_lr, group max,
top-M groups, attention over the gathered groups) for one batch of one layer
(all 36 layers for the c5 workload), on seeded synthetic tensors that are already
resident in HBM.  Steps rotate over several independent copies of the inputs so
that the working set of consecutive steps exceeds the on-chip caches (the 32K,
batch-1 working set alone would fit the 256 MB last-level cache).

    python bench.py --gpus 1 --steps K --warmup W [--config c4] [--extra c1,c2,c3,c5] [--mode graph|eager]

prints ONE JSON line.  The headline workload (default c4, the largest single-layer one:
128K context, batch 4) gives tokens/s (= batch / step latency) as `value`, the latency
itself in `ms_per_step` / `us_per_layer`, a `roofline` object for the dominant kernel
(algorithmic bytes / measured kernel time against 8 TB/s) and a `cpu_baseline` object (the
fp64 CPU oracle timed on this machine's host cores).  The other workloads follow under
`other_workloads`, each with its own latency, roofline and cpu_baseline: c1 (4K, fp32:
microseconds only), c2 and c3 (32K context, batch 1 and 8) and c5 (a whole 36-layer stack
per step, batch 16, replayed as one captured graph).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
METRIC = "decode step latency (µs/layer) + tokens/s; achieved HBM GB/s vs 8 TB/s peak"
CACHE_BYTES = 256e6 + 32e6     # last-level cache + the eight L2s


# --------------------------------------------------------------------------------------
# algorithmic bytes: what the method itself has to move per layer-step
# --------------------------------------------------------------------------------------
def algorithmic_bytes(cfg, meta_bytes: int = None) -> dict:
    """meta_bytes: bytes per element of K_lr (default: those of the workload's dtype)."""
    P = cfg.batch * cfg.n_kv_heads
    S = cfg.batch if cfg.joint else P      # selection sets: one K_lr, one score row, one idx each
    eb = cfg.elem_bytes
    NG, M = cfg.n_groups, cfg.n_select
    q_bytes = cfg.batch * cfg.n_q_heads * cfg.head_dim * eb
    a_bytes = cfg.n_kv_heads * cfg.head_dim * cfg.rank * 4
    predict = S * cfg.ctx_len * cfg.rank * (meta_bytes or eb) + q_bytes + a_bytes + S * NG * 4
    topk = S * NG * 4 + S * M * 4
    attn = S * M * 4 + 2 * P * M * cfg.group_size * cfg.head_dim * eb + q_bytes + q_bytes
    return {"predict": predict, "topk": topk, "attn": attn, "step": predict + topk + attn}


# --------------------------------------------------------------------------------------
# workload: device-resident rotating copies
# --------------------------------------------------------------------------------------
class Workload:
    def __init__(self, cfg, copies: int, log=print, meta: str = None):
        import torch
        import paper_2511_11907_amd as kv
        from workloads import make_layer

        self.cfg, self.kv, self.torch = cfg, kv, torch
        dev = "cuda:0"
        code = kv.KVS_F32 if cfg.dtype == "f32" else kv.KVS_BF16
        tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
        # 8-bit metadata: stored as K.A / 8 so that the heavy hitters stay inside the format
        mcode, mscale, mdt = (kv.KVS_FP8_E4M3, 0.125, torch.float8_e4m3fn) if meta == "fp8" else (code, 0.0, tdt)
        self.p = kv.Params(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.rank,
                           cfg.ctx_len, cfg.group_size, cfg.n_select, code, mcode, meta_scale=mscale,
                           head_mode=kv.KVS_HEADS_JOINT if cfg.joint else kv.KVS_HEADS_SEPARATE)
        self.ws = torch.empty(kv.kvs_workspace_bytes(self.p) // 4, dtype=torch.float32, device=dev)
        kv.kvs_workspace_init(self.p, self.ws)
        self.slots = []
        self.host0 = None
        B, Hk, N = cfg.batch, cfg.n_kv_heads, cfg.ctx_len

        def up(x):
            import numpy as np
            if x.dtype == np.uint16:
                return torch.from_numpy(x.view(np.int16)).to(dev).view(torch.bfloat16)
            return torch.from_numpy(x).to(dev)

        # c5: the copies ARE the 36 layers (distinct adapters); otherwise independent
        # sequences of layer 0 that share layer 0's adapter
        per_layer = cfg.layers > 1
        n = cfg.layers if per_layer else copies
        A0 = None
        t0 = time.time()
        for c in range(n):
            if per_layer:
                L = make_layer(cfg, layer=c, workers=16)
            else:
                L = make_layer(cfg, layer=0, workers=16, seq_offset=c * B, adapter_from=A0)
                A0 = L.A
            s = {"K": up(L.K), "V": up(L.V), "q": up(L.q), "A": up(L.A)}
            sets = self.p.sets
            s["K_lr"] = torch.empty(sets + (N, cfg.rank), dtype=mdt, device=dev)
            kv.kvs_build_metadata(self.p, s["K"], s["A"], s["K_lr"])
            s["idx"] = torch.empty(sets + (cfg.n_select,), dtype=torch.int32, device=dev)
            s["gs"] = torch.empty(sets + (cfg.n_groups,), dtype=torch.float32, device=dev)
            s["out"] = torch.empty((B, cfg.n_q_heads, cfg.head_dim), dtype=tdt, device=dev)
            # a workspace of its own, so that layer-steps in flight together do not share one
            s["ws"] = torch.empty_like(self.ws)
            kv.kvs_workspace_init(self.p, s["ws"])
            self.slots.append(s)
            if c == 0:
                self.host0 = L
            del L
        torch.cuda.synchronize()
        log(f"[bench] {cfg.name}: {n} input copies resident ({time.time() - t0:.1f}s to generate)")
        self.layers_per_step = cfg.layers if per_layer else 1

    # one layer-step on slot i through the single fused entry point
    def layer_step(self, i: int):
        s = self.slots[i % len(self.slots)]
        step = self.kv.kvs_decode_step_single_launch if getattr(self, "single_launch", False) else self.kv.kvs_decode_step
        step(self.p, s["q"], s["K_lr"], s["A"], s["K"], s["V"], s["idx"], None, s["out"], self.ws)

    def step(self, i: int):
        if self.layers_per_step == 1:
            self.layer_step(i)
        else:
            for l in range(self.layers_per_step):
                self.layer_step(l)

    def pipelined_in_two_launches(self) -> bool:
        """Whether kvs_attend_select_next covers this workload's layout (bf16, d = 128, 3..8
        query heads per KV head, at most 16384 groups per selection set)."""
        c = self.cfg
        return (c.dtype != "f32" and c.head_dim == 128 and 3 <= c.n_q_heads // c.n_kv_heads <= 8
                and c.n_groups <= 16384)

    def run(self, count: int, layer_ahead: bool = False):
        """`count` steps on the current stream.  With `layer_ahead`, the layer-steps are
        issued the way the method's runtime pipelines them (Sec. 3.3, 3.4: the groups of
        layer i+1 are predicted while layer i is still computing, from a query known one
        layer early).  Where kvs_attend_select_next covers the layout that is two launches
        per layer on ONE stream - the prediction of layer i+1, then the attention of layer i
        together with the selection of layer i+1 - with the ordinary calls at both ends, so
        that `count` steps still hold exactly `count` predictions, selections and
        attentions.  Elsewhere (fp32, d = 64): prediction, selection and attention each on
        a stream of their own, chained per layer by events, forked from and joined to the
        current stream so that the whole thing can be captured into a graph."""
        if not layer_ahead:
            for i in range(count):
                self.step(i)
            return
        torch, kv, p = self.torch, self.kv, self.p
        n = count * self.layers_per_step
        if self.pipelined_in_two_launches():
            ws = self.ws
            slot = lambda j: self.slots[j % len(self.slots)]
            s = slot(0)
            kv.kvs_predict_select(p, s["q"], s["K_lr"], s["A"], s["idx"], None, ws)
            for j in range(n):
                s = slot(j)
                if j + 1 < n:
                    t = slot(j + 1)
                    # (no workspace, i.e. no score histogram handed to the selection: hidden behind
                    # the attention the selection gains nothing from it, and the prediction kernel
                    # saves the atomics; joint-head mode keeps its low-rank queries there)
                    kv.kvs_predict_scores(p, t["q"], t["K_lr"], t["A"], t["gs"], ws if self.cfg.joint else None)
                    kv.kvs_attend_select_next(p, s["q"], s["K"], s["V"], s["idx"], s["out"], t["gs"], t["idx"], ws)
                else:
                    kv.kvs_sparse_decode_attn(p, s["q"], s["K"], s["V"], s["idx"], s["out"], ws)
            return
        main = torch.cuda.current_stream()
        if not hasattr(self, "side"):
            self.side = (torch.cuda.Stream(), torch.cuda.Stream())
        s_sel, s_att = self.side
        s_sel.wait_stream(main)
        s_att.wait_stream(main)
        last = {}                                       # slot -> event of its last attention
        for j in range(n):
            k = j % len(self.slots)
            s = self.slots[k]
            if k in last:                               # the slot's buffers are reused
                main.wait_event(last[k])
            kv.kvs_predict_scores(p, s["q"], s["K_lr"], s["A"], s["gs"], s["ws"])
            e_p = torch.cuda.Event()
            e_p.record(main)
            with torch.cuda.stream(s_sel):
                s_sel.wait_event(e_p)
                kv.kvs_select_topk(p, s["gs"], s["idx"], s["ws"])
                e_t = torch.cuda.Event()
                e_t.record(s_sel)
            with torch.cuda.stream(s_att):
                s_att.wait_event(e_t)
                kv.kvs_sparse_decode_attn(p, s["q"], s["K"], s["V"], s["idx"], s["out"], s["ws"])
                e_a = torch.cuda.Event()
                e_a.record(s_att)
            last[k] = e_a
        main.wait_stream(s_sel)
        main.wait_stream(s_att)


def time_steps(wl: Workload, steps: int, warmup: int, mode: str, layer_ahead: bool = False,
               regions: int = 1) -> list:
    """Seconds for exactly `steps` steps (after `warmup` untimed ones), measured `regions`
    times over: one entry per timed region, each bracketed by a device synchronisation."""
    torch = wl.torch
    # steps per captured graph: one rotation over the copies, and at least 24 so that the
    # launch of the graph itself stays a small part of a replay
    # (layer-ahead: exactly one rotation, so that no copy - standing in for a layer - is used
    # twice inside a graph and has to wait for its own previous use)
    # (the two-launch pipelined form runs on one stream and may reuse a copy like the serial form)
    one_rotation = layer_ahead and not wl.pipelined_in_two_launches()
    n = 1 if wl.layers_per_step != 1 else len(wl.slots) * (1 if one_rotation else max(1, -(-24 // len(wl.slots))))
    out = []
    if mode == "eager":
        wl.run(warmup, layer_ahead)
        for _ in range(regions):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            wl.run(steps, layer_ahead)
            torch.cuda.synchronize()
            out.append(time.perf_counter() - t0)
        return out
    # graph mode: one captured rotation (n steps), plus a tail graph if steps % n != 0
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        wl.run(max(2, min(warmup, n)), layer_ahead)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    def capture(count):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            wl.run(count, layer_ahead)
        return g

    full, tail = divmod(steps, n)
    g_full = capture(n) if full else None
    g_tail = capture(tail) if tail else None
    for _ in range(max(1, warmup // n)):
        (g_full or g_tail).replay()
    for _ in range(regions):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(full):
            g_full.replay()
        if g_tail is not None:
            g_tail.replay()
        torch.cuda.synchronize()
        out.append(time.perf_counter() - t0)
    return out


def median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2] if len(xs) % 2 else 0.5 * (xs[len(xs) // 2 - 1] + xs[len(xs) // 2])


def time_kernels(wl: Workload, reps: int) -> dict:
    """Average duration of each of the step's three kernels from HIP events on the launch
    stream: `reps` back-to-back launches over the rotating copies, through the split entry
    points (the same kernels kvs_decode_step launches), replayed as one captured graph
    between two events, so that the host's launch cost (longer than the small kernels) is
    not in the figure.  What remains beside the kernel's own duration is the gap between
    consecutive launches on the device (about a microsecond); the rocprofv3 kernel trace
    under profiles/ has the durations alone.
    The selection kernel consumes the histogram the prediction kernel leaves behind, so it
    is timed as (prediction + selection) minus prediction."""
    torch, kv, p = wl.torch, wl.kv, wl.p

    def timed(fn):
        for i in range(min(reps, len(wl.slots))):
            fn(wl.slots[i % len(wl.slots)])
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(reps):
                fn(wl.slots[i % len(wl.slots)])
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps   # us

    def pair(s):
        kv.kvs_predict_scores(p, s["q"], s["K_lr"], s["A"], s["gs"], wl.ws)
        kv.kvs_select_topk(p, s["gs"], s["idx"], wl.ws)

    out = {}
    both = timed(pair)
    # prediction alone keeps adding to the histograms; reset them afterwards
    out["predict"] = timed(lambda s: kv.kvs_predict_scores(p, s["q"], s["K_lr"], s["A"], s["gs"], wl.ws))
    kv.kvs_workspace_init(p, wl.ws)
    out["topk"] = max(both - out["predict"], 0.0)
    out["attn"] = timed(lambda s: kv.kvs_sparse_decode_attn(p, s["q"], s["K"], s["V"], s["idx"], s["out"], wl.ws))
    return out


def time_step_spread(wl: Workload, steps: int) -> dict:
    """Spread of the single-step latency: eager steps over the rotating copies with a HIP
    event between consecutive steps (each interval also holds one event record)."""
    torch = wl.torch
    wl.run(min(8, steps))
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    for i in range(steps):
        wl.step(i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    us = sorted(ev[i].elapsed_time(ev[i + 1]) * 1e3 / wl.layers_per_step for i in range(steps))
    pick = lambda f: us[min(len(us) - 1, int(f * len(us)))]
    return {"p10": pick(0.10), "median": pick(0.50), "p90": pick(0.90), "steps": steps, "mode": "eager"}


def time_build_metadata(wl: Workload, reps: int = 5) -> dict:
    """The metadata build (outside the step latency): reads all of K once, writes K_lr."""
    torch, kv, p = wl.torch, wl.kv, wl.p
    s = wl.slots[0]
    scratch = torch.empty_like(s["K_lr"])
    kv.kvs_build_metadata(p, s["K"], s["A"], scratch)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        sl = wl.slots[i % len(wl.slots)]
        kv.kvs_build_metadata(p, sl["K"], sl["A"], scratch)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / reps
    nbytes = s["K"].numel() * s["K"].element_size() + scratch.numel() * scratch.element_size()
    return {"us": us, "algorithmic_bytes": nbytes, "gbps": nbytes / us / 1e3,
            "frac": nbytes / us / 1e3 / HBM_PEAK_GBPS}


def load_traffic(cfg_name: str, kernel: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE, scaled
    by a plain copy of known size), if a summary for this workload has been committed."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f)[cfg_name][kernel]["bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def cpu_baseline(cfg, L, budget_s: float = 12.0, meta: str = None) -> dict:
    """The fp64 oracle as it stands, single-threaded, on the same inputs: whole steps
    (prediction + selection + sparse attention) of copy 0 until ~budget_s seconds."""
    import numpy as np
    import oracle

    code = oracle.F32 if cfg.dtype == "f32" else oracle.BF16
    # bound the sample: at most 8 (sequence, kv head) problems of the batch
    P = cfg.batch * cfg.n_kv_heads
    nb = max(1, min(cfg.batch, 8 // cfg.n_kv_heads if cfg.n_kv_heads <= 8 else 1))
    mcode, mscale = (oracle.FP8_E4M3, 0.125) if meta == "fp8" else (code, 0.0)
    sh = oracle.Shape(nb, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.rank, cfg.ctx_len,
                      cfg.group_size, cfg.n_select, code, mcode, n_threads=1, meta_scale=mscale,
                      head_mode=oracle.HEADS_JOINT if cfg.joint else oracle.HEADS_SEPARATE)
    K, V, q = (np.ascontiguousarray(x[:nb]) for x in (L.K, L.V, L.q))
    klr = oracle.build_metadata(oracle.Shape(**{**sh.__dict__, "n_threads": 8}), K, L.A)  # untimed set-up

    def timed(shape, budget):
        reps, spent = 0, 0.0
        while spent < budget and reps < 2000:
            t0 = time.perf_counter()
            r = oracle.predict_select(shape, q, klr, L.A)
            oracle.sparse_attn(shape, q, K, V, r["idx"])
            spent += time.perf_counter() - t0
            reps += 1
        return reps, spent

    reps, spent = timed(sh, budget_s)
    tokens = reps * nb                      # sequences advanced by one token
    frac = nb * cfg.n_kv_heads / P          # share of one layer-step that was timed
    # the same sample with the oracle's own threading over the independent problems
    threads = max(1, min(16, os.cpu_count() or 1, nb * cfg.n_kv_heads))
    reps_t, spent_t = timed(oracle.Shape(**{**sh.__dict__, "n_threads": threads}), budget_s / 3)
    return {"value": tokens / spent / cfg.layers, "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "sample": f"{reps} x (predict_select + sparse_attn) of {nb} of {cfg.batch} sequences, "
                      f"{cfg.n_kv_heads} kv heads, one layer, fp64 single thread; "
                      f"{spent / reps * 1e3:.1f} ms per sampled layer-step "
                      f"({frac:.3g} of a full layer-step); value scaled to all {cfg.layers} layer(s)",
            "threaded": {"value": reps_t * nb / spent_t / cfg.layers, "cores": threads,
                         "ms_per_sampled_layer_step": spent_t / reps_t * 1e3}}


def measure(cfg, steps, warmup, mode, copies=None, log=print, want_cpu=True, meta=None,
            layer_ahead=False, cpu_budget_s: float = 12.0) -> dict:
    ab = algorithmic_bytes(cfg, 1 if meta == "fp8" else None)
    if copies is None:
        copies = max(2, int(-(-3 * CACHE_BYTES // ab["step"])))   # rotation >= 3x the caches
        copies = min(copies, 32)
    wl = Workload(cfg, copies, log, meta)
    layers = wl.layers_per_step
    # The timed region is exactly `steps` steps; it is measured several times over (so that at
    # least ~200 steps are timed in all, whatever `steps` is) and the median region counts.
    regions = max(3, min(25, -(-200 // max(1, steps * layers))))
    secs = time_steps(wl, steps, warmup, mode, regions=regions)
    sec = median(secs)
    ms_step = sec / steps * 1e3
    us_layer = ms_step * 1e3 / layers
    region_us = sorted(x / steps * 1e6 / layers for x in secs)
    kern = time_kernels(wl, max(steps, 50))
    meta_build = time_build_metadata(wl)
    spread = time_step_spread(wl, max(steps, 50) if layers == 1 else max(3, min(steps, 10)))
    # warm-cache figure for reference: the same step repeated on one copy
    one = Workload.__new__(Workload)
    one.__dict__.update(wl.__dict__)
    one.slots = wl.slots[:1] if layers == 1 else wl.slots
    warm_ms = median(time_steps(one, steps, warmup, mode, regions=3)) / steps * 1e3 if layers == 1 else None
    # the same steps issued layer-ahead (prediction of later layers overlapping the
    # selection and attention of earlier ones); with a one-layer workload the rotating
    # copies stand in for the successive layers of a model
    ahead_ms = (median(time_steps(wl, steps, warmup, mode, layer_ahead=True, regions=3)) / steps * 1e3
                if layer_ahead else None)
    # the same steps as one launch each (kvs_decode_step_single_launch), where that entry
    # point covers the layout: reported beside the three-launch figure, never instead of it
    single_ms = None
    try:
        wl.single_launch = True
        single_ms = median(time_steps(wl, steps, warmup, mode, regions=3)) / steps * 1e3
    except wl.kv.KvsError as e:
        if e.status != 4:
            raise
    finally:
        wl.single_launch = False
    dom = max(("predict", "attn"), key=lambda k: kern[k])
    achieved = ab[dom] / (kern[dom] * 1e-6) / 1e9
    res = {
        "tokens_per_s": cfg.batch / (ms_step * 1e-3),
        "ms_per_step": ms_step,
        "us_per_layer": us_layer,
        "timed_regions": {"count": regions, "steps_each": steps,
                          "us_per_layer_min": region_us[0], "us_per_layer_median": us_layer,
                          "us_per_layer_max": region_us[-1]},
        "step_gbps": ab["step"] * layers / (ms_step * 1e-3) / 1e9,
        "kernel_us": kern,
        "dominant": dom,
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": load_traffic(cfg.name, dom) if meta is None else None,
                     "algorithmic_bytes": ab[dom], "kernel_us": kern[dom]},
        "algorithmic_bytes": ab,
        "copies": len(wl.slots),
        "warm_ms_per_step": warm_ms,
        "us_per_layer_spread": spread,
        "build_metadata": meta_build,
        "single_launch": None if single_ms is None else {
            "us_per_layer": single_ms * 1e3 / layers,
            "step_hbm_frac": ab["step"] * layers / (single_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "layer_ahead": None if ahead_ms is None else {
            "us_per_layer": ahead_ms * 1e3 / layers,
            "step_hbm_frac": ab["step"] * layers / (ahead_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "form": ("two launches per layer on one stream: kvs_predict_scores of layer i+1, then "
                     "kvs_attend_select_next (attention of layer i with the selection of layer i+1)"
                     if wl.pipelined_in_two_launches() else
                     "prediction, selection and attention on three streams chained by events")},
    }
    if want_cpu:
        res["cpu_baseline"] = cpu_baseline(cfg, wl.host0, budget_s=cpu_budget_s, meta=meta)
    del wl, one
    import torch
    torch.cuda.empty_cache()
    return res


def describe(cfg, meta=None) -> str:
    return (f"{cfg.name}: {cfg.n_q_heads}q/{cfg.n_kv_heads}kv d={cfg.head_dim} N={cfg.ctx_len} b={cfg.batch} "
            f"r={cfg.rank} G={cfg.group_size} M={cfg.n_select} layers={cfg.layers} {cfg.dtype}"
            + (" joint-head" if cfg.joint else "") + (" fp8-metadata" if meta else ""))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=240)
    ap.add_argument("--warmup", type=int, default=24)
    ap.add_argument("--config", default="c4",
                    choices=["c1", "c2", "c3", "c4", "c5", "c1j", "c2j", "c3j", "c4j", "c5j"],
                    help="workload; a trailing j = the same workload under the joint-head design")
    ap.add_argument("--mode", default="graph", choices=["graph", "eager"])
    ap.add_argument("--copies", type=int, default=None, help="rotating input copies (default: 3x the caches)")
    ap.add_argument("--extra", default="c1,c2,c3,c5",
                    help="further configs reported under 'other_workloads' ('' = none)")
    ap.add_argument("--meta", default="same", choices=["same", "fp8"],
                    help="dtype of the compressed K cache: that of the workload, or 8-bit E4M3")
    ap.add_argument("--layer-ahead", dest="layer_ahead", action="store_true", default=True,
                    help="also time the steps issued layer-ahead (three streams): reported beside the serial "
                         "figure, never instead of it (default)")
    ap.add_argument("--no-layer-ahead", dest="layer_ahead", action="store_false",
                    help="skip that pass, e.g. for a kernel trace that should hold no overlapped launches")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    # a workload's layer geometry can be changed, e.g. to that of another model of Sec. 4.1
    # (--q-heads 40 --group-size 12 --ctx-len 32760 --n-select 33: a Qwen3-14B layer at G = 12)
    for flag in ("batch", "q-heads", "kv-heads", "ctx-len", "rank", "group-size", "n-select"):
        ap.add_argument("--" + flag, type=int, default=None, help="override this field of the workload")
    ap.add_argument("--pmc-copy", action="store_true",
                    help="also run one 256 MiB device copy (calibration kernel for rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "run it with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from workloads import PRESETS

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    log = lambda *a: print(*a, file=sys.stderr, flush=True)
    import paper_2511_11907_amd as kv
    log(f"[bench] {kv.kvs_version()} from {kv.library_path()} on {torch.cuda.get_device_name(0)}")

    if args.pmc_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cfg = PRESETS[args.config]
    over = {field: getattr(args, arg) for arg, field in
            (("batch", "batch"), ("q_heads", "n_q_heads"), ("kv_heads", "n_kv_heads"), ("ctx_len", "ctx_len"),
             ("rank", "rank"), ("group_size", "group_size"), ("n_select", "n_select"))
            if getattr(args, arg) is not None}
    if over:
        cfg = cfg.replace(name=cfg.name + "*", **over)
        if "rank" in over:
            cfg = cfg.replace(planted_rank=min(cfg.rank, cfg.planted_rank))
    meta = None if args.meta == "same" else args.meta
    main_res = measure(cfg, args.steps, args.warmup, args.mode, args.copies, log,
                       want_cpu=not args.no_cpu_baseline, meta=meta, layer_ahead=args.layer_ahead)
    others = {}
    for name in [x for x in args.extra.split(",") if x and x != args.config]:
        c = PRESETS[name]
        # c5: a step is the whole 36-layer stack, replayed as one captured graph of 108 launches
        st = max(10, min(args.steps, 20)) if c.layers > 1 else max(20, min(args.steps, 60))
        r = measure(c, st, max(4, min(args.warmup, 8)), args.mode, None, log,
                    want_cpu=not args.no_cpu_baseline, meta=meta, layer_ahead=args.layer_ahead,
                    cpu_budget_s=3.0)
        keep = ["tokens_per_s", "ms_per_step", "us_per_layer", "timed_regions", "kernel_us", "copies",
                "layer_ahead", "single_launch", "us_per_layer_spread", "algorithmic_bytes"]
        if name.startswith("c1"):
            # 0.8 MB per step: bound by launch and memory latency, latency reported only
            others[name] = {k: r[k] for k in keep}
            others[name]["roofline"] = None
            others[name]["note"] = "latency-bound (0.8 MB per step): microseconds only, no roofline claim"
        else:
            others[name] = {k: r[k] for k in keep + ["step_gbps", "roofline", "build_metadata"]}
            others[name]["step_hbm_frac"] = r["step_gbps"] / HBM_PEAK_GBPS
        if "cpu_baseline" in r:
            others[name]["cpu_baseline"] = r["cpu_baseline"]
        others[name]["workload"] = describe(c, meta)

    line = {
        "metric": METRIC,
        "value": main_res["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"],
        "us_per_layer": main_res["us_per_layer"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": describe(cfg, meta), "mode": args.mode, "input_copies": main_res["copies"]},
        "step_hbm_gbps": main_res["step_gbps"],
        "step_hbm_frac": main_res["step_gbps"] / HBM_PEAK_GBPS,
        "warm_ms_per_step": main_res["warm_ms_per_step"],
        "timed_regions": main_res["timed_regions"],
        "us_per_layer_spread": main_res["us_per_layer_spread"],
        "layer_ahead": main_res["layer_ahead"],
        "single_launch": main_res["single_launch"],
        "build_metadata": main_res["build_metadata"],
        "kernel_us": main_res["kernel_us"],
        "algorithmic_bytes": main_res["algorithmic_bytes"],
        "roofline": main_res["roofline"],
    }
    if "cpu_baseline" in main_res:
        line["cpu_baseline"] = main_res["cpu_baseline"]
    if others:
        line["other_workloads"] = others
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
