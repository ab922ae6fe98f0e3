#!/usr/bin/env python3
"""Benchmark of the HACK hot path on one MI355X.

One "step" = one layer's whole scale schedule (score -> select -> compact ->
attend at every scale) on a batch of seeded synthetic inputs that are already
resident in HBM.  Prints ONE JSON line: full-schedule us/layer, plus the
roofline of the dominant kernel (attention, bf16 MFMA), per-stage rates and the
fp64 oracle timed on the host cores (a baseline, not the target).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16
HBM_PEAK_GBPS = 8000.0             # MI355X HBM3E
COPY_CALIBRATION_BYTES = 1 << 30   # read and written per launch in --mode copy
FP32_VALU_PEAK_TFLOPS = 157.3


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--config", type=int, default=2, help="workload family 0..4 (default: Infinity-2B-shaped 1024^2)")
    ap.add_argument("--layers", type=int, default=2, help="distinct layers of inputs kept resident and cycled")
    ap.add_argument("--mode", choices=["graph", "eager", "copy"], default="graph",
                    help="graph/eager: how the schedule is launched; copy: only run a plain 1 GiB-in/1 GiB-out "
                         "elementwise kernel --steps times (the known-size reference for HBM counter calibration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-breakdown", action="store_true")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--keep", type=float, default=None,
                    help="configs 2 and 4: retained fraction of the cache averaged over heads (default 0.3, i.e. rho = 70 %%)")
    ap.add_argument("--head-variance", action="store_true",
                    help="also time the offline head-classification kernels (attention variance of every unit at the "
                         "final step over the full cache) and report them in a head_variance object")
    ap.add_argument("--final-merge", action="store_true",
                    help="also time the schedule with the final-step merge of the contextual units in its last step")
    ap.add_argument("--no-full-cache-reference", action="store_true",
                    help="skip the extra run of the same schedule without compression (full_cache_reference)")
    ap.add_argument("--full-budget", action="store_true",
                    help="reference run: budgets = the whole cache, i.e. the same kernels with no compression "
                         "(plain KV-cache attention over all previous scales)")
    return ap.parse_args()


class LayerState:
    """Inputs of one layer resident on the device + its managed cache."""

    def __init__(self, hk, cfg, layer, wl, torch, full_budget=False):
        self.cfg, self.layer = cfg, layer
        self.types = wl.head_types(cfg, layer)
        self.budgets = [wl.step_budgets(cfg, layer, k) for k in range(1, cfg.n_steps + 1)]
        cap = np.minimum(np.tile(wl.head_budgets(cfg, layer), cfg.batch), cfg.T_K)
        if full_budget:
            self.budgets = [np.full(cfg.n_units, wl.NO_COMPRESSION, np.int32) for _ in self.budgets]
            cap = np.full(cfg.n_units, cfg.T_K, np.int64)
        self.cap = cap
        self.mc = hk.managed_cache(cap, with_pos=True)
        dev = torch.device("cuda", 0)
        self.q, self.k, self.v, self.o = [], [], [], []
        data = wl.gen_layer(cfg, layer)
        for kk in range(1, cfg.n_steps + 1):
            st = data[kk]
            for dst, src_f, src_b in ((self.q, st.q, st.q_bits), (self.k, st.k, st.k_bits), (self.v, st.v, st.v_bits)):
                if cfg.dtype == "bf16":
                    t = torch.from_numpy(src_b.view(np.int16)).to(dev).view(torch.bfloat16)
                else:
                    t = torch.from_numpy(src_f).to(dev)
                dst.append(t.contiguous())
            self.o.append(torch.empty_like(self.q[-1]))
        self.host = data
        self.final_merge = False   # the last step with the final-step merge of the contextual units

    def run(self, hk):
        c = self.cfg
        self.mc.reset()
        for i in range(c.n_steps):
            hk.step(self.mc, self.q[i], self.k[i], self.v[i], self.types, self.budgets[i], c.n_init, c.scale, self.o[i],
                    final=self.final_merge and i == c.n_steps - 1)


def plan_of(cfg, budgets):
    """Per step (L before, T_in, len_out) per unit for the budgets actually used."""
    L = np.zeros(cfg.n_units, np.int64)
    plan = []
    for i in range(cfg.n_steps):
        t_in = L + cfg.N[i]
        len_out = np.minimum(budgets[i].astype(np.int64), t_in)
        plan.append((L.copy(), t_in, len_out))
        L = len_out
    return plan


def time_events(torch, fn, reps):
    """Average ms of one fn() launch: reps launches are captured in a HIP graph
    (after one eager call that uploads the launch table) and the replay is
    bracketed by HIP events on the stream it runs on, so host-side launch cost
    does not leak into short kernels."""
    fn()
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(st):
        with torch.cuda.graph(g, stream=st):
            for _ in range(reps):
                fn()
        g.replay()                       # warm replay
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(st)
        g.replay()
        b.record(st)
    torch.cuda.synchronize()
    return float(a.elapsed_time(b)) / reps


def breakdown(hk, ls, wl, torch, reps=5):
    """Per-stage time of one layer: the same kernels hack_step launches, issued
    through the individual entry points on the same cache states, each bracketed
    by HIP events.  Returns dict stage -> list of ms per scale step."""
    from paper_2504_09261_amd.binding import Cache
    c = ls.cfg
    dev = torch.device("cuda", 0)
    stride = (c.T_K + 63) // 64 * 64
    imp = torch.zeros((c.n_units, stride), device=dev)
    kept = torch.zeros((c.n_units, stride), dtype=torch.int32, device=dev)
    cap = ls.cap
    off_s = np.concatenate([[0], np.cumsum((cap + 7) // 8 * 8)])[:-1].astype(np.int64)
    rows_s = int(((cap + 7) // 8 * 8).sum())
    ks = torch.empty((rows_s, c.head_dim), dtype=hk.torch_dtype, device=dev)
    vs = torch.empty_like(ks)
    t = dict(score=[], select=[], compact=[], attn=[])
    ls.mc.reset()
    plan = plan_of(c, ls.budgets)
    for i in range(c.n_steps):
        L, t_in, len_out = plan[i]
        comp = (len_out < t_in)
        if comp.any():
            pre = ls.mc.as_cache()
            act = comp.astype(np.uint8)
            t["score"].append(time_events(torch, lambda: hk.score(ls.q[i], pre, c.scale, imp, k_new=ls.k[i], active=act), reps))
            # select / compact are timed on the compressing units only, as in hack_step
            bud = np.where(comp, ls.budgets[i], 1 << 30).astype(np.int32)
            t["select"].append(time_events(torch, lambda: hk.select(c.batch, imp, t_in.astype(np.int32), ls.types, bud, c.n_init, c.N[i], kept), reps))
            out_len = np.where(comp, len_out, 0).astype(np.int32)
            scratch = Cache(ks, vs, off_s, out_len)
            t["compact"].append(time_events(torch, lambda: hk.compact(c.batch, c.N[i], pre, kept, scratch, ls.k[i], ls.v[i]), reps))
        else:
            for s in ("score", "select", "compact"):
                t[s].append(0.0)
        hk.step(ls.mc, ls.q[i], ls.k[i], ls.v[i], ls.types, ls.budgets[i], c.n_init, c.scale, ls.o[i])
        post = ls.mc.as_cache()
        t["attn"].append(time_events(torch, lambda: hk.attn(ls.q[i], post, c.scale, ls.o[i]), reps))
    return t


def cpu_baseline(cfg, layer, wl, budget_s=12.0, max_layers=4):
    """The oracle as it stands, on the host cores, on a bounded sample of the
    workload: whole schedules of single units, alternating head classes, over
    successive layers until about budget_s seconds of CPU work are spent."""
    from oracle import hack_oracle as ho
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    t_per, n_units, spent, layers_used = {}, 0, 0.0, 0
    for lay in range(layer, layer + max_layers):
        if spent > budget_s:
            break
        layers_used += 1
        types = wl.head_types(cfg, lay)
        data = wl.gen_layer(cfg, lay)
        steps = [(data[k].q, data[k].k, data[k].v) for k in range(1, cfg.n_steps + 1)]
        budgets = [wl.step_budgets(cfg, lay, k) for k in range(1, cfg.n_steps + 1)]
        ctx = [int(h) for h in np.where(types == 0)[0]]
        st = [int(h) for h in np.where(types == 1)[0]]
        if not ctx or not st:
            ctx = st = list(range(cfg.heads))
        # alternate classes so a cut-off sample keeps the workload's contextual/structural mix in view
        order = [u for pair in zip(st, ctx + st) for u in pair] + list(range(cfg.n_units))
        seen = set()
        for u in order:
            if u in seen:
                continue
            seen.add(u)
            t0 = time.perf_counter()
            ho.run_schedule(steps, types, budgets, cfg.n_init, cfg.scale, cfg.n_obs, units=[u], keep_outputs=False)
            dt = time.perf_counter() - t0
            t_per.setdefault(int(types[u % cfg.heads]), []).append(dt)
            n_units += 1
            spent += dt
            if spent > 2.5 * budget_s:
                break
    types0 = wl.head_types(cfg, layer)
    n_c = int((np.tile(types0, cfg.batch) == 0).sum())
    n_s = cfg.n_units - n_c
    mean_c = float(np.mean(t_per.get(0, t_per.get(1))))
    mean_s = float(np.mean(t_per.get(1, t_per.get(0))))
    layer_s = n_c * mean_c + n_s * mean_s
    return dict(value=layer_s * 1e6, unit="us/layer", cores=int(cores), kind="oracle",
                sample=f"{n_units} unit schedules from {layers_used} layer(s) starting at layer {layer}, "
                       f"{spent:.1f} s measured; per-class means scaled to one layer "
                       f"({n_c} contextual, {n_s} structural units)")


def head_variance_leg(hk, ls, torch, reps=5):
    """Times hack_head_variance on the final step of the layer: all N_K queries against the full cache."""
    from paper_2504_09261_amd.binding import Cache
    c = ls.cfg
    stride = (c.T_K + 7) // 8 * 8
    k_all = torch.cat(ls.k, dim=2).reshape(c.n_units, c.T_K, c.head_dim)
    kc = torch.zeros((c.n_units, stride, c.head_dim), dtype=k_all.dtype, device=k_all.device)
    kc[:, :c.T_K] = k_all
    kc = kc.reshape(c.n_units * stride, c.head_dim)
    cache = Cache(kc, kc, np.arange(c.n_units, dtype=np.int64) * stride, np.full(c.n_units, c.T_K, np.int32))
    sigma = torch.zeros(c.n_units, dtype=torch.float64, device=k_all.device)
    q = ls.q[-1]
    ms = time_events(torch, lambda: hk.head_variance(q, cache, c.scale, sigma), reps)
    flop = 2 * 2.0 * c.N[-1] * c.T_K * c.head_dim * c.n_units          # two passes of Q K^T
    return {"us": ms * 1e3, "gflop": flop / 1e9, "TFLOPs": flop / (ms * 1e-3) / 1e12,
            "frac_mfma": flop / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "sigma_contextual_mean": float(sigma.cpu().numpy().reshape(c.batch, c.heads)[:, ls.types == 0].mean()),
            "sigma_structural_mean": float(sigma.cpu().numpy().reshape(c.batch, c.heads)[:, ls.types == 1].mean())}


def committed_traffic(cfg, kernel, source):
    """HBM bytes per launch of `kernel` on this workload from the committed counter summary (rocprofv3
    --pmc FETCH_SIZE / WRITE_SIZE runs, calibrated on a plain copy).  The number is not measured in this
    run, so its provenance travels with it: the summary records the SHA-256 of the kernel source it was
    measured on, and `stale` says whether the source has changed since.  None when no summary is present."""
    import hashlib
    here = os.path.dirname(os.path.abspath(__file__))
    path = os.path.join(here, "profiles", f"{kernel}_cfg{cfg.cfg_id}_hbm_traffic.txt")
    value, measured_sha = None, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                value = float(line.split("=")[1].split()[0])
            if line.startswith("kernel_source_sha256"):
                measured_sha = line.split("=")[1].split()[0]
    except OSError:
        return None, None
    try:
        now_sha = hashlib.sha256(open(os.path.join(here, source), "rb").read()).hexdigest()
    except OSError:
        now_sha = None
    return value, {"file": os.path.relpath(path, here), "kernel_source": source, "measured_on_sha256": measured_sha,
                   "current_sha256": now_sha, "stale": measured_sha is None or measured_sha != now_sha,
                   "note": "committed rocprofv3 counter summary, not measured in this run"}


def parity_leg(hk, ls, wl, torch, n_units=4):
    """Device-vs-oracle parity of the timed workload (part of the cpu_baseline leg, outside the timed
    region): one more eager pass of layer 0 that keeps the kept indices, and the oracle walking the same
    schedule for a few units of both head classes (oracle.parity.ScheduleChecker)."""
    from oracle.parity import ScheduleChecker
    c = ls.cfg
    types = ls.types
    ctx = [int(h) for h in np.where(types == 0)[0]]
    st = [int(h) for h in np.where(types == 1)[0]]
    units = []
    for i in range(n_units):
        pool = ctx if (i % 2 == 0 and ctx) else (st or ctx)
        b = (i // 2) % c.batch
        units.append(b * c.heads + pool[(i // 2) % len(pool)])
    units = sorted(set(units))
    tol = 1e-4 if c.dtype == "f32" else 2e-2
    chk = ScheduleChecker(c.heads, c.head_dim, types, c.n_init, c.scale, c.n_obs, units, tol)
    stride = (c.T_K + 63) // 64 * 64
    kept = torch.full((c.n_units, stride), -1, dtype=torch.int32, device=ls.q[0].device)
    ls.mc.reset()
    L = np.zeros(c.n_units, np.int64)
    for i in range(c.n_steps):
        hk.step(ls.mc, ls.q[i], ls.k[i], ls.v[i], types, ls.budgets[i], c.n_init, c.scale, ls.o[i], kept_idx=kept)
        torch.cuda.synchronize()
        off, ln = ls.mc.view()
        t_in = L + c.N[i]
        L = np.minimum(ls.budgets[i].astype(np.int64), t_in)
        dev = {}
        for u in units:
            b, h = divmod(u, c.heads)
            dev[u] = dict(I=kept[u, :ln[u]].cpu().numpy() if L[u] < t_in[u] else None,
                          pos=ls.mc.pos[off[u]:off[u] + ln[u]].cpu().numpy(),
                          O=ls.o[i][b, h].float().cpu().numpy().astype(np.float64))
        hst = ls.host[i + 1]
        chk.step(hst.q, hst.k, hst.v, ls.budgets[i], dev)
    s = chk.summary()
    return {"workload": c.name, "layer": ls.layer, "units_checked": len(units), "steps": s["steps"],
            "kept_sets": {"compared": s["compress_events"], "exact": s["exact"], "excused": s["excused"],
                          "mismatch": s["mismatch"]},
            "near_tie_rel": s["near_tie_rel"], "token_id_mismatches": s["pos_mismatch"],
            "max_abs_dO": s["max_abs_dO"], "tolerance": tol, "ok": not chk.failures}


def full_cache_leg(hk, cfg, wl, torch, args, time_schedule, attn_last_us):
    """The same schedule with budgets that cover the whole cache (no compression: plain KV-cache
    attention over all previous scales), timed the same way: the reference of the paper's efficiency
    analysis (whole path and attention at the last scale with and without compression)."""
    ls = LayerState(hk, cfg, 0, wl, torch, full_budget=True)
    ls.run(hk)
    torch.cuda.synchronize()
    ms = time_schedule([ls], max(4, args.steps // 4), 2)
    post = ls.mc.as_cache()
    i = cfg.n_steps - 1
    last = time_events(torch, lambda: hk.attn(ls.q[i], post, cfg.scale, ls.o[i]), 3)
    ls.mc.close()
    return {"budgets": "whole cache", "us_per_layer": ms * 1e3, "attn_last_scale_us": last * 1e3,
            "keys_per_unit_last_scale": cfg.T_K,
            "attn_last_scale_us_compressed": attn_last_us,
            "attn_last_scale_speedup": (last * 1e3) / attn_last_us if attn_last_us else None}


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (units are independent; there is no multi-GPU path); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2504_09261_amd import workload as wl
    from paper_2504_09261_amd.binding import Hack

    torch.cuda.set_device(0)
    if args.mode == "copy":
        n = COPY_CALIBRATION_BYTES // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(args.steps):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"mode": "copy", "launches": args.steps, "bytes_read_per_launch": 4 * n,
                          "bytes_written_per_launch": 4 * n}))
        return
    cfg = wl.get_config(args.config, batch=args.batch, **({} if args.keep is None else {"keep": args.keep}))
    hk = Hack(cfg.heads, cfg.head_dim, cfg.dtype, cfg.n_units, cfg.T_K, max(cfg.N), cfg.n_obs)
    layers = [LayerState(hk, cfg, l, wl, torch, args.full_budget) for l in range(args.layers)]

    # eager warm-up: uploads every launch table once
    for ls in layers:
        ls.run(hk)
    torch.cuda.synchronize()

    stream = torch.cuda.Stream()

    def time_schedule(lstates, steps, warmup):
        """ms per layer schedule: `steps` schedules (cycling over lstates) after `warmup` untimed ones."""
        graphs = None
        if args.mode == "graph":
            graphs = []
            with torch.cuda.stream(stream):
                for l in lstates:
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=stream):
                        l.run(hk)
                    graphs.append(g)
            torch.cuda.synchronize()

        def one(i):
            if graphs is not None:
                graphs[i % len(lstates)].replay()
            else:
                lstates[i % len(lstates)].run(hk)

        with torch.cuda.stream(stream):
            for i in range(warmup):
                one(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(steps):
                one(i)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
        return (t1 - t0) * 1e3 / steps

    ms_per_step = time_schedule(layers, args.steps, args.warmup)

    work = wl.work_model(cfg, 0)
    if args.full_budget:   # no compression: every step attends over the whole cache
        for r in work:
            r.update(attn_flop=r["full_attn_flop"], score_flop=0.0, score_bytes=0.0, select_bytes=0.0,
                     compact_bytes=0.0, n_compress=0)
    tot = {k: sum(r[k] for r in work) for k in work[0] if k not in ("k", "N_k")}
    # KV-cache bytes of one layer: what plain caching would hold, the largest logical cache the schedule
    # passes through (right before a compression), what is retained at the end, and what is allocated
    plan = plan_of(cfg, layers[0].budgets)
    row_bytes = 2 * cfg.head_dim * cfg.elem_bytes
    kv_bytes = {"uncompressed": int(cfg.T_K) * cfg.n_units * row_bytes,
                "logical_peak": int(max(int(t_in.sum()) for _, t_in, _ in plan)) * row_bytes,
                "final": int(plan[-1][2].sum()) * row_bytes,
                "allocated": int(layers[0].mc.k.shape[0]) * row_bytes}
    result = {
        "metric": "full-schedule us/layer", "value": ms_per_step * 1e3, "unit": "us/layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "units": cfg.n_units, "heads": cfg.heads, "head_dim": cfg.head_dim,
                   "batch": cfg.batch, "scales": len(cfg.sides), "tokens": cfg.T_K, "launch": args.mode,
                   "layers_resident": args.layers},
        "budgets": "full cache (no compression)" if args.full_budget else "workload default",
        "kv_bytes_per_layer": kv_bytes,
        "attn_gflop_per_layer": tot["attn_flop"] / 1e9,
        "compress_mb_per_layer": (tot["score_bytes"] + tot["select_bytes"] + tot["compact_bytes"]) / 1e6,
    }

    if not args.no_breakdown:
        bd = breakdown(hk, layers[0], wl, torch)
        attn_ms = sum(bd["attn"])
        n_attn = len(bd["attn"])
        tf = tot["attn_flop"] / (attn_ms * 1e-3) / 1e12
        if cfg.dtype == "bf16":
            # The dominant kernel is attn_pipe (128-query work items); the early steps with few
            # queries run the key-split kernel attn_split.  The roofline entry is attn_pipe's own:
            # flop of the steps it serves / its launch time; every step together is listed beside it.
            own = [i for i in range(n_attn) if hk.attn_variant(cfg.batch, cfg.N[i]) == 0]
            own_flop = sum(work[i]["attn_flop"] for i in own)
            own_ms = sum(bd["attn"][i] for i in own)
            tf_own = own_flop / (own_ms * 1e-3) / 1e12
            big = [i for i, r in enumerate(work) if r["attn_flop"] > 0.05 * tot["attn_flop"]]
            tf_big = sum(work[i]["attn_flop"] for i in big) / (sum(bd["attn"][i] for i in big) * 1e-3) / 1e12
            kname = "attn_pipe" if os.environ.get("HACK_ATTN_PIPE", "1") != "0" else "attn_mfma"
            traffic, traffic_src = committed_traffic(cfg, kname, "paper_2504_09261_amd/csrc/kernels_attn.hip")
            result["roofline"] = {
                "bound": "mfma", "kernel": kname, "achieved": tf_own, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": tf_own / MFMA_BF16_PEAK_TFLOPS,
                "traffic": traffic, "traffic_source": traffic_src,
                "steps": [i + 1 for i in own], "launches_per_layer": len(own),
                "avg_launch_us": own_ms * 1e3 / len(own), "flop_per_launch": own_flop / len(own),
                "all_attention_launches": {"launches_per_layer": n_attn, "achieved": tf,
                                           "frac": tf / MFMA_BF16_PEAK_TFLOPS,
                                           "attn_split_steps": [i + 1 for i in range(n_attn) if i not in own]},
                "large_steps": {"steps": [i + 1 for i in big], "achieved": tf_big,
                                "frac": tf_big / MFMA_BF16_PEAK_TFLOPS},
            }
        else:
            result["roofline"] = {
                "bound": "alu", "kernel": "attn_generic", "achieved": tf, "peak": FP32_VALU_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": tf / FP32_VALU_PEAK_TFLOPS, "traffic": None,
            }
        stages = {}
        for s, key in (("score", "score_bytes"), ("select", "select_bytes"), ("compact", "compact_bytes")):
            ms = sum(bd[s])
            stages[s] = {"us_per_layer": ms * 1e3, "algorithmic_MB": tot[key] / 1e6,
                         "GBps": (tot[key] / 1e9) / (ms * 1e-3) if ms > 0 else None,
                         "frac_hbm": (tot[key] / 1e9) / (ms * 1e-3) / HBM_PEAK_GBPS if ms > 0 else None}
        ssc_ms = sum(sum(bd[s]) for s in ("score", "select", "compact"))
        ssc_b = tot["score_bytes"] + tot["select_bytes"] + tot["compact_bytes"]
        stages["score+select+compact"] = {"us_per_layer": ssc_ms * 1e3, "GBps": ssc_b / 1e9 / (ssc_ms * 1e-3) if ssc_ms else None,
                                          "frac_hbm": ssc_b / 1e9 / (ssc_ms * 1e-3) / HBM_PEAK_GBPS if ssc_ms else None}
        stages["attn"] = {"us_per_layer": attn_ms * 1e3, "per_step_us": [round(x * 1e3, 1) for x in bd["attn"]]}
        result["stages"] = stages

    if args.head_variance and cfg.dtype == "bf16":
        result["head_variance"] = head_variance_leg(hk, layers[0], torch)

    if args.final_merge and cfg.dtype == "bf16" and not args.full_budget:
        # the same schedule with the last step through hack_step_final (outside `value`: the merge belongs to the
        # last generation step of an image only)
        for ls in layers:
            ls.final_merge = True
        for ls in layers:
            ls.run(hk)   # uploads the launch tables of the merging step
        torch.cuda.synchronize()
        ms_merge = time_schedule(layers, args.steps, args.warmup)
        for ls in layers:
            ls.final_merge = False
        last = plan_of(cfg, layers[0].budgets)[-1]
        merging = [u for u in range(cfg.n_units) if layers[0].types[u % cfg.heads] == 0 and last[2][u] < last[1][u]]
        flop = sum(2.0 * float(last[1][u]) * float(last[2][u]) * cfg.head_dim for u in merging)
        result["final_merge"] = {"us_per_layer": ms_merge * 1e3, "extra_us": (ms_merge - ms_per_step) * 1e3,
                                 "units_merging": len(merging), "similarity_gflop": flop / 1e9}

    if not args.no_breakdown and not args.full_budget and not args.no_full_cache_reference:
        result["full_cache_reference"] = full_cache_leg(hk, cfg, wl, torch, args, time_schedule,
                                                        result["stages"]["attn"]["per_step_us"][-1])
        result["full_cache_reference"]["whole_path_speedup"] = result["full_cache_reference"]["us_per_layer"] / result["value"]

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, 0, wl)
        if not args.full_budget:
            # the same leg also checks the timed workload against the oracle (outside the timed region)
            result["parity"] = parity_leg(hk, layers[0], wl, torch)
            result["cpu_baseline"]["parity"] = result["parity"]

    print(json.dumps(result))


if __name__ == "__main__":
    main()
