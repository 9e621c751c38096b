#!/usr/bin/env python3
"""Benchmark of the packed variable-length attention hot path on one MI355X.

A step = one pass of the whole path over one synthetic batch: tile-list build
+ forward + backward (dQ pass, dK/dV pass), inputs resident in HBM.  The
workload is the BERT-large fwd+bwd batch (56 sequences, 16 heads, d = 64,
max length 512, seeded length mixture; fp16).  Prints ONE JSON line.

Useful FLOPs count only real tokens and the five backward contractions:
forward 4*sum(L^2)*H*d, backward 10*sum(L^2)*H*d.
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

PEAK_TFLOPS = {"f16": 2500.0, "bf16": 2500.0}   # MI355X dense MFMA, published
HBM_GBS = 8000.0
# HBM bytes per launch of the other --op modes on workload 3's shapes, from rocprofv3 FETCH_SIZE /
# WRITE_SIZE counter runs scaled by a plain-copy reference (profiles/*_kernels*.md)
MEASURED_TRAFFIC_OTHER_CFG3 = {"gather_rows": 32.9e6 + 32.3e6, "scatter_rows": 33.3e6 + 58.7e6,
                               "unpad_indices": 0.27e6 + 0.18e6,
                               "ln_fwd_kernel": 64.7e6 + 65.5e6,
                               "ln_bwd (rows + columns)": 65.3e6 + 67.0e6 + 2.1e6,
                               "embedding_bwd_window_kernel": 32.7e6 + 26.3e6}


def stored_traffic(workload, kernel):
    """HBM bytes per launch of an attention kernel from profiles/traffic.json (written by
    paper_2208_08124_amd/profile_traffic.py from counter runs), or None if the file is
    missing, is for another workload, or was measured on other kernel sources."""
    from paper_2208_08124_amd import build
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as fh:
            doc = json.load(fh)
    except (OSError, ValueError):
        return None
    if doc.get("source_id") != build.source_id() or doc.get("workload") != workload:
        return None
    k = doc.get("kernels", {}).get(kernel)
    return None if k is None else k["fetch_bytes"] + k["write_bytes"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, help="workload 2..5 (3 = headline)")
    ap.add_argument("--uniform", type=str, default=None, metavar="L,B",
                    help="kernel study: B sequences of exactly L tokens instead of --config's lengths")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="only run a plain device-to-device copy of this many MiB a few times "
                         "(reference reading for rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--dropout", type=float, default=0.0, metavar="P",
                    help="run every step through the dropout entry points with this probability "
                         "(the headline workload has none; a default run reports p = 0.1 beside it)")
    ap.add_argument("--op", choices=["attention", "unpad", "layernorm", "embedding"], default="attention",
                    help="attention (the headline path), the padded <-> unpadded row copies, or "
                         "Dropout+Add+LayerNorm on the packed rows")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-padded", action="store_true")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (sequences and heads are independent, so more "
              "GPUs would each run their own batch); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2208_08124_amd import fmha
    from paper_2208_08124_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    fmha.lib()  # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": n, "copies": 5}))
        return
    dev_dt = {"f16": torch.float16, "bf16": torch.bfloat16}
    if args.op == "unpad":
        bench_unpad(args, torch, fmha, wl)
        return
    if args.op == "layernorm":
        bench_layernorm(args, torch, fmha, wl)
        return
    if args.op == "embedding":
        bench_embedding(args, torch, fmha, wl)
        return

    b = wl.make_workload(args.config, backward=True)
    if args.uniform:
        ul, ub = (int(x) for x in args.uniform.split(","))
        w = wl.WORKLOADS[args.config]
        b = wl.make_batch([ul] * ub, w.heads, w.dtype, w.seed, backward=True)
        b["name"] = "uniform_%dx%d" % (ul, ub)
    dt = b["dtype"]
    lengths = b["lengths"]
    T, H = b["total_tokens"], b["heads"]
    sum_l2 = float((lengths.astype(np.float64) ** 2).sum())
    fl_fwd = 4.0 * sum_l2 * H * 64
    fl_dq = 2.0 * sum_l2 * H * 64    # of the dQ pass only dQ = dS K is new work
    fl_dkv = 8.0 * sum_l2 * H * 64   # S, dP, dV, dK
    fl_all = fl_fwd + fl_dq + fl_dkv

    def dev(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(dev_dt[dt])

    class Dev:
        drop = (args.dropout, 220808124) if args.dropout > 0 else None   # (p, seed)

        def __init__(self, bb):
            self.bb = bb
            self.q, self.k, self.v, self.do = (dev(bb[n]) for n in ("q", "k", "v", "do"))
            self.cu = torch.from_numpy(bb["cu_seqlens"]).cuda()
            self.su = torch.from_numpy(bb["seqused"]).cuda() if "seqused" in bb else None
            t = bb["total_tokens"]
            self.o = torch.empty_like(self.q)
            self.lse = torch.empty((H, t), dtype=torch.float32, device="cuda")
            self.dq, self.dk, self.dv = (torch.empty_like(self.q) for _ in range(3))
            self.ws = fmha.alloc_workspace(bb["batch"], t, H, True)

        def fwd(self, reuse=False):
            fmha.fmha_varlen_fwd(self.q, self.k, self.v, self.cu, self.bb["max_seqlen"], self.bb["scale"],
                                 self.o, self.lse, self.ws, seqused=self.su, reuse_schedule=reuse,
                                 dropout=self.drop)

        def bwd(self, only=None):
            fmha.fmha_varlen_bwd(self.q, self.k, self.v, self.o, self.do, self.lse, self.cu,
                                 self.bb["max_seqlen"], self.bb["scale"], self.dq, self.dk, self.dv,
                                 self.ws, seqused=self.su, reuse_schedule=True, only=only,
                                 dropout=self.drop)

        def step(self):
            self.fwd()      # builds the tile list, then the forward kernel
            self.bwd()      # reuses the list: dQ pass + dK/dV pass

    def precondition(fn, seconds=0.5):
        """Untimed steps for a fixed duration ahead of a timed region: a short run (the driver's
        20 steps take 5 ms) otherwise measures the chip on its way up from idle clocks."""
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            for _ in range(10):
                fn()
            torch.cuda.synchronize()

    def timed(fn, steps, warmup):
        """Seconds per step by the wall clock over exactly `steps` steps after `warmup` untimed
        ones; timed.events_ms holds the median and minimum of the same steps by HIP events."""
        precondition(fn)
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        t0 = time.perf_counter()
        evs[0].record()
        for i in range(steps):
            fn()
            evs[i + 1].record()
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / steps
        per = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(steps))
        timed.events_ms = {"median": round(per[len(per) // 2], 5), "min": round(per[0], 5)}
        return sec

    d = Dev(b)
    warm_sec = timed(d.step, args.steps, args.warmup)
    # Cold-cache timing: rotate over enough distinct buffer sets (each holds its own
    # Q, K, V, dO, outputs and workspace) to exceed 1 GB, so that no step finds its
    # inputs in the 256 MB last-level cache.  This is the headline: consecutive
    # layers of a model never touch the same tensors either.
    set_bytes = 8 * T * H * 64 * 2
    n_sets = max(2, min(8, -(-(1 << 30) // set_bytes) + 1))
    sets = [d] + [Dev(b) for _ in range(n_sets - 1)]
    turn = [0]

    def cold_step():
        sets[turn[0] % n_sets].step()
        turn[0] += 1

    sec = timed(cold_step, args.steps, max(args.warmup, n_sets))
    step_events = dict(timed.events_ms)

    # per-kernel durations: HIP events on the launch stream between the three kernels of a
    # step (forward with the tile list already built, dQ pass, dK/dV pass), in step order and
    # rotating over the buffer sets like the timed region, so every kernel sees the cache
    # state it has inside a step
    def kernel_times(steps):
        # the plain forward and the one with dropout are different kernels
        fwd_name = "fmha_fwd64_kernel" if Dev.drop is None else "fmha_fwd_kernel"
        legs = [(fwd_name, lambda x: x.fwd(reuse=True)), ("bwd_dq_kernel", lambda x: x.bwd(only="dq")),
                ("bwd_dkv_kernel", lambda x: x.bwd(only="dkv"))]
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(legs) + 1)] for _ in range(steps)]
        for i in range(n_sets):
            sets[i].step()
        torch.cuda.synchronize()
        for i in range(steps):
            x = sets[i % n_sets]
            evs[i][0].record()
            for j, (_, fn) in enumerate(legs):
                fn(x)
                evs[i][j + 1].record()
        torch.cuda.synchronize()
        per_step = sorted(e[0].elapsed_time(e[-1]) for e in evs)   # the kernels of a step, tile list reused
        kernel_times.step_stats = {"median_ms": round(per_step[len(per_step) // 2], 5), "min_ms": round(per_step[0], 5)}
        med = lambda v: sorted(v)[len(v) // 2]
        return {nm: med([e[j].elapsed_time(e[j + 1]) for e in evs]) for j, (nm, _) in enumerate(legs)}

    ksteps = max(20, min(args.steps, 200))
    k_ms = kernel_times(ksteps)
    reuse_stats = dict(kernel_times.step_stats)
    # the tile list is built once per batch and serves all layers and both directions: a step
    # that reuses it (what 47 of the 48 attention calls of a 24-layer model do), timed like `value`
    def reuse_step():
        x = sets[turn[0] % n_sets]
        turn[0] += 1
        x.fwd(reuse=True)
        x.bwd()
    reuse_sec = timed(reuse_step, args.steps, n_sets)
    # the same cold rotation with every buffer set's step captured once in a HIP graph and
    # replayed: what the launch gaps between the four kernels of a step cost in eager mode
    graph_replay = None
    try:
        graphs = []
        for x in sets:
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph):
                x.step()
            graphs.append(gph)

        def graph_step():
            graphs[turn[0] % n_sets].replay()
            turn[0] += 1
        gsec = timed(graph_step, args.steps, n_sets)
        graph_replay = {"ms_per_step": round(gsec * 1e3, 5), "value": round(fl_all / gsec / 1e12, 3),
                        "ms_per_step_events": dict(timed.events_ms)}
        del graphs
    except RuntimeError as e:   # capture not available: report why, keep the eager figures
        graph_replay = {"error": str(e)[:200]}
    with_dropout = None
    if args.dropout == 0:
        # the same cold rotation through the dropout entry points, p = 0.1 (BERT's setting)
        Dev.drop = (0.1, 220808124)
        dsec = timed(cold_step, max(20, args.steps // 2), n_sets)
        dk_ms = kernel_times(max(20, ksteps // 2))
        Dev.drop = None
        with_dropout = {"p": 0.1, "ms_per_step": round(dsec * 1e3, 5),
                        "value": round(fl_all / dsec / 1e12, 3),
                        "kernels_ms": {k: round(v, 5) for k, v in dk_ms.items()}}
    del sets
    k_fl = {"fmha_fwd_kernel": fl_fwd, "fmha_fwd64_kernel": fl_fwd, "bwd_dq_kernel": fl_dq, "bwd_dkv_kernel": fl_dkv}
    dom = max(k_ms, key=k_ms.get)
    ach = k_fl[dom] / (k_ms[dom] * 1e-3) / 1e12
    peak = PEAK_TFLOPS[dt]
    roofline = {"bound": "mfma", "kernel": dom, "achieved": round(ach, 2), "peak": peak,
                "unit": "TFLOP/s", "frac": round(ach / peak, 4),
                "traffic": None if args.uniform else stored_traffic(b["name"], dom),
                "avg_launch_ms": round(k_ms[dom], 5),
                "kernels_ms": {k: round(v, 5) for k, v in k_ms.items()},
                "kernels_tflops": {k: round(k_fl[k] / (k_ms[k] * 1e-3) / 1e12, 2) for k in k_ms},
                "hbm_algorithmic_GBs": round(12.0 * T * H * 64 * 2 / sec / 1e9, 1)}

    out = {
        "metric": "useful attention TFLOP/s fwd+bwd",
        "value": round(fl_all / sec / 1e12, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 5),
        "ms_per_step_events": step_events,   # the timed steps again, one by one, by HIP events
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dt, "data": "synthetic",
        "config": {"workload": b["name"], "baseline_config": args.config, "sequences": int(b["batch"]),
                   "heads": int(H), "head_dim": 64, "max_seqlen": int(b["max_seqlen"]),
                   "total_tokens": int(T), "sum_len_sq": sum_l2,
                   "step": "tile-list build + forward + backward (dQ pass, dK/dV pass)"},
        "pct_of_mfma_peak": round(100.0 * fl_all / sec / 1e12 / peak, 2),
        "peak_tflops": peak,
        "tokens_per_s": round(T / sec, 1),
        "useful_flop_per_step": fl_all,
        "tile_list": {"built_every_step_ms": round(sec * 1e3, 5), "reused_ms": round(reuse_sec * 1e3, 5),
                      "amortised_1_in_48_ms": round((sec + 47 * reuse_sec) / 48 * 1e3, 5),
                      "reused_step_events": reuse_stats},
        "cache": {"value_is": "cold", "buffer_sets": n_sets,
                  "warm_ms_per_step": round(warm_sec * 1e3, 5),
                  "warm_value": round(fl_all / warm_sec / 1e12, 3)},
        "roofline": roofline,
        "graph_replay": graph_replay,
    }
    if args.dropout > 0:
        out["config"]["dropout_p"] = args.dropout
    if with_dropout:
        out["with_dropout"] = with_dropout

    if not args.no_padded:
        # the same kernels on the padded layout (every sequence 512 rows, keys past the
        # true length masked): what a padded framework executes for this batch
        pd = Dev(wl.pad_batch(b, b["max_seqlen"]))
        psec = timed(pd.step, max(5, args.steps // 4), max(2, args.warmup // 4))
        out["padded_baseline"] = {"ms_per_step": round(psec * 1e3, 5),
                                  "tokens_per_s": round(T / psec, 1),
                                  "speedup_unpadded_vs_padded": round(psec / warm_sec, 3),
                                  "note": "same buffers every step, compared with the warm unpadded time"}
        del pd

    if not args.no_cpu_baseline:
        from oracle import oracle
        n = b["batch"]
        if args.config == 5:   # bounded sample: a seeded subset incl. first, last, shortest, longest
            rng = np.random.default_rng(0)
            pick = sorted(set([0, n - 1, int(lengths.argmin()), int(lengths.argmax())]
                              + rng.choice(n, 60, replace=False).tolist()))
        else:
            pick = list(range(n))
        cu = b["cu_seqlens"]
        rows = np.concatenate([np.arange(cu[i], cu[i + 1]) for i in pick])
        sub_cu = wl.cu_from_lengths(lengths[pick])
        x = {nm: wl.bits_to_f64(b[nm][rows], dt) for nm in ("q", "k", "v", "do")}
        t0 = time.perf_counter()
        o_ref, _ = oracle.fwd(x["q"], x["k"], x["v"], sub_cu, b["scale"])
        g_ref = oracle.bwd(x["q"], x["k"], x["v"], x["do"], sub_cu, b["scale"])
        csec = time.perf_counter() - t0
        # one more step (outside every timed region; without dropout, which the oracle call
        # above does not have either), against the oracle's results for the same sequences:
        # what the parity tests assert, as achieved numbers
        from oracle.parity import gradient_errors
        Dev.drop = None
        d.step()
        torch.cuda.synchronize()
        ridx = torch.from_numpy(rows).cuda()
        f64 = lambda t: t[ridx].double().cpu().numpy()
        parity = {"sequences": len(pick), "o_max_abs": float(np.abs(f64(d.o) - o_ref).max())}
        for nm, got, want in zip(("dq", "dk", "dv"), (d.dq, d.dk, d.dv), g_ref):
            rel, fro = gradient_errors(f64(got), want, sub_cu)
            parity[nm + "_worst_sequence_rel"] = round(rel, 6)
            parity[nm + "_frobenius_rel"] = round(fro, 6)
        parity["o_max_abs"] = round(parity["o_max_abs"], 6)
        parity["bar"] = "o_max_abs <= 5e-3 (+ half a bf16 ulp of O for bf16), gradients <= 1e-2"
        out["parity"] = parity
        sub_fl = 14.0 * float((lengths[pick].astype(np.float64) ** 2).sum()) * H * 64
        out["cpu_baseline"] = {"value": round(sub_fl / csec / 1e12, 6), "unit": "TFLOP/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "%d of %d sequences, all heads, fwd+bwd, %.2f s" % (len(pick), n, csec)}

    print(json.dumps(out))


def bench_unpad(args, torch, fmha, wl):
    """The steps either side of the attention path: input_mask -> nonzero_indices / batch_offset,
    gather (padded -> unpadded) and scatter (back), on hidden-state rows of the workload's
    batch: [B, max_seqlen, H*64] 16-bit.  Bound by HBM traffic; a step = indices + one gather
    + one scatter, rotating over buffer sets like the attention bench."""
    w = wl.WORKLOADS[args.config]
    b = wl.make_workload(args.config, backward=False)
    lengths = b["lengths"]
    nb, s, hid = int(b["batch"]), int(b["max_seqlen"]), int(b["heads"]) * 64
    rows, t = nb * s, int(b["total_tokens"])
    row_bytes = hid * 2
    mask_np = (np.arange(s)[None, :] < lengths[:, None]).astype(np.int32)
    n_sets = max(2, min(8, -(-(1 << 30) // (3 * rows * row_bytes)) + 1))

    class Set:
        def __init__(self):
            self.mask = torch.from_numpy(mask_np).cuda()
            self.x = torch.randint(-30000, 30000, (rows, hid), dtype=torch.int16, device="cuda")
            self.packed = torch.empty((rows, hid), dtype=torch.int16, device="cuda")   # worst-case room
            self.back = torch.empty((rows, hid), dtype=torch.int16, device="cuda")
            self.idx = torch.empty(rows, dtype=torch.int32, device="cuda")
            self.inv = torch.empty(rows, dtype=torch.int32, device="cuda")
            self.cu = torch.empty(nb + 1, dtype=torch.int32, device="cuda")

        def indices(self):
            fmha.fmha_unpad_indices(self.mask, self.idx, self.inv, self.cu)

        def gather(self):
            fmha.fmha_gather_rows(self.x, self.idx, self.cu[-1:], self.packed)

        def scatter(self):
            fmha.fmha_scatter_rows(self.packed, self.inv, self.cu[-1:], self.back)

    sets = [Set() for _ in range(n_sets)]
    names = ("unpad_indices", "gather_rows", "scatter_rows")
    for x in sets:
        x.indices(); x.gather(); x.scatter()
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        for x in sets:
            x.indices(); x.gather(); x.scatter()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        x = sets[i % n_sets]
        x.indices(); x.gather(); x.scatter()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    for i in range(args.steps):
        x = sets[i % n_sets]
        evs[i][0].record(); x.indices(); evs[i][1].record(); x.gather(); evs[i][2].record(); x.scatter(); evs[i][3].record()
    torch.cuda.synchronize()
    k_ms = {nm: sum(e[j].elapsed_time(e[j + 1]) for e in evs) / args.steps for j, nm in enumerate(names)}
    alg = {"unpad_indices": 2 * rows * 4 + (rows + t) * 4 + (nb + 1) * 4,          # mask twice, inverse, indices, offsets
           "gather_rows": 2 * t * row_bytes + t * 4,
           "scatter_rows": t * row_bytes + rows * row_bytes + rows * 4}
    dom = max(k_ms, key=k_ms.get)
    gbs = {k: alg[k] / (k_ms[k] * 1e-3) / 1e9 for k in names}
    out = {"metric": "padded <-> unpadded rows, algorithmic GB/s (indices + gather + scatter)",
           "value": round(sum(alg.values()) / sec / 1e9, 1), "unit": "GB/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 5),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u16", "data": "synthetic",
           "config": {"workload": w.name + "_hidden_rows", "baseline_config": args.config, "sequences": nb,
                      "max_seqlen": s, "row_bytes": row_bytes, "valid_rows": t, "padded_rows": rows,
                      "buffer_sets": n_sets},
           "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(gbs[dom], 1), "peak": HBM_GBS,
                        "unit": "GB/s", "frac": round(gbs[dom] / HBM_GBS, 4),
                        "traffic": MEASURED_TRAFFIC_OTHER_CFG3.get(dom) if args.config == 3 else None,
                        "avg_launch_ms": round(k_ms[dom], 5),
                        "kernels_ms": {k: round(v, 5) for k, v in k_ms.items()},
                        "kernels_GBs": {k: round(v, 1) for k, v in gbs.items()},
                        "algorithmic_bytes": alg}}
    if not args.no_cpu_baseline:
        from oracle import unpad
        xs = np.random.default_rng(0).integers(0, 65535, size=(rows, hid)).astype(np.uint16)
        t0 = time.perf_counter()
        idx, inv, cu = unpad.unpad_indices(mask_np)
        g = unpad.gather_rows(xs, idx)
        unpad.scatter_rows(g, idx, rows)
        csec = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(sum(alg.values()) / csec / 1e9, 4), "unit": "GB/s", "cores": 1,
                               "kind": "oracle", "sample": "the whole batch once, %.2f s" % csec}
    print(json.dumps(out))


def bench_layernorm(args, torch, fmha, wl):
    """Dropout + Add + LayerNorm, forward and backward, on the packed hidden states of the
    workload's batch ([T, H*64] 16-bit, p = --dropout or 0.1).  Bound by HBM traffic; a step =
    forward + backward, rotating over buffer sets like the attention bench."""
    w = wl.WORKLOADS[args.config]
    b = wl.make_workload(args.config, backward=False)
    t, hid = int(b["total_tokens"]), int(b["heads"]) * 64
    tdt = {"f16": torch.float16, "bf16": torch.bfloat16}[w.dtype]
    p = args.dropout if args.dropout > 0 else 0.1
    drop = (p, 220808124)
    n_sets = max(2, min(8, -(-(1 << 30) // (8 * t * hid * 2)) + 1))
    ws_bytes = fmha.fmha_dropout_add_ln_bwd_workspace_size(t, hid)

    class Set:
        def __init__(self):
            g = lambda: torch.randn((t, hid), dtype=torch.float32, device="cuda").to(tdt)
            self.x, self.r, self.dy = g(), g(), g()
            self.y, self.z, self.dx, self.dr = (torch.empty((t, hid), dtype=tdt, device="cuda") for _ in range(4))
            self.mu, self.rstd = (torch.empty(t, dtype=torch.float32, device="cuda") for _ in range(2))
            self.gamma = 1 + 0.1 * torch.randn(hid, dtype=torch.float32, device="cuda")
            self.beta = 0.1 * torch.randn(hid, dtype=torch.float32, device="cuda")
            self.dgamma, self.dbeta = (torch.empty(hid, dtype=torch.float32, device="cuda") for _ in range(2))
            self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

        def fwd(self):
            fmha.fmha_dropout_add_ln_fwd(self.x, self.r, self.gamma, self.beta, 1e-12, self.y, self.z, self.mu,
                                         self.rstd, dropout=drop)

        def bwd(self):
            fmha.fmha_dropout_add_ln_bwd(self.dy, self.z, self.mu, self.rstd, self.gamma, 1e-12, self.dx, self.dr,
                                         self.dgamma, self.dbeta, self.ws, dropout=drop)

    sets = [Set() for _ in range(n_sets)]
    for _ in range(max(1, args.warmup // n_sets)):
        for x in sets:
            x.fwd(); x.bwd()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        x = sets[i % n_sets]
        x.fwd(); x.bwd()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for i in range(args.steps):
        x = sets[i % n_sets]
        evs[i][0].record(); x.fwd(); evs[i][1].record(); x.bwd(); evs[i][2].record()
    torch.cuda.synchronize()
    names = ("ln_fwd_kernel", "ln_bwd (rows + columns)")
    k_ms = {nm: sum(e[j].elapsed_time(e[j + 1]) for e in evs) / args.steps for j, nm in enumerate(names)}
    row = hid * 2
    alg = {names[0]: t * (4 * row + 8) + 8 * hid,                       # x, r in; y, z out; mu, rstd; gamma, beta
           names[1]: t * (4 * row + 8) + 12 * hid + 2 * ws_bytes}       # dy, z in; dx, dr out; column sums out and in
    dom = max(k_ms, key=k_ms.get)
    gbs = {k: alg[k] / (k_ms[k] * 1e-3) / 1e9 for k in names}
    out = {"metric": "Dropout+Add+LayerNorm fwd+bwd, algorithmic GB/s",
           "value": round(sum(alg.values()) / sec / 1e9, 1), "unit": "GB/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 5),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": w.name + "_hidden_rows", "baseline_config": args.config, "rows": t,
                      "hidden": hid, "storage": w.dtype, "dropout_p": p, "buffer_sets": n_sets},
           "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(gbs[dom], 1), "peak": HBM_GBS,
                        "unit": "GB/s", "frac": round(gbs[dom] / HBM_GBS, 4),
                        "traffic": MEASURED_TRAFFIC_OTHER_CFG3.get(dom) if (args.config == 3 and args.dropout == 0) else None,
                        "avg_launch_ms": round(k_ms[dom], 5),
                        "kernels_ms": {k: round(v, 5) for k, v in k_ms.items()},
                        "kernels_GBs": {k: round(v, 1) for k, v in gbs.items()},
                        "algorithmic_bytes": alg}}
    if not args.no_cpu_baseline:
        from oracle import layernorm as oln
        n = min(t, 4096)
        f = lambda a: a[:n].double().cpu().numpy()
        x0 = sets[0]
        t0 = time.perf_counter()
        oln.fwd(f(x0.x), f(x0.r), x0.gamma.cpu().numpy(), x0.beta.cpu().numpy(), 1e-12)
        oln.bwd(f(x0.dy), f(x0.x), f(x0.r), x0.gamma.cpu().numpy(), 1e-12)
        csec = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(sum(alg.values()) * n / t / csec / 1e9, 4), "unit": "GB/s", "cores": 1,
                               "kind": "oracle", "sample": "%d of %d rows, no dropout, fwd+bwd, %.2f s" % (n, t, csec)}
    print(json.dumps(out))


def bench_embedding(args, torch, fmha, wl):
    """Embedding backward on the workload's token count: T gradient rows of H*64 16-bit values
    scattered onto a 30 522-row weight gradient (BERT's word-piece vocabulary) with Zipf-distributed
    ids.  A step = one accumulation into an already cleared weight gradient; both work splits are
    timed; the roofline entry prices the default (die-aware) one against HBM traffic."""
    w = wl.WORKLOADS[args.config]
    b = wl.make_workload(args.config, backward=False)
    t, hid, vocab = int(b["total_tokens"]), int(b["heads"]) * 64, 30522
    tdt = {"f16": torch.float16, "bf16": torch.bfloat16}[w.dtype]
    ids_np = wl.zipf_token_ids(t, vocab, w.seed + 100)
    distinct = int(np.unique(ids_np).size)
    top = int(np.bincount(ids_np).max())
    n_sets = max(2, min(8, -(-(1 << 30) // (t * hid * 2 + vocab * hid * 2)) + 1))

    class Set:
        def __init__(self):
            self.dy = torch.randn((t, hid), dtype=torch.float32, device="cuda").to(tdt)
            self.ids = torch.from_numpy(ids_np).cuda()
            self.dw = torch.zeros((vocab, hid), dtype=tdt, device="cuda")

    sets = [Set() for _ in range(n_sets)]

    def timed_events(plain, no_die=False):
        for x in sets:
            fmha.fmha_embedding_bwd(x.dy, x.ids, x.dw, plain_split=plain, no_die_split=no_die)
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
        for i in range(args.steps):
            x = sets[i % n_sets]
            evs[i][0].record()
            fmha.fmha_embedding_bwd(x.dy, x.ids, x.dw, plain_split=plain, no_die_split=no_die)
            evs[i][1].record()
        torch.cuda.synchronize()
        return sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps

    ms_die, ms_plain, ms_nodie = timed_events(False), timed_events(True), timed_events(False, True)

    # the variant without atomics: the sort (once per batch of indices) and the backward call
    # that uses it, timed separately
    ws = [torch.empty(fmha.fmha_embedding_sort_workspace_size(t, hid), dtype=torch.uint8, device="cuda") for _ in sets]

    def timed_sorted(which):
        def call(i):
            x = sets[i % n_sets]
            if which == "sort":
                fmha.fmha_embedding_sort(x.ids, hid, vocab, ws[i % n_sets])
            else:
                fmha.fmha_embedding_bwd_sorted(x.dy, ws[i % n_sets], x.dw)
        for i in range(n_sets):
            call(i)
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
        for i in range(args.steps):
            evs[i][0].record()
            call(i)
            evs[i][1].record()
        torch.cuda.synchronize()
        return sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps

    ms_sort, ms_sorted = timed_sorted("sort"), timed_sorted("bwd")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        x = sets[i % n_sets]
        fmha.fmha_embedding_bwd(x.dy, x.ids, x.dw)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    row = hid * 2
    alg = t * row + t * 4 + 2 * distinct * row     # gradient rows in, ids, one read-modify-write per touched weight row
    out = {"metric": "embedding backward, gradient rows per second", "value": round(t / sec, 1), "unit": "rows/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 5),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
           "config": {"workload": w.name + "_token_ids", "baseline_config": args.config, "rows": t, "hidden": hid,
                      "vocab": vocab, "ids": "Zipf(1.0), seeded", "distinct_ids": distinct,
                      "most_frequent_id_count": top, "buffer_sets": n_sets},
           "roofline": {"bound": "hbm", "kernel": "embedding_bwd_window_kernel",
                        "achieved": round(alg / (ms_die * 1e-3) / 1e9, 1), "peak": HBM_GBS, "unit": "GB/s",
                        "frac": round(alg / (ms_die * 1e-3) / 1e9 / HBM_GBS, 4),
                        "traffic": MEASURED_TRAFFIC_OTHER_CFG3["embedding_bwd_window_kernel"] if args.config == 3 else None,
                        "avg_launch_ms": round(ms_die, 5), "algorithmic_bytes": alg,
                        "kernels_ms": {"embedding_bwd_window_kernel (default: duplicates merged, split by die)": round(ms_die, 5),
                                       "embedding_bwd_window_kernel (duplicates merged, no die split)": round(ms_nodie, 5),
                                       "embedding_bwd_kernel (plain: one token per wavefront)": round(ms_plain, 5)},
                        "packed_atomics_per_s": round(t * hid / 2 / (ms_die * 1e-3), 1)},
           "sorted_variant": {"what": "fmha_embedding_sort once per batch of indices, then fmha_embedding_bwd_sorted: "
                                      "fp32 sums in sorted order, one write per weight row, no atomics",
                              "sort_ms": round(ms_sort, 5), "backward_ms": round(ms_sorted, 5),
                              "rows_per_s": round(t / (ms_sorted * 1e-3), 1),
                              "rows_per_s_with_sort": round(t / ((ms_sorted + ms_sort) * 1e-3), 1),
                              "hbm_GBs": round(alg / (ms_sorted * 1e-3) / 1e9, 1),
                              "hbm_frac": round(alg / (ms_sorted * 1e-3) / 1e9 / HBM_GBS, 4)}}
    if not args.no_cpu_baseline:
        from oracle import embedding as oemb
        n = min(t, 20000)
        x = sets[0].dy[:n].double().cpu().numpy()
        t0 = time.perf_counter()
        oemb.embedding_bwd(x, ids_np[:n], vocab)
        csec = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(n / csec, 1), "unit": "rows/s", "cores": 1, "kind": "oracle",
                               "sample": "%d of %d rows, %.2f s" % (n, t, csec)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
