#!/usr/bin/env python3
"""Benchmark of paged decode attention over prefix-aliased KV on one MI355X.

One step = one fea_decode_attention call (alias detection + KV sweep + merge)
for a whole batch: every request produces one token's attention output.  Tables,
q and the KV pool are resident in HBM before the timed region.  The KV pool is
replicated so that consecutive steps touch different memory and the 256 MB
memory-side cache cannot serve them ("cold", the headline); a warm figure on a
single replica is reported next to it.

Prints ONE JSON line on stdout.  --suite additionally measures all five batch
shapes and the homogeneous-vs-heterogeneous comparisons; it and the other extra
modes write their lines as .jsonl files into the folder given by --out.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as W  # noqa: E402

HBM_PEAK_GBS = 8000.0
OUT_DIR = os.path.join(ROOT, "gpurun_out")   # --out


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Case:
    """One batch on the device: tables from the library, q and a replicated KV pool."""

    def __init__(self, spec, replicas_bytes=1 << 30, seed_shift=0, tokens=None, max_group=0, label=None,
                 extra_blocks=0, extra_cols=0):
        import torch
        import paper_2605_06046_amd as fea
        self.fea, self.torch, self.spec = fea, torch, spec
        self.label = label or spec.name
        wl = W.generate(spec, with_kv=False) if tokens is None else tokens
        if extra_blocks or extra_cols:   # room for the history to grow (decode loop)
            import dataclasses
            wl = dataclasses.replace(wl, num_blocks=wl.num_blocks + extra_blocks,
                                     max_blocks_per_seq=wl.max_blocks_per_seq + extra_cols)
        self.wl = wl
        t0 = time.perf_counter()
        pool = fea.fea_kv_alloc(wl.num_blocks, 16, wl.perm_seed)
        bt, lens, _, _ = fea.fea_build_block_tables(pool, wl.tokens, wl.tok_offsets, wl.max_blocks_per_seq)
        self.table_build_s = time.perf_counter() - t0
        self.pool = pool
        self.bt, self.lens = bt, lens
        self.B = bt.shape[0]
        live = np.unique(bt[bt >= 0])
        self.unique_blocks = int(len(live))
        self.logical_blocks = int((bt >= 0).sum())
        es = 2 if spec.dtype == "bf16" else 4
        self.block_bytes = 16 * 2 * spec.num_kv_heads * spec.head_dim * es      # K and V of one block
        self.unique_bytes = self.unique_blocks * self.block_bytes
        self.logical_bytes = self.logical_blocks * self.block_bytes
        pool_bytes = wl.num_blocks * self.block_bytes
        self.R = max(1, min(8, -(-replicas_bytes // max(self.unique_bytes, 1)))) if pool_bytes < (2 << 30) else 1
        dt = torch.bfloat16 if spec.dtype == "bf16" else torch.float32
        g = torch.Generator(device="cuda")
        g.manual_seed(spec.seed + seed_shift)
        shape = (self.R, wl.num_blocks, spec.num_kv_heads, 16, spec.head_dim)
        self.k = torch.empty(shape, dtype=dt, device="cuda")
        self.v = torch.empty(shape, dtype=dt, device="cuda")
        for r in range(self.R):                      # chunked: randn makes float32 first
            for cache in (self.k, self.v):
                for b0 in range(0, wl.num_blocks, 8192):
                    b1 = min(wl.num_blocks, b0 + 8192)
                    cache[r, b0:b1] = torch.randn((b1 - b0,) + shape[2:], generator=g, device="cuda",
                                                  dtype=torch.float32).to(dt)
        q = wl.q
        self.q = (torch.from_numpy(q.view(np.int16)).cuda().view(torch.bfloat16) if q.dtype == np.uint16
                  else torch.from_numpy(q).cuda())
        self.dbt = torch.from_numpy(bt).cuda()
        self.dl = torch.from_numpy(lens).cuda()
        self.out = torch.empty_like(self.q)
        self.params = fea.AttnParams(spec.num_q_heads, spec.num_kv_heads, spec.head_dim,
                                     fea.FEA_DTYPE_BF16 if spec.dtype == "bf16" else fea.FEA_DTYPE_F32,
                                     max_group=max_group)
        nbytes = fea.fea_decode_workspace_bytes(self.params, self.B, bt.shape[1])
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        # argument lists prepared once: the timed loop only makes the foreign call
        lib = fea.load_library()
        self._fn = lib.fea_decode_attention
        vp = C.c_void_p
        self._args = [
            (C.byref(self.params), vp(self.q.data_ptr()), vp(self.k[r].data_ptr()), vp(self.v[r].data_ptr()),
             vp(self.dbt.data_ptr()), bt.shape[1], vp(self.dl.data_ptr()), self.B, vp(self.out.data_ptr()),
             vp(self.ws.data_ptr()), nbytes)
            for r in range(self.R)]

    def step(self, r, stream_ptr):
        rc = self._fn(*self._args[r], stream_ptr)
        if rc != 0:
            raise RuntimeError(self.fea.load_library().fea_last_error().decode())

    def time_steps(self, steps, warmup, cold=True, graph=False):
        """Mean milliseconds per step over `steps` back-to-back calls."""
        torch = self.torch
        R = self.R if cold else 1
        stream = torch.cuda.current_stream()
        sp = C.c_void_p(stream.cuda_stream)
        for s in range(warmup):
            self.step(s % R, sp)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if graph:
            side = torch.cuda.Stream()
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                spg = C.c_void_p(side.cuda_stream)
                for s in range(R):
                    self.step(s, spg)
                side.synchronize()
                with torch.cuda.graph(gr, stream=side):
                    for s in range(R):
                        self.step(s, spg)
            reps = max(1, steps // R)
            gr.replay()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                gr.replay()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / (reps * R)
        e0.record()
        for s in range(steps):
            self.step(s % R, sp)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    def kernel_times(self, steps, cold=True):
        """Average (plan, sweep, merge) durations in ms over `steps` back-to-back calls (no
        host sync between), from HIP events attached to each dispatch on the launch stream."""
        torch, fea = self.torch, self.fea
        if profiler_attached():          # the tool times the dispatches itself; the library refuses its own events then
            return None
        R = self.R if cold else 1
        sp = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        for s in range(4):
            self.step(s % R, sp)
        fea.fea_profile_enable(steps, -1)
        try:
            for s in range(steps):
                self.step(s % R, sp)
            return np.mean([fea.fea_profile_read(s) for s in range(steps)], axis=0)
        finally:
            fea.fea_profile_enable(0, -1)

    def time_model_step(self, layers=32, reps=10):
        """Mean ms per attention call when one plan serves `layers` calls (the layers of
        one decode step share tables and lengths): 1 planning call + layers-1 reusing calls."""
        torch, fea = self.torch, self.fea
        sp = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        reuse = fea.AttnParams(self.spec.num_q_heads, self.spec.num_kv_heads, self.spec.head_dim,
                               self.params.dtype, max_group=self.params.max_group, flags=fea.FEA_FLAG_REUSE_PLAN)
        args_reuse = [(C.byref(reuse),) + a[1:] for a in self._args]

        def one_step(base):
            self.step(base % self.R, sp)
            for l in range(1, layers):
                rc = self._fn(*args_reuse[(base + l) % self.R], sp)
                if rc != 0:
                    raise RuntimeError(fea.load_library().fea_last_error().decode())
        one_step(0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for r in range(reps):
            one_step(r)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (reps * layers)

    def measure(self, steps, warmup, graph=False, light=False):
        ms_cold = self.time_steps(steps, warmup, cold=True, graph=graph)
        ms_warm = self.time_steps(steps, warmup, cold=False, graph=graph)
        kt = self.kernel_times(min(steps, 200))
        info = self.fea.fea_decode_plan_info(self.ws)
        if kt is None:
            kt = [float("nan")] * 3
        return {
            "workload": self.label, "B": self.B, "ms_per_step": ms_cold, "ms_per_step_warm": ms_warm,
            "tokens_per_s": self.B / (ms_cold * 1e-3), "tokens_per_s_warm": self.B / (ms_warm * 1e-3),
            "unique_kv_bytes": self.unique_bytes, "logical_kv_bytes": self.logical_bytes,
            "unique_kv_gbs": self.unique_bytes / (ms_cold * 1e-3) / 1e9,
            "unique_kv_gbs_warm": self.unique_bytes / (ms_warm * 1e-3) / 1e9,
            "logical_kv_gbs": self.logical_bytes / (ms_cold * 1e-3) / 1e9,
            "frac_hbm_peak_step": self.unique_bytes / (ms_cold * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "kernel_us": {"plan": kt[0] * 1e3, "sweep": kt[1] * 1e3, "merge": kt[2] * 1e3},
            "sweep_gbs": self.unique_bytes / (kt[1] * 1e-3) / 1e9,
            "ms_per_call_plan_shared_by_32_layers": None if light else self.time_model_step(),
            "replicas": self.R, "plan": info, "table_build_ms": self.table_build_s * 1e3,
            "table_build_tokens_per_s": len(self.wl.tokens) / self.table_build_s,
        }


def profiler_attached():
    """rocprofv3 (and tools like it) announce themselves through this variable."""
    return bool(os.environ.get("ROCP_TOOL_LIBRARIES"))


def cpu_baseline(case, budget_s=14.0):
    """The float64 oracle, as it stands, on the host cores: whole requests of the same batch, for
    about half of `budget_s` with the numerical library's threads as they come (all cores) and for
    the other half limited to one thread."""
    from oracle.attention import decode_attention
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threadpool_limits, threads = None, os.cpu_count() or 1
    q = case.q.float().cpu().numpy()
    k = case.k[0].float().cpu().numpy()
    v = case.v[0].float().cpu().numpy()
    decode_attention(q, k, v, case.bt, case.lens, requests=[0])          # warm

    def leg(seconds):
        done, t0 = 0, time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            decode_attention(q, k, v, case.bt, case.lens, requests=[done % case.B])
            done += 1
        return done, time.perf_counter() - t0

    done, dt = leg(budget_s / 2)
    res = {"value": done / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
           "nproc": os.cpu_count(),
           "sample": f"{done} request-steps cycling over the {case.B} requests of {case.label} "
                     f"(all heads, full history each), {dt:.1f} s wall, numerical library threads as configured"}
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            done1, dt1 = leg(budget_s / 2)
        res["one_thread"] = {"value": done1 / dt1, "unit": "tokens/s", "cores": 1,
                             "sample": f"{done1} request-steps of the same batch, {dt1:.1f} s wall"}
    return res


def hbm_calibration(gib=2):
    """What the box streams through the sweep's own fetch path (no computation): GB/s over a buffer
    far larger than the memory-side cache, blocks in order and scattered."""
    import torch
    import paper_2605_06046_amd as fea
    buf = torch.empty(gib << 30, dtype=torch.uint8, device="cuda")
    buf.view(torch.int32).fill_(0x3F803F80)
    res = {"buffer_GiB": gib, "linear_gbs": fea.fea_stream_read_gbs(buf, scattered=False, repeats=5),
           "scattered_gbs": fea.fea_stream_read_gbs(buf, scattered=True, repeats=5)}
    del buf
    torch.cuda.empty_cache()
    return res


def compact(case, m):
    """One entry of the default line's `configs` block."""
    sweep_us = m["kernel_us"]["sweep"]
    return {"B": case.B, "ms_per_step": m["ms_per_step"], "ms_per_step_warm": m["ms_per_step_warm"],
            "tokens_per_s": m["tokens_per_s"],
            "unique_kv_MB": case.unique_bytes / 1e6, "logical_kv_MB": case.logical_bytes / 1e6,
            "kernel_us": m["kernel_us"],
            "sweep_frac_of_hbm_peak": case.unique_bytes / (sweep_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
            "step_frac_of_hbm_peak": m["frac_hbm_peak_step"],
            "groups": m["plan"]["groups"], "variant": m["plan"]["variant"], "kv_replicas_rotated": case.R,
            "traffic_over_unique": (lambda t: None if t is None else t / case.unique_bytes)(
                traffic_from_profile(case.label, m["plan"]))}


def config_cases():
    """(label, Case factory) for the other batch shapes of the measurement and the equal-size
    homogeneous-vs-mixed comparisons (H2: 32 requests from one prefix group vs 4 from each of 8;
    H3: the one-prefix batch vs the same lengths with nothing shared)."""
    import dataclasses
    base = W.CONFIGS["c3"]
    yield "c1", lambda: Case(W.CONFIGS["c1"])
    yield "c3", lambda: Case(W.CONFIGS["c3"])
    yield "c4", lambda: Case(W.CONFIGS["c4"])
    yield "c5", lambda: Case(W.CONFIGS["c5"])
    homo = dataclasses.replace(base, name="H2_homogeneous", groups=((32, 4096),), interleave=False)
    mixed = dataclasses.replace(base, name="H2_mixed", groups=tuple((4, 4096) for _ in range(8)))
    yield "H2_homogeneous", lambda: Case(homo, label=homo.name)
    yield "H2_mixed", lambda: Case(mixed, label=mixed.name)

    def unshared():
        c2 = W.CONFIGS["c2"]
        wl = W.generate(c2, with_kv=False)
        rng = np.random.default_rng(7)
        toks = wl.tokens.copy()
        for i in range(c2.batch):                     # re-draw every prefix: same lengths, no common tokens
            toks[wl.tok_offsets[i]:wl.tok_offsets[i] + 4096] = rng.integers(0, W.VOCAB, size=4096, dtype=np.int32)
        wl_u = dataclasses.replace(wl, tokens=toks, num_blocks=int(sum(-(-int(L) // 16) for L in wl.seq_lens)))
        return Case(dataclasses.replace(c2, name="H3_unshared"), tokens=wl_u, label="H3_unshared")
    yield "H3_unshared", unshared


def traffic_from_profile(workload, plan):
    """HBM bytes per sweep launch from the committed counter summary, if it is current: taken with
    this sweep kernel source and with the plan (items, partial rows, groups, piece size) that the
    kernel executes now."""
    path = os.path.join(ROOT, "profiles", f"sweep_mfma_{workload}_pmc.json")
    try:
        d = json.load(open(path))
        same = d.get("kernel_rev") == kernel_rev() and d.get("plan") == plan
        return d.get("traffic_bytes_per_launch") if same else None
    except Exception:
        return None


def kernel_rev():
    from paper_2605_06046_amd.profile_summary import kernel_rev as rev
    return rev(ROOT)


def main():
    global OUT_DIR
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="c2", choices=sorted(W.CONFIGS))
    ap.add_argument("--graph", action="store_true", help="replay the steps from a captured HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true",
                    help="measure only --workload (skip the other batch shapes and the homogeneous-vs-mixed comparisons)")
    ap.add_argument("--no-hbm-calibration", action="store_true",
                    help="skip the streaming-read measurement of what the box delivers to the sweep's fetch path")
    ap.add_argument("--out", default=OUT_DIR, help="folder for the .jsonl files of the extra modes")
    ap.add_argument("--suite", action="store_true", help="also run all shapes and the homogeneity comparisons")
    ap.add_argument("--decode-loop", type=int, default=0, metavar="N",
                    help="also run N decode steps (extend, append, attend over the KV replicas as layers)")
    ap.add_argument("--scheduler", action="store_true",
                    help="also compare first-come-first-served batches with batches formed by the Chunked Hash Tree")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="also sweep the batch size on one shared 10K-token prefix vs five of them (Experiment 5's shape)")
    ap.add_argument("--paper-shapes", action="store_true",
                    help="also run the batch shapes of the paper's Experiments 2 (shared fraction), 4 (sharing levels) "
                         "and 6 (batching strategies over eight prefix groups)")
    ap.add_argument("--policies", type=int, default=0, metavar="ROUNDS",
                    help="also form ROUNDS batches per stop policy (first-come-first-served, rule-based, bandit, "
                         "Q-learning) from a five-group queue, the measured decode throughput as the reward")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run a plain 1 GiB device-to-device copy three times (known traffic, for counter runs)")
    args = ap.parse_args()
    OUT_DIR = args.out
    if args.gpus != 1:
        log("bench.py: this library runs on one GPU only (no collectives, no sharding); use --gpus 1")
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(2)
    import paper_2605_06046_amd as fea
    fea.load_library()

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    calib = None if args.no_hbm_calibration else hbm_calibration()
    if calib:
        log(json.dumps({"hbm_calibration": calib}))
    spec = W.CONFIGS[args.workload]
    case = Case(spec)
    m = case.measure(args.steps, args.warmup, graph=args.graph)
    log(json.dumps(m))
    sweep_s = m["kernel_us"]["sweep"] * 1e-6
    achieved = case.unique_bytes / sweep_s / 1e9          # nan under a profiler (it times the kernels itself)
    nn = lambda x: None if x != x else x                  # NaN -> null
    line = {
        "metric": "decode-attn tokens/s (unique-KV HBM GB/s vs peak in roofline)",
        "value": m["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if spec.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: B={case.B}, Hq={spec.num_q_heads}, Hkv={spec.num_kv_heads}, "
                               f"d={spec.head_dim}, block 16, groups={[list(g) for g in spec.groups[:2]]}"
                               f"{'...' if len(spec.groups) > 2 else ''}, suffix U{list(spec.suffix)}",
                   "mode": "graph" if args.graph else "eager", "kv_replicas_rotated": case.R,
                   "unique_kv_MB": case.unique_bytes / 1e6, "logical_kv_MB": case.logical_bytes / 1e6},
        "unique_kv_gbs": m["unique_kv_gbs"], "frac_hbm_peak_whole_step": m["frac_hbm_peak_step"],
        "warm": {"tokens_per_s": m["tokens_per_s_warm"], "unique_kv_gbs": m["unique_kv_gbs_warm"]},
        "kernel_us": {k: nn(v) for k, v in m["kernel_us"].items()}, "plan": m["plan"],
        "plan_shared_by_32_layers": {"ms_per_call": m["ms_per_call_plan_shared_by_32_layers"],
                                     "tokens_per_s": case.B / (m["ms_per_call_plan_shared_by_32_layers"] * 1e-3)},
        "host_table_build": {"ms": m["table_build_ms"], "tokens_per_s": m["table_build_tokens_per_s"]},
        "roofline": {"bound": "hbm", "achieved": nn(achieved), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": nn(achieved / HBM_PEAK_GBS), "traffic": traffic_from_profile(args.workload, m["plan"]),
                     "kernel": ("sweep_generic_kernel", "sweep_mfma_kernel", "decode_small_kernel")[m["plan"]["variant"]],
                     "bytes_per_launch": case.unique_bytes,
                     "achievable_gbs": None if calib is None else calib["scattered_gbs"],
                     "frac_of_achievable": None if calib is None else nn(achieved / calib["scattered_gbs"])},
        "hbm_calibration": calib, "profiler_attached": profiler_attached(),
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(case)
    else:
        line["cpu_baseline"] = None

    if not args.no_configs:
        # every batch shape of the measurement in the same line, the headline workload included
        configs = {args.workload: compact(case, m)}
        del case
        case = None
        torch.cuda.empty_cache()
        for label, make in config_cases():
            if label == args.workload:
                continue
            c = make()
            heavy = label == "c5"
            mm = c.measure(40 if heavy else max(50, args.steps // 4), 5 if heavy else max(10, args.warmup // 4),
                           graph=args.graph, light=True)
            configs[label] = compact(c, mm)
            log(json.dumps({label: configs[label]}))
            del c
            torch.cuda.empty_cache()
        line["configs"] = {k: {kk: (nn(vv) if isinstance(vv, float) else vv) for kk, vv in v.items()} for k, v in configs.items()}
        ratio = lambda slow, fast: configs[slow]["ms_per_step"] / configs[fast]["ms_per_step"]
        line["homogeneous_vs_mixed"] = {
            "H2_equal_size_equal_logical_kv": {"homogeneous_ms": configs["H2_homogeneous"]["ms_per_step"],
                                               "mixed_ms": configs["H2_mixed"]["ms_per_step"],
                                               "speedup": ratio("H2_mixed", "H2_homogeneous")},
        }
        if "c2" in configs:
            line["homogeneous_vs_mixed"]["H3_shared_vs_unshared_same_lengths"] = {
                "shared_ms": configs["c2"]["ms_per_step"], "unshared_ms": configs["H3_unshared"]["ms_per_step"],
                "speedup": ratio("H3_unshared", "c2")}

    if args.decode_loop > 0:
        os.makedirs(OUT_DIR, exist_ok=True)
        with open(os.path.join(OUT_DIR, "decode_loop.jsonl"), "w") as f:
            for layers, every in ((None, 1), (None, 32), (1, 1), (1, 32)):
                res = decode_loop(args.decode_loop, layers, every)
                f.write(json.dumps(res) + "\n")
                log(json.dumps(res))
                torch.cuda.empty_cache()
    if args.scheduler and not args.suite:
        os.makedirs(OUT_DIR, exist_ok=True)
        with open(os.path.join(OUT_DIR, "scheduler.jsonl"), "w") as f:
            case = None
            torch.cuda.empty_cache()
            for res in scheduler_comparison(max(50, args.steps // 4), max(10, args.warmup // 2), args.graph):
                f.write(json.dumps(res) + "\n")
                log(json.dumps(res))
    for flag, name, gen in ((args.batch_sweep, "batch_sweep.jsonl", lambda: batch_sweep(max(50, args.steps // 4), max(10, args.warmup // 2))),
                            (args.paper_shapes, "paper_shapes.jsonl", lambda: paper_shapes(max(50, args.steps // 4), max(10, args.warmup // 2))),
                            (args.policies > 0, "policies.jsonl", lambda: policy_comparison(args.policies))):
        if flag:
            os.makedirs(OUT_DIR, exist_ok=True)
            case = None
            torch.cuda.empty_cache()
            with open(os.path.join(OUT_DIR, name), "w") as f:
                for res in gen():
                    f.write(json.dumps(res) + "\n")
                    f.flush()
                    log(json.dumps(res))
    if args.suite:
        os.makedirs(OUT_DIR, exist_ok=True)
        with open(os.path.join(OUT_DIR, "suite.jsonl"), "w") as f:
            f.write(json.dumps(m) + "\n")
            case = None
            torch.cuda.empty_cache()
            for res in run_suite(args):
                f.write(json.dumps(res) + "\n")
                f.flush()
                log(json.dumps(res))
    print(json.dumps(line), flush=True)


def run_suite(args):
    """All shapes, plus: H2 homogeneous vs mixed batch of equal size and logical KV,
    H3 shared vs unshared batch of equal lengths, H1 one mixed launch vs eight
    homogeneous launches over the same KV."""
    import dataclasses
    import torch
    steps, warm = max(50, args.steps // 4), max(10, args.warmup // 2)
    for name in ("c1", "c3", "c4", "c5"):
        c = Case(W.CONFIGS[name])
        yield c.measure(steps if name != "c5" else 40, warm if name != "c5" else 5, graph=args.graph)
        del c
        torch.cuda.empty_cache()
    base = W.CONFIGS["c3"]
    # H2: 32 requests of one group vs 32 requests drawn 4 from each of the 8 groups
    homo = dataclasses.replace(base, name="H2_homogeneous", groups=((32, 4096),), interleave=False)
    mixed = dataclasses.replace(base, name="H2_mixed", groups=tuple((4, 4096) for _ in range(8)))
    for sp in (homo, mixed):
        c = Case(sp, label=sp.name)
        yield c.measure(steps, warm, graph=args.graph)
        del c
        torch.cuda.empty_cache()
    # H3: c2 against the same lengths with nothing shared
    c2 = W.CONFIGS["c2"]
    wl = W.generate(c2, with_kv=False)
    rng = np.random.default_rng(7)
    toks = wl.tokens.copy()
    for i in range(c2.batch):                     # re-draw every prefix: same lengths, no common tokens
        toks[wl.tok_offsets[i]:wl.tok_offsets[i] + 4096] = rng.integers(0, W.VOCAB, size=4096, dtype=np.int32)
    wl_unshared = dataclasses.replace(wl, tokens=toks, num_blocks=int(sum(-(-int(L) // 16) for L in wl.seq_lens)))
    c = Case(dataclasses.replace(c2, name="H3_unshared"), tokens=wl_unshared, label="H3_unshared")
    yield c.measure(steps, warm, graph=args.graph)
    del c
    torch.cuda.empty_cache()
    # grouping switched off on the shared batch: the paper's own mechanism (cache locality only)
    c = Case(c2, max_group=1, label="c2_grouping_off")
    yield c.measure(steps, warm, graph=args.graph)
    del c
    torch.cuda.empty_cache()
    # H1: the 8 groups of c3 as 8 homogeneous launches of 32 (time summed) vs the one mixed launch above
    total_ms, total_ms_warm, B = 0.0, 0.0, 0
    for gi in range(8):
        sp = dataclasses.replace(base, name=f"H1_group{gi}", index=30 + gi, groups=((32, 4096),), interleave=False)
        c = Case(sp, replicas_bytes=1 << 30, label=sp.name)
        m = c.measure(steps, warm, graph=args.graph)
        total_ms += m["ms_per_step"]
        total_ms_warm += m["ms_per_step_warm"]
        B += c.B
        del c
        torch.cuda.empty_cache()
    yield {"workload": "H1_eight_homogeneous_launches_of_32", "B": B, "ms_per_step": total_ms,
           "ms_per_step_warm": total_ms_warm, "tokens_per_s": B / (total_ms * 1e-3)}
    yield from scheduler_comparison(steps, warm, args.graph)
    yield from device_hashing()


def device_hashing(reps=50):
    """Chunk hashes of a whole batch on the device (the chunk-parallel formulation) against the
    host function, on the token streams of c2 (64 long requests) and c5 (512 requests)."""
    import torch
    import paper_2605_06046_amd as fea
    for name in ("c2", "c5"):
        wl = W.generate(W.CONFIGS[name], with_kv=False)
        hoff = np.zeros(len(wl.tok_offsets), dtype=np.int64)
        hoff[1:] = np.cumsum(-(-np.diff(wl.tok_offsets) // 16))
        d_tok, d_toff, d_hoff = (torch.from_numpy(x).cuda() for x in (wl.tokens, wl.tok_offsets, hoff))
        d_h = torch.zeros(int(hoff[-1]), dtype=torch.int64, device="cuda")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for r in range(reps + 5):
            if r == 5:
                e0.record()
            fea.fea_chunk_hashes_device(d_tok, d_toff, d_hoff, d_h)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        t0 = time.perf_counter()
        host = [fea.fea_chunk_hashes(wl.request_tokens(i)) for i in range(wl.spec.batch)]
        host_us = (time.perf_counter() - t0) * 1e6
        same = bool(np.array_equal(np.concatenate(host), d_h.cpu().numpy().view(np.uint64)))
        yield {"workload": f"device_chunk_hashes_{name}", "B": wl.spec.batch, "tokens": int(len(wl.tokens)),
               "us_per_call": us, "tokens_per_s": len(wl.tokens) / (us * 1e-6), "host_us": host_us,
               "host_tokens_per_s": len(wl.tokens) / (host_us * 1e-6), "equal_to_host": same}


def decode_loop(n_steps, layers=None, replan_every=1):
    """A run of decode steps on the c2 batch: per step the host extends tables and lengths by one
    token, and every layer (a replica of the KV pool stands for a layer's cache) appends its new K/V
    rows and attends; the plan of a step is shared by its layers, and made anew (alias detection and
    work split) only every replan_every-th step: in between the first layer stretches the plan at hand
    to the lengths of now."""
    import torch
    import paper_2605_06046_amd as fea
    spec = W.CONFIGS["c2"]
    c = Case(spec, extra_blocks=spec.batch * (n_steps // 16 + 2), extra_cols=n_steps // 16 + 2)
    L = c.R if layers is None else min(layers, c.R)
    p_plan = c.params
    p_reuse = fea.AttnParams(spec.num_q_heads, spec.num_kv_heads, spec.head_dim, p_plan.dtype, flags=fea.FEA_FLAG_REUSE_PLAN)
    p_refresh = fea.AttnParams(spec.num_q_heads, spec.num_kv_heads, spec.head_dim, p_plan.dtype, flags=fea.FEA_FLAG_REFRESH_PLAN)
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    shape_new = (c.B, spec.num_kv_heads, spec.head_dim)
    k_new = torch.randn(shape_new, generator=g, device="cuda").to(c.k.dtype)
    v_new = torch.randn(shape_new, generator=g, device="cuda").to(c.k.dtype)
    bt, lens = c.bt, c.lens
    # One pinned staging slot per step: the device runs behind the host, and a slot that were written
    # again before its copy has run would hand the device lengths that are ahead of its tables.
    n_slots = n_steps + 5
    pin_l = torch.empty((n_slots,) + lens.shape, dtype=torch.int32).pin_memory()
    pin_t = torch.empty((n_slots,) + bt.shape, dtype=torch.int32).pin_memory()
    slot = [0]

    # the foreign calls with their arguments marshalled once: the loop is meant to show the device's
    # pace, and a Python driver that converts tensors on every call would set it instead
    lib = fea.load_library()
    vp = C.c_void_p
    sp = vp(torch.cuda.current_stream().cuda_stream)
    n_new = C.c_int32()
    ext_args = (c.pool.handle, vp(bt.ctypes.data), bt.shape[1], vp(lens.ctypes.data), c.B, C.byref(n_new))
    app_args = [(C.byref(p_plan), vp(k_new.data_ptr()), vp(v_new.data_ptr()), vp(c.k[l].data_ptr()), vp(c.v[l].data_ptr()),
                 vp(c.dbt.data_ptr()), bt.shape[1], vp(c.dl.data_ptr()), c.B, sp) for l in range(L)]
    att_args = [(C.byref(p_plan if l == 0 else p_reuse),) + c._args[l][1:] + (sp,) for l in range(L)]
    att_refresh = (C.byref(p_refresh),) + c._args[0][1:] + (sp,)
    t_lens, t_bt = torch.from_numpy(lens), torch.from_numpy(bt)      # views of the host arrays the library updates

    def check(rc):
        if rc != 0:
            raise RuntimeError(lib.fea_last_error().decode())

    def step():
        check(lib.fea_kv_extend(*ext_args))
        j = slot[0]
        slot[0] += 1
        if n_new.value:      # tables first: lengths never get ahead of them on the device
            pin_t[j].copy_(t_bt); c.dbt.copy_(pin_t[j], non_blocking=True)
        pin_l[j].copy_(t_lens); c.dl.copy_(pin_l[j], non_blocking=True)
        for l in range(L):
            check(lib.fea_kv_append(*app_args[l]))
            check(lib.fea_decode_attention(*(att_refresh if l == 0 and j % replan_every else att_args[l])))

    for _ in range(5):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(n_steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = e0.elapsed_time(e1) / n_steps
    return {"workload": f"decode_loop_c2_{L}_layers", "B": c.B, "decode_steps": n_steps, "layers": L,
            "new_plan_every": replan_every, "ms_per_decode_step": ms, "us_per_layer": ms * 1e3 / L, "tokens_per_s_per_layer_call": c.B / (ms * 1e-3 / L),
            "tokens_per_s_model_of_these_layers": c.B / (ms * 1e-3), "host_wall_ms_per_step": wall * 1e3 / n_steps,
            "final_len_mean": float(lens.mean())}


def scheduler_comparison(steps, warm, graph):
    """The 256 requests of c3 (8 prefix groups, arriving interleaved) served as batches of 32
    chosen first-come-first-served or by the Chunked Hash Tree with the rule-based stop
    policy: summed attention time over the 8 batches of each schedule, and the tree's
    time per operation."""
    import dataclasses
    import torch
    import paper_2605_06046_amd as fea
    base = W.CONFIGS["c3"]
    wl = W.generate(base, with_kv=False)
    B = base.batch
    reqs = [wl.request_tokens(i) for i in range(B)]
    t_ops = {}
    tree = fea.Cht()
    t0 = time.perf_counter()
    for i, r in enumerate(reqs):
        tree.insert(i, tokens=r)
    t_ops["insert_ns"] = (time.perf_counter() - t0) / B * 1e9
    policy = dict(small_batch=2, loss_small=1 << 30, loss_limit=8, peers_relax=16, loss_relaxed=32)
    cht_batches, t_build, t_finish = [], 0.0, 0.0
    while tree.stats()["waiting"] > 0:
        t0 = time.perf_counter()
        ids = tree.build_batch(32, **policy)
        t_build += time.perf_counter() - t0
        cht_batches.append(ids)
        t0 = time.perf_counter()
        for rid in ids:
            tree.finish(rid)
        t_finish += time.perf_counter() - t0
    t_ops["find_best_plus_add_ns"] = t_build / B * 1e9
    t_ops["finish_ns"] = t_finish / B * 1e9
    fcfs_batches = [list(range(b0, min(B, b0 + 32))) for b0 in range(0, B, 32)]

    def sub(sel):
        toks = np.concatenate([reqs[i] for i in sel])
        offs = np.zeros(len(sel) + 1, dtype=np.int64)
        offs[1:] = np.cumsum([len(reqs[i]) for i in sel])
        return dataclasses.replace(wl, tokens=toks, tok_offsets=offs, group_of=wl.group_of[sel], q=wl.q[sel],
                                   num_blocks=int(sum(-(-len(reqs[i]) // 16) for i in sel)))

    for name, batches in (("sched_fcfs_batches_of_32", fcfs_batches), ("sched_cht_batches_of_32", cht_batches)):
        total_ms, n, groups_per_batch = 0.0, 0, []
        for k, sel in enumerate(batches):
            sp = dataclasses.replace(base, name=f"{name}_{k}")
            c = Case(sp, tokens=sub(sel), label=sp.name)
            total_ms += c.measure(steps, warm, graph=graph)["ms_per_step"]
            n += c.B
            groups_per_batch.append(int(len(set(wl.group_of[sel].tolist()))))
            del c
            torch.cuda.empty_cache()
        out = {"workload": name, "B": n, "batches": len(batches), "prefix_groups_per_batch": groups_per_batch,
               "ms_per_step": total_ms, "tokens_per_s": n / (total_ms * 1e-3)}
        if name.startswith("sched_cht"):
            out["tree_ns_per_request"] = {k: round(v) for k, v in t_ops.items()}
        yield out


def batch_sweep(steps, warm):
    """Decode-attention throughput against the batch size for a homogeneous batch (every request
    on one 10K-token prefix) and a heterogeneous one (the requests spread over five such
    prefixes, in arrival order): the shape of the paper's Experiment 5 on a Llama-3-8B layer."""
    import torch
    base = W.CONFIGS["c2"]
    for B in (5, 10, 20, 40, 80, 160, 320, 500):
        for kind, groups in (("homogeneous", ((B, 10240),)), ("heterogeneous", tuple((B // 5, 10240) for _ in range(5)))):
            sp = W.Spec(f"sweep_{kind}_{B}", 60 + (B % 50), "bf16", base.num_q_heads, base.num_kv_heads, base.head_dim,
                        groups, (64, 256), interleave=True)
            c = Case(sp, label=sp.name)
            m = c.measure(steps, warm)
            yield {"workload": sp.name, "B": c.B, "kind": kind, "ms_per_step": m["ms_per_step"],
                   "tokens_per_s": m["tokens_per_s"], "unique_kv_MB": c.unique_bytes / 1e6,
                   "logical_kv_MB": c.logical_bytes / 1e6, "kernel_us": m["kernel_us"]}
            del c
            torch.cuda.empty_cache()


def _case_from_sequences(base, name, seqs, index):
    """A Case over explicit token sequences (shape parameters and q from `base`'s layer)."""
    import dataclasses
    sp = W.Spec(name, index, "bf16", base.num_q_heads, base.num_kv_heads, base.head_dim, ((len(seqs), 0),), (1, 1))
    wl = W.generate(sp, with_kv=False)
    offs = np.zeros(len(seqs) + 1, dtype=np.int64)
    offs[1:] = np.cumsum([len(x) for x in seqs])
    nblk = int(sum(-(-len(x) // 16) for x in seqs))
    wl = dataclasses.replace(wl, tokens=np.concatenate(seqs), tok_offsets=offs, num_blocks=nblk,
                             max_blocks_per_seq=max(-(-len(x) // 16) for x in seqs) + 1,
                             group_of=np.zeros(len(seqs), dtype=np.int32))
    return Case(sp, tokens=wl, label=name)


def paper_shapes(steps, warm):
    """The batch shapes of Section 3 on a Llama-3-8B layer, decode attention only.
    Experiment 2: 100 requests of 2 048 tokens sharing the first 2048 f tokens.
    Experiment 4: 64 requests of 4 096 tokens in four 1 024-token levels, the first k levels shared
    (level 1 by all, level 2 by 16, level 3 by 4 requests each), k = 0..3.
    Experiment 6: eight prefix groups (10 240 tokens) of 100 requests served as 1x800 ... 32x25:
    summed attention time of one decode step over all batches."""
    import torch
    base = W.CONFIGS["c2"]
    rng = np.random.default_rng(W.SEED_BASE + 90)
    draw = lambda n: rng.integers(0, W.VOCAB, size=n, dtype=np.int32)

    def run(name, seqs, index, extra):
        c = _case_from_sequences(base, name, seqs, index)
        m = c.measure(steps, warm)
        out = {"workload": name, "B": c.B, "ms_per_step": m["ms_per_step"], "tokens_per_s": m["tokens_per_s"],
               "unique_kv_MB": c.unique_bytes / 1e6, "logical_kv_MB": c.logical_bytes / 1e6,
               "kernel_us": m["kernel_us"], "groups": m["plan"]["groups"]}
        out.update(extra)
        del c
        torch.cuda.empty_cache()
        return out

    for f in (0.0, 0.25, 0.5, 0.75, 1.0):
        shared = draw(int(2048 * f) // 16 * 16)
        seqs = [np.concatenate([shared, draw(2048 - len(shared))]) if len(shared) < 2048 else shared.copy()
                for _ in range(100)]
        yield run(f"exp2_shared_fraction_{f:g}", seqs, 70, {"f": f})
    for k in range(4):
        lv1 = draw(1024)
        lv2 = [draw(1024) for _ in range(4)]
        lv3 = [draw(1024) for _ in range(16)]
        seqs = []
        for i in range(64):
            parts = [lv1 if k >= 1 else draw(1024), lv2[i % 4] if k >= 2 else draw(1024),
                     lv3[i % 16] if k >= 3 else draw(1024), draw(1024)]
            seqs.append(np.concatenate(parts))
        yield run(f"exp4_levels_shared_{k}", seqs, 71, {"levels_shared": k})
    prefixes = [draw(10240) for _ in range(8)]
    reqs = [(g, np.concatenate([prefixes[g], draw(int(rng.integers(64, 257)))])) for g in range(8) for _ in range(100)]
    for n_batches in (1, 2, 4, 8, 16, 32):
        per_group = max(1, n_batches // 8)                  # batches per prefix group (homogeneous strategies)
        groups_per_batch = max(1, 8 // n_batches)
        total_ms, total_b, kus = 0.0, 0, [0.0, 0.0, 0.0]
        for b in range(n_batches):
            if n_batches <= 8:
                gs = range(b * groups_per_batch, (b + 1) * groups_per_batch)
                seqs = [x for g, x in reqs if g in gs]
            else:
                g, part = b // per_group, b % per_group
                mine = [x for gg, x in reqs if gg == g]
                size = len(mine) // per_group
                seqs = mine[part * size:(part + 1) * size]
            r = run(f"exp6_{n_batches}x{800 // n_batches}_batch{b}", seqs, 72, {})
            total_ms += r["ms_per_step"]
            total_b += r["B"]
            for j, key in enumerate(("plan", "sweep", "merge")):
                kus[j] += r["kernel_us"][key]
        yield {"workload": f"exp6_{n_batches}x{800 // n_batches}", "batches": n_batches, "B": total_b,
               "prefix_groups_per_batch": groups_per_batch if n_batches <= 8 else 1, "ms_per_decode_step": total_ms,
               "tokens_per_s": total_b / (total_ms * 1e-3),
               "kernel_us_summed": {"plan": kus[0], "sweep": kus[1], "merge": kus[2]}}


def policy_comparison(rounds, max_batch=256, queue=320, n_groups=5, prefix=5120, ucb_c=0.1, q_every_step=True,
                      names=("fcfs", "rule_based", "bandit", "q_learning")):
    """Batch formation with the stop policies of Section 4.3 on a queue fed from five prefix groups
    (5K-token prefixes, equal shares; the queue is topped up to `queue` waiting requests before
    every batch).  Each formed batch runs one decode-attention step; its measured tokens/s is the
    reward of the learned policies.  Reported per policy over the second half of the rounds:
    tokens/s (summed tokens over summed attention time), mean batch size, prefix groups per batch."""
    import torch
    import paper_2605_06046_amd as fea
    base = W.CONFIGS["c2"]
    rng = np.random.default_rng(W.SEED_BASE + 77)
    prefixes = [rng.integers(0, 32000, size=prefix, dtype=np.int32) for _ in range(n_groups)]
    cols = (prefix + 256) // 16 + 2
    n_blocks = n_groups * (prefix // 16) + max_batch * 18 + 64
    params = fea.AttnParams(base.num_q_heads, base.num_kv_heads, base.head_dim, fea.FEA_DTYPE_BF16)
    R = 4
    g = torch.Generator(device="cuda"); g.manual_seed(9)
    kv = [[torch.randn((n_blocks, base.num_kv_heads, 16, base.head_dim), generator=g, device="cuda").to(torch.bfloat16)
           for _ in range(2)] for _ in range(R)]
    q = torch.randn((max_batch, base.num_q_heads, base.head_dim), generator=g, device="cuda").to(torch.bfloat16)
    out = torch.empty_like(q)
    ws = torch.empty(fea.fea_decode_workspace_bytes(params, max_batch, cols), dtype=torch.uint8, device="cuda")
    dbt = torch.empty((max_batch, cols), dtype=torch.int32, device="cuda")
    dl = torch.empty(max_batch, dtype=torch.int32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    bins = dict(b_bins=10, w_bins=10, loss_thresholds=(0, 16, 128))
    rule = dict(small_batch=16, loss_small=1 << 30, loss_limit=8, peers_relax=32, loss_relaxed=64)

    def run(name):
        prng = np.random.default_rng(W.SEED_BASE + 78)          # every policy sees the same arrivals and draws
        tree, pool = fea.Cht(), fea.fea_kv_alloc(n_blocks, 16, 0)
        pol = {"bandit": lambda: fea.Policy(fea.FEA_POLICY_UCB, c=ucb_c, **bins),
               "q_learning": lambda: fea.Policy(fea.FEA_POLICY_QLEARN, alpha=0.2, gamma=0.9, eps=1.0, eps_min=0.002,
                                                eps_decay=0.99, reward_every_step=q_every_step, **bins)}.get(name, lambda: None)()
        toks, grp, order, next_id = {}, {}, [], 0
        tok_s, t_s, sizes, mixes, form_s = 0.0, 0.0, [], [], 0.0
        for rnd in range(rounds):
            while len(order) < queue:
                gi = int(prng.integers(n_groups))
                t = np.concatenate([prefixes[gi], prng.integers(0, 32000, size=int(prng.integers(64, 257)), dtype=np.int32)])
                toks[next_id], grp[next_id] = t, gi
                tree.insert(next_id, tokens=t)
                order.append(next_id)
                next_id += 1
            t0 = time.perf_counter()
            if name == "fcfs":
                ids = order[:max_batch]
                for rid in ids:
                    tree.add_to_batch(rid)
            elif name == "rule_based":
                ids = tree.build_batch(max_batch, **rule)
            else:
                ids = tree.build_batch_learned(pol, max_batch, prng.random((max_batch, 2)))
            form_s += time.perf_counter() - t0
            if not ids:                                            # a learned policy may stop at once: nothing runs
                if pol is not None:
                    pol.reward(0.0)
                continue
            B = len(ids)
            offs = np.zeros(B + 1, dtype=np.int64)
            offs[1:] = np.cumsum([len(toks[i]) for i in ids])
            bt, lens, _, _ = fea.fea_build_block_tables(pool, np.concatenate([toks[i] for i in ids]), offs, cols)
            dbt[:B].copy_(torch.from_numpy(bt)); dl[:B].copy_(torch.from_numpy(lens))
            for r in range(R + 1):                                 # one untimed call, then one per KV replica
                if r == 1:
                    e0.record()
                fea.fea_decode_attention(params, q[:B], kv[r % R][0], kv[r % R][1], dbt[:B], dl[:B], out[:B], ws)
            e1.record()
            torch.cuda.synchronize()
            sec = e0.elapsed_time(e1) * 1e-3 / R
            if pol is not None:
                pol.reward(B / sec * 1e-6)                         # M tokens/s
            if rnd >= rounds // 2:
                tok_s += B; t_s += sec; sizes.append(B); mixes.append(len({grp[i] for i in ids}))
            for row, rid in zip(bt, ids):
                fea.fea_release(pool, row[row >= 0])
                tree.finish(rid)
                del toks[rid], grp[rid]
            done = set(ids)
            order = [i for i in order if i not in done]
        return {"workload": f"policy_{name}", "rounds": rounds, "max_batch": max_batch, "queue": queue,
                "tokens_per_s": tok_s / max(t_s, 1e-12), "mean_batch": float(np.mean(sizes)) if sizes else 0.0,
                "prefix_groups_per_batch": float(np.mean(mixes)) if mixes else 0.0,
                "formation_us_per_batch": form_s / rounds * 1e6,
                "policy": pol.info() if pol is not None else None}

    for name in names:
        yield run(name)


if __name__ == "__main__":
    main()
