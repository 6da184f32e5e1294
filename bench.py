#!/usr/bin/env python3
"""Benchmark of the fused-subgraph hot path on one MI355X.

A step is one pass of the hot path over one batch of synthetic input: the
fused execution of the bias + tanh-GELU gated product subgraph
(bf16 [8192,11008], one ew_flat kernel) followed by the error-scoring pass of
its output against the output of the op-by-op (unfused) run of the same DAG.
The planner and the kernel specialisation run once, before the timed region.

value = effective HBM GB/s of the step: bytes that must move (every external
input once + every output once for the fused subgraph, both buffers once for
the scorer) / time.  The roofline entry times the fused kernel alone with
events on the launch stream.  The other named configs and the op-by-op
baseline are timed with the paper's protocol (20 warmup, 100 trials, median,
IQR) and reported under "configs".
"""
import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch from hardware counters (FETCH_SIZE and WRITE_SIZE, each scaled by what the
# same counter reads for a 256 MiB plain copy; figures in profiles/bench_cfg3_hbm_traffic_pmc.md).
# Keyed by kernel name, which ends in a hash of the specialised source: a changed kernel has a
# new name and reports traffic = null until the counters are taken again.
MEASURED_TRAFFIC_BYTES = {"pf_ew_add_gelu_mul_fdee327e": 541146382}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the per-config table")
    ap.add_argument("--sets", type=int, default=2, help="distinct buffer sets rotated through (cold cache)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the main line: the ten-shape task instances, shape-aware tiling against a static one")
    ap.add_argument("--score-sizes", action="store_true",
                    help="time the scorer and the tolerance ladder on one pair of 1 k ... 90 M elements (bf16 and f32)")
    ap.add_argument("--dags", type=str, default="",
                    help="with --cfg5: only these DAG numbers (comma separated), e.g. for a run under rocprofv3")
    ap.add_argument("--cfg5", action="store_true",
                    help="instead of the main line: fused against op-by-op time of each of the 256 random DAGs")
    return ap.parse_args()


def stats(us):
    us = np.asarray(us, dtype=np.float64)
    q1, med, q3 = np.percentile(us, [25, 50, 75])
    return float(med), float(q3 - q1)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus %d refused)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2605_29357_amd as pf
    from paper_2605_29357_amd.hip_events import HipEvent
    from tests.device import Runner, alloc_outputs, to_host_bits
    from workloads import configs

    assert torch.cuda.is_available(), "no GPU"
    pf.lib()
    stream = torch.cuda.current_stream()
    if args.sweep:
        print(json.dumps({"sweep": sweep_table(torch, pf, Runner, alloc_outputs, stream),
                          "outer_extent_reuse": reuse_table(torch, pf, Runner, alloc_outputs, stream)}))
        return
    if args.score_sizes:
        print(json.dumps({"score_sizes": score_sizes_table(torch, pf, stream)}))
        return
    if args.cfg5:
        only = [int(k) for k in args.dags.split(",") if k.strip()] or None
        print(json.dumps({"cfg5": cfg5_table(torch, pf, Runner, alloc_outputs, stream, only)}))
        return

    # ---------------------------------------------------------------- workload
    w = configs.cfg3_bias_gelu_gate()
    fused = Runner(w, fuse=True)
    unfused = Runner(w, fuse=False, intermediates_f32=False)
    unfused.d_in = fused.d_in
    nsets = max(1, args.sets)
    in_sets = [fused.d_in] + [[t.clone() for t in fused.d_in] for _ in range(nsets - 1)]
    out_sets = [alloc_outputs(w) for _ in range(nsets)]
    ref = unfused.run()[0]                       # reference output: op-by-op execution
    torch.cuda.synchronize()
    dt = w.output_dtypes[0]
    n_out = ref.numel()
    score_bytes = 2 * n_out * configs.ITEMSIZE[dt]
    res = torch.zeros(ctypes.sizeof(pf.ScoreResult), dtype=torch.uint8, device="cuda")
    sws = torch.empty(max(pf.score_workspace_bytes(1), 256), dtype=torch.uint8, device="cuda")

    def make_pair(out):
        p = pf.Pair()
        p.d_cand, p.d_ref, p.n = out.data_ptr(), ref.data_ptr(), n_out
        p.cand_dtype = p.ref_dtype = pf.DTYPES[dt]
        p.rtol, p.atol, p.equal_nan = configs.RTOL[dt], configs.ATOL[dt], 0
        return [p]
    pairs = [make_pair(o[0]) for o in out_sets]

    def step(i, ev=None):
        k = i % nsets
        fused.d_in = in_sets[k]
        # ev[0], ev[1]: start and end of the fused kernel itself (dispatch timestamps);
        # ev[2]: recorded on the stream after the scoring launches
        fused.run(out_sets[k], stream, events=ev[:2] if ev else None)
        pf.score(pairs[k], res.data_ptr(), sws.data_ptr(), sws.numel(), stream.cuda_stream)
        if ev:
            ev[2].record(stream)

    # a plain copy of known size (256 MiB in, 256 MiB out): the reference point that scales
    # hardware byte counters when this command is run under a counter-collecting profiler
    cp_src = torch.empty(1 << 28, dtype=torch.uint8, device="cuda").random_(0, 255)
    cp_dst = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    for _ in range(3):
        pf.copy_bytes(cp_dst.data_ptr(), cp_src.data_ptr(), 1 << 28, stream.cuda_stream)
    torch.cuda.synchronize()
    del cp_src, cp_dst

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    evs = [[HipEvent() for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, evs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    k_us = [e[0].elapsed_us(e[1]) for e in evs]
    s_us = [e[1].elapsed_us(e[2]) for e in evs]
    kernel_us = float(np.mean(k_us))
    score_us = float(np.mean(s_us))
    sr = pf.ScoreResult.from_buffer_copy(res.cpu().numpy().tobytes())
    step_bytes = w.algorithmic_bytes + score_bytes
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    gi = fused.exe.group_info(0)
    src = fused.exe.source(0)
    kname = src[src.index('extern "C" __global__'):].split("(")[1].split()[-1]
    roofline = {"bound": "hbm", "kernel": kname + " (bias + tanh-GELU gate, bf16 [8192,11008])",
                "achieved": w.algorithmic_bytes / (kernel_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "traffic": MEASURED_TRAFFIC_BYTES.get(kname),
                "traffic_source": ("stored: FETCH_SIZE + WRITE_SIZE of this kernel from profiles/bench_cfg3_hbm_traffic_pmc.md, "
                                   "not collected in this run") if kname in MEASURED_TRAFFIC_BYTES else
                                  "none: the kernel has changed since the counters in profiles/bench_cfg3_hbm_traffic_pmc.md were taken",
                "avg_us": kernel_us, "median_us": stats(k_us)[0],
                "algorithmic_bytes": w.algorithmic_bytes, "grid": gi["grid_blocks"], "block": gi["block_threads"]}
    roofline["frac"] = roofline["achieved"] / roofline["peak"]

    out = {"metric": "effective HBM GB/s of fused subgraphs (% of peak); speedup vs unfused op-by-op",
           "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": "cfg3: bias + tanh-GELU gated product, bf16 a,b [8192,11008], bias [11008]; "
                                  "fused execute (1 kernel) + error scoring vs the op-by-op output",
                      "step_bytes": step_bytes, "buffer_sets": nsets},
           "pct_of_peak": 100.0 * value / HBM_PEAK_GBS,
           "roofline": roofline,
           "score": {"avg_us": score_us, "GBps": score_bytes / (score_us * 1e-6) / 1e9, "bytes": score_bytes,
                     "allclose": sr.allclose, "max_abs": sr.max_abs, "n_viol": sr.n_viol}}

    # the tolerance ladder and both results in one pass, on the same pair (outside the timed steps)
    lres = torch.zeros(ctypes.sizeof(pf.LadderResult), dtype=torch.uint8, device="cuda")
    aws = torch.empty(max(pf.score_all_workspace_bytes(1), 256), dtype=torch.uint8, device="cuda")
    for label, call in (("ladder_us", lambda p: pf.score_ladder(p, lres.data_ptr(), aws.data_ptr(), aws.numel(), stream.cuda_stream)),
                        ("both_us", lambda p: pf.score_all(p, res.data_ptr(), lres.data_ptr(), aws.data_ptr(), aws.numel(), stream.cuda_stream))):
        ts = []
        for i in range(12):
            a, b = HipEvent(), HipEvent()
            a.record(stream)
            call(pairs[i % nsets])
            b.record(stream)
            torch.cuda.synchronize()
            ts.append(a.elapsed_us(b))
        out["score"][label] = float(np.median(ts[4:]))

    # --------------------------------------------- per-config table (paper protocol)
    if not args.no_extra:
        out["configs"] = per_config_table(torch, pf, configs, Runner, alloc_outputs, stream, w, fused, unfused, in_sets)

    # --------------------------------------------------------------- CPU baseline
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, to_host_bits, ref, out_sets[0][0], dt, configs)
    print(json.dumps(out))


def time_runner(torch, runner, stream, in_sets, out_sets, warmup=20, trials=100, max_rounds=3):
    """Paper protocol: 20 warmup, 100 timed trials, median; re-run while IQR > 20% of the median.
    Times are device times from the start of the first kernel to the end of the last."""
    from paper_2605_29357_amd.hip_events import HipEvent
    n = len(in_sets)
    med = iqr = None
    for _ in range(max_rounds):
        for i in range(warmup):
            runner.d_in = in_sets[i % n]
            runner.run(out_sets[i % n], stream)
        evs = [(HipEvent(), HipEvent()) for _ in range(trials)]
        torch.cuda.synchronize()
        for i in range(trials):
            runner.d_in = in_sets[i % n]
            # start of the first kernel to end of the last one
            runner.run(out_sets[i % n], stream, events=evs[i])
        torch.cuda.synchronize()
        med, iqr = stats([a.elapsed_us(b) for a, b in evs])
        if iqr <= 0.2 * med:
            break
    return med, iqr


def per_config_table(torch, pf, configs, Runner, alloc_outputs, stream, w3, fused3, unfused3, in_sets3):
    table = {}
    # a plain copy of the same byte volume: the practical ceiling
    nbytes = 1 << 28
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 255)
    dsts = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
    for i in range(10):
        pf.copy_bytes(dsts[i % 2].data_ptr(), src.data_ptr(), nbytes, stream.cuda_stream)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(50)]
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(evs):
        a.record(stream)
        pf.copy_bytes(dsts[i % 2].data_ptr(), src.data_ptr(), nbytes, stream.cuda_stream)
        b.record(stream)
    torch.cuda.synchronize()
    med, iqr = stats([a.elapsed_time(b) * 1e3 for a, b in evs])
    table["copy_256MiB"] = {"us": med, "iqr_us": iqr, "GBps": 2 * nbytes / (med * 1e-6) / 1e9}
    del src, dsts

    def copy_same_bytes(total, sets):
        """A plain copy moving `total` bytes (half read, half written), cold: the ceiling for a kernel of that size."""
        half = max(total // 2 // 16 * 16, 16)
        srcs = [torch.empty(half, dtype=torch.uint8, device="cuda").random_(0, 255) for _ in range(sets)]
        dsts = [torch.empty(half, dtype=torch.uint8, device="cuda") for _ in range(sets)]
        from paper_2605_29357_amd.hip_events import HipEvent
        ts = []
        for i in range(60):
            a, b = HipEvent(), HipEvent()
            a.record(stream)
            pf.copy_bytes(dsts[i % sets].data_ptr(), srcs[i % sets].data_ptr(), half, stream.cuda_stream)
            b.record(stream)
            if i >= 10:
                ts.append((a, b))
        torch.cuda.synchronize()
        return stats([a.elapsed_us(b) for a, b in ts])[0]

    def entry(w, sets):
        f = Runner(w, fuse=True)
        u = Runner(w, fuse=False, intermediates_f32=False)
        ins = [f.d_in] + [[t.clone() for t in f.d_in] for _ in range(sets - 1)]
        outs = [alloc_outputs(w) for _ in range(sets)]
        fm, fi = time_runner(torch, f, stream, ins, outs)
        um, ui = time_runner(torch, u, stream, ins, outs)
        # warm: one buffer set, so repeat runs may be served from the Infinity Cache
        wm, wi = time_runner(torch, f, stream, ins[:1], outs[:1])
        unfused_kernels = u.info["n_kernels"]
        del u
        cp = copy_same_bytes(w.algorithmic_bytes, sets)
        return {"bytes": w.algorithmic_bytes, "fused_us": fm, "fused_iqr_us": fi, "fused_kernels": f.info["n_kernels"],
                "copy_same_bytes_us": cp, "pct_of_copy": 100 * cp / fm,
                "fused_GBps": w.algorithmic_bytes / (fm * 1e-6) / 1e9,
                "fused_pct_peak": 100 * w.algorithmic_bytes / (fm * 1e-6) / 1e9 / HBM_PEAK_GBS,
                "fused_warm_us": wm, "unfused_us": um, "unfused_iqr_us": ui, "unfused_kernels": unfused_kernels,
                "speedup_vs_unfused": um / fm}

    # cfg3 reuses the buffers of the main loop
    outs3 = [alloc_outputs(w3) for _ in range(len(in_sets3))]
    fm, fi = time_runner(torch, fused3, stream, in_sets3, outs3)
    um, ui = time_runner(torch, unfused3, stream, in_sets3, outs3, trials=30)
    table["cfg3_bias_gelu_gate"] = {"bytes": w3.algorithmic_bytes, "fused_us": fm, "fused_iqr_us": fi, "fused_kernels": 1,
                                    "fused_GBps": w3.algorithmic_bytes / (fm * 1e-6) / 1e9,
                                    "fused_pct_peak": 100 * w3.algorithmic_bytes / (fm * 1e-6) / 1e9 / HBM_PEAK_GBS,
                                    "unfused_us": um, "unfused_iqr_us": ui, "unfused_kernels": unfused3.info["n_kernels"],
                                    "speedup_vs_unfused": um / fm}
    del outs3
    table["cfg4_rmsnorm_rope"] = entry(configs.cfg4_rmsnorm_rope(), 5)          # 5 x 136 MB > 512 MB between reuses
    table["cfg2_masked_softmax"] = entry(configs.cfg2_masked_softmax(), 16)     # 16 x 34 MB
    table["cfg1_add_layernorm"] = entry(configs.cfg1_add_layernorm(), 4)        # launch-bound either way
    # the paper's Case 1 at its D96 route (roll + slice + add + LayerNorm, two outputs, bf16)
    table["case1_roll_slice_add_layernorm_D96"] = entry(configs.roll_slice_add_layernorm(), 40)
    table["case2_masked_mean_pooling"] = entry(configs.masked_mean_pooling(), 6)   # 6 x 101 MB
    # launch-bound steps: op-by-op and fused execution, each followed by scoring, enqueued one call at a time and
    # replayed from a captured HIP graph of 16 steps (wall time per step, host included)
    for name, w in (("cfg1_add_layernorm", configs.cfg1_add_layernorm()), ("cfg2_masked_softmax", configs.cfg2_masked_softmax())):
        table[name]["step_wall_us"] = graph_replay_step(torch, pf, configs, Runner, alloc_outputs, w)
    return table


def graph_replay_step(torch, pf, configs, Runner, alloc_outputs, w, steps=16, reps=30):
    """Wall-clock microseconds per (execute + score) step: eager calls against replays of a captured graph."""
    dt = w.output_dtypes[0]
    out = {}
    ref = Runner(w, fuse=False, intermediates_f32=True).run()
    for label, fuse in (("fused", True), ("op_by_op", False)):
        r = Runner(w, fuse=fuse, intermediates_f32=False)
        outs = alloc_outputs(w, poison=False)
        p = pf.Pair()
        p.d_cand, p.d_ref, p.n = outs[0].data_ptr(), ref[0].data_ptr(), outs[0].numel()
        p.cand_dtype = p.ref_dtype = pf.DTYPES[dt]
        p.rtol, p.atol, p.equal_nan = configs.RTOL[dt], configs.ATOL[dt], 0
        res = torch.zeros(ctypes.sizeof(pf.ScoreResult), dtype=torch.uint8, device="cuda")
        sws = torch.empty(max(pf.score_workspace_bytes(1), 256), dtype=torch.uint8, device="cuda")
        side = torch.cuda.Stream()

        def one(stream):
            r.run(outs, stream=stream)
            pf.score([p], res.data_ptr(), sws.data_ptr(), sws.numel(), stream.cuda_stream)

        with torch.cuda.stream(side):
            for _ in range(3):
                one(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(steps):
                one(side)
        times = {"eager": [], "graph": []}
        for _ in range(reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            with torch.cuda.stream(side):
                for _ in range(steps):
                    one(side)
            torch.cuda.synchronize()
            times["eager"].append((time.perf_counter() - t0) * 1e6 / steps)
            t0 = time.perf_counter()
            graph.replay()
            torch.cuda.synchronize()
            times["graph"].append((time.perf_counter() - t0) * 1e6 / steps)
        out[label] = {"kernels_per_step": r.info["n_kernels"] + 3, "eager_us": float(np.median(times["eager"])),
                      "graph_us": float(np.median(times["graph"]))}
        del graph
    return out


def _rotating(torch, r, w, alloc_outputs, min_bytes=600e6, max_sets=48):
    """Enough copies of a workload's buffers that more than the Infinity Cache is touched between reuses."""
    n = int(max(2, min(max_sets, min_bytes // max(w.algorithmic_bytes, 1) + 1)))
    ins = [r.d_in] + [[t.clone() for t in r.d_in] for _ in range(n - 1)]
    outs = [alloc_outputs(w, poison=False) for _ in range(n)]
    return ins, outs


def sweep_table(torch, pf, Runner, alloc_outputs, stream):
    """Task instances (one operator sequence at ten shapes): per member the fused kernel with the tiling the
    planner derives from the shape, the same kernel with the tiling of member 0 forced onto every member (a
    static tiling), and the op-by-op run.  A static tiling the template cannot realise is a compile failure."""
    from workloads import sweeps
    table = {}
    for fam in sweeps.FAMILIES:
        rows, static = [], None
        for k in range(10):
            w = sweeps.member(fam, k)
            f = Runner(w)
            gi = f.exe.group_info(0)
            if static is None and gi["template"] in ("row_resident", "col_reduce"):
                static = {"tune_row_lanes": gi["lanes_per_row"]}
                if gi["template"] == "col_reduce":
                    static["tune_col_block"] = gi["block_threads"]
            ins, outs = _rotating(torch, f, w, alloc_outputs)
            fm, _ = time_runner(torch, f, stream, ins, outs, warmup=10, trials=50, max_rounds=2)
            u = Runner(w, fuse=False, intermediates_f32=False, upload=False)
            um, _ = time_runner(torch, u, stream, ins, outs, warmup=5, trials=30, max_rounds=1)
            row = {"member": w.name, "bytes": w.algorithmic_bytes, "template": gi["template"], "lanes_per_row": gi["lanes_per_row"],
                   "block": gi["block_threads"], "fused_us": fm, "GBps": w.algorithmic_bytes / fm / 1e3, "unfused_us": um,
                   "unfused_kernels": u.info["n_kernels"]}
            if static:
                try:
                    s = Runner(w, upload=False, **static)
                    sm, _ = time_runner(torch, s, stream, ins, outs, warmup=10, trials=50, max_rounds=2)
                    row["static_us"] = sm
                except pf.PfError as e:
                    row["static_us"] = None                          # the paper's error class 2
                    row["static_error"] = str(e)[:120]
            rows.append(row)
            del f, u, ins, outs
        ok = [r for r in rows if r.get("static_us")]
        summary = {"geomean_speedup_vs_unfused": float(np.exp(np.mean([np.log(r["unfused_us"] / r["fused_us"]) for r in rows]))),
                   "static_tiling": static}
        if static:
            summary["static_compile_failures"] = len(rows) - len(ok)
            summary["geomean_static_over_shape_aware"] = float(np.exp(np.mean([np.log(r["static_us"] / r["fused_us"]) for r in ok])))
            summary["worst_static_over_shape_aware"] = float(max(r["static_us"] / r["fused_us"] for r in ok))
        table[fam] = {"members": rows, "summary": summary}
    return table


def reuse_table(torch, pf, Runner, alloc_outputs, stream):
    """One operator sequence at several outermost extents (batch, rows): flat and row kernels take that extent as
    an argument, so members with the same tiling run one code object.  Per member: kernel name, wall time of
    pf_compile (a JIT compilation or a cache hit) and the fused kernel's device time."""
    import time
    import types
    from tests.device import TORCH_DT
    from workloads import configs
    fams = {
        "bias_gelu_gate": (configs.cfg3_bias_gelu_gate(rows=8, cols=11008), lambda r: [(r, 11008), (11008,), (r, 11008)], (1024, 2048, 4096, 8192)),
        "masked_softmax": (configs.cfg2_masked_softmax(heads=2, seq=512), lambda h: [(h, 512, 512), (512, 512)], (8, 16, 32, 64)),
        "rmsnorm_rope": (configs.cfg4_rmsnorm_rope(2, 2048, 32, 128), lambda b: [(b, 2048, 32, 128), (128,), (2048, 1, 128), (2048, 1, 128)], (2, 4, 8)),
        "add_layernorm": (configs.cfg1_add_layernorm(rows=8, cols=768), lambda r: [(r, 768), (r, 768), (768,), (768,)], (16384, 32768, 65536, 131072)),
    }
    table = {}
    for fam, (base, shapes_of, extents) in fams.items():
        g0 = pf.Graph(base.text)
        rows = []
        for x in extents:
            shapes = shapes_of(x)
            before = pf.jit_stats()
            t0 = time.perf_counter()
            g = g0.variant(shapes)
            w = types.SimpleNamespace(text=g.text(), inputs=None, input_dtypes=base.input_dtypes, input_shapes=shapes,
                                      output_dtypes=base.output_dtypes, output_shapes=[shapes[0]] * len(base.output_dtypes), name=fam)
            f = Runner(w, upload=False)
            compile_ms = (time.perf_counter() - t0) * 1e3
            after = pf.jit_stats()
            w.algorithmic_bytes = f.info["algorithmic_bytes"]
            f.d_in = [(torch.rand(tuple(sh), device="cuda") + 0.5).to(TORCH_DT[dt]) for dt, sh in zip(w.input_dtypes, shapes)]
            ins, outs = _rotating(torch, f, w, alloc_outputs)
            fm, _ = time_runner(torch, f, stream, ins, outs, warmup=10, trials=50, max_rounds=2)
            rows.append({"outer_extent": x, "kernel": f.exe.kernel_name(0), "pf_compile_ms": compile_ms,
                         "jit_compiled": after["compiled"] - before["compiled"],
                         "cache_hits": after["memory_hits"] + after["disk_hits"] - before["memory_hits"] - before["disk_hits"],
                         "grid": f.exe.group_info(0)["grid_blocks"], "bytes": w.algorithmic_bytes, "fused_us": fm,
                         "GBps": w.algorithmic_bytes / fm / 1e3})
            del f, ins, outs
        table[fam] = {"members": rows, "code_objects": len({r["kernel"] for r in rows})}
    return table


def score_sizes_table(torch, pf, stream):
    """One (candidate, reference) pair per call, candidate = reference with 1e-3 relative noise: device time from
    just before the call's first kernel to just after its last (events on the stream; median of 30 calls after 10)."""
    from paper_2605_29357_amd.hip_events import HipEvent
    rows = []
    for n in (1024, 8192, 8193, 65536, 131072, 131073, 1 << 21, 1 << 24, 8192 * 11008):
        for dt, tdt in (("bf16", torch.bfloat16), ("f32", torch.float32)):
            x = torch.randn(n, device="cuda").to(tdt)
            y = (x.float() * (1 + 1e-3 * torch.randn(n, device="cuda"))).to(tdt)
            p = pf.Pair()
            p.d_cand, p.d_ref, p.n = y.data_ptr(), x.data_ptr(), n
            p.cand_dtype = p.ref_dtype = pf.DTYPES[dt]
            p.rtol, p.atol, p.equal_nan = 2e-2, 1e-5, 0
            res = torch.zeros(max(ctypes.sizeof(pf.ScoreResult), ctypes.sizeof(pf.LadderResult)), dtype=torch.uint8, device="cuda")
            res2 = torch.zeros(ctypes.sizeof(pf.LadderResult), dtype=torch.uint8, device="cuda")
            ws = torch.empty(max(pf.score_all_workspace_bytes(1), 256), dtype=torch.uint8, device="cuda")
            row = {"elements": n, "dtype": dt, "bytes": 2 * n * x.element_size(),
                   "route": "one workgroup, one launch" if n <= 8192 else "staging launch + walking launch"}

            def both(pairs, r, w, wn, st):
                pf.score_all(pairs, r, res2.data_ptr(), w, wn, st)

            for label, call in (("score_us", pf.score), ("ladder_us", pf.score_ladder), ("both_us", both)):
                ts = []
                for _ in range(40):
                    a, b = HipEvent(), HipEvent()
                    a.record(stream)
                    call([p], res.data_ptr(), ws.data_ptr(), ws.numel(), stream.cuda_stream)
                    b.record(stream)
                    torch.cuda.synchronize()
                    ts.append(a.elapsed_us(b))
                row[label] = float(np.median(ts[10:]))
            row["score_GBps"] = row["bytes"] / row["score_us"] / 1e3
            row["ladder_GBps"] = row["bytes"] / row["ladder_us"] / 1e3
            row["both_GBps"] = row["bytes"] / row["both_us"] / 1e3
            rows.append(row)
            del x, y
    return rows


def configs_tol(dt):
    from workloads import configs
    return (configs.RTOL[dt], configs.ATOL[dt])


# Vector-ALU issue slots one element costs per operator, in units of one wave instruction at half the fp32 FMA
# rate.  The chip's published fp32 vector peak, 157.3 TFLOP/s = 78.6e12 FMA lane-operations per second, is 32 lanes
# per SIMD and clock (256 CUs x 4 SIMDs x 2.4 GHz); compares, selects, conversions and fp64 operations issue at
# 16 lanes per clock (the unit: 39.3e12 lane-operations per second), transcendental instructions at 8.  So
# fp32 add / mul / fma and simple integer operations count 0.5, the 16-lane class 1, v_rcp / v_exp 2.  Counted from
# the instruction sequences the kernels use for each operator.
ALU_UNITS = {"add": 0.5, "sub": 0.5, "mul": 0.5, "div": 6.5, "exp": 6.5, "tanh": 13.5, "sigmoid": 9.5, "gelu": 11.0, "rsqrt": 2.0,
             "maximum": 3.0, "minimum": 3.0, "rot_pairs": 0.5, "transpose": 2.0, "sum": 1.5, "mean": 1.5, "max": 3.0, "var": 4.0,
             "roll": 0.0, "slice": 0.0}
ALU_UNITS_FAST = dict(ALU_UNITS, div=2.5, exp=2.5, tanh=5.5, sigmoid=5.0, gelu=5.5)      # bf16 / fp16 graphs (no refinement steps)
ALU_PEAK_UNITS = 256 * 4 * 16 * 2.4e9
LOAD_UNITS = {"f32": 0.25, "bf16": 1.0, "f16": 1.0}       # per element: address arithmetic amortised over a vector + widening
STORE_UNITS = {"f32": 0.25, "bf16": 0.75, "f16": 1.0}


def alu_bound_us(pf, exe, graph, dtype):
    """Lower bound on a plan's time from vector-ALU issue alone: for every kernel, the operators it evaluates
    times the elements of its iteration domain, over the chip's issue rate."""
    table = ALU_UNITS if dtype == "f32" else ALU_UNITS_FAST
    total = 0.0
    for gi in exe.groups():
        elems = gi["rows"] * gi["cols"]
        units = 0.0
        for n in gi["nodes"]:
            ni = graph.node_info(n)
            full = 1
            for d in ni["shape"]:
                full *= d
            # a value that is uniform along the row costs one evaluation per row, not per element
            units += table.get(ni["op"], 1.0) * (elems if full * 2 > elems or ni["op"] in ("sum", "mean", "max", "var") else full)
        units += elems * (LOAD_UNITS[dtype] * max(1.0, gi["bytes_read"] / max(1, elems * (4 if dtype == "f32" else 2))) +
                          STORE_UNITS[dtype] * gi["bytes_written"] / max(1, elems * (4 if dtype == "f32" else 2)))
        total += units / ALU_PEAK_UNITS * 1e6
    return total


def cfg5_table(torch, pf, Runner, alloc_outputs, stream, only=None):
    """The 256 random fusible DAGs on their seeded inputs: fused and op-by-op device time each (median of 30 runs
    after 5 warm-ups; HIP events attached to the dispatches).  Cold: the runs rotate through enough copies of the
    DAG's buffers that more than 512 MB is touched between two uses of the same copy (the Infinity Cache holds
    256 MB); DAGs so small that 48 copies do not reach that are marked warm-only (they are launch-bound).  Warm: one
    copy.  Beside each time the two lower bounds: HBM (algorithmic bytes / 8 TB/s) and vector-ALU issue
    (alu_bound_us), and which of them is the larger.  Then every output of every fused run is scored against its
    op-by-op counterpart in ONE batched scoring call."""
    from paper_2605_29357_amd.hip_events import HipEvent
    from tests.device import to_device
    from workloads import dags

    def med_time(r, ins, outs, n=30, warm=5):
        k = len(ins)
        for i in range(warm):
            r.d_in = ins[i % k]
            r.run(outs[i % k], stream)
        evs = [(HipEvent(), HipEvent()) for _ in range(n)]
        for i, e in enumerate(evs):
            r.d_in = ins[i % k]
            r.run(outs[i % k], stream, events=e)
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_us(b) for a, b in evs]))

    if only is not None:
        # a plain copy of known size (256 MiB in, 256 MiB out): scales the hardware byte counters when a few DAGs
        # are run under a counter-collecting profiler
        cp_src = torch.empty(1 << 28, dtype=torch.uint8, device="cuda").random_(0, 255)
        cp_dst = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
        for _ in range(3):
            pf.copy_bytes(cp_dst.data_ptr(), cp_src.data_ptr(), 1 << 28, stream.cuda_stream)
        torch.cuda.synchronize()
        del cp_src, cp_dst
    rows, kept, pairs = [], [], []
    t_start = time.perf_counter()
    for k in (only if only is not None else range(dags.N_DAGS)):
        w = dags.cfg5(k)                                     # seeded inputs, as certified with the oracle
        dt = w.meta["dtype"]
        f = Runner(w, fuse=True, guard=False)
        u = Runner(w, fuse=False, intermediates_f32=False, upload=False, guard=False)
        touched = w.algorithmic_bytes + f.info["workspace_bytes"]
        nsets = int(max(1, min(48, 600e6 // max(touched, 1) + 1)))
        ins = [f.d_in] + [[t.clone() for t in f.d_in] for _ in range(nsets - 1)]
        outs = [alloc_outputs(w, poison=False) for _ in range(nsets)]
        uouts = alloc_outputs(w, poison=False)
        cold_ok = nsets * touched >= 512e6
        fused_cold = med_time(f, ins, outs)
        fused_warm = med_time(f, ins[:1], outs[:1])
        unfused = med_time(u, ins, outs if nsets > 1 else [uouts])
        u.d_in = ins[0]
        u.run(uouts, stream)
        # what a plain copy of the same byte volume takes, cold (half read, half written): the practical ceiling
        # for a kernel of this size, measured for the DAGs the 16 MB summary is about
        copy_us = None
        if w.algorithmic_bytes >= 16e6:
            half = w.algorithmic_bytes // 2 // 16 * 16
            csets = int(max(2, min(48, 600e6 // (2 * half) + 1)))
            srcs = [torch.empty(half, dtype=torch.uint8, device="cuda").random_(0, 255) for _ in range(csets)]
            dsts = [torch.empty(half, dtype=torch.uint8, device="cuda") for _ in range(csets)]
            ts = []
            for i in range(35):
                a, b = HipEvent(), HipEvent()
                a.record(stream)
                pf.copy_bytes(dsts[i % csets].data_ptr(), srcs[i % csets].data_ptr(), half, stream.cuda_stream)
                b.record(stream)
                if i >= 5:
                    ts.append((a, b))
            torch.cuda.synchronize()
            copy_us = float(np.median([a.elapsed_us(b) for a, b in ts]))
            del srcs, dsts
        g = f.exe.graph
        hbm_us = w.algorithmic_bytes / (HBM_PEAK_GBS * 1e3)
        alu_us = alu_bound_us(pf, f.exe, g, dt)
        rows.append({"dag": w.name, "bytes": w.algorithmic_bytes, "planned_bytes": f.info["planned_bytes"], "buffer_sets": nsets,
                     "cold": bool(cold_ok), "fused_us": fused_cold, "fused_warm_us": fused_warm, "unfused_us": unfused,
                     "fused_kernels": f.info["n_kernels"], "unfused_kernels": u.info["n_kernels"],
                     "templates": [gi["template"] for gi in f.exe.groups()], "hbm_bound_us": hbm_us, "alu_bound_us": alu_us,
                     "copy_same_bytes_us": copy_us, "pct_of_copy": 100 * copy_us / fused_cold if copy_us else None,
                     "binds": "alu" if alu_us > hbm_us else "hbm", "pct_of_hbm_peak": 100 * hbm_us / fused_cold,
                     "pct_of_bound": 100 * max(hbm_us, alu_us) / fused_cold})
        # every output of the fused run against the op-by-op one: the pairs of one batched scoring call
        for o, uo, odt in zip(outs[0], uouts, w.output_dtypes):
            p = pf.Pair()
            p.d_cand, p.d_ref, p.n = o.data_ptr(), uo.data_ptr(), o.numel()
            p.cand_dtype = p.ref_dtype = pf.DTYPES[odt]
            p.rtol, p.atol, p.equal_nan = configs_tol(odt) + (0,)
            pairs.append(p)
        kept.append((outs[0], uouts))
        del f, u, ins, outs
        if k % 16 == 15:
            print("cfg5: %d DAGs timed, %.0f s" % (k + 1, time.perf_counter() - t_start), file=sys.stderr, flush=True)
    res = torch.zeros(len(pairs) * ctypes.sizeof(pf.ScoreResult), dtype=torch.uint8, device="cuda")
    sws = torch.empty(max(pf.score_workspace_bytes(len(pairs)), 256), dtype=torch.uint8, device="cuda")
    ts = []
    for i in range(8):
        a, b = HipEvent(), HipEvent()
        a.record(stream)
        pf.score(pairs, res.data_ptr(), sws.data_ptr(), sws.numel(), stream.cuda_stream)
        b.record(stream)
        torch.cuda.synchronize()
        ts.append(a.elapsed_us(b))
    raw = res.cpu().numpy().tobytes()
    results = [pf.ScoreResult.from_buffer_copy(raw, i * ctypes.sizeof(pf.ScoreResult)) for i in range(len(pairs))]
    pair_bytes = sum(2 * p.n * (4 if p.cand_dtype == pf.DTYPES["f32"] else 2) for p in pairs)
    scoring = {"pairs": len(pairs), "bytes": pair_bytes, "us": float(np.median(ts[2:])),
               "GBps": pair_bytes / float(np.median(ts[2:])) / 1e3, "pairs_allclose": int(sum(r.allclose for r in results)),
               "elements": int(sum(p.n for p in pairs))}
    del kept
    tf, tu = sum(r["fused_us"] for r in rows), sum(r["unfused_us"] for r in rows)
    big = [r for r in rows if r["bytes"] >= 16e6 and r["fused_kernels"] == 1 and r["cold"]]
    multi = [r for r in rows if r["fused_kernels"] >= 3]
    return {"dags": rows, "scoring": scoring,
            "summary": {"fused_us_total": tf, "fused_warm_us_total": sum(r["fused_warm_us"] for r in rows), "unfused_us_total": tu,
                        "speedup_total": tu / tf,
                        "geomean_speedup": float(np.exp(np.mean([np.log(r["unfused_us"] / r["fused_us"]) for r in rows]))),
                        "fused_kernels": sum(r["fused_kernels"] for r in rows), "unfused_kernels": sum(r["unfused_kernels"] for r in rows),
                        "algorithmic_GBps_total": sum(r["bytes"] for r in rows) / tf / 1e3,
                        "single_kernel_dags_over_16MB": len(big),
                        "their_median_pct_of_hbm_peak_cold": float(np.median([r["pct_of_hbm_peak"] for r in big])) if big else None,
                        "their_min_pct_of_hbm_peak_cold": float(min(r["pct_of_hbm_peak"] for r in big)) if big else None,
                        "their_median_pct_of_bound_cold": float(np.median([r["pct_of_bound"] for r in big])) if big else None,
                        "their_median_pct_of_equal_bytes_copy": float(np.median([r["pct_of_copy"] for r in big])) if big else None,
                        "their_min_pct_of_equal_bytes_copy": float(min(r["pct_of_copy"] for r in big)) if big else None,
                        "median_pct_of_hbm_peak_of_those_copies": float(np.median([100 * r["hbm_bound_us"] / r["copy_same_bytes_us"] for r in big])) if big else None,
                        "alu_bound_among_them": int(sum(r["binds"] == "alu" for r in big)),
                        "median_planned_over_algorithmic_3plus_kernels":
                            float(np.median([r["planned_bytes"] / r["bytes"] for r in multi])) if multi else None}}


def _cpu_rows(job):
    """One worker's share of the oracle run: rows lo .. hi of the workload, read from files in shared memory."""
    folder, lo, hi, cols, dt, rtol, atol = job
    sys.path.insert(0, ROOT)
    from oracle import dag as oracle_dag
    from oracle import score as oracle_score
    from workloads import configs
    a, bias, b, cand, ref = (np.load(os.path.join(folder, name + ".npy"), mmap_mode="r") for name in ("a", "bias", "b", "cand", "ref"))
    part = configs.cfg3_bias_gelu_gate(rows=hi - lo, cols=cols, dtype=dt)
    y = oracle_dag.run(part.text, [np.ascontiguousarray(a[lo:hi]), np.ascontiguousarray(bias), np.ascontiguousarray(b[lo:hi])])[0]
    s = oracle_score.score_pair(np.ascontiguousarray(cand[lo:hi]), dt, np.ascontiguousarray(ref[lo:hi]), dt, rtol, atol)
    return y.shape[0], int(s["n"]), int(s["n_viol"])


def cpu_baseline(w, to_host_bits, ref, cand, dt, configs):
    """The oracle as it stands on the whole workload (op-by-op fp64 DAG, then fp64 scoring): on one thread, and
    with the rows split evenly over one process per host core (the oracle itself is single-threaded)."""
    import multiprocessing
    import shutil
    import tempfile
    from oracle import dag as oracle_dag
    from oracle import score as oracle_score
    cand_bits = to_host_bits(cand, dt)
    ref_bits = to_host_bits(ref, dt)
    t0 = time.perf_counter()
    y = oracle_dag.run(w.text, w.inputs)[0]
    s = oracle_score.score_pair(cand_bits, dt, ref_bits, dt, configs.RTOL[dt], configs.ATOL[dt])
    t1 = time.perf_counter()
    nbytes = w.algorithmic_bytes + 2 * cand_bits.size * configs.ITEMSIZE[dt]
    assert y.shape == tuple(w.output_shapes[0]) and s["n"] == cand_bits.size
    out = {"value": nbytes / (t1 - t0) / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
           "sample": "the whole workload (all %d rows), one step: %.2f s" % (w.output_shapes[0][0], t1 - t0),
           "nproc": os.cpu_count()}
    # all cores: a GPU machine gives one GPU's job 16 of the host's cores, whatever the machine has
    rows, cols = w.output_shapes[0]
    workers = max(1, min(16, os.cpu_count() or 1, len(os.sched_getaffinity(0))))
    folder = tempfile.mkdtemp(prefix="pf_cpu_baseline_", dir="/dev/shm" if os.path.isdir("/dev/shm") else None)
    try:
        for name, arr in (("a", w.inputs[0]), ("bias", w.inputs[1]), ("b", w.inputs[2]),
                          ("cand", cand_bits.reshape(rows, cols)), ("ref", ref_bits.reshape(rows, cols))):
            np.save(os.path.join(folder, name + ".npy"), arr)
        cuts = [rows * k // workers for k in range(workers + 1)]
        jobs = [(folder, cuts[k], cuts[k + 1], cols, dt, configs.RTOL[dt], configs.ATOL[dt]) for k in range(workers)]
        # fresh interpreters (not forks of this process, which holds the GPU); started and warmed before the clock
        with multiprocessing.get_context("spawn").Pool(workers) as pool:
            pool.map(_cpu_rows, [(folder, 0, 1, cols, dt, 0.0, 0.0)] * workers)
            t2 = time.perf_counter()
            parts = pool.map(_cpu_rows, jobs, chunksize=1)
            t3 = time.perf_counter()
        assert sum(p[0] for p in parts) == rows and sum(p[1] for p in parts) == cand_bits.size
        assert sum(p[2] for p in parts) == s["n_viol"]
        out["all_cores"] = {"value": nbytes / (t3 - t2) / 1e9, "unit": "GB/s", "cores": workers,
                            "sample": "the same step, rows split evenly over %d processes: %.2f s" % (workers, t3 - t2)}
    finally:
        shutil.rmtree(folder, ignore_errors=True)
    return out


if __name__ == "__main__":
    main()
