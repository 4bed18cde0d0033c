#!/usr/bin/env python3
"""Benchmark of the NestedKV prefill compression pass on one MI355X.

A step is one pass of the whole hot path -- nkv_score, nkv_budget, nkv_select_compact back to back on one
stream -- over one batch of synthetic keys/values that are already resident in HBM.  The default workload is
the headline one: Qwen3-4B-shaped long prefill, 36 layers x 8 KV heads x 32768 tokens x 128, bf16, r = 0.75.

Prints ONE JSON line: prompt tokens compressed per second, the roofline record of the dominant kernel
(algorithmic bytes per launch over its HIP-event duration, against 8 TB/s), and the CPU oracle timed on this
machine's host cores on the same inputs.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published


def algorithmic_bytes(d, dv, esize, r):
    """Bytes the method has to move per (head, token): keys once, scores out and in twice, kept rows in and
    out, kept indices out.  Per kernel and in total."""
    keep = 1.0 - r
    scan = esize * d                      # read every key once
    gather = 2.0 * keep * esize * (d + dv)
    total = scan + 4 + 4 + 4 + 4 * keep + gather
    return {"scan": float(scan), "gather": float(gather), "total": float(total)}


def read_traffic(kernel, workload):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.txt")
    try:
        m = re.search(r"^hbm_bytes_per_launch\s*[:=]\s*([0-9.eE+]+)", open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def bench_decode(args):
    """--mode decode: a step is one new token's attention (all layers, all query heads) over a compressed
    cache of the workload's shape -- a synthetic ragged cache with head-wise lengths that add up to
    H * floor((1 - r) N) per layer, resident in HBM."""
    import numpy as np
    import torch
    import nkv_inputs
    import paper_2605_26678_amd as nkv

    nkv.lib()
    w = nkv_inputs.WORKLOADS[args.workload]
    r = args.ratio if args.ratio is not None else w.ratios[0]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, V = nkv_inputs.make_kv(w, dev)
    lens = nkv_inputs.synthetic_head_lengths(w, r)
    pk, pv, head_off = nkv_inputs.synthetic_cache(w, K, V, lens)
    Hq = args.q_heads or 4 * w.H
    q = nkv_inputs.make_queries(w, Hq, K)
    del K, V
    rows, P = int(pk.shape[0]), len(w.prompt_lens)
    dtype = {"fp32": nkv.DTYPE_F32, "bf16": nkv.DTYPE_BF16, "fp16": nkv.DTYPE_F16, "fp8": nkv.DTYPE_F8_E4M3}[w.dtype]
    shape = nkv.Shape(w.L, w.H, w.d, w.d_v, dtype, w.cu_seqlens)
    params = nkv.params_default()
    scale = 1.0 / float(np.sqrt(w.d))
    ws = torch.empty(max(nkv.decode_workspace_bytes(shape, Hq, rows), 256), dtype=torch.uint8, device=dev)
    out = torch.empty(P, w.L, Hq, w.d_v, dtype=torch.float32, device=dev)
    lse = torch.empty(P, w.L, Hq, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        nkv.decode_attention(q, pk, pv, head_off, rows, shape, params, Hq, scale, out, lse, ws, stream)
    torch.cuda.synchronize()
    evs = [{"decode": (nkv.HipEvent(), nkv.HipEvent())} for _ in range(args.steps)]
    timed = [nkv.with_kernel_timers(params, e) for e in evs]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        nkv.decode_attention(q, pk, pv, head_off, rows, shape, timed[i], Hq, scale, out, lse, ws, stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = statistics.fmean(e["decode"][0].elapsed_ms(e["decode"][1]) for e in evs)
    esize = 4 if w.dtype == "fp32" else 2
    nbytes = float(rows) * (w.d + w.d_v) * esize                 # every retained K and V row once
    achieved = nbytes / (kern_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "decode", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": read_traffic("decode", w.name), "bytes_per_launch": nbytes,
                "kernel_ms": {"decode": round(kern_ms, 4)}}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle.decode import decode_attention as oracle_decode
        ho = head_off.cpu().numpy()
        spent, done_rows, u = 0.0, 0, 0
        G = Hq // w.H
        while spent < 15.0 and u < ho.shape[0] - 1:
            a, b = int(ho[u]), int(ho[u + 1])
            pl, h = divmod(u, w.H)
            p_, l_ = divmod(pl, w.L)
            qq = q[p_, l_, h * G:(h + 1) * G].float().cpu().numpy()[None, None]
            kk, vv = pk[a:b].float().cpu().numpy(), pv[a:b].float().cpu().numpy()
            t = time.perf_counter()
            oracle_decode(qq, kk, vv, np.array([0, b - a]), 1, scale)
            spent += time.perf_counter() - t
            done_rows += b - a
            u += 1
        cpu = {"value": round(P / (spent * rows / max(done_rows, 1)), 3), "unit": "decoded tokens/s (attention only)",
               "cores": 1, "kind": "oracle", "seconds": round(spent, 2),
               "sample": f"the first {u} of {ho.shape[0] - 1} (prompt, layer, KV head) units, {done_rows} of {rows} "
                         f"rows, scaled by rows; numpy fp64, one thread apart from numpy's own"}
    out_line = {"metric": "decoded tokens/sec, attention over the compressed cache (all layers+heads)",
                "value": round(P / (wall / args.steps), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
                "warmup": args.warmup, "ms_per_step": round(wall * 1e3 / args.steps, 4), "higher_is_better": True,
                "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                "config": {"workload": f"decode over {w.name}: {w.L} layers x {w.H} KV heads x {Hq} query heads, "
                                       f"{rows} retained rows of {list(w.prompt_lens)} tokens (r={r}), d={w.d}, "
                                       f"{w.dtype} cache", "ratio": r, "kv_dtype": w.dtype,
                           "cache": "synthetic ragged cache: per layer the heads' lengths add up to "
                                    "H*floor((1-r)N), a fifth each plus a multinomial share",
                           "inputs": nkv_inputs.recipe(w)},
                "roofline": roofline, "cpu_baseline": cpu}
    print(json.dumps(out_line))
    return 0


def bench_prefill_overlap(args):
    """How much a prefill loop lengthens when every layer's K/V are compressed as soon as they exist (Section 2.1:
    the method runs once after prefill, layer by layer; Section 4.4 reports prefill time with and without it).

    The layer's own work is a stand-in: the four projection GEMMs of a Qwen3-4B-shaped decoder layer over the
    whole prompt in bf16 (torch.matmul; attention itself is left out, so a real layer takes longer and hides
    more).  Three runs over all layers: the GEMMs alone; the GEMMs with the layer's compression pass (L = 1 calls
    of the three entry points) on a second stream, started when the layer's K/V projection is done; and the
    same calls in line on the GEMMs' stream."""
    import torch
    import nkv_inputs
    import paper_2605_26678_amd as nkv

    nkv.lib()
    w = nkv_inputs.WORKLOADS[args.workload]
    r = args.ratio if args.ratio is not None else w.ratios[0]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, V = nkv_inputs.make_kv(w, dev)
    dtype = {"fp32": nkv.DTYPE_F32, "bf16": nkv.DTYPE_BF16, "fp16": nkv.DTYPE_F16, "fp8": nkv.DTYPE_F8_E4M3}[w.dtype]
    params = nkv.params_default()
    r_list = [r] * (len(w.cu_seqlens) - 1)
    shape1 = nkv.Shape(1, w.H, w.d, w.d_v, dtype, w.cu_seqlens)
    comps = [nkv.Compressor(shape1, r_list, params) for _ in range(w.L)]
    hidden, inter, q_dim, kv_dim = 2560, 9728, 4096, 2 * w.H * w.d
    g = torch.Generator(device=dev).manual_seed(0)
    def mat(m, n):
        return (torch.randn(m, n, device=dev, dtype=torch.float32, generator=g) * (m ** -0.5)).to(torch.bfloat16)
    Wqkv, Wo, Wgu, Wd = mat(hidden, q_dim + kv_dim), mat(q_dim, hidden), mat(hidden, 2 * inter), mat(inter, hidden)
    x = mat(w.T, hidden)
    flops_layer = 2.0 * w.T * (hidden * (q_dim + kv_dim) + q_dim * hidden + hidden * 2 * inter + inter * hidden)
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    kv_ready = [torch.cuda.Event() for _ in range(w.L)]
    side_done = torch.cuda.Event()

    def layer_gemms(l, after_kv):
        qkv = x @ Wqkv
        after_kv(l)
        h = qkv[:, :q_dim] @ Wo
        gu = h @ Wgu
        return gu[:, :inter] @ Wd

    def none(l):
        pass

    def on_side(l):
        kv_ready[l].record(main)
        side.wait_event(kv_ready[l])
        comps[l].run(K[l], V[l], side)

    def in_line(l):
        comps[l].run(K[l], V[l], main)

    def run(after_kv):
        for l in range(w.L):
            layer_gemms(l, after_kv)
        if after_kv is on_side:
            side_done.record(side)
            main.wait_event(side_done)

    out = {}
    for name, fn in (("gemms_alone", none), ("compression_on_second_stream", on_side), ("compression_in_line", in_line)):
        for _ in range(max(args.warmup, 1)):
            run(fn)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run(fn)
        torch.cuda.synchronize()
        out[name] = (time.perf_counter() - t0) / args.steps * 1e3
    base = out["gemms_alone"]
    res = {"metric": "prefill time added by compressing every layer's K/V as it is produced", "unit": "percent",
           "value": round((out["compression_on_second_stream"] - base) / base * 100, 3),
           "in_line_percent": round((out["compression_in_line"] - base) / base * 100, 3),
           "ms_per_step": {k: round(v, 3) for k, v in out.items()}, "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "higher_is_better": False, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"{w.name}: per layer {w.H} KV heads x {list(w.prompt_lens)} tokens x d={w.d}, {w.dtype} K/V, "
                                  f"r={r}; {w.L} layers",
                      "layer_stand_in": f"bf16 GEMMs [T,{hidden}]x[{hidden},{q_dim + kv_dim}], [T,{q_dim}]x[{q_dim},{hidden}], "
                                        f"[T,{hidden}]x[{hidden},{2 * inter}], [T,{inter}]x[{inter},{hidden}] (no attention)",
                      "stand_in_tflops": round(flops_layer * w.L / (base * 1e-3) / 1e12, 1),
                      "inputs": nkv_inputs.recipe(w)}}
    print(json.dumps(res))
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="qwen4b_32k")
    ap.add_argument("--ratio", type=float, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-layers", type=int, default=0, help="layers the oracle is timed on (0 = choose)")
    ap.add_argument("--generic", action="store_true", help="force the shape-generic scoring kernels")
    ap.add_argument("--two-pass", action="store_true", help="stable anomaly in a second pass over the keys")
    ap.add_argument("--vector-scan", action="store_true", help="vector-unit formulation of the fused scan also where the matrix-core one applies")
    ap.add_argument("--per-layer", action="store_true",
                    help="a step is L passes with L = 1, one per layer's K/V slice, as a prefill loop would call it")
    ap.add_argument("--layers-per-call", type=int, default=1,
                    help="with --per-layer: layers handed to one call (must divide the workload's layers)")
    ap.add_argument("--layer-tensors", action="store_true",
                    help="every layer's K and V in an allocation of its own (a framework's list of per-layer caches), "
                         "still one call over all layers")
    ap.add_argument("--graph", action="store_true",
                    help="record a step's calls in a HIP graph once and time replays of it (wall time only: no per-kernel "
                         "events inside a graph)")
    ap.add_argument("--mode", choices=("pass", "decode", "prefill-overlap"), default="pass",
                    help="pass: the compression pass (default); decode: attention over the compressed cache; "
                         "prefill-overlap: layer-by-layer calls beside a stand-in for the layers' own GEMMs")
    ap.add_argument("--q-heads", type=int, default=0, help="decode mode: query heads (default 4 per KV head)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2
    if args.mode == "decode":
        return bench_decode(args)
    if args.mode == "prefill-overlap":
        return bench_prefill_overlap(args)

    import torch
    import nkv_inputs
    import paper_2605_26678_amd as nkv

    nkv.lib()                                   # fails loudly if the HIP library is missing
    w = nkv_inputs.WORKLOADS[args.workload]
    r = args.ratio if args.ratio is not None else w.ratios[0]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, V = nkv_inputs.make_kv(w, dev)
    dtype = {"fp32": nkv.DTYPE_F32, "bf16": nkv.DTYPE_BF16, "fp16": nkv.DTYPE_F16, "fp8": nkv.DTYPE_F8_E4M3}[w.dtype]
    shape = nkv.Shape(w.L, w.H, w.d, w.d_v, dtype, w.cu_seqlens)
    params = nkv.params_default(flags=(nkv.FLAG_GENERIC_KERNELS if args.generic else 0)
                                | (nkv.FLAG_TWO_PASS_STABLE if args.two_pass else 0)
                                | (nkv.FLAG_VECTOR_SCAN if args.vector_scan else 0))
    r_list = [r] * shape.n_prompts
    if args.per_layer:
        lpc = args.layers_per_call
        if lpc < 1 or w.L % lpc:
            print(f"bench.py: --layers-per-call must divide {w.L}", file=sys.stderr)
            return 2
        shape1 = nkv.Shape(lpc, w.H, w.d, w.d_v, shape.dtype, w.cu_seqlens)
        calls = [(nkv.Compressor(shape1, r_list, params), K[l:l + lpc], V[l:l + lpc]) for l in range(0, w.L, lpc)]
    elif args.layer_tensors:
        args.no_cpu_baseline = True                      # the oracle leg reads the one-tensor layout
        Kl, Vl = [K[l].clone() for l in range(w.L)], [V[l].clone() for l in range(w.L)]
        del K, V
        shape = nkv.Shape(w.L, w.H, w.d, w.d_v, dtype, w.cu_seqlens, key_layers=Kl, value_layers=Vl)
        K, V = Kl[0], Vl[0]
        calls = [(nkv.Compressor(shape, r_list, params), K, V)]
    else:
        calls = [(nkv.Compressor(shape, r_list, params), K, V)]
    stream = torch.cuda.current_stream()

    def run_all(per_call_params=None):
        for c, (comp, Kc, Vc) in enumerate(calls):
            if per_call_params is not None:
                comp.params = per_call_params[c]
            comp.run(Kc, Vc, stream)

    for _ in range(args.warmup):
        run_all()
    torch.cuda.synchronize()

    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            stream = side
            run_all()                                                  # warm-up on the capture stream
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                stream = torch.cuda.current_stream()
                run_all()
        torch.cuda.synchronize()
        for _ in range(max(args.warmup, 1)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        print(json.dumps({"metric": "prompt tokens compressed/sec (all layers+heads)", "value": round(w.T / (ms * 1e-3), 1),
                          "unit": "prompt tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": round(ms, 4), "higher_is_better": True, "dtype": "f32", "data": "synthetic",
                          "config": {"workload": w.name, "ratio": r, "calls_per_step": len(calls),
                                     "launch": "one HIP graph per step, replayed"}}))
        return 0

    # Timed region: K steps; the kernel that dominates (the key scan) is bracketed by an event pair of its own,
    # recorded by the library on the launch stream.  An event pair costs a few microseconds of pipeline bubble,
    # so the other kernels are timed in K more steps after the timed region.
    def run_steps(names):
        evs = [[{name: (nkv.HipEvent(), nkv.HipEvent()) for name in names} for _ in calls] for _ in range(args.steps)]
        timed = [[nkv.with_kernel_timers(params, evs[i][c]) for c in range(len(calls))] for i in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            run_all(timed[i])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        # per step: a kernel's launches added up over the step's calls
        ms = {name: statistics.fmean(sum(e[name][0].elapsed_ms(e[name][1]) for e in evs[i])
                                     for i in range(args.steps)) for name in names}
        return wall, ms

    base_params = params
    wall, kern_ms = run_steps(("scan",))
    _, rest_ms = run_steps(tuple(k for k in nkv.PASS_KERNELS if k != "scan"))
    kern_ms.update(rest_ms)
    kern_ms = {name: kern_ms[name] for name in nkv.PASS_KERNELS}
    ms_per_step = wall * 1e3 / args.steps
    tokens = w.T
    value = tokens / (wall / args.steps)

    esize = {"fp32": 4, "bf16": 2, "fp16": 2, "fp8": 1}[w.dtype]
    ab = algorithmic_bytes(w.d, w.d_v, esize, r)
    head_tokens = w.L * w.H * w.T
    dominant = max(("scan", "gather"), key=lambda k: kern_ms[k])
    achieved = ab[dominant] * head_tokens / (kern_ms[dominant] * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": None if args.per_layer else read_traffic(dominant, w.name),
                "traffic_source": None if args.per_layer or read_traffic(dominant, w.name) is None
                else f"profiles/{dominant}_{w.name}_pmc.txt (rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier run of this "
                     f"build, not measured in this run)",
                "bytes_per_launch": ab[dominant] * head_tokens,
                "kernel_ms": {k: round(v, 4) for k, v in kern_ms.items()},
                "whole_pass": {"algorithmic_bytes": ab["total"] * head_tokens,
                               "achieved": round(ab["total"] * head_tokens / (ms_per_step * 1e-3) / 1e9, 1),
                               "frac": round(ab["total"] * head_tokens / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}}

    # copy yardstick: what a plain 16-byte-vector copy reaches on this machine
    src = K.view(torch.uint8).reshape(-1)[: min(K.numel() * K.element_size(), 1 << 30)]
    dst = torch.empty_like(src)
    for _ in range(2):
        nkv.copy_probe(dst, src, stream)
    a, b = nkv.HipEvent(), nkv.HipEvent()
    a.record(stream)
    for _ in range(10):
        nkv.copy_probe(dst, src, stream)
    b.record(stream)
    torch.cuda.synchronize()
    roofline["copy_probe_GBs"] = round(2 * src.numel() * 10 / (a.elapsed_ms(b) * 1e-3) / 1e9, 1)
    nkv.copy_probe(None, src, stream)                                  # the loads alone
    a.record(stream)
    for _ in range(10):
        nkv.copy_probe(None, src, stream)
    b.record(stream)
    torch.cuda.synchronize()
    roofline["read_probe_GBs"] = round(src.numel() * 10 / (a.elapsed_ms(b) * 1e-3) / 1e9, 1)
    del src, dst

    cpu = None
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from parity_util import oracle_params
        op = oracle_params(base_params)
        n_layers = args.cpu_layers or w.L
        cu = w.cu_seqlens
        spent = 0.0
        done = 0
        for l in range(n_layers):
            raw = {1: torch.uint8, 2: torch.int16, 4: torch.int32}[esize]
            Kl = K[l].cpu().float().numpy()
            Kb, Vb = K[l].cpu().view(raw).numpy(), V[l].cpu().view(raw).numpy()
            t = time.perf_counter()
            oracle.compress(Kl[None], Kb[None], Vb[None], cu, r_list, op)
            spent += time.perf_counter() - t
            done += 1
            if spent > 30.0:
                break
        threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
        threads = min(threads, w.H)                      # the oracle's only parallel loop runs over a layer's heads
        cpu = {"value": round(tokens / (spent * w.L / done), 1), "unit": "prompt tokens/s", "cores": threads,
               "kind": "oracle", "seconds": round(spent, 2),
               "sample": f"{done} of {w.L} layers of the same workload (all heads, all prompts), scaled by L/{done}; "
                         f"OpenMP over the {w.H} heads of a layer for scoring, the rest single-threaded"}

    out = {"metric": "prompt tokens compressed/sec (all layers+heads)", "value": round(value, 1),
           "unit": "prompt tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"{w.name}: {w.L} layers x {w.H} KV heads x {list(w.prompt_lens)} tokens x d={w.d}, "
                                  f"{w.dtype} K/V, r={r}", "ratio": r, "kv_dtype": w.dtype,
                      "scoring_kernels": "generic" if args.generic else "default",
                      "calls_per_step": len(calls),
                      "inputs": nkv_inputs.recipe(w)},
           "roofline": roofline, "cpu_baseline": cpu}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
