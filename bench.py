#!/usr/bin/env python3
"""Benchmark of the decode-step hot path (append + attention over the packed KV cache).

One "step" = one decode step of a LLaMA-3.1-8B-shaped model: 32 layers, each issuing
bd_decode_step (= bd_append_kv + bd_decode_attn with split-K combine) on its own,
independent cache, back to back on one stream.  Thirty-two distinct caches keep the working set (> 1 GB) far above the
256 MB last-level cache, so every step streams its KV bytes from HBM.

Prints ONE JSON line.  value = effective KV GB/s:
algorithmic bytes of the attention calls of a step / wall time of the step.
"""
from __future__ import annotations

import argparse
import gc
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
N_LAYERS = 32
# packed K + packed V + their parameters, per token and KV head
PER_TOKEN_BYTES = {"int4": 136, "int2": 72, "mxfp4": 136, "int4_kt": 136, "int2_kt": 72,
                   "int4_g64": 144, "int4_g32": 160, "int2_g64": 80, "int2_g32": 96,
                   "int4_kt_g64": 144, "int4_kt_g32": 160, "int2_kt_g64": 80, "int2_kt_g32": 96}
VARIANTS = {
    "": "the configuration as listed",
    "paged": "the same tokens in a paged cache (128-token pages scattered over a pool, lengths on the device): "
             "bd_paged_decode_step per layer",
    "kt": "K quantized per token instead of per channel (formats int4_kt / int2_kt)",
    "gq8": "8 query heads per KV head (64/8 heads)",
    "gq16": "16 query heads per KV head (128/8 heads)",
    "g64": "quantization groups of 64 instead of 128 (formats int4_g64 / int2_g64)",
    "g32": "quantization groups of 32 (formats int4_g32 / int2_g32)",
    "kt_g64": "K per token with quantization groups of 64 channels (formats int4_kt_g64 / int2_kt_g64)",
    "kt_g32": "K per token with quantization groups of 32 channels (formats int4_kt_g32 / int2_kt_g32)",
}


def algorithmic_bytes(w, packed_len: int, res_len: int) -> int:
    """Bytes one attention call must move: packed K and V codes, their parameters, the
    residual fp16 tokens present, the query and the output."""
    units = w.batch * w.n_kv_heads
    qo = 2 * w.batch * w.n_q_heads * w.head_dim * 2
    return units * (packed_len * PER_TOKEN_BYTES[w.fmt] + res_len * w.head_dim * 2 * 2) + qo


def measured_traffic(w, variant: str):
    """HBM bytes per decode-kernel launch from the committed rocprofv3 --pmc summary of this
    workload (FETCH_SIZE + WRITE_SIZE, calibrated against a plain copy), or None."""
    if variant:
        return None
    path = os.path.join(ROOT, "profiles", f"decode_{w.fmt}_{w.name}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(float(line.split(":")[1]))
    except OSError:
        pass
    return None


def _oracle_worker(job):
    """One host process of the cpu_baseline leg: the oracle's decode steps (append + attention) on one
    (sequence, KV head) unit for at least `seconds`; returns (steps, algorithmic bytes, seconds)."""
    from threadpoolctl import threadpool_limits
    from oracle import bitdecode_oracle as O
    from paper_2503_18773_amd import workloads as W
    w, unit, K1, V1, cap, seconds, sm_scale = job
    per_tok = PER_TOKEN_BYTES[w.fmt]
    with threadpool_limits(limits=1):
        if w.fmt == "mxfp4":
            oc = O.MxCache(1, 1, cap)
        else:
            oc = O.IntCache(1, 1, 4 if w.fmt.startswith("int4") else 2, cap, k_per_token="_kt" in w.fmt,
                            group=64 if w.fmt.endswith("_g64") else 32 if w.fmt.endswith("_g32") else 128)
        oc.quant_pack_kv(K1, V1)          # untimed: prefill
        b, h = divmod(unit, w.n_kv_heads)
        new = [(W.make_new_kv(w, s), W.make_q(w, s)) for s in range(4)]   # drawn before the clock starts
        nsteps, nbytes = 0, 0
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            (kn, vn), q = new[nsteps % 4]
            oc.append_kv(kn[b:b + 1, h:h + 1], vn[b:b + 1, h:h + 1])
            O.decode_attn(oc, q[b:b + 1, h * w.g_q:(h + 1) * w.g_q], sm_scale)
            nsteps += 1
            plen = getattr(oc, "packed_len", getattr(oc, "length", 0))
            nbytes += plen * per_tok + getattr(oc, "res_len", 0) * 512 + 2 * w.g_q * 256
        return nsteps, nbytes, time.perf_counter() - t0


def oracle_baseline(w, K, V, cap, seconds, sm_scale):
    """The oracle as it stands on the host cores: one process per (sequence, KV head) unit, up to 16."""
    import multiprocessing as mp
    units = list(range(min(16, w.batch * w.n_kv_heads, os.cpu_count() or 1)))
    jobs = []
    for u in units:
        b, h = divmod(u, w.n_kv_heads)
        jobs.append((w, u, np.ascontiguousarray(K[b:b + 1, h:h + 1]), np.ascontiguousarray(V[b:b + 1, h:h + 1]), cap,
                     seconds, sm_scale))
    with mp.get_context("spawn").Pool(len(jobs)) as pool:
        res = pool.map(_oracle_worker, jobs, chunksize=1)
    steps = sum(r[0] for r in res)
    wall = max(r[2] for r in res)
    return {"value": round(sum(r[1] for r in res) / wall / 1e9, 4), "unit": "GB/s", "cores": len(jobs), "kind": "oracle",
            "seconds": round(wall, 2),
            "sample": f"{steps} decode steps (append + attention) in all, on {len(jobs)} of the "
                      f"{w.batch * w.n_kv_heads} (sequence, KV head) units of one layer at context {w.context}, one "
                      f"single-threaded process per unit (numpy float64)"}


def kernel_roofline(B, W, torch, w, caches, qs_last, outs, splits, paged, sm_scale, variant, total_steps):
    """Roofline of the dominant kernel (decode attention), measured live with HIP events on the stream the
    kernels run on: one event pair around the bd_decode_attn launches (partials only, no combine) of all
    layers, enqueued back to back; the kernels run without gaps, so elapsed / launches is the average
    launch duration (cold caches: each layer has its own).  Also the streaming-read floor over the same
    caches (bd_probe_stream_read: the same loads, no arithmetic), measured the same way."""
    stream = torch.cuda.current_stream()
    mx = w.fmt == "mxfp4"
    c0 = caches[0]
    reps = 5

    def timed(launch):
        per_rep = []
        for rep_ in range(reps + 1):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for li, c in enumerate(caches):
                launch(li, c)
            b.record(stream)
            torch.cuda.synchronize()
            if rep_:
                per_rep.append(a.elapsed_time(b) * 1e3 / len(caches))
        return per_rep

    def decode(li, c):
        if paged:   # this entry point always merges: the figure includes the combine kernel
            c.decode_attn(qs_last, sm_scale, outs[li], splits)
        else:
            B.bd_decode_attn(c.desc, qs_last, c.packed_len, c.res_len, sm_scale, splits, c.workspace(splits), None)

    per_rep = timed(decode)
    kernel_us = float(np.mean(per_rep))
    if paged:
        n = w.context + total_steps
        pl, rl = (n, 0) if mx else (n - n % 128, n % 128)
    else:
        pl, rl = c0.packed_len, c0.res_len
    launch_bytes = algorithmic_bytes(w, pl, rl)
    achieved = launch_bytes / (kernel_us * 1e-6) / 1e9
    kernel_name = "decode_mx_kernel" if mx else "decode_grp_kernel" if "_g" in w.fmt else "decode_int_kernel"
    roofline = {"bound": "hbm", "kernel": kernel_name,
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(w, variant),
                "avg_launch_us": round(kernel_us, 3), "min_launch_us": round(float(np.min(per_rep)), 3),
                "bytes_per_launch": launch_bytes, "num_splits": splits,
                "timing": f"hip events around {len(caches)} back-to-back launches (one per cold layer cache), "
                          f"{reps} repetitions" + (" (paged entry point: decode + combine kernels)" if paged else "")}
    stream_roof = None
    if not paged:
        ppl = c0.packed_len - c0.packed_len % 128
        probe = timed(lambda li, c: B.bd_probe_stream_read(c.desc, ppl))
        code_bytes = w.batch * w.n_kv_heads * ppl * 128 * (2 if w.fmt.startswith("int2") else 4) // 8 * 2
        us = float(np.mean(probe))
        stream_roof = {"avg_launch_us": round(us, 3), "min_launch_us": round(float(np.min(probe)), 3),
                       "bytes_per_launch": code_bytes, "GB/s": round(code_bytes / us / 1e3, 1),
                       "frac_of_peak": round(code_bytes / us / 1e3 / HBM_PEAK_GBPS, 4),
                       "what": "bd_probe_stream_read: the packed K and V codes of the same caches read with the decode "
                               "kernel's loads and nothing else; same timing as the roofline (context, not a target)"}
    return roofline, stream_roof


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg1", help="cfg1 (32K int4, default), cfg3 (128K int4), cfg2, cfg0")
    ap.add_argument("--variant", default="", choices=sorted(VARIANTS),
                    help="a variation of the workload: " + "; ".join(f"{k or '(none)'}: {v}" for k, v in VARIANTS.items()))
    ap.add_argument("--layers", type=int, default=N_LAYERS)
    ap.add_argument("--mode", default="eager", choices=["graph", "eager"],
                    help="graph: the warm-up steps and the timed steps are each captured into one HIP graph "
                         "(every step distinct) so host launch cost is out of the timed region; eager: plain calls")
    ap.add_argument("--splits", type=int, default=0, help="override the library's split factor")
    ap.add_argument("--per-step", default="", metavar="FILE",
                    help="eager mode only: also time every step with its own event pair and write the list "
                         "(step, packed_len, res_len, microseconds) to FILE; steps that fill the residual block show "
                         "as spikes (they run the quantize kernel)")
    ap.add_argument("--flush", default="first", choices=["first", "lazy"],
                    help="the step that fills the residual block packs it before attending it (bd_decode_step = "
                         "bd_append_kv + bd_decode_attn) or attends it in fp16 and packs it afterwards "
                         "(bd_decode_step_lazy, the paper's Residual Kernel order)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-128k", action="store_true", help="cfg1 only: skip the second measurement at 128K (cfg3)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="lower bound on the oracle's timed CPU work")
    ap.add_argument("--calib-copy", action="store_true",
                    help="only run a plain 1 GiB device copy 5 times (calibrates the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (the path shards by batch / KV head / "
              "context, but no multi-GPU code exists)", file=sys.stderr)
        return 2

    import torch
    from paper_2503_18773_amd import binding as B
    from paper_2503_18773_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calib_copy:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calib_copy_bytes": 1 << 30, "launches": 5}))
        return 0
    B.lib()  # fail loudly if the HIP library is missing
    rec, cpu_job = run(args, args.workload, args.steps, args.warmup, not args.no_cpu_baseline)
    if args.workload == "cfg1" and not args.variant and not args.no_128k:
        # the metric is quoted at 32K and at 128K: the same measurement on cfg3 (fewer steps: each moves 4x the bytes)
        torch.cuda.empty_cache()
        r3, _ = run(args, "cfg3", max(args.steps // 4, 3), min(args.warmup, 2), False)
        rec["roofline_128k"] = r3["roofline"]
        rec["stream_roof_128k"] = r3["stream_roof"]
        rec["step_128k"] = {k: r3[k] for k in ("value", "unit", "steps", "warmup", "ms_per_step", "us_per_layer_call",
                                                 "pct_hbm_peak", "prefill_quant_pack_ms_per_layer")}
        rec["step_128k"]["workload"] = r3["config"]["workload"]
        rec["step_128k"]["num_splits"] = r3["config"]["num_splits"]
    if cpu_job is not None:
        rec["cpu_baseline"] = oracle_baseline(*cpu_job)
    print(json.dumps(rec))
    return 0


def run(args, workload: str, steps: int, warmup: int, with_cpu: bool) -> dict:
    """Everything bench.py measures on one workload; returns the record."""
    import torch
    from paper_2503_18773_amd import binding as B
    from paper_2503_18773_amd import workloads as W
    w = W.CONFIGS[workload]
    if args.variant in ("kt", "g64", "g32", "kt_g64", "kt_g32"):
        w = W.scaled(w, fmt=w.fmt + "_" + args.variant)
    elif args.variant in ("gq8", "gq16"):
        w = W.scaled(w, n_q_heads=int(args.variant[2:]) * w.n_kv_heads)
    paged = args.variant == "paged"
    total_steps = warmup + steps
    cap = ((w.context + total_steps + 1 + 127) // 128) * 128 + 128
    tdt = torch.float16 if w.in_dtype == "fp16" else torch.bfloat16

    def dev(x):
        if w.in_dtype == "fp16":
            return torch.from_numpy(np.ascontiguousarray(x)).cuda()
        return torch.from_numpy(W.bf16_bits(x).view(np.int16)).cuda().view(torch.bfloat16)

    # ---- synthetic inputs, resident in HBM before anything is timed
    t_setup = time.time()
    K, V = W.make_kv(w)
    Kd, Vd = dev(K), dev(V)
    caches = []
    max_pages = cap // 128
    for li in range(args.layers):
        if paged:
            # every layer its own pool; the pages of a sequence are scattered over it
            num_pages = w.batch * max_pages + 16
            table = np.random.default_rng(1000 + li).permutation(num_pages)[:w.batch * max_pages]
            c = B.PagedKVCache(w.batch, w.n_q_heads, w.n_kv_heads, w.fmt, num_pages,
                               table.reshape(w.batch, max_pages).astype(np.int32))
            for b in range(w.batch):
                c.quant_pack_kv(b, Kd[b], Vd[b])
        else:
            c = B.KVCache(w.batch, w.n_q_heads, w.n_kv_heads, w.fmt, cap)
            c.quant_pack_kv(Kd, Vd)
        caches.append(c)
    torch.cuda.synchronize()
    # prefill quantize+pack time of one layer (reported, not part of the step)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    if paged:
        for b in range(w.batch):
            caches[0].quant_pack_kv(b, Kd[b], Vd[b])
    else:
        caches[0].quant_pack_kv(Kd, Vd)
    e1.record(); torch.cuda.synchronize()
    prefill_ms = e0.elapsed_time(e1)
    del Kd, Vd
    new_kv = [tuple(dev(x) for x in W.make_new_kv(w, s)) for s in range(total_steps)]
    qs = [dev(W.make_q(w, s)) for s in range(total_steps)]
    outs = [torch.empty((w.batch, w.n_q_heads, 128), dtype=tdt, device="cuda:0") for _ in range(args.layers)]
    sm_scale = W.softmax_scale(w)
    shape = B.bd_cache(w.batch, w.n_q_heads, w.n_kv_heads, 128, B.FORMATS[w.fmt], cap, None, None, None, None, None,
                       None)
    splits = args.splits or B.bd_choose_splits(shape, w.context)
    for c in caches:
        c.workspace(splits)
    setup_s = time.time() - t_setup

    step_bytes = []
    mx = w.fmt == "mxfp4"

    def lengths(n_tokens: int):
        """(packed, residual) token counts of a sequence of n_tokens."""
        return (n_tokens, 0) if mx else (n_tokens - n_tokens % 128, n_tokens % 128)

    def run_step(s: int):
        kn, vn = new_kv[s]
        nbytes = 0
        for li, c in enumerate(caches):
            if paged:   # the lengths live on the device; the host knows them by counting
                c.decode_step(kn, vn, qs[s], sm_scale, outs[li], splits, lazy=args.flush == "lazy")
                nbytes += algorithmic_bytes(w, *lengths(w.context + s + 1))
            else:
                c.decode_step(kn, vn, qs[s], sm_scale, outs[li], num_splits=splits, lazy=args.flush == "lazy")
                nbytes += algorithmic_bytes(w, c.packed_len, c.res_len)
        step_bytes.append(nbytes)

    stream = torch.cuda.current_stream()
    gc.collect()
    gc.disable()   # (a collection inside the timed loop shows up as one multi-millisecond step)
    if args.mode == "graph" and paged:
        # lengths and the flush decision live on the device: ONE captured step (all layers) is replayed
        # for every step, its inputs copied into static buffers before each replay
        kn_s, vn_s, q_s = torch.zeros_like(new_kv[0][0]), torch.zeros_like(new_kv[0][1]), torch.zeros_like(qs[0])
        g_step = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_step):
            for li, c in enumerate(caches):
                c.decode_step(kn_s, vn_s, q_s, sm_scale, outs[li], splits, lazy=args.flush == "lazy")

        def replay_step(s: int):
            kn_s.copy_(new_kv[s][0]); vn_s.copy_(new_kv[s][1]); q_s.copy_(qs[s])
            g_step.replay()
            step_bytes.append(len(caches) * algorithmic_bytes(w, *lengths(w.context + s + 1)))

        for s in range(warmup):
            replay_step(s)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(warmup, total_steps):
            replay_step(s)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    elif args.mode == "graph":
        g_warm, g_timed = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
        if warmup:
            with torch.cuda.graph(g_warm):
                for s in range(warmup):
                    run_step(s)
        with torch.cuda.graph(g_timed):
            for s in range(warmup, total_steps):
                run_step(s)
        if warmup:
            g_warm.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g_timed.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    else:
        for s in range(warmup):
            run_step(s)
        torch.cuda.synchronize()
        step_events = []
        t0 = time.perf_counter()
        for s in range(warmup, total_steps):
            if args.per_step:
                ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                ea.record(stream)
            run_step(s)
            if args.per_step:
                eb.record(stream)
                step_events.append((s, *(lengths(w.context + s + 1) if paged else (caches[0].packed_len, caches[0].res_len)), ea, eb))
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        if args.per_step:
            with open(args.per_step, "w") as f:
                f.write(f"# {w.name} {w.fmt}: per-step time of {args.layers} layers (bd_decode_step each), num_splits {splits}\n")
                f.write("# step packed_len res_len(after the step) microseconds\n")
                for s, pl, rl, ea, eb in step_events:
                    f.write(f"{s} {pl} {rl} {ea.elapsed_time(eb) * 1e3:.1f}\n")
    gc.enable()
    elapsed = t1 - t0
    timed_bytes = sum(step_bytes[warmup:])
    ms_per_step = elapsed * 1e3 / steps
    value = timed_bytes / elapsed / 1e9

    roofline, stream_roof = kernel_roofline(B, W, torch, w, caches, qs[-1], outs, splits, paged, sm_scale, args.variant,
                                            total_steps)
    del caches, outs, new_kv, qs
    # ---- the oracle on the host cores, on a bounded sample of the same workload: after every GPU measurement
    #      of the run (ten idle seconds in between would let the GPU's clocks drop), so only its inputs are kept
    cpu_job = (w, K, V, cap, args.cpu_seconds, sm_scale) if with_cpu else None

    rec = {
        "metric": "effective KV GB/s per decode step (32-layer LLaMA-8B-shape step: append + split-K attention "
                  "over the packed cache)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"int4": "u4->f16 mfma, f32 accumulate", "int2": "u2->f16 mfma, f32 accumulate",
                  "mxfp4": "e2m1 mfma, f32 accumulate"}[w.fmt.split("_")[0]],
        "data": "synthetic",
        "config": {"workload": f"{w.name}: batch {w.batch}, {w.n_q_heads}/{w.n_kv_heads} heads, head_dim 128, "
                               f"context {w.context}, {w.fmt} KV" + (f", variant {args.variant}" if args.variant else ""),
                   "layers": args.layers, "mode": args.mode, "num_splits": splits, "flush": args.flush},
        "us_per_layer_call": round(ms_per_step * 1e3 / args.layers, 3),
        "us_per_decode_step": round(ms_per_step * 1e3, 2),
        "pct_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "prefill_quant_pack_ms_per_layer": round(prefill_ms, 4),
        "setup_s": round(setup_s, 1),
        "roofline": roofline,
        "stream_roof": stream_roof,
        "cpu_baseline": None,
    }
    return rec, cpu_job


if __name__ == "__main__":
    sys.exit(main())
