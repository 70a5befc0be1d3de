#!/usr/bin/env python3
"""Benchmark of libhfxattn on one MI355X.

A step is one pass of the whole hot path over one scheduled batch: the host builds the batch
descriptor and uploads it (hfx_build_batch_desc), then one persistent launch executes the mixed
prefill/decode paged attention (hfx_mixed_paged_attention).  Inputs are resident in HBM before
the timed region.  The headline workload is the Llama-3-8B-shaped mixed step (64 decodes with
log-normal contexts + 2 prompt chunks of 512); the decode-heavy and prefill-heavy steps are
timed as well and reported under "paths" because the metric names all three figures.

Prints ONE JSON line.
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


TRAFFIC_NOTE = os.path.join(ROOT, "profiles", "bench_hbm_traffic_fetch_write.txt")
KERNEL_SOURCES = ["hfx_kernels.hip", "hfx_desc.h", "hfx_plan.cpp"]


def sources_digest() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2508_15919_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic():
    """HBM bytes per launch of the headline step from the committed counter summary (FETCH_SIZE + WRITE_SIZE,
    scaled by the plain-copy calibration); None when the kernel or planner sources have changed since."""
    try:
        for line in open(TRAFFIC_NOTE):
            if line.startswith("headline_step_hbm_bytes_per_launch="):
                fields = dict(kv.split("=") for kv in line.split())
                if fields.get("sources_sha256") == sources_digest():
                    return int(fields["headline_step_hbm_bytes_per_launch"])
    except (OSError, ValueError):
        pass
    return None


def device_pool(torch, batch, seed, copies=1):
    """N(0,1) bf16 page pool(s) made on the device (for steps whose outputs are not compared here)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    pools = []
    for _ in range(copies):
        p = torch.empty(batch.pool_shape(), dtype=torch.bfloat16, device="cuda")
        p.normal_(generator=g)
        pools.append(p)
    return pools


def time_launches(torch, hb, step, pools, iters, warmup):
    """Average duration of one attention launch, HIP events on the launch stream; pools are rotated so that
    consecutive launches do not find their KV in the last-level cache."""
    stream = torch.cuda.current_stream()
    for i in range(warmup):
        step.pool = pools[i % len(pools)]
        step.run(stream)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for i in range(iters):
        step.pool = pools[i % len(pools)]
        evs[i][0].record(stream)
        step.run(stream)
        evs[i][1].record(stream)
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in evs)
    return sum(ms) / len(ms), ms[len(ms) // 2], ms[0]


def path_figures(torch, hb, batch, pools, iters, warmup):
    """Attention launches only of one step: time, and the figures of whichever kinds of work it holds."""
    step = hb.DeviceStep(batch, pool_dev=pools[0])
    avg, med, best = time_launches(torch, hb, step, pools, iters, warmup)
    out = {"workload": batch.name, "requests": batch.num_requests, "query_tokens": batch.total_q,
           "launch_ms_avg": round(avg, 4), "launch_ms_median": round(med, 4), "launch_ms_min": round(best, 4),
           "tokens_per_s": round(batch.total_q / avg * 1e3, 1)}
    n_dec = int((batch.kind == 0).sum())
    if n_dec == batch.num_requests:
        byt = batch.decode_io_bytes()
        out.update(bound="hbm", algorithmic_bytes=byt, achieved_GBs=round(byt / avg / 1e6, 1),
                   frac_of_hbm_peak=round(byt / avg / 1e6 / HBM_PEAK_GBS, 4),
                   kv_tokens_per_s=round(float(batch.ctx_len.sum()) / avg * 1e3, 1))
    elif n_dec == 0:
        fl = batch.prefill_flops()
        out.update(bound="mfma", algorithmic_flops=fl, achieved_TFLOPs=round(fl / avg / 1e9, 1),
                   frac_of_bf16_mfma_peak=round(fl / avg / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4))
    else:
        byt = batch.decode_io_bytes() + batch.prefill_io_bytes()
        out.update(algorithmic_bytes=byt, achieved_GBs=round(byt / avg / 1e6, 1),
                   algorithmic_flops=batch.prefill_flops())
    del step
    return out


def append_figures(torch, hb, batch, pool, iters, warmup):
    """hfx_append_kv of the step's chunk tokens (the call that precedes the attention of a step)."""
    step = hb.DeviceStep(batch, pool_dev=pool)
    T, Hkv, D = batch.total_q, batch.num_kv_heads, batch.head_dim
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    k_new = torch.empty((T, Hkv, D), dtype=torch.bfloat16, device="cuda").normal_(generator=g)
    v_new = torch.empty((T, Hkv, D), dtype=torch.bfloat16, device="cuda").normal_(generator=g)
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        step.append(k_new, v_new, stream)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for a, c in evs:
        a.record(stream)
        step.append(k_new, v_new, stream)
        c.record(stream)
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(c) for a, c in evs)
    avg = sum(ms) / len(ms)
    byt = 2 * (2 * T * Hkv * D * 2)        # K and V, read once and written once
    return {"workload": batch.name + "/append", "tokens": T, "launch_ms_avg": round(avg, 5),
            "launch_ms_min": round(ms[0], 5), "bound": "hbm", "algorithmic_bytes": byt,
            "achieved_GBs": round(byt / avg / 1e6, 1)}


def copy_figures(torch, hb, batch, src, dst, iters, warmup):
    """hfx_copy_pages of every page the step's requests hold, from one pool into another."""
    ids = np_unique_pages(batch)
    shape = hb.make_shape(batch.num_q_heads, batch.num_kv_heads, batch.head_dim, batch.num_pages, 0.0)
    host_stage = torch.empty(8 * len(ids), dtype=torch.uint8, pin_memory=True)
    dev_stage = torch.empty(8 * len(ids), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        hb.hfx_copy_pages(shape, src, dst, batch.num_pages, ids, ids, host_stage, dev_stage, stream)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for a, c in evs:
        a.record(stream)
        hb.hfx_copy_pages(shape, src, dst, batch.num_pages, ids, ids, host_stage, dev_stage, stream)
        c.record(stream)
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(c) for a, c in evs)
    avg = sum(ms) / len(ms)
    page_bytes = batch.num_kv_heads * 2 * 16 * batch.head_dim * 2
    byt = 2 * len(ids) * page_bytes          # every page read once and written once
    return {"workload": batch.name + "/page-copy", "pages": int(len(ids)), "launch_ms_avg": round(avg, 5),
            "launch_ms_min": round(ms[0], 5), "bound": "hbm", "algorithmic_bytes": byt,
            "achieved_GBs": round(byt / avg / 1e6, 1), "frac_of_hbm_peak": round(byt / avg / 1e6 / HBM_PEAK_GBS, 4)}


def np_unique_pages(batch):
    import numpy as np
    return np.unique(batch.bt_pages).astype(np.int32)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--pool-copies", type=int, default=4, help="distinct KV pools rotated across steps")
    ap.add_argument("--no-paths", action="store_true", help="skip the decode-heavy / prefill-heavy steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--event-every", type=int, default=8,
                    help="bracket every N-th timed step's attention call with HIP timing events (each pair "
                         "costs the stream about 6 us, so bracketing every step would slow the loop it measures)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy a few times (reference dispatches for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU; there is no sharded path to time (--gpus must be 1)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2508_15919_amd import binding as hb
    from paper_2508_15919_amd import synth

    hb.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.int32, device="cuda").fill_(7)      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    b = synth.config(2)
    pools = [torch.from_numpy(b.pool.view(np.int16)).cuda()]
    for i in range(1, max(1, args.pool_copies)):
        pools.append(pools[0].clone())
    ring = [hb.DeviceStep(b, pool_dev=pools[i % len(pools)]) for i in range(max(4, len(pools)))]
    torch.cuda.synchronize()

    # host cost of building + uploading the descriptor alone
    t0 = time.perf_counter()
    for i in range(50):
        ring[i % len(ring)].build(stream)
        torch.cuda.synchronize()
    desc_us = (time.perf_counter() - t0) / 50 * 1e6

    every = max(1, args.event_every)
    ev0 = {i: torch.cuda.Event(enable_timing=True) for i in range(0, args.steps, every)}
    ev1 = {i: torch.cuda.Event(enable_timing=True) for i in ev0}
    busy = [None] * len(ring)
    uploaded = [torch.cuda.Event() for _ in ring]
    upload_stream = torch.cuda.Stream()      # default priority; carries only the descriptor uploads

    def one_step(i, timed):
        # the descriptor of step i is planned on the host and uploaded on a side stream while the
        # launch of step i-1 is still running; the launch stream waits for the upload only
        k = i % len(ring)
        s = ring[k]
        if busy[k] is not None:
            busy[k].synchronize()        # the slot's previous upload and launch have drained
        s.build(upload_stream)
        uploaded[k].record(upload_stream)
        stream.wait_event(uploaded[k])
        if timed and i in ev0:
            ev0[i].record(stream)
            s.run(stream)
            ev1[i].record(stream)
            busy[k] = ev1[i]
        else:
            s.run(stream)
            busy[k] = torch.cuda.Event()
            busy[k].record(stream)

    for i in range(args.warmup):
        one_step(i, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(i, True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    launch_ms = [ev0[i].elapsed_time(ev1[i]) for i in ev0]
    launch_avg = sum(launch_ms) / len(launch_ms)

    T = b.total_q
    alg_bytes = b.decode_io_bytes() + b.prefill_io_bytes()
    achieved = alg_bytes / launch_avg / 1e6
    result = {
        "metric": "mixed-step attention tokens/s", "value": round(T / ms_per_step * 1e3, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg2: Llama-3-8B-shaped layer (32 q / 8 kv heads, D 128, page 16), 64 decodes "
                               "ctx~lognormal(median 1k, max 8k) + 2 prompt chunks of 512 (ctx 512 and 2048)",
                   "requests": b.num_requests, "query_tokens": T, "decode_kv_tokens": int(b.ctx_len[b.kind == 0].sum()),
                   "pool_copies_rotated": len(pools), "step": "descriptor build + upload (side stream, overlapping the previous launch) + one attention call"},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(),
                     "kernel": "mixed_attention_kernel<128> (+ merge_kernel<128>, same API call)",
                     "launch_ms_avg": round(launch_avg, 5), "launches_timed": len(launch_ms),
                     "algorithmic_bytes": alg_bytes},
        "launch_only_tokens_per_s": round(T / launch_avg * 1e3, 1),
        "desc_build_upload_us": round(desc_us, 1),
        "prefill_flops": b.prefill_flops(),
    }

    # the oracle runs last: its worker threads keep spinning for a while after a parallel region and
    # take the core from the thread that enqueues the launches timed below
    got_bits = None if args.no_cpu_baseline else ring[0].out_bits()

    if not args.no_paths:
        paths = {}

        def leg(name, fn):
            try:
                paths[name] = fn()
            except Exception as e:  # the headline above stands on its own
                paths[name] = {"error": repr(e)}

        # the two pure steps hidden in the headline step (the paper's E_d and E_p), over the same pools
        leg("cfg2_decode_only", lambda: path_figures(torch, hb, b.sub_batch(synth.DECODE), pools, 100, 10))
        leg("cfg2_prefill_only", lambda: path_figures(torch, hb, b.sub_batch(synth.PREFILL), pools, 100, 10))
        if all("launch_ms_avg" in paths[k] for k in ("cfg2_decode_only", "cfg2_prefill_only")):
            td, tp = paths["cfg2_decode_only"]["launch_ms_avg"], paths["cfg2_prefill_only"]["launch_ms_avg"]
            paths["cfg2_mixed_vs_parts"] = {"mixed_ms": round(launch_avg, 4), "max_of_parts_ms": round(max(td, tp), 4),
                                            "sum_of_parts_ms": round(td + tp, 4)}
        # the same step with one pool only: consecutive launches find most of their KV in the last-level cache
        leg("cfg2_warm_single_pool", lambda: path_figures(torch, hb, b, pools[:1], 100, 10))
        leg("cfg2_kv_append", lambda: append_figures(torch, hb, b, pools[0], 100, 10))
        if len(pools) > 1:      # the pools are copies of each other, so the move leaves their contents as they are
            leg("cfg2_page_copy", lambda: copy_figures(torch, hb, b, pools[0], pools[1], 50, 5))
        del ring
        pools.clear()
        torch.cuda.empty_cache()

        def big(which, part=None):
            bb = synth.config(which, fill_pool=False)
            if part is not None:
                bb = bb.sub_batch(part)
            pp = device_pool(torch, bb, 1000 + which, copies=1 if bb.num_pages * bb.num_kv_heads > (1 << 19) else 2)
            try:
                return path_figures(torch, hb, bb, pp, 30, 5)
            finally:
                del pp
                torch.cuda.empty_cache()

        leg("decode_heavy", lambda: big(3))
        leg("prefill_heavy", lambda: big(4, synth.PREFILL))
        # the long-context tensor-parallel share (8 q-heads on 1 kv-head), its two halves
        leg("cfg5_decode_part", lambda: big(5, synth.DECODE))
        leg("cfg5_prefill_part", lambda: big(5, synth.PREFILL))

        def short_context():
            bb = synth.table1_short_context(seed=7, requests_per_task=64)
            pp = [torch.from_numpy(bb.pool.view(np.int16)).cuda()]
            out = path_figures(torch, hb, bb, pp, 100, 10)
            st = hb.DeviceStep(bb, pool_dev=pp[0])
            t0 = time.perf_counter()
            for _ in range(50):
                st.build(stream)
                torch.cuda.synchronize()
            out["desc_build_upload_us"] = round((time.perf_counter() - t0) / 50 * 1e6, 1)
            return out

        leg("table1_short_context", short_context)

        def latency_model():
            # E_p = a + b*n_token (the linear model of the paper's token-budget formula), fitted to this
            # kernel on prompt batches with Table-1 lengths; E_d = the headline step's decode part
            ns, ts = [], []
            for rpt in (4, 8, 16, 32, 64, 128):
                bb = synth.table1_short_context(seed=11, requests_per_task=rpt).sub_batch(synth.PREFILL)
                pp = [torch.from_numpy(bb.pool.view(np.int16)).cuda()]
                f = path_figures(torch, hb, bb, pp, 50, 5)
                ns.append(bb.total_q)
                ts.append(f["launch_ms_avg"] * 1e-3)
            e_d = paths.get("cfg2_decode_only", {}).get("launch_ms_avg", 0.11) * 1e-3
            model, r2 = hb.hfx_fit_latency_model(ns, ts, e_d)
            ttft, tpot = 100 * e_d, 4 * e_d          # an example SLO pair in units of this layer's decode time
            return {"n_token": ns, "seconds": [round(t, 7) for t in ts], "a_s": model.a, "b_s_per_token": model.b,
                    "r_squared": round(r2, 5), "e_d_s": e_d,
                    "example": {"ttft_s": ttft, "tpot_s": tpot, "token_budget": hb.hfx_token_budget(ttft, tpot, model)}}

        leg("latency_model", latency_model)
        result["paths"] = paths

    if not args.no_cpu_baseline:
        from oracle import hfx_oracle
        hfx_oracle.attention_batch(synth.config(1))            # load + warm the library
        t0 = time.perf_counter()
        ref = hfx_oracle.attention_batch(b)
        cpu_s = time.perf_counter() - t0
        got = synth.bf16_bits_to_f64(got_bits)
        err = np.abs(got - ref)
        result["cpu_baseline"] = {"value": round(T / cpu_s, 2), "unit": "tokens/s", "cores": hfx_oracle.num_threads(),
                                  "kind": "oracle", "sample": "the whole cfg2 step, one run (%.2f s)" % cpu_s}
        result["parity_vs_oracle"] = {"max_abs": float(err.max()), "mean_abs": float(err.mean())}


    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
