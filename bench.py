#!/usr/bin/env python3
"""Benchmark of libhfxattn on one MI355X.

A step is one pass of the whole hot path over one scheduled batch: the host builds the batch
descriptor and uploads it (hfx_build_batch_desc), then one persistent launch executes the mixed
prefill/decode paged attention (hfx_mixed_paged_attention).  Inputs are resident in HBM before
the timed region.  The headline workload is the whole prefill-heavy mixed step (4 prompt chunks
of 2048 tokens on prior contexts 0/4k/8k/12k plus 32 decodes at about 2k context; Llama-3-8B head
shape), whose dominant kernel is bound by the bf16 matrix cores; the decode-heavy step (HBM-bound)
rides inside "roofline" as its "hbm" part, and the other configurations, the pure-prefill and
pure-decode parts of the mixed steps, the KV append, the page copy, the short-context step and
the fitted latency model are reported under "paths".

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
            if line.startswith("cfg4_step_hbm_bytes_per_launch="):
                fields = dict(kv.split("=") for kv in line.split())
                if fields.get("sources_sha256") == sources_digest():
                    return int(fields["cfg4_step_hbm_bytes_per_launch"])
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
    """Durations (ms, sorted) of `iters` attention launches after `warmup` untimed ones, HIP events on the
    launch stream; pools are rotated so that consecutive launches do not find their KV in the last-level cache."""
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
    return sorted(a.elapsed_time(b) for a, b in evs)


def path_figures(torch, hb, batch, pools, iters=60, warmup=10):
    """Attention launches only of one step: median of `iters` launches after `warmup`, and the figures of
    whichever kinds of work the step holds (computed on the median)."""
    step = hb.DeviceStep(batch, pool_dev=pools[0])
    ms = time_launches(torch, hb, step, pools, iters, warmup)
    avg, med, best = sum(ms) / len(ms), ms[len(ms) // 2], ms[0]
    out = {"workload": batch.name, "requests": batch.num_requests, "query_tokens": batch.total_q,
           "launches": iters, "warmup": warmup,
           "launch_ms_median": round(med, 4), "launch_ms_avg": round(avg, 4), "launch_ms_min": round(best, 4),
           "tokens_per_s": round(batch.total_q / med * 1e3, 1)}
    n_dec = int((batch.kind == 0).sum())
    if n_dec > 0:
        byt = batch.decode_io_bytes() + (batch.prefill_io_bytes() if n_dec < batch.num_requests else 0)
        out.update(algorithmic_bytes=byt, achieved_GBs=round(byt / med / 1e6, 1),
                   frac_of_hbm_peak=round(byt / med / 1e6 / HBM_PEAK_GBS, 4))
    if n_dec == batch.num_requests:
        out.update(bound="hbm", kv_tokens_per_s=round(float(batch.ctx_len.sum()) / med * 1e3, 1))
    if n_dec < batch.num_requests:
        fl = batch.prefill_flops()
        out.update(algorithmic_flops=fl, achieved_TFLOPs=round(fl / med / 1e9, 1),
                   frac_of_bf16_mfma_peak=round(fl / med / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4))
        if n_dec == 0:
            out.update(bound="mfma")
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
    med = ms[len(ms) // 2]
    byt = 2 * (2 * T * Hkv * D * 2)        # K and V, read once and written once
    return {"workload": batch.name + "/append", "tokens": T, "launch_ms_median": round(med, 5),
            "launch_ms_min": round(ms[0], 5), "bound": "hbm", "algorithmic_bytes": byt,
            "achieved_GBs": round(byt / med / 1e6, 1)}


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
    med = ms[len(ms) // 2]
    page_bytes = batch.num_kv_heads * 2 * 16 * batch.head_dim * 2
    byt = 2 * len(ids) * page_bytes          # every page read once and written once
    return {"workload": batch.name + "/page-copy", "pages": int(len(ids)), "launch_ms_median": round(med, 5),
            "launch_ms_min": round(ms[0], 5), "bound": "hbm", "algorithmic_bytes": byt,
            "achieved_GBs": round(byt / med / 1e6, 1), "frac_of_hbm_peak": round(byt / med / 1e6 / HBM_PEAK_GBS, 4)}


def np_unique_pages(batch):
    import numpy as np
    return np.unique(batch.bt_pages).astype(np.int32)


def mixed_vs_parts(paths, whole, dec, pre):
    """The mixed step against its pure-decode and pure-prefill parts (medians)."""
    if all("launch_ms_median" in paths.get(k, {}) for k in (whole, dec, pre)):
        td, tp = paths[dec]["launch_ms_median"], paths[pre]["launch_ms_median"]
        return {"mixed_ms": paths[whole]["launch_ms_median"], "max_of_parts_ms": round(max(td, tp), 4),
                "sum_of_parts_ms": round(td + tp, 4)}
    return {"error": "a part is missing"}


def oracle_sample(batch, every):
    """(request, chunk row, q-head) triples for the timed oracle run: every decode request and every
    `every`-th row of each prompt chunk (the first row shifted by the request index, so that the rows fall on
    all positions of a tile), all q-heads; and the share of the step's multiply-adds they stand for."""
    req, row, head = [], [], []
    work = total = 0
    for r in range(batch.num_requests):
        q, c = int(batch.q_len[r]), int(batch.ctx_len[r])
        p = c - q
        total += q * p + q * (q + 1) // 2
        rows = [0] if batch.kind[r] == 0 else list(range(r % every, q, every))
        for i in rows:
            work += p + i + 1
            for h in range(batch.num_q_heads):
                req.append(r); row.append(i); head.append(h)
    return req, row, head, work / total


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--pool-copies", type=int, default=2, help="distinct KV pools rotated across steps")
    ap.add_argument("--no-paths", action="store_true", help="headline step only (no roofline.hbm, no paths)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--event-every", type=int, default=1,
                    help="bracket every N-th timed step's attention call with HIP timing events (a pair costs "
                         "the stream about 6 us, half a percent of this step)")
    ap.add_argument("--oracle-every", type=int, default=3,
                    help="the timed oracle run takes every N-th row of each prompt chunk (1 = the whole step)")
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

    b = synth.config(4)
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
    launch_ms = sorted(ev0[i].elapsed_time(ev1[i]) for i in ev0)
    launch_avg = sum(launch_ms) / len(launch_ms)

    T = b.total_q
    flops = b.prefill_flops()
    alg_bytes = b.decode_io_bytes() + b.prefill_io_bytes()
    achieved = flops / launch_avg / 1e9
    result = {
        "metric": "mixed-step attention tokens/s", "value": round(T / ms_per_step * 1e3, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg4: prefill-heavy mixed step, whole (32 q / 8 kv heads, D 128, page 16): 4 prompt chunks "
                               "of 2048 tokens on prior contexts 0/4096/8192/12288 + 32 decodes at 2048+-256 context",
                   "requests": b.num_requests, "query_tokens": T, "decode_kv_tokens": int(b.ctx_len[b.kind == 0].sum()),
                   "pool_copies_rotated": len(pools), "step": "descriptor build + upload (side stream, overlapping the previous launch) + one attention call"},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": measured_traffic(),
                     "kernel": "mixed_attention_kernel<128> (+ merge_kernel<128>, same API call)",
                     "launch_ms_avg": round(launch_avg, 5), "launch_ms_median": round(launch_ms[len(launch_ms) // 2], 5),
                     "launches_timed": len(launch_ms),
                     "algorithmic_flops": flops, "algorithmic_bytes": alg_bytes, "hbm": None},
        "launch_only_tokens_per_s": round(T / launch_avg * 1e3, 1),
        "desc_build_upload_us": round(desc_us, 1),
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

        # the headline step again (launches only, median) and the two pure steps hidden in it (the paper's
        # E_p and E_d), over the same pools
        leg("cfg4_mixed", lambda: path_figures(torch, hb, b, pools))
        leg("cfg4_prefill_only", lambda: path_figures(torch, hb, b.sub_batch(synth.PREFILL), pools))
        leg("cfg4_decode_only", lambda: path_figures(torch, hb, b.sub_batch(synth.DECODE), pools, 100, 10))
        paths["cfg4_mixed_vs_parts"] = mixed_vs_parts(paths, "cfg4_mixed", "cfg4_decode_only", "cfg4_prefill_only")
        leg("cfg4_kv_append", lambda: append_figures(torch, hb, b, pools[0], 100, 10))
        if len(pools) > 1:      # the pools are copies of each other, so the move leaves their contents as they are
            leg("cfg4_page_copy", lambda: copy_figures(torch, hb, b, pools[0], pools[1], 50, 10))
        del ring
        pools.clear()
        torch.cuda.empty_cache()

        def with_pools(bb, seed, copies, fn):
            pp = device_pool(torch, bb, seed, copies=copies)
            try:
                return fn(pp)
            finally:
                del pp
                torch.cuda.empty_cache()

        # the decode-heavy step: the HBM-bound half of the metric
        b3 = synth.config(3, fill_pool=False)
        leg("decode_heavy", lambda: with_pools(b3, 1003, 1, lambda pp: path_figures(torch, hb, b3, pp)))
        dh = paths["decode_heavy"]
        if "achieved_GBs" in dh:
            result["roofline"]["hbm"] = {
                "workload": "cfg3: decode-heavy step, 256 decodes, contexts uniform 2048..16384, no prefill",
                "bound": "hbm", "achieved": dh["achieved_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": dh["frac_of_hbm_peak"], "algorithmic_bytes": dh["algorithmic_bytes"],
                "launch_ms_median": dh["launch_ms_median"], "launches_timed": dh["launches"]}

        # the Llama-3-8B-shaped mixed step (64 decodes + 2 chunks of 512) and its parts, 4 pools rotated
        b2 = synth.config(2, fill_pool=False)

        def cfg2_legs(pp):
            paths["cfg2_mixed"] = path_figures(torch, hb, b2, pp, 100, 10)
            paths["cfg2_decode_only"] = path_figures(torch, hb, b2.sub_batch(synth.DECODE), pp, 100, 10)
            paths["cfg2_prefill_only"] = path_figures(torch, hb, b2.sub_batch(synth.PREFILL), pp, 100, 10)
            paths["cfg2_mixed_vs_parts"] = mixed_vs_parts(paths, "cfg2_mixed", "cfg2_decode_only", "cfg2_prefill_only")
            # one pool only: consecutive launches find most of their KV in the last-level cache
            return path_figures(torch, hb, b2, pp[:1], 100, 10)

        leg("cfg2_warm_single_pool", lambda: with_pools(b2, 1002, 4, cfg2_legs))

        # the long-context tensor-parallel share (8 q-heads on 1 kv-head): whole step and its two halves
        b5 = synth.config(5, fill_pool=False)

        def cfg5_legs(pp):
            paths["cfg5_decode_only"] = path_figures(torch, hb, b5.sub_batch(synth.DECODE), pp, 100, 10)
            paths["cfg5_prefill_only"] = path_figures(torch, hb, b5.sub_batch(synth.PREFILL), pp)
            return path_figures(torch, hb, b5, pp)

        leg("cfg5_mixed", lambda: with_pools(b5, 1005, 2, cfg5_legs))
        paths["cfg5_mixed_vs_parts"] = mixed_vs_parts(paths, "cfg5_mixed", "cfg5_decode_only", "cfg5_prefill_only")

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
            # kernel on prompt batches with Table-1 lengths; E_d = the Llama-8B-shaped step's decode part
            ns, ts = [], []
            for rpt in (4, 8, 16, 32, 64, 128):
                bb = synth.table1_short_context(seed=11, requests_per_task=rpt).sub_batch(synth.PREFILL)
                pp = [torch.from_numpy(bb.pool.view(np.int16)).cuda()]
                f = path_figures(torch, hb, bb, pp, 50, 10)
                ns.append(bb.total_q)
                ts.append(f["launch_ms_median"] * 1e-3)
            e_d = paths.get("cfg2_decode_only", {}).get("launch_ms_median", 0.11) * 1e-3
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
        every = max(1, args.oracle_every)
        req, row, head, share = oracle_sample(b, every)
        t0 = time.perf_counter()
        ref = hfx_oracle.attention_rows_batch(b, req, row, head)
        cpu_s = time.perf_counter() - t0
        qi = b.q_indptr()
        got = synth.bf16_bits_to_f64(got_bits)[qi[np.array(req)] + np.array(row), np.array(head)]
        err = np.abs(got - ref)
        result["cpu_baseline"] = {
            "value": round(T * share / cpu_s, 2), "unit": "tokens/s", "cores": hfx_oracle.num_threads(), "kind": "oracle",
            "sample": "cfg4 step: all 32 decode requests and every %d-th row of each of the 4 prompt chunks, all 32 q-heads "
                      "(%d rows, %.1f %% of the step's multiply-adds) in %.2f s; value = step tokens x that share / seconds"
                      % (every, len(req), 100 * share, cpu_s)}
        result["parity_vs_oracle"] = {"rows": len(req), "max_abs": float(err.max()), "mean_abs": float(err.mean())}

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
