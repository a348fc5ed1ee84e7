#!/usr/bin/env python3
"""Benchmark of libjigsaw_decode: paged decode attention on one MI355X.

A step is one jd_decode_attention call (work partition + split-KV partial pass + combine) over
one synthetic decode batch that is already resident in HBM.  The default workload is the
long-tailed Qwen3-8B-like rollout step (batch 256, 32 q / 8 kv heads, head_dim 128, 16-token
pages, 512-token prompt + lognormal response); `--cfg` selects another of the five configs.

Prints ONE JSON line: the metric (KV bytes read per second, i.e. T * 2 * Hkv * D * 2 bytes per
step over the step time), a `roofline` object for the dominant kernel (the partial pass, timed
with HIP events on the launch stream inside the timed region), and a `cpu_baseline` object (the
fp64 CPU oracle timed on the host cores on a bounded sample of the same workload).
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--cfg", type=int, default=2, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--variant", type=int, default=0, help="0 default, 1 vector, 2 mfma")
    ap.add_argument("--cu-budget", type=int, default=0)
    ap.add_argument("--sweep", choices=["none", "cu", "batch", "merge", "loop", "prefill"], default="none",
                    help="extra measurements after the timed region: 'cu' = step time at 25/50/75/100 %% of the "
                         "compute units (the library's cu_budget), 'batch' = step time as the batch shrinks to its "
                         "longest requests, 'merge' = the straggler batches of n = 1, 2, 4, 8 workers (cfg3 draws) merged into one, "
                         "'loop' = the closed decode loop (KV append + attention) eager and as a replayed "
                         "HIP graph, 'prefill' = causal prefill over the paged cache (KV recomputation of migrated requests, "
                         "a new turn after a context) against the matrix-core peak")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="CPU-seconds budget of the oracle sample")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU by design (decode attention shards by request or by kv head "
              "with no exchange); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2604_23838_amd import binding as jb
    from paper_2604_23838_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = torch.device("cuda:0")
    t0 = time.time()
    w = W.gen_config(args.cfg, args.seed, threads=min(16, os.cpu_count() or 8))
    s = w.shape
    print(f"[bench] generated cfg{args.cfg} ({s.name}) T={w.total_tokens} KV={w.kv_bytes / 1e9:.3f} GB "
          f"in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)
    q = torch.from_numpy(w.q.view(np.int16)).to(dev).view(torch.bfloat16)
    kp = torch.from_numpy(w.k_pages.view(np.int16)).to(dev).view(torch.bfloat16)
    vp = torch.from_numpy(w.v_pages.view(np.int16)).to(dev).view(torch.bfloat16)
    bt = torch.from_numpy(w.block_table).to(dev)
    sl = torch.from_numpy(w.seq_lens).to(dev)
    out = torch.empty((s.batch, s.num_q_heads, s.head_dim), dtype=torch.float32, device=dev)
    op = jb.DecodeAttention(s.batch, s.num_q_heads, s.num_kv_heads, s.head_dim, w.max_pages_per_seq, w.num_pages,
                            variant=args.variant, cu_budget=args.cu_budget)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for _ in range(args.warmup):
            op(q, kp, vp, bt, sl, out)
        torch.cuda.synchronize()
        # HIP events around the kernels of every 8th step of the timed region (an event record costs
        # stream time, so timing every step would slow down the very steps being measured)
        every = 8
        jb.jd_profile_enable(op.handle, (args.steps + every - 1) // every, every)
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for _ in range(args.steps):
            op(q, kp, vp, bt, sl, out)
        torch.cuda.synchronize()
        t_end = time.perf_counter()
        ms_sum, calls = jb.jd_profile_read(op.handle)
        jb.jd_profile_enable(op.handle, 0, 1)
    # measured ceiling of a plain read sweep over the K pool (same stream, same process)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    nbytes = kp.numel() * 2
    with torch.cuda.stream(stream):
        for _ in range(3):
            jb.jd_debug_stream_read(kp.data_ptr(), nbytes, sink.data_ptr(), stream.cuda_stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(20):
            jb.jd_debug_stream_read(kp.data_ptr(), nbytes, sink.data_ptr(), stream.cuda_stream)
        e1.record(stream)
        torch.cuda.synchronize()
    read_ceiling = nbytes * 20 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    # a plain copy of known size (256 MiB read + 256 MiB written), so that a profiler run of this
    # command has a kernel to scale its byte counters against
    copy_bytes = min(256 << 20, nbytes // 2 // 16 * 16)
    dst = torch.empty(copy_bytes, dtype=torch.uint8, device=dev)
    with torch.cuda.stream(stream):
        for _ in range(3):
            jb.jd_debug_stream_copy(dst.data_ptr(), kp.data_ptr(), copy_bytes, stream.cuda_stream)
        torch.cuda.synchronize()
    del dst
    op.check_flags()
    # spread of single steps: an event pair around each of 100 more steps (the records add ~5 us of stream time
    # to each interval, so these sit a little above the timed region's mean)
    with torch.cuda.stream(stream):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(100)]
        for a, b in evs:
            a.record(stream)
            op(q, kp, vp, bt, sl, out)
            b.record(stream)
        torch.cuda.synchronize()
    single = np.sort(np.array([a.elapsed_time(b) * 1e3 for a, b in evs]))
    ms_per_step = (t_end - t_start) * 1e3 / args.steps
    kv_bytes = w.kv_bytes
    tbs = kv_bytes / (ms_per_step * 1e-3) / 1e12
    partial_ms = ms_sum[1] / max(calls, 1)
    achieved = kv_bytes / (partial_ms * 1e-3) / 1e9 if partial_ms > 0 else 0.0

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            with open(tpath) as f:
                traffic = json.load(f).get(f"cfg{args.cfg}_variant{args.variant}")
        except Exception:
            traffic = None

    result = {
        "metric": "decode_attention_kv_bandwidth",
        "value": round(tbs, 4),
        "unit": "TB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "us_per_step": round(ms_per_step * 1e3, 2),
        "single_step_us": {"p10": round(float(single[10]), 2), "median": round(float(single[50]), 2),
                           "p90": round(float(single[90]), 2), "note": "event pair per step, 100 steps"},
        "pct_of_hbm_peak": round(100.0 * tbs * 1e3 / HBM_PEAK_GBS, 2),
        "stream_read_ceiling_gbs": round(read_ceiling, 1),
        "calibration_copy_bytes": copy_bytes,
        "pct_of_stream_read_ceiling": round(100.0 * tbs * 1e3 / read_ceiling, 2),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "accumulate": "f32",
        "data": "synthetic",
        "config": {"workload": f"cfg{args.cfg} {s.name}: batch {s.batch}, {s.num_q_heads}q/{s.num_kv_heads}kv heads, "
                               f"head_dim {s.head_dim}, page 16, seed {args.seed}, T={w.total_tokens} tokens",
                   "kv_bytes_per_step": kv_bytes, "variant": args.variant, "cu_budget": args.cu_budget,
                   "derived_us_per_model_step": round(ms_per_step * 1e3 * s.layers, 1), "layers": s.layers},
        "kernel_ms": {"partition": round(ms_sum[0] / max(calls, 1), 5), "partial": round(partial_ms, 5),
                      "combine": round(ms_sum[2] / max(calls, 1), 5)},
        "roofline": {"bound": "hbm", "kernel": "decode_fused_kernel (partition + split-KV partial attention + combine)" if args.variant != 1 else "partial_vector_kernel", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic},
    }

    def time_steps(o, lens_t, steps=60, warm=10):
        with torch.cuda.stream(stream):
            for _ in range(warm):
                o(q, kp, vp, bt, lens_t, out)
            torch.cuda.synchronize()
            t0_ = time.perf_counter()
            for _ in range(steps):
                o(q, kp, vp, bt, lens_t, out)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0_) * 1e6 / steps

    if args.sweep == "cu":
        # the paper bounds the SMs a sub-stage may use and finds small-batch rollout insensitive to them
        # (Sub-stage Multiplexing, "Compute Resource Utilization"); the same experiment with the library's CU budget
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        rows = []
        for pct in (25, 50, 75, 100):
            o2 = jb.DecodeAttention(s.batch, s.num_q_heads, s.num_kv_heads, s.head_dim, w.max_pages_per_seq,
                                    w.num_pages, variant=args.variant, cu_budget=cus * pct // 100)
            us = time_steps(o2, sl)
            o2.close()
            rows.append({"cu_pct": pct, "cu_budget": cus * pct // 100, "us_per_step": round(us, 2),
                         "kv_tb_per_s": round(kv_bytes / us / 1e6, 4)})
        result["cu_budget_sweep"] = rows
    if args.sweep == "batch":
        # the effective batch shrinks as short responses finish (Motivation, "Varied Decoding Lengths"):
        # keep the k longest requests active, the others are finished rows (seq_len 0) of the same batch
        order = np.argsort(-w.seq_lens.astype(np.int64), kind="stable")
        rows = []
        k = s.batch
        while k >= 1:
            lens_k = np.zeros_like(w.seq_lens)
            lens_k[order[:k]] = w.seq_lens[order[:k]]
            lt = torch.from_numpy(lens_k).to(dev)
            us = time_steps(op, lt)
            kvb = int(lens_k.astype(np.int64).sum()) * 2 * s.num_kv_heads * s.head_dim * 2
            rows.append({"active_requests": k, "tokens": int(lens_k.astype(np.int64).sum()), "us_per_step": round(us, 2),
                         "kv_tb_per_s": round(kvb / us / 1e6, 4)})
            k //= 2
        result["shrinking_batch_sweep"] = rows
        with torch.cuda.stream(stream):
            op(q, kp, vp, bt, sl, out)     # restore the full batch's output for the parity check below
            torch.cuda.synchronize()

    if args.sweep == "merge":
        # long-tail migration aggregates the stragglers of n DP workers on one target (Sub-stage Merging):
        # n independent cfg3 draws merged into one batch; a bandwidth-bound kernel should charge the sum of the bytes
        s3 = W.SHAPES[3]
        rows = []
        for n in (1, 2, 4, 8):
            lens_m = np.concatenate([W.draw_seq_lens(3, np.random.default_rng(args.seed + i)) for i in range(n)])
            wm = W.build(dataclasses.replace(s3, batch=len(lens_m)), lens_m, seed=args.seed, cfg=30 + n,
                         threads=min(16, os.cpu_count() or 8))
            qm = torch.from_numpy(wm.q.view(np.int16)).to(dev).view(torch.bfloat16)
            km = torch.from_numpy(wm.k_pages.view(np.int16)).to(dev).view(torch.bfloat16)
            vm = torch.from_numpy(wm.v_pages.view(np.int16)).to(dev).view(torch.bfloat16)
            btm = torch.from_numpy(wm.block_table).to(dev)
            slm = torch.from_numpy(wm.seq_lens).to(dev)
            om = torch.empty((len(lens_m), s3.num_q_heads, s3.head_dim), dtype=torch.float32, device=dev)
            o2 = jb.DecodeAttention(len(lens_m), s3.num_q_heads, s3.num_kv_heads, s3.head_dim, wm.max_pages_per_seq,
                                    wm.num_pages, variant=args.variant)
            with torch.cuda.stream(stream):
                for _ in range(10):
                    o2(qm, km, vm, btm, slm, om)
                torch.cuda.synchronize()
                t0_ = time.perf_counter()
                for _ in range(100):
                    o2(qm, km, vm, btm, slm, om)
                torch.cuda.synchronize()
                us = (time.perf_counter() - t0_) * 1e6 / 100
            o2.close()
            rows.append({"workers_merged": n, "requests": len(lens_m), "tokens": wm.total_tokens,
                         "us_per_step": round(us, 2), "kv_tb_per_s": round(wm.kv_bytes / us / 1e6, 4)})
            del qm, km, vm, om
        for r in rows:
            r["us_vs_n_times_single"] = round(r["us_per_step"] / (rows[0]["us_per_step"] * r["workers_merged"]), 3)
        result["merged_straggler_sweep"] = rows

    if args.sweep == "loop":
        # a closed decode loop: every step appends one token per request and attends over the grown cache.
        # The requests start 64 tokens short of their generated length, so they grow back into pages they own.
        steps_l = 64
        start = np.maximum(w.seq_lens - steps_l, 1).astype(np.int32)
        lt = torch.from_numpy(start).to(dev)
        kn = torch.randn((s.batch, s.num_kv_heads, s.head_dim), device=dev).bfloat16()
        vn = torch.randn((s.batch, s.num_kv_heads, s.head_dim), device=dev).bfloat16()
        res = {}
        with torch.cuda.stream(stream):
            for mode in ("eager", "graph"):
                lt.copy_(torch.from_numpy(start))
                op.append(kn, vn, kp, vp, bt, lt)
                op(q, kp, vp, bt, lt, out)
                torch.cuda.synchronize()
                lt.copy_(torch.from_numpy(start))
                if mode == "graph":
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=stream):
                        op.append(kn, vn, kp, vp, bt, lt)
                        op(q, kp, vp, bt, lt, out)
                torch.cuda.synchronize()
                t0_ = time.perf_counter()
                for _ in range(steps_l - 1):
                    if mode == "graph":
                        g.replay()
                    else:
                        op.append(kn, vn, kp, vp, bt, lt)
                        op(q, kp, vp, bt, lt, out)
                torch.cuda.synchronize()
                res[mode] = (time.perf_counter() - t0_) * 1e6 / (steps_l - 1)
            lt.copy_(torch.from_numpy(start))
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(steps_l - 1):
                op.append(kn, vn, kp, vp, bt, lt)
            e1.record(stream)
            torch.cuda.synchronize()
            append_us = e0.elapsed_time(e1) * 1e3 / (steps_l - 1)
        result["decode_loop"] = {"steps": steps_l - 1, "us_per_step_eager": round(res["eager"], 2),
                                 "us_per_step_graph": round(res["graph"], 2),
                                 "append_only_us": round(append_us, 2),
                                 "append_bytes": 4 * s.batch * s.num_kv_heads * s.head_dim * 2,
                                 "note": "the K/V pool now holds 64 synthetic tokens per request: parity check skipped"}
        args.no_cpu_baseline = True

    if args.sweep == "prefill":
        # KV recomputation after a migration and the prefill of a new turn (Sub-stage Merging; Motivation,
        # "Multi-turn Rollout Idling"), on this config's head shape and length distribution
        MFMA_PEAK_TFLOPS = 2500.0   # dense bf16
        rows = []
        nreq = min(32, s.batch)
        base = w.seq_lens[:nreq].astype(np.int64)
        for name, lens_p, ql_p in (("recompute_whole_request", base, base),
                                    ("new_turn_512_after_context", base + 512, np.full(nreq, 512, dtype=np.int64))):
            wp = W.build(dataclasses.replace(s, batch=nreq), lens_p.astype(np.int32), seed=args.seed + 1, cfg=70,
                         threads=min(16, os.cpu_count() or 8))
            offs = np.concatenate([[0], np.cumsum(ql_p)[:-1]]).astype(np.int32)
            tq = int(ql_p.sum())
            qp = torch.randn((tq, s.num_q_heads, s.head_dim), device=dev).bfloat16()
            kpp = torch.from_numpy(wp.k_pages.view(np.int16)).to(dev).view(torch.bfloat16)
            vpp = torch.from_numpy(wp.v_pages.view(np.int16)).to(dev).view(torch.bfloat16)
            btp = torch.from_numpy(wp.block_table).to(dev)
            slp = torch.from_numpy(wp.seq_lens).to(dev)
            qlp = torch.from_numpy(ql_p.astype(np.int32)).to(dev)
            ofp = torch.from_numpy(offs).to(dev)
            outp = torch.empty((tq, s.num_q_heads, s.head_dim), dtype=torch.float32, device=dev)
            o2 = jb.DecodeAttention(nreq, s.num_q_heads, s.num_kv_heads, s.head_dim, wp.max_pages_per_seq, wp.num_pages)
            reps = 10
            with torch.cuda.stream(stream):
                for _ in range(2):
                    o2.prefill(qp, kpp, vpp, btp, slp, qlp, ofp, int(ql_p.max()), out=outp)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(reps):
                    o2.prefill(qp, kpp, vpp, btp, slp, qlp, ofp, int(ql_p.max()), out=outp)
                e1.record(stream)
                torch.cuda.synchronize()
            o2.check_flags()
            o2.close()
            ms = e0.elapsed_time(e1) / reps
            ctx = lens_p - ql_p
            pairs = int((ql_p * ctx + ql_p * (ql_p + 1) // 2).sum())      # (query, key) pairs under the causal mask
            flops = 4.0 * s.num_q_heads * s.head_dim * pairs
            rows.append({"case": name, "requests": nreq, "new_tokens": tq, "kv_tokens": int(lens_p.sum()),
                         "ms": round(ms, 4), "new_tokens_per_s": round(tq / ms * 1e3, 1),
                         "roofline": {"bound": "mfma", "achieved": round(flops / ms / 1e9, 2), "peak": MFMA_PEAK_TFLOPS,
                                      "unit": "TFLOP/s", "frac": round(flops / ms / 1e9 / MFMA_PEAK_TFLOPS, 4),
                                      "traffic": None}})
            del kpp, vpp, qp, outp
        result["prefill_sweep"] = rows

    if not args.no_cpu_baseline:
        from oracle import jo
        cores = jo.max_threads()
        # bounded sample: whole requests, taken in batch order until the CPU-seconds budget is used
        # (the oracle does ~4*L*Hq*D fp64 flops per request at a few GFLOP/s per core)
        flops_budget = args.cpu_seconds * 1.0e9
        rows, used = [], 0.0
        for b in range(s.batch):
            f = 4.0 * float(w.seq_lens[b]) * s.num_q_heads * s.head_dim
            if rows and used + f > flops_budget:
                break
            rows.append(b)
            used += f
        sub = W.subset_requests(w, rows)
        passes, dt = 0, 0.0
        while passes == 0 or (dt * cores < 0.75 * args.cpu_seconds and passes < 16):
            t1 = time.perf_counter()
            ref = jo.decode_attention(sub.q, sub.k_pages, sub.v_pages, sub.block_table, sub.seq_lens)
            dt += time.perf_counter() - t1
            passes += 1
        dt /= passes
        got = out[torch.tensor(rows, device=dev)].cpu().numpy()
        diff = np.abs(got.astype(np.float64) - ref.astype(np.float64))
        max_abs = float(diff.max())
        max_rel = float((diff / np.maximum(np.abs(ref.astype(np.float64)), 1e-3)).max())
        result["cpu_baseline"] = {"value": round(sub.kv_bytes / dt / 1e12, 6), "unit": "TB/s", "cores": cores,
                                  "kind": "oracle",
                                  "sample": f"first {len(rows)} of {s.batch} requests ({sub.total_tokens} tokens, "
                                            f"{sub.kv_bytes / 1e9:.3f} GB of KV), fp64, {passes} passes, "
                                            f"{dt:.2f}s wall each"}
        # the same oracle on one core, on the first requests only (a few seconds)
        rows1, used1 = [], 0.0
        for b in rows:
            f = 4.0 * float(w.seq_lens[b]) * s.num_q_heads * s.head_dim
            if rows1 and used1 + f > 0.25 * args.cpu_seconds * 1.0e9:
                break
            rows1.append(b)
            used1 += f
        sub1 = W.subset_requests(w, rows1)
        t1 = time.perf_counter()
        jo.decode_attention(sub1.q, sub1.k_pages, sub1.v_pages, sub1.block_table, sub1.seq_lens, threads=1)
        dt1 = time.perf_counter() - t1
        result["cpu_baseline"]["one_core"] = {"value": round(sub1.kv_bytes / dt1 / 1e12, 6), "unit": "TB/s",
                                              "sample": f"first {len(rows1)} requests ({sub1.total_tokens} tokens), "
                                                        f"{dt1:.2f}s wall"}
        result["parity_on_sample"] = {"max_abs": max_abs, "max_rel_floor1e-3": max_rel,
                                      "ok": bool(max_abs <= 5e-3 and max_rel <= 1e-2)}
    op.close()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
