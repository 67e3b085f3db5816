#!/usr/bin/env python3
"""Benchmark of PQ decode attention on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--copies C] [--no-cpu-baseline] [--warm]
                    [--no-others] [--no-next]

A step is one pass of the hot path over one batch: pq_attn_decode (table build,
score pass, softmax, value pass, recent rows, split merge — one fused kernel) on
the configured workload; with --config 4 the step is pq_encode_append of 64 new
tokens per head followed by pq_attn_decode.  The default workload is the
Llama-2-7B-shaped layer at 32K context (batch 1, 32 heads, 4-bit PQ, 128 recent
tokens).  Inputs are synthetic and already resident in HBM.  The timed steps
rotate through several distinct copies of the code tensors (1 GiB in total) so
that the codes come from HBM and not from the 256 MB memory-side cache.

Prints ONE JSON line.  `value` = context tokens scanned per second
(sum_b (N_b + R_b) per step / wall time per step).  `roofline` prices the decode
kernel against HBM: algorithmic bytes per launch / average kernel duration, the
span between two HIP events on the launching stream around the K back-to-back
launches divided by K (so it includes the gap between kernels).
`cpu_baseline` is the double-precision oracle on the same workload on the host.
The default run (workload 1) also times the other named workloads — batched, grouped-query 128K, 2-bit +
encode — with fewer launches each and lists them under `other_workloads` (kernel time, algorithmic bytes,
fraction of the HBM peak); `value` stays the metric's workload.  It then runs the measurements of
bench_extra.py for the operations around the path (bulk encode at prompt shape, encode on a second stream,
codebook training, 12-bit codes) and lists their results under `next_rows`, each with its own roofline figure.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published


def algorithmic_bytes(w, data):
    """Bytes the method itself must move for one decode launch: K and V codes of every
    cached token (2*M per token per KV head), the recent rows, each KV head's two
    codebooks once, q in and the fp32 output row out."""
    import numpy as np
    eb = 2 if w.dtype == "f16" else 4
    n_tok = int(np.asarray(data["ctx_len"], dtype=np.int64).sum()) + (w.n_new * w.batch)
    codes = n_tok * w.n_kv_heads * 2 * w.n_subspaces
    recent = int(np.asarray(data["recent_len"], dtype=np.int64).sum()) * w.n_kv_heads * w.head_dim * eb * 2
    codebooks = w.n_kv_heads * 2 * w.n_subspaces * 256 * w.sub_dim * eb
    qo = w.batch * w.n_q_heads * w.head_dim * (eb + 4)
    return {"codes": codes, "recent": recent, "codebooks": codebooks, "q_out": qo,
            "total": codes + recent + codebooks + qo}


def time_other_workload(index, steps, warmup):
    """Decode kernel time (HIP-event span / launches on the launching stream, rotating code copies) of another
    named workload, and for the workload with an append the whole step as well."""
    import numpy as np
    import torch

    from paper_2504_03661_amd.harness import PQSession
    from synth import workloads as W

    w = W.config(index)
    data = W.generate(w)
    scale = W.attention_scale(w)
    bytes_alg = algorithmic_bytes(w, data)
    one_copy = 2 * w.batch * w.n_kv_heads * w.context * w.n_subspaces
    copies = max(2, min(8, -(-(1 << 30) // one_copy)))
    sess = PQSession(data, w.n_q_heads, w.dtype, code_copies=copies)
    dec = [sess.prepared_decode(scale, copy=c) for c in range(copies)]
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    if w.n_new > 0:
        sess.ctx_len.fill_(w.context)          # decode alone: the cache as it is after the append

    def span(fn, n):
        torch.cuda.synchronize()
        ev0.record()
        for i in range(n):
            fn(i)
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / n

    span(lambda i: dec[i % copies](), warmup)
    kernel_ms = span(lambda i: dec[i % copies](), steps)
    out = {"workload": w.name, "n_splits": sess.n_splits, "launches": steps, "kernel_ms": round(kernel_ms, 5),
           "algorithmic_bytes": bytes_alg["total"], "code_bytes": bytes_alg["codes"],
           "achieved_gbps": round(bytes_alg["total"] / (kernel_ms * 1e-3) / 1e9, 1),
           "frac": round(bytes_alg["total"] / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
           "code_read_frac_of_peak": round(bytes_alg["codes"] / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
    tokens = int(np.asarray(data["ctx_len"], dtype=np.int64).sum() + w.n_new * w.batch +
                 np.asarray(data["recent_len"], dtype=np.int64).sum())
    out["context_tokens_per_s"] = round(tokens / (kernel_ms * 1e-3), 1)
    if w.n_new > 0:
        new_k = torch.from_numpy(data["new_k"]).cuda()
        new_v = torch.from_numpy(data["new_v"]).cuda()
        base_len = torch.from_numpy(data["ctx_len"]).cuda()
        app = [sess.prepared_append(new_k, new_v, copy=c) for c in range(copies)]

        def step(i):
            sess.ctx_len.copy_(base_len)
            app[i % copies]()
            dec[i % copies]()

        span(step, max(warmup // 4, 10))
        out["step_ms_append_then_decode"] = round(span(step, steps), 5)
        out["n_new"] = w.n_new
    sess.close()
    del sess, dec, data
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # Defaults: the first 10-20 ms of back-to-back launches after an idle period run about 8 % slower than the
    # steady state (clocks ramping up), so the warm-up is longer than that and the timed region a few times longer.
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=1000)
    ap.add_argument("--config", type=int, default=1, help="workload index 0..4 (default 1: the metric's workload)")
    ap.add_argument("--copies", type=int, default=0, help="distinct code-tensor copies to rotate (0 = 1 GiB worth)")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--warm", action="store_true", help="also time the same-buffer (cache-warm) case")
    ap.add_argument("--no-others", action="store_true", help="skip the other named workloads and the bench_extra.py measurements (only with --config 1 they run)")
    ap.add_argument("--no-next", action="store_true",
                    help="skip only the bench_extra.py measurements")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy a few times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2504_03661_amd import load_library
    from paper_2504_03661_amd.harness import PQSession
    from synth import workloads as W

    load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    if args.calibrate_copy:
        # known traffic: every launch reads 1 GiB and writes 1 GiB
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": {"bytes_read_per_launch": 1 << 30, "bytes_written_per_launch": 1 << 30,
                                             "launches": 10}}))
        return

    w = W.config(args.config)
    data = W.generate(w)
    scale = W.attention_scale(w)
    bytes_alg = algorithmic_bytes(w, data)
    one_copy = 2 * w.batch * w.n_kv_heads * w.context * w.n_subspaces
    copies = args.copies if args.copies > 0 else max(2, min(8, -(-(1 << 30) // one_copy)))

    sess = PQSession(data, w.n_q_heads, w.dtype, n_splits=args.splits, code_copies=copies)
    new_k = new_v = None
    if w.n_new > 0:
        new_k = torch.from_numpy(data["new_k"]).cuda()
        new_v = torch.from_numpy(data["new_v"]).cuda()
        base_len = torch.from_numpy(data["ctx_len"]).cuda()

    dec = [sess.prepared_decode(scale, copy=c) for c in range(copies)]
    app = [sess.prepared_append(new_k, new_v, copy=c) for c in range(copies)] if w.n_new > 0 else None

    def step(i):
        c = i % copies
        if app is not None:
            sess.ctx_len.copy_(base_len)      # the cache holds context - n_new tokens before every step
            app[c]()
        dec[c]()

    # Device pre-warm, not a step of the path: about 40 ms of the library's read-only probe, so that the
    # clocks have left their idle state before the warm-up steps start even when few of those are asked for.
    from paper_2504_03661_amd import pq_stream_read_probe
    prewarm = torch.empty(1 << 28, dtype=torch.uint8, device="cuda").fill_(1)
    t_pre = time.perf_counter()
    while time.perf_counter() - t_pre < 0.04:
        for _ in range(20):
            pq_stream_read_probe(sess.ctx, prewarm, prewarm.numel())
        torch.cuda.synchronize()
    device_prewarm_ms = (time.perf_counter() - t_pre) * 1e3
    del prewarm

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # Exactly K steps, bracketed by synchronize (wall clock) and by one HIP event pair on the
    # launching stream.  With one fused kernel per decode the event span / K is the kernel's
    # average duration including the launch gap between back-to-back kernels.
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    span_ms = ev0.elapsed_time(ev1) / args.steps
    ms_per_step = wall * 1e3 / args.steps

    # The decode kernel alone (for workloads whose step also encodes): the same loop without appends.
    kernel_ms = span_ms
    if app is not None:
        torch.cuda.synchronize()
        ev0.record()
        for i in range(args.steps):
            dec[i % copies]()
        ev1.record()
        torch.cuda.synchronize()
        kernel_ms = ev0.elapsed_time(ev1) / args.steps

    # Same-buffer ("warm") figure, on request: every step reads copy 0, which the 256 MB memory-side
    # cache can hold for the 128 MiB workloads.  For reference only; never used for `value`.  Off by
    # default so that a kernel trace of the default run holds warm-up and timed launches only.
    warm_ms = None
    if args.warm:
        torch.cuda.synchronize()
        ev0.record()
        for i in range(args.steps):
            dec[0]()
        ev1.record()
        torch.cuda.synchronize()
        warm_ms = ev0.elapsed_time(ev1) / args.steps

    # What HBM delivers to a kernel that only reads, on this machine: the library's read probe (same load
    # instruction as the code stream) over a 1 GiB buffer, five passes.
    probe = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(7)
    for _ in range(2):
        pq_stream_read_probe(sess.ctx, probe, probe.numel())
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(5):
        pq_stream_read_probe(sess.ctx, probe, probe.numel())
    ev1.record()
    torch.cuda.synchronize()
    stream_gbps = 5 * probe.numel() / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del probe

    tokens_per_step = int(np.asarray(data["ctx_len"], dtype=np.int64).sum() + w.n_new * w.batch +
                          np.asarray(data["recent_len"], dtype=np.int64).sum())
    value = tokens_per_step / (ms_per_step * 1e-3)

    achieved = bytes_alg["total"] / (kernel_ms * 1e-3) / 1e9
    # HBM bytes per launch from rocprofv3 counters cannot be read inside this process: the figure is the one a
    # separate counter run of this same command left under profiles/ (static; the file names the commands)
    traffic = None
    traffic_source = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{w.name}.txt")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
        traffic_source = f"profiles/traffic_{w.name}.txt (static: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, not measured in this run)"
    kernel_name = {True: "pq_decode_grouped_kernel", False: "pq_decode_kernel"}[w.n_q_heads != w.n_kv_heads and w.dtype == "f16"]
    roofline = {"bound": "hbm", "kernel": kernel_name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "traffic_source": traffic_source,
                "kernel_ms": round(kernel_ms, 5), "event_span_ms_per_step": round(span_ms, 5),
                "measured_stream_read_gbps": round(stream_gbps, 1),
                "frac_of_measured_stream_read": round(achieved / stream_gbps, 4),
                "warm_same_buffer_kernel_ms": None if warm_ms is None else round(warm_ms, 5),
                "algorithmic_bytes": bytes_alg,
                "code_read_gbps": round(bytes_alg["codes"] / (kernel_ms * 1e-3) / 1e9, 1),
                "code_read_frac_of_peak": round(bytes_alg["codes"] / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}

    out_gpu = sess.out.cpu().numpy().astype(np.float64)
    n_splits = sess.n_splits
    sess.close()

    others = None
    if args.config == 1 and not args.no_others:
        others = [time_other_workload(k, steps=n, warmup=wu) for k, n, wu in ((3, 1500, 800), (2, 400, 200), (4, 200, 100))]

    next_rows = None
    if args.config == 1 and not args.no_next and not args.no_others:
        import bench_extra
        next_rows = {}
        for name, fn in (("prefill_encode", bench_extra.prefill), ("pq12", bench_extra.pq12),
                         ("kmeans_train", bench_extra.train), ("async_encode", bench_extra.async_encode)):
            t = time.perf_counter()
            next_rows[name] = fn()
            next_rows[name]["wall_s"] = round(time.perf_counter() - t, 1)
            torch.cuda.empty_cache()

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import pq_oracle
        # bounded sample: at most 64 (sequence, head) rows of the same workload
        rng = np.random.default_rng(0)
        all_pairs = [(b, h) for b in range(w.batch) for h in range(w.n_q_heads)]
        pairs = all_pairs if len(all_pairs) <= 64 else [all_pairs[i] for i in rng.choice(len(all_pairs), 64, False)]
        ctx_len = np.asarray(data["ctx_len"]) if w.n_new == 0 else np.asarray(data["ctx_len"])
        # repeat until about one second of wall time (ten or more core-seconds) has been spent
        best = None
        ref = None
        reps = 0
        spent = 0.0
        while reps < 3 or (spent < 1.0 and reps < 50):
            t = time.perf_counter()
            ref = pq_oracle.decode(data["q"], data["k_codes"], data["v_codes"], ctx_len, data["k_codebook"],
                                   data["v_codebook"], data["recent_k"], data["recent_v"], data["recent_len"],
                                   scale=scale, pairs=pairs)
            dt = time.perf_counter() - t
            best = dt if best is None else min(best, dt)
            spent += dt
            reps += 1
        # the same oracle on one thread, two rows
        threads = pq_oracle.num_threads()
        pq_oracle.set_num_threads(1)
        t = time.perf_counter()
        pq_oracle.decode(data["q"], data["k_codes"], data["v_codes"], ctx_len, data["k_codebook"], data["v_codebook"],
                         data["recent_k"], data["recent_v"], data["recent_len"], scale=scale, pairs=all_pairs[:2])
        one_thread = time.perf_counter() - t
        pq_oracle.set_num_threads(threads)
        frac_rows = len(pairs) / len(all_pairs)
        cpu_tokens = tokens_per_step * frac_rows
        cpu = {"value": round(cpu_tokens / best, 1), "unit": "context tokens/s", "cores": pq_oracle.num_threads(),
               "kind": "oracle", "seconds": round(best, 4),
               "value_one_thread": round(tokens_per_step * min(2, len(all_pairs)) / len(all_pairs) / one_thread, 1),
               "sample": f"{len(pairs)} of {len(all_pairs)} (sequence, head) rows of {w.name}, best of {reps}; "
                         "tokens counted pro rata"}
        if w.n_new == 0:
            sel = np.array(pairs)
            err = float(np.abs(out_gpu[sel[:, 0], sel[:, 1]] - ref[sel[:, 0], sel[:, 1]]).max())
            cpu["max_abs_err_vs_gpu"] = err

    line = {
        "metric": "context tokens scanned/sec & HBM GB/s (% peak), PQ decode attn @32K, 1 GPU",
        "value": round(value, 1), "unit": "context tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "device_prewarm_ms": round(device_prewarm_ms, 1), "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "context": w.context, "pq": f"M={w.n_subspaces} x ds={w.sub_dim} x 256",
                   "io_dtype": w.dtype, "recent_cap": w.recent_cap, "n_new": w.n_new, "n_splits": n_splits,
                   "code_copies_rotated": copies, "seed": w.seed},
        "roofline": roofline,
        "other_workloads": others,
        "next_rows": next_rows,
        "cpu_baseline": cpu,
        "paper_context": "MILLION reports 2.09x end-to-end and 2.01x attention speed-up at 32K on one A40 "
                         "(Llama-2-7B, TPOT 63.41 ms vs 132.97 ms); no kernel-level figure is published",
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
