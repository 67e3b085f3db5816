#!/usr/bin/env python3
"""Measurements beyond the headline benchmark (one MI355X):

    python bench_extra.py prefill   # bulk encode of a 32K-token prompt, all heads, K and V
    python bench_extra.py async     # encode on a second stream while decode runs
    python bench_extra.py train     # offline codebook training (k-means), 64K samples x 32 heads
    python bench_extra.py pq12 [shape]  # 12-bit codes: decode at 1 x 32 heads x 32K, 8 x 32 x 32K, 32 query / 8 KV heads x
                                    # 128K and 8 x 32q/8kv x 32K (or the one shape named), 64-token append
    python bench_extra.py ctx       # decode time against context length (1K .. 128K), 32 heads and 32 query / 8 KV heads
    python bench_extra.py step1     # one decoding step of one sequence: one-token append + decode, 8-bit and 12-bit
    python bench_extra.py batch     # many short sequences: 8 x 32K .. 256 x 1K tokens (32 heads, 128 recent rows), decode and
                                    # the one-token-per-sequence append

prefill: the nearest-centroid encode at prompt shape (Section III-A, "Online Prefill with KV Cache
Quantization"): vectors per second against the vector-ALU roofline (256 CUs x 64 lanes x 2.4 GHz = 39.3 T
operations/s) at the instruction count of the fp16 filter kernel, and the time the plain fp64 scan (2 ds + 3
operations per (sub-vector, centroid)) would need at that peak.

async: Section III-B's asynchronous quantization with what this pool allows — two streams of DEFAULT
priority.  Decode reads the visible lengths, encode appends behind them using a second length array, so the
two kernels touch disjoint data; the caller publishes the new lengths between steps.

train: Lloyd iterations of the per-subspace k-means (Section III-A, "Offline PQ Codebook Training") on 65 536
sampled vectors per head, 32 heads, M = 64: time per iteration against the vector-ALU roofline at the instruction
count of the assignment (the encode's matrix-core filter), and the time the plain fp64 scan would need at that peak.

pq12: the 12-bit setting (M = 32, 4096 centroids, 48 bytes per token and tensor; Section IV-A).  Decode
against HBM: algorithmic bytes = codes + recent rows + both codebooks once per KV head (2 MiB per head: at 32K
tokens they are 40 % of the bytes) + q / out.  With few (sequence, head) pairs the decode runs in two passes
(partial scores per subspace group, then softmax and values): "n_passes" in the output.
ctx: decode kernel time against context length, 1K .. 128K tokens (and short sequences in a 128K-capacity cache), for 1 x 32 heads (one query head per KV head) and for
32 query / 8 KV heads (the grouped-query kernel); split counts as the library chooses them.

step1: one decoding step of a single sequence, 32 heads at 32K tokens: append of one token per head, then decode, for
8-bit codes (M = 64) and 12-bit codes (M = 32, 4096 centroids).
batch: the same number of cached tokens as 8 sequences x 32K, cut into more and shorter sequences (a serving batch):
decode time against the bytes the method must move (codes, the recent rows — a large share at 1K tokens — codebooks,
q / out), and the append of one new token per sequence.
Each mode prints one JSON line.
"""
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

ALU_LANE_OPS_PER_S = 256 * 64 * 2.4e9


def _span_ms(fn, steps, warmup=3):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def prefill():
    import numpy as np
    import torch
    from paper_2504_03661_amd.harness import PQSession
    from synth import workloads as W

    n_new = 32768
    w = W.Workload("prefill_encode_32k", 1, 32, 32, 128, 64, n_new, "f16", n_new=n_new, seed=W.BASE_SEED + 11)
    data = W.generate(w)
    with PQSession(data, w.n_q_heads, w.dtype) as s:
        nk = torch.from_numpy(data["new_k"]).cuda()
        nv = torch.from_numpy(data["new_v"]).cuda()
        app = s.prepared_append(nk, nv)

        def step():
            s.ctx_len.zero_()
            app()
        ms = _span_ms(step, 5)
    vectors = 2 * w.batch * w.n_kv_heads * n_new
    # vector instructions the fp16 filter kernel issues per (token, subspace), matrix instructions not counted: 2 + 3
    # per group of 4 centroids in its two passes, about 180 for token set-up, the fp64 evaluation of 4 to 8 candidates
    # and the store (rocprofv3 SQ_INSTS_VALU - SQ_INSTS_MFMA: 499); 2 matrix instructions per group of 4
    ops_per_subvector = 256 * 1.25 + 180
    mfma_per_subvector = 2 * 64 * (w.sub_dim // 2)
    ops = vectors * w.n_subspaces * ops_per_subvector
    achieved = ops / (ms * 1e-3)
    scan_ops = vectors * w.n_subspaces * 256 * (2 * w.sub_dim + 3)
    return ({"mode": "prefill_encode", "workload": w.name, "ms": round(ms, 3),
                      "vectors_per_s": round(vectors / (ms * 1e-3)), "tokens_per_s": round(n_new / (ms * 1e-3)),
                      "roofline": {"bound": "alu", "unit": "lane-op/s", "achieved": achieved,
                                   "peak": ALU_LANE_OPS_PER_S, "frac": round(achieved / ALU_LANE_OPS_PER_S, 4),
                                   "ops_per_subvector": ops_per_subvector},
                      # a SIMD issues a 64-lane vector instruction in 4 cycles and a 4x4x4 matrix instruction in 8
                      "ms_at_the_issue_limit": round(vectors * w.n_subspaces / 64 * (4 * ops_per_subvector + 8 * mfma_per_subvector)
                                                     / (1024 * 2.4e9) * 1e3, 3),
                      "ms_of_the_fp64_scan_at_alu_peak": round(scan_ops / ALU_LANE_OPS_PER_S * 1e3, 3)})


def async_encode():
    import numpy as np
    import torch
    from paper_2504_03661_amd import binding as B
    from paper_2504_03661_amd.harness import PQSession
    from synth import workloads as W

    w = W.config(4)
    data = W.generate(w)
    scale = W.attention_scale(w)
    with PQSession(data, w.n_q_heads, w.dtype) as s:
        nk = torch.from_numpy(data["new_k"]).cuda()
        nv = torch.from_numpy(data["new_v"]).cuda()
        visible = s.ctx_len                                  # decode reads these lengths
        pending = visible.clone()                            # encode appends behind them
        side = torch.cuda.Stream()                           # default priority
        main = torch.cuda.current_stream()

        def decode_only():
            B.pq_attn_decode(s.ctx, s.q, s.k_codes[0], s.v_codes[0], visible, None, None, None, None, None, scale,
                             s.out, main)

        def encode_only():
            pending.copy_(visible)
            B.pq_encode_append(s.ctx, nk, nv, w.n_new, None, None, s.k_codes[0], s.v_codes[0], pending, main)

        def overlapped():
            # decode is submitted first: its workgroups take most of every CU's LDS, the encode
            # workgroups (one wavefront, a few KiB of LDS) then fit beside them
            side.wait_stream(main)
            decode_only()
            with torch.cuda.stream(side):
                pending.copy_(visible)
                B.pq_encode_append(s.ctx, nk, nv, w.n_new, None, None, s.k_codes[0], s.v_codes[0], pending, side)
            main.wait_stream(side)

        steps = 50
        t_dec = _span_ms(decode_only, steps, warmup=50)   # warm-ups pass the clock ramp after an idle period
        t_enc = _span_ms(encode_only, steps, warmup=50)
        t_both = _span_ms(overlapped, steps, warmup=50)
    return ({"mode": "async_encode", "workload": w.name, "decode_ms": round(t_dec, 4),
                      "encode_ms": round(t_enc, 4), "serial_ms": round(t_dec + t_enc, 4),
                      "overlapped_ms": round(t_both, 4),
                      "hidden_fraction_of_encode": round((t_dec + t_enc - t_both) / t_enc, 3),
                      "streams": "two streams of default priority"})


def train():
    import numpy as np
    import torch
    from paper_2504_03661_amd import binding as B
    from synth import workloads as W

    Hkv, M, n, iters = 32, 64, 65536, 5
    d = W.training_samples(Hkv, n, 128, M, seed=5)
    cfg = B.PQAttnConfig(batch=1, n_q_heads=Hkv, n_kv_heads=Hkv, head_dim=128, n_subspaces=M, n_centroids=256,
                         max_context=64, max_recent=0, dtype=B.PQ_F16, device=0, n_splits=0)
    ctx = B.pq_attn_create(cfg)
    x = torch.from_numpy(d["samples"]).cuda()
    init = torch.from_numpy(d["init"]).cuda()
    cb = init.clone()
    nbytes = B.pq_kmeans_workspace_bytes(ctx)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")

    def run():
        cb.copy_(init)
        B.pq_kmeans_fit(ctx, x, n, cb, iters, ws, nbytes)

    ms = _span_ms(run, 3, warmup=1) / iters
    ds = 128 // M
    # vector instructions of the assignment per (sample, subspace): the encode's matrix-core filter (2 + 3 per group
    # of 4 centroids, 4 to 8 candidates in fp64, set-up) and the LDS atomics of the member sums
    ops = Hkv * M * n * (256 * 1.25 + 200)
    scan_ops = Hkv * M * n * 256 * (2 * ds + 3)
    trained = cb.cpu().numpy()
    B.pq_attn_destroy(ctx)

    return ({"mode": "kmeans_train", "workload": f"{Hkv} heads x {n} samples, M={M}, {iters} Lloyd iterations",
                      "ms_per_iteration": round(ms, 3),
                      "sub_vectors_per_s": round(Hkv * M * n / (ms * 1e-3), 1),
                      "alu": {"bound": "alu", "achieved": round(ops / (ms * 1e-3) / 1e12, 2),
                              "peak": round(ALU_LANE_OPS_PER_S / 1e12, 1), "unit": "T vector operations/s",
                              "frac": round(ops / (ms * 1e-3) / ALU_LANE_OPS_PER_S, 4)},
                      "ms_of_the_fp64_scan_at_alu_peak": round(scan_ops / ALU_LANE_OPS_PER_S * 1e3, 3),
                      "trained_codebook_finite": bool(np.isfinite(trained.astype(np.float32)).all())})


def pq12(only=None):
    import numpy as np
    import torch
    from paper_2504_03661_amd.harness import PQSession
    from synth import workloads as W

    res = {"mode": "pq12"}
    # one query head per KV head (the metric's layer shape, one and eight sequences), then grouped queries: 32 query /
    # 8 KV heads at 128K tokens and eight sequences at 32K (the grouped-query kernel)
    for name, Bn, hkv, n in (("1x32x32k", 1, 32, 32768), ("8x32x32k", 8, 32, 32768),
                             ("1x32q8kv_128k", 1, 8, 131072), ("8x32q8kv_32k", 8, 8, 32768)):
        if only is not None and name != only:
            continue
        w = W.Workload("pq12_" + name, Bn, 32, hkv, 128, 32, n, "f16", recent_cap=128, recent_fixed=128,
                       seed=W.BASE_SEED + 12, n_centroids=4096)
        data = W.generate(w)
        one_copy = 2 * Bn * hkv * n * 48
        copies = max(2, min(8, -(-(1 << 30) // one_copy)))
        with PQSession(data, 32, "f16", code_copies=copies) as s:
            dec = [s.prepared_decode(W.attention_scale(w), copy=c) for c in range(copies)]
            it = [0]

            def step():
                dec[it[0] % copies]()
                it[0] += 1
            # warm-up past the clock ramp that follows an idle period (the first 10-20 ms run slower)
            ms = _span_ms(step, 400, warmup=max(100, int(30e-3 / (70e-6 * Bn))))
            n_splits, n_passes, hpw = s.n_splits, s.n_passes, s.heads_per_workgroup
        codes = Bn * hkv * n * 96
        total = codes + Bn * hkv * 128 * 128 * 2 * 2 + hkv * 2 * 32 * 4096 * 4 * 2 + Bn * 32 * 128 * 6
        res[name] = {"decode_ms": round(ms, 4), "n_passes": n_passes, "n_splits": n_splits, "heads_per_workgroup": hpw,
                     "ctx_tokens_per_s": round(Bn * (n + 128) / (ms * 1e-3), 1),
                     "roofline": {"bound": "hbm", "achieved": round(total / (ms * 1e-3) / 1e9, 1), "peak": 8000.0,
                                  "unit": "GB/s", "frac": round(total / (ms * 1e-3) / 1e9 / 8000.0, 4),
                                  "algorithmic_bytes": total, "code_bytes": codes}}
    if only is not None:
        return res
    # append of 64 tokens per head, 16 sequences x 32 heads (the shape of the 8-bit encode workload)
    w = W.Workload("pq12_append", 16, 32, 32, 128, 32, 4096, "f16", n_new=64, seed=W.BASE_SEED + 13, n_centroids=4096)
    data = W.generate(w)
    with PQSession(data, 32, "f16") as s:
        nk, nv = torch.from_numpy(data["new_k"]).cuda(), torch.from_numpy(data["new_v"]).cuda()
        base = s.ctx_len.clone()
        app = s.prepared_append(nk, nv)

        def step2():
            s.ctx_len.copy_(base)
            app()
        ms = _span_ms(step2, 20, warmup=10)
    # vector instructions of the matrix-core filter per (token, subspace), matrix instructions not counted: 2 + 2.25
    # per group of 4 centroids in its two passes, about 1100 for 16-32 candidates evaluated in fp64, set-up and store
    # (rocprofv3 SQ_INSTS_VALU - SQ_INSTS_MFMA: 5470); the plain fp64 scan has 4096 x 11
    pairs = 2 * 16 * 32 * 64 * 32
    ops = pairs * (4096 * 4.25 / 4 + 1100)
    res["append_16x32x64"] = {"ms": round(ms, 4), "vectors_per_s": round(2 * 16 * 32 * 64 / (ms * 1e-3), 1),
                              "alu": {"bound": "alu", "achieved": round(ops / (ms * 1e-3) / 1e12, 2),
                                      "peak": round(ALU_LANE_OPS_PER_S / 1e12, 1), "unit": "T vector operations/s",
                                      "frac": round(ops / (ms * 1e-3) / ALU_LANE_OPS_PER_S, 4)},
                              # 4 cycles of a SIMD per 64-lane vector instruction, 8 per 4x4x4 matrix instruction (4 per group)
                              "ms_at_the_issue_limit": round(pairs / 64 * (4 * (4096 * 4.25 / 4 + 1100) + 8 * 4096) / (1024 * 2.4e9) * 1e3, 3),
                              "ms_of_the_fp64_scan_at_alu_peak": round(pairs * 4096 * 11 / ALU_LANE_OPS_PER_S * 1e3, 3)}
    return res


def ctx():
    import torch
    from paper_2504_03661_amd.harness import PQSession
    from synth import workloads as W

    res = {"mode": "decode_vs_context", "unit": "us per decode"}
    for label, hq, hkv in (("32_heads", 32, 32), ("32q_8kv", 32, 8)):
        rows = {}
        for n in (1024, 2048, 4096, 8192, 16384, 32768, 65536, 131072):
            w = W.Workload("ctx", 1, hq, hkv, 128, 64, n, "f16", recent_cap=128, recent_fixed=128, seed=W.BASE_SEED + 21)
            data = W.generate(w)
            copies = max(2, min(16, -(-(1 << 30) // (2 * hkv * n * 64))))
            with PQSession(data, hq, "f16", code_copies=copies) as s:
                dec = [s.prepared_decode(W.attention_scale(w), copy=c) for c in range(copies)]
                it = [0]

                def step():
                    dec[it[0] % copies]()
                    it[0] += 1
                rows[str(n)] = {"us": round(_span_ms(step, 400, warmup=1500) * 1e3, 2), "n_splits": s.n_splits}
        res[label] = rows
    # a short sequence in a long cache: the grid is sized for the 128K capacity, the live splits follow the length
    for label, hq, hkv in (("32_heads_in_128k_cache", 32, 32), ("32q_8kv_in_128k_cache", 32, 8)):
        w = W.Workload("ctx_cap", 1, hq, hkv, 128, 64, 131072, "f16", recent_cap=128, recent_fixed=128, seed=W.BASE_SEED + 22)
        data = W.generate(w)
        copies = max(2, min(16, -(-(1 << 30) // (2 * hkv * 131072 * 64))))
        rows = {}
        with PQSession(data, hq, "f16", code_copies=copies) as s:
            dec = [s.prepared_decode(W.attention_scale(w), copy=c) for c in range(copies)]
            it = [0]

            def step():
                dec[it[0] % copies]()
                it[0] += 1
            for n in (256, 2048, 16384, 131072):
                s.ctx_len.fill_(n)
                live = min(s.n_splits, max(1, ((n + 63) // 64) // 4, 128 // 16))
                rows[str(n)] = {"us": round(_span_ms(step, 400, warmup=1500) * 1e3, 2), "launched_splits": s.n_splits,
                                "live_splits": live}
        res[label] = rows
    return res


def step1():
    import torch
    from paper_2504_03661_amd.harness import PQSession
    from synth import workloads as W

    res = {"mode": "single_sequence_step", "unit": "us"}
    for label, m, c in (("8bit_M64", 64, 256), ("12bit_M32", 32, 4096)):
        w = W.Workload("step1_" + label, 1, 32, 32, 128, m, 32768, "f16", recent_cap=128, recent_fixed=128, n_new=1,
                       seed=W.BASE_SEED + 22, n_centroids=c)
        data = W.generate(w)
        with PQSession(data, 32, "f16", code_copies=8) as s:
            nk, nv = torch.from_numpy(data["new_k"]).cuda(), torch.from_numpy(data["new_v"]).cuda()
            base = s.ctx_len.clone()
            apps = [s.prepared_append(nk, nv, copy=k) for k in range(8)]
            decs = [s.prepared_decode(W.attention_scale(w), copy=k) for k in range(8)]
            it = [0]

            def reset_only():
                s.ctx_len.copy_(base)

            def append_only():
                s.ctx_len.copy_(base)
                apps[it[0] % 8]()
                it[0] += 1

            def whole():
                s.ctx_len.copy_(base)
                apps[it[0] % 8]()
                decs[it[0] % 8]()
                it[0] += 1
            t_reset = _span_ms(reset_only, 400, warmup=400) * 1e3
            t_app = _span_ms(append_only, 400, warmup=400) * 1e3
            t_all = _span_ms(whole, 400, warmup=800) * 1e3
        res[label] = {"length_reset_copy": round(t_reset, 2), "append_one_token_per_head": round(t_app - t_reset, 2),
                      "append_and_decode": round(t_all - t_reset, 2)}
    return res


def batch():
    import torch
    from paper_2504_03661_amd.harness import PQSession
    from synth import workloads as W

    res = {"mode": "batched_short_sequences", "heads": 32, "recent_rows": 128}
    for Bn, n in ((8, 32768), (32, 8192), (64, 4096), (128, 2048), (256, 1024)):
        w = W.Workload("batch", Bn, 32, 32, 128, 64, n, "f16", recent_cap=128, recent_fixed=128, n_new=1,
                       seed=W.BASE_SEED + 31)
        data = W.generate(w)
        with PQSession(data, 32, "f16", code_copies=2) as s:
            dec = [s.prepared_decode(W.attention_scale(w), copy=c) for c in range(2)]
            nk, nv = torch.from_numpy(data["new_k"]).cuda(), torch.from_numpy(data["new_v"]).cuda()
            base = s.ctx_len.clone()
            app = [s.prepared_append(nk, nv, copy=c) for c in range(2)]
            it = [0]

            def step():
                dec[it[0] % 2]()
                it[0] += 1

            def reset_only():
                s.ctx_len.copy_(base)

            def append_step():
                s.ctx_len.copy_(base)
                app[it[0] % 2]()
                it[0] += 1
            ms = _span_ms(step, 100, warmup=100)
            t_app = (_span_ms(append_step, 100, warmup=50) - _span_ms(reset_only, 100, warmup=50)) * 1e3
        total = Bn * 32 * (n - 1) * 128 + Bn * 32 * 128 * 128 * 2 * 2 + 32 * 2 * 64 * 256 * 2 * 2 + Bn * 32 * 128 * 6
        res[f"{Bn}x{n // 1024}k"] = {"decode_us": round(ms * 1e3, 1), "append_one_token_per_sequence_us": round(t_app, 1),
                                     "algorithmic_bytes": total,
                                     "frac_of_hbm_peak": round(total / (ms * 1e-3) / 1e9 / 8000.0, 4)}
    # ragged batches in a 128K-capacity cache: with 256 (sequence, head) pairs the library chooses one split, and a
    # long sequence is then scanned by one workgroup per head while the compute units of the short ones idle; a
    # caller who expects ragged batches asks for splits (the live splits follow each sequence's length and its share
    # of the batch's tokens, the surplus workgroups leave at once)
    for label, lens in (("one_128k_seven_1k", (131072,) + (1024,) * 7), ("64k_halving_to_512", tuple(65536 >> k for k in range(8))),
                        ("eight_32k", (32768,) * 8)):
        row = {}
        for n_splits in (0, 8):
            w = W.Workload("ragged", 8, 32, 32, 128, 64, 131072, "f16", recent_cap=128, recent_fixed=128,
                           seed=W.BASE_SEED + 51, ctx_lens=lens)
            data = W.generate(w)
            with PQSession(data, 32, "f16", n_splits=n_splits) as s:
                dec = s.prepared_decode(W.attention_scale(w))
                row[f"n_splits_{n_splits}"] = {"splits": s.n_splits, "decode_us": round(_span_ms(dec, 50, warmup=50) * 1e3, 1)}
            del data
        res["ragged_" + label] = row
    return res


if __name__ == "__main__":
    modes = {"batch": batch, "prefill": prefill, "async": async_encode, "train": train, "pq12": pq12, "ctx": ctx, "step1": step1}
    mode = sys.argv[1] if len(sys.argv) > 1 else ""
    if mode not in modes:
        print(__doc__)
        sys.exit(2)
    print(json.dumps(modes[mode](*sys.argv[2:3]) if mode == "pq12" else modes[mode]()))
