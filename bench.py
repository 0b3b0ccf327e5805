#!/usr/bin/env python3
"""Benchmark of the verify step on one MI355X.

A step is one aurora_verify call (chunk attention, LM head + softmax statistics, acceptance)
over one batch of synthetic input that is already resident in HBM.  The default workload is the
Llama-3-8B-shaped chain verify (batch 32, k = 4, contexts 1024..4096, paged KV, vocab 128256).
Prints ONE JSON line: verified draft tokens/s, the roofline of the dominant kernel (the LM-head
vocabulary sweep) from HIP-event timing, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {4: 157.3, 2: 2500.0, 1: 5000.0}  # dense, by bytes per operand element (fp32 vector, bf16, fp8), published

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on `bench.py --stage <stage> --workload <name>`
# (seed 1), scaled by what the same counters read for `--stage copy` (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0).  Each entry
# names the file under profiles/ that holds the counters it was computed from (attention = sweep kernel + combine).
# Constants of an earlier profiling run, not measured live: None for workloads and seeds that were not profiled.
MEASURED_TRAFFIC = {
    ("llama", 1, "lmhead"): {"read_bytes": 1061782509, "write_bytes": 92701395,
        "source": "profiles/lmhead_counters_llama3_8b_chain_k4.txt"},
    ("llama", 1, "attn"): {"read_bytes": 314706187 + 8241253, "write_bytes": 7954598 + 1310720,
        "source": "profiles/attn_counters_llama3_8b_chain_k4.txt"},
    ("qwen_greedy", 1, "lmhead"): {"read_bytes": 1582910131, "write_bytes": 306656812,
        "source": "profiles/lmhead_counters_qwen3_8b_greedy_k6.txt"},
    ("qwen_greedy", 1, "attn"): {"read_bytes": 1167539001 + 15271195, "write_bytes": 14873830 + 3670016,
        "source": "profiles/attn_counters_qwen3_8b_greedy_k6.txt"},
    ("tree", 1, "lmhead"): {"read_bytes": 1185215020, "write_bytes": 296291315,
        "source": "profiles/lmhead_counters_llama3_8b_tree32.txt"},
    ("tree", 1, "attn"): {"read_bytes": 277109115 + 34725227, "write_bytes": 34078816 + 4194304,
        "source": "profiles/attn_counters_llama3_8b_tree32.txt"},
    ("stress", 1, "lmhead"): {"read_bytes": 9448627009, "write_bytes": 1161910137,
        "source": "profiles/lmhead_counters_stress_b256.txt"},
    ("stress", 1, "attn"): {"read_bytes": 8113377592 + 42115614, "write_bytes": 40029894 + 15728640,
        "source": "profiles/attn_counters_stress_b256.txt"},
}


def make_workload(name, seed):
    import gen
    if name == "llama":
        return gen.llama_chain(seed)
    if name == "llama_fp8head":
        return gen.llama_chain(seed, head_fp8=True)
    if name == "llama_fp8kv":
        return gen.llama_chain(seed, kv_fp8=True)
    if name == "llama_fp8":
        return gen.llama_chain(seed, kv_fp8=True, head_fp8=True)
    if name == "llama_draft32k":
        return gen.llama_chain(seed, draft_vocab=32000, draft_noise=0.5)
    if name == "llama_k10":
        return gen.llama_chain(seed, num_q=11)   # lookahead 10 (paper section 5, the discard-token experiment)
    if name == "tiny":
        return gen.tiny_chain(seed)
    if name == "qwen_greedy":
        return gen.qwen_greedy_chain(seed)
    if name == "tree":
        return gen.llama_tree(seed)
    if name == "tree_fp8kv":
        return gen.llama_tree(seed, kv_fp8=True)
    if name == "tree_fp8":
        return gen.llama_tree(seed, kv_fp8=True, head_fp8=True)
    if name == "stress":
        import torch
        pool_bytes = int(0.40 * torch.cuda.get_device_properties(0).total_memory)
        return gen.stress_chain(seed, pool_pages=pool_bytes // (2 * 8 * 16 * 128 * 2))
    raise SystemExit(f"unknown workload {name}")


def event_time_ms(fn, iters, torch):
    """Average duration of fn() over `iters` back-to-back launches, by HIP events on the launch stream."""
    st = torch.cuda.current_stream()
    fn()  # untimed: the first call of a stage may set up its buffers
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for _ in range(iters):
        fn()
    e1.record(st)
    e1.synchronize()
    return e0.elapsed_time(e1) / iters


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="llama", choices=["llama", "llama_fp8head", "llama_fp8kv", "llama_fp8", "llama_draft32k", "llama_k10", "tiny", "qwen_greedy", "tree", "tree_fp8kv", "tree_fp8", "stress"])
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--cpu-sample", type=int, default=32, help="requests given to the CPU oracle (0 = skip)")
    ap.add_argument("--steps-only", action="store_true",
                    help="skip the back-to-back stage timings: every kernel launch of the run then belongs to a step "
                         "sequence (for kernel traces whose averages should be the in-step durations)")
    ap.add_argument("--stage", default=None, choices=["attn", "lmhead", "accept", "verify", "trace", "copy", "loss", "attn_bwd",
                                                      "vendor_gemm", "ceiling"],
                    help="profiling aid: launch only this stage --steps times (after --warmup) and exit; "
                         "'copy' runs a plain device-to-device copy of 1 GiB for counter calibration; 'vendor_gemm' times "
                         "the vendor GEMM library (torch.matmul, bf16, product only) on the workload's LM-head shape and "
                         "on a large square, as a reference for what dense bf16 contraction reaches on this box; "
                         "'ceiling' runs the library's calibration probe (matrix cores alone, + operand reads from LDS, "
                         "+ LDS-direct loads from L2, loads alone) on random and on zero operands")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on exactly one GPU (--gpus 1); multi-GPU sharding of the "
                         "verify step is a design note in the repository's documentation, not built")

    import numpy as np
    import torch
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (no CPU fallback exists)")
    import paper_2602_06932_amd as av
    from paper_2602_06932_amd.device import DeviceVerify
    av.load()

    if args.stage == "ceiling":
        # what a dense bf16 contraction reaches on this device, part by part, and how much the values matter
        g = torch.Generator(device="cuda").manual_seed(args.seed)
        rows = torch.randn((4, 512, 4096), device="cuda", generator=g)
        rows[:, :256] *= 0.02                      # the first 256 rows of a tile stand for LM-head rows, the rest for tokens
        data = {"random (LM-head-like values)": rows.to(torch.bfloat16).contiguous(), "zeros": torch.zeros((4, 512, 4096), dtype=torch.bfloat16, device="cuda")}
        sink = torch.zeros(1, device="cuda")
        wgs, stages = 1024, 96
        names = ["matrix cores only", "+ operand reads from LDS", "+ LDS-direct loads from L2", "LDS-direct loads alone"]
        res = []
        for dname, buf in data.items():
            for mode in range(4):
                fn = lambda: av.aurora_probe_contraction(mode, buf, wgs, stages, sink)
                for _ in range(args.warmup):
                    fn()
                torch.cuda.synchronize()
                ms = event_time_ms(fn, args.steps, torch)
                flops = 0.0 if mode == 3 else 2.0 * wgs * stages * 256 * 256 * 64
                loaded = wgs * stages * 65536.0 if mode >= 2 else 0.0
                res.append({"operands": dname, "mode": names[mode], "avg_ms": ms, "TFLOPs": flops / (ms * 1e-3) / 1e12,
                            "TBps_into_LDS": loaded / (ms * 1e-3) / 1e12})
        # the vocabulary sweep alone: 1 GiB streamed once from HBM in the LM head's tile shape
        big = torch.empty((1 << 30) // 2, dtype=torch.bfloat16, device="cuda").normal_(0, 0.02, generator=g)
        fn = lambda: av.aurora_probe_contraction(4, big, 1, 1, sink)
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        ms = event_time_ms(fn, args.steps, torch)
        res.append({"operands": "1 GiB", "mode": "vocabulary sweep alone (HBM -> LDS, LM-head tile shape)", "avg_ms": ms,
                    "TFLOPs": 0.0, "TBps_into_LDS": (1 << 30) / (ms * 1e-3) / 1e12})
        print(json.dumps({"stage": "ceiling", "workgroups": wgs, "stages": stages, "results": res}))
        return

    if args.stage == "loss":
        # the training side's first kernel on a batch of trace rows: 32K-entry draft vocabulary, 1024 kept target
        # logits per row (paper appendix A.2), 4096 rows - 25 verify steps of the headline configuration
        import gen
        rows, vd, k = 4096, 32000, 1024
        z, ids, bits, traj = gen.loss_inputs(args.seed, rows, vd, top_k=k)
        d = av.aurora_loss_desc(rows=rows, draft_vocab=vd, top_k=k, discard_top_k=64, lambda_discard=0.5)
        dz, di = torch.from_numpy(z).cuda(), torch.from_numpy(ids).cuda()
        db, dt = torch.from_numpy(bits.view(np.int16)).cuda(), torch.from_numpy(traj).cuda()
        row_kl, loss = torch.empty(rows, device="cuda"), torch.empty(5, device="cuda")
        grad = torch.empty((rows, vd), device="cuda")
        fn = lambda: av.aurora_draft_loss(d, dz, di, db, dt, row_kl, loss, grad)
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        ms = event_time_ms(fn, args.steps, torch)
        alg = rows * vd * 4 * 2 + rows * k * 6
        print(json.dumps({"stage": "loss", "steps": args.steps, "avg_ms": ms, "rows": rows, "draft_vocab": vd, "top_k": k,
                          "loss": float(loss[0].item()), "algorithmic_bytes": alg,
                          "roofline": {"bound": "hbm", "achieved": alg / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                                       "unit": "GB/s", "frac": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}}))
        return

    t0 = time.time()
    w = make_workload(args.workload, args.seed)
    gen_s = time.time() - t0
    dv = DeviceVerify(w)
    torch.cuda.synchronize()

    if args.stage == "attn_bwd":
        # training-side backward of the chunk / tree attention of this workload (forward included in the call)
        dout = torch.randn(dv.q.shape, device="cuda").to(dv.q.dtype)
        dq = torch.empty(dv.q.shape, dtype=torch.float32, device="cuda")
        dk = torch.zeros(dv.k_pages.shape, dtype=torch.float32, device="cuda")
        dvp = torch.zeros(dv.v_pages.shape, dtype=torch.float32, device="cuda")
        wsb = torch.empty(av.aurora_attn_backward_workspace_bytes(dv.attn_desc), dtype=torch.uint8, device="cuda")
        fn = lambda: av.aurora_attn_backward(dv.attn_desc, dv.q, dv.k_pages, dv.v_pages, dv.block_table, dv.seq_lens,
                                             dv.parents, dout, dq, dk, dvp, wsb)
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        ms = event_time_ms(fn, args.steps, torch)
        ms_fwd = event_time_ms(dv.attn, args.steps, torch)
        # the same backward on an output and logsumexp kept from aurora_attn_forward (no recomputation)
        out_s = torch.empty_like(dv.q)
        lse_s = torch.empty(dv.q.shape[:3], dtype=torch.float32, device="cuda")
        av.aurora_attn_forward(dv.attn_desc, dv.q, dv.k_pages, dv.v_pages, dv.block_table, dv.seq_lens, dv.parents,
                               out_s, lse_s, wsb)
        fn_saved = lambda: av.aurora_attn_backward_saved(dv.attn_desc, dv.q, dv.k_pages, dv.v_pages, dv.block_table,
                                                         dv.seq_lens, dv.parents, out_s, lse_s, dout, dq, dk, dvp, wsb)
        fn_saved()
        ms_saved = event_time_ms(fn_saved, args.steps, torch)
        tok = int(w.seq_lens.astype(np.int64).sum())
        esz = 2 if w.dtype == "bf16" else 4
        kv_elems = tok * w.num_kv_heads * w.head_dim
        alg = 2 * kv_elems * esz * 2 + 2 * kv_elems * 4    # K, V read by the forward and by the backward; dK, dV written
        rows = w.num_q * w.num_q_heads // w.num_kv_heads
        flops = 2.0 * rows * w.head_dim * tok * w.num_kv_heads * (2 + 5)
        print(json.dumps({"stage": "attn_bwd", "steps": args.steps, "avg_ms": ms, "forward_alone_ms": ms_fwd,
                          "backward_from_saved_ms": ms_saved,
                          "workload": w.name, "algorithmic_bytes": alg, "flops": flops,
                          "roofline": {"bound": "hbm", "achieved": alg / (ms * 1e-3) / 1e9, "peak": 8000.0,
                                       "unit": "GB/s", "frac": alg / (ms * 1e-3) / 1e9 / 8000.0,
                                       "note": "whole call (forward, delta, backward, dq merge); bf16 matrix-core kernels "
                                               "when the shape allows, fp32 gradients written once"},
                          "mfma_TFLOPs": flops / (ms * 1e-3) / 1e12,
                          "hbm_GBps": alg / (ms * 1e-3) / 1e9}))
        return

    if args.stage == "vendor_gemm":
        res = []
        for (m, n, k) in [(w.batch * w.num_q, w.vocab, w.hidden_size), (8192, 8192, 8192)]:
            a_ = torch.randn(m, k, device="cuda").to(torch.bfloat16)
            b_ = (torch.randn(n, k, device="cuda") * 0.02).to(torch.bfloat16)
            fn = lambda: torch.matmul(a_, b_.T)
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            ms = event_time_ms(fn, args.steps, torch)
            res.append({"M": m, "N": n, "K": k, "avg_ms": ms, "TFLOPs": 2.0 * m * n * k / (ms * 1e-3) / 1e12})
            del a_, b_
        print(json.dumps({"stage": "vendor_gemm", "workload": w.name, "dtype": "bf16 in, bf16 out", "results": res}))
        return

    if args.stage:
        if args.stage == "copy":
            src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
            dst = torch.empty_like(src)
            fn = lambda: dst.copy_(src)
        else:
            if args.stage == "trace":
                dv.verify()  # the emission reads the logits and acceptance outputs of a verify step
            fn = getattr(dv, args.stage)
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        ms = event_time_ms(fn, args.steps, torch)
        print(json.dumps({"stage": args.stage, "steps": args.steps, "avg_ms": ms, "workload": w.name}))
        return

    # ---- per-stage HIP-event timing (back-to-back launches of one stage, same stream) ----------------
    # Done first: it also brings the GPU out of its idle clocks before the timed region.
    it = 20
    dv.verify()
    torch.cuda.synchronize()
    ms_attn_b2b = ms_lmhead_b2b = ms_accept_half = ms_verify_ev = ms_trace = ms_step_emit = None
    if not args.steps_only:
        ms_attn_b2b = event_time_ms(dv.attn, it, torch)
        ms_lmhead_b2b = event_time_ms(dv.lmhead, it, torch)
        ms_accept_half = event_time_ms(dv.accept, it, torch)
        ms_verify_ev = event_time_ms(dv.verify, it, torch)
        ms_trace = event_time_ms(dv.trace, it, torch)  # not part of a step: the emission that follows a verify
        # ... and as it runs in serving, once after every step (the logits are then cold): step + emission, minus the step
        def step_and_emit():
            dv.verify()
            dv.trace()
        ms_step_emit = event_time_ms(step_and_emit, it, torch)

    # ---- timed region: K whole verify steps (one aurora_verify call each) ---------------------------
    for _ in range(args.warmup):
        dv.verify()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        dv.verify()
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t0
    ms_step = 1e3 * t_total / args.steps
    res = dv.results_host()
    draft_tokens = w.batch * (w.num_q - 1)
    emitted = int(res["accept_len"].sum()) + w.batch

    # ---- the same K steps once more with a HIP event pair on the launch stream around every step: the median of
    # the stream-timed steps (what the measurement plan asks for) beside the host-wall mean above -------------
    st = torch.cuda.current_stream()
    sev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    for e in sev:
        e[0].record(st)
        dv.verify()
        e[1].record(st)
    torch.cuda.synchronize()
    per_step = sorted(e[0].elapsed_time(e[1]) for e in sev)
    ms_step_median = per_step[len(per_step) // 2]

    # ---- the same K steps again as three calls (attention, LM head, acceptance on its logits: the very
    # kernels aurora_verify enqueues, in its order) with HIP events on the launch stream around the
    # attention and LM-head stages of every step: the kernels' durations inside the step sequence --------
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e in ev:
        e[0].record(st)
        dv.attn()
        e[1].record(st)
        dv.lmhead()
        e[2].record(st)
        dv.accept_logits()
    torch.cuda.synchronize()
    ms_step_split = 1e3 * (time.perf_counter() - t0) / args.steps
    ms_attn = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps
    ms_lmhead = sum(e[1].elapsed_time(e[2]) for e in ev) / args.steps
    res2 = dv.results_host()
    assert all(np.array_equal(res[k], res2[k]) for k in ("accept_len", "next_token", "accept_mask"))

    esz = 2 if w.dtype == "bf16" else 4
    hsz = 1 if getattr(w, "head_dtype", "") == "fp8" else esz  # bytes per LM-head operand element
    w_bytes = w.vocab * w.hidden_size * hsz + w.batch * w.num_q * w.hidden_size * hsz
    ksz = 1 if getattr(w, "kv_dtype", "") == "fp8" else esz    # bytes per cached K / V element
    kv_bytes = int(w.seq_lens.astype(np.int64).sum()) * 2 * w.num_kv_heads * w.head_dim * ksz
    lm_gbs = w_bytes / (ms_lmhead * 1e-3) / 1e9
    kv_gbs = kv_bytes / (ms_attn * 1e-3) / 1e9
    lm_flops = 2.0 * w.batch * w.num_q * w.hidden_size * w.vocab

    tr_lm = MEASURED_TRAFFIC.get((args.workload, args.seed, "lmhead"))
    # The LM head streams W once per 160 (small kernel) or per 256 rows: with few rows it is bound by that sweep, with many
    # by the matrix cores.  The bound reported is the one the shape puts nearer: flop per algorithmic byte against
    # the ratio of the two peaks (2.5e15 / 8e12 = 312 flop per byte).
    lm_tflops = lm_flops / (ms_lmhead * 1e-3) / 1e12
    lm_roof = {"kernel": "lmhead (LM-head GEMM + softmax statistics)"}
    if lm_flops / w_bytes > MFMA_PEAK_TFLOPS[hsz] * 1e12 / (HBM_PEAK_GBS * 1e9):
        lm_roof.update({"bound": "mfma", "achieved": lm_tflops, "peak": MFMA_PEAK_TFLOPS[hsz], "unit": "TFLOP/s",
                        "frac": lm_tflops / MFMA_PEAK_TFLOPS[hsz], "hbm_GBs": lm_gbs})
    else:
        lm_roof.update({"bound": "hbm", "achieved": lm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": lm_gbs / HBM_PEAK_GBS, "mfma_tflops": lm_tflops})
    lm_roof.update({"traffic": (tr_lm["read_bytes"] + tr_lm["write_bytes"]) if tr_lm else None,
                    "traffic_detail": tr_lm, "algorithmic_bytes": w_bytes, "flops": lm_flops})
    tr_at = MEASURED_TRAFFIC.get((args.workload, args.seed, "attn"))
    out = {
        "metric": "verified draft tokens/sec on 1 GPU (Llama-3-8B shape, k=4)" if args.workload == "llama"
                  else f"verified draft tokens/sec on 1 GPU ({w.name})",
        "value": draft_tokens / (ms_step * 1e-3),
        "unit": "draft tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "ms_per_step_median_stream_timed": ms_step_median,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype + ("" if ksz == esz else ", KV cache fp8 (e4m3, per-head scales)")
                 + ("" if hsz == esz else ", LM head fp8 (e4m3, per-row scales)"),
        "data": "synthetic",
        "config": {"workload": w.recipe, "name": w.name, "batch": w.batch, "k": w.num_q - 1,
                   "context": [int(w.seq_lens.min()), int(w.seq_lens.max())], "page_size": w.page_size,
                   "heads": [w.num_q_heads, w.num_kv_heads, w.head_dim], "hidden": w.hidden_size,
                   "vocab": w.vocab, "temperature": w.temperature, "seed": w.seed},
        "emitted_tokens_per_s": emitted / (ms_step * 1e-3),
        "mean_accept_len": float(res["accept_len"].mean()),
        "stage_ms": {"attn_in_step": ms_attn, "lmhead_in_step": ms_lmhead, "step_as_three_calls": ms_step_split,
                     "attn_back_to_back": ms_attn_b2b, "lmhead_back_to_back": ms_lmhead_b2b,
                     "accept_half(lmhead+walk)": ms_accept_half, "verify_by_events": ms_verify_ev,
                     "trace_emit_after_verify(top-1024)": ms_trace,
                     "verify_step_plus_trace_emit": ms_step_emit},
        "roofline": lm_roof,
        "roofline_attn": {"kernel": "chunk attention (KV sweep)", "bound": "hbm", "achieved": kv_gbs,
                          "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kv_gbs / HBM_PEAK_GBS,
                          "traffic": (tr_at["read_bytes"] + tr_at["write_bytes"]) if tr_at else None,
                          "traffic_detail": tr_at, "algorithmic_bytes": kv_bytes},
        "host_generation_s": gen_s,
    }

    # ---- CPU oracle on a bounded sample of the same workload ---------------------------------------
    if args.cpu_sample > 0:
        import oracle
        n = min(args.cpu_sample, w.batch)
        ws = w.take_requests(np.arange(n))
        t0 = time.perf_counter()
        oracle.verify(ws)
        t_cpu = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": n * (w.num_q - 1) / t_cpu, "unit": "draft tokens/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"first {n} of {w.batch} requests of the same workload, "
                                         f"attention + LM head + acceptance, {t_cpu:.1f} s wall"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
