#!/usr/bin/env python3
"""Benchmark of the fused generation + inference stage on one MI355X.

One "step" is one whole stage over one synthetic long-tail batch: Actor prefill + decode of
every sample, fused at sample level with the Reference / Critic / Reward scoring forwards
(rlhf_run_stage, fused = 1).  Prints ONE JSON line:

  value      (generated + scored sequence tokens) / stage time, tokens/s, inputs resident in HBM
  roofline   the kernel class with the largest share of GPU time, its algorithmic bytes (or
             flops) per launch over its HIP-event duration, against the MI355X peak
  cpu_baseline  the numpy oracle timed on this machine's host cores on a bounded sample
  plus: fused vs sequential stage time, per-class kernel figures, the long-tail phase lens.

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 7b|gpt2s|tiny|13b|70b_slice]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "fp32": 157.3}
# what the arithmetic actually is: bf16 models keep bf16 weights, feed IEEE-half activations to
# v_mfma_f32_16x16x32_f16 (same peak as bf16) and accumulate in float; the KV cache is half
ARITH = {"bf16": "bf16 weights x f16 activations, f32 accumulate (f16 KV cache)", "fp32": "f32"}
ROLE_MASK_DEFAULT = 0b1110      # Reference, Critic, Reward; Actor log-probs come from decoding

# bounded oracle sample per workload: (samples, output-length cap, oracle dtype)
CPU_SAMPLE = {"tiny": (8, 64, "float64"), "gpt2s": (4, 24, "float64"), "7b": (4, 32, "float32"),
              "13b": (1, 8, "float32"), "70b_slice": (1, 8, "float32")}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_stage(cfg, args):
    import torch

    import paper_2409_13221_amd as R
    from workload import make_weights, make_workload

    m = cfg.model
    t0 = time.time()
    if args.weights == "seeded":
        weights = [make_weights(cfg, r, device="cuda") for r in range(4)]
    else:
        # same distribution from torch's own generator: for runs under a counter-collecting profiler,
        # whose tool aborts in the integer kernels of the counter-based generator
        from workload.generate import weight_shapes
        torch.manual_seed(cfg.seed)
        wdt = torch.float32 if m.dtype == "fp32" else torch.bfloat16
        weights = [{k: (torch.ones(sh, device="cuda") if k.startswith("g_") else
                        torch.empty(sh, device="cuda", dtype=wdt).normal_(0.0, 0.02))
                    for k, sh in weight_shapes(m, r).items()} for r in range(4)]
    torch.cuda.synchronize()
    log(f"[bench] weights for 4 roles on device in {time.time() - t0:.1f}s")
    wl = make_workload(cfg)
    po, out_len = wl["prompt_offsets"], wl["out_len"]
    plen = np.diff(po).astype(np.int32)
    n = len(plen)
    max_new = np.full(n, cfg.length_cap, np.int32)          # reservation is for the cap, as in production
    max_ctx = int(plen.max()) + cfg.length_cap + 1
    page_b = m.n_layers * 2 * m.n_kv_heads * cfg.page_tokens * m.head_dim * m.elem_bytes()
    need_pages = int(np.ceil((plen + max_new) / cfg.page_tokens).sum())
    free_b, total_b = torch.cuda.mem_get_info()
    max_batch_tokens = max(args.max_batch_tokens, max_ctx)
    ws_est = 3 * max_batch_tokens * (12 * m.d_model + 8 * m.ffn + 16 * m.n_q_heads * m.head_dim) + (8 << 30)
    # half copies of the matrices for the prefill / scoring passes (made by rlhf_load_weights, after the pool)
    half_copies = int(args.half_weight_copies and m.dtype == "bf16")
    copies_b = 4 * m.decode_weight_bytes() if half_copies else 0
    pool_pages = int(min(need_pages, max(1, (free_b - ws_est - copies_b) // page_b)))
    mc = R.model_cfg_of(m)
    ec = R.rlhf_engine_cfg(cfg.page_tokens, pool_pages * page_b, n, max_ctx, min(n, args.max_active),
                           max_batch_tokens, cfg.eos_id, 0, args.corun_decode_cus, int(args.admission == "optimistic"), None, None,
                           half_copies)
    ctx = R.rlhf_create(mc, ec)
    for role, w in enumerate(weights):
        R.rlhf_load_weights(ctx, role, w)
    log(f"[bench] {cfg.name}: {n} samples, prompts {plen.min()}..{plen.max()}, outputs mean {out_len.mean():.1f} "
        f"max {out_len.max()}; KV pool {pool_pages} pages ({pool_pages * page_b / 2**30:.1f} GiB) of {need_pages} "
        f"reserved at the cap; HBM free {free_b / 2**30:.0f} of {total_b / 2**30:.0f} GiB")
    return R, ctx, weights, wl, max_new


def run_stage(R, ctx, wl, max_new, fused, args, trace=False):
    R.rlhf_submit(ctx, wl["prompt_tokens"], wl["prompt_offsets"], max_new, wl["out_len"])
    n = len(max_new)
    R_t = args.R_t if args.R_t >= 0 else n + 1
    t0 = time.perf_counter()
    stats, tr = R.rlhf_run_stage(ctx, "auto" if fused == "auto" else bool(fused), R_t, args.score_chunk_tokens, args.role_mask,
                                 trace_cap=(1 << 15) if trace else 0, trace_time=trace)
    return (time.perf_counter() - t0) * 1e3, stats, tr


def cpu_baseline(cfg, weights):
    """The oracle, as it stands, on a bounded sample of the same workload: generation of the
    first few samples (output length capped) and their three scoring forwards."""
    import threadpoolctl

    from oracle import transformer as OT
    from workload import make_workload

    n, cap, dt = CPU_SAMPLE[cfg.name]
    dtype = np.float64 if dt == "float64" else np.float32
    wl = make_workload(cfg, n)
    po = wl["prompt_offsets"]
    prompts = [wl["prompt_tokens"][po[i]:po[i + 1]].tolist() for i in range(n)]
    out_len = np.minimum(wl["out_len"], cap)
    shape = OT.Shape.of(cfg.model)
    elapsed, toks = 0.0, None
    for role in range(4):
        model = OT.Model(shape, {k: v.float().cpu().numpy() for k, v in weights[role].items()}, dtype)
        t0 = time.perf_counter()
        if role == 0:
            gen = OT.greedy_generate_cached(model, prompts, out_len, cfg.eos_id)
            toks = [g.tokens.tolist() for g in gen]
        elif role == 1:
            [OT.score_logprobs(model, p, y) for p, y in zip(prompts, toks)]
        elif role == 2:
            [OT.score_values(model, p, y) for p, y in zip(prompts, toks)]
        else:
            [OT.score_reward(model, p, y) for p, y in zip(prompts, toks)]
        elapsed += time.perf_counter() - t0
        del model
        log(f"[bench] cpu oracle role {role} done, cumulative {elapsed:.1f}s")
    G = int(out_len.sum())
    S = int(sum(len(p) for p in prompts) + G)
    threads = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] or [1])
    return {"value": (G + S) / elapsed, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {n} sample(s) of '{cfg.name}', outputs capped at {cap}: {G} generated + {S} "
                      f"scored tokens in {elapsed:.1f}s, numpy {dt}, full depth"}


CLASS_BOUND = {"gemm_decode": "hbm", "attn_decode": "hbm", "gemm_batch": "mfma", "attn_batch": "mfma"}


def rooflines(prof, dtype, steps):
    """One roofline object per kernel class.  Clock: HIP events on the stream the kernel runs on,
    around every sample_every-th launch of the class over ALL timed stages (rlhf_profile_*); what a
    bracket costs beyond its kernels (launch + signalling latency: twice the median bracket of one
    empty kernel minus that of two, measured on the same stream when profiling starts) is taken off
    each bracket, which is what makes the average comparable with the kernel durations rocprofv3
    reports (within about 2 us either way).  achieved = algorithmic bytes (or flops) of the sampled
    launches / their corrected time."""
    out = {}
    for k, v in prof.items():
        if not v["sampled"]:
            continue
        raw_ms = v["sampled_ms"]
        ms = max(raw_ms - v["sampled"] * v["bracket_overhead_ms"], 1e-9)
        if CLASS_BOUND[k] == "hbm":
            ach, peak, unit = v["sampled_bytes"] / (ms * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            ach, peak, unit = v["sampled_flops"] / (ms * 1e-3) / 1e12, MFMA_PEAK_TFLOPS[dtype], "TFLOP/s"
        avg_us = ms / v["sampled"] * 1e3
        out[k] = {"bound": CLASS_BOUND[k], "kernel": k, "achieved": round(ach, 2), "peak": peak, "unit": unit,
                  "frac": round(ach / peak, 4), "traffic": None,
                  "avg_launch_us": round(avg_us, 2), "avg_bracket_us": round(raw_ms / v["sampled"] * 1e3, 2),
                  "bracket_overhead_us": round(v["bracket_overhead_ms"] * 1e3, 2),
                  "launches_per_stage": int(v["launches"] // steps), "sampled": int(v["sampled"]),
                  "dropped": int(v["dropped"]),
                  "est_ms_per_stage": round(avg_us * v["launches"] / steps / 1e3, 1),
                  "alg_bytes_per_stage": v["total_bytes"] / steps, "alg_flops_per_stage": v["total_flops"] / steps,
                  "GBps": round(v["sampled_bytes"] / (ms * 1e-3) / 1e9, 1),
                  "TFLOPs": round(v["sampled_flops"] / (ms * 1e-3) / 1e12, 2)}
    return out


def micro(args):
    """Kernel-level cases at the 7B layer shapes through the ops ABI, for rocprofv3 counter runs and
    per-kernel timings.  In dispatch order: a 1 GiB device copy (calibrates FETCH_SIZE / WRITE_SIZE);
    the four projections of a scoring pass at M = --micro_rows (half activations, half copies of the
    weights, rotary fused into QKV and SwiGLU into gate||up, as the stage runs them) and the LM head
    fused with the log-softmax gather at M = 2048; the four projections in the decode regime at
    M = 8, 32, 64, 128, 256 (the five tilings of a decode step); paged decode attention (32 samples x
    1024 cached tokens, 32 heads x 128, half).  Each case launches exactly one GEMM / attention /
    copy kernel per call, 1 + --micro_reps calls."""
    import torch

    import paper_2409_13221_amd as R
    torch.cuda.set_device(0)
    dev = "cuda"
    out = []

    def timed(name, fn, bytes_, flops, reps=args.micro_reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        out.append({"case": name, "us": round(us, 1), "GBps": round(bytes_ / us / 1e3, 1),
                    "TFLOPs": round(flops / us / 1e6, 1), "alg_bytes": bytes_, "alg_flops": flops})
        log(f"[micro] {name}: {us:.1f} us, {bytes_ / us / 1e3:.0f} GB/s, {flops / us / 1e6:.0f} TFLOP/s")

    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    timed("copy_1GiB", lambda: dst.copy_(src), 2.0 * src.numel() * 4, 0)
    del src, dst
    shapes = [("qkv", 12288, 4096), ("o", 4096, 4096), ("gate_up", 22016, 4096), ("down", 4096, 11008)]
    half_w = bool(args.half_weight_copies)
    M = args.micro_rows
    for name, N, K in shapes:
        A = torch.randn(M, K, device=dev).to(torch.float16)
        W = (torch.randn(N, K, device=dev) * 0.02).to(torch.bfloat16)
        Wx = R.rlhf_op_bf16_to_half(W) if half_w else W
        if name == "gate_up":          # as the stage runs it: SwiGLU in the epilogue
            act = torch.empty(M, N // 2, device=dev, dtype=torch.float16)
            timed(f"gemm_{name}_swiglu_M{M}", lambda: R.rlhf_op_gemm_swiglu(A, Wx, act),
                  (N * K + M * K) * 2.0 + M * (N // 2) * 2.0, 2.0 * M * N * K)
        elif name == "qkv":            # as the stage runs it: rotary and the q / k / v scatter in the epilogue
            Hq, hd = 32, 128
            pos = torch.randint(0, 2048, (M,), device=dev, dtype=torch.int32)
            ang = torch.arange(2048, device=dev)[:, None] * 10000.0 ** (-2.0 * torch.arange(hd // 2, device=dev) / hd)[None, :]
            tab = torch.stack([torch.cos(ang), torch.sin(ang)], dim=-1).float().contiguous()
            q, k, v = (torch.empty(M, Hq * hd, device=dev, dtype=torch.float16) for _ in range(3))
            timed(f"gemm_{name}_rope_M{M}", lambda: R.rlhf_op_gemm_rope(A, Wx, pos, tab, q, k, v, n_q_heads=Hq,
                                                                        n_kv_heads=Hq, head_dim=hd, check_indices=False),
                  (N * K + M * K) * 2.0 + M * N * 2.0, 2.0 * M * N * K)
        else:
            C = torch.empty(1, M, N, device=dev)
            timed(f"gemm_{name}_M{M}", lambda: R.rlhf_op_gemm(A, Wx, C, 1, 0 if half_w else 7),
                  (N * K + M * K) * 2.0 + M * N * 4.0, 2.0 * M * N * K)
    # LM head of a scoring pass fused with the log-softmax gather
    Mh, V, K = 2048, 32000, 4096
    A = torch.randn(Mh, K, device=dev).to(torch.float16)
    W = (torch.randn(V, K, device=dev) * 0.02).to(torch.bfloat16)
    Wx = R.rlhf_op_bf16_to_half(W) if half_w else W
    toks = torch.randint(0, V, (Mh,), device=dev, dtype=torch.int32)
    idx = torch.arange(Mh, device=dev, dtype=torch.int32)
    lp = torch.empty(Mh, device=dev)
    scratch = torch.empty(int(R.lib().rlhf_op_lm_head_logprob_scratch_floats(Mh, V)), device=dev)
    timed(f"gemm_lm_head_logprob_M{Mh}", lambda: R.rlhf_op_lm_head_logprob(A, Wx, toks, idx, lp, idx, scratch),
          (V * K + Mh * K) * 2.0 + scratch.numel() * 4.0, 2.0 * Mh * V * K)
    del A, W, Wx
    for M in (8, 32, 64, 128, 256):
        for name, N, K in shapes:
            A = torch.randn(M, K, device=dev).to(torch.float16)
            W = (torch.randn(N, K, device=dev) * 0.02).to(torch.bfloat16)
            ns = R.rlhf_op_gemm_nsplit(R.RLHF_BF16, M, N, K, 16)
            C = torch.empty(ns, M, N, device=dev)
            timed(f"gemm_{name}_M{M}", lambda: R.rlhf_op_gemm(A, W, C, ns),
                  (N * K + M * K) * 2.0 + ns * M * N * 4.0, 2.0 * M * N * K)
    rows, ctx, Hq, hd, Ly = 32, 1024, 32, 128, 1
    n_pages = rows * ctx // 16
    pool = torch.randn(n_pages, Ly, 2, Hq, 16, hd, device=dev).to(torch.float16)
    q = torch.randn(rows, Hq * hd, device=dev).to(torch.float16)
    pt = torch.randperm(n_pages, device=dev).to(torch.int32).reshape(rows, ctx // 16).contiguous()
    rs = torch.arange(rows, dtype=torch.int32, device=dev)
    cl = torch.full((rows,), ctx, dtype=torch.int32, device=dev)
    o = torch.empty_like(q)
    timed("decode_attn_B32_ctx1024", lambda: R.rlhf_op_paged_decode_attention(q, pool, pt, rs, cl, o, None, None, 0, 1, Ly,
                                                                            Hq, Hq, hd),
          rows * ctx * 2.0 * Hq * hd * 2, 4.0 * rows * ctx * Hq * hd)
    print(json.dumps({"micro": out}), flush=True)


def rt_sweep(cfg, args):
    """Fused stage time against the trigger R_t (Section 4.2, Figure 9's single-GPU analogue):
    R_t = 0 is the serial plan, R_t > N scores from the first retirement on."""
    R, ctx, weights, wl, max_new = build_stage(cfg, args)
    n = len(max_new)
    out = []
    run_stage(R, ctx, wl, max_new, True, args)                      # warm-up
    for frac in (0.0, 0.05, 0.1, 0.2, 0.35, 0.5, 0.75, 1.01):
        args.R_t = int(round(frac * n)) if frac <= 1.0 else n + 1
        ms, st, _ = run_stage(R, ctx, wl, max_new, args.R_t > 0, args)
        out.append({"R_t_over_N": frac, "R_t": args.R_t, "stage_ms": round(ms, 1), "batches": int(st.n_batches),
                    "decode_stream_ms": round(st.decode_stream_ms, 1), "score_stream_ms": round(st.score_stream_ms, 1)})
        log(f"[rt_sweep] R_t/N = {frac}: {ms:.0f} ms")
    R.rlhf_destroy(ctx)
    print(json.dumps({"rt_sweep": out, "workload": cfg.name, "score_chunk_tokens": args.score_chunk_tokens}), flush=True)


def bs_curve(cfg, args):
    """Decode step latency against the batch size B at a fixed context (the BS_max of
    Section 4.2: latency stays flat while decoding is bandwidth-bound)."""
    import torch

    import paper_2409_13221_amd as R
    from workload import make_weights
    m = cfg.model
    actor = make_weights(cfg, 0, device="cuda")
    P, steps = args.bs_ctx, 24
    page_b = m.n_layers * 2 * m.n_kv_heads * cfg.page_tokens * m.head_dim * m.elem_bytes()
    out = []
    for B in [int(b) for b in args.bs_list.split(",")]:
        pages = B * -(-(P + steps + 2) // cfg.page_tokens)
        ec = R.rlhf_engine_cfg(cfg.page_tokens, pages * page_b, B, P + steps + 2, B, max(8192, P + steps + 2),
                               cfg.eos_id, 0, 0, 0, None, None)
        ctx = R.rlhf_create(R.model_cfg_of(m), ec)
        R.rlhf_load_weights(ctx, 0, actor)
        rng = np.random.default_rng(B)
        toks = rng.integers(3, m.vocab, B * P).astype(np.int32)
        offs = (np.arange(B + 1) * P).astype(np.int64)
        lens = np.full(B, steps + 1, np.int32)
        med = []
        for rep in range(2):
            R.rlhf_submit(ctx, toks, offs, lens, lens)
            st, tr = R.rlhf_run_stage(ctx, False, 0, 1 << 30, 0, trace_cap=64, trace_time=True)
            med.append(float(np.median(tr["step_ms"][2:])))          # step 0 holds the prefill
        kv = B * (P + steps // 2) * m.kv_bytes_per_token()
        ms = min(med)
        out.append({"B": B, "ctx": P, "step_ms": round(ms, 3), "tokens_per_s": round(B / ms * 1e3, 1),
                    "hbm_GBps": round((m.decode_weight_bytes() + kv) / ms / 1e6, 1)})
        log(f"[bs_curve] B = {B}: {ms:.3f} ms/step")
        R.rlhf_destroy(ctx)
    print(json.dumps({"bs_curve": out, "workload": cfg.name}), flush=True)


def migrate_probe(cfg, args):
    """Cost of the re-prefill migration mechanism (Section 4.2, "Migration mechanism"): a sample
    at context ctx loses its KV cache and rebuilds it by one prefill; set beside the time to move
    the same cache as bytes (the first mechanism), at HBM copy speed and at one xGMI link."""
    import time

    import paper_2409_13221_amd as R
    from workload import make_weights
    m = cfg.model
    actor = make_weights(cfg, 0, device="cuda")
    page_b = m.n_layers * 2 * m.n_kv_heads * cfg.page_tokens * m.head_dim * m.elem_bytes()
    out = []
    for ctx_len in [int(c) for c in args.migrate_ctx.split(",")]:
        P, extra = ctx_len - 8, 24
        pages = -(-(P + extra + 2) // cfg.page_tokens)
        ec = R.rlhf_engine_cfg(cfg.page_tokens, pages * page_b, 1, P + extra + 2, 1, max(8192, P + extra + 2),
                               cfg.eos_id, 0, 0, 0, None, None)
        ctx = R.rlhf_create(R.model_cfg_of(m), ec)
        R.rlhf_load_weights(ctx, 0, actor)
        toks = np.random.default_rng(ctx_len).integers(3, m.vocab, P).astype(np.int32)
        lens = np.array([extra], np.int32)
        R.rlhf_submit(ctx, toks, np.array([0, P], np.int64), lens, lens)

        def step_ms():
            R.rlhf_sync(ctx)
            t0 = time.perf_counter()
            R.rlhf_generate_step(ctx)
            R.rlhf_sync(ctx)
            return (time.perf_counter() - t0) * 1e3
        first = step_ms()                                   # prompt prefill + one decode
        plain = min(step_ms() for _ in range(7))            # plain decode steps; context is now ctx_len
        R.rlhf_migrate(ctx, [0])
        moved = step_ms()                                   # re-prefill of ctx_len tokens + one decode
        after = step_ms()
        kv = ctx_len * m.kv_bytes_per_token()
        out.append({"ctx": ctx_len, "first_step_ms": round(first, 2), "decode_step_ms": round(plain, 2),
                    "reprefill_step_ms": round(moved, 2), "reprefill_ms": round(moved - plain, 2),
                    "decode_step_after_ms": round(after, 2), "kv_MB": round(kv / 1e6, 1),
                    "kv_copy_ms_at_5TBps": round(kv / 5.0e9, 3), "kv_xgmi_ms_at_153GBps": round(kv / 153e6, 2)})
        log(f"[migrate_probe] ctx {ctx_len}: re-prefill {moved - plain:.2f} ms, KV {kv / 1e6:.0f} MB")
        R.rlhf_destroy(ctx)
    print(json.dumps({"migrate_probe": out, "workload": cfg.name}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="7b")
    ap.add_argument("--R_t", type=int, default=-1, help="scoring trigger; -1 = n_samples + 1 (always on)")
    ap.add_argument("--score_chunk_tokens", type=int, default=8192)
    ap.add_argument("--max_batch_tokens", type=int, default=8192)
    ap.add_argument("--max_active", type=int, default=256)
    ap.add_argument("--role_mask", type=int, default=ROLE_MASK_DEFAULT)
    ap.add_argument("--corun_decode_cus", type=int, default=0,
                    help="compute units given to decoding while scoring is in flight (0 = no partition)")
    ap.add_argument("--sample_every", type=int, default=7,
                    help="time every n-th launch of a kernel class (co-prime with the 4 GEMMs per layer)")
    ap.add_argument("--fused", action="store_true", help="force the fused plan (default: the library chooses)")
    ap.add_argument("--sequential", action="store_true",
                    help="time the serial generate-then-score plan instead (clean per-kernel figures)")
    ap.add_argument("--rt_sweep", action="store_true", help="fused stage time vs the trigger R_t")
    ap.add_argument("--bs_curve", action="store_true", help="decode step latency vs batch size (BS_max)")
    ap.add_argument("--admission", choices=["reserve", "optimistic"], default="optimistic",
                    help="reserve: a sample is admitted when its KV reservation at the length cap fits; "
                         "optimistic: on present need, with preemption by re-prefill")
    ap.add_argument("--half_weight_copies", type=int, default=1,
                    help="1: the library keeps IEEE-half copies of the bf16 matrices for prefill / scoring passes "
                         "(both GEMM operands direct to LDS); 0: bf16 weights converted on the fly")
    ap.add_argument("--weights", choices=["seeded", "normal"], default="seeded",
                    help="seeded: the workload's counter-based generator; normal: torch's (profiler runs only)")
    ap.add_argument("--micro_rows", type=int, default=8192, help="rows of the scoring-pass cases of --micro")
    ap.add_argument("--migrate_probe", action="store_true", help="cost of migration by re-prefill vs moving the KV cache")
    ap.add_argument("--migrate_ctx", default="512,1024,2048", help="contexts of --migrate_probe")
    ap.add_argument("--bs_list", default="1,2,4,8,16,32,64,128,256", help="batch sizes of --bs_curve")
    ap.add_argument("--bs_ctx", type=int, default=512)
    ap.add_argument("--micro", action="store_true", help="run the kernel-level cases instead of the stage")
    ap.add_argument("--micro_reps", type=int, default=5)
    ap.add_argument("--no_cpu", action="store_true")
    ap.add_argument("--no_sequential", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the stage shards by sample across GPUs with no collective "
              "inside it, so N GPUs are N independent copies of this run).  Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch

    from workload import CONFIGS
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.micro:
        micro(args)
        return
    torch.cuda.set_device(0)
    cfg = CONFIGS[args.config]
    if args.rt_sweep:
        rt_sweep(cfg, args)
        return
    if args.migrate_probe:
        migrate_probe(cfg, args)
        return
    if args.bs_curve:
        bs_curve(cfg, args)
        return
    R, ctx, weights, wl, max_new = build_stage(cfg, args)
    # the library picks the plan (fused unless a decode step of this model is launch-bound) unless told otherwise
    plan = False if args.sequential else True if args.fused else "auto"

    for i in range(args.warmup):
        ms, st, _ = run_stage(R, ctx, wl, max_new, plan, args)
        log(f"[bench] warmup {i}: {ms:.1f} ms, {st.n_steps} steps, {st.n_batches} scoring batches, "
            f"plan {'fused' if st.fused_used else 'serial'}")
    R.rlhf_profile_begin(ctx, args.sample_every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    times, last = [], None
    for i in range(args.steps):
        ms, st, tr = run_stage(R, ctx, wl, max_new, plan, args, trace=(i == args.steps - 1))
        times.append(ms)
        last = (st, tr)
        log(f"[bench] step {i}: {ms:.1f} ms")
    torch.cuda.synchronize()
    total_ms = (time.perf_counter() - t0) * 1e3
    prof = R.rlhf_profile_end(ctx)
    st, tr = last
    ms_per_step = total_ms / args.steps
    G, S = int(st.generated_tokens), int(st.scored_tokens)
    value = (G + S) / (ms_per_step * 1e-3)

    # one roofline object per kernel class; `roofline` is the class with the largest share of GPU time
    roofs = rooflines(prof, cfg.model.dtype, args.steps)
    for k, r in roofs.items():
        if r["dropped"]:
            log(f"[bench] WARNING: {r['dropped']} launches of {k} were due for timing but found no free event pair; "
                f"raise --sample_every")
    # HBM-side bytes per launch from the committed rocprofv3 counter summary (FETCH_SIZE and WRITE_SIZE runs
    # over the kernel-level cases of --micro, each scaled by a 1 GiB copy): a per-kernel micro-case figure,
    # not a counter run over this stage
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{cfg.name}.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            f = line.split()
            if len(f) >= 4 and f[0] in roofs:
                roofs[f[0]]["traffic"] = float(f[1]) + float(f[2])
                roofs[f[0]]["traffic_detail"] = {"fetched_bytes": float(f[1]), "written_bytes": float(f[2]),
                                                 "algorithmic_bytes": float(f[3]), "scope": "kernel-level micro cases",
                                                 "source": f"profiles/hbm_traffic_{cfg.name}.txt"}
    roof = max(roofs.values(), key=lambda r: r["est_ms_per_stage"]) if roofs else None

    # long-tail lens: steps with at most 20 % of the batch still active; decode-only steps
    lens = {}
    if tr is not None and "step_ms" in tr:
        n = len(max_new)
        dec_only = tr["prefill_tokens"] == 0
        tail = (tr["active"] <= 0.2 * n) & dec_only
        def gbps(mask):
            t = float(tr["step_ms"][mask].sum())
            return round(float(tr["step_bytes"][mask].sum()) / (t * 1e-3) / 1e9, 1) if t > 0 else None
        lens = {"decode_steps": int(st.n_steps), "tail_steps_frac": round(float(tail.mean()), 4),
                "tail_time_frac": round(float(tr["step_ms"][tail].sum() / max(tr["step_ms"].sum(), 1e-9)), 4),
                "decode_hbm_GBps": gbps(dec_only), "tail_hbm_GBps": gbps(tail),
                "decode_hbm_frac": round((gbps(dec_only) or 0) / HBM_PEAK_GBS, 4),
                "decode_stream_ms": round(st.decode_stream_ms, 1), "score_stream_ms": round(st.score_stream_ms, 1),
                "generated_tokens": G, "scored_tokens": S, "scoring_batches": int(st.n_batches)}

    # the serial plan (generate everything, then score) under the same conditions: profiler on, the same
    # sampling stride; up to three runs, mean
    seq = None
    if not args.no_sequential and not args.sequential:
        n_seq = min(args.steps, 3)
        R.rlhf_profile_begin(ctx, args.sample_every)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n_seq):
            ms_i, _, _ = run_stage(R, ctx, wl, max_new, False, args)
            log(f"[bench] sequential generate-then-score {i}: {ms_i:.1f} ms")
        torch.cuda.synchronize()
        ms_seq = (time.perf_counter() - t0) * 1e3 / n_seq
        prof_seq = R.rlhf_profile_end(ctx)
        rs = rooflines(prof_seq, cfg.model.dtype, n_seq)
        seq = {"sequential_ms": round(ms_seq, 1), "fused_ms": round(ms_per_step, 1),
               "speedup": round(ms_seq / ms_per_step, 3), "runs": {"fused": args.steps, "sequential": n_seq},
               "profiler": "on in both, same stride",
               "sequential_kernels": {k: {"avg_launch_us": r["avg_launch_us"], "achieved": r["achieved"],
                                          "unit": r["unit"], "frac": r["frac"],
                                          "est_ms_per_stage": r["est_ms_per_stage"]} for k, r in rs.items()}}
    R.rlhf_destroy(ctx)

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(cfg, weights)

    out = {"metric": "gen+scored tokens/s per GPU (long-tail lens)", "value": round(value, 1), "unit": "tokens/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 2),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": ARITH[cfg.model.dtype],
           "data": "synthetic",
           "config": {"workload": cfg.name, "n_samples": int(len(max_new)), "length_law": cfg.length_law,
                      "length_params": list(cfg.length_params), "length_cap": cfg.length_cap,
                      "plan": "fused" if st.fused_used else "sequential",
                      "corun_decode_cus": args.corun_decode_cus, "admission": args.admission,
                      "half_weight_copies": int(args.half_weight_copies and cfg.model.dtype == "bf16"),
                      "score_chunk_tokens": args.score_chunk_tokens, "R_t": args.R_t, "role_mask": args.role_mask,
                      "page_tokens": cfg.page_tokens},
           "roofline": roof, "cpu_baseline": cpu, "fused_vs_sequential": seq, "roofline_all": roofs,
           "roofline_clock": "HIP events on the kernel's own stream around every "
                             f"{args.sample_every}th launch of a class over all {args.steps} timed stages, minus the "
                             "bracket's own cost (2 x median bracket of one empty kernel - that of two)",
           "long_tail": lens}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
