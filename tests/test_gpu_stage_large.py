"""Parity at the real layer shapes (7B / 13B / 70B-slice widths), and the full-size runs in
the benchmark's launch configuration checked on sampled outputs and by properties."""
import numpy as np
import pytest

from tests import stage_harness as H
from workload import CONFIGS

pytestmark = pytest.mark.gpu


def _slice_case(name, n_layers, n, prompt_len, max_len):
    cfg = CONFIGS[name].with_(prompt_len=prompt_len, gain_jitter=0.05)
    inp = H.make_inputs(cfg, n=n, max_len=max_len, n_layers=n_layers, weight_device="cuda")
    return cfg, H.oracle_stage(cfg, inp=inp, dtype=np.float32)


@pytest.mark.parametrize("name,n_layers,n,prompt_len,max_len", [
    ("7b", 3, 4, (40, 150), 20),          # d 4096, 32 x 128 heads, ffn 11008, vocab 32000
    ("13b", 2, 3, (40, 100), 12),         # d 5120 (two RMSNorm iterations), 40 heads, ffn 13824
    ("70b_slice", 1, 3, (40, 100), 12),   # d 8192, 64 query / 8 KV heads, ffn 28672
])
def test_real_width_layer_slices_match_oracle(name, n_layers, n, prompt_len, max_len):
    """Real widths, reduced depth and sample count so that the float32 oracle finishes in
    seconds; fused and serial plans."""
    cfg, ref = _slice_case(name, n_layers, n, prompt_len, max_len)
    print(f"[{name}] oracle done", flush=True)
    got = H.run_gpu_stage(cfg, ref, fused=True, R_t=n + 1, chunk_tokens=200)
    worst = H.compare_stage(cfg, ref, got)
    print(f"[{name}] fused worst errors:", worst, flush=True)
    seq = H.run_gpu_stage(cfg, ref, fused=False, R_t=0, chunk_tokens=200)
    H.compare_stage(cfg, ref, seq)
    np.testing.assert_array_equal(got["tokens"], seq["tokens"])


def test_7b_full_depth_matches_oracle():
    """All 32 layers of the 7B shape on two short samples (Actor generation + re-scoring and
    Critic values; the float32 oracle holds one 27 GB model at a time)."""
    cfg = CONFIGS["7b"].with_(prompt_len=(48, 64), gain_jitter=0.05)
    inp = H.make_inputs(cfg, n=2, max_len=6, weight_device="cuda")
    print("[7b full depth] weights ready", flush=True)
    # generation by the oracle (Actor), with forcing decided by its own margins
    import oracle.transformer as OT
    shape = OT.Shape.of(cfg.model)
    actor = OT.Model(shape, {k: v.float().cpu().numpy() for k, v in inp["weights"][0].items()}, np.float32)
    po = inp["prompt_offsets"]
    prompts = [inp["prompt_tokens"][po[i]:po[i + 1]].tolist() for i in range(2)]
    gen = OT.greedy_generate_cached(actor, prompts, inp["out_len"], cfg.eos_id)
    del actor
    print("[7b full depth] oracle generation done", flush=True)
    ref = dict(inp)
    ref["forced"] = [np.where(g.margin < H.MARGIN, g.tokens, -1).astype(np.int32) for g in gen]
    got = H.run_gpu_stage(cfg, ref, fused=True, R_t=3, chunk_tokens=64, role_mask=0b0101)
    for i, g in enumerate(gen):
        np.testing.assert_array_equal(H.unpack(got, "tokens")[i], g.tokens)
        assert np.abs(H.unpack(got, "lp_actor")[i] - g.logprob).max() <= 2e-2
        assert np.abs(H.unpack(got, "lp_actor_rescored")[i] - g.logprob).max() <= 2e-2
    worst = H.check_samples_by_teacher_forcing(cfg, inp, got, [0, 1], roles=(2,), value_tol=H.DEEP)
    print("[7b full depth] worst:", worst, flush=True)


def test_gpt2s_full_config_sampled_outputs_and_bookkeeping():
    """The whole GPT-2-small-shape workload (64 samples, outputs up to 1024) as bench.py runs
    it; bookkeeping bit-exact against the scheduler model, three samples (the longest one
    included) checked through the oracle by teacher forcing."""
    cfg = CONFIGS["gpt2s"]
    inp = H.make_inputs(cfg, weight_device="cuda")
    with H.GpuStage(cfg, inp, max_new_cap=cfg.length_cap, max_batch_tokens=8192) as g:
        g.submit(None)
        model = H.scheduler_model_for(g)
        trace = model.run_stage(True, g.n + 1, 6144)
        stats, tr = g.R.rlhf_run_stage(g.ctx, True, g.n + 1, 6144, H.ALL_ROLES, trace_cap=4096)
        snap = g.snapshot()
        got = g.results()
    assert stats.n_steps == len(trace) and snap["batches"] == model.batches
    assert snap["retired"] == model.retired and snap["batch_step"] == model.batch_step
    assert tr["decoded"].tolist() == [t[0].n_decoded for t in trace]
    assert got["gen_len"].tolist() == inp["out_len"].tolist()
    ids = sorted({int(np.argmax(inp["out_len"])), 0, 17})
    worst = H.check_samples_by_teacher_forcing(cfg, inp, got, ids, dtype=np.float64)
    print("gpt2s full config, sampled:", ids, worst, flush=True)
    # the re-scored Actor log-probs (full forward) agree with those captured while decoding
    assert np.abs(got["lp_actor"] - got["lp_actor_rescored"]).max() <= 4e-2


def test_gpt2s_full_config_optimistic_admission_under_memory_pressure():
    """The same workload with a KV pool of 300 pages (the cap reservations add up to 5120, the
    samples' own lengths to 1751): admission on present need and preemption by re-prefill.  The
    scheduler model predicts every step (10 preemptions, 1267 steps instead of the 3729 of cap
    reservations); the longest sample and two others are checked through the oracle; and for ALL
    samples the log-probs captured while decoding (over caches that were partly rebuilt by
    prefill) agree with a full forward."""
    cfg = CONFIGS["gpt2s"]
    inp = H.make_inputs(cfg, weight_device="cuda")
    with H.GpuStage(cfg, inp, pool_pages=300, max_new_cap=cfg.length_cap, max_batch_tokens=8192,
                    optimistic=True) as g:
        g.submit(None)
        model = H.scheduler_model_for(g)
        trace = model.run_stage(True, g.n + 1, 6144)
        stats, tr = g.R.rlhf_run_stage(g.ctx, True, g.n + 1, 6144, H.ALL_ROLES, trace_cap=4096)
        snap = g.snapshot()
        got = g.results()
    assert model.n_preempted == 10 and len(trace) == 1267
    assert stats.n_steps == len(trace) and snap["batches"] == model.batches
    assert snap["retired"] == model.retired and snap["free"] == model.free
    assert tr["decoded"].tolist() == [t[0].n_decoded for t in trace]
    assert tr["prefill_tokens"].tolist() == [t[0].n_prefill_tokens for t in trace]
    assert got["gen_len"].tolist() == inp["out_len"].tolist()
    ids = sorted({int(np.argmax(inp["out_len"])), 5, 40})
    worst = H.check_samples_by_teacher_forcing(cfg, inp, got, ids, dtype=np.float64)
    print("gpt2s full config, optimistic admission, sampled:", ids, worst, flush=True)
    assert np.abs(got["lp_actor"] - got["lp_actor_rescored"]).max() <= 4e-2


@pytest.mark.parametrize("optimistic", [True, False])
def test_7b_full_config_properties(optimistic):
    """The 7B-shape workload at full size in bench.py's configuration (optimistic admission is
    what bench.py times by default; cap reservations, where the KV pool gates admission, is its
    --admission reserve): bookkeeping bit-exact against the scheduler model, fused and serial
    plans give identical tokens, and the Actor log-probs captured by cached decoding agree with
    their re-scoring by a full forward (cached decode = full recompute).  In the benchmark's
    configuration the run is also checked against the oracle: the longest sample (more than a
    thousand output tokens, context past 1500) and a short one go through the float32 oracle at
    full depth for all four roles (teacher forcing on the GPU's own tokens)."""
    import torch
    cfg = CONFIGS["7b"]
    inp = H.make_inputs(cfg, weight_device="cuda")
    print("[7b full] weights ready", flush=True)
    free_b, _ = torch.cuda.mem_get_info()
    # as bench.py: half copies of the four roles' matrices live beside the pool
    pool_pages = int((free_b - (24 << 30) - 4 * cfg.model.decode_weight_bytes()) // H.page_bytes(cfg))
    with H.GpuStage(cfg, inp, pool_pages=pool_pages, max_new_cap=cfg.length_cap, max_batch_tokens=8192,
                    optimistic=optimistic, half_weight_copies=True) as g:
        assert g.pool_pages < int(np.ceil((g.plen + g.max_new) / 16).sum())      # cap reservations would not fit
        g.submit(None)
        model = H.scheduler_model_for(g)
        trace = model.run_stage(True, g.n + 1, 6144)
        stats, tr = g.R.rlhf_run_stage(g.ctx, True, g.n + 1, 6144, H.ALL_ROLES, trace_cap=4096)
        snap = g.snapshot()
        fused = g.results()
        print(f"[7b full] fused stage {stats.wall_ms:.0f} ms", flush=True)
        assert stats.n_steps == len(trace) and snap["batches"] == model.batches
        assert snap["retired"] == model.retired and snap["free"] == model.free
        assert tr["decoded"].tolist() == [t[0].n_decoded for t in trace]
        assert tr["active"].tolist() == [t[0].n_active - len(t[1]) for t in trace]
        assert tr["prefill_tokens"].tolist() == [t[0].n_prefill_tokens for t in trace]   # re-prefills included
        if optimistic:
            assert trace[0][0].n_admitted == g.n                                  # nobody waits for a reservation
        else:
            assert max(t[0].n_admitted for t in trace[1:]) > 0                    # late admissions happened
        g.submit(None)
        stats2, _ = g.R.rlhf_run_stage(g.ctx, False, 0, 6144, 0b1110, trace_cap=0)
        serial = g.results()
        print(f"[7b full] serial stage {stats2.wall_ms:.0f} ms", flush=True)
    assert fused["gen_len"].tolist() == inp["out_len"].tolist()
    np.testing.assert_array_equal(fused["tokens"], serial["tokens"])
    np.testing.assert_array_equal(fused["lp_actor"], serial["lp_actor"])
    for k in ("lp_ref", "values"):
        assert np.abs(fused[k] - serial[k]).max() <= 2e-3, k                      # batch composition differs
    # two evaluations, each within 2e-2 of the exact log-prob, differ by at most 4e-2
    gap = float(np.abs(fused["lp_actor"] - fused["lp_actor_rescored"]).max())
    print(f"[7b full] max |lp_actor - lp_actor_rescored| over {fused['lp_actor'].size} tokens: {gap:.4f}", flush=True)
    assert gap <= 4e-2
    assert np.all(np.isfinite(fused["reward"])) and np.all(fused["lp_ref"] <= 0)
    if optimistic:
        longest = int(np.argmax(inp["out_len"]))
        short = int(np.argmin(np.where(inp["out_len"] >= 8, inp["out_len"] + np.diff(inp["prompt_offsets"]), 1 << 30)))
        po = inp["prompt_offsets"]
        print(f"[7b full] oracle check of sample {longest} (prompt {po[longest + 1] - po[longest]}, output "
              f"{inp['out_len'][longest]}) and sample {short} (prompt {po[short + 1] - po[short]}, output "
              f"{inp['out_len'][short]}), all four roles", flush=True)
        worst = H.check_samples_by_teacher_forcing(cfg, inp, fused, [longest, short], dtype=np.float32,
                                                   roles=(0, 1, 2, 3), value_tol=H.DEEP, deep_tokens=True)
        print("[7b full] sampled outputs against the oracle:", worst, flush=True)


def _deep_stage_against_oracle(name, n_layers, n, max_len, prompt_len, role_samples):
    """A stage at (nearly) full depth of a wide shape on a few samples with contexts beyond a
    thousand tokens: the GPU generates and scores (fused plan); every sample's tokens, Actor
    log-probs and, per role_samples, Reference log-probs / values / rewards go through the float32
    oracle by teacher forcing.  The serial plan must give the same tokens."""
    cfg = CONFIGS[name].with_(gain_jitter=0.05) if prompt_len is None else \
        CONFIGS[name].with_(gain_jitter=0.05, prompt_len=prompt_len)
    inp = H.make_inputs(cfg, n=n, max_len=max_len, n_layers=n_layers, weight_device="cuda")
    print(f"[{name} x{n_layers}] weights ready; outputs {inp['out_len'].tolist()}, prompts "
          f"{np.diff(inp['prompt_offsets']).tolist()}", flush=True)
    got = H.run_gpu_stage(cfg, inp, fused=True, R_t=n + 1, chunk_tokens=1024, max_batch_tokens=4096)
    seq = H.run_gpu_stage(cfg, inp, fused=False, R_t=0, chunk_tokens=1024, max_batch_tokens=4096)
    np.testing.assert_array_equal(got["tokens"], seq["tokens"])
    np.testing.assert_array_equal(got["lp_actor"], seq["lp_actor"])
    assert np.abs(got["lp_actor"] - got["lp_actor_rescored"]).max() <= 4e-2
    worst = H.check_samples_by_teacher_forcing(cfg, inp, got, list(range(n)), dtype=np.float32, roles=(0, 1, 2, 3),
                                               value_tol=H.DEEP, role_samples=role_samples, deep_tokens=True)
    print(f"[{name} x{n_layers}] against the oracle:", worst, flush=True)
    assert (np.diff(inp["prompt_offsets"]) + inp["out_len"]).max() >= 1000


def test_70b_slice_full_depth_stage_matches_oracle():
    """All 10 layers of the 70B-slice shape (64 query / 8 KV heads: the grouped-head MFMA decode
    attention and the grouped flash attention inside a deep stage), prompts of 1024 tokens."""
    _deep_stage_against_oracle("70b_slice", None, n=2, max_len=24, prompt_len=None,
                               role_samples={1: [1], 2: [0], 3: [1]})


def test_13b_eight_layer_stage_matches_oracle():
    """8 of the 40 layers of the 13B shape (d 5120, 40 heads), one context beyond a thousand tokens."""
    _deep_stage_against_oracle("13b", 8, n=2, max_len=200, prompt_len=(880, 900), role_samples={1: [0], 3: [0]})
