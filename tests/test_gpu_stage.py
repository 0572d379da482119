"""Stage-level parity through the C ABI: the HIP path against the oracle on the same seeded
inputs -- token ids, log-probs, values, rewards, and bit-exact bookkeeping."""
import numpy as np
import pytest

from tests import stage_harness as H
from workload import CONFIGS

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tiny_ref():
    cfg = CONFIGS["tiny"].with_(gain_jitter=0.05)
    return cfg, H.oracle_stage(cfg)


def test_tiny_fused_stage_matches_oracle(tiny_ref):
    cfg, ref = tiny_ref
    got = H.run_gpu_stage(cfg, ref, fused=True, R_t=9, chunk_tokens=128)
    worst = H.compare_stage(cfg, ref, got)
    print("tiny fused worst errors:", worst)
    assert got["stats"].generated_tokens == int(ref["out_len"].sum())


def test_tiny_sequential_equals_fused(tiny_ref):
    """Section 4.1: fusing the stages does not change any sample's result."""
    cfg, ref = tiny_ref
    a = H.run_gpu_stage(cfg, ref, fused=True, R_t=9, chunk_tokens=128)
    b = H.run_gpu_stage(cfg, ref, fused=False, R_t=0, chunk_tokens=128)
    H.compare_stage(cfg, ref, b)
    np.testing.assert_array_equal(a["tokens"], b["tokens"])
    np.testing.assert_array_equal(a["lp_actor"], b["lp_actor"])     # same decode batches: bit-identical
    for k in ("lp_ref", "values", "reward", "lp_actor_rescored"):   # different scoring batches
        np.testing.assert_allclose(a[k], b[k], rtol=0, atol=2e-5)
    assert a["snapshot"]["retired"] == b["snapshot"]["retired"]
    assert a["stats"].n_steps == b["stats"].n_steps


@pytest.mark.parametrize("pool_factor,max_active", [(1.0, None), (0.45, None), (1.0, 3)])
def test_tiny_bookkeeping_is_bit_exact_step_by_step(tiny_ref, pool_factor, max_active):
    cfg, ref = tiny_ref
    with H.GpuStage(cfg, ref, max_active=max_active) as probe:
        need = probe.pool_pages
        biggest = int(np.ceil((probe.plen + probe.max_new) / cfg.page_tokens).max())
    pool = max(biggest, int(need * pool_factor))
    with H.GpuStage(cfg, ref, pool_pages=pool, max_active=max_active) as g:
        g.submit(ref["forced"])
        model = H.scheduler_model_for(g)
        while True:
            snap = g.snapshot()
            assert snap["n_waiting"] == len(model.waiting)
            if model.generation_done():
                break
            info = g.R.rlhf_generate_step(g.ctx)
            want = model.generate_step()
            assert (info.step, info.n_admitted, info.n_prefill_tokens, info.n_decoded, info.n_active) == \
                   (want.step, want.n_admitted, want.n_prefill_tokens, want.n_decoded, want.n_active)
            gone = g.R.rlhf_retire(g.ctx, g.n).tolist()
            assert gone == model.retire()
            snap, ms = g.snapshot(), model.snapshot()
            for k in ("step", "active", "ctx", "gen_len", "pages", "free", "reserved", "retired"):
                assert snap[k] == ms[k], k
        g.R.rlhf_score(g.ctx, model.retired, H.ALL_ROLES, True)
        got = g.results()
    H.compare_stage(cfg, ref, got)


@pytest.mark.parametrize("fused,R_t,chunk", [(True, 9, 64), (True, 3, 64), (False, 0, 100), (True, 9, 1)])
def test_tiny_run_stage_batches_match_scheduler_model(tiny_ref, fused, R_t, chunk):
    cfg, ref = tiny_ref
    with H.GpuStage(cfg, ref) as g:
        g.submit(ref["forced"])
        model = H.scheduler_model_for(g)
        trace = model.run_stage(fused, R_t, chunk)
        stats, tr = g.R.rlhf_run_stage(g.ctx, fused, R_t, chunk, H.ALL_ROLES, trace_cap=4096)
        snap = g.snapshot()
        got = g.results()
    assert stats.n_steps == len(trace) and stats.n_batches == len(model.batches)
    assert snap["batches"] == model.batches and snap["batch_step"] == model.batch_step
    assert snap["retired"] == model.retired and snap["free"] == model.free
    assert tr["decoded"].tolist() == [t[0].n_decoded for t in trace]
    assert tr["active"].tolist() == [t[0].n_active - len(t[1]) for t in trace]
    H.compare_stage(cfg, ref, got)


def test_tiny_small_batch_workspace_splits_passes(tiny_ref):
    """Prefill and scoring passes bounded by max_batch_tokens give the same results."""
    cfg, ref = tiny_ref
    got = H.run_gpu_stage(cfg, ref, fused=True, R_t=9, chunk_tokens=10_000, max_batch_tokens=100)
    H.compare_stage(cfg, ref, got)


def test_errors_are_reported_not_fatal(tiny_ref):
    cfg, ref = tiny_ref
    import paper_2409_13221_amd as R
    mc = R.model_cfg_of(cfg.model)
    bad = R.rlhf_engine_cfg(8, 1 << 20, 4, 64, 4, 64, 2, 0, 0, 0, None, None)
    with pytest.raises(R.RlhfError) as e:
        R.rlhf_create(mc, bad)
    assert e.value.code == R.RLHF_EINVAL and "page_tokens" in str(e.value)
    with H.GpuStage(cfg, ref) as g:
        with pytest.raises(R.RlhfError) as e:
            R.rlhf_generate_step(g.ctx)              # nothing submitted
        assert e.value.code == R.RLHF_ESTATE
        g.submit(ref["forced"])
        with pytest.raises(R.RlhfError) as e:
            R.rlhf_score(g.ctx, [0], H.ALL_ROLES)    # still generating
        assert e.value.code == R.RLHF_ESTATE
        with pytest.raises(R.RlhfError) as e:
            R.rlhf_score(g.ctx, [99], H.ALL_ROLES)
        assert e.value.code == R.RLHF_EINVAL
    with H.GpuStage(cfg, ref, pool_pages=2) as g:
        with pytest.raises(R.RlhfError) as e:
            g.submit(ref["forced"])                  # one sample's reservation exceeds the pool
        assert e.value.code == R.RLHF_ENOMEM


# ------------------------------------------------------------------------------ bf16 path

@pytest.fixture(scope="module")
def gpt2s_ref():
    """GPT-2-small shape, bf16, real depth; 6 samples with outputs capped at 24 so that the
    float64 oracle finishes in seconds.  Weights are drawn on the GPU and copied to the host."""
    cfg = CONFIGS["gpt2s"].with_(gain_jitter=0.05)
    inp = H.make_inputs(cfg, n=6, max_len=24, weight_device="cuda")
    return cfg, H.oracle_stage(cfg, inp=inp)


def test_gpt2s_bf16_stage_matches_oracle(gpt2s_ref):
    cfg, ref = gpt2s_ref
    got = H.run_gpu_stage(cfg, ref, fused=True, R_t=7, chunk_tokens=600)
    worst = H.compare_stage(cfg, ref, got)
    print("gpt2s bf16 worst errors:", worst, "forced positions:",
          int(sum((f >= 0).sum() for f in ref["forced"])), "of", int(ref["out_len"].sum()))
    seq = H.run_gpu_stage(cfg, ref, fused=False, R_t=0, chunk_tokens=600)
    H.compare_stage(cfg, ref, seq)
    np.testing.assert_array_equal(got["tokens"], seq["tokens"])


def test_gqa_bf16_small_model_matches_oracle():
    """Grouped KV heads (8 query heads per KV head, head_dim 128) on a small bf16 model."""
    from workload.configs import ModelCfg
    base = CONFIGS["tiny"]
    m = ModelCfg(n_layers=2, d_model=512, n_q_heads=16, n_kv_heads=2, head_dim=128, ffn=1024, vocab=2048,
                 dtype="bf16")
    cfg = base.with_(name="gqa_small", model=m, n_samples=5, prompt_len=(20, 45), gain_jitter=0.05)
    ref = H.oracle_stage(cfg, max_len=20)
    got = H.run_gpu_stage(cfg, ref, fused=True, R_t=6, chunk_tokens=64)
    print("gqa worst errors:", H.compare_stage(cfg, ref, got))
