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


@pytest.mark.parametrize("to_back,pool_factor", [(False, 1.0), (True, 1.0), (False, 0.4)])
def test_tiny_migration_by_reprefill(tiny_ref, to_back, pool_factor):
    """Section 4.2, second migration mechanism: stragglers lose their KV cache and get it back by
    a prefill over prompt + generated tokens.  Bookkeeping follows the scheduler model bit for bit
    and tokens, log-probs, values and rewards are those of an undisturbed run."""
    cfg, ref = tiny_ref
    with H.GpuStage(cfg, ref) as probe:
        need = probe.pool_pages
        biggest = int(np.ceil((probe.plen + probe.max_new) / cfg.page_tokens).max())
    pool = max(biggest, int(need * pool_factor))
    r = np.random.default_rng(5)
    with H.GpuStage(cfg, ref, pool_pages=pool) as g:
        g.submit(ref["forced"])
        model = H.scheduler_model_for(g)
        moved = 0
        while not model.generation_done():
            info = g.R.rlhf_generate_step(g.ctx)
            want = model.generate_step()
            assert (info.step, info.n_admitted, info.n_prefill_tokens, info.n_decoded, info.n_active) == \
                   (want.step, want.n_admitted, want.n_prefill_tokens, want.n_decoded, want.n_active)
            assert g.R.rlhf_retire(g.ctx, g.n).tolist() == model.retire()
            movable = [i for i in model.active if model.gen_len[i] < model.target[i]]
            if movable and info.step % 3 == 1:
                ids = [int(i) for i in r.permutation(movable)[:max(1, len(movable) // 2)]]
                g.R.rlhf_migrate(g.ctx, ids, to_back)
                model.migrate(ids, to_back)
                moved += len(ids)
            snap, ms = g.snapshot(), model.snapshot()
            for k in ("step", "n_waiting", "active", "ctx", "gen_len", "pages", "free", "reserved", "retired"):
                assert snap[k] == ms[k], k
        assert moved >= 3
        # what cannot move: retired, waiting or unknown samples, duplicates
        for bad in ([model.retired[0]], [g.n], [-1]):
            with pytest.raises(g.R.RlhfError):
                g.R.rlhf_migrate(g.ctx, bad)
        g.R.rlhf_score(g.ctx, model.retired, H.ALL_ROLES, True)
        got = g.results()
    H.compare_stage(cfg, ref, got)


@pytest.mark.parametrize("pool_pages,max_new_cap,n_preempted", [(48, 64, 0), (16, 64, 0), (9, 64, 1), (7, 64, 2),
                                                                 (16, None, 0)])
def test_tiny_optimistic_admission_and_preemption(tiny_ref, pool_pages, max_new_cap, n_preempted):
    """Admission on present need with preemption by re-prefill: under pools from ample down to one
    page more than a single sample's cap, every step's bookkeeping (who is admitted, who is preempted,
    which pages) equals the scheduler model's, and the outputs are those of the undisturbed run."""
    cfg, ref = tiny_ref
    pool = pool_pages          # the cap reservations of the 8 samples add up to 48 (33 at their own lengths)
    with H.GpuStage(cfg, ref, pool_pages=pool, max_new_cap=max_new_cap, optimistic=True) as g:
        g.submit(ref["forced"])
        model = H.scheduler_model_for(g)
        preempted = 0
        while not model.generation_done():
            info = g.R.rlhf_generate_step(g.ctx)
            before = model.n_preempted
            want = model.generate_step()
            assert (info.step, info.n_admitted, info.n_prefill_tokens, info.n_decoded, info.n_active) == \
                   (want.step, want.n_admitted, want.n_prefill_tokens, want.n_decoded, want.n_active)
            assert info.n_preempted == model.n_preempted - before
            preempted += info.n_preempted
            assert g.R.rlhf_retire(g.ctx, g.n).tolist() == model.retire()
            snap, ms = g.snapshot(), model.snapshot()
            for k in ("step", "n_waiting", "active", "ctx", "gen_len", "pages", "free", "reserved", "retired"):
                assert snap[k] == ms[k], k
        assert preempted == n_preempted
        g.R.rlhf_score(g.ctx, model.retired, H.ALL_ROLES, True)
        got = g.results()
    H.compare_stage(cfg, ref, got)
    # the whole-stage entry point runs the same policy
    with H.GpuStage(cfg, ref, pool_pages=pool, max_new_cap=max_new_cap, optimistic=True) as g:
        g.submit(ref["forced"])
        stats, _ = g.R.rlhf_run_stage(g.ctx, True, g.n + 1, 64, H.ALL_ROLES)
        assert stats.n_steps == model.step
        H.compare_stage(cfg, ref, g.results())


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


def test_gpt2s_bf16_migration_by_reprefill(gpt2s_ref):
    """The same migration on the bf16 path, where the rebuilt cache comes from the MFMA prefill
    kernels instead of the decode kernels: results stay within the stage's tolerances, and
    tokens are those of the undisturbed run except where the oracle itself is within MARGIN of
    a tie (those positions are teacher-forced in both runs)."""
    cfg, ref = gpt2s_ref
    plain = H.run_gpu_stage(cfg, ref, fused=True, R_t=7, chunk_tokens=600)
    with H.GpuStage(cfg, ref) as g:
        g.submit(ref["forced"])
        model = H.scheduler_model_for(g)
        while not model.generation_done():
            info = g.R.rlhf_generate_step(g.ctx)
            model.generate_step()
            assert g.R.rlhf_retire(g.ctx, g.n).tolist() == model.retire()
            movable = [i for i in model.active if model.gen_len[i] < model.target[i]]
            if movable and info.step in (4, 9, 10):
                ids = movable[::2]
                g.R.rlhf_migrate(g.ctx, ids, info.step == 9)
                model.migrate(ids, info.step == 9)
        g.R.rlhf_score(g.ctx, model.retired, H.ALL_ROLES, True)
        got = g.results()
    print("gpt2s migrated worst errors:", H.compare_stage(cfg, ref, got))
    np.testing.assert_array_equal(got["tokens"], plain["tokens"])
    assert np.abs(got["lp_actor"] - plain["lp_actor"]).max() <= 2 * H.LP_TOL["bf16"]


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


# --------------------------------------------------------------- termination on EOS, GAE

def test_tiny_stop_on_eos_matches_oracle():
    """Generation "until reaching a termination token": the Actor's LM-head row of eos_id is
    scaled up so that EOS becomes the greedy choice at scattered positions; samples end there,
    earlier than their cap, and the bookkeeping follows."""
    import torch
    from oracle import transformer as OT
    cfg = CONFIGS["tiny"].with_(gain_jitter=0.05)
    inp = H.make_inputs(cfg, n=8)
    inp["weights"][0]["head"][cfg.eos_id] *= 4.5
    cap = 40
    actor = H.oracle_models(cfg, inp)[0]
    po = inp["prompt_offsets"]
    prompts = [inp["prompt_tokens"][po[i]:po[i + 1]].tolist() for i in range(8)]
    gen = OT.greedy_generate_cached(actor, prompts, [cap] * 8, cfg.eos_id, stop_at_eos=True)
    lens = np.array([len(g.tokens) for g in gen], np.int32)
    assert lens.min() < cap and len(set(lens.tolist())) > 2, lens          # EOS really ends samples early
    inp["out_len"] = lens
    forced = [np.where(g.margin < H.MARGIN, g.tokens, -1).astype(np.int32) for g in gen]
    with H.GpuStage(cfg, inp, stop_on_eos=True, max_new_cap=cap) as g:
        g.submit(forced, use_forced_len=False)
        model = H.scheduler_model_for(g)
        while not model.generation_done():
            info, want = g.R.rlhf_generate_step(g.ctx), model.generate_step()
            assert (info.n_admitted, info.n_decoded, info.n_active) == (want.n_admitted, want.n_decoded, want.n_active)
            assert g.R.rlhf_retire(g.ctx, g.n).tolist() == model.retire()
            snap = g.snapshot()
            assert snap["active"] == model.active and snap["free"] == model.free
        got = g.results()
    assert got["gen_len"].tolist() == lens.tolist()
    for i, gi in enumerate(gen):
        np.testing.assert_array_equal(H.unpack(got, "tokens")[i], gi.tokens)
        assert np.abs(H.unpack(got, "lp_actor")[i] - gi.logprob).max() <= 1e-4
        assert gi.tokens[-1] == cfg.eos_id or len(gi.tokens) == cap


@pytest.mark.parametrize("which", ["tiny", "gpt2s"])
def test_gae_single_matmul_matches_recursion(which, tiny_ref, gpt2s_ref):
    """Section 6: GAE unrolled into one matrix multiply, against the backward recursion fed with
    the oracle's own log-probs, values and rewards."""
    from oracle.gae import gae, token_rewards
    cfg, ref = tiny_ref if which == "tiny" else gpt2s_ref
    gamma, lam, kl = 0.99, 0.95, 0.1
    with H.GpuStage(cfg, ref) as g:
        g.submit(ref["forced"])
        g.R.rlhf_run_stage(g.ctx, True, g.n + 1, 256, 0b1110)
        res = g.results()
        adv, ret = g.R.rlhf_compute_gae(g.ctx, gamma, lam, kl, int(g.max_new.sum()))
    o = res["resp_offsets"]
    want_a, want_r = [], []
    for i in range(g.n):
        a, r = gae(token_rewards(ref["lp_actor"][i], ref["lp_ref"][i], ref["reward"][i], kl), ref["values"][i], gamma, lam)
        want_a.append(a); want_r.append(r)
    want_a, want_r = np.concatenate(want_a), np.concatenate(want_r)
    got_a, got_r = adv[:o[-1]], ret[:o[-1]]
    if which == "tiny":          # float model: inputs agree to 1e-6, the product adds float32 rounding
        np.testing.assert_allclose(got_a, want_a, rtol=0, atol=2e-5)
        np.testing.assert_allclose(got_r, want_r, rtol=0, atol=2e-5)
    else:                        # bf16 model: the inputs carry the activation rounding of the stage
        assert H.rel_err(got_a, want_a) <= 1e-2 and H.rel_err(got_r, want_r) <= 1e-2


def test_cu_partition_gives_identical_results(gpt2s_ref):
    """Splitting the chip between the two streams while scoring is in flight changes where
    kernels run, not what they compute."""
    cfg, ref = gpt2s_ref
    a = H.run_gpu_stage(cfg, ref, fused=True, R_t=7, chunk_tokens=300)
    b = H.run_gpu_stage(cfg, ref, fused=True, R_t=7, chunk_tokens=300, corun_decode_cus=128)
    H.compare_stage(cfg, ref, b)
    for k in ("tokens", "lp_actor", "lp_ref", "values", "reward", "lp_actor_rescored"):
        np.testing.assert_array_equal(a[k], b[k])
    assert a["snapshot"]["batches"] == b["snapshot"]["batches"]


def test_degenerate_workloads(tiny_ref):
    """Empty batch, a single one-token sample (it ends at its prefill), role subsets, and a
    context reused for a second stage."""
    cfg, ref = tiny_ref
    import paper_2409_13221_amd as R
    with H.GpuStage(cfg, ref) as g:
        # nothing submitted: a stage over zero samples is zero steps
        R.rlhf_submit(g.ctx, np.zeros(0, np.int32), np.zeros(1, np.int64), np.zeros(0, np.int32))
        st, _ = R.rlhf_run_stage(g.ctx, True, 1, 64, H.ALL_ROLES)
        assert (st.n_steps, st.n_batches, st.generated_tokens) == (0, 0, 0)
        assert R.rlhf_get_results(g.ctx, 0, 0)["tokens"].size == 0
        # one sample of length 1: prefill emits the termination token, no decode step follows
        p0 = ref["prompts"][0]
        R.rlhf_submit(g.ctx, np.array(p0, np.int32), np.array([0, len(p0)], np.int64), np.array([1], np.int32),
                      np.array([1], np.int32))
        info = R.rlhf_generate_step(g.ctx)
        assert (info.n_admitted, info.n_decoded) == (1, 0)
        assert R.rlhf_retire(g.ctx, 1).tolist() == [0]
        R.rlhf_score(g.ctx, [0], 0b0110, True)              # Reference and Critic only
        out = R.rlhf_get_results(g.ctx, 1, 1)
        assert out["tokens"].tolist() == [cfg.eos_id] and out["gen_len"].tolist() == [1]
        assert np.isfinite(out["lp_actor"]).all() and np.isfinite(out["lp_ref"]).all() and np.isfinite(out["values"]).all()
        assert np.isnan(out["reward"]).all() and np.isnan(out["lp_actor_rescored"]).all()   # never scored
        # the same context runs the full workload afterwards, twice, with identical results
        g.submit(ref["forced"])
        R.rlhf_run_stage(g.ctx, True, 9, 128, H.ALL_ROLES)
        a = g.results()
        g.submit(ref["forced"])
        R.rlhf_run_stage(g.ctx, True, 9, 128, H.ALL_ROLES)
        b = g.results()
    H.compare_stage(cfg, ref, a)
    for k in ("tokens", "lp_actor", "lp_ref", "values", "reward"):
        np.testing.assert_array_equal(a[k], b[k])


# ------------------------------------------------- exact logit ties, non-finite results

@pytest.mark.parametrize("which", ["tiny", "gpt2s"])
def test_exact_logit_ties_emit_the_lower_id(which):
    """Every odd row of the Actor's LM head is a copy of the even row before it, so every
    position's best logit is an exact tie between ids 2k and 2k + 1.  Both picks (the one after
    prefill, over one logit plane, and the one of a decode step, over split-K planes) must emit
    the even id.  Nothing is teacher-forced; the oracle checks the path by teacher forcing."""
    import copy
    if which == "tiny":
        cfg = CONFIGS["tiny"].with_(gain_jitter=0.05)
        inp = H.make_inputs(cfg, n=6, max_len=14)
    else:
        cfg = CONFIGS["gpt2s"].with_(gain_jitter=0.05)
        inp = H.make_inputs(cfg, n=4, max_len=10, weight_device="cuda")
    inp = dict(inp)
    inp["weights"] = [dict(w) for w in inp["weights"]]
    head = inp["weights"][0]["head"].clone()
    head[1::2] = head[0::2]
    inp["weights"][0]["head"] = head
    with H.GpuStage(cfg, inp) as g:
        g.submit(None)
        g.R.rlhf_run_stage(g.ctx, True, g.n + 1, 64, 0b0001)
        got = g.results()
    toks = H.unpack(got, "tokens")
    assert sum(len(t) for t in toks) == int(inp["out_len"].sum())
    for i, t in enumerate(toks):
        assert np.all(t % 2 == 0), f"sample {i} emitted an odd id: {t}"
        assert t[-1] == cfg.eos_id
    # first tokens come from the prefill pick, the others from decode picks
    assert all(len(t) >= 3 for t in toks)
    H.check_samples_by_teacher_forcing(cfg, inp, got, list(range(g.n)), dtype=np.float64, roles=(0,))


def test_non_finite_results_are_reported():
    """A model whose activations leave the range of the 16-bit path: the stage still runs to its
    end (every kernel stays in bounds), and rlhf_get_results reports RLHF_ENONFINITE."""
    import paper_2409_13221_amd as R
    cfg = CONFIGS["gpt2s"].with_(gain_jitter=0.0)
    inp = H.make_inputs(cfg, n=3, max_len=5, n_layers=2, weight_device="cuda")
    ok = H.run_gpu_stage(cfg, inp, fused=True, R_t=4, chunk_tokens=64)           # finite as drawn
    assert np.isfinite(ok["lp_actor"]).all() and np.isfinite(ok["values"]).all()
    inp = dict(inp)
    inp["weights"] = [dict(w) for w in inp["weights"]]
    inp["weights"][1]["g_final"] = inp["weights"][1]["g_final"] * 1.0e6          # Reference: final-norm rows overflow half
    with H.GpuStage(cfg, inp) as g:
        g.submit(None)
        g.R.rlhf_run_stage(g.ctx, True, g.n + 1, 64, H.ALL_ROLES)
        with pytest.raises(R.RlhfError) as e:
            g.results()
        assert e.value.code == R.RLHF_ENONFINITE
        # the flag belongs to the stage: a new submit clears it
        g.submit(None)
        g.R.rlhf_run_stage(g.ctx, True, g.n + 1, 64, 0b1101)                     # without the Reference
        assert np.isfinite(g.results()["values"]).all()


def test_auto_plan_picks_serial_for_launch_bound_models(tiny_ref, gpt2s_ref):
    """fused = 2 leaves the plan to the library: both small shapes are launch-bound, so it runs
    the serial plan (one scoring pass after generation), with the serial plan's batches."""
    for cfg, ref in (tiny_ref, gpt2s_ref):
        with H.GpuStage(cfg, ref) as g:
            g.submit(ref["forced"])
            model = H.scheduler_model_for(g)
            model.run_stage(False, 0, 64)
            stats, _ = g.R.rlhf_run_stage(g.ctx, "auto", g.n + 1, 64, H.ALL_ROLES)
            assert stats.fused_used == 0
            assert g.snapshot()["batches"] == model.batches
            H.compare_stage(cfg, ref, g.results())


def test_half_weight_copies_do_not_change_results(gpt2s_ref):
    """The engine option that keeps IEEE-half copies of the matrices for prefill / scoring passes:
    the whole GPT-2-small-shape stage (prefill passes of more than 512 rows included) gives
    bit-identical outputs with and without it, and they match the oracle."""
    cfg, ref = gpt2s_ref
    a = H.run_gpu_stage(cfg, ref, fused=True, R_t=7, chunk_tokens=600)
    b = H.run_gpu_stage(cfg, ref, fused=True, R_t=7, chunk_tokens=600, half_weight_copies=True)
    H.compare_stage(cfg, ref, b)
    for k in ("tokens", "lp_actor", "lp_ref", "values", "reward", "lp_actor_rescored"):
        np.testing.assert_array_equal(a[k], b[k])
