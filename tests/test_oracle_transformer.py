"""Pins for oracle/transformer.py: everything here is checked against something other than
the oracle itself -- an independent library implementation of the same decoder, a library
attention routine, scalar brute force, closed forms and invariants.  (The paper prints no
numeric example for this path, so there is no printed value to pin to.)"""
import math

import numpy as np
import pytest
import torch

from oracle import transformer as T
from workload import CONFIGS, make_weights
from workload.configs import ModelCfg


def rand_model(seed, n_layers=2, d=32, hq=4, hkv=4, hd=8, ffn=48, vocab=50, head_rows=None,
               scale=1.0, dtype=np.float64):
    """A small model whose attention is far from uniform (weights ~ N(0, scale^2 / fan_in)
    with a boosted Q/K so that scores spread over several units)."""
    r = np.random.default_rng(seed)
    s = T.Shape(n_layers, d, hq, hkv, hd, ffn, vocab, 1e-5, 10000.0)
    qkv_rows = (hq + 2 * hkv) * hd
    w = {
        "embed": r.normal(0, 1.0, (vocab, d)),
        "wqkv": r.normal(0, 2.0 * scale / math.sqrt(d), (n_layers, qkv_rows, d)),
        "wo": r.normal(0, scale / math.sqrt(hq * hd), (n_layers, d, hq * hd)),
        "w_gate_up": r.normal(0, scale / math.sqrt(d), (n_layers, 2 * ffn, d)),
        "w_down": r.normal(0, scale / math.sqrt(ffn), (n_layers, d, ffn)),
        "g_attn": 1 + 0.2 * r.normal(size=(n_layers, d)),
        "g_mlp": 1 + 0.2 * r.normal(size=(n_layers, d)),
        "g_final": 1 + 0.2 * r.normal(size=(d,)),
        "head": r.normal(0, 1.0 / math.sqrt(d), (vocab if head_rows is None else head_rows, d)),
    }
    return T.Model(s, w, dtype), w, s


# ------------------------------------------------------- independent implementation

def _hf_llama(m, w):
    from transformers import LlamaConfig, LlamaForCausalLM
    hc = LlamaConfig(hidden_size=m.d_model, intermediate_size=m.ffn, num_hidden_layers=m.n_layers,
                     num_attention_heads=m.n_q_heads, num_key_value_heads=m.n_kv_heads,
                     vocab_size=m.vocab, rms_norm_eps=m.rms_eps, rope_theta=m.rope_base,
                     attention_bias=False, mlp_bias=False, tie_word_embeddings=False,
                     head_dim=m.head_dim, max_position_embeddings=1024,
                     attn_implementation="eager")
    hf = LlamaForCausalLM(hc).to(torch.float64).eval()
    qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    sd = {"model.embed_tokens.weight": w["embed"], "model.norm.weight": w["g_final"],
          "lm_head.weight": w["head"]}
    for l in range(m.n_layers):
        p = f"model.layers.{l}."
        sd[p + "self_attn.q_proj.weight"] = w["wqkv"][l, :qd]
        sd[p + "self_attn.k_proj.weight"] = w["wqkv"][l, qd:qd + kvd]
        sd[p + "self_attn.v_proj.weight"] = w["wqkv"][l, qd + kvd:]
        sd[p + "self_attn.o_proj.weight"] = w["wo"][l]
        sd[p + "mlp.gate_proj.weight"] = w["w_gate_up"][l, :m.ffn]
        sd[p + "mlp.up_proj.weight"] = w["w_gate_up"][l, m.ffn:]
        sd[p + "mlp.down_proj.weight"] = w["w_down"][l]
        sd[p + "input_layernorm.weight"] = w["g_attn"][l]
        sd[p + "post_attention_layernorm.weight"] = w["g_mlp"][l]
    sd = {k: torch.as_tensor(np.asarray(v), dtype=torch.float64) for k, v in sd.items()}
    missing, unexpected = hf.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in k or "inv_freq" in k for k in missing), (missing, unexpected)
    return hf


@pytest.mark.parametrize("case", ["tiny_workload", "gqa_sharp"])
def test_forward_matches_independent_llama(case):
    """The whole block structure (pre-norm, rotary pairing and base, GQA head mapping,
    SwiGLU, final norm, untied head) against the transformers library's Llama in float64."""
    if case == "tiny_workload":
        cfg = CONFIGS["tiny"].with_(gain_jitter=0.1)
        m = cfg.model
        w = {k: v.double().numpy() for k, v in make_weights(cfg, 0).items()}
        model = T.Model(T.Shape.of(m), w)
    else:
        model, w, s = rand_model(5, n_layers=3, d=48, hq=6, hkv=2, hd=8, ffn=80, vocab=97)
        m = ModelCfg(s.n_layers, s.d_model, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn,
                     s.vocab, "fp32", s.rms_eps, s.rope_base)
    hf = _hf_llama(m, w)
    toks = np.random.default_rng(1).integers(0, m.vocab, 37)
    with torch.no_grad():
        out = hf(torch.as_tensor(toks)[None, :], output_hidden_states=True)
    H, Z = model.forward_full(toks)
    zr = out.logits[0].numpy()
    assert np.abs(zr).max() > 0.5
    # the library builds its rotary tables in float32, hence 1e-6 rather than 1e-12; any
    # wrong convention (pairing, base, head mapping, norm placement) shows at 1e-1
    np.testing.assert_allclose(Z, zr, rtol=0, atol=2e-6 * max(1.0, np.abs(zr).max()))
    np.testing.assert_allclose(H, out.hidden_states[-1][0].numpy(), rtol=0, atol=2e-5)


def test_attention_matches_library_sdpa():
    r = np.random.default_rng(2)
    Tn, Hq, Hkv, hd = 19, 6, 3, 16
    q, k, v = r.normal(size=(Tn, Hq, hd)), r.normal(size=(Tn, Hkv, hd)), r.normal(size=(Tn, Hkv, hd))
    got = T.attention(q, k, v, np.arange(Tn))
    tq = torch.as_tensor(q).permute(1, 0, 2)[None]
    tk = torch.as_tensor(k).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    tv = torch.as_tensor(v).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0]
    np.testing.assert_allclose(got, ref.permute(1, 0, 2).numpy(), atol=1e-12)


# ------------------------------------------------------------------------ brute force

def test_attention_brute_force_scalar_loops():
    r = np.random.default_rng(3)
    Tn, S, Hq, Hkv, hd = 5, 8, 4, 2, 6
    q, k, v = r.normal(size=(Tn, Hq, hd)), r.normal(size=(S, Hkv, hd)), r.normal(size=(S, Hkv, hd))
    q_pos = np.array([3, 4, 5, 6, 7])           # 5 new queries after 3 cached positions
    got, probs = T.attention(q, k, v, q_pos, return_probs=True)
    for t in range(Tn):
        for h in range(Hq):
            kh = h // (Hq // Hkv)
            sc = []
            for s_ in range(q_pos[t] + 1):
                dot = 0.0
                for e in range(hd):
                    dot += q[t, h, e] * k[s_, kh, e]
                sc.append(dot / math.sqrt(hd))
            mx = max(sc)
            ex = [math.exp(x - mx) for x in sc]
            den = sum(ex)
            for e in range(hd):
                acc = 0.0
                for s_ in range(q_pos[t] + 1):
                    acc += ex[s_] / den * v[s_, kh, e]
                assert abs(acc - got[t, h, e]) < 1e-12
            assert abs(probs[h, t].sum() - 1.0) < 1e-12               # rows sum to 1
            assert np.all(probs[h, t, q_pos[t] + 1:] == 0.0)          # the future is masked


def test_uniform_attention_is_running_mean_of_values():
    """Closed form: with W_q = 0 every visible key scores alike, so position t's attention
    output is the mean of v_0..v_t (catches an off-by-one in the causal mask)."""
    r = np.random.default_rng(4)
    Tn, H, hd = 9, 2, 4
    k, v = r.normal(size=(Tn, H, hd)), r.normal(size=(Tn, H, hd))
    out = T.attention(np.zeros((Tn, H, hd)), k, v, np.arange(Tn))
    want = np.cumsum(v, axis=0) / np.arange(1, Tn + 1)[:, None, None]
    np.testing.assert_allclose(out, want, atol=1e-14)


# ---------------------------------------------------------------- rotary and RMSNorm

def test_rope_closed_forms():
    r = np.random.default_rng(6)
    hd = 16
    q, k = r.normal(size=(1, 1, hd)), r.normal(size=(1, 1, hd))
    assert np.array_equal(T.rope(q, np.array([0]), 10000.0), q)       # position 0: identity
    for m_, n_ in [(5, 3), (40, 17), (1000, 999)]:
        a = np.sum(T.rope(q, np.array([m_]), 10000.0) * T.rope(k, np.array([n_]), 10000.0))
        b = np.sum(T.rope(q, np.array([m_ - n_]), 10000.0) * k)        # relative property
        assert abs(a - b) < 1e-10
    x = r.normal(size=(7, 3, hd))
    y = T.rope(x, np.arange(7) * 13, 10000.0)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), atol=1e-12)
    # hand value: hd = 2 has the single pair (0, 1) turning by pos radians
    y2 = T.rope(np.array([[[1.0, 0.0]]]), np.array([1]), 10000.0)
    np.testing.assert_allclose(y2[0, 0], [math.cos(1.0), math.sin(1.0)], atol=1e-15)
    # pairing is (k, k + hd/2), frequency base^(-2k/hd): hd = 4, pos = 2
    y4 = T.rope(np.array([[[1.0, 1.0, 0.0, 0.0]]]), np.array([2]), 100.0)
    np.testing.assert_allclose(y4[0, 0], [math.cos(2.0), math.cos(0.2), math.sin(2.0), math.sin(0.2)],
                               atol=1e-15)


def test_rmsnorm_properties():
    r = np.random.default_rng(7)
    x = r.normal(size=(5, 64)) * 3.0
    y = T.rmsnorm(x, np.ones(64), 1e-12)
    np.testing.assert_allclose(np.mean(y * y, axis=-1), 1.0, atol=1e-9)
    np.testing.assert_allclose(T.rmsnorm(7.5 * x, np.ones(64), 1e-12), y, atol=1e-9)
    g = r.normal(size=64)
    np.testing.assert_allclose(T.rmsnorm(x, g, 1e-5), T.rmsnorm(x, np.ones(64), 1e-5) * g, atol=1e-14)
    # eps sits inside the square root, added to the mean square: x = (3, 4) -> ms = 12.5
    np.testing.assert_allclose(T.rmsnorm(np.array([3.0, 4.0]), np.ones(2), 0.5),
                               np.array([3.0, 4.0]) / math.sqrt(13.0), atol=1e-15)


# ---------------------------------------------------------------- structure of forward

def test_gqa_equals_mha_on_replicated_heads():
    model, w, s = rand_model(8, hq=4, hkv=2, hd=8)
    qd, kvd = 32, 16
    wq, wk, wv = w["wqkv"][:, :qd], w["wqkv"][:, qd:qd + kvd], w["wqkv"][:, qd + kvd:]
    rep = lambda a: a.reshape(s.n_layers, 2, 8, -1).repeat(2, axis=1).reshape(s.n_layers, 32, -1)
    w2 = dict(w, wqkv=np.concatenate([wq, rep(wk), rep(wv)], axis=1))
    mha = T.Model(T.Shape(s.n_layers, s.d_model, 4, 4, 8, s.ffn, s.vocab), w2)
    toks = np.arange(11) % s.vocab
    np.testing.assert_allclose(model.forward_full(toks)[1], mha.forward_full(toks)[1], atol=1e-12)


def test_zero_layers_and_dead_branches():
    model, w, s = rand_model(9)
    toks = np.array([3, 1, 4, 1, 5])
    want = T.rmsnorm(w["embed"][toks], w["g_final"], s.rms_eps) @ w["head"].T
    m0 = T.Model(T.Shape(0, s.d_model, 4, 4, 8, s.ffn, s.vocab),
                 {k: (v[:0] if v.ndim == 3 or k in ("g_attn", "g_mlp") else v) for k, v in w.items()})
    np.testing.assert_allclose(m0.forward_full(toks)[1], want, atol=1e-13)
    # zero output projections make both residual branches vanish
    dead = T.Model(s, dict(w, wo=np.zeros_like(w["wo"]), w_down=np.zeros_like(w["w_down"])))
    np.testing.assert_allclose(dead.forward_full(toks)[1], want, atol=1e-13)


def test_one_layer_one_head_by_hand():
    """d = 2, one head, identity-like weights, two tokens: every number written out."""
    s = T.Shape(1, 2, 1, 1, 2, 2, 3, 0.0, 10000.0)
    I = np.eye(2)
    w = {"embed": np.array([[1.0, 0.0], [0.0, 2.0], [1.0, 1.0]]),
         "wqkv": np.concatenate([I, I, I])[None], "wo": I[None],
         "w_gate_up": np.concatenate([I, I])[None], "w_down": np.zeros((1, 2, 2)),
         "g_attn": np.ones((1, 2)), "g_mlp": np.ones((1, 2)), "g_final": np.ones(2),
         "head": np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])}
    H, Z = T.Model(s, w).forward_full([0, 1])
    r2 = math.sqrt(2.0)
    # position 0: n1 = (r2, 0); q = k = v = n1 (angle 0); attends to itself: a = (r2, 0)
    h0 = np.array([1.0 + r2, 0.0])
    # position 1: n1 = (0, r2); rotary at pos 1, pair (0,1): q1 = k1 = (-r2 sin1, r2 cos1)
    q1 = np.array([-r2 * math.sin(1.0), r2 * math.cos(1.0)])
    s10 = q1 @ np.array([r2, 0.0]) / r2
    s11 = q1 @ q1 / r2
    p0 = math.exp(s10) / (math.exp(s10) + math.exp(s11))
    a1 = p0 * np.array([r2, 0.0]) + (1 - p0) * np.array([0.0, r2])
    h1 = np.array([0.0, 2.0]) + a1
    for t, h in enumerate((h0, h1)):
        hn = h / math.sqrt(np.mean(h * h))
        np.testing.assert_allclose(H[t], hn, atol=1e-14)
        np.testing.assert_allclose(Z[t], [hn[0], hn[1], hn[0] + hn[1]], atol=1e-14)


def test_causal_prefix_invariance():
    model, _, s = rand_model(10)
    r = np.random.default_rng(0)
    toks = r.integers(0, s.vocab, 20)
    _, Z = model.forward_full(toks)
    other = toks.copy()
    other[12:] = r.integers(0, s.vocab, 8)
    _, Z2 = model.forward_full(other)
    np.testing.assert_array_equal(Z[:12], Z2[:12])
    assert np.abs(Z[12:] - Z2[12:]).max() > 1e-3
    _, Z3 = model.forward_full(toks[:12])
    np.testing.assert_allclose(Z[:12], Z3, atol=1e-12)


# ------------------------------------------------------------- generation and scoring

def test_cached_decode_equals_full_recompute():
    model, _, s = rand_model(11, n_layers=3)
    r = np.random.default_rng(1)
    prompts = [r.integers(3, s.vocab, n).tolist() for n in (5, 9, 1)]
    lens = [7, 1, 4]
    full = [T.greedy_generate(model, p, L, eos_id=2) for p, L in zip(prompts, lens)]
    cached = T.greedy_generate_cached(model, prompts, lens, eos_id=2)
    for a, b, L in zip(full, cached, lens):
        assert len(a.tokens) == L
        np.testing.assert_array_equal(a.tokens, b.tokens)
        np.testing.assert_array_equal(a.greedy, b.greedy)
        np.testing.assert_allclose(a.logprob, b.logprob, atol=1e-12)
        np.testing.assert_allclose(a.margin, b.margin, atol=1e-12)


def test_reprefill_migration_changes_nothing():
    """Section 4.2, second migration mechanism: discarding a sample's KV cache and rebuilding it
    by a prefill over prompt + generated tokens leaves tokens and log-probs as they were."""
    model, _, s = rand_model(13, n_layers=2)
    r = np.random.default_rng(4)
    prompts = [r.integers(3, s.vocab, n).tolist() for n in (6, 3, 8)]
    lens = [9, 5, 2]
    plain = T.greedy_generate_cached(model, prompts, lens, eos_id=2)
    moved = T.greedy_generate_cached(model, prompts, lens, eos_id=2, migrate_after={1: [0, 2], 3: [1, 0], 4: [1]})
    for a, b in zip(plain, moved):
        np.testing.assert_array_equal(a.tokens, b.tokens)
        np.testing.assert_allclose(a.logprob, b.logprob, atol=1e-12)
        np.testing.assert_allclose(a.margin, b.margin, atol=1e-12)


def test_cached_decode_equals_full_recompute_tiny_workload_fp32():
    """The same at the Tiny workload's shape in float32 (tolerance 1e-5)."""
    cfg = CONFIGS["tiny"]
    w = {k: v.numpy() for k, v in make_weights(cfg, 0).items()}
    model = T.Model(T.Shape.of(cfg.model), w, dtype=np.float32)
    prompt = np.random.default_rng(2).integers(3, cfg.model.vocab, 32).tolist()
    a = T.greedy_generate(model, prompt, 6, eos_id=2)
    b = T.greedy_generate_cached(model, [prompt], [6], eos_id=2)[0]
    np.testing.assert_array_equal(a.tokens, b.tokens)
    np.testing.assert_allclose(a.logprob, b.logprob, atol=1e-5)
    m64 = T.Model(T.Shape.of(cfg.model), w, dtype=np.float64)
    c = T.greedy_generate(m64, prompt, 6, eos_id=2, forced=a.tokens)
    np.testing.assert_allclose(a.logprob, c.logprob, atol=1e-4)       # float32 vs float64


def test_generation_semantics():
    model, _, s = rand_model(12)
    prompt = [5, 6, 7, 8]
    g = T.greedy_generate(model, prompt, 6, eos_id=2)
    assert g.tokens[-1] == 2                               # termination token imposed at L
    free = g.tokens[:-1]
    np.testing.assert_array_equal(free, g.greedy[:-1])     # greedy elsewhere
    # the greedy token's log-prob is the row maximum of the log-softmax; probabilities sum to 1
    x = list(prompt)
    for j in range(6):
        _, Z = model.forward_full(x)
        ls = T.log_softmax_rows(Z[-1:])[0]
        assert abs(np.exp(ls).sum() - 1.0) < 1e-12
        if j < 5:
            assert g.logprob[j] == ls.max() and int(np.argmax(ls)) == g.tokens[j]
        else:
            assert abs(g.logprob[j] - ls[2]) < 1e-15       # EOS gets its true log-prob
        top = np.sort(Z[-1])
        assert abs(g.margin[j] - (top[-1] - top[-2])) < 1e-15
        x.append(int(g.tokens[j]))
    # teacher forcing: imposed tokens are followed and are what gets fed back
    forced = np.array([-1, 9, -1, 11, -1, -1])
    f = T.greedy_generate(model, prompt, 6, eos_id=2, forced=forced)
    assert f.tokens[1] == 9 and f.tokens[3] == 11 and f.tokens[0] == g.tokens[0]
    _, Z = model.forward_full(prompt + [int(f.tokens[0]), 9])
    assert f.greedy[2] == int(np.argmax(Z[-1]))
    # lowest index wins a tie
    assert T._pick(np.array([0.0, 3.0, 3.0, 1.0]), -1)[0] == 1


def test_stop_at_eos_semantics():
    """"Until reaching a termination token": with stop_at_eos the response ends at the first
    emitted eos_id; both generation variants agree, and the prefix equals free greedy decoding."""
    model, w, s = rand_model(21)
    prompt = [4, 9, 3]
    free = T.greedy_generate(model, prompt, 12, eos_id=2, stop_at_eos=True)
    # make the free run's 4th token the termination token and generate again
    eos = int(free.tokens[3])
    a = T.greedy_generate(model, prompt, 12, eos_id=eos, stop_at_eos=True)
    first = int(np.argmax(free.tokens == eos))
    assert len(a.tokens) == first + 1 <= 4 and a.tokens[-1] == eos
    np.testing.assert_array_equal(a.tokens, free.tokens[:first + 1])
    b = T.greedy_generate_cached(model, [prompt, prompt], [12, 2], eos, stop_at_eos=True)
    np.testing.assert_array_equal(a.tokens, b[0].tokens)
    assert len(b[1].tokens) == min(2, first + 1)                # the cap still applies, nothing imposed
    np.testing.assert_array_equal(b[1].tokens, free.tokens[:len(b[1].tokens)])


def test_scoring_alignment_and_heads():
    actor, _, s = rand_model(13)
    critic, wc, _ = rand_model(14, head_rows=1)
    reward, wr, _ = rand_model(15, head_rows=1)
    prompt = [4, 9, 3, 7, 7]
    g = T.greedy_generate(actor, prompt, 5, eos_id=2)
    resp = g.tokens.tolist()
    # re-scoring the Actor's own response by one full forward reproduces generation's log-probs
    np.testing.assert_allclose(T.score_logprobs(actor, prompt, resp), g.logprob, atol=1e-12)
    # value[j] is read at position P+j-1: it sees y_1..y_{j-1} but not y_j
    v = T.score_values(critic, prompt, resp)
    assert v.shape == (5,)
    alt = list(resp); alt[2] = (alt[2] + 1) % s.vocab
    v2 = T.score_values(critic, prompt, alt)
    np.testing.assert_array_equal(v[:3], v2[:3])
    assert abs(v[3] - v2[3]) > 1e-6
    H, _ = critic.forward_full(prompt + resp)
    np.testing.assert_allclose(v, H[4:9] @ wc["head"][0], atol=1e-13)
    # reward reads the last token (the imposed EOS)
    Hr, _ = reward.forward_full(prompt + resp)
    assert abs(T.score_reward(reward, prompt, resp) - Hr[-1] @ wr["head"][0]) < 1e-13
    alt = list(resp); alt[-1] = 3
    assert abs(T.score_reward(reward, prompt, alt) - T.score_reward(reward, prompt, resp)) > 1e-6


def test_packed_scoring_equals_alone():
    model, _, s = rand_model(16)
    r = np.random.default_rng(5)
    seqs = [r.integers(0, s.vocab, n).tolist() for n in (7, 3, 12)]
    packed = T.score_packed(model, seqs)
    for x, (H, Z) in zip(seqs, packed):
        H1, Z1 = model.forward_full(x)
        np.testing.assert_allclose(Z, Z1, atol=1e-12)
        np.testing.assert_allclose(H, H1, atol=1e-12)
