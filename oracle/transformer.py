"""Plain numpy decoder-only transformer: generation and scoring of ONE sample at a time.

TEST INFRASTRUCTURE ONLY -- see the package docstring.

The paper takes the model as given ("LLaMA"); the block below is the reading this build
fixes: pre-norm residual block, RMSNorm with float statistics, rotary embedding pairing
dimension k with k + hd/2, causal softmax attention scaled by 1/sqrt(hd) with grouped KV
heads, SwiGLU MLP, no biases, untied LM head.  Critic and Reward replace the LM head by a
single row applied to the final-norm hidden state.

What is computed (Section 2.1):
  Generation stage -- prefill over the prompt gives the first output token; each decoding
  step appends one token chosen greedily (lowest id on ties) until the termination point.
  Inference stage -- Reference / Critic / Reward each run one causal forward over
  prompt + response; per-token log-probabilities, per-token values, one scalar reward.

All arithmetic is in `dtype` (float64 by default).  Weights arrive already rounded to the
storage precision of the GPU path and are only upcast here.
"""
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np


# --------------------------------------------------------------------------- primitives

def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """y = x * rsqrt(mean(x^2) + eps) * g, over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding.  x: [T, H, hd]; pos: [T] absolute positions (0 = first prompt
    token).  Pair (k, k + hd/2) is rotated by angle pos * base^(-2k/hd)."""
    hd = x.shape[-1]
    half = hd // 2
    k = np.arange(half, dtype=np.float64)
    ang = pos.astype(np.float64)[:, None] * base ** (-2.0 * k / hd)[None, :]   # [T, half]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def softmax_rows(s: np.ndarray) -> np.ndarray:
    s = s - np.max(s, axis=-1, keepdims=True)
    e = np.exp(s)
    return e / np.sum(e, axis=-1, keepdims=True)


def log_softmax_rows(z: np.ndarray) -> np.ndarray:
    m = np.max(z, axis=-1, keepdims=True)
    return z - m - np.log(np.sum(np.exp(z - m), axis=-1, keepdims=True))


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_pos: np.ndarray,
              return_probs: bool = False):
    """Causal attention.  q: [T, Hq, hd] for queries at absolute positions q_pos [T];
    k, v: [S, Hkv, hd] for keys at positions 0..S-1.  Query head h reads KV head
    h // (Hq / Hkv).  Key s is visible to query t iff s <= q_pos[t].  Returns [T, Hq, hd]."""
    T, Hq, hd = q.shape
    S, Hkv, _ = k.shape
    group = Hq // Hkv
    visible = np.arange(S)[None, :] <= q_pos[:, None]                          # [T, S]
    out = np.empty_like(q)
    probs = np.empty((Hq, T, S), dtype=q.dtype) if return_probs else None
    for h in range(Hq):
        kh = h // group
        s = (q[:, h, :] @ k[:, kh, :].T) / np.sqrt(np.asarray(hd, dtype=q.dtype))
        s = np.where(visible, s, -np.inf)
        p = softmax_rows(s)
        out[:, h, :] = p @ v[:, kh, :]
        if return_probs:
            probs[h] = p
    return (out, probs) if return_probs else out


def silu(a: np.ndarray) -> np.ndarray:
    return a / (1.0 + np.exp(-a))


# -------------------------------------------------------------------------------- model

@dataclass
class Shape:
    """Model dimensions (duck-typed copy of whatever config object the caller has)."""
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    @classmethod
    def of(cls, m, n_layers: Optional[int] = None) -> "Shape":
        return cls(m.n_layers if n_layers is None else n_layers, m.d_model, m.n_q_heads,
                   m.n_kv_heads, m.head_dim, m.ffn, m.vocab, m.rms_eps, m.rope_base)


class Model:
    """One role's weights, upcast to the oracle's working precision.

    `weights` maps names to arrays in the generator's layout: embed [V,d]; wqkv
    [Ly, (Hq+2Hkv)*hd, d] with Q rows, then K rows, then V rows; wo [Ly, d, Hq*hd];
    w_gate_up [Ly, 2f, d] with gate rows then up rows; w_down [Ly, d, f]; g_attn, g_mlp
    [Ly, d]; g_final [d]; head [V, d] (LM head) or [1, d] (value / reward head)."""

    def __init__(self, shape: Shape, weights: Dict[str, np.ndarray], dtype=np.float64):
        self.s = shape
        self.dtype = dtype
        w = {k: np.asarray(a, dtype=dtype) for k, a in weights.items()}
        s = shape
        qd, kvd = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
        self.embed = w["embed"]
        self.wq = w["wqkv"][:, :qd, :]
        self.wk = w["wqkv"][:, qd:qd + kvd, :]
        self.wv = w["wqkv"][:, qd + kvd:, :]
        self.wo = w["wo"]
        self.wg = w["w_gate_up"][:, :s.ffn, :]
        self.wu = w["w_gate_up"][:, s.ffn:, :]
        self.wd = w["w_down"]
        self.g_attn, self.g_mlp, self.g_final = w["g_attn"], w["g_mlp"], w["g_final"]
        self.head = w["head"]

    # -- the definition: one causal forward over a whole sequence, nothing cached
    def forward_full(self, tokens: Sequence[int]):
        """Returns (H, Z): final-norm hidden states [T, d] and head outputs [T, rows]."""
        s = self.s
        tok = np.asarray(tokens, dtype=np.int64)
        T = tok.shape[0]
        pos = np.arange(T)
        h = self.embed[tok].copy()
        for l in range(s.n_layers):
            n1 = rmsnorm(h, self.g_attn[l], s.rms_eps)
            q = rope((n1 @ self.wq[l].T).reshape(T, s.n_q_heads, s.head_dim), pos, s.rope_base)
            k = rope((n1 @ self.wk[l].T).reshape(T, s.n_kv_heads, s.head_dim), pos, s.rope_base)
            v = (n1 @ self.wv[l].T).reshape(T, s.n_kv_heads, s.head_dim)
            a = attention(q, k, v, pos).reshape(T, -1)
            h = h + a @ self.wo[l].T
            n2 = rmsnorm(h, self.g_mlp[l], s.rms_eps)
            h = h + (silu(n2 @ self.wg[l].T) * (n2 @ self.wu[l].T)) @ self.wd[l].T
        H = rmsnorm(h, self.g_final, s.rms_eps)
        return H, H @ self.head.T

    # -- second implementation: incremental forward with a per-sequence KV cache
    def new_cache(self) -> "KVCache":
        return KVCache([None] * self.s.n_layers, [None] * self.s.n_layers, 0)

    def forward_incremental(self, caches: List["KVCache"], new_tokens: List[Sequence[int]]):
        """Feed new_tokens[i] (>= 1 token) to sequence i, whose cache holds its earlier
        positions.  Projections of all sequences' new tokens go through one matmul (rows
        are independent); attention is per sequence over its own cache.  Returns (H, Z) for
        the new tokens only, rows in sequence order, and extends the caches."""
        s = self.s
        lens = [len(t) for t in new_tokens]
        tok = np.concatenate([np.asarray(t, dtype=np.int64) for t in new_tokens])
        pos = np.concatenate([c.length + np.arange(n) for c, n in zip(caches, lens)])
        offs = np.concatenate([[0], np.cumsum(lens)])
        Ttot = tok.shape[0]
        h = self.embed[tok].copy()
        for l in range(s.n_layers):
            n1 = rmsnorm(h, self.g_attn[l], s.rms_eps)
            q = rope((n1 @ self.wq[l].T).reshape(Ttot, s.n_q_heads, s.head_dim), pos, s.rope_base)
            k = rope((n1 @ self.wk[l].T).reshape(Ttot, s.n_kv_heads, s.head_dim), pos, s.rope_base)
            v = (n1 @ self.wv[l].T).reshape(Ttot, s.n_kv_heads, s.head_dim)
            a = np.empty((Ttot, s.n_q_heads, s.head_dim), dtype=self.dtype)
            for i, c in enumerate(caches):
                lo, hi = offs[i], offs[i + 1]
                c.k[l] = k[lo:hi] if c.k[l] is None else np.concatenate([c.k[l], k[lo:hi]])
                c.v[l] = v[lo:hi] if c.v[l] is None else np.concatenate([c.v[l], v[lo:hi]])
                a[lo:hi] = attention(q[lo:hi], c.k[l], c.v[l], pos[lo:hi])
            h = h + a.reshape(Ttot, -1) @ self.wo[l].T
            n2 = rmsnorm(h, self.g_mlp[l], s.rms_eps)
            h = h + (silu(n2 @ self.wg[l].T) * (n2 @ self.wu[l].T)) @ self.wd[l].T
        for c, n in zip(caches, lens):
            c.length += n
        H = rmsnorm(h, self.g_final, s.rms_eps)
        return H, H @ self.head.T


@dataclass
class KVCache:
    k: list
    v: list
    length: int


# --------------------------------------------------------------------------- generation

@dataclass
class Generated:
    tokens: np.ndarray    # [L] emitted tokens y_1..y_L
    logprob: np.ndarray   # [L] Actor log-prob of each emitted token
    margin: np.ndarray    # [L] top-1 minus top-2 logit at the position that chose y_j
    greedy: np.ndarray    # [L] the argmax token at each position (before any override)


def _pick(z: np.ndarray, override: int):
    """Greedy choice on one logit row: (emitted token, its log-prob, margin, argmax)."""
    y_star = int(np.argmax(z))                    # numpy returns the lowest index on ties
    top2 = np.partition(z, -2)[-2:]
    y = y_star if override < 0 else int(override)
    lp = log_softmax_rows(z[None, :])[0, y]
    return y, lp, float(top2[1] - top2[0]), y_star


def _override(j: int, out_len: int, eos_id: int, forced: Optional[Sequence[int]],
              impose_eos: bool = True) -> int:
    """Token imposed at output index j (1-based), or -1.  The termination token is imposed
    at j = out_len (unless impose_eos is off: then out_len is only a cap); `forced` (teacher
    forcing, -1 = free) may impose earlier ones."""
    if j == out_len and impose_eos:
        return eos_id
    if forced is not None and forced[j - 1] >= 0:
        return int(forced[j - 1])
    return -1


def greedy_generate(actor: Model, prompt: Sequence[int], out_len: int, eos_id: int,
                    forced: Optional[Sequence[int]] = None, stop_at_eos: bool = False) -> Generated:
    """Generation of one sample by full recompute: every step runs the whole sequence
    through the Actor and reads the last position (Section 2.1, Generation stage).
    Default: the sample has exactly out_len tokens, the last one imposed to be eos_id (the
    synthetic workloads' termination rule).  stop_at_eos: generation runs "until reaching a
    termination token" -- it ends when eos_id is emitted, out_len is only a cap and nothing is
    imposed there."""
    x = list(int(t) for t in prompt)
    toks, lps, margins, greedy = [], [], [], []
    for j in range(1, out_len + 1):
        _, Z = actor.forward_full(x)
        y, lp, mg, ys = _pick(Z[-1], _override(j, out_len, eos_id, forced, not stop_at_eos))
        toks.append(y); lps.append(lp); margins.append(mg); greedy.append(ys)
        x.append(y)
        if stop_at_eos and y == eos_id:
            break
    return Generated(np.array(toks, np.int32), np.array(lps, actor.dtype),
                     np.array(margins, actor.dtype), np.array(greedy, np.int32))


def greedy_generate_cached(actor: Model, prompts: List[Sequence[int]], out_lens: Sequence[int],
                           eos_id: int, forced: Optional[List[Optional[Sequence[int]]]] = None,
                           stop_at_eos: bool = False,
                           migrate_after: Optional[dict] = None) -> List[Generated]:
    """The same results by prefill + KV-cached decoding steps, all samples advanced in
    lock step (sample i drops out after out_lens[i] tokens).  Equal to `greedy_generate`
    per sample; this is the variant that is affordable beyond toy sizes.

    migrate_after = {j: [ids]}: after output index j, the listed unfinished samples are
    migrated by the second mechanism of Section 4.2 ("Migration mechanism"): their KV cache
    is discarded, only their tokens are kept, and the cache is regenerated by rerunning the
    prefill over prompt + generated tokens before generation goes on."""
    n = len(prompts)
    forced = forced if forced is not None else [None] * n
    caches = [actor.new_cache() for _ in range(n)]
    rec = [([], [], [], []) for _ in range(n)]
    feed = [list(int(t) for t in p) for p in prompts]
    live = list(range(n))
    j = 1
    while live:
        _, Z = actor.forward_incremental([caches[i] for i in live], [feed[i] for i in live])
        ends = np.cumsum([len(feed[i]) for i in live]) - 1
        nxt = []
        for row, i in zip(ends, live):
            y, lp, mg, ys = _pick(Z[row], _override(j, out_lens[i], eos_id, forced[i], not stop_at_eos))
            for lst, val in zip(rec[i], (y, lp, mg, ys)):
                lst.append(val)
            feed[i] = [y]
            if j < out_lens[i] and not (stop_at_eos and y == eos_id):
                nxt.append(i)
        for i in (migrate_after or {}).get(j, []):
            if i in nxt:
                caches[i] = actor.new_cache()
                feed[i] = [int(t) for t in prompts[i]] + [int(t) for t in rec[i][0]]
        live = nxt
        j += 1
    return [Generated(np.array(t, np.int32), np.array(lp, actor.dtype),
                      np.array(mg, actor.dtype), np.array(g, np.int32)) for t, lp, mg, g in rec]


# ------------------------------------------------------------------------------ scoring

def score_logprobs(model: Model, prompt: Sequence[int], response: Sequence[int]) -> np.ndarray:
    """Actor/Reference scoring from one causal forward over prompt + response: for
    j = 1..L, lp[j] = log_softmax(z)[y_j] with z the logits at the position just before
    y_j (0-based row P+j-2 of Z: the last prompt token predicts y_1)."""
    P, L = len(prompt), len(response)
    _, Z = model.forward_full(list(prompt) + list(response))
    ls = log_softmax_rows(Z[P - 1:P + L - 1])
    return ls[np.arange(L), np.asarray(response, dtype=np.int64)]


def score_values(critic: Model, prompt: Sequence[int], response: Sequence[int]) -> np.ndarray:
    """Critic: value[j] = <w_v, H[row]> at the same row that predicts y_j (0-based P+j-2),
    i.e. the value of the state before y_j is chosen; j = 1..L."""
    P, L = len(prompt), len(response)
    _, Z = critic.forward_full(list(prompt) + list(response))
    return Z[P - 1:P + L - 1, 0]


def score_reward(reward: Model, prompt: Sequence[int], response: Sequence[int]) -> float:
    """Reward: <w_r, H[T-1]> at the last token of prompt + response."""
    _, Z = reward.forward_full(list(prompt) + list(response))
    return Z[-1, 0]


def score_packed(model: Model, seqs: List[Sequence[int]]):
    """Forward over several sequences at once (projections batched, attention per
    sequence).  Must equal `forward_full` sequence by sequence; returns lists (H_i, Z_i)."""
    caches = [model.new_cache() for _ in seqs]
    H, Z = model.forward_incremental(caches, seqs)
    offs = np.concatenate([[0], np.cumsum([len(x) for x in seqs])])
    return [(H[offs[i]:offs[i + 1]], Z[offs[i]:offs[i + 1]]) for i in range(len(seqs))]
