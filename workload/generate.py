"""Counter-based seeded generators for weights, prompts and output lengths.

Every drawn number is a pure function of (seed, stream, element index): a 64-bit
mixing hash of the counter gives two 32-bit uniforms, and a Box-Muller transform in
float64 turns them into a standard normal.  Being position-addressable, any slice of
any tensor can be produced without producing the rest, on the CPU or on the GPU, with
torch integer/float64 elementwise ops (which are this module's only dependency).

Integer draws (prompt tokens, lengths) are always made on the CPU.  Weight tensors may
be made on either device; across devices the float64 log/cos may differ in the last
place, so a test that needs both sides to see identical bytes makes a tensor once and
copies it.
"""
import math
from typing import Dict, Tuple

import numpy as np
import torch

from .configs import ModelCfg, WorkloadCfg

ROLE_NAMES = ("actor", "ref", "critic", "reward")

_M64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB

# stream ids (combined with the seed into a 64-bit key)
_S_PROMPT_LEN, _S_PROMPT_TOK, _S_OUT_LEN = 1, 2, 3
_TENSOR_STREAM = {"embed": 16, "wqkv": 17, "wo": 18, "w_gate_up": 19, "w_down": 20,
                  "g_attn": 21, "g_mlp": 22, "g_final": 23, "head": 24}


def _s64(x: int) -> int:
    """Python int in [0, 2^64) -> the same bits as a signed 64-bit value."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_py(x: int) -> int:
    x = (x + _GAMMA) & _M64
    x = ((x ^ (x >> 30)) * _C1) & _M64
    x = ((x ^ (x >> 27)) * _C2) & _M64
    return x ^ (x >> 31)


def stream_key(seed: int, stream: int) -> int:
    return _mix_py(_mix_py(seed & _M64) ^ ((stream * 0xD1342543DE82EF95) & _M64))


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 bit patterns."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix_t(x: torch.Tensor) -> torch.Tensor:
    x = x + _s64(_GAMMA)
    x = (x ^ _lsr(x, 30)) * _s64(_C1)
    x = (x ^ _lsr(x, 27)) * _s64(_C2)
    return x ^ _lsr(x, 31)


def hash_bits(key: int, start: int, count: int, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """(hi32, lo32) of the hash of counters start .. start+count-1, as int64 in [0, 2^32)."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    h = _mix_t(idx + _s64(key))
    return _lsr(h, 32), h & 0xFFFFFFFF


def normals(key: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """float64 standard normals for counters start .. start+count-1."""
    hi, lo = hash_bits(key, start, count, device)
    u1 = (hi.to(torch.float64) + 1.0) * (2.0 ** -32)        # (0, 1]
    u2 = lo.to(torch.float64) * (2.0 ** -32)                # [0, 1)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def uniforms_open(key: int, start: int, count: int) -> torch.Tensor:
    """float64 uniforms in (0, 1] (CPU)."""
    hi, _ = hash_bits(key, start, count)
    return (hi.to(torch.float64) + 1.0) * (2.0 ** -32)


def uniform_ints(key: int, start: int, count: int, lo: int, hi: int) -> torch.Tensor:
    """int64 uniform in [lo, hi) (CPU), by multiply-shift of the high 32 bits."""
    h, _ = hash_bits(key, start, count)
    return lo + ((h * (hi - lo)) >> 32)


# ----------------------------------------------------------------------------- weights

def weight_shapes(m: ModelCfg, role: int, n_layers: int = None) -> Dict[str, Tuple[int, ...]]:
    """Shapes of one role's tensors, in the layout the C-ABI takes them.

    wqkv rows are the Q heads, then the K heads, then the V heads; w_gate_up rows are the
    gate projection then the up projection.  `head` is the LM head for Actor/Reference and
    a single row (value head, reward head) for Critic/Reward.
    """
    ly = m.n_layers if n_layers is None else n_layers
    head_rows = m.vocab if role in (0, 1) else 1
    return {
        "embed": (m.vocab, m.d_model),
        "wqkv": (ly, m.qkv_rows, m.d_model),
        "wo": (ly, m.d_model, m.q_dim),
        "w_gate_up": (ly, 2 * m.ffn, m.d_model),
        "w_down": (ly, m.d_model, m.ffn),
        "g_attn": (ly, m.d_model),
        "g_mlp": (ly, m.d_model),
        "g_final": (m.d_model,),
        "head": (head_rows, m.d_model),
    }


def _fill_normal(out: torch.Tensor, key: int, std: float, mean: float, chunk: int = 1 << 24):
    flat = out.view(-1)
    n = flat.numel()
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        z = normals(key, s, c, device=out.device)
        flat[s:s + c] = (mean + std * z).to(torch.float32).to(out.dtype)


def make_weights(cfg: WorkloadCfg, role: int, device="cpu", n_layers: int = None,
                 init_std: float = 0.02) -> Dict[str, torch.Tensor]:
    """One role's tensors.  Matrices are i.i.d. N(0, init_std^2), drawn in float64, cast to
    float32 and then (bf16 configs) rounded once to bfloat16; norm gains are float32,
    1 + gain_jitter * z.  The role's seed is cfg.seed + role."""
    m = cfg.model
    tdtype = torch.float32 if m.dtype == "fp32" else torch.bfloat16
    out = {}
    for name, shape in weight_shapes(m, role, n_layers).items():
        key = stream_key(cfg.seed + role, _TENSOR_STREAM[name])
        if name.startswith("g_"):
            t = torch.empty(shape, dtype=torch.float32, device=device)
            if cfg.gain_jitter == 0.0:
                t.fill_(1.0)
            else:
                _fill_normal(t, key, cfg.gain_jitter, 1.0)
        else:
            t = torch.empty(shape, dtype=tdtype, device=device)
            _fill_normal(t, key, init_std, 0.0)
        out[name] = t
    return out


# ------------------------------------------------------------------- prompts and lengths

def draw_lengths(cfg: WorkloadCfg, n: int = None) -> np.ndarray:
    """Output lengths L_i >= 1 (int32).  lognormal: clamp(round(exp(mu + sigma z)), 1, cap);
    pareto: clamp(floor(x_min * u^(-1/alpha)), 1, cap) with u uniform in (0, 1]."""
    n = cfg.n_samples if n is None else n
    key = stream_key(cfg.seed, _S_OUT_LEN)
    a, b = cfg.length_params
    if cfg.length_law == "lognormal":
        z = normals(key, 0, n).numpy()
        raw = np.rint(np.exp(a + b * z))
    elif cfg.length_law == "pareto":
        u = uniforms_open(key, 0, n).numpy()
        raw = np.floor(b * u ** (-1.0 / a))
    else:
        raise ValueError(cfg.length_law)
    return np.clip(raw, 1, cfg.length_cap).astype(np.int32)


def make_prompts(cfg: WorkloadCfg, n: int = None) -> Tuple[np.ndarray, np.ndarray]:
    """(packed prompt tokens int32[sum P], offsets int64[n+1]).  Lengths are uniform on the
    inclusive range cfg.prompt_len; tokens are uniform in [3, vocab)."""
    n = cfg.n_samples if n is None else n
    lo, hi = cfg.prompt_len
    if lo == hi:
        plen = np.full(n, lo, dtype=np.int64)
    else:
        plen = uniform_ints(stream_key(cfg.seed, _S_PROMPT_LEN), 0, n, lo, hi + 1).numpy()
    offs = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(plen, out=offs[1:])
    toks = uniform_ints(stream_key(cfg.seed, _S_PROMPT_TOK), 0, int(offs[-1]), 3, cfg.model.vocab)
    return toks.numpy().astype(np.int32), offs


def make_workload(cfg: WorkloadCfg, n: int = None) -> Dict[str, np.ndarray]:
    toks, offs = make_prompts(cfg, n)
    return {"prompt_tokens": toks, "prompt_offsets": offs, "out_len": draw_lengths(cfg, n)}
