"""Named model shapes and workload recipes.

The five entries mirror the five synthetic configurations this build is measured on:
a Llama-style decoder (pre-norm, rotary, SwiGLU, no biases, untied LM head) used four
times over (Actor, Reference, Critic, Reward = four seeds of one shape), a prompt-length
law and a long-tailed output-length law.  The long tail is the point of the exercise:
the generation stage's length distribution (Section 2.2, Figure 2) is what inter-stage
fusion (Section 4) exploits.
"""
from dataclasses import dataclass, field, replace
from typing import Tuple

BASE_SEED = 20240913
EOS_ID = 2
PAGE_TOKENS = 16


@dataclass(frozen=True)
class ModelCfg:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    dtype: str  # "fp32" or "bf16": storage type of weights / KV cache on the GPU path
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def qkv_rows(self) -> int:
        return self.q_dim + 2 * self.kv_dim

    def n_params(self, head_rows: int = None) -> int:
        """Parameter count of one model (matrices only plus norm gains)."""
        hr = self.vocab if head_rows is None else head_rows
        per_layer = (self.qkv_rows * self.d_model + self.d_model * self.q_dim
                     + 3 * self.d_model * self.ffn + 2 * self.d_model)
        return (self.vocab * self.d_model + self.n_layers * per_layer
                + self.d_model + hr * self.d_model)

    def elem_bytes(self) -> int:
        return 4 if self.dtype == "fp32" else 2

    def decode_weight_bytes(self) -> int:
        """Bytes of weights one decode step must read (no embedding table: one row per
        sample is gathered from it)."""
        per_layer = (self.qkv_rows * self.d_model + self.d_model * self.q_dim
                     + 3 * self.d_model * self.ffn)
        return (self.n_layers * per_layer + self.vocab * self.d_model) * self.elem_bytes()

    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_layers * self.kv_dim * self.elem_bytes()


@dataclass(frozen=True)
class WorkloadCfg:
    name: str
    model: ModelCfg
    n_samples: int
    prompt_len: Tuple[int, int]          # inclusive range, (lo, hi); lo == hi => fixed
    length_law: str                      # "lognormal" or "pareto"
    length_params: Tuple[float, float]   # (mu, sigma) or (alpha, x_min)
    length_cap: int
    page_tokens: int = PAGE_TOKENS
    eos_id: int = EOS_ID
    seed: int = BASE_SEED
    gain_jitter: float = 0.0             # std of (norm gain - 1); 0 => gains are exactly 1

    @property
    def max_ctx(self) -> int:
        return self.prompt_len[1] + self.length_cap

    def with_(self, **kw) -> "WorkloadCfg":
        return replace(self, **kw)


CONFIGS = {
    "tiny": WorkloadCfg(
        name="tiny",
        model=ModelCfg(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64,
                       ffn=688, vocab=4096, dtype="fp32"),
        n_samples=8, prompt_len=(32, 32),
        length_law="lognormal", length_params=(3.0, 0.8), length_cap=64),
    "gpt2s": WorkloadCfg(
        name="gpt2s",
        model=ModelCfg(n_layers=12, d_model=768, n_q_heads=12, n_kv_heads=12, head_dim=64,
                       ffn=2048, vocab=32000, dtype="bf16"),
        n_samples=64, prompt_len=(256, 256),
        length_law="lognormal", length_params=(4.8, 1.0), length_cap=1024),
    "7b": WorkloadCfg(
        name="7b",
        model=ModelCfg(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=32, head_dim=128,
                       ffn=11008, vocab=32000, dtype="bf16"),
        n_samples=256, prompt_len=(128, 512),
        length_law="pareto", length_params=(1.5, 64.0), length_cap=2048),
    "13b": WorkloadCfg(
        name="13b",
        model=ModelCfg(n_layers=40, d_model=5120, n_q_heads=40, n_kv_heads=40, head_dim=128,
                       ffn=13824, vocab=32000, dtype="bf16"),
        n_samples=32, prompt_len=(512, 512),
        length_law="pareto", length_params=(1.2, 128.0), length_cap=4096),
    "70b_slice": WorkloadCfg(
        name="70b_slice",
        model=ModelCfg(n_layers=10, d_model=8192, n_q_heads=64, n_kv_heads=8, head_dim=128,
                       ffn=28672, vocab=32000, dtype="bf16"),
        n_samples=128, prompt_len=(1024, 1024),
        length_law="lognormal", length_params=(6.0, 1.0), length_cap=4096),
}


def get_config(name: str) -> WorkloadCfg:
    if name not in CONFIGS:
        raise KeyError(f"unknown workload {name!r}; have {sorted(CONFIGS)}")
    return CONFIGS[name]
