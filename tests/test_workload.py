"""The input generators: determinism, ranges, and the closed-form means of the length laws."""
import math
import os

import numpy as np
import pytest
import torch

from workload import CONFIGS, draw_lengths, make_prompts, make_weights, weight_shapes
from workload.generate import normals, stream_key, _mix_py, _mix_t, _s64

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "length_laws.txt")


def _phi(x):
    return 0.5 * (1.0 + math.erf(x / math.sqrt(2.0)))


def closed_form(law, a, b, cap):
    """E[L] = sum_{k=1..cap} P(L >= k) and P(L == cap) for the clamped integer laws."""
    def tail(k):  # P(L >= k), k >= 1
        if k <= 1:
            return 1.0
        if law == "pareto":          # floor(X) >= k  <=>  X >= k, X ~ Pareto(alpha=a, x_min=b)
            return 1.0 if k <= b else (b / k) ** a
        # round(X) >= k  <=>  X >= k - 1/2, X lognormal(mu=a, sigma=b)
        return 1.0 - _phi((math.log(k - 0.5) - a) / b)
    return sum(tail(k) for k in range(1, cap + 1)), tail(cap)


def _golden_rows():
    rows = []
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            name, law, a, b, cap, mean, pcap = line.split()
            rows.append((name, law, float(a), float(b), int(cap), float(mean), float(pcap)))
    return rows


@pytest.mark.parametrize("row", _golden_rows(), ids=lambda r: r[0])
def test_length_law_means(row):
    name, law, a, b, cap, mean, pcap = row
    cfg = CONFIGS[name]
    assert (cfg.length_law, cfg.length_params, cfg.length_cap) == (law, (a, b), cap)
    m, p = closed_form(law, a, b, cap)
    assert abs(m - mean) <= 0.005 * mean + 0.06          # tabulated to 3-4 digits
    assert abs(p - pcap) <= 0.02 * pcap + 5e-5
    L = draw_lengths(cfg, 1_000_000).astype(np.float64)
    assert L.min() >= 1 and L.max() <= cap
    se = L.std() / 1000.0
    assert abs(L.mean() - m) < 5 * se
    assert abs((L == cap).mean() - p) < 5 * math.sqrt(p / 1e6) + 1e-6


def test_long_tail_shape():
    """Section 2.2: the tail is long -- P99.9 is far above the median (for the 7B law,
    more than ten times)."""
    L = draw_lengths(CONFIGS["7b"], 200_000)
    assert np.percentile(L, 99.9) > 10 * np.median(L)


def test_hash_matches_python_ints():
    x = torch.tensor([0, 1, 2, 12345678901234, -1, -(1 << 63)], dtype=torch.int64)
    got = _mix_t(x).tolist()
    want = [_s64(_mix_py(v & ((1 << 64) - 1))) for v in x.tolist()]
    assert got == want


def test_normals_are_position_addressable_and_standard():
    key = stream_key(7, 3)
    a = normals(key, 0, 100_000)
    b = normals(key, 40_000, 1000)
    assert torch.equal(a[40_000:41_000], b)
    assert abs(a.mean().item()) < 0.02 and abs(a.std().item() - 1) < 0.02
    assert abs((a ** 4).mean().item() - 3.0) < 0.15
    assert not torch.equal(a[:1000], normals(stream_key(7, 4), 0, 1000))


def test_prompts_and_weights():
    cfg = CONFIGS["7b"]
    toks, offs = make_prompts(cfg)
    plen = np.diff(offs)
    assert plen.min() >= 128 and plen.max() <= 512 and len(plen) == 256
    assert toks.min() >= 3 and toks.max() < cfg.model.vocab and toks.dtype == np.int32
    t2, o2 = make_prompts(cfg)
    assert np.array_equal(toks, t2) and np.array_equal(offs, o2)

    tiny = CONFIGS["tiny"]
    w0, w0b, w1 = make_weights(tiny, 0), make_weights(tiny, 0), make_weights(tiny, 1)
    for k, shp in weight_shapes(tiny.model, 0).items():
        assert tuple(w0[k].shape) == shp
        assert torch.equal(w0[k], w0b[k])
    assert not torch.equal(w0["wqkv"], w1["wqkv"])
    assert abs(w0["wqkv"].std().item() - 0.02) < 2e-4
    assert torch.all(w0["g_attn"] == 1)
    assert tuple(make_weights(tiny, 2)["head"].shape) == (1, tiny.model.d_model)
    # a layer slice is a prefix of the full stream
    w_slice = make_weights(tiny, 0, n_layers=1)
    assert torch.equal(w_slice["wqkv"][0], w0["wqkv"][0])
    # bf16 configs are rounded once from the same float values
    tb = tiny.with_(model=tiny.model.__class__(**{**tiny.model.__dict__, "dtype": "bf16"}))
    wb = make_weights(tb, 0)
    assert wb["wo"].dtype == torch.bfloat16
    assert torch.equal(wb["wo"], w0["wo"].to(torch.bfloat16))
    assert tiny.model.n_params() == sum(v.numel() for v in w0.values())
