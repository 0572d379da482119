"""Row-wise kernels through the C ABI (include/rlhf_ops.h) against the oracle's primitives:
RMSNorm fused with the residual add, rotary + KV append, SwiGLU, the greedy pick (with exact
ties), the log-softmax gather, the value / reward head."""
import numpy as np
import pytest
import torch

from oracle import transformer as OT

pytestmark = pytest.mark.gpu

TDT = {"fp32": torch.float32, "bf16": torch.bfloat16, "half": torch.float16}
ROUND = {"fp32": 1e-6, "bf16": 2.0 ** -8, "half": 2.0 ** -11}     # unit roundoff of the output type


def _R():
    import paper_2409_13221_amd as R
    return R


@pytest.mark.parametrize("act", ["fp32", "bf16", "half"])
@pytest.mark.parametrize("rows,d,nsplit", [(1, 256, 0), (5, 768, 1), (3, 4096, 4), (2, 5120, 3), (4, 8192, 16),
                                           (70, 1032, 5)])
def test_rmsnorm_with_residual_planes(act, rows, d, nsplit):
    R = _R()
    r = np.random.default_rng(rows * 31 + d + nsplit)
    h = r.normal(size=(rows, d)).astype(np.float32)
    part = (r.normal(size=(max(nsplit, 1), rows, d)) * 0.3).astype(np.float32)
    g = (1.0 + 0.1 * r.normal(size=d)).astype(np.float32)
    eps = 1e-5
    v = h.astype(np.float64) + (part[:nsplit].astype(np.float64).sum(0) if nsplit else 0.0)
    want = OT.rmsnorm(v, g.astype(np.float64), eps)
    hd, pd, gd = torch.from_numpy(h).cuda(), torch.from_numpy(part).cuda(), torch.from_numpy(g).cuda()
    xn = torch.full((rows, d), float("nan"), device="cuda", dtype=TDT[act])
    R.rlhf_op_rmsnorm(hd, pd[:nsplit] if nsplit else None, gd, xn, eps)
    torch.cuda.synchronize()
    got = xn.double().cpu().numpy()
    np.testing.assert_allclose(got, want, rtol=2 * ROUND[act], atol=1e-6)
    # the residual stream now holds the sum (float)
    np.testing.assert_allclose(hd.double().cpu().numpy(), v, rtol=0, atol=2e-6 * (nsplit + 1))


def test_rmsnorm_selected_rows_leave_the_stream_alone():
    R = _R()
    r = np.random.default_rng(3)
    rows_h, d = 9, 512
    h = r.normal(size=(rows_h, d)).astype(np.float32)
    part = r.normal(size=(2, rows_h, d)).astype(np.float32)
    g = np.ones(d, np.float32)
    sel = np.array([7, 0, 3], np.int32)
    hd = torch.from_numpy(h).cuda()
    xn = torch.zeros(3, d, device="cuda")
    R.rlhf_op_rmsnorm(hd, torch.from_numpy(part).cuda(), torch.from_numpy(g).cuda(), xn, 1e-5,
                      row_idx=torch.from_numpy(sel).cuda())
    torch.cuda.synchronize()
    v = h.astype(np.float64) + part.astype(np.float64).sum(0)
    np.testing.assert_allclose(xn.double().cpu().numpy(), OT.rmsnorm(v[sel], g.astype(np.float64), 1e-5), rtol=3e-6,
                               atol=1e-6)
    np.testing.assert_array_equal(hd.cpu().numpy(), h)


@pytest.mark.parametrize("act,Hq,Hkv,hd", [("fp32", 4, 4, 64), ("half", 8, 2, 128), ("bf16", 3, 3, 64),
                                           ("half", 32, 32, 128)])
@pytest.mark.parametrize("nsplit", [1, 4])
def test_rope_kv_append(act, Hq, Hkv, hd, nsplit):
    R = _R()
    r = np.random.default_rng(Hq * 5 + hd + nsplit)
    rows, n_layers, layer, n_pages, max_pos = 6, 2, 1, 5, 300
    width = (Hq + 2 * Hkv) * hd
    planes = r.normal(size=(nsplit, rows, width)).astype(np.float32)
    pos = np.array([0, 1, 17, 299, 64, 5], np.int32)
    slots = r.permutation(n_pages * 16)[:rows].astype(np.int32)
    k_ = np.arange(hd // 2, dtype=np.float64)
    ang = np.arange(max_pos, dtype=np.float64)[:, None] * 10000.0 ** (-2.0 * k_ / hd)[None, :]
    table = np.stack([np.cos(ang), np.sin(ang)], -1).astype(np.float32)
    x = planes.astype(np.float64).sum(0)
    q_want = OT.rope(x[:, :Hq * hd].reshape(rows, Hq, hd), pos, 10000.0).reshape(rows, -1)
    k_want = OT.rope(x[:, Hq * hd:(Hq + Hkv) * hd].reshape(rows, Hkv, hd), pos, 10000.0).reshape(rows, -1)
    v_want = x[:, (Hq + Hkv) * hd:]
    t = TDT[act]
    q = torch.zeros(rows, Hq * hd, device="cuda", dtype=t)
    k = torch.zeros(rows, Hkv * hd, device="cuda", dtype=t)
    v = torch.zeros(rows, Hkv * hd, device="cuda", dtype=t)
    pool = torch.zeros(n_pages, n_layers, 2, Hkv, 16, hd, device="cuda", dtype=t)
    R.rlhf_op_rope_kv(torch.from_numpy(planes).cuda(), torch.from_numpy(pos).cuda(), torch.from_numpy(table).cuda(),
                      q, k, v, pool, torch.from_numpy(slots).cuda(), layer, n_layers, Hq, Hkv, hd)
    torch.cuda.synchronize()
    tol = dict(rtol=2 * ROUND[act], atol=2e-5 * nsplit)
    np.testing.assert_allclose(q.double().cpu().numpy(), q_want, **tol)
    np.testing.assert_allclose(k.double().cpu().numpy(), k_want, **tol)
    np.testing.assert_allclose(v.double().cpu().numpy(), v_want, **tol)
    pc = pool.double().cpu().numpy()
    for rr in range(rows):
        pg, off = divmod(int(slots[rr]), 16)
        np.testing.assert_allclose(pc[pg, layer, 0, :, off, :].reshape(-1), k_want[rr], **tol)
        np.testing.assert_allclose(pc[pg, layer, 1, :, off, :].reshape(-1), v_want[rr], **tol)
    assert not pc[:, 0].any()                      # the other layer is untouched


@pytest.mark.parametrize("act", ["fp32", "bf16", "half"])
@pytest.mark.parametrize("rows,ffn,nsplit", [(1, 688, 1), (7, 2048, 3), (33, 11008, 2)])
def test_swiglu(act, rows, ffn, nsplit):
    R = _R()
    r = np.random.default_rng(rows + ffn)
    gu = (r.normal(size=(nsplit, rows, 2 * ffn)) * 1.5).astype(np.float32)
    x = gu.astype(np.float64).sum(0)
    want = OT.silu(x[:, :ffn]) * x[:, ffn:]
    actb = torch.zeros(rows, ffn, device="cuda", dtype=TDT[act])
    R.rlhf_op_swiglu(torch.from_numpy(gu).cuda(), actb)
    torch.cuda.synchronize()
    np.testing.assert_allclose(actb.double().cpu().numpy(), want, rtol=2 * ROUND[act] + 2e-6, atol=1e-5)


def _pick_case(logits64, forced):
    """Oracle side of the greedy pick on summed logits."""
    toks, lps = [], []
    for r_ in range(logits64.shape[0]):
        y, lp, _, _ = OT._pick(logits64[r_], -1 if forced is None else int(forced[r_]))
        toks.append(y); lps.append(lp)
    return np.array(toks), np.array(lps)


@pytest.mark.parametrize("vocab,nsplit", [(4096, 1), (32000, 1), (32000, 4), (1000, 2), (37, 1)])
def test_pick_greedy_with_exact_ties_takes_the_lowest_id(vocab, nsplit):
    """Exact ties inside a column chunk of the first stage, across chunks, between the first and
    the last id, and ties that exist only after the split planes are summed."""
    R = _R()
    r = np.random.default_rng(vocab + nsplit)
    rows = 9
    # multiples of 1/8 keep every partial sum exact in float, so ties survive the summation
    planes = (r.integers(-40, 40, size=(nsplit, rows, vocab)) / 8.0).astype(np.float32)
    tot = planes.astype(np.float64).sum(0)
    top = tot.max() + 1.0
    chunk = -(-vocab // 32)

    def plant(row, ids):
        for i in ids:
            planes[0, row, i] += np.float32(top - tot[row, i])
    plant(0, [vocab - 1, 0])                               # first and last id
    plant(1, [min(chunk + 1, vocab - 1), min(chunk + 2, vocab - 1)])          # same chunk
    plant(2, [min(5 * chunk + 3, vocab - 1), min(2 * chunk, vocab - 1), vocab - 2])   # three chunks
    plant(3, [vocab // 2, vocab // 2 - 1])
    plant(4, list(range(0, vocab, max(1, vocab // 50))))   # many
    tot = planes.astype(np.float64).sum(0)
    forced = np.full(rows, -1, np.int32)
    forced[6] = vocab - 1                                  # an imposed token gets its true log-prob
    forced[7] = 2
    want_tok, want_lp = _pick_case(tot, forced)
    assert want_tok[0] == 0 and want_tok[2] == min(2 * chunk, vocab - 1) and want_tok[4] == 0
    lg = torch.from_numpy(planes).cuda()
    tokens = torch.full((rows * 2,), -7, dtype=torch.int32, device="cuda")
    lp = torch.zeros(rows * 2, device="cuda")
    dst = torch.arange(rows, dtype=torch.int32, device="cuda") * 2 + 1
    picked = torch.zeros(rows, dtype=torch.int32, device="cuda")
    R.rlhf_op_pick(lg, torch.from_numpy(forced).cuda(), tokens, dst, lp, dst, picked)
    torch.cuda.synchronize()
    got_tok = tokens.cpu().numpy()[1::2]
    np.testing.assert_array_equal(got_tok, want_tok)
    np.testing.assert_array_equal(picked.cpu().numpy(), want_tok)
    np.testing.assert_array_equal(tokens.cpu().numpy()[0::2], -7)
    np.testing.assert_allclose(lp.cpu().numpy()[1::2], want_lp, rtol=0, atol=1e-4)


@pytest.mark.parametrize("vocab,nsplit", [(32000, 1), (4096, 3)])
def test_gather_logprob(vocab, nsplit):
    R = _R()
    r = np.random.default_rng(vocab)
    rows = 11
    planes = (r.normal(size=(nsplit, rows, vocab)) * 2.0).astype(np.float32)
    tokens = r.integers(0, vocab, size=40).astype(np.int32)
    target = r.integers(0, 40, size=rows).astype(np.int32)
    ls = OT.log_softmax_rows(planes.astype(np.float64).sum(0))
    want = ls[np.arange(rows), tokens[target]]
    out = torch.zeros(rows + 3, device="cuda")
    dst = torch.from_numpy(r.permutation(rows + 3)[:rows].astype(np.int32)).cuda()
    R.rlhf_op_gather_lp(torch.from_numpy(planes).cuda(), torch.from_numpy(tokens).cuda(),
                        torch.from_numpy(target).cuda(), out, dst)
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy()[dst.cpu().numpy()], want, rtol=0, atol=1e-4)


@pytest.mark.parametrize("act,wdt", [("fp32", "fp32"), ("fp32", "bf16"), ("half", "bf16"), ("bf16", "bf16")])
def test_value_head_dot(act, wdt):
    R = _R()
    r = np.random.default_rng(9)
    rows, d = 13, 4096
    xn = torch.from_numpy(r.normal(size=(rows, d)).astype(np.float32)).to(TDT[act]).cuda()
    w = torch.from_numpy((r.normal(size=d) * 0.02).astype(np.float32)).to(TDT[wdt]).cuda()
    want = xn.double().cpu().numpy() @ w.double().cpu().numpy()
    out = torch.zeros(rows, device="cuda")
    R.rlhf_op_head_dot(xn, w, out, torch.arange(rows, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=0, atol=2e-5)


def test_gemm_half_activations_near_the_top_of_the_range():
    """Activations close to IEEE half's largest finite value (65504): products and sums are taken
    in float, so the result is finite and exact to float accumulation."""
    R = _R()
    r = np.random.default_rng(4)
    M, N, K = 16, 256, 512
    a = (r.choice([-1.0, 1.0], size=(M, K)) * r.uniform(3.0e4, 6.5e4, size=(M, K))).astype(np.float32)
    A = torch.from_numpy(a).half().cuda()
    assert torch.isfinite(A).all() and float(A.abs().max()) > 6.0e4
    W = torch.from_numpy((r.normal(size=(N, K)) * 0.02).astype(np.float32)).to(torch.bfloat16).cuda()
    want = A.double().cpu().numpy() @ W.double().cpu().numpy().T
    out = torch.zeros(1, M, N, device="cuda")
    R.rlhf_op_gemm(A, W, out, 1)
    torch.cuda.synchronize()
    got = out[0].double().cpu().numpy()
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-6 * np.abs(want).max() * np.sqrt(K))


@pytest.mark.parametrize("act", ["half", "bf16"])
@pytest.mark.parametrize("M,vocab,K", [(1, 32000, 768), (300, 32000, 512), (700, 2048, 512), (130, 1000, 64),
                                       (515, 4100, 128)])
def test_lm_head_fused_with_logsoftmax_gather(act, M, vocab, K):
    """The scoring pass's LM head with the log-softmax gather in the GEMM epilogue (logits are
    never written) against the oracle's log_softmax over float64 logits of the same inputs;
    vocabularies that fill whole 256-column tiles, part of one, and part of a 128-column half."""
    R = _R()
    r = np.random.default_rng(M + vocab + K)
    A = torch.from_numpy(r.normal(size=(M, K)).astype(np.float32)).to(TDT[act]).cuda()
    W = torch.from_numpy((r.normal(size=(vocab, K)) * 0.05).astype(np.float32)).to(torch.bfloat16).cuda()
    tokens = r.integers(0, vocab, size=2 * M + 5).astype(np.int32)
    tokens[:4] = [0, vocab - 1, min(255, vocab - 1), min(256, vocab - 1)]
    target = r.permutation(2 * M + 5)[:M].astype(np.int32)
    target[:min(4, M)] = np.arange(min(4, M))
    z = A.double().cpu().numpy() @ W.double().cpu().numpy().T
    want = OT.log_softmax_rows(z)[np.arange(M), tokens[target]]
    out = torch.full((M + 2,), float("nan"), device="cuda")
    dst = torch.from_numpy(r.permutation(M + 2)[:M].astype(np.int32)).cuda()
    keep = R.rlhf_op_lm_head_logprob(A, W, torch.from_numpy(tokens).cuda(), torch.from_numpy(target).cuda(), out, dst)
    torch.cuda.synchronize()
    del keep
    got = out.cpu().numpy()[dst.cpu().numpy()]
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-4)
    assert np.isnan(out.cpu().numpy()).sum() == 2          # only the M destinations were written
