"""Kernel-level parity through the C ABI (include/rlhf_ops.h) against the oracle's primitives
(numpy float64 matmul; oracle.transformer.attention)."""
import numpy as np
import pytest
import torch

from oracle import transformer as OT

pytestmark = pytest.mark.gpu


def _R():
    import paper_2409_13221_amd as R
    return R


def _bf16_round(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16)


@pytest.mark.parametrize("dtype", ["bf16", "bf16_half_act", "fp32"])
@pytest.mark.parametrize("M,N,K,nsplit", [
    (1, 256, 512, 1), (5, 130, 72, 1), (16, 768, 256, 4), (17, 1376, 256, 2), (33, 200, 688, 3),
    (64, 512, 2048, 1), (100, 4100, 328, 1), (257, 384, 1000, 2), (300, 1024, 64, 1),
])
def test_gemm(dtype, M, N, K, nsplit):
    R = _R()
    r = np.random.default_rng(M * 7 + N)
    a, w = r.normal(size=(M, K)), r.normal(size=(N, K))
    if dtype == "bf16":
        A, W = _bf16_round(a).cuda(), _bf16_round(w).cuda()
    elif dtype == "bf16_half_act":      # activations in IEEE half, weights bf16 (scaled into half's normal range)
        A, W = torch.from_numpy(a.astype(np.float32)).half().cuda(), _bf16_round(w * 0.02).cuda()
    else:
        A, W = torch.from_numpy(a.astype(np.float32)).cuda(), torch.from_numpy(w.astype(np.float32)).cuda()
    want = A.double().cpu().numpy() @ W.double().cpu().numpy().T
    out = torch.full((nsplit, M, N), float("nan"), device="cuda")
    R.rlhf_op_gemm(A, W, out, nsplit)
    torch.cuda.synchronize()
    got = out.double().sum(0).cpu().numpy()
    # inputs are exact in both paths; only float32 accumulation order differs
    np.testing.assert_allclose(got, want, rtol=0, atol=3e-5 * np.sqrt(K) * 4)
    assert np.abs(want).max() > 0.05


def test_gemm_nsplit_choice_is_sane():
    R = _R()
    for (M, N, K) in [(1, 4096, 4096), (16, 22016, 4096), (256, 4096, 11008), (8192, 4096, 4096)]:
        ns = R.rlhf_op_gemm_nsplit(R.RLHF_BF16, M, N, K, 16)
        assert 1 <= ns <= 16
        assert (ns - 1) * (-(-K // ns)) < K
    assert R.rlhf_op_gemm_nsplit(R.RLHF_BF16, 8192, 4096, 4096, 16) == 1


def _paged_case(seed, rows, Hq, Hkv, hd, n_layers, layer, ctx_lens, dtype):
    r = np.random.default_rng(seed)
    n_pages_each = [-(-c // 16) for c in ctx_lens]
    pool_pages = sum(n_pages_each) + 3
    perm = r.permutation(pool_pages)
    pt_stride = max(n_pages_each) + 1
    page_table = np.full((rows + 2, pt_stride), 0, np.int32)
    row_sample = r.permutation(rows + 2)[:rows].astype(np.int32)
    tdt = {"bf16": torch.bfloat16, "half": torch.float16, "fp32": torch.float32}[dtype]
    pool = (torch.randn(pool_pages, n_layers, 2, Hkv, 16, hd) * 1.0).to(tdt)
    q = (torch.randn(rows, Hq, hd) * 2.0).to(tdt)
    nxt = 0
    want = np.zeros((rows, Hq, hd))
    for rr in range(rows):
        pages = perm[nxt:nxt + n_pages_each[rr]]
        nxt += n_pages_each[rr]
        page_table[row_sample[rr], :len(pages)] = pages
        kv = pool[pages, layer].double().numpy()                  # [np, 2, Hkv, 16, hd]
        k = kv[:, 0].transpose(0, 2, 1, 3).reshape(-1, Hkv, hd)[:ctx_lens[rr]]
        v = kv[:, 1].transpose(0, 2, 1, 3).reshape(-1, Hkv, hd)[:ctx_lens[rr]]
        want[rr] = OT.attention(q[rr:rr + 1].double().numpy(), k, v, np.array([ctx_lens[rr] - 1]))[0]
    return q, pool, page_table, row_sample, want


@pytest.mark.parametrize("dtype,Hq,Hkv,hd", [("bf16", 4, 4, 128), ("bf16", 16, 2, 128), ("bf16", 3, 3, 64),
                                             ("half", 4, 4, 128), ("half", 16, 2, 128), ("half", 3, 3, 64),
                                             ("fp32", 4, 4, 64), ("fp32", 2, 2, 128)])
@pytest.mark.parametrize("nsplit", [1, 3, 8])
def test_paged_decode_attention(dtype, Hq, Hkv, hd, nsplit):
    R = _R()
    ctx_lens = [1, 16, 17, 5, 250, 64, 33, 129]
    rows, n_layers, layer = len(ctx_lens), 3, 1
    q, pool, pt, rs, want = _paged_case(11, rows, Hq, Hkv, hd, n_layers, layer, ctx_lens, dtype)
    qd, pd = q.cuda().reshape(rows, Hq * hd).contiguous(), pool.cuda().contiguous()
    out = torch.zeros_like(qd)
    pa = torch.zeros(rows * Hq * nsplit * hd, device="cuda")
    pm = torch.zeros(rows * Hq * nsplit * 2, device="cuda")
    R.rlhf_op_paged_decode_attention(qd, pd, torch.from_numpy(pt).cuda(), torch.from_numpy(rs).cuda(),
                                     torch.tensor(ctx_lens, dtype=torch.int32).cuda(), out, pa, pm, layer,
                                     nsplit, n_layers, Hq, Hkv, hd)
    torch.cuda.synchronize()
    got = out.double().cpu().numpy().reshape(rows, Hq, hd)
    tol = {"bf16": 2e-2, "half": 3e-3, "fp32": 2e-5}[dtype]   # 16-bit: output rounding of values of size ~1-3
    np.testing.assert_allclose(got, want, rtol=0, atol=tol)


@pytest.mark.parametrize("Hq,Hkv", [(16, 2), (4, 4)])
@pytest.mark.parametrize("nsplit", [1, 5, 16])
def test_paged_decode_attention_long_contexts(Hq, Hkv, nsplit):
    """Contexts of thousands of tokens (many pages per wave, splits with and without pages), for
    the grouped-head MFMA kernel and the one-head-per-KV-head kernel."""
    R = _R()
    ctx_lens = [4000, 33, 2047, 1000, 16, 3009]
    rows, n_layers, layer, hd = len(ctx_lens), 2, 1, 128
    q, pool, pt, rs, want = _paged_case(21, rows, Hq, Hkv, hd, n_layers, layer, ctx_lens, "half")
    qd, pd = q.cuda().reshape(rows, Hq * hd).contiguous(), pool.cuda().contiguous()
    out = torch.zeros_like(qd)
    pa = torch.zeros(rows * Hq * nsplit * hd, device="cuda")
    pm = torch.zeros(rows * Hq * nsplit * 2, device="cuda")
    R.rlhf_op_paged_decode_attention(qd, pd, torch.from_numpy(pt).cuda(), torch.from_numpy(rs).cuda(),
                                     torch.tensor(ctx_lens, dtype=torch.int32).cuda(), out, pa, pm, layer,
                                     nsplit, n_layers, Hq, Hkv, hd)
    torch.cuda.synchronize()
    got = out.double().cpu().numpy().reshape(rows, Hq, hd)
    # long contexts average many values: outputs are small and so is their half rounding
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-3)


@pytest.mark.parametrize("Hq,Hkv,hd", [(4, 4, 128), (8, 1, 128), (3, 3, 64)])
def test_flash_attention(Hq, Hkv, hd):
    """MFMA attention of bf16 models: several query tiles, ragged tails, tiny sequences."""
    R = _R()
    lens = [1, 130, 64, 300, 17, 128, 257]
    T = sum(lens)
    torch.manual_seed(5)
    q, k, v = (torch.randn(T, Hq, hd) * 1.5).half(), torch.randn(T, Hkv, hd).half(), torch.randn(T, Hkv, hd).half()
    want, o = np.zeros((T, Hq, hd)), 0
    for n in lens:
        want[o:o + n] = OT.attention(q[o:o + n].double().numpy(), k[o:o + n].double().numpy(),
                                     v[o:o + n].double().numpy(), np.arange(n))
        o += n
    out = torch.zeros(T, Hq * hd, dtype=torch.float16, device="cuda")
    keep = R.rlhf_op_flash_attention(q.cuda().reshape(T, -1).contiguous(), k.cuda().reshape(T, -1).contiguous(),
                                     v.cuda().reshape(T, -1).contiguous(), lens, out, Hq, Hkv, hd)
    torch.cuda.synchronize()
    del keep
    # probabilities and the output are rounded to half: 2^-11 relative on values of size ~1-3
    np.testing.assert_allclose(out.double().cpu().numpy().reshape(T, Hq, hd), want, rtol=0, atol=4e-3)


@pytest.mark.parametrize("dtype,Hq,Hkv,hd", [("fp32", 4, 4, 64), ("fp32", 2, 2, 128)])
def test_varlen_attention(dtype, Hq, Hkv, hd):
    R = _R()
    lens = [1, 7, 16, 17, 40, 3]
    T = sum(lens)
    tdt = torch.float16 if dtype == "half" else torch.float32
    torch.manual_seed(3)
    q, k, v = torch.randn(T, Hq, hd) * 1.5, torch.randn(T, Hkv, hd), torch.randn(T, Hkv, hd)
    row_start, row_pos, want = [], [], np.zeros((T, Hq, hd))
    o = 0
    for n in lens:
        row_start += [o] * n
        row_pos += list(range(n))
        want[o:o + n] = OT.attention(q[o:o + n].double().numpy(), k[o:o + n].double().numpy(),
                                     v[o:o + n].double().numpy(), np.arange(n))
        o += n
    out = torch.zeros(T, Hq * hd, dtype=tdt, device="cuda")
    R.rlhf_op_varlen_attention(q.cuda().reshape(T, -1).contiguous(), k.cuda().reshape(T, -1).contiguous(),
                               v.cuda().reshape(T, -1).contiguous(),
                               torch.tensor(row_start, dtype=torch.int32).cuda(),
                               torch.tensor(row_pos, dtype=torch.int32).cuda(), out, Hq, Hkv, hd)
    torch.cuda.synchronize()
    tol = 3e-3 if dtype == "half" else 2e-5      # half: output rounding of values of size ~1-3
    np.testing.assert_allclose(out.double().cpu().numpy().reshape(T, Hq, hd), want, rtol=0, atol=tol)


@pytest.mark.parametrize("variant", [5, 6, 7])
@pytest.mark.parametrize("half_act", [False, True])
def test_gemm_compute_bound_tilings(variant, half_act):
    """Every large-M tiling (XCD-aware tile order, ragged M/N/K edges, more tiles than one
    super-tile in N) against float64."""
    R = _R()
    M, N, K = 700, 4200, 328
    r = np.random.default_rng(variant)
    a, w = r.normal(size=(M, K)), r.normal(size=(N, K)) * 0.02
    A = torch.from_numpy(a.astype(np.float32)).half().cuda() if half_act else _bf16_round(a).cuda()
    W = _bf16_round(w).cuda()
    want = A.double().cpu().numpy() @ W.double().cpu().numpy().T
    out = torch.full((1, M, N), float("nan"), device="cuda")
    R.rlhf_op_gemm(A, W, out, 1, variant)
    torch.cuda.synchronize()
    np.testing.assert_allclose(out[0].double().cpu().numpy(), want, rtol=0, atol=2e-5)


@pytest.mark.parametrize("half_act", [True, False])
@pytest.mark.parametrize("M,f,K", [(512, 688, 256), (700, 1000, 328), (1024, 11008, 512)])
def test_gemm_swiglu_fused(half_act, M, f, K):
    """Gate||up projection with the SwiGLU epilogue against float64 (ragged M, f, K edges)."""
    R = _R()
    r = np.random.default_rng(f)
    a, w = r.normal(size=(M, K)), r.normal(size=(2 * f, K)) * 0.06
    A = torch.from_numpy(a.astype(np.float32)).half().cuda() if half_act else _bf16_round(a).cuda()
    W = _bf16_round(w).cuda()
    z = A.double().cpu().numpy() @ W.double().cpu().numpy().T
    want = OT.silu(z[:, :f]) * z[:, f:]
    act = torch.full((M, f), float("nan"), dtype=A.dtype, device="cuda")
    R.rlhf_op_gemm_swiglu(A, W, act)
    torch.cuda.synchronize()
    got = act.double().cpu().numpy()
    assert np.isfinite(got).all() and np.abs(want).max() > 0.3
    tol = (2 ** -11 if half_act else 2 ** -8) * np.maximum(np.abs(want), 1e-2) + 1e-4   # output rounding
    assert np.all(np.abs(got - want) <= tol), np.abs(got - want).max()


@pytest.mark.parametrize("half_act", [True, False])
@pytest.mark.parametrize("M,K,Hq,Hkv,hd,with_pool", [(512, 256, 4, 4, 64, False), (700, 320, 5, 1, 64, True),
                                                     (1000, 192, 3, 1, 128, True), (1024, 512, 8, 2, 128, False)])
def test_gemm_rope_fused(half_act, M, K, Hq, Hkv, hd, with_pool):
    """QKV projection with rotary embedding, rounding and the q / k / v / paged-pool scatter in
    the epilogue against float64 (ragged M and N edges, grouped heads, both head sizes)."""
    R = _R()
    r = np.random.default_rng(M + K)
    base, n_layers, layer, max_pos = 10000.0, 3, 1, 300
    N = (Hq + 2 * Hkv) * hd
    a, w = r.normal(size=(M, K)), r.normal(size=(N, K)) * 0.06
    A = torch.from_numpy(a.astype(np.float32)).half().cuda() if half_act else _bf16_round(a).cuda()
    W = _bf16_round(w).cuda()
    pos = r.integers(0, max_pos, size=M).astype(np.int32)
    ang = np.arange(max_pos)[:, None] * base ** (-2.0 * np.arange(hd // 2) / hd)[None, :]
    table = torch.from_numpy(np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)).cuda()
    z = A.double().cpu().numpy() @ W.double().cpu().numpy().T
    want_q = OT.rope(z[:, :Hq * hd].reshape(M, Hq, hd), pos, base).reshape(M, -1)
    want_k = OT.rope(z[:, Hq * hd:(Hq + Hkv) * hd].reshape(M, Hkv, hd), pos, base).reshape(M, -1)
    want_v = z[:, (Hq + Hkv) * hd:]
    nan = lambda *s: torch.full(s, float("nan"), dtype=A.dtype, device="cuda")
    q, k, v = nan(M, Hq * hd), nan(M, Hkv * hd), nan(M, Hkv * hd)
    n_pages = (M + 15) // 16 + 2
    pool = nan(n_pages, n_layers, 2, Hkv, 16, hd) if with_pool else None
    slots = r.permutation(n_pages * 16)[:M].astype(np.int32)          # every row its own token slot
    R.rlhf_op_gemm_rope(A, W, torch.from_numpy(pos).cuda(), table, q, k if not with_pool else None,
                        v if not with_pool else None, pool, torch.from_numpy(slots).cuda() if with_pool else None,
                        layer, n_layers, Hq, Hkv, hd)
    torch.cuda.synchronize()
    eps = 2 ** -11 if half_act else 2 ** -8

    def close(got, want):
        got = got.double().cpu().numpy()
        assert np.isfinite(got).all() and np.abs(want).max() > 0.3
        assert np.all(np.abs(got - want) <= eps * np.maximum(np.abs(want), 1e-2) + 1e-4), np.abs(got - want).max()

    close(q, want_q)
    if with_pool:
        p = pool.double().cpu().numpy()
        got = p[slots // 16, layer, :, :, slots % 16, :]              # [M, 2, Hkv, hd]
        close(torch.from_numpy(got[:, 0].reshape(M, -1)), want_k)
        close(torch.from_numpy(got[:, 1].reshape(M, -1)), want_v)
        p[slots // 16, layer, :, :, slots % 16, :] = np.nan
        assert np.isnan(p).all()                                      # nothing else was written
        assert torch.isnan(k).all() and torch.isnan(v).all()
    else:
        close(k, want_k)
        close(v, want_v)


@pytest.mark.parametrize("M,N,K", [(200, 12288, 4096), (256, 4096, 11008), (129, 22016, 4096)])
def test_gemm_mid_rows_take_the_tall_tiling_with_split_k(M, N, K):
    """129..256 rows of a large matrix run as one row of 256 x 256 tiles with K split over the
    compute units (the split the stage itself chooses); uneven last split included."""
    R = _R()
    r = np.random.default_rng(M + N)
    A = torch.from_numpy(r.normal(size=(M, K)).astype(np.float32)).half().cuda()
    W = _bf16_round(r.normal(size=(N, K)) * 0.02).cuda()
    ns = R.rlhf_op_gemm_nsplit(R.RLHF_BF16, M, N, K, 16)
    assert ns > 1 and -(-N // 256) * ns <= 256
    want = A.double().cpu().numpy() @ W.double().cpu().numpy().T
    out = torch.full((ns, M, N), float("nan"), device="cuda")
    R.rlhf_op_gemm(A, W, out, ns)
    torch.cuda.synchronize()
    got = out.double().sum(0).cpu().numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=3e-5 * np.sqrt(K))


# ------------------------------------------- half copies of the weights (both operands direct to LDS)

def test_half_weight_gemm_rejects_operands_of_4_gib():
    """The half-weight kernels address an operand with 32-bit byte offsets: an A of 4 GiB is refused with
    an error before anything is launched (nothing in it is read, so it need not be initialised)."""
    R = _R()
    K, N, M = 2048, 256, 1 << 20                       # M * K * 2 bytes = 4 GiB
    A = torch.empty(M, K, dtype=torch.float16, device="cuda")
    Wh = R.rlhf_op_bf16_to_half(_bf16_round(np.zeros((N, K)) + 0.01).cuda())
    C = torch.empty(1, M, N, device="cuda")
    with pytest.raises(Exception) as err:
        R.rlhf_op_gemm(A, Wh, C, 1)
    assert "rlhf_op_gemm" in str(err.value) or "EINVAL" in str(err.value)
    del A, C
    # one row less fits
    A = torch.zeros(M - 1, K, dtype=torch.float16, device="cuda")
    C = torch.empty(1, M - 1, N, device="cuda")
    R.rlhf_op_gemm(A, Wh, C, 1)
    torch.cuda.synchronize()
    assert float(C.abs().max()) == 0.0


def test_half_weight_copies_give_bit_identical_tall_gemms():
    """With an IEEE-half copy of the bf16 matrix (the library's own conversion) the tall kernels load
    both operands global -> LDS directly; plain, split-K, SwiGLU, rotary and LM-head epilogues must
    reproduce the bf16-weight path bit for bit (same half values, same accumulation order) and so
    match float64 like it does."""
    R = _R()
    r = np.random.default_rng(77)
    M, K = 700, 512
    A = torch.from_numpy(r.normal(size=(M, K)).astype(np.float32)).half().cuda()
    # a share of tiny weights exercises half's subnormal range in the conversion
    w = r.normal(size=(1300, K)) * 0.02
    w[::7] *= 1e-4
    W = _bf16_round(w).cuda()
    Wh = R.rlhf_op_bf16_to_half(W)
    torch.cuda.synchronize()
    wd, whd = W.double().cpu().numpy(), Wh.double().cpu().numpy()
    big = np.abs(wd) >= 2.0 ** -14
    np.testing.assert_array_equal(whd[big], wd[big])                         # exact in the normal range
    assert np.all(np.abs(whd - wd) < 2.0 ** -24) and np.all(np.abs(whd) <= np.abs(wd))   # toward zero below it
    # plain, one split and three
    for ns in (1, 3):
        a = torch.full((ns, M, 1300), float("nan"), device="cuda")
        b = torch.full((ns, M, 1300), float("nan"), device="cuda")
        R.rlhf_op_gemm(A, W, a, ns, 7)
        R.rlhf_op_gemm(A, Wh, b, ns)
        torch.cuda.synchronize()
        assert torch.equal(a, b)
        np.testing.assert_allclose(b.double().sum(0).cpu().numpy(), A.double().cpu().numpy() @ whd.T, rtol=0, atol=3e-5)
    # SwiGLU epilogue (648 output columns: a ragged last tile)
    act_a = torch.full((M, 648), float("nan"), dtype=torch.float16, device="cuda")
    act_b = torch.full_like(act_a, float("nan"))
    R.rlhf_op_gemm_swiglu(A, W[:1296].contiguous(), act_a)
    R.rlhf_op_gemm_swiglu(A, Wh[:1296].contiguous(), act_b)
    # rotary epilogue: 6 query + 2 x 2 KV heads of 128 -> 1280 rows of W
    Hq, Hkv, hd = 6, 2, 128
    pos = torch.from_numpy(r.integers(0, 300, size=M).astype(np.int32)).cuda()
    ang = np.arange(300)[:, None] * 10000.0 ** (-2.0 * np.arange(hd // 2) / hd)[None, :]
    table = torch.from_numpy(np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)).cuda()
    outs = []
    for Wx in (W[:1280].contiguous(), Wh[:1280].contiguous()):
        q = torch.full((M, Hq * hd), float("nan"), dtype=torch.float16, device="cuda")
        k = torch.full((M, Hkv * hd), float("nan"), dtype=torch.float16, device="cuda")
        v = torch.full_like(k, float("nan"))
        R.rlhf_op_gemm_rope(A, Wx, pos, table, q, k, v, None, None, 0, 1, Hq, Hkv, hd)
        outs.append((q, k, v))
    # LM head fused with the log-softmax gather over a vocabulary of 1300
    tokens = torch.from_numpy(r.integers(0, 1300, size=M).astype(np.int32)).cuda()
    idx = torch.arange(M, dtype=torch.int32, device="cuda")
    lp_a, lp_b = torch.zeros(M, device="cuda"), torch.zeros(M, device="cuda")
    keep = [R.rlhf_op_lm_head_logprob(A, W, tokens, idx, lp_a, idx), R.rlhf_op_lm_head_logprob(A, Wh, tokens, idx, lp_b, idx)]
    torch.cuda.synchronize()
    del keep
    assert torch.equal(act_a, act_b) and torch.isfinite(act_b).all()
    for x, y in zip(*outs):
        assert torch.equal(x, y) and torch.isfinite(y).all()
    assert torch.equal(lp_a, lp_b)
    z = A.double().cpu().numpy() @ whd.T
    want = OT.log_softmax_rows(z)[np.arange(M), tokens.cpu().numpy()]
    np.testing.assert_allclose(lp_b.cpu().numpy(), want, rtol=0, atol=1e-4)


# ------------------------------------------- few rows, no K split, the consumer in the epilogue

@pytest.mark.parametrize("half_act", [True, False])
@pytest.mark.parametrize("M,f,K", [(1, 688, 256), (7, 1000, 768), (16, 11008, 4096), (9, 40, 512)])
def test_few_row_gate_up_with_swiglu_epilogue(half_act, M, f, K):
    """Decode-step gate||up projection: up to 16 rows, every workgroup walks the whole K range
    through its register ring (depth 8 or 4), SwiGLU in the epilogue; ragged last column block."""
    R = _R()
    r = np.random.default_rng(f + M)
    a, w = r.normal(size=(M, K)), r.normal(size=(2 * f, K)) * 0.06
    A = torch.from_numpy(a.astype(np.float32)).half().cuda() if half_act else _bf16_round(a).cuda()
    W = _bf16_round(w).cuda()
    z = A.double().cpu().numpy() @ W.double().cpu().numpy().T
    want = OT.silu(z[:, :f]) * z[:, f:]
    act = torch.full((M, f), float("nan"), dtype=A.dtype, device="cuda")
    R.rlhf_op_gemm_swiglu(A, W, act)
    torch.cuda.synchronize()
    got = act.double().cpu().numpy()
    assert np.isfinite(got).all()
    tol = (2 ** -11 if half_act else 2 ** -8) * np.maximum(np.abs(want), 1e-2) + 1e-4
    assert np.all(np.abs(got - want) <= tol), np.abs(got - want).max()


@pytest.mark.parametrize("half_act", [True, False])
@pytest.mark.parametrize("M,K,Hq,Hkv,hd,with_pool", [(1, 256, 4, 4, 64, True), (5, 768, 5, 1, 64, False),
                                                     (16, 4096, 8, 2, 128, True), (11, 512, 3, 3, 128, True)])
def test_few_row_qkv_with_rotary_epilogue(half_act, M, K, Hq, Hkv, hd, with_pool):
    """Decode-step QKV projection: rotary embedding and the q / paged-pool (or k, v) scatter in the
    epilogue of the no-split kernel; both head sizes, grouped heads."""
    R = _R()
    r = np.random.default_rng(M + K)
    base, n_layers, layer, max_pos = 10000.0, 2, 1, 300
    N = (Hq + 2 * Hkv) * hd
    a, w = r.normal(size=(M, K)), r.normal(size=(N, K)) * 0.06
    A = torch.from_numpy(a.astype(np.float32)).half().cuda() if half_act else _bf16_round(a).cuda()
    W = _bf16_round(w).cuda()
    pos = r.integers(0, max_pos, size=M).astype(np.int32)
    ang = np.arange(max_pos)[:, None] * base ** (-2.0 * np.arange(hd // 2) / hd)[None, :]
    table = torch.from_numpy(np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)).cuda()
    z = A.double().cpu().numpy() @ W.double().cpu().numpy().T
    want_q = OT.rope(z[:, :Hq * hd].reshape(M, Hq, hd), pos, base).reshape(M, -1)
    want_k = OT.rope(z[:, Hq * hd:(Hq + Hkv) * hd].reshape(M, Hkv, hd), pos, base).reshape(M, -1)
    want_v = z[:, (Hq + Hkv) * hd:]
    nan = lambda *s: torch.full(s, float("nan"), dtype=A.dtype, device="cuda")
    q, k, v = nan(M, Hq * hd), nan(M, Hkv * hd), nan(M, Hkv * hd)
    n_pages = 4
    pool = nan(n_pages, n_layers, 2, Hkv, 16, hd) if with_pool else None
    slots = r.permutation(n_pages * 16)[:M].astype(np.int32)
    R.rlhf_op_gemm_rope(A, W, torch.from_numpy(pos).cuda(), table, q, k if not with_pool else None,
                        v if not with_pool else None, pool, torch.from_numpy(slots).cuda() if with_pool else None,
                        layer, n_layers, Hq, Hkv, hd)
    torch.cuda.synchronize()
    eps = 2 ** -11 if half_act else 2 ** -8

    def close(got, want):
        got = got.double().cpu().numpy()
        assert np.isfinite(got).all()
        assert np.all(np.abs(got - want) <= eps * np.maximum(np.abs(want), 1e-2) + 1e-4), np.abs(got - want).max()

    close(q, want_q)
    if with_pool:
        p = pool.double().cpu().numpy()
        got = p[slots // 16, layer, :, :, slots % 16, :]
        close(torch.from_numpy(got[:, 0].reshape(M, -1)), want_k)
        close(torch.from_numpy(got[:, 1].reshape(M, -1)), want_v)
        p[slots // 16, layer, :, :, slots % 16, :] = np.nan
        assert np.isnan(p).all()
        assert torch.isnan(k).all() and torch.isnan(v).all()
    else:
        close(k, want_k)
        close(v, want_v)


@pytest.mark.parametrize("M,N,K", [(3, 200, 256), (16, 4100, 1024), (8, 12288, 4096)])
def test_few_row_gemm_without_k_split(M, N, K):
    R = _R()
    r = np.random.default_rng(N)
    A = torch.from_numpy(r.normal(size=(M, K)).astype(np.float32)).half().cuda()
    W = _bf16_round(r.normal(size=(N, K)) * 0.02).cuda()
    want = A.double().cpu().numpy() @ W.double().cpu().numpy().T
    out = torch.full((1, M, N), float("nan"), device="cuda")
    R.rlhf_op_gemm(A, W, out, 1, 8)
    torch.cuda.synchronize()
    np.testing.assert_allclose(out[0].double().cpu().numpy(), want, rtol=0, atol=3e-5 * np.sqrt(K))
