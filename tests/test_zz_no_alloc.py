"""The allocation-free decode-attention entry point against the ordinary one (same kernels, the
split partials in the library's built-in scratch instead of caller buffers): two calls in a row,
the second on a smaller input, so that leftovers of the first call in the shared scratch would
show; and the size limit is an error, not a fault."""
import numpy as np
import pytest
import torch

from tests.test_gpu_ops import _paged_case

pytestmark = pytest.mark.gpu


def _run_both(R, seed, ctx_lens, Hq, Hkv, hd, nsplit, dtype):
    rows, n_layers, layer = len(ctx_lens), 2, 1
    q, pool, pt, rs, want = _paged_case(seed, rows, Hq, Hkv, hd, n_layers, layer, ctx_lens, dtype)
    qd, pd = q.cuda().reshape(rows, Hq * hd).contiguous(), pool.cuda().contiguous()
    ptd, rsd = torch.from_numpy(pt).cuda(), torch.from_numpy(rs).cuda()
    cl = torch.tensor(ctx_lens, dtype=torch.int32).cuda()
    ref = torch.zeros_like(qd)
    pa = torch.zeros(rows * Hq * nsplit * hd, device="cuda")
    pm = torch.zeros(rows * Hq * nsplit * 2, device="cuda")
    R.rlhf_op_paged_decode_attention(qd, pd, ptd, rsd, cl, ref, pa, pm, layer, nsplit, n_layers, Hq, Hkv, hd)
    out = torch.full_like(qd, float("nan"))
    before = torch.cuda.memory_allocated()
    R.rlhf_op_paged_decode_attention_noalloc(qd, pd, ptd, rsd, cl, out, layer, nsplit, n_layers, Hq, Hkv, hd)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), ref.float().cpu().numpy(), want.reshape(rows, Hq * hd)


@pytest.mark.parametrize("dtype,Hq,Hkv,hd,tol", [("half", 16, 2, 128, 3e-3), ("half", 4, 4, 128, 3e-3),
                                                 ("fp32", 4, 4, 64, 2e-5)])
def test_no_alloc_decode_attention_two_calls(dtype, Hq, Hkv, hd, tol):
    import paper_2409_13221_amd as R
    # first call: long contexts, many splits; second: fewer rows, shorter contexts, fewer splits
    for seed, ctx_lens, nsplit in ((31, [900, 33, 2047, 1000, 16, 1500, 257, 64], 8), (32, [40, 5, 130], 3)):
        got, ref, want = _run_both(R, seed, ctx_lens, Hq, Hkv, hd, nsplit, dtype)
        np.testing.assert_array_equal(got, ref)                      # same kernels, same split: bit-identical
        np.testing.assert_allclose(got, want, rtol=0, atol=tol)      # and both match the oracle's attention


def test_no_alloc_decode_attention_rejects_oversize():
    import paper_2409_13221_amd as R
    rows, Hq, hd = 64, 32, 128
    q = torch.zeros(rows, Hq * hd, device="cuda", dtype=torch.float16)
    pool = torch.zeros(4, 1, 2, Hq, 16, hd, device="cuda", dtype=torch.float16)
    pt = torch.zeros(rows, 2, dtype=torch.int32, device="cuda")
    rs = torch.arange(rows, dtype=torch.int32, device="cuda")
    cl = torch.ones(rows, dtype=torch.int32, device="cuda")
    with pytest.raises(R.RlhfError) as e:       # 64 * 32 * 16 = 32768 slots > 16384
        R.rlhf_op_paged_decode_attention_noalloc(q, pool, pt, rs, cl, torch.empty_like(q), 0, 16, 1, Hq, Hq, hd)
    assert e.value.code == R.RLHF_EINVAL and "16384" in str(e.value)
