"""The allocation-free attention entry point (svoo_block_sparse_attn_static: its schedule scratch is a
device array inside the library) against svoo_block_sparse_attn through the C boundary: same bits,
on two calls in a row, the second with a smaller input (the shared array keeps the first call's
contents, and nothing of them may leak into the second)."""
import numpy as np
import pytest
import torch

from paper_2603_18636_amd import svoo, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


def layout(rng, bh, n, d, kq, kk, dtype):
    q = (1.5 * rng.standard_normal((bh, n, d))).astype(np.float32)
    k = (1.5 * rng.standard_normal((bh, n, d))).astype(np.float32)
    v = rng.standard_normal((bh, n, d)).astype(np.float32)
    if dtype == "bf16":
        q, k, v = (synth.round_to_bf16(x) for x in (q, k, v))
    lq = rng.integers(0, kq, (bh, n)).astype(np.int32)
    lk = rng.integers(0, kk, (bh, n)).astype(np.int32)
    mask = rng.random((bh, kq, kk)) < 0.4
    mask[:, np.arange(kq), rng.integers(0, kk, kq)] = True
    cnt = mask.sum(2).astype(np.int32)
    lst = np.full((bh, kq, kk), -1, dtype=np.int32)
    for b in range(bh):
        for r in range(kq):
            lst[b, r, :cnt[b, r]] = np.nonzero(mask[b, r])[0]
    qd, kd, vd = (H.to_dev(x, dtype) for x in (q, k, v))
    perm_q, q_off, (qs,) = svoo.permute(H.to_dev(lq), kq, [qd])
    perm_k, k_off, (ks, vs) = svoo.permute(H.to_dev(lk), kk, [kd, vd])
    return qs, ks, vs, q_off, k_off, H.to_dev(cnt), H.to_dev(lst)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_static_entry_point_equals_workspace_entry_point_twice(dtype, d):
    rng = np.random.default_rng(77 + d)
    scale = H.scale_of(d)
    bits = torch.int16 if dtype == "bf16" else torch.int32
    for bh, n, kq, kk in ((3, 2000, 40, 33), (2, 700, 9, 11)):          # the second call is the smaller one
        args = layout(rng, bh, n, d, kq, kk, dtype)
        want, want_lse = svoo.block_sparse_attn(*args, scale, want_lse=True)
        out = torch.full_like(args[0], float("nan"))
        lse = torch.full((bh, n), float("nan"), dtype=torch.float32, device=H.DEV)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        svoo.block_sparse_attn_static(*args, scale, out, lse)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(out.view(bits), want.view(bits))
        assert torch.equal(lse, want_lse)


def test_static_entry_point_rejects_shapes_beyond_its_scratch():
    bh, n, d, kq, kk = 300, 1024, 64, 1024, 2
    x = torch.zeros((bh, n, d), dtype=torch.bfloat16, device=H.DEV)
    q_off = torch.zeros((bh, kq + 1), dtype=torch.int32, device=H.DEV)
    k_off = torch.zeros((bh, kk + 1), dtype=torch.int32, device=H.DEV)
    cnt = torch.zeros((bh, kq), dtype=torch.int32, device=H.DEV)
    lst = torch.zeros((bh, kq, kk), dtype=torch.int32, device=H.DEV)
    out = torch.ones_like(x)
    with pytest.raises(svoo.SvooError) as err:
        svoo.block_sparse_attn_static(x, x, x, q_off, k_off, cnt, lst, 0.125, out)
    assert err.value.status == 5
    torch.cuda.synchronize()
    assert (out == 1).all()            # nothing was launched
