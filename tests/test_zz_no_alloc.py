"""The allocation-free entry point esa_select_topk_static against esa_select_topk, through the C ABI.

The library keeps the scratch of this call in an array of its own on the GPU; the array survives from
call to call, so the test makes two calls in a row, the second on a smaller input, and a third on a
batch, each compared bit for bit with the call that takes a caller workspace."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def esa():
    import paper_2502_14477_amd as lib
    return lib


def _raw_call(esa, score, k, base, idx):
    """The C entry point itself, with plain pointers: no workspace argument, nothing allocated here."""
    B, n = (1, score.shape[0]) if score.dim() == 1 else score.shape
    rc = esa.lib.esa_select_topk_static(ctypes.c_void_p(score.data_ptr()), n, k, base, ctypes.c_void_p(idx.data_ptr()), B,
                                        score.stride(0) if score.dim() == 2 else n, min(k, n),
                                        ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    return rc


def test_select_topk_static_matches_select_topk_on_consecutive_calls(esa):
    print("[case] esa_select_topk_static: n=200000 k=2048, then n=5000 k=300, then batch 4 x 70000", flush=True)
    rng = np.random.default_rng(2024)
    esa.esa_select_topk_static_prepare()
    assert esa.esa_select_topk_static_capacity() >= 1 << 20
    cases = [(1, 200000, 2048, 77), (1, 5000, 300, 3), (4, 70000, 1000, 0), (1, 40, 64, 5)]
    for B, n, k, base in cases:
        s = rng.standard_normal((B, n)).astype(np.float32)
        s[:, rng.choice(n, size=min(n, 50), replace=False)] = 0.25           # exact ties near the top
        sd = torch.from_numpy(s).cuda()
        sd = sd[0] if B == 1 else sd
        want = esa.esa_select_topk(sd, k, base=base)
        idx = torch.full(want.shape, -1, dtype=torch.int32, device="cuda")
        before = torch.cuda.memory_allocated()
        rc = _raw_call(esa, sd, k, base, idx)
        assert rc == 0, esa.lib.esa_last_error()
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert torch.equal(idx, want), (B, n, k)
        # and through the binding
        assert torch.equal(esa.esa_select_topk_static(sd, k, base=base), want)


def test_select_topk_static_rejects_what_does_not_fit(esa):
    print("[case] esa_select_topk_static: oversize request", flush=True)
    cap = esa.esa_select_topk_static_capacity()
    n = 1 << 22
    B = 1
    while esa.lib.esa_select_topk_workspace_bytes(n, 16, B) <= cap:
        B *= 2
    score = torch.zeros(8, dtype=torch.float32, device="cuda")           # never read: the call must refuse first
    idx = torch.zeros(8, dtype=torch.int32, device="cuda")
    rc = esa.lib.esa_select_topk_static(ctypes.c_void_p(score.data_ptr()), n, 16, 0, ctypes.c_void_p(idx.data_ptr()), B, n, 16,
                                        ctypes.c_void_p(0))
    assert rc == -3 and b"scratch" in esa.lib.esa_last_error()
