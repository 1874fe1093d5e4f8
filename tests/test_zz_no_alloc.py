"""The entry point that allocates nothing (clt_norm_accumulate_static: the per-block partial sums live in
the library's own static device array) against the entry point it is a variant of (clt_norm_accumulate,
partial sums in the caller's workspace): same kernels, so the per-layer norm sums must agree bit for bit --
and with the oracle's factor.  Two calls in a row, the second on a smaller input, so that whatever the
first call left in the shared array cannot leak into the second."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import clt_oracle as O

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(L, B, d, kind, seed):
    g = torch.Generator().manual_seed(seed)
    a = torch.randn((L, B, d), generator=g) * (1.0 + 0.5 * torch.arange(L, dtype=torch.float32))[:, None, None]
    if kind == "f32":
        return a.to(DEV), None, a.double().numpy()
    if kind == "bf16":
        a16 = a.to(torch.bfloat16)
        return a16.to(DEV), None, a16.double().numpy()
    absmax = a.abs().amax(dim=2)
    s = (absmax / 127.0).float()
    q = torch.clamp(torch.round(a / s[:, :, None]), -127, 127).to(torch.int8)
    return q.to(DEV), s.to(DEV), O.dequantize_rows(q.numpy(), s.numpy())


@pytest.mark.parametrize("kind", ["f32", "bf16", "int8"])
def test_static_scratch_entry_point_matches_workspace_entry_point(kind):
    from paper_2603_21014_amd import binding as K
    results = []
    for call, (L, B, d) in enumerate([(5, 1000, 264), (3, 77, 72)]):      # the second call is the smaller one
        a, scale, a_np = _inputs(L, B, d, kind, 11 + call)
        step = K.CLTStep(L, d, 64, B, dtype="f32" if kind == "f32" else "bf16", int8_inputs=kind == "int8")
        want = torch.zeros(L, dtype=torch.float64, device=DEV)
        got = torch.full((L,), 0.0, dtype=torch.float64, device=DEV)
        K.clt_norm_accumulate(step.H, a, want, scale)
        # cumulative count of allocations made through torch (memory freed meanwhile by the garbage collector,
        # e.g. of earlier tests, does not change it)
        held = torch.cuda.memory_stats()["allocation.all.allocated"]
        K.clt_norm_accumulate_static(a, got, scale)
        K.clt_norm_accumulate_static(a, got, scale)                      # accumulates: twice the sum
        K.clt_norm_accumulate(step.H, a, want, scale)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == held, "the static entry point allocated device memory"
        assert torch.equal(got, want), (got, want)
        ref = 2.0 * np.sqrt((a_np * a_np).sum(axis=2)).sum(axis=1)
        np.testing.assert_allclose(got.cpu().numpy(), ref, rtol=1e-5 if kind != "f32" else 1e-6)
        np.testing.assert_allclose(got.cpu().numpy() / (2 * B), O.normalisation_factor([a_np]), rtol=1e-5)
        results.append(got.cpu())
    assert len(results) == 2


def test_static_scratch_entry_point_rejects_what_it_cannot_hold():
    from paper_2603_21014_amd import binding as K
    lib = K._lib
    a = torch.zeros((2, 64, 64), dtype=torch.float32, device=DEV)
    s = torch.zeros(2, dtype=torch.float64, device=DEV)
    f = lib.clt_norm_accumulate_static
    # 128 layers x ceil(20000 / 32) blocks = 80000 partial sums > 65536: refused before any launch
    assert f(None, 128, 20000, 64, K.DTYPE_F32, K.INPUT_NATIVE, a.data_ptr(), None, s.data_ptr()) == -4
    assert b"static scratch" in lib.clt_last_error(None)
    assert f(None, 2, 64, 60, K.DTYPE_F32, K.INPUT_NATIVE, a.data_ptr(), None, s.data_ptr()) == -2
    assert f(None, 2, 64, 64, K.DTYPE_F32, K.INPUT_NATIVE, None, None, s.data_ptr()) == -1
    assert f(None, 2, 64, 64, K.DTYPE_F32, K.INPUT_INT8_ROWSCALE, a.data_ptr(), None, s.data_ptr()) == -1
    assert f(None, 2, 64, 64, K.DTYPE_F32, K.INPUT_NATIVE, a.data_ptr() + 4, None, s.data_ptr()) == -3
    assert f(None, 2, 64, 64, 9, K.INPUT_NATIVE, a.data_ptr(), None, s.data_ptr()) == -1
    torch.cuda.synchronize()
    assert not s.any()
