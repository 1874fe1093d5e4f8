"""GPU parity of the activation normalisation (Sec. 3.1): the per-layer norm sums over several batches, the
division (folded into the row scales for int8 rows), and a whole train step on the normalised inputs, each
against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import clt_oracle as O
from workloads import clt_synth as S

from clt_testlib import GpuRun, OracleRun, compare_step, theta_for_density, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _batches(w, n):
    """n seeded batches of inputs and targets (float32 on the host, already rounded to the storage type)."""
    return [S.make_inputs(S.scaled(w, seed=w.seed + 101 * i)) for i in range(n)]


def _handle(K, w):
    return K.CLTStep(w.L, w.d, w.F, w.B, dtype=w.dtype, int8_inputs=w.int8_inputs, device=DEV, matrix_grads=False)


@pytest.mark.parametrize("kind", ["f32", "bf16", "int8"])
def test_norm_sums_over_batches_and_division(kind):
    from paper_2603_21014_amd import binding as K
    base = S.WORKLOADS["llama1b_int8"] if kind == "int8" else S.scaled(S.WORKLOADS["llama1b"], dtype=kind)
    w = S.scaled(base, L=3, d=264, F=72, B=300, k_active=8)      # 10 row blocks, the last one ragged; d not a multiple of 256
    step = _handle(K, w)
    T = torch.float32 if kind == "f32" else torch.bfloat16
    sums = torch.zeros(w.L, dtype=torch.float64, device=DEV)
    ref_batches, dev_batches = [], []
    for x, _ in _batches(w, 3):
        if kind == "int8":
            q, s = S.quantize_rows_int8(x)
            ref_batches.append(O.dequantize_rows(q.numpy(), s.numpy()))
            dev_batches.append((q.to(DEV), s.to(DEV)))
            K.clt_norm_accumulate(step.H, dev_batches[-1][0], sums, dev_batches[-1][1])
        else:
            ref_batches.append(to_np(x))
            dev_batches.append((x.to(DEV, T).contiguous(), None))
            K.clt_norm_accumulate(step.H, dev_batches[-1][0], sums)
    n_tokens = 3 * w.B
    c = O.normalisation_factor(ref_batches)
    got = sums.cpu().numpy()
    print(f"[norm {kind}] c = {c}, rel err of sums = {np.abs(got / (c * n_tokens) - 1).max():.2e}", flush=True)
    np.testing.assert_allclose(got, c * n_tokens, rtol=2e-6)

    # a second pass over the same batches gives the same bits (fixed summation order)
    again = torch.zeros_like(sums)
    for a, s in dev_batches:
        K.clt_norm_accumulate(step.H, a, again, s)
    assert torch.equal(again, sums)

    a, s = dev_batches[1]
    if kind == "int8":
        out = torch.empty_like(s)
        K.clt_normalise(step.H, sums, n_tokens, scale_in=s, scale_out=out)
        np.testing.assert_allclose(out.cpu().numpy(), s.cpu().numpy().astype(np.float64) / c[:, None], rtol=1e-6)
        K.clt_normalise(step.H, sums, n_tokens, scale_in=s, scale_out=s)          # in place
        assert torch.equal(s, out)
    else:
        out = torch.empty_like(a)
        K.clt_normalise(step.H, sums, n_tokens, a_in=a, a_out=out)
        want = O.normalise_activations(ref_batches[1], c)
        # one rounding of the quotient to the storage type (plus the fp32 factor)
        rel = 2.0 ** -8 if kind == "bf16" else 1e-6
        assert np.all(np.abs(to_np(out) - want) <= rel * np.abs(want) + 1e-30)
        K.clt_normalise(step.H, sums, n_tokens, a_in=a, a_out=a)                  # in place
        assert torch.equal(a, out)


def test_all_zero_layer_is_left_unscaled():
    from paper_2603_21014_amd import binding as K
    w = S.scaled(S.WORKLOADS["tiny"], L=2, d=64, F=64, B=40)
    step = _handle(K, w)
    x = torch.randn(w.L, w.B, w.d, generator=torch.Generator().manual_seed(5))
    x[0] = 0.0
    xg = x.to(DEV)
    sums = torch.zeros(w.L, dtype=torch.float64, device=DEV)
    K.clt_norm_accumulate(step.H, xg, sums)
    c = O.normalisation_factor([to_np(x)])
    assert sums[0].item() == 0.0 and c[0] == 1.0
    out = torch.full_like(xg, 7.0)
    K.clt_normalise(step.H, sums, w.B, a_in=xg, a_out=out)
    assert torch.all(out[0] == 0.0)
    np.testing.assert_allclose(to_np(out), O.normalise_activations(to_np(x), c), rtol=3e-6)


def test_train_step_on_normalised_int8_cache():
    """Factors from three batches, folded into the row scales on the device; the step on a fourth batch then
    matches the oracle's step on the dequantised inputs divided by the oracle's own factors."""
    from paper_2603_21014_amd import binding as K
    w = S.scaled(S.WORKLOADS["llama1b_int8"], L=3, d=264, F=520, B=300, k_active=8)
    step = _handle(K, w)
    sx = torch.zeros(w.L, dtype=torch.float64, device=DEV)
    sy = torch.zeros(w.L, dtype=torch.float64, device=DEV)
    ref_x, ref_y = [], []
    for x, y in _batches(w, 3):
        for t, sums, ref in ((x, sx, ref_x), (y, sy, ref_y)):
            q, s = S.quantize_rows_int8(t)
            ref.append(O.dequantize_rows(q.numpy(), s.numpy()))
            K.clt_norm_accumulate(step.H, q.to(DEV), sums, s.to(DEV))
    cx, cy = O.normalisation_factor(ref_x), O.normalisation_factor(ref_y)

    x, y = S.make_inputs(S.scaled(w, seed=w.seed + 999))
    (qx, s_x), (qy, s_y) = S.quantize_rows_int8(x), S.quantize_rows_int8(y)
    fx, fy = torch.empty_like(s_x, device=DEV), torch.empty_like(s_y, device=DEV)
    K.clt_normalise(step.H, sx, 3 * w.B, scale_in=s_x.to(DEV), scale_out=fx)
    K.clt_normalise(step.H, sy, 3 * w.B, scale_in=s_y.to(DEV), scale_out=fy)
    xo = O.normalise_activations(O.dequantize_rows(qx.numpy(), s_x.numpy()), cx)
    yo = O.normalise_activations(O.dequantize_rows(qy.numpy(), s_y.numpy()), cy)
    # normalised inputs have mean norm near one per layer (the generator's layers differ by up to 1.5x before)
    assert np.all(np.abs(np.sqrt((xo * xo).sum(2)).mean(1) - 1.0) < 0.1)

    params = S.make_params(w)
    # thresholds for the normalised scale: a fraction of the features active
    theta = theta_for_density(torch.from_numpy(xo).float(), params["W_enc"], params["b_enc"], 0.05)
    g = GpuRun(w, params, qx, qy, x_scale=fx.cpu(), y_scale=fy.cpu(), theta=theta)
    o = OracleRun(w, params, x, y, gpu_active=g.active, gpu_window=g.window, theta=theta, x_np=xo, y_np=yo,
                  gpu_below=g.below)
    assert 0.01 < g.active.mean() < 0.2
    errs = compare_step(w, g, o, 2e-2)
    worst = sorted(errs.items(), key=lambda kv: -kv[1])[:4]
    print("[normalised int8 step] worst: " + ", ".join(f"{k}={e:.2e}" for k, e in worst), flush=True)


def test_normalisation_argument_errors():
    from paper_2603_21014_amd import binding as K
    w8 = S.scaled(S.WORKLOADS["llama1b_int8"], L=2, d=64, F=64, B=40)
    wn = S.scaled(S.WORKLOADS["tiny"], L=2, d=64, F=64, B=40)
    s8, sn = _handle(K, w8), _handle(K, wn)
    sums = torch.ones(2, dtype=torch.float64, device=DEV)
    q = torch.zeros(2, 40, 64, dtype=torch.int8, device=DEV)
    sc = torch.ones(2, 40, device=DEV)
    xf = torch.ones(2, 40, 64, device=DEV)
    with pytest.raises(K.CLTError) as e:          # int8 rows need their scales
        K.clt_norm_accumulate(s8.H, q, sums)
    assert "a_scale" in str(e.value)
    with pytest.raises(K.CLTError):               # native rows have none
        K.clt_norm_accumulate(sn.H, xf, sums, sc)
    with pytest.raises(K.CLTError) as e:
        K.clt_normalise(s8.H, sums, 0, scale_in=sc, scale_out=sc)
    assert "n_tokens" in str(e.value)
    with pytest.raises(K.CLTError):               # int8 codes are never rewritten
        K._check(K._lib.clt_normalise(s8.H.h, K._stream(), sums.data_ptr(), 40, q.data_ptr(), sc.data_ptr(), q.data_ptr(),
                                      sc.data_ptr()), s8.H.h)
    with pytest.raises(K.CLTError):
        K.clt_normalise(sn.H, sums, 40, a_in=xf, a_out=xf, scale_in=sc, scale_out=sc)
    with pytest.raises(K.CLTError):
        K.clt_normalise(sn.H, sums, 40, scale_in=sc, scale_out=sc)
    assert torch.all(xf == 1.0) and torch.all(sc == 1.0)
