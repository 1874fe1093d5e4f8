"""Pins for the oracle's dead-feature penalty and log-threshold parameterisation
(App. B objective, third term; theta = exp(tau)).  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import clt_oracle as O
from test_oracle_pins import _JumpSTE, rand_problem


def full_loss(p, tau_or_theta, lambda0, lambda1, C, log_threshold):
    theta = O.threshold_value(tau_or_theta, log_threshold)
    fwd = O.forward(p["x"], p["W_enc"], p["b_enc"], theta, p["W_dec"], p["b_dec"])
    n = O.decoder_norms(p["W_dec"], p["x"].shape[0])
    tot = O.loss_terms(fwd["y_hat"], p["y"], fwd["z"], n, lambda0, C)[0]
    return tot + O.dead_feature_term(fwd["pre"], theta, n, lambda1), fwd, theta


def test_dead_term_closed_forms():
    rng = np.random.default_rng(1)
    L, B, F = 2, 5, 4
    pre = rng.standard_normal((L, B, F))
    n = 0.5 + rng.random((L, F))
    # threshold below every pre-activation: nothing is penalised
    assert O.dead_feature_term(pre, np.full((L, F), pre.min() - 1.0), n, 3.0) == 0.0
    # threshold above every pre-activation: the term is linear, (lambda1/B) sum (theta - pre) n
    th = np.full((L, F), pre.max() + 1.0)
    want = 3.0 * np.sum((th[:, None, :] - pre) * n[:, None, :]) / B
    assert abs(O.dead_feature_term(pre, th, n, 3.0) - want) < 1e-12
    # brute force
    tot = 0.0
    th = rng.standard_normal((L, F)) * 0.3
    for l in range(L):
        for b in range(B):
            for f in range(F):
                tot += max(th[l, f] - pre[l, b, f], 0.0) * n[l, f]
    assert abs(O.dead_feature_term(pre, th, n, 0.7) - 0.7 * tot / B) < 1e-12
    assert np.allclose(O.threshold_value(np.log(th * 0 + 0.03), True), 0.03)


@pytest.mark.parametrize("log_threshold", [False, True])
def test_all_gradients_by_finite_differences_with_empty_ste_window(log_threshold):
    """With an STE window too narrow to hold any pre-activation the objective is a genuine
    differentiable function of every parameter, including the threshold (only the
    dead-feature term depends on it), so central differences pin all five gradients."""
    rng = np.random.default_rng(7)
    L, d, F, B = 3, 5, 7, 4
    p = rand_problem(rng, L, d, F, B, theta=0.15, wscale=0.8)
    param = np.log(p["theta"]) if log_threshold else p["theta"].copy()
    lambda0, lambda1, C = 0.3, 0.9, 2.0
    _, fwd, theta = full_loss(p, param, lambda0, lambda1, C, log_threshold)
    assert np.min(np.abs(fwd["pre"] - theta[:, None, :])) > 1e-3
    assert (~fwd["active"]).sum() > 10
    gr = O.backward(p["x"], p["y"], theta, p["W_dec"], fwd, lambda0, C, eps=1e-7,
                    lambda1=lambda1, log_threshold=log_threshold)
    assert not gr["window"].any()
    h = 1e-6
    for name in ("W_enc", "b_enc", "W_dec", "b_dec", "theta"):
        g = gr["d" + name]
        for _ in range(20):
            idx = tuple(rng.integers(0, s) for s in g.shape)
            q = {k: v.copy() for k, v in p.items()}
            par = param.copy()
            if name == "theta":
                par[idx] += h
            else:
                q[name][idx] += h
            lp_, f1, _ = full_loss(q, par, lambda0, lambda1, C, log_threshold)
            if name == "theta":
                par[idx] -= 2 * h
            else:
                q[name][idx] -= 2 * h
            lm_, f2, _ = full_loss(q, par, lambda0, lambda1, C, log_threshold)
            assert (f1["active"] == fwd["active"]).all() and (f2["active"] == fwd["active"]).all()
            fd = (lp_ - lm_) / (2 * h)
            assert abs(fd - g[idx]) <= 2e-6 * max(1.0, abs(g[idx])), (name, idx, fd, g[idx])


@pytest.mark.parametrize("log_threshold", [False, True])
def test_against_torch_autograd_with_ste(log_threshold):
    rng = np.random.default_rng(9)
    L, d, F, B = 3, 6, 10, 16
    p = rand_problem(rng, L, d, F, B, theta=0.2, wscale=0.6)
    param = np.log(p["theta"]) if log_threshold else p["theta"].copy()
    lambda0, lambda1, C, eps = 0.7, 1.3, 2.0, 0.3
    tot, fwd, theta = full_loss(p, param, lambda0, lambda1, C, log_threshold)
    gr = O.backward(p["x"], p["y"], theta, p["W_dec"], fwd, lambda0, C, eps, lambda1=lambda1,
                    log_threshold=log_threshold)
    assert gr["window"].sum() > 10

    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=k not in ("x", "y", "theta")) for k, v in p.items()}
    tpar = torch.tensor(param, dtype=torch.float64, requires_grad=True)
    tth = torch.exp(tpar) if log_threshold else tpar
    blk, c = {}, 0
    for l in range(L):
        for lp in range(l, L):
            blk[(l, lp)] = c
            c += 1
    pres = [t["x"][l] @ t["W_enc"][l] + t["b_enc"][l] for l in range(L)]
    zs = [_JumpSTE.apply(pres[l], tth[l], eps) for l in range(L)]
    loss = 0.0
    for lp in range(L):
        yh = t["b_dec"][lp] + sum(zs[l] @ t["W_dec"][blk[(l, lp)]] for l in range(lp + 1))
        loss = loss + ((yh - t["y"][lp]) ** 2).sum() / B
    for l in range(L):
        nrm = torch.cat([t["W_dec"][blk[(l, lp)]] for lp in range(l, L)], dim=1).norm(dim=1)
        loss = loss + lambda0 * torch.tanh(C * zs[l] * nrm).sum() / B
        loss = loss + lambda1 * (torch.relu(tth[l] - pres[l]) * nrm).sum() / B
    loss.backward()
    assert abs(float(loss.detach()) - tot) < 1e-12 * max(1.0, abs(tot))
    for k in ("W_enc", "b_enc", "W_dec", "b_dec"):
        np.testing.assert_allclose(gr["d" + k], t[k].grad.numpy(), rtol=1e-10, atol=1e-12, err_msg=k)
    np.testing.assert_allclose(gr["dtheta"], tpar.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_train_step_with_dead_term_moves_threshold_parameter():
    rng = np.random.default_rng(11)
    L, d, F, B = 2, 4, 6, 8
    p = rand_problem(rng, L, d, F, B, theta=0.1)
    params = {k: p[k] for k in O.PARAM_NAMES}
    params["theta"] = np.log(params["theta"])
    zeros = {k: np.zeros_like(v) for k, v in params.items()}
    newp, m, v, info = O.train_step(p["x"], p["y"], params, zeros, zeros, 1, 2e-4, 0.0, 2.0, 1e-7,
                                    lambda1=1.0, log_threshold=True)
    g = info["grads"]["dtheta"]
    assert (g >= 0).all() and (g > 0).any()          # only the dead term acts: it lowers the thresholds
    assert ((newp["theta"] - params["theta"])[g > 1e-6] < 0).all()


def test_below_tie_break_is_honoured_only_inside_the_band():
    rng = np.random.default_rng(13)
    L, d, F, B = 2, 4, 6, 8
    p = rand_problem(rng, L, d, F, B, theta=0.1)
    fwd = O.forward(p["x"], p["W_enc"], p["b_enc"], p["theta"], p["W_dec"], p["b_dec"])
    below = fwd["pre"] < p["theta"][:, None, :]
    dist = np.abs(fwd["pre"] - p["theta"][:, None, :])
    idx = np.unravel_index(np.argmin(dist), dist.shape)
    band = 0.5 * (float(dist[idx]) + float(np.sort(dist.ravel())[1]))
    assert (dist < band).sum() == 1
    forced = below.copy()
    forced[idx] = ~forced[idx]
    kw = dict(lambda0=0.3, C=2.0, eps=0.05, lambda1=0.8)
    base = O.backward(p["x"], p["y"], p["theta"], p["W_dec"], fwd, **kw)
    flip = O.backward(p["x"], p["y"], p["theta"], p["W_dec"], fwd, band=band, below_tie_break=forced, **kw)
    l, b, f = idx
    n = O.decoder_norms(p["W_dec"], L)
    sign = 1.0 if forced[idx] else -1.0        # one more (or one fewer) entry counted as below
    assert abs((flip["dtheta"] - base["dtheta"])[l, f] - sign * 0.8 / B * n[l, f]) < 1e-12
    assert abs((flip["dpre"] - base["dpre"])[idx] + sign * 0.8 / B * n[l, f]) < 1e-12
    d_th = flip["dtheta"] - base["dtheta"]
    d_th[l, f] = 0.0
    assert not d_th.any()
    with pytest.raises(ValueError):
        O.backward(p["x"], p["y"], p["theta"], p["W_dec"], fwd, band=float(dist[idx]) * 0.5, below_tie_break=forced, **kw)
