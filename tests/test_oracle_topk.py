"""Pins for the oracle's TopK activation (Sec. 3.2 names TopK as the alternative to
JumpReLU; reading: per token and layer the k largest pre-activations).  CPU only."""
import numpy as np
import pytest
import torch

from oracle import clt_oracle as O
from test_oracle_pins import rand_problem


def test_topk_against_python_sort_and_handmade_rows():
    rng = np.random.default_rng(3)
    pre = rng.standard_normal((2, 3, 9))
    pre[0, 1, 2] = pre[0, 1, 5]                      # an exact tie
    for k in (0, 1, 4, 9):
        z, act = O.topk_activation(pre, k)
        for l in range(2):
            for b in range(3):
                order = sorted(range(9), key=lambda f: (-pre[l, b, f], f))     # value descending, index ascending
                want = set(order[:k])
                assert set(np.nonzero(act[l, b])[0]) == want
                for f in range(9):
                    assert z[l, b, f] == (pre[l, b, f] if f in want else 0.0)
    row = np.array([[[1.0, 3.0, 3.0, 2.0]]])
    assert O.topk_activation(row, 1)[1].tolist() == [[[False, True, False, False]]]    # lower index wins the tie
    assert O.topk_activation(row, 2)[1].tolist() == [[[False, True, True, False]]]
    neg = np.array([[[-1.0, -2.0, -3.0]]])
    assert O.topk_activation(neg, 1)[0].tolist() == [[[-1.0, 0.0, 0.0]]]                # the sign does not matter
    with pytest.raises(ValueError):
        O.topk_activation(row, 5)


def test_topk_against_torch_topk():
    rng = np.random.default_rng(4)
    pre = rng.standard_normal((3, 17, 64))
    for k in (1, 7, 63):
        z, act = O.topk_activation(pre, k)
        vals, idx = torch.topk(torch.tensor(pre), k, dim=2)
        want = torch.zeros(pre.shape, dtype=torch.float64).scatter_(2, idx, vals).numpy()
        assert (z == want).all()
        assert (act.sum(axis=2) == k).all()


def test_topk_limits_reduce_to_known_models():
    """k = F keeps everything (the linear model, as JumpReLU with theta = -inf); k = 0 keeps
    nothing (every target is reconstructed by its decoder bias)."""
    rng = np.random.default_rng(5)
    L, d, F, B = 3, 4, 6, 5
    p = rand_problem(rng, L, d, F, B)
    full = O.forward(p["x"], p["W_enc"], p["b_enc"], None, p["W_dec"], p["b_dec"], topk=F)
    lin = O.forward(p["x"], p["W_enc"], p["b_enc"], np.full((L, F), -np.inf), p["W_dec"], p["b_dec"])
    assert (full["z"] == full["pre"]).all() and np.allclose(full["y_hat"], lin["y_hat"], rtol=0, atol=1e-13)
    none = O.forward(p["x"], p["W_enc"], p["b_enc"], None, p["W_dec"], p["b_dec"], topk=0)
    assert not none["z"].any()
    for lp in range(L):
        assert (none["y_hat"][lp] == p["b_dec"][lp][None, :]).all()


def test_topk_tie_break_rule():
    rng = np.random.default_rng(6)
    pre = rng.standard_normal((1, 2, 12))
    k = 4
    _, act = O.topk_activation(pre, k)
    srt = np.sort(pre[0, 0])[::-1]
    kth, nxt = srt[k - 1], srt[k]
    band = (kth - nxt) * 1.01                        # holds the k-th and the (k+1)-th value of row 0, nothing more of it
    i_k, i_n = int(np.where(pre[0, 0] == kth)[0][0]), int(np.where(pre[0, 0] == nxt)[0][0])
    forced = act.copy()
    forced[0, 0, i_k], forced[0, 0, i_n] = False, True       # the other valid choice inside the band
    z, a2 = O.topk_activation(pre, k, tie_break=forced, band=band)
    assert a2[0, 0, i_n] and not a2[0, 0, i_k] and z[0, 0, i_n] == nxt
    with pytest.raises(ValueError):                  # same swap, band too narrow
        O.topk_activation(pre, k, tie_break=forced, band=(kth - nxt) * 0.5)
    bad = act.copy()
    bad[0, 0, i_n] = True                            # k + 1 entries
    with pytest.raises(ValueError):
        O.topk_activation(pre, k, tie_break=bad, band=band)


def topk_loss(p, k, lambda0, C):
    fwd = O.forward(p["x"], p["W_enc"], p["b_enc"], None, p["W_dec"], p["b_dec"], topk=k)
    n = O.decoder_norms(p["W_dec"], p["x"].shape[0])
    return O.loss_terms(fwd["y_hat"], p["y"], fwd["z"], n, lambda0, C)[0], fwd


@pytest.mark.parametrize("lambda0", [0.0, 0.4])
def test_topk_gradients_by_finite_differences(lambda0):
    """Away from rank changes the selected set is constant and the objective is smooth."""
    rng = np.random.default_rng(8)
    L, d, F, B = 3, 5, 8, 4
    p = rand_problem(rng, L, d, F, B, wscale=0.8)
    k, C = 3, 2.0
    _, fwd = topk_loss(p, k, lambda0, C)
    gr = O.backward(p["x"], p["y"], np.zeros((L, F)), p["W_dec"], fwd, lambda0, C, eps=0.05, topk=True)
    assert not gr["dtheta"].any() and not gr["window"].any()
    h = 1e-6
    for name in ("W_enc", "b_enc", "W_dec", "b_dec"):
        g = gr["d" + name]
        for _ in range(25):
            idx = tuple(rng.integers(0, s) for s in g.shape)
            q = {kk: v.copy() for kk, v in p.items()}
            q[name][idx] += h
            lp_, f1 = topk_loss(q, k, lambda0, C)
            q[name][idx] -= 2 * h
            lm_, f2 = topk_loss(q, k, lambda0, C)
            assert (f1["active"] == fwd["active"]).all() and (f2["active"] == fwd["active"]).all()
            fd = (lp_ - lm_) / (2 * h)
            assert abs(fd - g[idx]) <= 2e-6 * max(1.0, abs(g[idx])), (name, idx, fd, g[idx])


def test_topk_gradients_against_torch_autograd():
    rng = np.random.default_rng(9)
    L, d, F, B = 3, 6, 10, 12
    p = rand_problem(rng, L, d, F, B, wscale=0.6)
    k, lambda0, C = 4, 0.7, 2.0
    tot, fwd = topk_loss(p, k, lambda0, C)
    gr = O.backward(p["x"], p["y"], np.zeros((L, F)), p["W_dec"], fwd, lambda0, C, eps=0.05, topk=True)
    t = {kk: torch.tensor(v, dtype=torch.float64, requires_grad=kk in ("W_enc", "b_enc", "W_dec", "b_dec"))
         for kk, v in p.items()}
    blk, c = {}, 0
    for l in range(L):
        for lp in range(l, L):
            blk[(l, lp)] = c
            c += 1
    zs = []
    for l in range(L):
        pre = t["x"][l] @ t["W_enc"][l] + t["b_enc"][l]
        vals, idx = torch.topk(pre, k, dim=1)
        zs.append(torch.zeros_like(pre).scatter(1, idx, vals))
    loss = 0.0
    for lp in range(L):
        yh = t["b_dec"][lp] + sum(zs[l] @ t["W_dec"][blk[(l, lp)]] for l in range(lp + 1))
        loss = loss + ((yh - t["y"][lp]) ** 2).sum() / B
    for l in range(L):
        nrm = torch.cat([t["W_dec"][blk[(l, lp)]] for lp in range(l, L)], dim=1).norm(dim=1)
        loss = loss + lambda0 * torch.tanh(C * zs[l] * nrm).sum() / B
    loss.backward()
    assert abs(float(loss.detach()) - tot) < 1e-12 * max(1.0, abs(tot))
    for kk in ("W_enc", "b_enc", "W_dec", "b_dec"):
        np.testing.assert_allclose(gr["d" + kk], t[kk].grad.numpy(), rtol=1e-10, atol=1e-12, err_msg=kk)


def test_dead_feature_term_is_refused_with_topk():
    rng = np.random.default_rng(10)
    p = rand_problem(rng, 2, 3, 4, 3)
    _, fwd = topk_loss(p, 2, 0.0, 1.0)
    with pytest.raises(ValueError):
        O.backward(p["x"], p["y"], np.zeros((2, 4)), p["W_dec"], fwd, 0.0, 1.0, 0.05, lambda1=0.5, topk=True)
