"""Pins for the CPU oracle (no GPU): each check ties oracle/clt_oracle.py to
something other than itself -- brute-force loops, closed forms, library special
cases, finite differences, a torch-autograd re-derivation, a hand-worked example
and the paper's printed parameter count."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import clt_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split()
            out[k] = float(v)
    return out


def rand_problem(rng, L, d, F, B, theta=0.1, wscale=None):
    P = O.num_blocks(L)
    ws = wscale if wscale is not None else 1.0 / math.sqrt(d)
    return dict(
        x=rng.standard_normal((L, B, d)),
        y=rng.standard_normal((L, B, d)),
        W_enc=rng.uniform(-ws, ws, (L, d, F)),
        b_enc=0.1 * rng.standard_normal((L, F)),
        theta=np.full((L, F), theta),
        W_dec=rng.uniform(-ws, ws, (P, F, d)),
        b_dec=0.1 * rng.standard_normal((L, d)),
    )


# ---------------------------------------------------------------- packing, sizes
def test_packed_index_is_source_major_bijection():
    L = 4
    seen = [O.packed_index(l, lp, L) for l in range(L) for lp in range(l, L)]
    assert seen == list(range(O.num_blocks(L)))           # row by row, no gaps
    assert [O.packed_index(0, t, L) for t in range(4)] == [0, 1, 2, 3]
    assert [O.packed_index(1, t, L) for t in range(1, 4)] == [4, 5, 6]
    assert [O.packed_index(2, t, L) for t in range(2, 4)] == [7, 8]
    assert O.packed_index(3, 3, L) == 9
    with pytest.raises(ValueError):
        O.packed_index(2, 1, L)


def test_param_count_matches_paper_value():
    g = read_golden("param_count.txt")
    n = O.decoder_param_count(int(g["L"]), int(g["d"]), int(g["e"]))
    assert abs(n - g["approx_params"]) / g["approx_params"] < g["rel_tol"]
    # the same number from the packed layout: P blocks of F x d with F = e d
    L, d, e = int(g["L"]), int(g["d"]), int(g["e"])
    assert n == O.num_blocks(L) * (e * d) * d


# ---------------------------------------------------------------- forward pins
def brute_forward(p, L, d, F, B):
    """Pure-Python triple loops straight from eq. (1) and eq. (3)."""
    pre = [[[p["b_enc"][l][f] + sum(p["x"][l][b][i] * p["W_enc"][l][i][f] for i in range(d))
             for f in range(F)] for b in range(B)] for l in range(L)]
    z = [[[pre[l][b][f] if pre[l][b][f] > p["theta"][l][f] else 0.0
           for f in range(F)] for b in range(B)] for l in range(L)]
    yh = [[[0.0] * d for _ in range(B)] for _ in range(L)]
    # enumerate blocks in packed order instead of calling packed_index
    blk = 0
    for l in range(L):
        for lp in range(l, L):
            for b in range(B):
                for j in range(d):
                    yh[lp][b][j] += sum(z[l][b][f] * p["W_dec"][blk][f][j] for f in range(F))
            blk += 1
    for lp in range(L):
        for b in range(B):
            for j in range(d):
                yh[lp][b][j] += p["b_dec"][lp][j]
    return np.array(pre), np.array(z), np.array(yh)


def test_forward_against_brute_force_loops():
    rng = np.random.default_rng(1)
    L, d, F, B = 3, 4, 5, 3
    p = rand_problem(rng, L, d, F, B, theta=0.2, wscale=1.0)
    fwd = O.forward(p["x"], p["W_enc"], p["b_enc"], p["theta"], p["W_dec"], p["b_dec"])
    pre, z, yh = brute_forward(p, L, d, F, B)
    np.testing.assert_allclose(fwd["pre"], pre, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(fwd["z"], z, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(fwd["y_hat"], yh, rtol=1e-12, atol=1e-12)
    assert 0 < fwd["active"].sum() < fwd["active"].size        # both branches exercised


def test_decode_equals_concatenated_sources_per_target():
    """eq. (3) as one matmul per target over the concatenated sources."""
    rng = np.random.default_rng(2)
    L, d, F, B = 4, 6, 7, 5
    p = rand_problem(rng, L, d, F, B)
    z = np.abs(rng.standard_normal((L, B, F))) * (rng.random((L, B, F)) < 0.3)
    got = O.decode(z, p["W_dec"], p["b_dec"])
    starts = np.cumsum([0] + [L - l for l in range(L)])       # first block of each source
    for lp in range(L):
        zcat = np.concatenate([z[l] for l in range(lp + 1)], axis=1)
        Wcat = np.concatenate([p["W_dec"][starts[l] + (lp - l)] for l in range(lp + 1)], axis=0)
        np.testing.assert_allclose(got[lp], zcat @ Wcat + p["b_dec"][lp], rtol=1e-12, atol=1e-12)


def test_single_layer_reduces_to_standard_transcoder():
    """L = 1: eq. (3) is eq. (2), one affine map; check with torch's linear."""
    rng = np.random.default_rng(3)
    d, F, B = 5, 9, 4
    p = rand_problem(rng, 1, d, F, B, theta=-np.inf)
    fwd = O.forward(p["x"], p["W_enc"], p["b_enc"], p["theta"], p["W_dec"], p["b_dec"])
    x = torch.tensor(p["x"][0])
    pre = torch.nn.functional.linear(x, torch.tensor(p["W_enc"][0]).T, torch.tensor(p["b_enc"][0]))
    yh = torch.nn.functional.linear(pre, torch.tensor(p["W_dec"][0]).T, torch.tensor(p["b_dec"][0]))
    np.testing.assert_allclose(fwd["pre"][0], pre.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(fwd["z"][0], pre.numpy(), rtol=1e-12, atol=1e-12)   # theta=-inf: linear
    np.testing.assert_allclose(fwd["y_hat"][0], yh.numpy(), rtol=1e-12, atol=1e-12)


def test_zero_decoder_gives_bias_and_inf_theta_gives_no_activations():
    rng = np.random.default_rng(4)
    L, d, F, B = 3, 4, 6, 5
    p = rand_problem(rng, L, d, F, B)
    fwd = O.forward(p["x"], p["W_enc"], p["b_enc"], p["theta"], np.zeros_like(p["W_dec"]), p["b_dec"])
    for lp in range(L):
        np.testing.assert_array_equal(fwd["y_hat"][lp], np.tile(p["b_dec"][lp], (B, 1)))
    fwd = O.forward(p["x"], p["W_enc"], p["b_enc"], np.full((L, F), np.inf), p["W_dec"], p["b_dec"])
    assert not fwd["z"].any() and fwd["l0_per_layer"].sum() == 0
    n = O.decoder_norms(p["W_dec"], L)
    tot, rec, sp = O.loss_terms(fwd["y_hat"], p["y"], fwd["z"], n, 2.0, 4.0)
    assert sp == 0.0
    want = sum(np.sum((p["b_dec"][lp][None] - p["y"][lp]) ** 2) for lp in range(L)) / B
    assert abs(rec - want) < 1e-12 and tot == rec


def test_one_hot_feature_reads_decoder_rows_and_is_triangular():
    L, d, F, B = 4, 3, 5, 1
    rng = np.random.default_rng(5)
    W_dec = rng.standard_normal((O.num_blocks(L), F, d))
    b_dec = rng.standard_normal((L, d))
    for l in range(L):
        for f in (0, F - 1):
            z = np.zeros((L, B, F))
            z[l, 0, f] = 1.0
            yh = O.decode(z, W_dec, b_dec)
            # enumerate packed order by hand
            blk = sum(L - s for s in range(l))
            for lp in range(L):
                if lp < l:
                    np.testing.assert_array_equal(yh[lp, 0], b_dec[lp])
                else:
                    np.testing.assert_allclose(yh[lp, 0] - b_dec[lp], W_dec[blk + (lp - l), f],
                                               rtol=0, atol=1e-15)


def test_decoder_norm_is_norm_of_concatenated_rows():
    rng = np.random.default_rng(6)
    L, d, F = 3, 4, 5
    W_dec = rng.standard_normal((O.num_blocks(L), F, d))
    n = O.decoder_norms(W_dec, L)
    blk = 0
    for l in range(L):
        rows = np.concatenate([W_dec[blk + t] for t in range(L - l)], axis=1)   # [F, (L-l) d]
        np.testing.assert_allclose(n[l], np.linalg.norm(rows, axis=1), rtol=1e-13)
        blk += L - l


def test_sparsity_term_limits():
    rng = np.random.default_rng(7)
    L, B, F = 2, 6, 8
    z = np.abs(rng.standard_normal((L, B, F))) * (rng.random((L, B, F)) < 0.4)
    n = 0.5 + rng.random((L, F))
    yh = np.zeros((L, B, 3))
    lam = 1.7
    # C large: each active feature costs lambda0, so L_sp -> lambda0 * mean active count
    _, _, sp = O.loss_terms(yh, yh, z, n, lam, 1e9)
    assert abs(sp - lam * (z > 0).sum() / B) < 1e-9
    # C small: tanh(u) ~ u
    C = 1e-7
    _, _, sp = O.loss_terms(yh, yh, z, n, lam, C)
    assert abs(sp - lam * C * np.sum(z * n[:, None, :]) / B) < 1e-18
    # no activations: zero
    assert O.loss_terms(yh, yh, np.zeros_like(z), n, lam, 4.0)[2] == 0.0


# ---------------------------------------------------------------- worked example
def test_hand_worked_example():
    g = read_golden("worked_example.txt")
    x = np.array([[[1.0], [0.5]]])
    y = np.array([[[1.0], [1.0]]])
    W_enc = np.array([[[1.0]]]); b_enc = np.zeros((1, 1)); theta = np.array([[0.4]])
    W_dec = np.array([[[2.0]]]); b_dec = np.zeros((1, 1))
    fwd = O.forward(x, W_enc, b_enc, theta, W_dec, b_dec)
    n = O.decoder_norms(W_dec, 1)
    tot, rec, sp = O.loss_terms(fwd["y_hat"], y, fwd["z"], n, 0.1, 1.0)
    gr = O.backward(x, y, theta, W_dec, fwd, 0.1, 1.0, 0.4)
    tol = 2e-10
    assert abs(rec - g["L_rec"]) < tol and abs(sp - g["L_sp"]) < tol
    assert abs(gr["dz"][0, 0, 0] - g["dz0"]) < tol and abs(gr["dz"][0, 1, 0] - g["dz1"]) < tol
    assert abs(gr["dtheta"][0, 0] - g["dtheta"]) < tol
    assert abs(gr["dW_enc"][0, 0, 0] - g["dW_enc"]) < tol
    assert abs(gr["db_enc"][0, 0] - g["db_enc"]) < tol
    assert abs(gr["dW_dec"][0, 0, 0] - g["dW_dec"]) < tol
    assert abs(gr["db_dec"][0, 0] - g["db_dec"]) < tol


# ---------------------------------------------------------------- gradients
def total_loss(p, lambda0, C):
    fwd = O.forward(p["x"], p["W_enc"], p["b_enc"], p["theta"], p["W_dec"], p["b_dec"])
    n = O.decoder_norms(p["W_dec"], p["x"].shape[0])
    return O.loss_terms(fwd["y_hat"], p["y"], fwd["z"], n, lambda0, C)[0], fwd


@pytest.mark.parametrize("seed,lambda0,C", [(11, 0.0, 1.0), (12, 0.1, 1.0), (13, 2.0, 4.0)])
def test_smooth_gradients_by_central_finite_differences(seed, lambda0, C):
    rng = np.random.default_rng(seed)
    L, d, F, B = 3, 5, 7, 4
    p = rand_problem(rng, L, d, F, B, theta=0.15, wscale=0.8)
    _, fwd = total_loss(p, lambda0, C)
    # stay away from the threshold so no mask entry can flip under the perturbation
    assert np.min(np.abs(fwd["pre"] - p["theta"][:, None, :])) > 1e-3
    assert 0.2 < fwd["active"].mean() < 0.8
    gr = O.backward(p["x"], p["y"], p["theta"], p["W_dec"], fwd, lambda0, C, eps=1e-6)
    h = 1e-6
    for name in ("W_enc", "b_enc", "W_dec", "b_dec"):
        g = gr["d" + name]
        idxs = [tuple(rng.integers(0, s) for s in g.shape) for _ in range(25)]
        for idx in idxs:
            q = {k: v.copy() for k, v in p.items()}
            q[name][idx] += h
            lp_, f1 = total_loss(q, lambda0, C)
            q[name][idx] -= 2 * h
            lm_, f2 = total_loss(q, lambda0, C)
            assert (f1["active"] == fwd["active"]).all() and (f2["active"] == fwd["active"]).all()
            fd = (lp_ - lm_) / (2 * h)
            assert abs(fd - g[idx]) <= 1e-6 * max(1.0, abs(g[idx])), (name, idx, fd, g[idx])


class _JumpSTE(torch.autograd.Function):
    """JumpReLU with the rectangle-kernel pseudo-gradient for the threshold."""

    @staticmethod
    def forward(ctx, pre, theta, eps):
        ctx.save_for_backward(pre, theta)
        ctx.eps = eps
        return torch.where(pre > theta, pre, torch.zeros_like(pre))

    @staticmethod
    def backward(ctx, gout):
        pre, theta = ctx.saved_tensors
        eps = ctx.eps
        gpre = gout * (pre > theta)
        rect = ((pre - theta).abs() < eps / 2).to(gout.dtype)
        gtheta = (-(theta / eps) * rect * gout).sum(dim=0)
        return gpre, gtheta, None


def torch_autograd_grads(p, lambda0, C, eps):
    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=k not in ("x", "y")) for k, v in p.items()}
    L, B, _ = p["x"].shape
    zs, loss = [], 0.0
    for l in range(L):
        pre = t["x"][l] @ t["W_enc"][l] + t["b_enc"][l]
        zs.append(_JumpSTE.apply(pre, t["theta"][l], eps))
    blk = {}
    c = 0
    for l in range(L):
        for lp in range(l, L):
            blk[(l, lp)] = c
            c += 1
    for lp in range(L):
        yh = t["b_dec"][lp] + sum(zs[l] @ t["W_dec"][blk[(l, lp)]] for l in range(lp + 1))
        loss = loss + ((yh - t["y"][lp]) ** 2).sum() / B
    for l in range(L):
        rows = torch.cat([t["W_dec"][blk[(l, lp)]] for lp in range(l, L)], dim=1)
        loss = loss + lambda0 * torch.tanh(C * zs[l] * rows.norm(dim=1)).sum() / B
    loss.backward()
    return float(loss.detach()), {k: t[k].grad.numpy() for k in ("W_enc", "b_enc", "theta", "W_dec", "b_dec")}


@pytest.mark.parametrize("seed", [21, 22])
def test_all_gradients_against_torch_autograd(seed):
    rng = np.random.default_rng(seed)
    L, d, F, B = 3, 6, 10, 16
    p = rand_problem(rng, L, d, F, B, theta=0.2, wscale=0.6)
    lambda0, C, eps = 0.7, 2.0, 0.3
    tot, fwd = total_loss(p, lambda0, C)
    gr = O.backward(p["x"], p["y"], p["theta"], p["W_dec"], fwd, lambda0, C, eps)
    assert gr["window"].sum() > 10            # the pseudo-gradient path is exercised
    assert (gr["window"] & ~fwd["active"]).sum() > 0    # ... also on inactive entries
    tl, tg = torch_autograd_grads(p, lambda0, C, eps)
    assert abs(tl - tot) < 1e-12 * max(1, abs(tot))
    for k in tg:
        np.testing.assert_allclose(gr["d" + k], tg[k], rtol=1e-10, atol=1e-12, err_msg=k)


def test_dtheta_zero_when_window_is_empty():
    rng = np.random.default_rng(31)
    L, d, F, B = 2, 4, 6, 5
    p = rand_problem(rng, L, d, F, B, theta=0.3)
    _, fwd = total_loss(p, 1.0, 2.0)
    gap = np.min(np.abs(fwd["pre"] - p["theta"][:, None, :]))
    gr = O.backward(p["x"], p["y"], p["theta"], p["W_dec"], fwd, 1.0, 2.0, eps=gap)   # strict <
    assert not gr["window"].any() and not gr["dtheta"].any()


def test_zero_decoder_row_gives_finite_zero_norm_gradient():
    rng = np.random.default_rng(32)
    L, d, F, B = 2, 3, 4, 3
    p = rand_problem(rng, L, d, F, B, theta=-1.0)
    p["W_dec"][:, 1, :] = 0.0
    _, fwd = total_loss(p, 1.0, 2.0)
    gr = O.backward(p["x"], p["y"], p["theta"], p["W_dec"], fwd, 1.0, 2.0, 0.1)
    assert np.isfinite(gr["dW_dec"]).all()


def test_tie_break_only_inside_band():
    pre = np.array([[[0.1005, 0.5]]]); theta = np.array([[0.1, 0.1]])
    z, act = O.jumprelu(pre, theta)
    assert act.tolist() == [[[True, True]]]
    z2, act2 = O.jumprelu(pre, theta, tie_break=np.array([[[False, True]]]), band=1e-3)
    assert act2.tolist() == [[[False, True]]] and z2[0, 0, 0] == 0.0
    with pytest.raises(ValueError):
        O.jumprelu(pre, theta, tie_break=np.array([[[True, False]]]), band=1e-3)


def test_window_tie_break_only_inside_band():
    """Hand-made distances to the window edge eps/2 = 0.05: well inside, just inside the edge, just outside it,
    well outside.  A forced decision is taken only for the two entries within the band around the edge, changes
    the threshold gradient by exactly those entries' terms, and is refused anywhere else."""
    theta = np.array([[0.2, 0.2, 0.2, 0.2]])
    pre = np.array([[[0.21, 0.2496, 0.1497, 0.4]]])          # |pre - theta| = 0.01, 0.0496, 0.0503, 0.2
    eps, band = 0.1, 1e-3
    assert O.ste_window(pre, theta, eps).tolist() == [[[True, True, False, False]]]
    forced = np.array([[[True, False, True, False]]])         # both edge entries flipped
    assert O.ste_window(pre, theta, eps, tie_break=forced, band=band).tolist() == forced.tolist()
    for bad in ([[[False, True, False, False]]], [[[True, True, False, True]]]):     # flips outside the band
        with pytest.raises(ValueError):
            O.ste_window(pre, theta, eps, tie_break=np.array(bad), band=band)
    with pytest.raises(ValueError):                           # the same edge flip with a band too narrow to hold it
        O.ste_window(pre, theta, eps, tie_break=forced, band=1e-4)
    # through backward: d theta = -(theta/eps) * (sum of dz over the window), so the forced window moves it by
    # -(theta/eps) * (dz[entry 2] - dz[entry 1]) and nothing else changes
    rng = np.random.default_rng(35)
    L, d, F, B = 1, 3, 4, 1
    p = rand_problem(rng, L, d, F, B, theta=0.2)
    fwd = {"pre": pre, "active": pre > theta[:, None, :], "z": np.where(pre > theta[:, None, :], pre, 0.0)}
    fwd["y_hat"] = O.decode(fwd["z"], p["W_dec"], p["b_dec"])
    own = O.backward(p["x"], p["y"], theta, p["W_dec"], fwd, 1.0, 2.0, eps)
    flip = O.backward(p["x"], p["y"], theta, p["W_dec"], fwd, 1.0, 2.0, eps, window_tie_break=forced, band=band)
    dz = own["dz"][0, 0]
    np.testing.assert_allclose(flip["dtheta"][0] - own["dtheta"][0],
                               -(0.2 / eps) * np.array([0.0, -dz[1], dz[2], 0.0]), rtol=1e-12, atol=1e-15)
    for k in ("dW_enc", "db_enc", "dW_dec", "db_dec", "dpre"):
        assert (flip[k] == own[k]).all(), k


@pytest.mark.parametrize("inf", [np.inf, -np.inf])
def test_infinite_threshold_has_zero_threshold_gradient(inf):
    """theta = +inf (nothing active, eq. 1 reduces to z = 0) and theta = -inf (JumpReLU is the identity, the linear
    model): no pre-activation is within eps/2 of the threshold, so the rectangle kernel is zero everywhere and the
    threshold pseudo-gradient is exactly 0 -- a sum over an empty set, not (theta/eps) times an empty sum, which
    would be inf * 0.  Every other gradient stays finite; at -inf they are those of the linear model."""
    rng = np.random.default_rng(36)
    L, d, F, B = 2, 3, 5, 4
    p = rand_problem(rng, L, d, F, B)
    theta = np.full((L, F), inf)
    fwd = O.forward(p["x"], p["W_enc"], p["b_enc"], theta, p["W_dec"], p["b_dec"])
    gr = O.backward(p["x"], p["y"], theta, p["W_dec"], fwd, 1.0, 2.0, 0.1)
    assert not gr["window"].any()
    assert (gr["dtheta"] == 0.0).all()
    for k in ("dW_enc", "db_enc", "dW_dec", "db_dec"):
        assert np.isfinite(gr[k]).all(), k
    if inf > 0:
        assert not fwd["active"].any() and not gr["dW_enc"].any() and not gr["db_enc"].any()
    else:
        assert fwd["active"].all() and (fwd["z"] == fwd["pre"]).all()
        assert (gr["dpre"] == gr["dz"]).all()
        # the linear model's encoder-bias gradient by central differences (no mask can flip)
        def loss_at(b_enc):
            f = O.forward(p["x"], p["W_enc"], b_enc, theta, p["W_dec"], p["b_dec"])
            return O.loss_terms(f["y_hat"], p["y"], f["z"], O.decoder_norms(p["W_dec"], L), 1.0, 2.0)[0]
        h = 1e-6
        for (l, f) in ((0, 0), (1, 3)):
            bp, bm = p["b_enc"].copy(), p["b_enc"].copy()
            bp[l, f] += h; bm[l, f] -= h
            assert abs((loss_at(bp) - loss_at(bm)) / (2 * h) - gr["db_enc"][l, f]) < 1e-6 * max(1.0, abs(gr["db_enc"][l, f]))


# ---------------------------------------------------------------- Adam
def test_adam_first_step_closed_form():
    rng = np.random.default_rng(41)
    g = rng.standard_normal(50) * 10.0 ** rng.integers(-4, 2, 50)
    p0 = rng.standard_normal(50)
    p1, m1, v1 = O.adam_update(p0, g, np.zeros(50), np.zeros(50), 1, 2e-4)
    np.testing.assert_allclose(p1 - p0, -2e-4 * g / (np.abs(g) + 1e-8), rtol=1e-9, atol=0)
    np.testing.assert_allclose(m1, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v1, 0.001 * g * g, rtol=1e-12)


def test_adam_two_steps_against_torch_optim():
    rng = np.random.default_rng(42)
    p0 = rng.standard_normal((7, 3))
    gs = [rng.standard_normal((7, 3)), rng.standard_normal((7, 3))]
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([tp], lr=2e-4, betas=(0.9, 0.999), eps=1e-8)
    p, m, v = p0, np.zeros_like(p0), np.zeros_like(p0)
    for t, g in enumerate(gs, start=1):
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        p, m, v = O.adam_update(p, g, m, v, t, 2e-4, 0.9, 0.999, 1e-8)
        np.testing.assert_allclose(p, tp.detach().numpy(), rtol=1e-12, atol=1e-15)


def test_train_step_moves_every_parameter_against_its_gradient():
    rng = np.random.default_rng(43)
    L, d, F, B = 2, 4, 6, 8
    p = rand_problem(rng, L, d, F, B, theta=0.1)
    params = {k: p[k] for k in O.PARAM_NAMES}
    zeros = {k: np.zeros_like(v) for k, v in params.items()}
    newp, m, v, info = O.train_step(p["x"], p["y"], params, zeros, zeros, 1, 2e-4, 1.0, 2.0, 0.3)
    for k in O.PARAM_NAMES:
        g = info["grads"]["d" + k]
        nz = np.abs(g) > 1e-6
        np.testing.assert_allclose((newp[k] - params[k])[nz], -2e-4 * np.sign(g[nz]), rtol=1e-2)
        assert ((newp[k] - params[k])[g == 0] == 0).all()


# ---------------------------------------------------------------- int8 rows
def test_dequantize_rows_roundtrip_bound():
    from workloads import clt_synth as S
    g = torch.Generator().manual_seed(5)
    x = torch.randn((2, 7, 16), generator=g) * 3
    x[1, 3] = 0.0
    q, s = S.quantize_rows_int8(x)
    assert q.dtype == torch.int8 and int(q.abs().max()) <= 127 and float(s[1, 3]) == 1.0
    xd = O.dequantize_rows(q.numpy(), s.numpy())
    assert np.all(np.abs(xd - x.numpy().astype(np.float64)) <= 0.5 * s.numpy()[:, :, None] * (1 + 1e-6))
    assert not xd[1, 3].any()
