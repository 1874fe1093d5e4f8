"""CPU oracle for one cross-layer-transcoder (CLT) training step.

TEST INFRASTRUCTURE ONLY.  This module is the plain, slow, obviously-correct
definition that the HIP library is checked against.  It may be imported only by
tests, by the smoke check and by the benchmark's CPU-baseline leg; the product
path never calls it and it shares no code with the HIP path.

Everything is numpy float64.  Each function is the paper's definition written
out, with matmul as the only library step and no blocking, fusion or
reordering:

  encoder pre-activation ........ Sec. 2.1, eq. (1)
  JumpReLU ...................... Sec. 2.1 / Sec. 3.2 (named there; the form
                                  z = pre * H(pre - theta), strict ">", is the
                                  one of the JumpReLU literature the paper
                                  follows for its training recipe)
  TopK .......................... Sec. 3.2 names it as the alternative activation
                                  without a formula; taken as: per token and
                                  layer keep the k largest pre-activations
  cross-layer decode ............ Sec. 2.1, eq. (3); eq. (2) is its L = 1 case
  decoder norms ................. App. B: norm of the concatenation of all
                                  decoders that leave a source layer
  objective ..................... App. B training objective: reconstruction,
                                  sparsity and (optional, lambda_1 > 0) the
                                  dead-feature penalty with theta = exp(tau)
  backward ...................... chain rule through the above; the threshold
                                  gets the rectangle-kernel straight-through
                                  pseudo-gradient
  Adam .......................... App. C, Table 1 (betas, learning rate); bias
                                  correction on, eps outside the square root
  activation normalisation ...... Sec. 3.1, last paragraph: every activation is
                                  divided by a factor estimated from the first
                                  N batches so that norms come out near one;
                                  taken as: one factor per layer (and per side,
                                  inputs and targets), the mean L2 norm of that
                                  layer's token vectors over those batches

Storage conventions (they only transpose the paper's matrices):
  x      [L, B, d]   MLP inputs h_l per layer and token
  y      [L, B, d]   MLP outputs m_l (reconstruction targets)
  W_enc  [L, d, F]   pre = x @ W_enc[l] + b_enc[l]
  b_enc  [L, F], theta [L, F]
  W_dec  [P, F, d]   P = L(L+1)/2 blocks, block p(l, l') maps source l to
                     target l' >= l; source-major packing, see packed_index
  b_dec  [L, d]

Readings taken where the paper is silent: the loss sums over layers, model dims
and features and takes the mean over the B tokens; the decoder norm is
differentiated; dn/dW uses max(n, 1e-30) so an all-zero decoder row gives 0; the
dead-feature term has its true derivatives (no straight-through), ReLU'(0) = 0.

Parity pins (tests/test_oracle_*.py): brute-force Python loops, closed forms,
special cases that reduce to torch.nn.functional.linear / torch.optim.Adam,
central finite differences, a torch-autograd re-derivation, a hand-worked
example, and the paper's printed parameter count.  The threshold
pseudo-gradient is a definition, not a derivative, so finite differences cannot
pin it; it is pinned by the hand-worked example, by the autograd re-derivation
and by the "empty window gives zero" invariant.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# packed triangular decoder (eq. 3: sum over source layers l <= l')
# --------------------------------------------------------------------------
def num_blocks(L: int) -> int:
    """Number of (source, target) decoder blocks with l <= l' (eq. 3)."""
    return L * (L + 1) // 2


def packed_index(l: int, lp: int, L: int) -> int:
    """Block index of the decoder W_dec^{l -> l'} in source-major packing.

    Source 0 owns blocks 0..L-1 (targets 0..L-1), source 1 the next L-1
    (targets 1..L-1), and so on, so that all decoders leaving one source layer
    are contiguous (the "concatenation" whose norm App. B uses).
    """
    if not (0 <= l <= lp < L):
        raise ValueError("need 0 <= l <= l' < L")
    return l * L - l * (l - 1) // 2 + (lp - l)


def decoder_param_count(L: int, d: int, e: int) -> int:
    """App. B parameter formula: (L(L-1)/2 + L) * e * d^2."""
    return (L * (L - 1) // 2 + L) * e * d * d


# --------------------------------------------------------------------------
# forward
# --------------------------------------------------------------------------
def encoder_preact(x, W_enc, b_enc):
    """eq. (1) before the nonlinearity: pre[l] = x[l] @ W_enc[l] + b_enc[l]."""
    x = np.asarray(x, F64)
    W_enc = np.asarray(W_enc, F64)
    b_enc = np.asarray(b_enc, F64)
    L = x.shape[0]
    pre = np.empty((L, x.shape[1], W_enc.shape[2]), F64)
    for l in range(L):
        pre[l] = x[l] @ W_enc[l] + b_enc[l][None, :]
    return pre


def jumprelu(pre, theta, tie_break=None, band=0.0):
    """JumpReLU: z = pre where pre > theta (strictly), else 0.

    `tie_break`, if given, is a boolean array of forced decisions that is
    honoured only where |pre - theta| < band: there both decisions are valid
    results for an implementation whose pre-activation differs from this one by
    rounding, and a caller may ask which of the valid results to continue with.
    Outside the band the forced value must agree with the oracle's own.
    """
    pre = np.asarray(pre, F64)
    theta = np.asarray(theta, F64)
    active = pre > theta[:, None, :]
    if tie_break is not None:
        tb = np.asarray(tie_break, bool)
        inband = np.abs(pre - theta[:, None, :]) < band
        if np.any((tb != active) & ~inband):
            raise ValueError("tie_break disagrees with the oracle outside the band")
        active = np.where(inband, tb, active)
    z = np.where(active, pre, 0.0)
    return z, active


def topk_activation(pre, k, tie_break=None, band=0.0):
    """TopK activation: for every (layer, token) row of pre [L, B, F] keep the k
    largest entries (z = pre there, whatever its sign) and zero the rest; among
    equal values the lower feature index wins.  Returns (z, active).

    `tie_break` (boolean, same shape) is honoured only for entries within `band`
    of the row's k-th largest value, where an implementation whose
    pre-activation differs by rounding may rank differently; it must select
    exactly k entries per row and agree with the oracle outside the band.
    """
    pre = np.asarray(pre, F64)
    L, B, F = pre.shape
    k = int(k)
    if not 0 <= k <= F:
        raise ValueError("k out of range")
    active = np.zeros(pre.shape, bool)
    if k > 0:
        # stable sort of -pre: descending values, ascending index among equals
        order = np.argsort(-pre, axis=2, kind="stable")
        np.put_along_axis(active, order[:, :, :k], True, axis=2)
    if tie_break is not None and 0 < k < F:
        tb = np.asarray(tie_break, bool)
        kth = np.take_along_axis(pre, order[:, :, k - 1:k], axis=2)      # [L, B, 1]
        inband = np.abs(pre - kth) < band
        if np.any((tb != active) & ~inband):
            raise ValueError("top-k tie_break disagrees with the oracle outside the band")
        if np.any(tb.sum(axis=2) != k):
            raise ValueError("top-k tie_break does not select k entries in every row")
        active = tb
    z = np.where(active, pre, 0.0)
    return z, active


def ste_window(pre, theta, eps, tie_break=None, band=0.0):
    """Support of the rectangle kernel: |pre - theta| < eps / 2 (strict)."""
    pre = np.asarray(pre, F64)
    theta = np.asarray(theta, F64)
    dist = np.abs(pre - theta[:, None, :])
    win = dist < 0.5 * eps
    if tie_break is not None:
        tb = np.asarray(tie_break, bool)
        inband = np.abs(dist - 0.5 * eps) < band
        if np.any((tb != win) & ~inband):
            raise ValueError("window tie_break disagrees outside the band")
        win = np.where(inband, tb, win)
    return win


def decode(z, W_dec, b_dec):
    """eq. (3): y_hat[l'] = b_dec[l'] + sum_{l <= l'} z[l] @ W_dec[p(l, l')].

    Written as the explicit loop over (target, source) pairs.
    """
    z = np.asarray(z, F64)
    b_dec = np.asarray(b_dec, F64)
    L, B, _ = z.shape
    d = b_dec.shape[1]
    y_hat = np.empty((L, B, d), F64)
    for lp in range(L):
        acc = np.tile(b_dec[lp][None, :], (B, 1))
        for l in range(lp + 1):
            acc += z[l] @ np.asarray(W_dec[packed_index(l, lp, L)], F64)
        y_hat[lp] = acc
    return y_hat


def decoder_norms(W_dec, L):
    """App. B: n[l, f] = l2 norm of feature f's rows over all blocks l -> l'."""
    F = W_dec.shape[1]
    n2 = np.zeros((L, F), F64)
    for l in range(L):
        for lp in range(l, L):
            Wb = np.asarray(W_dec[packed_index(l, lp, L)], F64)
            n2[l] += np.sum(Wb * Wb, axis=1)
    return np.sqrt(n2)


def loss_terms(y_hat, y, z, n, lambda0, C):
    """App. B objective, lambda_1 = 0, mean over the B tokens.

    L_rec = (1/B) sum_{l', b, j} (y_hat - y)^2
    L_sp  = (lambda0/B) sum_{l, b, f} tanh(C * z * n[l, f])
    """
    y = np.asarray(y, F64)
    B = y.shape[1]
    r = y_hat - y
    L_rec = np.sum(r * r) / B
    L_sp = lambda0 * np.sum(np.tanh(C * z * n[:, None, :])) / B
    return L_rec + L_sp, L_rec, L_sp


def dead_feature_term(pre, theta, n, lambda1):
    """App. B dead-feature penalty, mean over the B tokens:

    L_dead = (lambda1/B) sum_{l, b, f} ReLU(theta[l,f] - pre[l,b,f]) * n[l,f]

    where theta = exp(tau) is the JumpReLU threshold in its log parameterisation
    and n the decoder norm of the feature.
    """
    pre = np.asarray(pre, F64)
    theta = np.asarray(theta, F64)
    B = pre.shape[1]
    return lambda1 * np.sum(np.maximum(theta[:, None, :] - pre, 0.0) * n[:, None, :]) / B


def threshold_value(param, log_threshold):
    """The threshold theta from its stored parameter: theta itself, or exp(tau)."""
    param = np.asarray(param, F64)
    return np.exp(param) if log_threshold else param


def forward(x, W_enc, b_enc, theta, W_dec, b_dec, tie_break=None, band=0.0, topk=None):
    """Encoder, activation (JumpReLU with thresholds theta, or TopK with k = topk and
    theta ignored), cross-layer decode.  Returns a dict of intermediates."""
    pre = encoder_preact(x, W_enc, b_enc)
    if topk is None:
        z, active = jumprelu(pre, theta, tie_break, band)
    else:
        z, active = topk_activation(pre, topk, tie_break, band)
    y_hat = decode(z, W_dec, b_dec)
    return {"pre": pre, "z": z, "active": active, "y_hat": y_hat,
            "l0_per_layer": active.sum(axis=(1, 2))}


# --------------------------------------------------------------------------
# backward
# --------------------------------------------------------------------------
def sparsity_norm_sums(z, n, lambda0, C):
    """G[l,f] = (lambda0/B) sum_b C z sech^2(C z n): derivative of L_sp w.r.t. the decoder norm n[l,f]."""
    z = np.asarray(z, F64)
    B = z.shape[1]
    u = C * z * n[:, None, :]
    with np.errstate(over="ignore"):
        sech2 = 1.0 / np.cosh(u) ** 2
    return (lambda0 / B) * np.sum(C * z * sech2, axis=1)


def backward(x, y, theta, W_dec, fwd, lambda0, C, eps,
             window_tie_break=None, band=0.0, lambda1=0.0, log_threshold=False,
             below_tie_break=None, topk=False):
    """Gradients of L_rec + L_sp (+ L_dead when lambda1 > 0) w.r.t. the five
    parameter tensors.  `theta` is the threshold value; with log_threshold the
    stored parameter is tau = log(theta) and "dtheta" is the gradient w.r.t. tau.

    d y_hat = 2 (y_hat - y) / B
    dz[l]   = sum_{l' >= l} d y_hat[l'] @ W_dec[p(l,l')]^T
              + (lambda0/B) C n sech^2(C z n)
    dpre    = dz where active, else 0              (no pseudo-term on pre)
    dtheta  = -(theta/eps) sum_b [ |pre-theta| < eps/2 ] dz
    dW_dec[p(l,l')] = z[l]^T @ d y_hat[l'] + (G[l,f]/n[l,f]) W_dec[p(l,l')][f,:]
              with G[l,f] = (lambda0/B) sum_b C z sech^2(C z n)
    db_dec  = sum_b d y_hat,  dW_enc[l] = x[l]^T @ dpre[l],  db_enc = sum_b dpre
    Dead-feature term (true derivatives of ReLU(theta - pre) n, ReLU'(0) = 0):
      dpre   += -(lambda1/B) n      where pre < theta
      dtheta += +(lambda1/B) n sum_b [pre < theta]
      G      += (lambda1/B) sum_b ReLU(theta - pre)      (the term's d/dn, enters dW_dec as G W / n)
    `below_tie_break` forces the decision pre < theta where |pre - theta| < band,
    under the same rule as jumprelu's tie_break.
    With topk the activation was TopK: the selected set is piecewise constant in
    the parameters, so d pre = dz on it and there is no threshold (dtheta = 0).
    """
    x = np.asarray(x, F64)
    y = np.asarray(y, F64)
    theta = np.asarray(theta, F64)
    L, B, d = x.shape
    z, pre, active, y_hat = fwd["z"], fwd["pre"], fwd["active"], fwd["y_hat"]
    F = z.shape[2]
    n = decoder_norms(W_dec, L)

    d_yhat = 2.0 * (y_hat - y) / B
    u = C * z * n[:, None, :]
    with np.errstate(over="ignore"):
        sech2 = 1.0 / np.cosh(u) ** 2
    g_sp = (lambda0 / B) * C * n[:, None, :] * sech2
    G = sparsity_norm_sums(z, n, lambda0, C)                   # [L, F]

    dz = g_sp.copy()
    for l in range(L):
        for lp in range(l, L):
            dz[l] += d_yhat[lp] @ np.asarray(W_dec[packed_index(l, lp, L)], F64).T
    dpre = np.where(active, dz, 0.0)
    below = pre < theta[:, None, :]
    if below_tie_break is not None:
        tb = np.asarray(below_tie_break, bool)
        inband = np.abs(pre - theta[:, None, :]) < band
        if np.any((tb != below) & ~inband):
            raise ValueError("below tie_break disagrees with the oracle outside the band")
        below = np.where(inband, tb, below)
    if lambda1 != 0.0:
        dpre = dpre + np.where(below, -(lambda1 / B) * n[:, None, :], 0.0)
        G = G + (lambda1 / B) * np.sum(np.maximum(theta[:, None, :] - pre, 0.0), axis=1)
    if topk:
        if lambda1 != 0.0:
            raise ValueError("the dead-feature term needs a threshold")
        win = np.zeros(pre.shape, bool)
    else:
        win = ste_window(pre, theta, eps, window_tie_break, band)
    # sum over the window entries of the per-entry pseudo-derivative -(theta/eps) dz;
    # an empty window contributes exactly 0, also for a non-finite threshold
    with np.errstate(invalid="ignore"):
        dtheta = np.sum(np.where(win, -(theta[:, None, :] / eps) * dz, 0.0), axis=1)
    if lambda1 != 0.0:
        dtheta = dtheta + (lambda1 / B) * n * below.sum(axis=1)
    if log_threshold:
        dtheta = dtheta * theta          # chain rule through theta = exp(tau)
    db_enc = dpre.sum(axis=1)

    dW_dec = np.empty((num_blocks(L), F, d), F64)
    n_safe = np.maximum(n, 1e-30)
    for l in range(L):
        for lp in range(l, L):
            p = packed_index(l, lp, L)
            Wb = np.asarray(W_dec[p], F64)
            dW_dec[p] = z[l].T @ d_yhat[lp] + (G[l] / n_safe[l])[:, None] * Wb
    db_dec = d_yhat.sum(axis=1)

    dW_enc = np.empty((L, d, F), F64)
    for l in range(L):
        dW_enc[l] = x[l].T @ dpre[l]

    return {"dW_enc": dW_enc, "db_enc": db_enc, "dtheta": dtheta,
            "dW_dec": dW_dec, "db_dec": db_dec,
            "d_yhat": d_yhat, "dz": dz, "dpre": dpre, "window": win,
            "n": n, "G": G}


# --------------------------------------------------------------------------
# Adam (App. C Table 1: betas (0.9, 0.999), learning rate 2e-4)
# --------------------------------------------------------------------------
def adam_update(p, g, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam step, 1-based step count t.  Returns (p, m, v) as new arrays."""
    p = np.asarray(p, F64)
    g = np.asarray(g, F64)
    m = beta1 * np.asarray(m, F64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, F64) + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    p = p - lr * m_hat / (np.sqrt(v_hat) + eps)
    return p, m, v


PARAM_NAMES = ("W_enc", "b_enc", "theta", "W_dec", "b_dec")


def train_step(x, y, params, m, v, t, lr, lambda0, C, eps,
               beta1=0.9, beta2=0.999, adam_eps=1e-8, lambda1=0.0, log_threshold=False, topk=None):
    """Forward, loss, backward and Adam on all five tensors.

    `params`, `m`, `v` are dicts keyed by PARAM_NAMES (params["theta"] holds tau
    when log_threshold).  Returns (new_params, new_m, new_v, info) with info
    holding forward values, loss terms and gradients.
    """
    theta = threshold_value(params["theta"], log_threshold)
    fwd = forward(x, params["W_enc"], params["b_enc"], theta, params["W_dec"], params["b_dec"], topk=topk)
    L = np.asarray(x).shape[0]
    n = decoder_norms(params["W_dec"], L)
    total, rec, sp = loss_terms(fwd["y_hat"], y, fwd["z"], n, lambda0, C)
    total = total + dead_feature_term(fwd["pre"], theta, n, lambda1)
    grads = backward(x, y, theta, params["W_dec"], fwd, lambda0, C, eps,
                     lambda1=lambda1, log_threshold=log_threshold, topk=topk is not None)
    new_p, new_m, new_v = {}, {}, {}
    for k in PARAM_NAMES:
        new_p[k], new_m[k], new_v[k] = adam_update(
            params[k], grads["d" + k], m[k], v[k], t, lr, beta1, beta2, adam_eps)
    info = {"fwd": fwd, "loss": (total, rec, sp), "grads": grads}
    return new_p, new_m, new_v, info


# --------------------------------------------------------------------------
# int8 activation cache (Sec. 3.1): the step consumes dequantised values
# --------------------------------------------------------------------------
def dequantize_rows(q, s):
    """x[l, b, :] = q[l, b, :] * s[l, b] for symmetric int8 codes q."""
    return np.asarray(q, F64) * np.asarray(s, F64)[:, :, None]


# --------------------------------------------------------------------------
# activation normalisation (Sec. 3.1): factor from the first N batches
# --------------------------------------------------------------------------
def normalisation_factor(batches):
    """c[l] = mean over every token of every batch of ||a[l, b, :]||_2.

    batches: iterable of [L, B_i, d] arrays (the first N batches of one side,
    inputs or targets).  A layer whose activations are all zero has no scale;
    it gets c = 1 so that dividing by it leaves the zeros alone."""
    total, count = None, 0
    for a in batches:
        a = np.asarray(a, F64)
        row_norms = np.sqrt((a * a).sum(axis=2))      # [L, B_i]
        s = row_norms.sum(axis=1)
        total = s if total is None else total + s
        count += a.shape[1]
    c = total / count
    return np.where(c > 0.0, c, 1.0)


def normalise_activations(a, c):
    """a[l, b, :] / c[l]."""
    return np.asarray(a, F64) / np.asarray(c, F64)[:, None, None]

