"""Helpers shared by the GPU parity tests: run one CLT train step through the
C ABI and through the CPU oracle on the same seeded inputs, and compare."""
from __future__ import annotations

import numpy as np
import torch

from oracle import clt_oracle as O
from workloads import clt_synth as S

MATS = ("W_enc", "W_dec")
MASK_BAND = 1e-3     # pre-activations this close to a decision boundary may fall either way


def rel_l2(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


class GpuRun:
    """One forward/loss/backward/Adam pass of the HIP library; results as numpy."""

    def __init__(self, w: S.CLTWorkload, params, x, y, t=1, m=None, v=None, x_scale=None, y_scale=None,
                 theta=None, decode_mode=1, gather_density_threshold=0.004, fused=False):
        from paper_2603_21014_amd import binding as K
        dev = "cuda:0"
        T = torch.float32 if w.dtype == "f32" else torch.bfloat16
        TX = torch.int8 if w.int8_inputs else T
        gp = {k: p.to(dev, T if k in MATS else torch.float32).contiguous() for k, p in params.items()}
        if theta is not None:
            gp["theta"] = theta.to(dev, torch.float32).contiguous()
        zeros = lambda: {k: torch.zeros(p.shape, dtype=torch.float32, device=dev) for k, p in gp.items()}
        gm = zeros() if m is None else {k: a.to(dev, torch.float32).contiguous() for k, a in m.items()}
        gv = zeros() if v is None else {k: a.to(dev, torch.float32).contiguous() for k, a in v.items()}
        master = None
        if w.master_weights:
            master = {k: params[k].to(dev, torch.float32).contiguous() for k in MATS}
        step = K.CLTStep(w.L, w.d, w.F, w.B, dtype=w.dtype, int8_inputs=w.int8_inputs,
                         master_weights=w.master_weights, C_=w.C, ste_bandwidth=w.ste_eps, device=dev,
                         decode_mode=decode_mode, gather_density_threshold=gather_density_threshold,
                         log_threshold=w.log_threshold, topk=w.topk or None)
        xg, yg = x.to(dev, TX).contiguous(), y.to(dev, TX).contiguous()
        xs = x_scale.to(dev) if x_scale is not None else None
        ys = y_scale.to(dev) if y_scale is not None else None
        step.forward(xg, gp, xs)
        self.loss = step.loss(yg, w.lambda0, ys, to_host=True, lambda1=w.lambda1, params=gp)
        self.norms = to_np(K.clt_workspace_view(step.H, "norms"))
        self.d_yhat = to_np(K.clt_workspace_view(step.H, "d_yhat"))
        self.G = to_np(K.clt_workspace_view(step.H, "G"))
        if fused:     # backward and Adam in one call, Adam inside the weight-gradient GEMM epilogues
            step.backward_adam_step(xg, gp, gm, gv, t, w.lr, master, xs)
        else:
            step.backward(xg, gp, xs)
        self.dpre = to_np(K.clt_workspace_view(step.H, "dpre"))
        torch.cuda.synchronize()
        self.pre, self.z, self.y_hat = to_np(step.pre), to_np(step.z), to_np(step.y_hat)
        cls = step.act_class.cpu().numpy()
        self.active, self.window = (cls & 1).astype(bool), (cls & 2).astype(bool)
        self.below = (cls & 4).astype(bool)
        self.l0 = step.l0.cpu().numpy()
        self.decode_switch = K.clt_workspace_view(step.H, "decode_switch").cpu().numpy()
        self.grads = {k: to_np(g) for k, g in step.grads.items()}
        if not fused:
            step.adam_step(t, w.lr, gp, gm, gv, master)
        torch.cuda.synchronize()
        self.new_params = {k: to_np(p) for k, p in gp.items()}
        self.new_m = {k: to_np(a) for k, a in gm.items()}
        self.new_v = {k: to_np(a) for k, a in gv.items()}
        self.new_master = {k: to_np(a) for k, a in master.items()} if master else None
        self.step = step


class OracleRun:
    """The same step through oracle/clt_oracle.py.  If the GPU took the other valid
    decision for pre-activations inside MASK_BAND of a boundary, the oracle is
    asked to continue from that decision (it verifies the band itself)."""

    def __init__(self, w, params, x, y, t=1, m=None, v=None, gpu_active=None, gpu_window=None, theta=None,
                 x_np=None, y_np=None, gpu_below=None):
        npar = {k: to_np(p) for k, p in params.items()}
        if theta is not None:
            npar["theta"] = to_np(theta)
        xn = to_np(x) if x_np is None else x_np
        yn = to_np(y) if y_np is None else y_np
        self.x_np, self.y_np = xn, yn
        self.theta = O.threshold_value(npar["theta"], w.log_threshold)
        self.fwd = O.forward(xn, npar["W_enc"], npar["b_enc"], self.theta, npar["W_dec"], npar["b_dec"],
                             tie_break=gpu_active, band=MASK_BAND, topk=w.topk or None)
        self.n = O.decoder_norms(npar["W_dec"], w.L)
        tot, rec, sp = O.loss_terms(self.fwd["y_hat"], yn, self.fwd["z"], self.n, w.lambda0, w.C)
        dead = O.dead_feature_term(self.fwd["pre"], self.theta, self.n, w.lambda1)
        self.loss = (tot + dead, rec, sp, dead)
        self.bwd = O.backward(xn, yn, self.theta, npar["W_dec"], self.fwd, w.lambda0, w.C, w.ste_eps,
                              window_tie_break=None if w.topk else gpu_window, band=MASK_BAND, lambda1=w.lambda1,
                              log_threshold=w.log_threshold, below_tie_break=None if w.topk else gpu_below,
                              topk=bool(w.topk))
        zeros = {k: np.zeros_like(a) for k, a in npar.items()}
        m = zeros if m is None else {k: to_np(a) for k, a in m.items()}
        v = zeros if v is None else {k: to_np(a) for k, a in v.items()}
        self.new_params, self.new_m, self.new_v = {}, {}, {}
        for k in O.PARAM_NAMES:
            self.new_params[k], self.new_m[k], self.new_v[k] = O.adam_update(
                npar[k], self.bwd["d" + k], m[k], v[k], t, w.lr)
        self.params = npar


def compare_step(w, g: GpuRun, o: OracleRun, tol, check_adam=True):
    """Element-wise parity of every output of the step.  Returns the error table."""
    L = w.L
    theta = o.theta
    pre_o = o.fwd["pre"]
    errs = {}
    if w.topk:
        # the oracle has verified the selection against its own ranking outside the band around each row's
        # k-th value and that every row holds exactly k entries; there is no threshold, window or gradient of it
        assert (g.active == o.fwd["active"]).all() and (g.active.sum(axis=2) == w.topk).all()
        assert not g.window.any() and not g.below.any() and not g.grads["theta"].any()
        theta = np.full(theta.shape, np.inf)             # keeps the threshold-based checks below trivially true
        assert not o.bwd["window"].any()
    # masks: identical except inside the band around the boundary
    band = np.abs(pre_o - theta[:, None, :]) < MASK_BAND
    assert ((g.active == o.fwd["active"]) | band | bool(w.topk)).all(), "active mask differs outside the band"
    wband = np.abs(np.abs(pre_o - theta[:, None, :]) - 0.5 * w.ste_eps) < MASK_BAND
    assert ((g.window == o.bwd["window"]) | wband).all(), "window mask differs outside the band"
    assert ((g.below == (pre_o < theta[:, None, :])) | band | bool(w.topk)).all(), "below-threshold mask differs outside the band"
    assert not (g.below & g.active).any()
    assert (g.l0 == g.active.sum(axis=(1, 2))).all(), "l0_per_layer does not count the active mask"
    errs["pre"] = rel_l2(g.pre, pre_o)
    errs["z"] = rel_l2(g.z, o.fwd["z"])
    errs["norms"] = rel_l2(g.norms, o.n)
    for lp in range(L):
        errs[f"y_hat[{lp}]"] = rel_l2(g.y_hat[lp], o.fwd["y_hat"][lp])
    for i, name in enumerate(("loss", "L_rec", "L_sp", "L_dead")):
        errs[name] = abs(g.loss[i] - o.loss[i]) / max(abs(o.loss[i]), 1e-30)
    errs["d_yhat"] = rel_l2(g.d_yhat, o.bwd["d_yhat"])
    # Column sums of the objective's decoder-norm derivative.  z sech^2(C z n) amplifies a relative
    # error of z by about 2 C z n, so with bf16 storage the reference is the oracle's sum over the
    # oracle's z rounded the way it is stored (the dead-feature part is linear and needs no such care).
    G_ref = o.bwd["G"]
    if w.dtype == "bf16":
        z_r = torch.from_numpy(o.fwd["z"]).to(torch.bfloat16).double().numpy()
        G_ref = G_ref - O.sparsity_norm_sums(o.fwd["z"], o.n, w.lambda0, w.C) \
            + O.sparsity_norm_sums(z_r, o.n, w.lambda0, w.C)
    errs["G"] = rel_l2(g.G, G_ref)
    if not w.int8_inputs:      # with int8 inputs the buffer holds dpre times the row scale of x
        errs["dpre"] = rel_l2(g.dpre, o.bwd["dpre"])
    for k in ("W_enc", "b_enc", "theta", "b_dec"):
        if k == "theta" and w.topk:
            continue                                     # exactly zero on both sides (asserted above)
        errs["d" + k] = rel_l2(g.grads[k], o.bwd["d" + k])
    for p in range(O.num_blocks(L)):
        errs[f"dW_dec[{p}]"] = rel_l2(g.grads["W_dec"][p], o.bwd["dW_dec"][p])
    bad = {k: e for k, e in errs.items() if not e <= tol}
    assert not bad, f"parity failures (tol {tol}): {bad}"
    if check_adam:
        check_adam_outputs(w, g, o, tol)
    return errs


def bf16_ulp(a):
    a = np.abs(np.asarray(a, np.float64))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -126)))
    return 2.0 ** (e - 7)


def check_adam_outputs(w, g: GpuRun, o: OracleRun, tol):
    """Moments within tol (they are linear / quadratic in the gradient).  The first
    update is -lr * g / (|g| + eps): it is compared where it is well conditioned
    (|g| >> eps and both gradients agree in sign and scale), up to the rounding of
    the stored parameter; everywhere it must stay within one learning rate."""
    for k in O.PARAM_NAMES:
        assert rel_l2(g.new_m[k], o.new_m[k]) <= tol, f"Adam m[{k}]"
        assert rel_l2(g.new_v[k], o.new_v[k]) <= 2 * tol, f"Adam v[{k}]"
        master = w.master_weights and k in MATS
        got = g.new_master[k] if master else g.new_params[k]
        want, old = o.new_params[k], o.params[k]
        g_o, g_g = o.bwd["d" + k], g.grads[k]
        cond = (np.abs(g_o) > 1e-5) & (np.abs(g_g - g_o) <= 0.5 * np.abs(g_o))
        if w.dtype == "bf16" and k in MATS and not master:
            quant = 0.51 * bf16_ulp(np.maximum(np.abs(got), np.abs(want)))
        else:
            quant = 2e-7 * np.abs(want) + 1e-12
        err = np.abs(got - want)
        assert (err[cond] <= quant[cond] + 2e-3 * w.lr).all(), f"Adam update {k}"
        assert (np.abs(got - old) <= 1.001 * w.lr + quant).all(), f"Adam step bound {k}"
        if master:
            rounded = g.new_params[k]
            assert (np.abs(rounded - got) <= 0.51 * bf16_ulp(got)).all(), f"bf16 copy of master {k}"


def run_both(w, theta=None, t=1, m=None, v=None, **gpu_kw):
    params = S.make_params(w)
    x, y = S.make_inputs(w)
    xs = ys = None
    xo = yo = None
    xin, yin = x, y
    if w.int8_inputs:
        xin, xs = S.quantize_rows_int8(x)
        yin, ys = S.quantize_rows_int8(y)
        xo = O.dequantize_rows(xin.numpy(), xs.numpy())
        yo = O.dequantize_rows(yin.numpy(), ys.numpy())
    g = GpuRun(w, params, xin, yin, t=t, m=m, v=v, x_scale=xs, y_scale=ys, theta=theta, **gpu_kw)
    o = OracleRun(w, params, x, y, t=t, m=m, v=v, gpu_active=g.active, gpu_window=g.window, theta=theta,
                  x_np=xo, y_np=yo, gpu_below=g.below)
    return g, o
