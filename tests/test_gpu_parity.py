"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.  Tolerances: 1e-4 relative (per tensor, per decoder
block) for the fp32 path, 2e-2 for the bf16 MFMA path; masks bit-exact except
for pre-activations within 1e-3 of a decision boundary."""
import numpy as np
import pytest
import torch

from oracle import clt_oracle as O
from workloads import clt_synth as S

from clt_testlib import GpuRun, OracleRun, compare_step, rel_l2, run_both, theta_for_density, to_np

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
DENSE, GATHER, AUTO = 1, 2, 0


def show(name, errs):
    worst = sorted(errs.items(), key=lambda kv: -kv[1])[:4]
    print(f"[{name}] worst: " + ", ".join(f"{k}={e:.2e}" for k, e in worst), flush=True)


def test_tiny_config_fp32_full_step():
    """The smallest configuration: L=4, d=64, F=256, B=128, fp32 storage, one forward + backward + Adam step."""
    w = S.WORKLOADS["tiny"]
    g, o = run_both(w)
    assert 0.2 < g.active.mean() < 0.8
    assert g.window.sum() > 100
    show("tiny f32", compare_step(w, g, o, TOL["f32"]))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L,d,F,B", [
    (3, 40, 72, 77),        # nothing is a multiple of any tile size
    (2, 264, 520, 300),     # 256-tiles plus ragged tails in every dimension
    (1, 64, 128, 1),        # single layer, single token
    (5, 128, 256, 130),
])
def test_ragged_shapes_full_step(dtype, L, d, F, B):
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=L, d=d, F=F, B=B, seed=7 + L + d)
    g, o = run_both(w)
    show(f"{dtype} L{L} d{d} F{F} B{B}", compare_step(w, g, o, TOL[dtype]))


def test_bf16_several_tiles_and_segments():
    """Spans 2x3 output tiles of 256x256 per group and up to 4 K segments."""
    w = S.scaled(S.WORKLOADS["gpt2"], L=4, d=512, F=768, B=512, k_active=16)
    g, o = run_both(w)
    show("bf16 multi-tile", compare_step(w, g, o, TOL["bf16"]))


@pytest.mark.parametrize("fused", [False, True])
def test_bf16_more_interior_tiles_than_cus(fused):
    """Every matrix extent is a multiple of the 256-tile and the launches hold more workgroup slots than the GPU has
    CUs, empty slots included (encoder 5 groups x 72 tiles in 432 slots, decode 5 x 8, dW_dec up to 5 blocks x 36
    tiles in 288 slots): the kernels without edge code walk their tiles in a loop, one workgroup per CU."""
    w = S.scaled(S.WORKLOADS["gpt2"], L=5, d=512, F=4608, B=1024, k_active=32, seed=77)
    g, o = run_both(w, fused=fused)
    show(f"bf16 tile loop fused={fused}", compare_step(w, g, o, TOL["bf16"]))


def test_bf16_outlier_inputs_llama_shaped_slice():
    """Config 3's input recipe (log-normal norms, outlier dims) at a slice of its shape."""
    w = S.scaled(S.WORKLOADS["llama1b"], L=3, d=2048, F=512, B=256)
    g, o = run_both(w)
    show("bf16 llama slice", compare_step(w, g, o, TOL["bf16"]))


@pytest.mark.parametrize("name,F,B", [("gpt2", 512, 256), ("gemma2b", 256, 128)])
def test_config_shaped_slices_full_depth(name, F, B):
    """The GPT-2 and Gemma-2 configs at their full depth and model width (L = 12 / 26 layers, d = 768 / 2304: all
    decoder blocks, up to 26 K segments per tile, 3 / 9 column tiles), on a slice of features and tokens the
    oracle can do in seconds; the call the benchmark times (Adam fused, fp32 master weights for Gemma)."""
    w = S.scaled(S.WORKLOADS[name], F=F, B=B, k_active=8)
    g, o = run_both(w, fused=True)
    show(f"{name} slice L{w.L} d{w.d}", compare_step(w, g, o, TOL["bf16"]))


def test_master_weights_bf16():
    w = S.scaled(S.WORKLOADS["gemma2b"], L=2, d=64, F=256, B=96)
    g, o = run_both(w)
    show("bf16 master", compare_step(w, g, o, TOL["bf16"]))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_infinite_threshold_gives_bias_only(dtype):
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype)
    theta = torch.full((w.L, w.F), float("inf"))
    params = S.make_params(w)
    params["b_dec"] = torch.randn((w.L, w.d), generator=torch.Generator().manual_seed(3))
    x, y = S.make_inputs(w)
    g = GpuRun(w, params, x, y, theta=theta)
    assert not g.active.any() and not g.z.any() and g.l0.sum() == 0
    for lp in range(w.L):
        assert (g.y_hat[lp] == params["b_dec"][lp].numpy()[None, :]).all()
    want = np.sum((params["b_dec"].numpy()[:, None, :].astype(np.float64) - to_np(y)) ** 2) / w.B
    assert abs(g.loss[1] - want) / want < 1e-5 and g.loss[2] == 0.0
    assert not g.grads["W_enc"].any() and not g.grads["theta"].any()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_zero_decoder_rows_do_not_produce_nan(dtype):
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=2, B=64)
    params = S.make_params(w)
    params["W_dec"][:, 5, :] = 0.0
    x, y = S.make_inputs(w)
    g = GpuRun(w, params, x, y)
    o = OracleRun(w, params, x, y, gpu_active=g.active, gpu_window=g.window)
    assert np.isfinite(g.grads["W_dec"]).all()
    show(f"zero rows {dtype}", compare_step(w, g, o, TOL[dtype]))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_adam_later_step_with_given_moments(dtype):
    """Adam at t = 7 from non-zero moments: m, v and the update against the oracle."""
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=2, B=64, master_weights=(dtype == "bf16"))
    params = S.make_params(w)
    gen = torch.Generator().manual_seed(11)
    m = {k: 1e-3 * torch.randn(p.shape, generator=gen) for k, p in params.items()}
    v = {k: 1e-6 * torch.rand(p.shape, generator=gen) for k, p in params.items()}
    x, y = S.make_inputs(w)
    g = GpuRun(w, params, x, y, t=7, m=m, v=v)
    o = OracleRun(w, params, x, y, t=7, m=m, v=v, gpu_active=g.active, gpu_window=g.window)
    tol = TOL[dtype]
    for k in O.PARAM_NAMES:
        assert rel_l2(g.new_m[k], o.new_m[k]) <= tol, k
        assert rel_l2(g.new_v[k], o.new_v[k]) <= tol, k
        got = g.new_master[k] if (w.master_weights and k in ("W_enc", "W_dec")) else g.new_params[k]
        assert rel_l2(got - o.params[k], o.new_params[k] - o.params[k]) <= tol, k


def test_five_training_steps_follow_the_oracle_trajectory():
    """Five consecutive fused steps on the fp32 config, parameters and moments carried on the device, against
    five oracle steps: the loss falls and follows the oracle's, the parameters stay within a fraction of the
    distance they travelled (Adam's early steps move every weight by about lr whatever the gradient's size, so a
    gradient near zero may take the other sign; that bounds the per-entry difference by 2 lr per step)."""
    from paper_2603_21014_amd import binding as K
    w = S.scaled(S.WORKLOADS["tiny"], L=3, d=64, F=128, B=96, seed=61)
    params = S.make_params(w)
    x, y = S.make_inputs(w)
    dev = "cuda:0"
    gp = {k: p.to(dev).contiguous() for k, p in params.items()}
    gm = {k: torch.zeros_like(p) for k, p in gp.items()}
    gv = {k: torch.zeros_like(p) for k, p in gp.items()}
    step = K.CLTStep(w.L, w.d, w.F, w.B, dtype="f32", C_=w.C, ste_bandwidth=w.ste_eps, matrix_grads=False)
    op = {k: to_np(p) for k, p in params.items()}
    om = {k: np.zeros_like(v) for k, v in op.items()}
    ov = {k: np.zeros_like(v) for k, v in op.items()}
    xg, yg = x.to(dev), y.to(dev)
    xn, yn = to_np(x), to_np(y)
    g_losses, o_losses = [], []
    for t in range(1, 6):
        step.train_step(xg, yg, gp, gm, gv, t, w.lr, w.lambda0)
        g_losses.append(step.loss_dev.cpu().numpy()[0])
        op, om, ov, info = O.train_step(xn, yn, op, om, ov, t, w.lr, w.lambda0, w.C, w.ste_eps)
        o_losses.append(info["loss"][0])
    print("losses gpu", g_losses, "oracle", o_losses, flush=True)
    assert all(b < a for a, b in zip(g_losses, g_losses[1:])), "the loss must fall on this problem"
    for a, b in zip(g_losses, o_losses):
        assert abs(a - b) <= 1e-3 * abs(b)
    for k in O.PARAM_NAMES:
        travelled = np.abs(op[k] - to_np(params[k]))
        diff = np.abs(to_np(gp[k]) - op[k])
        assert diff.max() <= 2 * 5 * w.lr * 1.001, k
        assert np.linalg.norm(diff) <= 0.05 * np.linalg.norm(travelled), k


# ---------------------------------------------------------------- backward + Adam in one call
@pytest.mark.parametrize("dtype,master", [("f32", False), ("bf16", False), ("bf16", True)])
@pytest.mark.parametrize("L,d,F,B", [(3, 40, 72, 77), (2, 264, 520, 300)])
def test_fused_backward_adam_step(dtype, master, L, d, F, B):
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=L, d=d, F=F, B=B, seed=31 + d, master_weights=master)
    g, o = run_both(w, fused=True)
    show(f"fused {dtype} master={master} L{L} d{d}", compare_step(w, g, o, TOL[dtype]))


@pytest.mark.parametrize("B,master", [(2048, False), (4096, True)])
def test_bf16_fused_update_many_tiles_per_cu(B, master):
    """The fused update at a size where every CU sees several tiles of both weight-gradient launches (dW_dec 21
    blocks x 88 tiles, dW_enc 6 x 88, no edge tiles, 32 / 64 K steps per tile), with and without master weights."""
    w = S.scaled(S.WORKLOADS["gpt2"], L=6, d=1024, F=5632, B=B, k_active=32, seed=78, master_weights=master)
    g, o = run_both(w, fused=True)
    show(f"bf16 fused update, many tiles, B={B} master={master}", compare_step(w, g, o, TOL["bf16"]))


def test_decoder_norms_reused_from_the_fused_update():
    """reuse_decoder_norms: the fused update of step t leaves the row sums of squares of the new decoder weights
    and the forward pass of step t + 1 forms the norms from them instead of reading W_dec.  The third step of a
    run is compared with the oracle started from the device's state after two steps; without the option the same
    step reads W_dec and must agree up to the summation order."""
    w = S.scaled(S.WORKLOADS["gpt2"], L=3, d=512, F=768, B=300, k_active=16, seed=88)
    params = S.make_params(w)
    x, y = S.make_inputs(w)
    g = GpuRun(w, params, x, y, fused=True, pre_steps=2, reuse_decoder_norms=True)
    assert g.kernel_launches.get("decoder_norms_from_update") == 1 and "decoder_norms" not in g.kernel_launches
    o = OracleRun(w, g.start_params, x, y, t=3, m=g.start_m, v=g.start_v, gpu_active=g.active, gpu_window=g.window)
    show("norms from the update, step 3", compare_step(w, g, o, TOL["bf16"], check_adam=False))
    for k in O.PARAM_NAMES:      # Adam from two steps of history: moments and the distance moved
        assert rel_l2(g.new_m[k], o.new_m[k]) <= TOL["bf16"] and rel_l2(g.new_v[k], o.new_v[k]) <= 2 * TOL["bf16"], k
    plain = GpuRun(w, params, x, y, fused=True, pre_steps=2)
    assert plain.kernel_launches.get("decoder_norms") == 1 and "decoder_norms_from_update" not in plain.kernel_launches
    assert rel_l2(g.norms, plain.norms) < 1e-6 and (g.active == plain.active).all()
    # the two runs differ by the summation order of the norms (1e-7 relative); after three steps that flips the bf16
    # rounding of a few updated weights (one flip in a thousand weights is a relative L2 distance of 1.2e-4)
    for k in O.PARAM_NAMES:
        assert rel_l2(g.new_params[k], plain.new_params[k]) < 1e-4, k
    # the list-driven row kernel of dW_dec leaves the same row sums (forced gather mode, same workload)
    gg = GpuRun(w, params, x, y, fused=True, pre_steps=2, reuse_decoder_norms=True, decode_mode=GATHER)
    assert gg.kernel_launches.get("decoder_norms_from_update") == 1 and "decoder_norms" not in gg.kernel_launches
    assert gg.kernel_launches.get("sparse_dW_dec") == 1
    og = OracleRun(w, gg.start_params, x, y, t=3, m=gg.start_m, v=gg.start_v, gpu_active=gg.active, gpu_window=gg.window)
    show("norms from the list-driven update, step 3", compare_step(w, gg, og, TOL["bf16"], check_adam=False))
    pg = GpuRun(w, params, x, y, fused=True, pre_steps=2, decode_mode=GATHER)
    assert pg.kernel_launches.get("decoder_norms") == 1
    assert rel_l2(gg.norms, pg.norms) < 1e-6
    # automatic mode: whichever of the two kernels the device-side switch picked leaves the sums, and the norms
    # kernel reads the same switch to know their layout
    # (sparse thresholds, so that the lists fit the room the automatic mode gives them; third case: dense decode,
    #  list-driven backward -- the row kernel's layout although the forward was dense)
    th = sparse_theta(w, 0.02)
    for thr, thr_bwd, switch in ((0.1, 0.0, 3), (0.001, 0.0, 0), (0.001, 0.1, 2)):
        ga = GpuRun(w, params, x, y, theta=th, fused=True, pre_steps=2, reuse_decoder_norms=True, decode_mode=AUTO,
                    gather_density_threshold=thr, list_backward_density_threshold=thr_bwd)
        assert ga.kernel_launches.get("decoder_norms_from_update") == 1 and "decoder_norms" not in ga.kernel_launches
        assert (ga.decode_switch[0] & 3) == switch and (ga.decode_switch[3] > 0) == (switch >= 2)
        pa = GpuRun(w, params, x, y, theta=th, fused=True, pre_steps=2, decode_mode=AUTO, gather_density_threshold=thr,
                    list_backward_density_threshold=thr_bwd)
        assert rel_l2(ga.norms, pa.norms) < 1e-6, (thr, thr_bwd, rel_l2(ga.norms, pa.norms))
        oa = OracleRun(w, ga.start_params, x, y, t=3, m=ga.start_m, v=ga.start_v, gpu_active=ga.active, gpu_window=ga.window)
        show(f"norms from the update, automatic mode, thresholds {thr} / {thr_bwd}",
             compare_step(w, ga, oa, TOL["bf16"], check_adam=False))
    # an unfused update in between changes W_dec without new row sums: the next forward must read W_dec again
    from paper_2603_21014_amd import binding as K
    step, (gp, gm, gv, _) = g.step, g.device_state
    xg, yg = x.to("cuda:0", torch.bfloat16), y.to("cuda:0", torch.bfloat16)
    step.train_step(xg, yg, gp, gm, gv, 4, w.lr, w.lambda0, fused=False)
    K.clt_profile_enable(step.H, True)
    step.forward(xg, gp)
    launches = {k: n for k, (_, n) in K.clt_profile_query(step.H).items() if n}
    assert launches.get("decoder_norms") == 1 and "decoder_norms_from_update" not in launches
    want = O.decoder_norms(to_np(gp["W_dec"]), w.L)
    assert rel_l2(to_np(K.clt_workspace_view(step.H, "norms")), want) < 1e-5


def test_fused_equals_unfused_with_fp32_storage():
    """With fp32 storage the gradient enters Adam unrounded on both paths: same gradients
    bit for bit, same update up to the contraction order of the two compiled epilogues."""
    w = S.scaled(S.WORKLOADS["tiny"], L=3, d=72, F=136, B=90, seed=33)
    params = S.make_params(w)
    x, y = S.make_inputs(w)
    gen = torch.Generator().manual_seed(12)
    m = {k: 1e-3 * torch.randn(p.shape, generator=gen) for k, p in params.items()}
    v = {k: 1e-6 * torch.rand(p.shape, generator=gen) for k, p in params.items()}
    a = GpuRun(w, params, x, y, t=5, m=m, v=v, fused=False)
    b = GpuRun(w, params, x, y, t=5, m=m, v=v, fused=True)
    old = {k: to_np(p) for k, p in params.items()}
    for k in O.PARAM_NAMES:
        assert (a.grads[k] == b.grads[k]).all(), k
        assert rel_l2(b.new_m[k], a.new_m[k]) < 1e-6 and rel_l2(b.new_v[k], a.new_v[k]) < 1e-6, k
        assert rel_l2(b.new_params[k] - old[k], a.new_params[k] - old[k]) < 1e-4, k


# ---------------------------------------------------------------- int8 activation cache
@pytest.mark.parametrize("L,d,F,B", [(2, 64, 256, 96), (3, 264, 520, 300)])
def test_int8_row_scaled_inputs(L, d, F, B):
    """x and y as int8 codes with per-(layer, token) scales, dequantised inside the
    kernels; the oracle consumes the dequantised values."""
    w = S.scaled(S.WORKLOADS["llama1b_int8"], L=L, d=d, F=F, B=B, k_active=8)
    g, o = run_both(w)
    show(f"int8 L{L} d{d} F{F} B{B}", compare_step(w, g, o, TOL["bf16"]))


# ---------------------------------------------------------------- dead-feature penalty, log threshold
def dead_term_matters(w, o, tol):
    """The oracle with the term switched off differs from the oracle with it by far more than
    the parity tolerance, in every output the term reaches: parity then proves it was computed."""
    off = OracleRun(S.scaled(w, lambda1=0.0), {k: torch.tensor(v) for k, v in o.params.items()},
                    None, None, gpu_active=o.fwd["active"], gpu_window=o.bwd["window"], x_np=o.x_np, y_np=o.y_np)
    for k in ("dW_enc", "db_enc", "dtheta", "G", "dpre"):      # G is the term's way into dW_dec
        assert rel_l2(off.bwd[k], o.bwd[k]) > 10 * tol, k
    assert o.loss[3] > 10 * tol * o.loss[0]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("log_threshold", [False, True])
@pytest.mark.parametrize("fused", [False, True])
def test_dead_feature_term_full_step(dtype, log_threshold, fused):
    """App. B third term, with the threshold stored directly or as its logarithm."""
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=3, d=72, F=136, B=90, seed=41, lambda1=5.0,
                 log_threshold=log_threshold)
    g, o = run_both(w, fused=fused)
    assert 0.2 < g.below.mean() < 0.8
    dead_term_matters(w, o, TOL[dtype])
    show(f"dead {dtype} log={log_threshold} fused={fused}", compare_step(w, g, o, TOL[dtype]))


def test_dead_feature_term_bf16_several_tiles():
    w = S.scaled(S.WORKLOADS["llama1b_dead"], L=3, d=512, F=768, B=300, k_active=16, lambda1=5.0)
    g, o = run_both(w, fused=True)
    dead_term_matters(w, o, TOL["bf16"])
    show("dead bf16 multi-tile", compare_step(w, g, o, TOL["bf16"]))


def test_dead_feature_term_int8_inputs():
    """The row scale of the int8 codes also multiplies the dead-feature part of d pre on its
    way into the encoder-weight gradient."""
    w = S.scaled(S.WORKLOADS["llama1b_int8"], L=2, d=264, F=520, B=300, k_active=8, lambda1=5.0, log_threshold=True)
    g, o = run_both(w)
    dead_term_matters(w, o, TOL["bf16"])
    show("dead int8", compare_step(w, g, o, TOL["bf16"]))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_log_threshold_without_dead_term(dtype):
    """Pure reparameterisation: same forward as theta = exp(tau), threshold gradient times theta."""
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=2, d=64, F=256, B=128, seed=43, log_threshold=True)
    g, o = run_both(w)
    assert g.window.sum() > 100 and np.abs(o.bwd["dtheta"]).max() > 0
    show(f"log-threshold {dtype}", compare_step(w, g, o, TOL[dtype]))


def test_dead_term_needs_pre_and_theta():
    from paper_2603_21014_amd import binding as K
    w = S.scaled(S.WORKLOADS["tiny"], L=2, d=64, F=128, B=32)
    step = K.CLTStep(w.L, w.d, w.F, w.B, dtype="f32", keep_pre=False)
    params = {k: p.cuda() for k, p in S.make_params(w).items()}
    x, y = (t.cuda() for t in S.make_inputs(w))
    step.forward(x, params)
    with pytest.raises(ValueError):
        step.loss(y, 1.0, lambda1=0.5, params=params)          # no pre buffer was kept
    with pytest.raises(K.CLTError) as e:                       # the ABI itself refuses the NULL pointer
        K._check(K._lib.clt_loss(step.H.h, None, y.data_ptr(), None, step.y_hat.data_ptr(), step.z.data_ptr(),
                                 None, None, 1.0, 0.5, step.loss_dev.data_ptr(), None), step.H.h)
    assert e.value.code == -1
    with pytest.raises(K.CLTError):
        step.loss(y, 1.0, lambda1=-1.0, params=params)
    torch.cuda.synchronize()


# ---------------------------------------------------------------- TopK activation
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L,d,F,B,k", [(3, 40, 72, 77, 5), (2, 264, 520, 300, 33), (2, 64, 1032, 40, 1)])
def test_topk_activation_full_step(dtype, L, d, F, B, k):
    """TopK instead of JumpReLU: exactly k features per token and layer, selected on the fp32 pre-activation."""
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=L, d=d, F=F, B=B, seed=91 + F, topk=k)
    for fused in (False, True):
        g, o = run_both(w, fused=fused)
        assert (g.l0 == k * B).all()
        show(f"topk {dtype} F{F} k{k} fused={fused}", compare_step(w, g, o, TOL[dtype]))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("F,k", [(2056, 61), (4096, 1), (8192, 61), (8192, 64), (8192, 8192), (8200, 67), (16384, 1),
                                 (16384, 61), (16384, 64), (16384, 16384)])
def test_topk_wide_rows(dtype, F, k):
    """Rows wider than 2048 features: 2048 < F <= 8192 keeps the row in registers (eight float4 per lane, with
    padding lanes when F is not a multiple of 1024), F > 8192 re-reads the row in every radix pass.  Two token rows
    are built to tie at the k-th value across more than one 256-lane round of the selection: an all-zero input row
    (every pre-activation equals the bias, the first k features win) and, in layer 1, encoder columns that repeat
    with a period of 1024 features (each value occurs F/1024 or more times, once per round; the copies are the same
    sum of the same products in the same order, so they tie exactly, and with k not a multiple of the repeat count
    the k-th value's copies are selected only in part)."""
    L, d, B = 2, 64, 40
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=L, d=d, F=F, B=B, seed=95 + F, topk=k, k_active=8)
    params = S.make_params(w)
    period = 1024
    params["W_enc"][1] = params["W_enc"][1][:, :period].repeat(1, (F + period - 1) // period)[:, :F]
    x, y = S.make_inputs(w)
    x[:, 3, :] = 0.0
    g = GpuRun(w, params, x, y, fused=True)
    assert (g.l0 == k * B).all() and (g.active.sum(axis=2) == k).all()
    assert g.active[:, 3, :k].all() and not g.active[:, 3, k:].any()
    o = OracleRun(w, params, x, y, gpu_active=g.active)
    # among exact copies the lower feature index wins: a copy is selected only if the copy one period below it is
    partial = False
    for lo in range(period, F, period):
        n = min(period, F - lo)
        upper, lower = g.active[1][:, lo:lo + n], g.active[1][:, lo - period:lo - period + n]
        assert not (upper & ~lower).any(), "tie order among equal values"
        partial |= bool((lower & ~upper).any())
    assert partial or k == F or k % (F // period) == 0, "no row had a tie group cut by the k-th value"
    show(f"topk wide {dtype} F{F} k{k}", compare_step(w, g, o, TOL[dtype]))


def test_topk_limits_and_ties():
    """k = 0 (nothing), k = F (everything, the linear model) and a zero input row, whose pre-activations are all
    equal to the bias: the first k features by index are selected."""
    w = S.scaled(S.WORKLOADS["tiny"], L=2, d=64, F=128, B=32, topk=7)
    params = S.make_params(w)
    x, y = S.make_inputs(w)
    x[:, 3, :] = 0.0
    g = GpuRun(w, params, x, y)
    o = OracleRun(w, params, x, y, gpu_active=g.active)
    assert (g.active[:, 3, :7]).all() and not g.active[:, 3, 7:].any()
    show("topk tie row", compare_step(w, g, o, TOL["f32"]))
    for k, frac in ((0, 0.0), (w.F, 1.0)):
        wk = S.scaled(w, topk=k)
        if k == 0:       # topk = 0 means JumpReLU to the workload helper: drive the library directly
            from paper_2603_21014_amd import binding as K
            step = K.CLTStep(w.L, w.d, w.F, w.B, dtype="f32", topk=0)
            gp = {kk: p.cuda() for kk, p in params.items()}
            step.forward(x.cuda(), gp)
            torch.cuda.synchronize()
            assert not step.z.any() and not step.act_class.any() and not step.l0.any()
            assert (step.y_hat.cpu() == params["b_dec"][:, None, :]).all()
        else:
            g = GpuRun(wk, params, x, y)
            assert g.active.all() and rel_l2(g.z, g.pre) == 0.0
            o = OracleRun(wk, params, x, y, gpu_active=g.active)
            show("topk k=F", compare_step(wk, g, o, TOL["f32"]))


def test_topk_with_gather_decode_and_sparse_backward():
    w = S.scaled(S.WORKLOADS["tiny"], dtype="bf16", L=3, d=128, F=512, B=130, seed=93, topk=12)
    g, o = run_both(w, decode_mode=2, fused=True)
    assert g.decode_switch[2] == 2
    show("topk + gather", compare_step(w, g, o, TOL["bf16"]))


def test_topk_refuses_dead_feature_term():
    from paper_2603_21014_amd import binding as K
    w = S.scaled(S.WORKLOADS["tiny"], L=2, d=64, F=128, B=32)
    step = K.CLTStep(w.L, w.d, w.F, w.B, dtype="f32", topk=4)
    params = {k: p.cuda() for k, p in S.make_params(w).items()}
    x, y = (t.cuda() for t in S.make_inputs(w))
    step.forward(x, params)
    with pytest.raises(K.CLTError) as e:
        step.loss(y, 1.0, lambda1=0.5, params=params)
    assert e.value.code == -1
    with pytest.raises(K.CLTError):
        K.clt_workspace_bytes(K.make_config(2, 64, 128, 32, topk=129))
    torch.cuda.synchronize()


# ---------------------------------------------------------------- seeded sweep over shapes and modes
def _sweep_cases():
    rng = np.random.default_rng(2024)
    cases = []
    for i in range(16):
        L = int(rng.integers(1, 6))
        d = 8 * int(rng.integers(1, 70))          # 8 .. 552: below, at and above one 256-wide tile
        F = 8 * int(rng.integers(1, 80))
        B = int(rng.integers(1, 330))
        cases.append((i, L, d, F, B))
    return cases


@pytest.mark.parametrize("i,L,d,F,B", _sweep_cases())
def test_seeded_shape_and_mode_sweep(i, L, d, F, B):
    """Random shapes (every dimension ragged against every tile size) crossed with the options: storage type,
    fused update, master weights, int8 inputs, dead-feature term / log threshold, TopK, list-driven kernels."""
    rng = np.random.default_rng(100 + i)
    dtype = "bf16" if rng.random() < 0.6 else "f32"
    int8 = dtype == "bf16" and rng.random() < 0.3
    topk = int(rng.integers(1, F + 1)) if rng.random() < 0.25 else 0
    dead = (not topk) and rng.random() < 0.4
    base = S.WORKLOADS["llama1b_int8"] if int8 else S.WORKLOADS["tiny"]
    w = S.scaled(base, dtype=dtype, L=L, d=d, F=F, B=B, seed=500 + i, k_active=max(1, F // 16),
                 master_weights=dtype == "bf16" and rng.random() < 0.4, topk=topk,
                 lambda1=2.0 if dead else 0.0, log_threshold=dead and rng.random() < 0.5)
    mode = [DENSE, GATHER, AUTO][int(rng.integers(0, 3))]
    fused = bool(rng.random() < 0.5)
    theta = None
    if mode != DENSE and not topk and rng.random() < 0.7:        # a sparse regime for the list-driven kernels
        theta = sparse_theta(w, 0.05)
        if w.log_threshold:
            theta = torch.log(theta.clamp_min(1e-3))
    g, o = run_both(w, theta=theta, decode_mode=mode, fused=fused, gather_density_threshold=0.1)
    show(f"sweep {i}: L{L} d{d} F{F} B{B} {dtype} int8={int8} topk={topk} dead={dead} log={w.log_threshold} "
         f"master={w.master_weights} mode={mode} fused={fused} path={g.decode_switch[2]}",
         compare_step(w, g, o, TOL[dtype]))


# ---------------------------------------------------------------- gather decode and the switch


def sparse_theta(w, rho):
    params = S.make_params(w)
    x, _ = S.make_inputs(w)
    return theta_for_density(x, params["W_enc"], params["b_enc"], rho)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rho", [0.02, 0.3])
def test_gather_decode_full_step_against_oracle(dtype, rho):
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=3, d=264, F=520, B=100, seed=77)
    theta = sparse_theta(w, rho)
    g, o = run_both(w, theta=theta, decode_mode=GATHER)
    assert g.decode_switch[2] == 2, "the gather path did not run"
    assert abs(g.active.mean() - rho) < 0.3 * rho
    show(f"gather {dtype} rho={rho}", compare_step(w, g, o, TOL[dtype]))


def test_gather_wide_model_dim_and_empty_rows():
    """d > 2048 takes two column passes; an infinite threshold leaves every list empty."""
    w = S.scaled(S.WORKLOADS["gpt2"], L=2, d=2304, F=256, B=40, seed=78)
    theta = sparse_theta(w, 0.05)
    g, o = run_both(w, theta=theta, decode_mode=GATHER)
    assert g.decode_switch[2] == 2
    show("gather d=2304", compare_step(w, g, o, TOL["bf16"]))
    params = S.make_params(w)
    params["b_dec"] = torch.randn((w.L, w.d), generator=torch.Generator().manual_seed(3))
    x, y = S.make_inputs(w)
    g = GpuRun(w, params, x, y, theta=torch.full((w.L, w.F), float("inf")), decode_mode=GATHER)
    assert g.decode_switch[1] == 0
    for lp in range(w.L):
        assert (g.y_hat[lp] == params["b_dec"][lp].numpy()[None, :]).all()


def test_gather_dz_lds_chunks_and_fallback(monkeypatch):
    """Backward through the lists when a token's d y_hat rows exceed 64 KB of LDS (fp32, d=2048: eight targets per
    chunk, nine targets from layer 0, so a second chunk of one), and the one-wave-per-entry kernel, which otherwise
    runs only when d is not a multiple of 8, forced on the same input: both against the oracle."""
    w = S.scaled(S.WORKLOADS["tiny"], dtype="f32", L=9, d=2048, F=256, B=24, seed=84)
    theta = sparse_theta(w, 0.3)                 # about 77 entries a row: two batches of 64
    g, o = run_both(w, theta=theta, decode_mode=GATHER)
    assert g.decode_switch[2] == 2
    show("gather_dz, chunked LDS staging", compare_step(w, g, o, TOL["f32"]))
    monkeypatch.setenv("CLT_GDZ_NO_LDS", "1")
    params = S.make_params(w)
    x, y = S.make_inputs(w)
    h = GpuRun(w, params, x, y, theta=theta, decode_mode=GATHER)
    for k in O.PARAM_NAMES:                      # same products, other summation order
        assert rel_l2(h.grads[k], g.grads[k]) < 1e-5, k


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gather_equals_dense(dtype):
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=4, d=128, F=512, B=130, seed=79)
    theta = sparse_theta(w, 0.03)
    params = S.make_params(w)
    x, y = S.make_inputs(w)
    a = GpuRun(w, params, x, y, theta=theta, decode_mode=DENSE)
    b = GpuRun(w, params, x, y, theta=theta, decode_mode=GATHER)
    assert (a.z == b.z).all()
    assert rel_l2(b.y_hat, a.y_hat) < 1e-5       # same fp32 sums, different order
    c = GpuRun(w, params, x, y, theta=theta, decode_mode=GATHER)
    assert (b.y_hat == c.y_hat).all()            # the gather path is deterministic
    tol = 1e-5 if dtype == "f32" else 1e-2
    for k in O.PARAM_NAMES:                      # sparse backward: same sums as the dense GEMMs, other order
        assert rel_l2(b.grads[k], a.grads[k]) < tol, k
        assert (b.grads[k] == c.grads[k]).all(), k
        assert (b.new_params[k] == c.new_params[k]).all(), k


@pytest.mark.parametrize("dtype,master", [("f32", False), ("bf16", False), ("bf16", True)])
def test_sparse_backward_fused_adam(dtype, master):
    """Backward through the decoder on the active-feature lists, Adam inside the row kernel."""
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=3, d=264, F=520, B=150, seed=81, master_weights=master)
    theta = sparse_theta(w, 0.04)
    g, o = run_both(w, theta=theta, decode_mode=GATHER, fused=True)
    assert g.decode_switch[2] == 2 and g.window.sum() > 20
    show(f"sparse bwd fused {dtype} master={master}", compare_step(w, g, o, TOL[dtype]))


@pytest.mark.parametrize("dtype,d", [("bf16", 256), ("f32", 96), ("bf16", 2304)])
def test_sparse_backward_column_slices_match_whole_rows(monkeypatch, dtype, d):
    """The row kernel of dW_dec cut into eight column slices (one per XCD; d a multiple of 32) against the kernel that
    takes whole rows.  With fp32 storage both sum a feature's tokens in the same order, one multiply-add each:
    gradients and the fused update must agree bit for bit; with bf16 storage the slices use packed dot products and
    agree to rounding.  d = 2304: two passes of lanes per slice, the second one ragged."""
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=4, d=d, F=264, B=90, seed=85, master_weights=dtype == "bf16")
    theta = sparse_theta(w, 0.06)
    params = S.make_params(w)
    x, y = S.make_inputs(w)
    monkeypatch.setenv("CLT_NO_FUSED_DZ", "1")       # (dz from the separate gather kernel both times)
    for fused in (False, True):
        monkeypatch.delenv("CLT_SD_ROWS", raising=False)
        a = GpuRun(w, params, x, y, theta=theta, decode_mode=GATHER, fused=fused)
        monkeypatch.setenv("CLT_SD_ROWS", "1")
        b = GpuRun(w, params, x, y, theta=theta, decode_mode=GATHER, fused=fused)
        assert a.decode_switch[2] == 2
        if dtype == "f32":
            if not fused:
                assert (a.grads["W_dec"] == b.grads["W_dec"]).all()
            for k in O.PARAM_NAMES:
                assert (a.new_params[k] == b.new_params[k]).all(), k
                assert (a.new_m[k] == b.new_m[k]).all() and (a.new_v[k] == b.new_v[k]).all(), k
        else:      # bf16: the slices take two tokens per packed dot product, the whole rows one per multiply-add
            if not fused:
                assert rel_l2(a.grads["W_dec"], b.grads["W_dec"]) < 3e-3      # (the gradient is stored as bf16)
            for k in O.PARAM_NAMES:
                assert rel_l2(a.new_m[k], b.new_m[k]) < 1e-5 and rel_l2(a.new_v[k], b.new_v[k]) < 1e-5, k


@pytest.mark.parametrize("dtype,d,rho", [("bf16", 256, 0.05), ("f32", 96, 0.05), ("bf16", 2304, 0.05), ("f32", 64, 0.6)])
def test_dz_taken_inside_the_row_kernel_of_dw_dec(monkeypatch, dtype, d, rho):
    """With lists of at most 128 entries per token the row kernel of dW_dec also takes the dot products that make up
    dz at the listed entries (per target and column slice, summed by a second kernel) and the separate gather kernel
    stands down; CLT_NO_FUSED_DZ switches that off.  Both ways against each other (same products, other summation
    order) and against the oracle; rho = 0.6 makes lists longer than the room for partial sums, so the separate
    kernel runs either way and the results are identical."""
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=4, d=d, F=264, B=90, seed=86, master_weights=dtype == "bf16")
    theta = sparse_theta(w, rho)
    params = S.make_params(w)
    x, y = S.make_inputs(w)
    for fused in (False, True):
        monkeypatch.delenv("CLT_NO_FUSED_DZ", raising=False)
        a = GpuRun(w, params, x, y, theta=theta, decode_mode=GATHER, fused=fused)
        monkeypatch.setenv("CLT_NO_FUSED_DZ", "1")
        b = GpuRun(w, params, x, y, theta=theta, decode_mode=GATHER, fused=fused)
        monkeypatch.delenv("CLT_NO_FUSED_DZ", raising=False)
        assert a.decode_switch[2] == 2 and a.window.sum() > 0
        longest = int(a.decode_switch[3])
        assert longest == int((a.active | a.window).sum(axis=(1, 2)).max())
        took_dz = longest <= w.B * 128
        assert took_dz == (rho < 0.5)
        tol = 1e-5 if dtype == "f32" else 1e-2
        assert rel_l2(a.dpre, b.dpre) < tol
        if not took_dz:
            assert (a.dpre == b.dpre).all()
        if not fused:
            for k in O.PARAM_NAMES:
                assert rel_l2(a.grads[k], b.grads[k]) < tol, k
    o = OracleRun(w, params, x, y, theta=theta, gpu_active=a.active, gpu_window=a.window)
    show(f"fused dz {dtype} d={d} rho={rho}", compare_step(w, a, o, TOL[dtype]))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_dz_inside_the_row_kernel_long_feature_lists(dtype):
    """Features listed by more than 64 tokens (about 90 of 300 here, up to about 120): the row kernel hands the
    dz sums of a feature over 64 tokens at a time, the last group ragged.  Lists stay under 128 entries per token
    (about 80), so dz is taken inside the row kernel."""
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=3, d=256, F=264, B=300, seed=89)
    theta = sparse_theta(w, 0.3)
    g, o = run_both(w, theta=theta, decode_mode=GATHER, fused=True)
    per_feature = (g.active | g.window).sum(axis=1)
    assert per_feature.max() > 100 and int(g.decode_switch[3]) <= 128 * w.B
    show(f"fused dz, long feature lists {dtype}", compare_step(w, g, o, TOL[dtype]))


def test_sparse_backward_many_layers():
    """More than 8 targets per source: the row kernel walks them in two chunks."""
    w = S.scaled(S.WORKLOADS["tiny"], dtype="bf16", L=11, d=64, F=256, B=48, seed=82)
    theta = sparse_theta(w, 0.05)
    for fused in (False, True):
        g, o = run_both(w, theta=theta, decode_mode=GATHER, fused=fused)
        show(f"sparse bwd L=11 fused={fused}", compare_step(w, g, o, TOL["bf16"]))


def test_sparse_backward_with_dead_feature_term():
    w = S.scaled(S.WORKLOADS["tiny"], dtype="bf16", L=3, d=128, F=512, B=130, seed=83, lambda1=5.0,
                 log_threshold=True)
    theta = torch.log(sparse_theta(w, 0.03))
    g, o = run_both(w, theta=theta, decode_mode=GATHER, fused=True)
    assert g.decode_switch[2] == 2
    dead_term_matters(w, o, TOL["bf16"])
    show("sparse bwd + dead term", compare_step(w, g, o, TOL["bf16"]))


@pytest.mark.parametrize("d", [264, 256])      # whole-row kernel + separate gather dz / column slices with dz inside
def test_sparse_backward_int8_inputs(d):
    w = S.scaled(S.WORKLOADS["llama1b_int8"], L=2, d=d, F=520, B=300, k_active=8)
    theta = sparse_theta(w, 0.03)
    g, o = run_both(w, theta=theta, decode_mode=GATHER, fused=True)
    show(f"sparse bwd int8 d={d}", compare_step(w, g, o, TOL["bf16"]))


def test_auto_switch_follows_measured_density():
    w = S.scaled(S.WORKLOADS["tiny"], dtype="bf16", L=3, d=128, F=1024, B=256, seed=80)
    params = S.make_params(w)
    x, y = S.make_inputs(w)
    # early-training density (about half the features active): dense path
    g = GpuRun(w, params, x, y, decode_mode=AUTO, gather_density_threshold=0.02)
    assert (g.decode_switch[0] & 3) == 0 and g.decode_switch[2] == 1
    # sparse regime: gather path, same result as the oracle
    theta = sparse_theta(w, 0.01)
    g = GpuRun(w, params, x, y, theta=theta, decode_mode=AUTO, gather_density_threshold=0.02)
    o = OracleRun(w, params, x, y, gpu_active=g.active, gpu_window=g.window, theta=theta)
    assert (g.decode_switch[0] & 3) == 3 and g.decode_switch[2] == 2      # both the decode and the backward on the lists
    show("auto -> gather", compare_step(w, g, o, TOL["bf16"]))
    # one token with a huge norm lights up far more features than a capped list holds: the mean density is still
    # below the threshold, but the step must decode densely; the backward, which takes dz inside the row kernel of
    # dW_dec and so works from the per-feature lists alone, stays on the lists
    x2 = x.clone()
    x2[:, 7, :] *= 300.0
    x2 = x2.bfloat16().float()
    theta = sparse_theta(w, 0.004)               # (rows are capped at 32 x threshold x F + 64 = 328 entries here)
    g = GpuRun(w, params, x2, y, theta=theta, decode_mode=AUTO, gather_density_threshold=0.008)
    o = OracleRun(w, params, x2, y, gpu_active=g.active, gpu_window=g.window, theta=theta)
    kcap = (int(32.0 * 0.008 * w.F) + 64 + 7) // 8 * 8
    assert g.active.mean() < 0.008
    assert g.decode_switch[0] == 7 and g.decode_switch[1] > kcap and g.decode_switch[2] == 1 and g.decode_switch[3] > 0
    show("auto -> dense fallback", compare_step(w, g, o, TOL["bf16"]))


@pytest.mark.parametrize("dtype,fused", [("bf16", True), ("f32", False), ("bf16", False)])
def test_auto_dense_decode_with_list_driven_backward(dtype, fused):
    """The automatic mode has two thresholds: between them the forward decode stays a dense GEMM while dz, dW_dec and
    its Adam update run on the active-feature lists (whose kernels pay up to a higher density).  Against the oracle,
    and the forward bit-identical to the dense mode's."""
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=3, d=128, F=1024, B=256, seed=87, master_weights=dtype == "bf16")
    params = S.make_params(w)
    x, y = S.make_inputs(w)
    theta = sparse_theta(w, 0.01)
    g = GpuRun(w, params, x, y, theta=theta, decode_mode=AUTO, gather_density_threshold=0.002,
               list_backward_density_threshold=0.05, fused=fused)
    assert (g.decode_switch[0] & 3) == 2 and g.decode_switch[2] == 1      # backward on the lists, decode dense
    dn = GpuRun(w, params, x, y, theta=theta, decode_mode=DENSE, fused=fused)
    assert (g.y_hat == dn.y_hat).all() and g.loss[0] == dn.loss[0]
    # the list-driven kernels did the work: the scan of the feature lists left their longest layer total
    assert int(g.decode_switch[3]) == int((g.active | g.window).sum(axis=(1, 2)).max())
    o = OracleRun(w, params, x, y, gpu_active=g.active, gpu_window=g.window, theta=theta)
    show(f"auto: dense decode, lists backward {dtype} fused={fused}", compare_step(w, g, o, TOL[dtype]))
    # above both thresholds everything is dense, below both everything on the lists
    hi = GpuRun(w, params, x, y, theta=theta, decode_mode=AUTO, gather_density_threshold=0.002,
                list_backward_density_threshold=0.005, fused=fused)
    assert (hi.decode_switch[0] & 3) == 0 and hi.decode_switch[2] == 1 and hi.decode_switch[3] == 0
    lo = GpuRun(w, params, x, y, theta=theta, decode_mode=AUTO, gather_density_threshold=0.02,
                list_backward_density_threshold=0.05, fused=fused)
    assert (lo.decode_switch[0] & 3) == 3 and lo.decode_switch[2] == 2


@pytest.mark.parametrize("dtype,lambda1", [("bf16", 0.0), ("f32", 0.0), ("bf16", 3.0)])
def test_auto_hands_long_lists_back_to_the_dense_backward(dtype, lambda1):
    """Automatic mode, mean density below the backward threshold, but one layer's lists are longer than the room for
    the partial sums of the fused dz (sized from that threshold): the scan of the feature lists clears the backward
    bit and dz / dW_dec run as dense GEMMs -- the separate gather dz kernel would be slower than those."""
    w = S.scaled(S.WORKLOADS["tiny"], dtype=dtype, L=3, d=128, F=1024, B=256, seed=88, lambda1=lambda1)
    params = S.make_params(w)
    x, y = S.make_inputs(w)
    theta = sparse_theta(w, 0.01)
    theta[0] = sparse_theta(w, 0.12)[0]          # 123 of 1024 per token in layer 0, mean density 0.047
    room = int(1.25 * 0.05 * w.F) + 32           # 96 entries per token
    g = GpuRun(w, params, x, y, theta=theta, decode_mode=AUTO, gather_density_threshold=0.002,
               list_backward_density_threshold=0.05, fused=True)
    assert abs(g.active.mean() - 0.047) < 0.01
    assert int(g.decode_switch[3]) > room * w.B and (g.decode_switch[0] & 3) == 0 and g.decode_switch[2] == 1
    dn = GpuRun(w, params, x, y, theta=theta, decode_mode=DENSE, fused=True)
    # the dense kernels ran: the decoder update has the dense mode's bits (the vectors' gradients are reduced by
    # another kernel in the automatic mode, in another order)
    assert (g.new_params["W_dec"] == dn.new_params["W_dec"]).all()
    for k in O.PARAM_NAMES:
        assert rel_l2(g.new_params[k], dn.new_params[k]) < 1e-3, k
    o = OracleRun(w, params, x, y, gpu_active=g.active, gpu_window=g.window, theta=theta)
    if lambda1:
        dead_term_matters(w, o, TOL[dtype])
    show(f"auto: long lists -> dense backward {dtype} lambda1={lambda1}", compare_step(w, g, o, TOL[dtype]))


def test_restored_state_reproduces_the_step_bitwise():
    """Two fused steps from a saved copy of (parameters, moments) against the same two steps after restoring that
    copy into the same buffers: every bit of the state and of the loss must come out the same (the step keeps no
    hidden state in its workspace between calls, and the dense path has a fixed summation order)."""
    from paper_2603_21014_amd import binding as K
    w = S.scaled(S.WORKLOADS["gpt2"], L=3, d=256, F=520, B=300, seed=62, master_weights=True)
    dev = "cuda:0"
    params = S.make_params(w)
    x, y = (t.to(dev, torch.bfloat16) for t in S.make_inputs(w))
    gp = {k: p.to(dev, torch.bfloat16 if k in ("W_enc", "W_dec") else torch.float32) for k, p in params.items()}
    gm = {k: torch.zeros(p.shape, dtype=torch.float32, device=dev) for k, p in gp.items()}
    gv = {k: torch.zeros(p.shape, dtype=torch.float32, device=dev) for k, p in gp.items()}
    master = {k: params[k].to(dev) for k in ("W_enc", "W_dec")}
    step = K.CLTStep(w.L, w.d, w.F, w.B, dtype="bf16", master_weights=True, C_=w.C, ste_bandwidth=w.ste_eps,
                     matrix_grads=False)
    step.train_step(x, y, gp, gm, gv, 1, w.lr, w.lambda0, master)          # some history in the moments
    state = [gp, gm, gv, master]
    saved = [{k: t.clone() for k, t in s.items()} for s in state]

    def two_steps():
        losses = []
        for t in (2, 3):
            step.train_step(x, y, gp, gm, gv, t, w.lr, w.lambda0, master)
            losses.append(step.loss_dev.cpu().clone())
        return losses, [{k: t.clone() for k, t in s.items()} for s in state]

    loss_a, end_a = two_steps()
    step.workspace_fill(0xCD)                                            # nothing may survive in the workspace
    for s, c in zip(state, saved):
        for k in s:
            s[k].copy_(c[k])
    loss_b, end_b = two_steps()
    torch.cuda.synchronize()
    for a, b in zip(loss_a, loss_b):
        assert torch.equal(a, b)
    for sa, sb in zip(end_a, end_b):
        for k in sa:
            assert torch.equal(sa[k], sb[k]), k
    assert not torch.equal(end_a[0]["W_dec"], saved[0]["W_dec"])


def test_rerun_is_bitwise_deterministic():
    w = S.scaled(S.WORKLOADS["gpt2"], L=3, d=256, F=512, B=300)
    params = S.make_params(w)
    x, y = S.make_inputs(w)
    a = GpuRun(w, params, x, y)
    b = GpuRun(w, params, x, y)
    assert a.loss == b.loss
    for k in O.PARAM_NAMES:
        assert (a.grads[k] == b.grads[k]).all(), k
        assert (a.new_params[k] == b.new_params[k]).all(), k


def test_call_order_and_argument_errors():
    from paper_2603_21014_amd import binding as K
    step = K.CLTStep(2, 64, 128, 32, dtype="f32")
    w = S.scaled(S.WORKLOADS["tiny"], L=2, d=64, F=128, B=32)
    params = {k: p.cuda() for k, p in S.make_params(w).items()}
    x, y = (t.cuda() for t in S.make_inputs(w))
    with pytest.raises(K.CLTError) as e:
        step.loss(y, 1.0)
    assert e.value.code == -6
    step.forward(x, params)
    with pytest.raises(K.CLTError) as e:
        step.backward(x, params)
    assert e.value.code == -6
    with pytest.raises(ValueError):
        step.forward(x[:, :16], params)                 # wrong shape is caught before the ABI
    with pytest.raises(K.CLTError) as e:                # misaligned pointer is caught by the ABI
        K._check(K._lib.clt_forward(step.H.h, None, x.data_ptr() + 4, None, params["W_enc"].data_ptr(),
                                    params["b_enc"].data_ptr(), params["theta"].data_ptr(),
                                    params["W_dec"].data_ptr(), params["b_dec"].data_ptr(), step.z.data_ptr(),
                                    None, step.act_class.data_ptr(), step.y_hat.data_ptr(), None), step.H.h)
    assert e.value.code == -3
    torch.cuda.synchronize()
