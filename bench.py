#!/usr/bin/env python3
"""Benchmark of the CLT train step (forward + loss + backward + Adam) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama1b]

Prints ONE JSON line: tokens/s of the whole step on synthetic inputs resident in
HBM, the roofline entry of the dominant kernel (timed live with HIP events on
the stream the kernels run on) and the CPU oracle timed on a bounded sample.
Everything runs on one GPU; --gpus above 1 exits with a message.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
GEMM_PAIRS = {"encoder_jumprelu_gemm": "L", "dW_enc_gemm": "L", "decode_gemm": "P", "dz_gemm": "P",
              "dW_dec_gemm": "P"}


KERNEL_SYMBOL = {"decode_gemm": "gemm_bf16_kernel<DecPolicy>", "dz_gemm": "gemm_bf16_kernel<DzPolicy>",
                 "dW_dec_gemm": "gemm_bf16_kernel<DWdecPolicy>", "encoder_jumprelu_gemm": "gemm_bf16_kernel<EncPolicy>",
                 "dW_enc_gemm": "gemm_bf16_kernel<DWencPolicy>"}


def profiled_traffic_bytes(workload, kernel):
    """HBM-side bytes per step of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE,
    calibrated against a plain copy) and the name of that file, or (None, None).  Hardware counters cannot be
    read from inside this process; the figure is the one of the profiled run, labelled with its source."""
    rel = os.path.join("profiles", f"train_step_{workload}_hbm_traffic.md")
    try:
        for line in open(os.path.join(ROOT, rel)):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) > 3 and cells[1] == KERNEL_SYMBOL.get(kernel):
                return (float(cells[2]) + float(cells[3])) * 1e9, rel
    except (OSError, ValueError):
        pass
    return None, None


def theta_for_density(x, W_enc, b_enc, rho):
    """Input recipe of the density sweep: per-layer thresholds (constant over features) at which a fraction rho of
    that layer's pre-activations lies above them, from a quantile of a subsample.  Chooses an input tensor only."""
    import torch
    L, F = x.shape[0], W_enc.shape[2]
    out = torch.empty((L, F), device=x.device, dtype=torch.float32)
    for l in range(L):
        s = (x[l] @ W_enc[l] + b_enc[l]).reshape(-1)
        if s.numel() > (1 << 22):
            s = s[:: s.numel() // (1 << 22)]
        kth = min(s.numel(), max(1, int(round(s.numel() * (1.0 - rho)))))
        out[l] = torch.kthvalue(s, kth).values
    return out


DIAG_VARIANTS = (
    # (name, mode bits of clt_diag_mfma_loop without the data bit)
    ("mfma_only", 0),
    ("mfma_only_32x32x16_shape", 128),
    ("mfma+lds_reads", 2),
    ("mfma+lds_reads+lds_writes", 6),
    ("mfma+lds+loads_from_L2", 14),
    ("mfma+lds+loads_half_from_infinity_cache", 30),
    # the same parts arranged for one wavefront per SIMD (4 waves, 8x8 accumulators each), and with direct-to-LDS staging
    ("one_wave_per_simd:mfma_only", 32),
    ("one_wave_per_simd:mfma+lds+loads_from_L2", 46),
    ("one_wave_per_simd:mfma+lds+loads_half_from_infinity_cache", 62),
    ("one_wave_per_simd:mfma+lds_reads+direct_to_lds_loads_from_L2", 110),
    ("one_wave_per_simd:mfma+lds_reads+direct_to_lds_loads_half_from_infinity_cache", 126),
)


def run_diag(dev, mode, iters, counters, buf):
    """One timed launch of the diagnostic loop: (TFLOP/s, ms, shader clock in GHz or None)."""
    import torch
    from paper_2603_21014_amd import binding as K
    K.clt_diag_mfma_loop(max(1, iters // 8), mode, counters, buf)      # warm-up (and the buffer fill)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    flop, hz = K.clt_diag_mfma_loop(iters, mode, counters, buf)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    c = counters.cpu().tolist()
    clock = c[0] / c[1] * hz / 1e9 if c[1] > 0 else None
    return {"tflops": round(flop / (ms * 1e-3) / 1e12, 1), "ms": round(ms, 3),
            "shader_clock_ghz": round(clock, 3) if clock else None}


def mfma_ceiling(dev, log, iters=40000, all_variants=False):
    """The MFMA stream of the contraction kernel on this GPU with its operands in registers (no memory traffic
    at all), on all-zero and on pseudo-random bf16 data: TFLOP/s from HIP events on the launch stream and the
    shader clock from the kernel's own cycle counters.  The bf16 MFMA rate is limited by board power and the
    power depends on the operand bits, so the two differ; the random-data figure is the ceiling for real data.
    all_variants adds the LDS and memory traffic of the real kernel back one part at a time (same loop, no data
    flow between the parts): what each part costs in clock and rate."""
    import torch
    out = {}
    counters = torch.zeros(4, dtype=torch.int64, device=dev)
    buf = None
    if all_variants:
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        buf = torch.empty(cus * (576 << 10), dtype=torch.uint8, device=dev)
    for vname, mode in (DIAG_VARIANTS if all_variants else DIAG_VARIANTS[:1]):
        for dname, rnd in (("zero_data", 0), ("random_data", 1)):
            r = run_diag(dev, mode | rnd, iters, counters, buf if mode & 8 else None)
            out.setdefault(vname, {})[dname] = r
            log(f"diagnostic loop {vname}, {dname}: {r['tflops']} TFLOP/s at {r['shader_clock_ghz']} GHz")
    out["what"] = ("v_mfma_f32_16x16x32_bf16 stream of the contraction kernel, 8 wavefronts per CU, operands in "
                   "registers (mfma_only: no LDS or global memory access)")
    return out


def library_gemm_reference(w, dev, log):
    """Context for the MFMA figures, not part of the step: what the vendor library (torch.matmul) sustains on this
    very GPU for one plain bf16 GEMM of the decode's shape (M = tokens, N = d_model, K = 16 F: the longest group
    of the triangular decode at L = 16) on random normal operands, measured after the timed region."""
    import torch
    M, N, Kd = w.B, w.d, 16 * w.F
    g = torch.Generator(device=dev).manual_seed(1)
    a = torch.randn((M, Kd), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    b = torch.randn((Kd, N), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    for _ in range(2):
        torch.matmul(a, b)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    iters = 10
    for _ in range(iters):
        torch.matmul(a, b)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    tf = 2.0 * M * N * Kd / (ms * 1e-3) / 1e12
    log(f"vendor library bf16 GEMM {M}x{N}x{Kd}: {ms:.3f} ms, {tf:.0f} TFLOP/s")
    del a, b
    return {"what": "torch.matmul, bf16, random normal operands", "M": M, "N": N, "K": Kd, "ms": round(ms, 4),
            "tflops": round(tf, 1)}


def cpu_oracle_baseline(w, log):
    """The oracle as it stands on a bounded sample of the workload: full L and d,
    F/4 features and B/8 tokens (about 10-20 s of host time).  The contraction cost
    is linear in B*F, Adam and the decoder norms in F, so the sample time is scaled
    back to the full shape and expressed in tokens/s."""
    import numpy as np
    import torch
    from oracle import clt_oracle as O
    from workloads import clt_synth as S
    fs, bs = max(8, w.F // 4), max(1, w.B // 8)
    ws = S.scaled(w, F=fs, B=bs, k_active=max(1, w.k_active // 4))
    params = {k: v.numpy().astype(np.float64) for k, v in S.make_params(ws).items()}
    x, y = (t.numpy().astype(np.float64) for t in S.make_inputs(ws))
    zeros = {k: np.zeros_like(v) for k, v in params.items()}
    t0 = time.perf_counter()
    theta = O.threshold_value(params["theta"], ws.log_threshold)
    topk = max(1, ws.topk // 4) if ws.topk else None          # the sample has a quarter of the features
    fwd = O.forward(x, params["W_enc"], params["b_enc"], theta, params["W_dec"], params["b_dec"], topk=topk)
    n = O.decoder_norms(params["W_dec"], ws.L)
    O.loss_terms(fwd["y_hat"], y, fwd["z"], n, ws.lambda0, ws.C)
    O.dead_feature_term(fwd["pre"], theta, n, ws.lambda1)
    grads = O.backward(x, y, theta, params["W_dec"], fwd, ws.lambda0, ws.C, ws.ste_eps, lambda1=ws.lambda1,
                       log_threshold=ws.log_threshold, topk=topk is not None)
    t1 = time.perf_counter()
    for k in O.PARAM_NAMES:
        O.adam_update(params[k], grads["d" + k], zeros[k], zeros[k], 1, ws.lr)
    t2 = time.perf_counter()
    t_fb, t_adam = t1 - t0, t2 - t1
    full = t_fb * (w.F / fs) * (w.B / bs) + t_adam * (w.F / fs)
    log(f"cpu oracle sample: fwd+loss+bwd {t_fb:.2f}s, adam {t_adam:.2f}s -> full step est {full:.0f}s")
    # the oracle is numpy: its matmuls run on the BLAS pool's threads, everything else on one
    threads = 1
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    except Exception:
        threads = int(os.environ.get("OMP_NUM_THREADS", "1") or 1)
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"value": w.B / full, "unit": "tokens/s", "cores": threads, "host_cpus": os.cpu_count(), "cpu_model": model,
            "kind": "oracle",
            "sample": f"L={ws.L} d={ws.d} F={fs} (1/{w.F // fs}) B={bs} (1/{w.B // bs}) of {w.name}; "
                      f"measured {t_fb + t_adam:.1f}s, scaled by B*F (contractions) and F (Adam)"}


def density_sweep(args, log):
    """Sec. 3.2 crossover on this GPU: the dense decode against the gather decode
    (compaction + gather) at forced activation densities, and the whole train step
    with the dense and with the list-driven backward.  Two input recipes at the int8
    Llama shape: token norms with a heavy tail (a few tokens carry most of the active
    features) and uniform token norms (what Sec. 3.1's normalisation produces).
    Prints one JSON line of its own."""
    import torch
    from paper_2603_21014_amd import binding as K
    from workloads import clt_synth as S
    dev, T = "cuda:0", torch.bfloat16
    out = {"metric": "gather vs dense decode crossover (active features per token and layer)", "recipes": {}}
    for recipe, w in (("heavy_tailed_tokens", S.WORKLOADS["llama1b_int8"]),
                      ("uniform_tokens", S.scaled(S.WORKLOADS["llama1b_int8"], outliers=False))):
        p32 = S.make_params(w, device=dev)
        x32, y32 = S.make_inputs(w, device=dev)
        xq, xs = S.quantize_rows_int8(x32)
        yq, ys = S.quantize_rows_int8(y32)
        xdq = xq.float() * xs[:, :, None]
        del x32, y32
        params = {k: (v.to(T) if k in ("W_enc", "W_dec") else v.clone()) for k, v in p32.items()}
        m = {k: torch.zeros(v.shape, dtype=torch.float32, device=dev) for k, v in params.items()}
        v_ = {k: torch.zeros(v.shape, dtype=torch.float32, device=dev) for k, v in params.items()}
        rows = []
        steps = {name: K.CLTStep(w.L, w.d, w.F, w.B, dtype="bf16", int8_inputs=True, C_=w.C,
                                 ste_bandwidth=w.ste_eps, device=dev, keep_pre=False, decode_mode=mode,
                                 matrix_grads=False)
                 for name, mode in (("dense", K.DECODE_DENSE), ("gather", K.DECODE_GATHER))}
        # dense forward decode, list-driven backward: the automatic mode with the first threshold at 0, the second at 1
        steps["hybrid"] = K.CLTStep(w.L, w.d, w.F, w.B, dtype="bf16", int8_inputs=True, C_=w.C,
                                    ste_bandwidth=w.ste_eps, device=dev, keep_pre=False, decode_mode=K.DECODE_AUTO,
                                    gather_density_threshold=0.0, list_backward_density_threshold=1.0,
                                    matrix_grads=False)
        t = 0
        for rho in (0.00025, 0.0005, 0.001, 0.0025, 0.005, 0.01, 0.015, 0.02, 0.05):
            theta = theta_for_density(xdq, p32["W_enc"], p32["b_enc"], rho)
            row = {"density": rho}
            for name, st in steps.items():
                params["theta"].copy_(theta)
                for it in range(3):
                    if it == 1:
                        K.clt_profile_enable(st.H, True)
                    t += 1
                    # lr 0: the density stays put
                    st.train_step(xq, yq, params, m, v_, t, 0.0, w.lambda0, None, xs, ys)
                torch.cuda.synchronize()
                prof = K.clt_profile_query(st.H)
                K.clt_profile_enable(st.H, False)
                ms = {k: v[0] / 2.0 for k, v in prof.items()}    # two profiled steps
                row[name + "_step_ms"] = round(sum(ms.values()), 2)
                if name == "hybrid":      # (lists too long for the fused dz: the automatic mode goes back to the dense kernels)
                    row["hybrid_backward_on_lists"] = bool(int(K.clt_workspace_view(st.H, "decode_switch")[0].item()) & 2)
                    continue
                if name == "dense":
                    row["dense_decode_ms"] = round(ms["decode_gemm"], 3)
                    row["dense_dz_ms"] = round(ms["dz_gemm"], 3)
                    row["dense_dW_dec_ms"] = round(ms["dW_dec_gemm"], 3)
                else:
                    row["gather_decode_ms"] = round(ms["compact_active"] + ms["gather_decode"], 3)
                    row["compact_ms"] = round(ms["compact_active"], 3)
                    row["gather_dz_ms"] = round(ms["sparse_dpre_fill"] + ms["gather_dz"], 3)
                    row["sparse_dW_dec_ms"] = round(ms["feature_lists"] + ms["sparse_dW_dec"], 3)
                    k_mean = st.l0.double().mean().item() / w.B
                    row["active_per_token_layer"] = round(k_mean, 1)
                    gbytes = w.B * k_mean * w.P * w.d * 2.0
                    row["gather_GBps"] = round(gbytes / (ms["gather_decode"] * 1e-3) / 1e9, 1)
                    # lists of at most 128 entries per token: the row kernel of dW_dec takes the dot products of dz
                    # as well and "gather_dz" is only the kernel that sums them
                    longest = int(K.clt_workspace_view(st.H, "decode_switch")[3].item())
                    row["dz_in_row_kernel"] = longest <= w.B * 128
                    row["gather_dz_GBps"] = (None if row["dz_in_row_kernel"]
                                             else round(gbytes / (ms["gather_dz"] * 1e-3) / 1e9, 1))
                    row["lists_backward_decoder_ms"] = round(row["gather_dz_ms"] + row["sparse_dW_dec_ms"], 3)
                    row["dense_backward_decoder_ms"] = None
                    # every parameter's weight, moments read and written once by the row kernel
                    row["sparse_dW_dec_GBps"] = round(w.P * w.F * w.d * 20.0 / (ms["sparse_dW_dec"] * 1e-3) / 1e9, 1)
            row["dense_backward_decoder_ms"] = round(row["dense_dz_ms"] + row["dense_dW_dec_ms"], 3)
            log(recipe + " " + str(row))
            rows.append(row)
        cross = None
        for a, b in zip(rows, rows[1:]):
            fa, fb = a["gather_decode_ms"] - a["dense_decode_ms"], b["gather_decode_ms"] - b["dense_decode_ms"]
            if fa <= 0 < fb:
                tt = fa / (fa - fb)
                cross = a["active_per_token_layer"] + tt * (b["active_per_token_layer"] - a["active_per_token_layer"])
        out["recipes"][recipe] = {"workload": w.name, "expansion": w.F / w.d, "crossover_k": cross, "rows": rows}
        del steps, params, m, v_, p32, xq, yq, xdq
        torch.cuda.empty_cache()
    print(json.dumps(out), flush=True)


def power_probe(args, log):
    """What limits the bf16 MFMA rate on this board (one JSON line): the diagnostic loop's variants, then the
    forward pass of the library on the workload's data and on all-zero inputs and weights (same kernels, same
    instruction count; only the operand bits differ), with the decode contraction's time for each."""
    import torch
    from paper_2603_21014_amd import binding as K
    from workloads import clt_synth as S
    dev, T = "cuda:0", torch.bfloat16
    out = {"metric": "bf16 MFMA rate against operand content and data movement", "loop": mfma_ceiling(dev, log, all_variants=True)}
    w = S.WORKLOADS[args.workload]
    p32 = S.make_params(w, device=dev)
    params = {k: (v.to(T) if k in ("W_enc", "W_dec") else v) for k, v in p32.items()}
    del p32
    x, _ = S.make_inputs(w, device=dev)
    x = x.to(T)
    step = K.CLTStep(w.L, w.d, w.F, w.B, dtype="bf16", C_=w.C, ste_bandwidth=w.ste_eps, device=dev, keep_pre=False,
                     matrix_grads=False)
    pair = 2.0 * w.B * w.F * w.d
    out["decode_gemm"] = {}
    for name in ("workload_data", "zero_data"):
        if name == "zero_data":
            x.zero_(); params["W_dec"].zero_(); params["W_enc"].zero_()
        for it in range(4):
            if it == 1:
                K.clt_profile_enable(step.H, True)
            step.forward(x, params)
        torch.cuda.synchronize()
        prof = K.clt_profile_query(step.H)
        K.clt_profile_enable(step.H, False)
        ms = prof["decode_gemm"][0] / prof["decode_gemm"][1]
        ems = prof["encoder_jumprelu_gemm"][0] / prof["encoder_jumprelu_gemm"][1]
        out["decode_gemm"][name] = {"ms": round(ms, 3), "tflops": round(w.P * pair / (ms * 1e-3) / 1e12, 1),
                                    "encoder_ms": round(ems, 3), "encoder_tflops": round(w.L * pair / (ems * 1e-3) / 1e12, 1),
                                    "active_fraction": round(step.l0.double().sum().item() / (w.L * w.B * w.F), 4)}
        log(f"forward on {name}: decode {ms:.3f} ms = {out['decode_gemm'][name]['tflops']} TFLOP/s, "
            f"encoder {ems:.3f} ms = {out['decode_gemm'][name]['encoder_tflops']} TFLOP/s")
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama1b")
    ap.add_argument("--no-library-gemm", action="store_true",
                    help="skip the vendor-library GEMM reference measured after the timed region")
    ap.add_argument("--decode-mode", default="dense", choices=["dense", "gather", "auto"],
                    help="dense GEMMs (default), the list-driven kernels of the sparse regime, or the device-side switch")
    ap.add_argument("--gather-density-threshold", type=float, default=0.0045,
                    help="auto mode: the forward decode gathers at or below this mean active fraction (measured "
                         "break-even on an MI355X: 0.0047-0.0052)")
    ap.add_argument("--list-backward-density-threshold", type=float, default=0.016,
                    help="auto mode: the backward through the decoder runs on the active-feature lists at or below "
                         "this mean active fraction (measured break-even: about 0.02)")
    ap.add_argument("--density", type=float, default=None,
                    help="force the activation density of a JumpReLU workload: per-layer thresholds at which this "
                         "fraction of the pre-activations is active (the recipe of --density-sweep), learning rate 0 so "
                         "that it stays put; the step does all of its work as usual")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="skip the per-kernel HIP-event brackets (roofline entry becomes null)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="end with one plain 1 GiB device copy (the last dispatch): reference for HBM byte counters")
    ap.add_argument("--power-probe", action="store_true",
                    help="instead of the train step: the contraction kernel's instruction stream taken apart (MFMA "
                         "only, + LDS reads, + LDS writes, + loads), on zero and on random data, and the decode "
                         "contraction itself on zero and on the workload's data")
    ap.add_argument("--density-sweep", action="store_true",
                    help="time dense vs gather decode at forced densities instead of the train step")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs the CLT train step on ONE GPU only (no sharding, no collectives); "
                 "use --gpus 1")

    def log(msg):
        print(f"[bench] {msg}", file=sys.stderr, flush=True)

    if args.density_sweep:
        return density_sweep(args, log)
    if args.power_probe:
        return power_probe(args, log)

    import torch
    from paper_2603_21014_amd import binding as K
    from workloads import clt_synth as S

    w = S.WORKLOADS[args.workload]
    assert w.dtype == "bf16", "the benchmark times the bf16 path"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    t0 = time.perf_counter()
    T = torch.bfloat16
    params32 = S.make_params(w, device=dev)
    params = {k: (v.to(T) if k in ("W_enc", "W_dec") else v) for k, v in params32.items()}
    master = {k: params32[k] for k in ("W_enc", "W_dec")} if w.master_weights else None
    x, y = S.make_inputs(w, device=dev)
    xs = ys = None
    if w.int8_inputs:
        x, xs = S.quantize_rows_int8(x)
        y, ys = S.quantize_rows_int8(y)
    else:
        x, y = x.to(T), y.to(T)
    lr = w.lr
    if args.density is not None:
        assert not w.topk and not w.log_threshold, "--density sets the thresholds of a JumpReLU workload"
        xf = x.float() * xs[:, :, None] if w.int8_inputs else x.float()
        params["theta"] = theta_for_density(xf, params32["W_enc"], params32["b_enc"], args.density)
        lr = 0.0
        del xf
    del params32
    m = {k: torch.zeros(v.shape, dtype=torch.float32, device=dev) for k, v in params.items()}
    v_ = {k: torch.zeros(v.shape, dtype=torch.float32, device=dev) for k, v in params.items()}
    step = K.CLTStep(w.L, w.d, w.F, w.B, dtype="bf16", int8_inputs=w.int8_inputs, master_weights=w.master_weights,
                     C_=w.C, ste_bandwidth=w.ste_eps, device=dev, keep_pre=w.lambda1 > 0,
                     log_threshold=w.log_threshold, topk=w.topk or None,
                     decode_mode={"dense": K.DECODE_DENSE, "gather": K.DECODE_GATHER, "auto": K.DECODE_AUTO}[args.decode_mode],
                     gather_density_threshold=args.gather_density_threshold,
                     list_backward_density_threshold=args.list_backward_density_threshold, matrix_grads=False,
                     reuse_decoder_norms=True)
    torch.cuda.synchronize()
    log(f"workload {w.name}: L={w.L} d={w.d} F={w.F} B={w.B}, inputs ready in {time.perf_counter() - t0:.1f}s, "
        f"{torch.cuda.memory_allocated() / 2**30:.1f} GiB allocated")

    def one_step(t):
        step.train_step(x, y, params, m, v_, t, lr, w.lambda0, master, xs, ys, lambda1=w.lambda1)

    t = 0
    for _ in range(args.warmup):
        t += 1
        one_step(t)
    torch.cuda.synchronize()
    log("warmup done")
    # timed region: exactly `steps` steps, no per-kernel event brackets, no host synchronisation inside
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        t += 1
        one_step(t)
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    loss = step.loss_dev.cpu().tolist()
    l0 = (step.l0.double().mean() / w.B).item()
    log(f"{ms_per_step:.2f} ms/step, loss {loss[0]:.4g}, mean active features/token/layer {l0:.1f}")

    flop = w.dense_flop_per_step()
    roof, kernels, median_ms = None, None, None
    if not args.no_kernel_timing:
        # second pass over the same steps: every kernel bracketed by HIP events on the launch stream (about 40
        # event records per step, kept out of the timed region above), and each step timed on its own
        K.clt_profile_enable(step.H, True)
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        evs[0].record()
        for i in range(args.steps):
            t += 1
            one_step(t)
            evs[i + 1].record()
        torch.cuda.synchronize()
        per = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps))
        median_ms = per[len(per) // 2] if len(per) % 2 else 0.5 * (per[len(per) // 2 - 1] + per[len(per) // 2])
        prof = K.clt_profile_query(step.H)
        K.clt_profile_enable(step.H, False)
        pair = 2.0 * w.B * w.F * w.d
        kernels = {}
        for name, (ms, n) in prof.items():
            if n == 0:
                continue
            avg = ms / n
            ent = {"avg_ms": round(avg, 4), "launches_per_step": n / args.steps}
            if name in GEMM_PAIRS:
                fl = pair * (w.L if GEMM_PAIRS[name] == "L" else w.P)
                ent["tflops"] = round(fl / (avg * 1e-3) / 1e12, 1)
                ent["flop"] = fl
            kernels[name] = ent
        # algorithmic bytes of the list-driven kernels: decoder rows of the listed features (decode, dz), the
        # weights and moments read and written once (row kernel of dW_dec)
        rows_bytes = w.B * l0 * w.P * w.d * 2.0
        hbm_bytes = {"gather_decode": rows_bytes, "gather_dz": rows_bytes, "sparse_dW_dec": 20.0 * w.P * w.F * w.d}
        # the two weight-gradient kernels carry the fused Adam update: per parameter the bf16 weight and the fp32
        # moments (and master copy) are read and written once (20 or 30 bytes), plus the operands once.  Where
        # that takes longer at 8 TB/s than the kernel's flop at the MFMA peak, HBM is the roof that bounds it.
        per_param = 30.0 if w.master_weights else 20.0
        act = 2.0 * w.L * w.B          # bytes of one bf16 [L, B, .] activation per unit of width
        fused_bytes = {"dW_dec_gemm": per_param * w.P * w.F * w.d + act * (w.F + w.d),
                       "dW_enc_gemm": per_param * w.L * w.F * w.d + act * (w.F + w.d) * (0.5 if w.int8_inputs else 1.0)}
        for k, b in fused_bytes.items():
            if k in kernels and b / 8e12 > kernels[k]["flop"] / (PEAK_BF16_TFLOPS * 1e12):
                hbm_bytes[k] = b
        per_step = lambda k: kernels[k]["avg_ms"] * kernels[k]["launches_per_step"]
        dom = max((k for k in kernels if k in GEMM_PAIRS or k in hbm_bytes), key=per_step)
        if dom in GEMM_PAIRS and dom not in hbm_bytes:
            ach = kernels[dom]["tflops"]
            traffic, source = profiled_traffic_bytes(w.name, dom)
            roof = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(ach / PEAK_BF16_TFLOPS, 4), "traffic": traffic, "traffic_source": source,
                    "avg_launch_ms": kernels[dom]["avg_ms"], "flop_per_launch": kernels[dom]["flop"]}
        else:
            ach = hbm_bytes[dom] / (kernels[dom]["avg_ms"] * 1e-3) / 1e9
            roof = {"kernel": dom, "bound": "hbm", "achieved": round(ach, 1), "peak": 8000.0, "unit": "GB/s",
                    "frac": round(ach / 8000.0, 4), "traffic": None, "traffic_source": None,
                    "avg_launch_ms": kernels[dom]["avg_ms"], "bytes_per_launch": hbm_bytes[dom]}
            if dom in GEMM_PAIRS:     # context: the same kernel against the MFMA roof it is not bound by
                roof["mfma_tflops"] = kernels[dom]["tflops"]
        for name, ent in sorted(kernels.items(), key=lambda kv: -kv[1]["avg_ms"] * kv[1]["launches_per_step"]):
            log(f"  {name:24s} {ent['avg_ms']:9.3f} ms x {ent['launches_per_step']:.0f}"
                + (f"  {ent['tflops']:7.1f} TFLOP/s" if "tflops" in ent else ""))

    if args.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        src.fill_(1)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()

    lib_gemm = ceiling = None
    if not args.no_library_gemm:
        lib_gemm = library_gemm_reference(w, dev, log)
        ceiling = mfma_ceiling(dev, log)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_oracle_baseline(w, log)

    out = {
        "metric": "CLT train-step tokens/s (fwd+bwd+Adam, bf16)", "value": w.B / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "L": w.L, "d_model": w.d, "features_per_layer": w.F, "tokens": w.B,
                   "decoder_blocks": w.P, "int8_inputs": w.int8_inputs, "master_weights": w.master_weights,
                   "activation": f"topk{w.topk}" if w.topk else "jumprelu", "decode_mode": args.decode_mode,
                   "fused_adam": True, "reuse_decoder_norms": True, "forced_density": args.density,
                   "active_per_token_layer": l0},
        "median_ms_per_step_profiled_pass": median_ms,
        "step_dense_tflops": flop / (ms_per_step * 1e-3) / 1e12,
        "step_frac_of_bf16_mfma_peak": flop / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "roofline": roof, "cpu_baseline": cpu, "kernels": kernels, "library_gemm": lib_gemm, "mfma_ceiling": ceiling,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
