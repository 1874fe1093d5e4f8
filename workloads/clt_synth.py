"""Seeded synthetic workloads shaped like the paper's CLT training runs.

This module only *generates inputs* (activations, targets, initial parameters,
int8 codes).  It holds none of the training step's arithmetic and is the one
module that both the tests' oracle side and the HIP side draw data from.  All
tensors are produced with torch on the requested device from per-tensor seeded
generators and returned as float32 (values rounded to bf16-representable
numbers when the workload's storage type is bf16), so both sides start from
bit-identical numbers.

The shapes follow the paper's setups (App. C Table 1: GPT-2 with L=12, d=768;
Llama-3.2-1B with L=16, d=2048; token batches of thousands) at one GPU's share
of the feature dimension under feature sharding (Sec. 3.3).  The paper trains
on cached OpenWebText activations (Sec. 3.1), which are not available here; the
generator below stands in for them:

* learned parameters: W_enc, W_dec ~ U(-1/sqrt(d), 1/sqrt(d)), biases 0,
  theta = 0.03 (the dense, early-training regime of Sec. 3.2), stored as
  log(0.03) by the workloads that use the log-threshold parameterisation;
* inputs: per-layer Gaussians scaled by (1 + 0.25 l); the "outlier" variant
  multiplies each token by a LogNormal(0, 0.5) norm and 4 fixed dims by 20
  (un-normalised residual-stream structure, cf. Sec. 3.1's normalisation);
* targets: a ground-truth sparse CLT with about k active features per token
  and layer, Exp(1) magnitudes, decoders D[l->l'] = 0.7^(l'-l) D[l], plus
  N(0, 0.01) noise.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class CLTWorkload:
    name: str
    L: int
    d: int
    F: int
    B: int
    dtype: str            # "f32" or "bf16": storage type of x, y, W_enc, W_dec
    k_active: int         # ground-truth active features per token and layer
    outliers: bool        # log-normal token norms + 4 outlier dims
    lambda0: float
    seed: int
    C: float = 4.0
    ste_eps: float = 0.05
    lr: float = 2e-4
    theta0: float = 0.03
    int8_inputs: bool = False
    master_weights: bool = False
    lambda1: float = 0.0          # dead-feature coefficient of the App. B objective (0 = term off)
    log_threshold: bool = False   # the theta tensor stores tau = log(theta)
    topk: int = 0                 # > 0: TopK activation with this k instead of JumpReLU (theta unused)

    @property
    def P(self) -> int:
        return self.L * (self.L + 1) // 2

    def dense_flop_per_step(self) -> float:
        """(2L + 3P) GEMMs of 2*B*F*d flop: encoder fwd + dW_enc per layer,
        decode fwd + dz + dW_dec per decoder block."""
        return (2 * self.L + 3 * self.P) * 2.0 * self.B * self.F * self.d


WORKLOADS = {
    "tiny": CLTWorkload("tiny", 4, 64, 256, 128, "f32", 8, False, 2.0, 1001),
    "gpt2": CLTWorkload("gpt2", 12, 768, 6144, 4096, "bf16", 32, False, 2.0, 1002),
    "llama1b": CLTWorkload("llama1b", 16, 2048, 8192, 4096, "bf16", 64, True, 12.0, 1003),
    "gemma2b": CLTWorkload("gemma2b", 26, 2304, 16384, 2048, "bf16", 64, False, 12.0, 1004,
                           master_weights=True),
    "llama1b_dead": CLTWorkload("llama1b_dead", 16, 2048, 8192, 4096, "bf16", 64, True, 12.0, 1003,
                                lambda1=0.1, log_threshold=True),
    "llama1b_topk": CLTWorkload("llama1b_topk", 16, 2048, 8192, 4096, "bf16", 64, True, 0.0, 1003, topk=64),
    "llama1b_topk16": CLTWorkload("llama1b_topk16", 16, 2048, 8192, 4096, "bf16", 64, True, 0.0, 1003, topk=16),
    "llama1b_int8": CLTWorkload("llama1b_int8", 16, 2048, 8192, 4096, "bf16", 64, True, 12.0,
                                1005, int8_inputs=True),
}


def scaled(w: CLTWorkload, **kw) -> CLTWorkload:
    """A copy of a workload with some sizes replaced (for parity-test slices)."""
    return replace(w, **kw)


def _gen(device, seed: int, idx: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000003 + idx)
    return g


def _round_storage(t: torch.Tensor, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        return t.to(torch.bfloat16).to(torch.float32)
    return t


def make_params(w: CLTWorkload, device="cpu"):
    """Initial learned parameters (float32 tensors on `device`)."""
    a = 1.0 / math.sqrt(w.d)
    W_enc = (torch.rand((w.L, w.d, w.F), generator=_gen(device, w.seed, 1), device=device,
                        dtype=torch.float32) * 2 - 1) * a
    W_dec = torch.empty((w.P, w.F, w.d), device=device, dtype=torch.float32)
    g = _gen(device, w.seed, 2)
    for p in range(w.P):      # block by block: bounded temporaries at large sizes
        W_dec[p] = (torch.rand((w.F, w.d), generator=g, device=device, dtype=torch.float32) * 2 - 1) * a
    return {
        "W_enc": _round_storage(W_enc, w.dtype),
        "b_enc": torch.zeros((w.L, w.F), device=device, dtype=torch.float32),
        "theta": torch.full((w.L, w.F), math.log(w.theta0) if w.log_threshold else w.theta0, device=device,
                            dtype=torch.float32),
        "W_dec": _round_storage(W_dec, w.dtype),
        "b_dec": torch.zeros((w.L, w.d), device=device, dtype=torch.float32),
    }


def make_inputs(w: CLTWorkload, device="cpu"):
    """x (MLP inputs) and y (MLP-output targets), float32 [L, B, d] each."""
    L, B, d, F = w.L, w.B, w.d, w.F
    x = torch.randn((L, B, d), generator=_gen(device, w.seed, 3), device=device, dtype=torch.float32)
    if w.outliers:
        r = torch.exp(0.5 * torch.randn((B,), generator=_gen(device, w.seed, 4), device=device))
        x = x * r[None, :, None]
        dims = torch.randperm(d, generator=_gen("cpu", w.seed, 5))[:4].to(device)
        x[:, :, dims] *= 20.0
    x = x * (1.0 + 0.25 * torch.arange(L, device=device, dtype=torch.float32))[:, None, None]
    x = _round_storage(x, w.dtype)

    # ground-truth sparse CLT
    y = torch.zeros((L, B, d), device=device, dtype=torch.float32)
    carry = torch.zeros((B, d), device=device, dtype=torch.float32)
    gD, gE, gA = _gen(device, w.seed, 6), _gen(device, w.seed, 7), _gen(device, w.seed, 8)
    for l in range(L):
        D = torch.randn((F, d), generator=gD, device=device) / math.sqrt(d)
        E = torch.randn((d, F), generator=gE, device=device) / math.sqrt(d)
        s = x[l] @ E
        flat = s.reshape(-1)
        if flat.numel() > (1 << 22):
            flat = flat[:: flat.numel() // (1 << 22)]
        kth = max(1, int(round(flat.numel() * (1.0 - w.k_active / F))))
        tau = torch.kthvalue(flat, min(kth, flat.numel())).values
        a = -torch.log1p(-torch.rand((B, F), generator=gA, device=device))   # Exp(1)
        a = torch.where(s > tau, a, torch.zeros_like(a))
        carry = 0.7 * carry + a @ D
        y[l] = carry
    y = y + 0.1 * torch.randn((L, B, d), generator=_gen(device, w.seed, 9), device=device)
    y = _round_storage(y, w.dtype)
    return x, y


def quantize_rows_int8(t: torch.Tensor):
    """Symmetric int8 codes with one absmax scale per (layer, token) row.

    s = absmax / 127 (1 for an all-zero row); q = clamp(round_half_even(t / s),
    -127, 127).  Returns (q int8 [L, B, d], s float32 [L, B]).
    """
    absmax = t.abs().amax(dim=2)
    s = torch.where(absmax > 0, absmax / 127.0, torch.ones_like(absmax))
    q = torch.clamp(torch.round(t / s[:, :, None]), -127, 127).to(torch.int8)
    return q, s.to(torch.float32)
