"""ctypes binding of libclt.so (include/clt.h).

Argument marshalling only: every step of the CLT train step runs in the HIP
kernels of the library.  torch is used for device memory and streams.  The
module-level functions carry the C names and take torch tensors; `CLTStep`
bundles a handle with its workspace and output buffers.

Importing this module without a built libclt.so raises: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libclt.so")

CLT_OK = 0
DTYPE_F32, DTYPE_BF16 = 0, 1
INPUT_NATIVE, INPUT_INT8_ROWSCALE = 0, 1
DECODE_AUTO, DECODE_DENSE, DECODE_GATHER = 0, 1, 2

EXPORTS = ("clt_workspace_bytes", "clt_init", "clt_destroy", "clt_last_error", "clt_forward",
           "clt_loss", "clt_backward", "clt_adam_step", "clt_backward_adam_step", "clt_workspace_view",
           "clt_profile_enable", "clt_profile_num_kernels", "clt_profile_query", "clt_norm_accumulate",
           "clt_normalise", "clt_diag_mfma_loop", "clt_norm_accumulate_static")


class CLTError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libclt error {code}: {msg}")
        self.code = code


class clt_config(C.Structure):
    _fields_ = [("size", C.c_uint32), ("L", C.c_int32), ("d", C.c_int32), ("F", C.c_int32), ("B", C.c_int32),
                ("dtype", C.c_int32), ("input_format", C.c_int32), ("master_weights", C.c_int32),
                ("decode_mode", C.c_int32), ("log_threshold", C.c_int32), ("activation", C.c_int32), ("topk_k", C.c_int32),
                ("reuse_decoder_norms", C.c_int32),
                ("gather_density_threshold", C.c_float), ("list_backward_density_threshold", C.c_float),
                ("C", C.c_float),
                ("ste_bandwidth", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("adam_eps", C.c_float)]


class clt_tensors(C.Structure):
    _fields_ = [("W_enc", C.c_void_p), ("b_enc", C.c_void_p), ("theta", C.c_void_p),
                ("W_dec", C.c_void_p), ("b_dec", C.c_void_p)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = C.CDLL(LIB_PATH)
    vp, fp = C.c_void_p, C.c_void_p
    lib.clt_workspace_bytes.argtypes = [C.POINTER(clt_config), C.POINTER(C.c_size_t)]
    lib.clt_init.argtypes = [C.POINTER(vp), C.POINTER(clt_config), vp, C.c_size_t]
    lib.clt_destroy.argtypes = [vp]
    lib.clt_last_error.argtypes = [vp]
    lib.clt_last_error.restype = C.c_char_p
    lib.clt_forward.argtypes = [vp, vp] + [vp] * 12
    lib.clt_loss.argtypes = [vp, vp, vp, fp, fp, vp, vp, fp, C.c_float, C.c_float, fp, C.POINTER(C.c_float)]
    lib.clt_backward.argtypes = [vp, vp, vp, fp, fp, vp, vp, vp, C.POINTER(clt_tensors)]
    lib.clt_adam_step.argtypes = [vp, vp, C.c_int64, C.c_float] + [C.POINTER(clt_tensors)] * 5
    lib.clt_backward_adam_step.argtypes = [vp, vp, vp, fp, vp, vp, C.c_int64, C.c_float] + [C.POINTER(clt_tensors)] * 5
    lib.clt_workspace_view.argtypes = [vp, C.c_int, C.POINTER(vp), C.POINTER(C.c_size_t)]
    lib.clt_norm_accumulate.argtypes = [vp, vp, vp, fp, vp]
    lib.clt_normalise.argtypes = [vp, vp, vp, C.c_int64, vp, fp, vp, fp]
    lib.clt_profile_enable.argtypes = [vp, C.c_int]
    lib.clt_profile_num_kernels.argtypes = []
    lib.clt_profile_query.argtypes = [vp, C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_double),
                                      C.POINTER(C.c_int64)]
    lib.clt_norm_accumulate_static.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, fp, vp]
    lib.clt_diag_mfma_loop.argtypes = [vp, C.c_int, C.c_int, vp, C.c_size_t, vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    for n in EXPORTS:
        if n != "clt_last_error":
            getattr(lib, n).restype = C.c_int
    return lib


_lib = _load()

_TORCH_T = {DTYPE_F32: torch.float32, DTYPE_BF16: torch.bfloat16}


def _check(rc, handle=None):
    if rc != CLT_OK:
        raise CLTError(rc, _lib.clt_last_error(handle).decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, shape, dtype, name, optional=False):
    """Device pointer of a tensor after checking what the kernels assume."""
    if t is None:
        if optional:
            return None
        raise ValueError(f"{name} is required")
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    if t.dtype != dtype or tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected {tuple(shape)} {dtype}, got {tuple(t.shape)} {t.dtype}")
    return t.data_ptr()


def make_config(L, d, F, B, dtype=DTYPE_BF16, input_format=INPUT_NATIVE, master_weights=False,
                decode_mode=DECODE_DENSE, gather_density_threshold=0.0045, C_=4.0, ste_bandwidth=0.05,
                beta1=0.9, beta2=0.999, adam_eps=1e-8, log_threshold=False, topk=None, reuse_decoder_norms=False,
                list_backward_density_threshold=0.0):
    """topk: None for JumpReLU, else k of the TopK activation.  reuse_decoder_norms: see include/clt.h (the caller
    promises that only clt_backward_adam_step writes W_dec between steps).  list_backward_density_threshold: AUTO
    mode's second threshold, for the backward through the decoder (0 = the same as gather_density_threshold)."""
    return clt_config(C.sizeof(clt_config), L, d, F, B, dtype, input_format, int(master_weights), decode_mode,
                      int(log_threshold), 0 if topk is None else 1, 0 if topk is None else int(topk),
                      int(reuse_decoder_norms), gather_density_threshold, list_backward_density_threshold, C_, ste_bandwidth,
                      beta1, beta2, adam_eps)


def clt_workspace_bytes(cfg: clt_config) -> int:
    n = C.c_size_t(0)
    _check(_lib.clt_workspace_bytes(C.byref(cfg), C.byref(n)))
    return n.value


class Handle:
    """A clt_handle plus the shapes needed to validate tensors on the Python side."""

    def __init__(self, cfg: clt_config, workspace: torch.Tensor):
        self.cfg = cfg
        self.workspace = workspace          # keeps the device memory alive
        h = C.c_void_p()
        _check(_lib.clt_init(C.byref(h), C.byref(cfg), workspace.data_ptr(), workspace.numel()))
        self.h = h
        self.T = _TORCH_T[cfg.dtype]
        self.TX = torch.int8 if cfg.input_format == INPUT_INT8_ROWSCALE else self.T
        L, d, F, B = cfg.L, cfg.d, cfg.F, cfg.B
        P = L * (L + 1) // 2
        self.shapes = {"x": (L, B, d), "y": (L, B, d), "scale": (L, B), "W_enc": (L, d, F), "b_enc": (L, F),
                       "theta": (L, F), "W_dec": (P, F, d), "b_dec": (L, d), "z": (L, B, F), "y_hat": (L, B, d)}

    def close(self):
        if self.h:
            _lib.clt_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def clt_init(cfg: clt_config, workspace: torch.Tensor) -> Handle:
    if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous uint8 device tensor")
    return Handle(cfg, workspace)


def clt_norm_accumulate(H: Handle, a, norm_sum, a_scale=None):
    s = H.shapes
    rc = _lib.clt_norm_accumulate(H.h, _stream(), _ptr(a, s["x"], H.TX, "a"),
                                  _ptr(a_scale, s["scale"], torch.float32, "a_scale", True),
                                  _ptr(norm_sum, (H.cfg.L,), torch.float64, "norm_sum"))
    _check(rc, H.h)


def clt_norm_accumulate_static(a, norm_sum, a_scale=None):
    """clt_norm_accumulate without a handle or workspace (the library's own static scratch); a is [L,B,d] float32,
    bfloat16 or int8 (then a_scale [L,B] float32 is required)."""
    if a is None or a.dim() != 3:
        raise ValueError("a must be a [L, B, d] device tensor")
    L, B, d = a.shape
    int8 = a.dtype == torch.int8
    dt = DTYPE_F32 if a.dtype == torch.float32 else DTYPE_BF16
    if a.dtype not in (torch.float32, torch.bfloat16, torch.int8):
        raise ValueError(f"a: unsupported dtype {a.dtype}")
    rc = _lib.clt_norm_accumulate_static(_stream(), L, B, d, dt, INPUT_INT8_ROWSCALE if int8 else INPUT_NATIVE,
                                         _ptr(a, (L, B, d), a.dtype, "a"),
                                         _ptr(a_scale, (L, B), torch.float32, "a_scale", True),
                                         _ptr(norm_sum, (L,), torch.float64, "norm_sum"))
    _check(rc)


def clt_normalise(H: Handle, norm_sum, n_tokens, a_in=None, scale_in=None, a_out=None, scale_out=None):
    s, f32 = H.shapes, torch.float32
    rc = _lib.clt_normalise(H.h, _stream(), _ptr(norm_sum, (H.cfg.L,), torch.float64, "norm_sum"), int(n_tokens),
                            _ptr(a_in, s["x"], H.T, "a_in", True), _ptr(scale_in, s["scale"], f32, "scale_in", True),
                            _ptr(a_out, s["x"], H.T, "a_out", True), _ptr(scale_out, s["scale"], f32, "scale_out", True))
    _check(rc, H.h)


def clt_forward(H: Handle, x, W_enc, b_enc, theta, W_dec, b_dec, z, act_class, y_hat,
                pre=None, l0_per_layer=None, x_scale=None):
    s, f32 = H.shapes, torch.float32
    rc = _lib.clt_forward(
        H.h, _stream(), _ptr(x, s["x"], H.TX, "x"), _ptr(x_scale, s["scale"], f32, "x_scale", True),
        _ptr(W_enc, s["W_enc"], H.T, "W_enc"), _ptr(b_enc, s["b_enc"], f32, "b_enc"),
        _ptr(theta, s["theta"], f32, "theta"), _ptr(W_dec, s["W_dec"], H.T, "W_dec"),
        _ptr(b_dec, s["b_dec"], f32, "b_dec"), _ptr(z, s["z"], H.T, "z"), _ptr(pre, s["z"], H.T, "pre", True),
        _ptr(act_class, s["z"], torch.uint8, "act_class"), _ptr(y_hat, s["y_hat"], f32, "y_hat"),
        _ptr(l0_per_layer, (H.cfg.L,), torch.int32, "l0_per_layer", True))
    _check(rc, H.h)


def clt_loss(H: Handle, y, y_hat, z, lambda0, loss_dev, y_scale=None, to_host=False, lambda1=0.0, pre=None,
             theta=None):
    s, f32 = H.shapes, torch.float32
    host = (C.c_float * 4)() if to_host else None
    dead = lambda1 > 0.0
    rc = _lib.clt_loss(H.h, _stream(), _ptr(y, s["y"], H.TX, "y"), _ptr(y_scale, s["scale"], f32, "y_scale", True),
                       _ptr(y_hat, s["y_hat"], f32, "y_hat"), _ptr(z, s["z"], H.T, "z"),
                       _ptr(pre, s["z"], H.T, "pre", not dead), _ptr(theta, s["theta"], f32, "theta", not dead),
                       float(lambda0), float(lambda1), _ptr(loss_dev, (4,), f32, "loss_dev"), host)
    _check(rc, H.h)
    return tuple(host) if to_host else None


def _tensors(H: Handle, t: dict, name: str, matrix_dtype, matrices_only=False) -> clt_tensors:
    s, f32 = H.shapes, torch.float32
    out = clt_tensors()
    out.W_enc = _ptr(t["W_enc"], s["W_enc"], matrix_dtype, f"{name}.W_enc")
    out.W_dec = _ptr(t["W_dec"], s["W_dec"], matrix_dtype, f"{name}.W_dec")
    if not matrices_only:
        out.b_enc = _ptr(t["b_enc"], s["b_enc"], f32, f"{name}.b_enc")
        out.theta = _ptr(t["theta"], s["theta"], f32, f"{name}.theta")
        out.b_dec = _ptr(t["b_dec"], s["b_dec"], f32, f"{name}.b_dec")
    return out


def clt_backward(H: Handle, x, theta, W_dec, z, act_class, grads: dict, x_scale=None):
    s, f32 = H.shapes, torch.float32
    g = _tensors(H, grads, "grads", H.T)
    rc = _lib.clt_backward(H.h, _stream(), _ptr(x, s["x"], H.TX, "x"),
                           _ptr(x_scale, s["scale"], f32, "x_scale", True), _ptr(theta, s["theta"], f32, "theta"),
                           _ptr(W_dec, s["W_dec"], H.T, "W_dec"), _ptr(z, s["z"], H.T, "z"),
                           _ptr(act_class, s["z"], torch.uint8, "act_class"), C.byref(g))
    _check(rc, H.h)


def clt_adam_step(H: Handle, t: int, lr: float, params: dict, grads: dict, m: dict, v: dict, master: dict = None):
    f32 = torch.float32
    p = _tensors(H, params, "params", H.T)
    g = _tensors(H, grads, "grads", H.T)
    mm = _tensors(H, m, "m", f32)
    vv = _tensors(H, v, "v", f32)
    ms = _tensors(H, master, "master", f32, matrices_only=True) if master is not None else None
    rc = _lib.clt_adam_step(H.h, _stream(), int(t), float(lr), C.byref(p), C.byref(g), C.byref(mm), C.byref(vv),
                            C.byref(ms) if ms is not None else None)
    _check(rc, H.h)


def clt_backward_adam_step(H: Handle, x, z, act_class, t: int, lr: float, params: dict, grads: dict, m: dict, v: dict,
                           master: dict = None, x_scale=None):
    """grads must hold b_enc, theta, b_dec; W_enc / W_dec entries are optional (written when present)."""
    s, f32 = H.shapes, torch.float32
    p = _tensors(H, params, "params", H.T)
    mm = _tensors(H, m, "m", f32)
    vv = _tensors(H, v, "v", f32)
    ms = _tensors(H, master, "master", f32, matrices_only=True) if master is not None else None
    g = clt_tensors()
    g.b_enc = _ptr(grads["b_enc"], s["b_enc"], f32, "grads.b_enc")
    g.theta = _ptr(grads["theta"], s["theta"], f32, "grads.theta")
    g.b_dec = _ptr(grads["b_dec"], s["b_dec"], f32, "grads.b_dec")
    g.W_enc = _ptr(grads.get("W_enc"), s["W_enc"], H.T, "grads.W_enc", True)
    g.W_dec = _ptr(grads.get("W_dec"), s["W_dec"], H.T, "grads.W_dec", True)
    rc = _lib.clt_backward_adam_step(H.h, _stream(), _ptr(x, s["x"], H.TX, "x"),
                                     _ptr(x_scale, s["scale"], f32, "x_scale", True), _ptr(z, s["z"], H.T, "z"),
                                     _ptr(act_class, s["z"], torch.uint8, "act_class"), int(t), float(lr),
                                     C.byref(p), C.byref(g), C.byref(mm), C.byref(vv),
                                     C.byref(ms) if ms is not None else None)
    _check(rc, H.h)


_VIEWS = {"norms": (0, torch.float32, lambda c: (c.L, c.F)), "d_yhat": (1, None, lambda c: (c.L, c.B, c.d)),
          "dpre": (2, None, lambda c: (c.L, c.B, c.F)), "G": (3, torch.float32, lambda c: (c.L, c.F)),
          "decode_switch": (4, torch.int32, lambda c: (4,))}


def clt_workspace_view(H: Handle, which: str) -> torch.Tensor:
    """A tensor aliasing one of the workspace regions (norms, d_yhat, dpre, G)."""
    idx, dt, shp = _VIEWS[which]
    dt = dt or H.T
    ptr, nbytes = C.c_void_p(), C.c_size_t()
    _check(_lib.clt_workspace_view(H.h, idx, C.byref(ptr), C.byref(nbytes)), H.h)
    off = ptr.value - H.workspace.data_ptr()
    return H.workspace[off:off + nbytes.value].view(dt).view(shp(H.cfg))


def clt_profile_enable(H: Handle, on: bool):
    _check(_lib.clt_profile_enable(H.h, int(on)), H.h)


def clt_profile_query(H: Handle) -> dict:
    """{kernel name: (total device ms, launches)} since profiling was enabled."""
    out = {}
    for k in range(_lib.clt_profile_num_kernels()):
        name, ms, n = C.c_char_p(), C.c_double(), C.c_int64()
        _check(_lib.clt_profile_query(H.h, k, C.byref(name), C.byref(ms), C.byref(n)), H.h)
        out[name.value.decode()] = (ms.value, n.value)
    return out


DIAG_RANDOM_DATA, DIAG_LDS_READS, DIAG_LDS_WRITES, DIAG_LOADS_L2, DIAG_LOADS_FAR = 1, 2, 4, 8, 16


def clt_diag_mfma_loop(iters: int, mode: int, counters: torch.Tensor, buf: torch.Tensor = None):
    """Enqueues the diagnostic MFMA loop (see include/clt.h for the mode bits); returns (flop of the launch, rate
    of the constant-rate counter in Hz).  counters: int64 device tensor of 4 elements; [0] shader cycles, [1]
    constant-rate ticks of one wavefront.  buf: uint8 device scratch for the modes that load from memory."""
    flop, hz = C.c_double(), C.c_double()
    if buf is not None and (buf.dtype != torch.uint8 or not buf.is_cuda or not buf.is_contiguous()):
        raise ValueError("buf must be a contiguous uint8 device tensor")
    _check(_lib.clt_diag_mfma_loop(_stream(), int(iters), int(mode), buf.data_ptr() if buf is not None else None,
                                   buf.numel() if buf is not None else 0,
                                   _ptr(counters, (4,), torch.int64, "counters"), C.byref(flop), C.byref(hz)))
    return flop.value, hz.value


class CLTStep:
    """A handle with its workspace and the per-step buffers of one configuration."""

    def __init__(self, L, d, F, B, dtype="bf16", int8_inputs=False, master_weights=False, C_=4.0,
                 ste_bandwidth=0.05, beta1=0.9, beta2=0.999, adam_eps=1e-8, device="cuda:0", keep_pre=True,
                 decode_mode=DECODE_DENSE, gather_density_threshold=0.0045, matrix_grads=True, log_threshold=False,
                 topk=None, workspace=None, reuse_decoder_norms=False, list_backward_density_threshold=0.016):
        """workspace: a uint8 device tensor of at least clt_workspace_bytes(config) bytes that the caller
        owns (256-byte aligned); by default one is allocated here."""
        dt = DTYPE_BF16 if dtype == "bf16" else DTYPE_F32
        self.cfg = make_config(L, d, F, B, dt, INPUT_INT8_ROWSCALE if int8_inputs else INPUT_NATIVE,
                               master_weights, decode_mode, gather_density_threshold, C_, ste_bandwidth, beta1,
                               beta2, adam_eps, log_threshold, topk, reuse_decoder_norms,
                               list_backward_density_threshold)
        self.device = torch.device(device)
        ws = workspace
        if ws is None:
            ws = torch.empty(clt_workspace_bytes(self.cfg), dtype=torch.uint8, device=self.device)
        self.H = clt_init(self.cfg, ws)
        T = self.H.T
        P = L * (L + 1) // 2
        e = lambda *s, dtype=T: torch.empty(s, dtype=dtype, device=self.device)
        self.z = e(L, B, F)
        self.pre = e(L, B, F) if keep_pre else None
        self.act_class = e(L, B, F, dtype=torch.uint8)
        self.y_hat = e(L, B, d, dtype=torch.float32)
        self.l0 = e(L, dtype=torch.int32)
        self.loss_dev = e(4, dtype=torch.float32)
        self.grads = {"b_enc": e(L, F, dtype=torch.float32), "theta": e(L, F, dtype=torch.float32),
                      "b_dec": e(L, d, dtype=torch.float32)}
        if matrix_grads:    # not needed by the fused backward + Adam path
            self.grads["W_enc"] = e(L, d, F)
            self.grads["W_dec"] = e(P, F, d)

    def workspace_fill(self, byte: int):
        """Overwrites the whole workspace (nothing in it is meant to outlive a step)."""
        self.H.workspace.fill_(byte)

    def forward(self, x, params, x_scale=None):
        clt_forward(self.H, x, params["W_enc"], params["b_enc"], params["theta"], params["W_dec"], params["b_dec"],
                    self.z, self.act_class, self.y_hat, self.pre, self.l0, x_scale)

    def loss(self, y, lambda0, y_scale=None, to_host=False, lambda1=0.0, params=None):
        """`params` (for its theta tensor) is needed only when the dead-feature term is on (lambda1 > 0)."""
        theta = params["theta"] if lambda1 > 0.0 else None
        pre = self.pre if lambda1 > 0.0 else None
        return clt_loss(self.H, y, self.y_hat, self.z, lambda0, self.loss_dev, y_scale, to_host, lambda1, pre, theta)

    def backward(self, x, params, x_scale=None):
        clt_backward(self.H, x, params["theta"], params["W_dec"], self.z, self.act_class, self.grads, x_scale)

    def adam_step(self, t, lr, params, m, v, master=None):
        clt_adam_step(self.H, t, lr, params, self.grads, m, v, master)

    def backward_adam_step(self, x, params, m, v, t, lr, master=None, x_scale=None):
        clt_backward_adam_step(self.H, x, self.z, self.act_class, t, lr, params, self.grads, m, v, master, x_scale)

    def train_step(self, x, y, params, m, v, t, lr, lambda0, master=None, x_scale=None, y_scale=None, fused=True,
                   lambda1=0.0):
        """forward, loss, backward and Adam; `fused` runs Adam inside the weight-gradient GEMMs."""
        self.forward(x, params, x_scale)
        self.loss(y, lambda0, y_scale, False, lambda1, params)
        if fused:
            self.backward_adam_step(x, params, m, v, t, lr, master, x_scale)
        else:
            self.backward(x, params, x_scale)
            self.adam_step(t, lr, params, m, v, master)
