"""Host-side checks that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad configurations before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def K():
    import __graft_entry__ as g
    if not os.path.exists(os.path.join(ROOT, "paper_2603_21014_amd", "libclt.so")):
        g.build()
    from paper_2603_21014_amd import binding
    return binding


def test_library_exports_every_declared_symbol(K):
    header = open(os.path.join(ROOT, "include", "clt.h")).read()
    declared = set(re.findall(r"^(?:int|const char\*)\s+(clt_\w+)\s*\(", header, flags=re.M))
    assert declared == set(K.EXPORTS)
    lib = ctypes.CDLL(K.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_config_struct_matches_header(K):
    assert ctypes.sizeof(K.clt_config) == 4 * 13 + 4 * 7
    assert ctypes.sizeof(K.clt_tensors) == 5 * ctypes.sizeof(ctypes.c_void_p)


def test_workspace_size_and_shape_validation(K):
    cfg = K.make_config(4, 64, 256, 128, dtype=K.DTYPE_F32)
    n = K.clt_workspace_bytes(cfg)
    # at least norms + G + d_yhat + dpre
    assert n >= 2 * 4 * 256 * 4 + 4 * 128 * 64 * 4 + 4 * 128 * 256 * 4
    for bad in (dict(d=63), dict(F=12), dict(L=0), dict(B=0), dict(L=200)):
        kw = dict(L=4, d=64, F=256, B=128)
        kw.update(bad)
        with pytest.raises(K.CLTError) as e:
            K.clt_workspace_bytes(K.make_config(**kw))
        assert e.value.code == -2, bad
    with pytest.raises(K.CLTError) as e:
        K.clt_workspace_bytes(K.make_config(4, 64, 256, 128, dtype=7))
    assert e.value.code == -1
    with pytest.raises(K.CLTError) as e:
        K.clt_workspace_bytes(K.make_config(4, 64, 256, 128, dtype=K.DTYPE_F32, input_format=K.INPUT_INT8_ROWSCALE))
    assert e.value.code == -1
    cfg = K.make_config(4, 64, 256, 128)
    cfg.size = 8
    with pytest.raises(K.CLTError):
        K.clt_workspace_bytes(cfg)


def test_automatic_mode_thresholds_and_workspace(K):
    """The two density thresholds of the automatic mode are checked, and the workspace grows with the larger of them
    (capped lists, their transpose and the room for the partial sums of the fused dz)."""
    base = dict(L=4, d=64, F=256, B=128, decode_mode=K.DECODE_AUTO)
    for bad in (dict(gather_density_threshold=-0.1), dict(gather_density_threshold=1.5),
                dict(list_backward_density_threshold=-0.1), dict(list_backward_density_threshold=2.0)):
        with pytest.raises(K.CLTError) as e:
            K.clt_workspace_bytes(K.make_config(**base, **bad))
        assert e.value.code == -1, bad
    dense = K.clt_workspace_bytes(K.make_config(4, 64, 256, 128))
    small = K.clt_workspace_bytes(K.make_config(**base, gather_density_threshold=0.004))
    same = K.clt_workspace_bytes(K.make_config(**base, gather_density_threshold=0.004,
                                               list_backward_density_threshold=0.004))
    large = K.clt_workspace_bytes(K.make_config(**base, gather_density_threshold=0.004,
                                                list_backward_density_threshold=0.1))
    assert dense < small == same < large      # 0 for the second threshold means: the same as the first


def test_init_rejects_bad_workspace_before_any_device_call(K):
    cfg = K.make_config(4, 64, 256, 128)
    h = ctypes.c_void_p()
    rc = K._lib.clt_init(ctypes.byref(h), ctypes.byref(cfg), None, 0)
    assert rc == -4 and not h.value
    assert b"workspace" in K._lib.clt_last_error(None)


def test_generator_is_seeded_and_bf16_representable():
    import torch
    from workloads import clt_synth as S
    w = S.scaled(S.WORKLOADS["gpt2"], L=2, d=32, F=64, B=40)
    p1, p2 = S.make_params(w), S.make_params(w)
    x1, y1 = S.make_inputs(w)
    x2, y2 = S.make_inputs(w)
    assert all(torch.equal(p1[k], p2[k]) for k in p1) and torch.equal(x1, x2) and torch.equal(y1, y2)
    for t in (p1["W_enc"], p1["W_dec"], x1, y1):
        assert torch.equal(t, t.bfloat16().float())
    assert p1["W_dec"].shape == (3, 64, 32) and float(p1["theta"][0, 0]) == pytest.approx(0.03)
