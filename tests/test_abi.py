"""The C-ABI library loads, exports every symbol include/*.h declares and
rejects bad arguments on the host, before anything is launched (so these
run without a GPU)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import dk_inputs
import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def dk():
    import paper_2207_00083_amd as dk
    if not os.path.exists(dk.lib_path()):
        from paper_2207_00083_amd.build import build_library
        build_library()
    dk.load()
    return dk


def declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            text = open(os.path.join(inc, f)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(dkf?_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(dk):
    names = declared_symbols()
    for must in ("dk_encode", "dk_linear_fwd", "dk_conv_fwd", "dk_wgrad", "dk_decode", "dk_verify",
                 "dk_coeffs", "dk_workspace_bytes", "dkf_coeffs", "dkf_quantize", "dkf_dequantize",
                 "dkf_encode", "dkf_linear_fwd", "dkf_decode_verify", "dkf_wgrad",
                 "dkf_fwd_workspace_bytes", "dkf_wgrad_workspace_bytes", "dkf_conv_fwd",
                 "dkf_conv_fwd_workspace_bytes"):
        assert must in names
    lib = C.CDLL(dk.lib_path())
    for n in names:
        assert hasattr(lib, n), n


def test_no_torch_or_oracle_in_the_library(dk):
    blob = open(dk.lib_path(), "rb").read()
    assert b"libtorch" not in blob and b"dk_oracle" not in blob


def test_status_strings(dk):
    assert dk.dk_status_str(0) == "ok"
    assert len({dk.dk_status_str(i) for i in range(9)}) == 9


def test_null_and_shape_errors_before_launch(dk):
    lib = dk.load()
    one = C.c_void_p(16)      # non-NULL, never dereferenced: every call below fails validation first
    null = C.c_void_p(0)
    assert lib.dk_encode(null, one, one, one, 1, 2, 8, null) == 1
    assert lib.dk_encode(one, one, one, one, 0, 2, 8, null) == 2
    assert lib.dk_encode(one, one, one, one, 1, 0, 8, null) == 2
    assert lib.dk_encode(one, one, one, one, 1, dk.DK_MAX_K + 1, 8, null) == 2
    assert lib.dk_encode(one, one, one, one, 1, 2, 0, null) == 2
    assert lib.dk_encode(C.c_void_p(18), one, one, one, 1, 2, 8, null) == 4
    assert lib.dk_decode(one, null, one, 1, 2, 8, null) == 1
    assert lib.dk_decode(one, one, one, 1, 2, -1, null) == 2
    assert lib.dk_verify(one, one, 1e-3, null, null, 1, 2, 8, one, 1 << 20, null) == 1
    assert lib.dk_verify(one, one, 1e-3, one, null, 1, 2, 8, null, 0, null) == 5
    assert lib.dk_verify(one, one, 1e-3, one, null, 1, 2, 8, one, 8, null) == 5
    assert lib.dk_verify(one, one, -1.0, one, null, 1, 2, 8, one, 1 << 20, null) == 2
    assert lib.dk_linear_fwd(one, one, null, 4, 4, 4, one, 1 << 20, null) == 1
    assert lib.dk_linear_fwd(one, one, one, 4, 0, 4, one, 1 << 20, null) == 2
    assert lib.dk_linear_fwd(one, one, one, 4, 4, 4, null, 0, null) == 5
    lay = dk.DkLayer.of(dk_inputs.conv(4, 4, 8, 8, 3))
    one256, f32 = C.c_void_p(256), C.c_float
    assert lib.dk_conv_fwd(None, one, one, one, 4, one, 1 << 20, null) == 1
    assert lib.dk_conv_fwd(C.byref(lay), one, one, one, 0, one, 1 << 20, null) == 2
    assert lib.dk_conv_fwd(C.byref(lay), one, one, one, 4, one, 8, null) == 5
    lin = dk.DkLayer.of(dk_inputs.linear(4, 4))
    assert lib.dk_conv_fwd(C.byref(lin), one, one, one, 4, one, 1 << 20, null) == 3
    bad = dk.DkLayer.of(dk_inputs.conv(4, 4, 2, 2, 5, 1, 0))      # filter larger than padded image
    assert lib.dk_conv_fwd(C.byref(bad), one, one, one, 4, one, 1 << 20, null) == 2
    assert lib.dk_wgrad(C.byref(lay), one, one, one, one, null, 1, 2, 1.0, 0, one, 1 << 20, null) == 1
    assert lib.dk_wgrad(C.byref(lay), one, one, one, one, one, 1, 2, 1.0, 0, one, 8, null) == 5
    assert lib.dk_wgrad(C.byref(lay), one, one, one, one, one, 1, 99, 1.0, 0, one, 1 << 20, null) == 2
    # forward + decode + verify in one call
    assert lib.dk_conv_fwd_decode_verify(C.byref(lay), one, one, one, one, f32(1e-3), null, one, null, 1, 2,
                                         one256, 1 << 30, null) == 1
    assert lib.dk_conv_fwd_decode_verify(C.byref(lay), one, one, one, one, f32(1e-3), one, one, null, 0, 2,
                                         one256, 1 << 30, null) == 2
    assert lib.dk_conv_fwd_decode_verify(C.byref(lin), one, one, one, one, f32(1e-3), one, one, null, 1, 2,
                                         one256, 1 << 30, null) == 3
    assert lib.dk_conv_fwd_decode_verify(C.byref(lay), one, one, one, one, f32(1e-3), one, one, null, 1, 2,
                                         one256, 64, null) == 5
    assert lib.dk_conv_fwd_decode_verify(C.byref(lay), one, one, one, one, f32(1e-3), one, one, null, 1, 2,
                                         one, 1 << 30, null) == 4
    assert dk.dk_conv_fwd_decode_verify_workspace_bytes(dk_inputs.conv(4, 4, 8, 8, 3), 2, 2) > 0
    assert dk.dk_conv_fwd_decode_verify_workspace_bytes(dk_inputs.linear(4, 4), 2, 2) == 0
    # tuning switches
    assert lib.dk_set_option(7, 1) == 2 and lib.dk_set_option(0, 5) == 2
    assert lib.dk_set_option(dk.DK_OPT_FUSE_WGRAD, dk.DK_FUSE_NEVER) == 0
    assert dk.dk_get_option(dk.DK_OPT_FUSE_WGRAD) == dk.DK_FUSE_NEVER
    assert lib.dk_set_option(dk.DK_OPT_FUSE_WGRAD, dk.DK_FUSE_AUTO) == 0
    assert dk.dk_get_option(99) == -1
    # the entry point without a workspace: argument errors first, then its group limit
    assert lib.dk_decode_verify_static(one, one, one, 1e-3, null, one, null, 1, 2, 8, null) == 1
    assert lib.dk_decode_verify_static(one, one, one, 1e-3, one, one, null, 1, 0, 8, null) == 2
    assert lib.dk_decode_verify_static(one, one, one, 1e-3, one, one, null, 4097, 2, 8, null) == 8
    assert lib.dk_static_scratch_bytes() == 4 << 20


def test_workspace_queries(dk):
    L = dk_inputs.conv(64, 64, 32, 32, 3)
    assert dk.dk_workspace_bytes(L, dk.DK_OP_FWD, 64, 4) >= 256
    m = dk.dk_layer_out_len(L)
    assert m == 64 * 32 * 32 and dk.dk_layer_in_len(L) == 64 * 32 * 32
    assert dk.dk_workspace_bytes(L, dk.DK_OP_WGRAD, 64, 4) >= 64 * 6 * m * 4
    assert dk.dk_workspace_bytes(None, dk.DK_OP_VERIFY, 64, 4) > 0
    assert dk.dk_workspace_bytes(L, dk.DK_OP_FWD, 0, 4) == 0
    assert dk.dk_workspace_bytes(L, 7, 4, 4) == 0
    assert dk.dk_layer_out_len(dk_inputs.conv(3, 64, 224, 224, 7, 2, 3)) == 64 * 112 * 112


@pytest.mark.parametrize("K", [1, 2, 4, 8, 16])
def test_host_coefficients_match_the_oracle(dk, K):
    rng = np.random.default_rng(K)
    A, gamma = dk_inputs.sample_coeff_draws(rng, 7, K)
    Ainv, nvec, B = dk.dk_coeffs(A, gamma)
    oAinv, onvec, oB = oracle.coefficients(A, gamma)
    for got, ref in ((Ainv, oAinv), (nvec, onvec), (B, oB)):
        assert got.dtype == np.float32
        assert np.max(np.abs(got - ref)) <= 2e-7 * np.max(np.abs(ref)) + 1e-12


def test_host_coefficients_reject_singular(dk):
    A = np.ones((1, 4, 4), dtype=np.float32)
    g = np.ones((1, 4), dtype=np.float32)
    with pytest.raises(dk.DkError) as e:
        dk.dk_coeffs(A, g)
    assert e.value.status == 7
    A = np.eye(4, dtype=np.float32)[None]
    g[0, 2] = 0.0
    with pytest.raises(dk.DkError) as e:
        dk.dk_coeffs(A, g)
    assert e.value.status == 7


def test_product_does_not_import_the_oracle():
    import subprocess, sys
    code = ("import sys; import paper_2207_00083_amd; "
            "assert not any(m == 'oracle' or m.startswith('oracle.') for m in sys.modules), 'oracle imported'")
    subprocess.run([sys.executable, "-c", code], check=True, cwd=ROOT)
    for root, _, files in os.walk(os.path.join(ROOT, "paper_2207_00083_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                assert "oracle" not in open(os.path.join(root, f)).read().lower().replace("no fallback", ""), f


def test_field_errors_before_launch(dk):
    lib = dk.load()
    one, null = C.c_void_p(256), C.c_void_p(0)
    assert lib.dkf_quantize(null, one, 8, 8, null) == 1
    assert lib.dkf_quantize(one, one, 0, 8, null) == 2
    assert lib.dkf_quantize(one, one, 8, 13, null) == 2
    assert lib.dkf_dequantize(one, one, 8, -1, null) == 2
    assert lib.dkf_encode(one, one, one, null, 1, 2, 8, 8, null) == 1
    assert lib.dkf_encode(one, one, one, one, 1, 17, 8, 8, null) == 2
    assert lib.dkf_encode(one, C.c_void_p(258), one, one, 1, 2, 8, 8, null) == 4
    assert lib.dkf_linear_fwd(one, one, one, 4, 4, 4, null, 0, null) == 5
    assert lib.dkf_linear_fwd(one, one, one, 4, 4, 4, one, 16, null) == 5
    assert lib.dkf_linear_fwd(one, one, one, 0, 4, 4, one, 1 << 30, null) == 2
    assert lib.dkf_decode_verify(one, one, one, one, null, null, 1, 2, 8, 8, null) == 1
    lin = dk.DkLayer.of(dk_inputs.linear(4, 4))
    conv = dk.DkLayer.of(dk_inputs.conv(4, 4, 8, 8, 3))
    assert lib.dkf_wgrad(C.byref(conv), one, one, one, one, one, null, 1, 2, 8, 1.0, 0, one, 64, null) == 5
    assert lib.dkf_conv_fwd(C.byref(lin), one, one, one, 4, one, 1 << 30, null) == 3
    assert lib.dkf_conv_fwd(C.byref(conv), one, one, one, 0, one, 1 << 30, null) == 2
    assert lib.dkf_conv_fwd(C.byref(conv), one, one, one, 4, one, 64, null) == 5
    assert lib.dkf_wgrad(C.byref(lin), one, one, one, one, one, null, 1, 2, 8, 1.0, 0, one, 64, null) == 5
    f = C.c_float
    assert lib.dkf_norm_scales(null, one, 1, 8, f(1.0), null) == 1
    assert lib.dkf_norm_scales(one, one, 0, 8, f(1.0), null) == 2
    assert lib.dkf_norm_scales(one, one, 65536, 8, f(1.0), null) == 2
    assert lib.dkf_norm_scales(one, one, 1, 8, f(0.0), null) == 2
    assert lib.dkf_quantize_norm(one, null, one, 1, 8, 8, null) == 1
    assert lib.dkf_quantize_norm(one, one, one, 1, 8, 13, null) == 2
    assert lib.dkf_encode_norm(one, null, one, one, one, 1, 2, 8, 8, null) == 1
    assert lib.dkf_encode_rng_norm(one, null, one, one, 1, 2, 8, 8, 0, null) == 1
    assert lib.dkf_encode_rng_norm(one, one, one, one, 1, 17, 8, 8, 0, null) == 2
    assert lib.dkf_decode_verify_norm(one, one, one, one, null, one, null, one, 1, 2, 8, 8, null) == 1
    assert lib.dkf_wgrad_norm(C.byref(lin), one, null, one, one, one, one, null, 1, 2, 8, f(1.0), 0, one, 64,
                              null) == 1
    assert dk.dkf_fwd_workspace_bytes(4, 4, 4) > 0 and dk.dkf_fwd_workspace_bytes(0, 4, 4) == 0
    assert dk.dkf_wgrad_workspace_bytes(dk_inputs.linear(4, 4), 1, 2) > 0
    # entry points added later: real weights into the dense forward, the bias, depthwise layers, the rate probe
    assert lib.dkf_linear_fwd_w(null, 8, one, one, 4, 4, 4, one, 1 << 30, null) == 1
    assert lib.dkf_linear_fwd_w(one, 13, one, one, 4, 4, 4, one, 1 << 30, null) == 2
    assert lib.dkf_linear_fwd_w(one, 8, one, one, 4, 4, 4, one, 16, null) == 5
    assert lib.dkf_add_bias(null, null, one, 4, 8, 1, 8, null) == 1
    assert lib.dkf_add_bias(one, null, one, 4, 8, 3, 8, null) == 2          # per does not divide m
    assert lib.dkf_add_bias(one, null, one, 4, 8, 1, 13, null) == 2
    assert lib.dkf_add_bias(C.c_void_p(258), null, one, 4, 8, 1, 8, null) == 4
    dw = dk_inputs.dwconv(4, 8, 8, 3)
    assert dk.dkf_conv_fwd_workspace_bytes(dw, 4) > 0 and dk.dkf_wgrad_workspace_bytes(dw, 1, 2) > 0
    assert lib.dkf_wgrad(C.byref(dk.DkLayer.of(dw)), one, one, one, one, one, null, 1, 2, 8, 1.0, 0, one, 64,
                         null) == 5
    assert lib.dkf_probe_mfma_rate(0, 0, null, null) == 2
    assert lib.dkf_probe_mfma_rate(3, 10, null, null) == 2


def test_field_coeffs_match_the_oracle_and_report_singular(dk):
    from oracle import field as F
    rng = np.random.default_rng(3)
    for K in (1, 4, 16):
        S = K + 2
        A = rng.integers(0, F.P, size=(3, S, S), dtype=np.uint32)
        gamma = rng.integers(1, F.P, size=(3, S), dtype=np.uint32)
        for got, want in zip(dk.dkf_coeffs(A, gamma), F.coefficients(A, gamma)):
            assert np.array_equal(got, want)
    A = np.ones((1, 3, 3), dtype=np.uint32)
    with pytest.raises(dk.DkError) as e:
        dk.dkf_coeffs(A, np.ones((1, 3), dtype=np.uint32))
    assert e.value.status == 7
    A = np.eye(3, dtype=np.uint32)[None]
    with pytest.raises(dk.DkError) as e:
        dk.dkf_coeffs(A, np.array([[1, 0, 1]], dtype=np.uint32))
    assert e.value.status == 7
    with pytest.raises(dk.DkError) as e:
        dk.dkf_coeffs(A * np.uint32(F.P), np.ones((1, 3), dtype=np.uint32))
    assert e.value.status == 2
