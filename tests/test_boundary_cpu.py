"""The C-ABI library loads without a GPU, exports every symbol the header declares, and rejects
bad arguments on the host before anything is launched (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2605_29727_amd", "libbastion_tv.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2605_29727_amd import build
        build.build()
    L = C.CDLL(LIB)
    L.btv_last_error.restype = C.c_char_p
    for n in ("btv_tree_build_workspace", "btv_tree_verify_attn_workspace", "btv_tree_verify_attn_paged_workspace",
              "btv_tree_accept_workspace"):
        getattr(L, n).restype = C.c_size_t
    return L


def _declared():
    names = set()
    for f in os.listdir(os.path.join(ROOT, "include")):
        if f.endswith(".h"):
            names |= set(re.findall(r"\b(btv_[a-z_0-9]+)\s*\(", open(os.path.join(ROOT, "include", f)).read()))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert getattr(lib, n) is not None


def test_binding_names_match_header():
    from paper_2605_29727_amd import binding
    assert sorted(binding.EXPORTS) == _declared()
    for n in binding.EXPORTS:
        if n != "btv_last_error":
            assert hasattr(binding, n), n


def test_version_and_workspace_queries(lib):
    assert lib.btv_version() >= 1
    assert lib.btv_tree_verify_attn_workspace(64, 8192, 32, 8, 128, 1) > 64 * 8 * 4
    assert lib.btv_tree_verify_attn_workspace(16, 128, 1, 1, 64, 0) >= 256
    assert lib.btv_tree_verify_attn_workspace(0, 128, 1, 1, 64, 0) == 0          # invalid shape -> 0
    assert lib.btv_tree_verify_attn_workspace(16, 128, 3, 2, 64, 0) == 0
    assert lib.btv_tree_verify_attn_fp8kv_workspace(64, 8192, 32, 8, 128) > 64 * 8 * 4
    assert lib.btv_tree_verify_attn_fp8kv_workspace(64, 8192, 32, 8, 64) == 0        # D = 64 is not built for FP8 K/V
    assert lib.btv_tree_verify_attn_paged_fp8kv_workspace(8, 64, 8192, 32, 8, 128) > 0
    assert lib.btv_tree_build_workspace(16, 128256, 64) > 0
    assert lib.btv_tree_build_workspace(17, 128256, 64) == 0
    assert lib.btv_tree_accept_workspace(64, 128256, 0) > 0
    assert lib.btv_tree_accept_workspace(64, 128256, 1) >= 128256 * 4      # the softmax numerators of one row


def test_bad_arguments_are_rejected_on_the_host(lib):
    fake = C.c_void_p(4096)   # never dereferenced: every call below fails validation first
    f0 = C.c_float(0.0)
    rc = lib.btv_tree_verify_attn(fake, fake, fake, fake, 1000, 10, 8, 8, 128, 1, f0, fake, None, C.c_size_t(0), None)
    assert rc == -1 and b"M=1000" in lib.btv_last_error()
    rc = lib.btv_tree_verify_attn(None, fake, fake, fake, 16, 10, 8, 8, 128, 1, f0, fake, None, C.c_size_t(0), None)
    assert rc == -1
    rc = lib.btv_tree_verify_attn(fake, fake, fake, fake, 16, 10, 8, 8, 96, 1, f0, fake, None, C.c_size_t(0), None)
    assert rc == -1 and b"D=96" in lib.btv_last_error()
    rc = lib.btv_tree_verify_attn(fake, fake, fake, fake, 16, 10, 8, 8, 128, 7, f0, fake, None, C.c_size_t(0), None)
    assert rc == -1
    rc = lib.btv_tree_verify_attn(fake, fake, fake, fake, 16, 10, 8, 8, 128, 1, f0, fake, None, C.c_size_t(0), None)
    assert rc == -2 and b"workspace" in lib.btv_last_error()
    rc = lib.btv_tree_verify_attn(fake, fake, fake, fake, 16, 10, 8, 8, 128, 1, f0, fake, C.c_void_p(4096 + 8),
                                  C.c_size_t(1 << 20), None)
    assert rc == -2 and b"aligned" in lib.btv_last_error()
    rc = lib.btv_tree_verify_attn(fake, fake, fake, fake, 16, 10, 8, 8, 128, 1, f0, fake, fake, C.c_size_t(16), None)
    assert rc == -2 and b"too small" in lib.btv_last_error()
    rc = lib.btv_tree_verify_attn(C.c_void_p(4096 + 8), fake, fake, fake, 16, 10, 8, 8, 128, 1, f0, fake, None, C.c_size_t(0),
                                  None)
    assert rc == -1 and b"16-byte aligned" in lib.btv_last_error()
    # FP8 KV cache: D = 128 only, positive finite scales, the same shape checks
    one, zero, nan = C.c_float(1.0), C.c_float(0.0), C.c_float(float("nan"))
    rc = lib.btv_tree_verify_attn_fp8kv(fake, fake, fake, one, one, fake, 16, 10, 8, 8, 64, f0, fake, None, C.c_size_t(0), None)
    assert rc == -1 and b"D=64" in lib.btv_last_error()
    for ks, vs in ((zero, one), (one, zero), (nan, one), (one, C.c_float(float("inf"))), (C.c_float(-2.0), one)):
        rc = lib.btv_tree_verify_attn_fp8kv(fake, fake, fake, ks, vs, fake, 16, 10, 8, 8, 128, f0, fake, None,
                                            C.c_size_t(0), None)
        assert rc == -1 and b"scales" in lib.btv_last_error()
    rc = lib.btv_tree_verify_attn_fp8kv(fake, fake, fake, one, one, fake, 1000, 10, 8, 8, 128, f0, fake, None,
                                        C.c_size_t(0), None)
    assert rc == -1 and b"M=1000" in lib.btv_last_error()
    rc = lib.btv_tree_verify_attn_fp8kv(fake, fake, fake, one, one, fake, 16, 10, 8, 8, 128, f0, fake, None,
                                        C.c_size_t(0), None)
    assert rc == -2 and b"workspace" in lib.btv_last_error()
    rc = lib.btv_tree_verify_attn_paged_fp8kv(fake, fake, fake, one, one, 10, fake, 4, fake, fake, fake, 2, 10, 8, 1 << 20,
                                              8, 8, 128, f0, fake, fake, C.c_size_t(1 << 30), None)
    assert rc == -1 and b"max_blocks" in lib.btv_last_error()
    rc = lib.btv_tree_build(fake, 16, 128256, 1000, fake, fake, None, None, fake, None, fake, C.c_size_t(1 << 30), None)
    assert rc == -1
    rc = lib.btv_tree_build(fake, 99, 128256, 64, fake, fake, None, None, fake, None, fake, C.c_size_t(1 << 30), None)
    assert rc == -1
    rc = lib.btv_tree_accept_greedy(fake, 1, fake, fake, 0, 100, fake, fake, fake, None, fake, C.c_size_t(1 << 20), None)
    assert rc == -1
    rc = lib.btv_tree_accept_stochastic(fake, 0, None, 16, fake, fake, 8, 100, fake, fake, fake, fake, fake,
                                        C.c_size_t(1 << 20), None)
    assert rc == -1
    rc = lib.btv_tree_verify_attn_paged(fake, fake, fake, 10, fake, 4, fake, fake, fake, 2, 10, 8, 1 << 20, 8, 8, 128,
                                        f0, fake, fake, C.c_size_t(1 << 30), None)
    assert rc == -1 and b"max_blocks" in lib.btv_last_error()


def test_host_cost_model_matches_the_oracle(oracle):
    """btv_verify_cost is host arithmetic only (App. E), so it is compared here, without a GPU."""
    from paper_2605_29727_amd import binding as btv
    cfgs = [(64, 8192, 32, 4096, 32, 8, 128, 14336, 128256, 2, 2.5e15, 8e12, 1.0, 0.0),
            (128, 32768, 80, 8192, 64, 8, 128, 28672, 128256, 2, 2.5e15, 8e12, 1.3, 2e-4),
            (1, 2, 1, 2, 1, 1, 2, 3, 5, 1, 56.0, 37.0, 2.0, 0.5),
            (0, 100, 2, 16, 2, 1, 8, 32, 50, 4, 1e9, 1e9, 1.0, 0.0)]
    for cfg in cfgs:
        got, ref = btv.btv_verify_cost(*cfg), oracle.verify_cost(*cfg)
        for k in ("flops", "bytes", "roofline_s", "latency_s"):
            assert got[k] == pytest.approx(ref[k], rel=1e-14), (cfg, k)
    with pytest.raises(btv.BtvError):
        btv.btv_verify_cost(1, 1, 1, 0, 1, 1, 1, 1, 1, 1, 1.0, 1.0)          # zero hidden size
    with pytest.raises(btv.BtvError):
        btv.btv_verify_cost(1, 1, 1, 8, 1, 1, 1, 1, 1, 1, 0.0, 1.0)          # zero peak


def test_host_calibration_matches_the_oracle(oracle):
    """The calibration entry points (Sec. 5.2) and the controller's cost curve (Eq. 6) are host arithmetic only."""
    import numpy as np
    from paper_2605_29727_amd import binding as btv, synth
    for seed in range(3):
        pred = 1e-3 * (1.0 + 10.0 * synth.uniform(seed, "calib_pred", (30,)))
        obs = 1.4 * pred + 3e-4 + 1e-4 * synth.uniform(seed, "calib_noise", (30,))
        got, ref = btv.btv_calib_fit_linear(pred, obs), oracle.calib_fit(pred, obs)
        assert got[0] == pytest.approx(ref[0], rel=1e-11) and got[1] == pytest.approx(ref[1], rel=1e-11)
    with pytest.raises(btv.BtvError):
        btv.btv_calib_fit_linear([2.0, 2.0], [1.0, 3.0])
    with pytest.raises(btv.BtvError):
        btv.btv_calib_fit_linear([2.0], [1.0])
    c_lib = c_orc = 1.0
    for i in range(20):
        obs, pred = 2.0 + 0.1 * i, 1.5 + 0.05 * i
        c_lib, c_orc = btv.btv_calib_ema_update(c_lib, 0.2, obs, pred), oracle.calib_ema(c_orc, 0.2, obs, pred)
        assert c_lib == pytest.approx(c_orc, rel=1e-14)
    with pytest.raises(btv.BtvError):
        btv.btv_calib_ema_update(1.0, 1.5, 1.0, 1.0)                           # alpha outside [0, 1]
    with pytest.raises(btv.BtvError):
        btv.btv_calib_ema_update(1.0, 0.5, 1.0, 0.0)                           # zero prediction
    args = (8192, 32, 4096, 32, 8, 128, 14336, 128256, 2, 2.5e15, 8e12, 1.3, 2e-4, 0.9, 1e-3)
    got, ref = np.array(btv.btv_verify_cost_curve(256, *args)), oracle.cost_curve(256, *args)
    assert np.allclose(got, ref, rtol=1e-14, atol=0)
    assert btv.btv_verify_cost_curve(0, *args) == []
    with pytest.raises(btv.BtvError):
        btv.btv_verify_cost_curve(257, *args)
