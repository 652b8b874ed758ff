"""Host-only checks of the C boundary: the library loads, exports every symbol
the header declares, validates arguments before touching a device, and its
schedule builder agrees with the oracle's."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import schedule
from paper_2505_03983_amd import binding, probe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header, macro="ASD_API"):
    src = open(os.path.join(ROOT, "include", header)).read()
    return sorted(set(re.findall(macro + r"[^;(]*?\b(asd_\w+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["asd.h", "asd_probe.h", "asd_testing.h"]
    names = _declared("asd.h")
    assert len(names) >= 15 and "asd_init" in names and "asd_sample" in names
    for n in ("asd_draft", "asd_verify", "asd_accept", "asd_destroy"):
        assert n in names
    testing = _declared("asd_testing.h")
    assert "asd_profile_read" in testing and "asd_debug_philox" in testing
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names + testing:
        assert hasattr(lib, n), n
    # and the binding binds them all
    L = binding.lib()
    for n in names + testing:
        assert getattr(L, n).argtypes is not None, n
    # the measurement probe is a library of its own; the sampling library does not carry it
    pnames = _declared("asd_probe.h", "ASD_PROBE_API")
    assert pnames == ["asd_probe_last_error", "asd_probe_mfma_ceiling"]
    plib = ctypes.CDLL(probe.LIB_PATH)
    for n in pnames:
        assert hasattr(plib, n), n
        assert not hasattr(lib, n), n


def test_status_strings():
    assert binding.status_string(0) == "ASD_OK"
    assert binding.status_string(-5) == "ASD_EUNSUPPORTED"


def test_schedule_matches_oracle_tables():
    for K in (1, 2, 100, 1000):
        s = binding.asd_schedule_ddpm_linear(K)
        T = schedule.ddpm_tables(K)
        for k in ("c_x", "c_0", "sigma", "abar"):
            np.testing.assert_allclose(s[k], T[k], rtol=2e-7, atol=1e-30)
        assert np.array_equal(s["tau"], T["tau"])
        assert s["sigma"][K - 1] == 0.0
    with pytest.raises(binding.AsdError):
        binding.asd_schedule_ddpm_linear(0)
    with pytest.raises(binding.AsdError):
        binding.asd_schedule_ddpm_linear(10, 0.5, 0.1)


def test_general_and_cosine_schedules_match_the_oracle():
    for K in (1, 7, 100, 1000):
        ab = binding.asd_abar_cosine(K)
        np.testing.assert_allclose(ab, schedule.cosine_abar(K), rtol=1e-13)
        s = binding.asd_schedule_from_abar(ab)
        T = schedule.tables_from_abar(schedule.cosine_abar(K))
        for k in ("c_x", "c_0", "sigma", "abar"):
            np.testing.assert_allclose(s[k], T[k], rtol=3e-7, atol=1e-30)
        assert np.array_equal(s["tau"], T["tau"])
    for bad in ([0.9, 0.5], [1.0, 0.5, 0.5], [1.0, 0.5, 0.0], [1.0, 1.2]):
        with pytest.raises(binding.AsdError):
            binding.asd_schedule_from_abar(np.array(bad))
    t = np.array([0.01, 0.5, 0.7, 40.0])
    s = binding.asd_schedule_sl_euler(t)
    np.testing.assert_allclose(s["c_0"], np.diff(t), rtol=2e-7)
    np.testing.assert_allclose(s["sigma"], np.sqrt(np.diff(t)), rtol=2e-7)
    assert np.all(s["c_x"] == 1.0) and list(s["tau"]) == [0, 1, 2] and s["sl_time"].dtype == np.float32
    for bad in ([0.0, 1.0], [1.0, 1.0], [2.0, 1.0], [-1.0, 1.0]):
        with pytest.raises(binding.AsdError):
            binding.asd_schedule_sl_euler(np.array(bad))
    with pytest.raises(binding.AsdError):
        binding.asd_abar_cosine(10, -1.0)
    with pytest.raises(binding.AsdError):
        binding.asd_abar_cosine(0)


def _cfg(**over):
    s = binding.asd_schedule_ddpm_linear(10)
    den = dict(kind="gmm", d=4, C=3, var=0.25, means=16, log_w=16, abar=s["abar"], n_tau=11)
    kw = dict(L=4, chains=2)
    for k, v in over.items():
        if k in kw:
            kw[k] = v
        elif k in den or k not in s:
            den[k] = v
        else:
            s[k] = v
    return s, den, kw


@pytest.mark.parametrize("over,status", [
    (dict(L=0), binding.ASD_EINVAL),
    (dict(chains=0), binding.ASD_EINVAL),
    (dict(d=0), binding.ASD_EINVAL),
    (dict(C=0), binding.ASD_EINVAL),
    (dict(means=None), binding.ASD_EINVAL),
    (dict(abar=None), binding.ASD_EINVAL),                        # neither abar nor sl_time
    (dict(sl_time=np.ones(11, np.float32)), binding.ASD_EINVAL),  # both
    (dict(abar=None, sl_time=np.full(11, -1.0, np.float32)), binding.ASD_EINVAL),
    (dict(var=-1.0), binding.ASD_EINVAL),
    (dict(n_tau=5), binding.ASD_EINVAL),                         # tau values out of range
    (dict(sigma=np.full(10, -1.0, np.float32)), binding.ASD_EINVAL),
    (dict(c_x=np.full(10, np.nan, np.float32)), binding.ASD_EINVAL),
    (dict(kind=7), binding.ASD_EINVAL),
])
def test_init_rejects_bad_configs_on_the_host(over, status):
    s, den, kw = _cfg(**over)
    with pytest.raises(binding.AsdError) as ei:
        binding.Ctx(s, den, kw["L"], kw["chains"])
    assert ei.value.status == status


def test_mlp_shape_rules():
    s = binding.asd_schedule_ddpm_linear(10)
    den = dict(kind="mlp", d=12, n_tau=11, width=16, n_blocks=1, temb_dim=8, w_in=16, w_blk=16, w_out=16, temb=16)
    with pytest.raises(binding.AsdError) as ei:
        binding.Ctx(s, den, 4, 2)
    assert ei.value.status == binding.ASD_EUNSUPPORTED           # d not a multiple of 8
    den.update(d=16, linears_per_block=2)
    with pytest.raises(binding.AsdError) as ei:
        binding.Ctx(s, den, 4, 2)
    assert ei.value.status == binding.ASD_EUNSUPPORTED
    den.update(linears_per_block=1, act_terms=3)
    with pytest.raises(binding.AsdError) as ei:
        binding.Ctx(s, den, 4, 2)
    assert ei.value.status == binding.ASD_EINVAL                 # activations: one bf16 term or two
    den.update(act_terms=2, w_out=None)
    with pytest.raises(binding.AsdError) as ei:
        binding.Ctx(s, den, 4, 2)
    assert ei.value.status == binding.ASD_EINVAL
    den.update(w_out=16, predict_eps=True)                       # a noise-predicting network needs abar
    with pytest.raises(binding.AsdError) as ei:
        binding.Ctx(s, den, 4, 2)
    assert ei.value.status == binding.ASD_EINVAL
    den.update(abar=np.full(11, 1.5, np.float32))
    with pytest.raises(binding.AsdError) as ei:
        binding.Ctx(s, den, 4, 2)
    assert ei.value.status == binding.ASD_EINVAL


def test_null_handles():
    L = binding.lib()
    assert L.asd_destroy(None) == binding.ASD_OK
    assert L.asd_init(None, None) == binding.ASD_EINVAL
    assert L.asd_sample(None, None, None, None, None) == binding.ASD_EINVAL
    assert L.asd_last_round_count(None) == -1
    assert "NULL" in binding.last_error()
    for name in ("asd_use_graphs", "asd_use_resident", "asd_use_adaptive_window", "asd_use_split_gemm"):
        assert getattr(L, name)(None, 1) == binding.ASD_EINVAL, name
    assert L.asd_resident_active(None) == 0
    assert L.asd_split_gemm_active(None) == 0
    # argument checks of the ceiling probe come before any device call
    P = probe.lib()
    assert P.asd_probe_mfma_ceiling(1, 1, 100, None) == -1
    t = ctypes.c_double(0.0)
    assert P.asd_probe_mfma_ceiling(1, 1, 0, ctypes.addressof(t)) == -1
    assert P.asd_probe_mfma_ceiling(0, 0, 5001, ctypes.addressof(t)) == -1
    assert P.asd_probe_mfma_ceiling(3, 1, 100, ctypes.addressof(t)) == -1          # dtype is 0, 1 or 2
    assert b"ms_target" in P.asd_probe_last_error()
