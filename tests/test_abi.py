"""The C-ABI library loads, exports what the header declares, and rejects bad arguments
before touching a device (CPU only: no compute call is made)."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2205_05248_amd import binding, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2205_05248_amd import build
        build.build(verbose=False)
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "marl_qnet.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(marl_[a-z_]+)\s*\(", header))
    assert {"marl_qnet_create", "marl_act_step", "marl_unroll_td", "marl_destroy"} <= declared
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(binding.EXPORTS)
    mixer = open(os.path.join(ROOT, "include", "marl_mixer.h")).read()
    mixer = re.sub(r"/\*.*?\*/", "", mixer, flags=re.S)
    declared = set(re.findall(r"\b(marl_[a-z_]+)\s*\(", mixer))
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(binding.MIXER_EXPORTS)
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["marl_mixer.h", "marl_qnet.h"]


def test_param_count_matches_packing(lib):
    for i in range(5):
        c = wl.config(i)
        N, D, A, H = wl.dims(c)
        assert binding.marl_param_count(N, D, A, H) == wl.param_count(N, D, A, H)
    assert binding.marl_param_count(3, 30, 9, 48) == 0          # hidden must be 64 or 128
    assert binding.marl_param_count(3, 30, 65, 64) == 0         # too many actions


def test_status_strings(lib):
    texts = {lib.marl_strerror(s).decode() for s in range(0, -8, -1)}
    assert len(texts) == 8 and "ok" in texts
    assert lib.marl_strerror(-99).decode() == "unknown status"


def test_create_rejects_bad_descriptions_before_using_a_device(lib):
    w = np.zeros(wl.param_count(3, 30, 9, 64), np.float32)
    mk = lambda **k: binding.Desc(**{**dict(n_agents=3, obs_dim=30, n_actions=9, hidden=64, weight_dtype=0, device=0), **k})
    out = ctypes.c_void_p()
    wp = w.ctypes.data_as(ctypes.c_void_p)
    create = lib.marl_qnet_create
    assert create(None, wp, w.size, ctypes.byref(out)) == -1
    assert create(ctypes.byref(mk()), None, w.size, ctypes.byref(out)) == -1
    assert create(ctypes.byref(mk()), wp, w.size, None) == -1
    for bad in (dict(n_agents=0), dict(obs_dim=-1), dict(n_actions=0), dict(n_actions=65), dict(hidden=100),
                dict(n_agents=65), dict(obs_dim=100000), dict(device=-1)):
        assert create(ctypes.byref(mk(**bad)), wp, w.size, ctypes.byref(out)) == -2, bad
    assert create(ctypes.byref(mk(weight_dtype=2)), wp, w.size, ctypes.byref(out)) == -3
    assert create(ctypes.byref(mk()), wp, w.size - 1, ctypes.byref(out)) == -4
    assert out.value is None


def test_calls_reject_null_handles(lib):
    assert lib.marl_act_step(None, 4, None, None, None, None, None, 0.0, 0, None, None, None, None) == -1
    assert lib.marl_unroll_td(None, None, 1, 1, None, None, None, None, None, None, 0.9, None, None, None, None, None) == -1
    assert lib.marl_act_step_indexed(None, 4, None, 2, None, None, None, None, None, 0.0, 0, None, None, None, None) == -1
    assert lib.marl_unroll_td_indexed(None, None, 8, None, 1, 1, None, None, None, None, None, None, 0.9, None, None, None,
                                      None, None) == -1
    assert lib.marl_unroll_td_double(None, None, 8, None, 1, 1, None, None, None, None, None, None, 0.9, None, None, None,
                                     None, None, None) == -1
    assert lib.marl_qnet_grad_workspace_bytes(None, 1, 1, None) == -1
    assert lib.marl_mixer_grad_workspace_bytes(None, 1, 1, None) == -1
    assert lib.marl_mixer_sgd_step(None, None, None, 0.1, None) == -1
    assert lib.marl_mixer_rmsprop_step(None, None, None, None, 0.1, 0.9, 1e-5, None) == -1
    assert lib.marl_qnet_rmsprop_step(None, None, None, None, 0.1, 0.9, 1e-5, None) == -1
    assert lib.marl_mixer_grad(None, 1, 1, None, None, None, None, 0, None, None, None) == -1
    assert lib.marl_qnet_grad(None, 1, 1, None, None, None, None, None, 0, None, None) == -1
    assert lib.marl_qnet_grad_kept(None, 1, 1, None, None, None, None, None, 0, None, None) == -1
    assert lib.marl_unroll_td_keep(None, None, 1, 1, None, None, None, None, None, None, 0.9, None, None, None, None, None, 0, None) == -1
    assert lib.marl_qnet_reserve_unroll(None, 1, 1) == -1
    assert lib.marl_qnet_get_desc(None, None) == -1
    assert lib.marl_destroy(None) == 0


def test_binding_fails_loudly_without_library(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libmarl_qnet.so")
    with pytest.raises(FileNotFoundError):
        binding.load()


def test_mixer_rejects_bad_arguments_before_using_a_device(lib):
    assert binding.marl_mixer_param_count(3, 32, 48) == wl.mixer_param_count(3, 32, 48)
    assert binding.marl_mixer_param_count(3, 24, 48) == 0           # embed must be 16, 32 or 64
    assert binding.marl_mixer_param_count(3, 32, 513) == 0          # fp32 state limit
    assert binding.marl_mixer_param_count(3, 32, 1024, binding.MARL_DTYPE_BF16) == wl.mixer_param_count(3, 32, 1024)
    assert binding.marl_mixer_param_count(65, 32, 48) == 0
    w = np.zeros(wl.mixer_param_count(3, 32, 48), np.float32)
    wp = w.ctypes.data_as(ctypes.c_void_p)
    out = ctypes.c_void_p()
    mk = lambda **k: binding.MixerDesc(**{**dict(n_agents=3, embed=32, state_dim=48, weight_dtype=0, device=0), **k})
    create = lib.marl_mixer_create
    assert create(None, wp, w.size, ctypes.byref(out)) == -1
    assert create(ctypes.byref(mk()), wp, w.size, None) == -1
    assert create(ctypes.byref(mk(embed=20)), wp, w.size, ctypes.byref(out)) == -2
    assert create(ctypes.byref(mk(state_dim=0)), wp, w.size, ctypes.byref(out)) == -2
    assert create(ctypes.byref(mk(weight_dtype=5)), wp, w.size, ctypes.byref(out)) == -3
    assert create(ctypes.byref(mk()), wp, w.size - 1, ctypes.byref(out)) == -4
    assert lib.marl_mixer_td(None, None, 1, 1, None, None, None, None, None, None, 0.5, None, None, None, None, None) == -1
    assert lib.marl_mixer_set_weights(None, wp, w.size, None) == -1
    lib.marl_mixer_destroy(None)


@pytest.mark.parametrize("ci,dtype", [(0, "fp32"), (1, "fp32"), (3, "bf16"), (4, "bf16"), (4, "fp32")])
def test_refresh_map_reproduces_the_packer_on_the_host(lib, ci, dtype):
    """The device-side weight refresh rebuilds the image through a map found by probing the packer; applied
    on the host to random weights (extreme magnitudes included) it must give the packer's own bytes."""
    cfg = wl.config(ci)
    N, D, A, H = wl.dims(cfg)
    w = wl.make_weights(cfg, 3).copy()
    rng = np.random.default_rng(ci)
    w[rng.integers(0, w.size, 50)] *= np.float32(1e6)
    w[rng.integers(0, w.size, 50)] *= np.float32(1e-20)
    w[rng.integers(0, w.size, 20)] = 0.0
    d = binding.Desc(N, D, A, H, binding.DTYPES[dtype], 0)
    assert lib.marl_qnet_check_refresh_map(ctypes.byref(d), w.ctypes.data_as(ctypes.c_void_p), w.size) == 0
    assert lib.marl_qnet_check_refresh_map(ctypes.byref(d), w.ctypes.data_as(ctypes.c_void_p), w.size - 1) == -4
    assert lib.marl_qnet_check_refresh_map(None, w.ctypes.data_as(ctypes.c_void_p), w.size) == -1
