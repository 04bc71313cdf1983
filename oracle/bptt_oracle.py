"""ctypes front end of the CPU oracle of back-propagation through time (oracle/bptt_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
cpu_baseline leg of bench.py.  The GPU library never imports or calls it, and
this module never imports the GPU package.  It only marshals numpy arrays; all
arithmetic is in the C file (learner step, Alg. 3: the gradient with respect to
the network's parameters).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bptt_oracle.c")
_LIB = os.path.join(_HERE, "libbptt_oracle.so")
_lib = None


def build(force=False):
    """Compile with gcc (-O2, no fast-math, no BLAS)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
                               "-o", _LIB, _SRC, "-lm", "-lpthread"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.bptt_param_count.restype = ctypes.c_long
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def default_threads():
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        return int(env)
    return max(1, min(os.cpu_count() or 1, 16))


def qnet_grad(dims, weights, obs, actions, filled, g, nthreads=None, relu_band=None, inputs_as_bf16=False):
    """grad [param count] f64 of sum(g * q_taken) with respect to the packed weights.

    obs [B,T+1,N,D], actions [B,T,N], filled [B,T], g [B,T,N] = dL/dq_taken.
    relu_band = delta: returns (grad, amb), amb the ambiguity budget of the first layer's entries for
    pre-activations within delta of zero.
    inputs_as_bf16: diagnostic mode for a network held in bf16, whose first layer takes every observation
    entry rounded to bf16 (nearest, ties to even): the gradient of that network, so that the first layer's
    yes/no decisions are taken on the values an implementation in that precision sees.
    """
    N, D, A, H = (int(v) for v in dims)
    weights = _c(weights, np.float32)
    count = int(_load().bptt_param_count(N, D, A, H))
    assert weights.size == count
    obs = _c(obs, np.float32)
    B, T = obs.shape[0], obs.shape[1] - 1
    assert obs.shape == (B, T + 1, N, D)
    if inputs_as_bf16:
        from oracle import marl_oracle
        obs = marl_oracle.round_bf16(obs).reshape(obs.shape)
    actions = _c(actions, np.int32); assert actions.shape == (B, T, N)
    assert actions.min(initial=0) >= 0 and actions.max(initial=0) < A
    filled = _c(filled, np.uint8); assert filled.shape == (B, T)
    g = _c(g, np.float64); assert g.shape == (B, T, N)
    grad = np.zeros(count)
    amb = None if relu_band is None else np.zeros(count)
    _load().bptt_qnet_grad(N, D, A, H, _p(weights), B, T, _p(obs), _p(actions), _p(filled), _p(g), _p(grad),
                           ctypes.c_double(0.0 if relu_band is None else float(relu_band)),
                           None if amb is None else _p(amb), int(nthreads or default_threads()))
    return grad if amb is None else (grad, amb)
