"""ctypes front end of the CPU oracle of the mixing network (oracle/mixer_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
cpu_baseline leg of bench.py.  The GPU library never imports or calls it, and
this module never imports the GPU package.  It only marshals numpy arrays; all
arithmetic is in the C file (learner step, Alg. 3: Q_total and y^total).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mixer_oracle.c")
_LIB = os.path.join(_HERE, "libmixer_oracle.so")
_lib = None


def build(force=False):
    """Compile with gcc (-O2, no fast-math, no BLAS)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.mixer_param_count.restype = ctypes.c_long
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def param_count(N, M, S):
    return int(_load().mixer_param_count(int(N), int(M), int(S)))


def forward(dims, w, q, state):
    """Q_total [R] for q [R, N] and state [R, S]; dims = (N, M, S)."""
    N, M, S = (int(v) for v in dims)
    w = _c(w, np.float32); assert w.size == param_count(N, M, S)
    q = _c(q, np.float64); state = _c(state, np.float32)
    R = q.shape[0]
    assert q.shape == (R, N) and state.shape == (R, S)
    out = np.zeros(R)
    _load().mixer_forward(N, M, S, _p(w), ctypes.c_long(R), _p(q), _p(state), _p(out))
    return out


def td(dims, w_online, w_target, state, q_taken, next_max, reward, terminated, filled, gamma):
    """dict(q_total, y_total, td_err [B, T] f64, loss [2] = (sum of squared errors, filled count)).
    w_target=None means target == online."""
    N, M, S = (int(v) for v in dims)
    w_online = _c(w_online, np.float32)
    w_target = w_online if w_target is None else _c(w_target, np.float32)
    assert w_online.size == w_target.size == param_count(N, M, S)
    state = _c(state, np.float32)
    B, T = state.shape[0], state.shape[1] - 1
    assert state.shape == (B, T + 1, S)
    q_taken = _c(q_taken, np.float64); next_max = _c(next_max, np.float64)
    assert q_taken.shape == (B, T, N) and next_max.shape == (B, T, N)
    reward = _c(reward, np.float32); assert reward.shape == (B, T)
    terminated = _c(terminated, np.uint8); assert terminated.shape == (B, T)
    filled = _c(filled, np.uint8); assert filled.shape == (B, T)
    out = dict(q_total=np.zeros((B, T)), y_total=np.zeros((B, T)), td_err=np.zeros((B, T)), loss=np.zeros(2))
    _load().mixer_td(N, M, S, _p(w_online), _p(w_target), B, T, _p(state), _p(q_taken), _p(next_max), _p(reward),
                     _p(terminated), _p(filled), ctypes.c_float(float(np.float32(gamma))),
                     _p(out["q_total"]), _p(out["y_total"]), _p(out["td_err"]), _p(out["loss"]))
    return out


def grad(dims, w, state, q, e, switch_band=None, inputs_as_bf16=False):
    """Backward pass: returns (grad_q [B,T,N], grad_w [param count]) for upstream e [B,T] = dL/dQ_total;
    with switch_band = delta also the ambiguity budget [param count] of the sign / step switches.
    inputs_as_bf16: diagnostic mode for a mixer held in bf16, whose generating layers take every state entry
    rounded to bf16 (nearest, ties to even): the gradient of that mixer, so that the switches are set on the
    values an implementation in that precision sees."""
    N, M, S = (int(v) for v in dims)
    w = _c(w, np.float32)
    assert w.size == param_count(N, M, S)
    state = _c(state, np.float32)
    B, T = state.shape[0], state.shape[1] - 1
    assert state.shape == (B, T + 1, S)
    if inputs_as_bf16:
        from oracle import marl_oracle
        state = marl_oracle.round_bf16(state).reshape(state.shape)
    q = _c(q, np.float64); assert q.shape == (B, T, N)
    e = _c(e, np.float64); assert e.shape == (B, T)
    grad_q = np.zeros((B, T, N))
    grad_w = np.zeros(w.size)
    amb = None if switch_band is None else np.zeros(w.size)
    _load().mixer_grad(N, M, S, _p(w), B, T, _p(state), _p(q), _p(e), _p(grad_q), _p(grad_w),
                       ctypes.c_double(0.0 if switch_band is None else float(switch_band)),
                       None if amb is None else _p(amb))
    return (grad_q, grad_w) if amb is None else (grad_q, grad_w, amb)
