"""ctypes front end of the CPU oracle (oracle/marl_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
cpu_baseline leg of bench.py.  The GPU library never imports or calls it, and
this module never imports the GPU package.  It only marshals numpy arrays; all
arithmetic is in the C file, which follows the definitions cited there
(worker decision step, Alg. 2; learner TD step, Alg. 3; hidden-state layout,
Fig. 3).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "marl_oracle.c")
_LIB = os.path.join(_HERE, "libmarl_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (-O2, no fast-math, no BLAS)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
             "-o", _LIB, _SRC, "-lm", "-lpthread"])
    return _LIB


def default_threads():
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        return int(env)
    return max(1, min(os.cpu_count() or 1, 16))


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_param_count.restype = ctypes.c_long
        _lib.oracle_S.restype = ctypes.c_uint64
        _lib.oracle_S.argtypes = [ctypes.c_uint64]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def param_count(N, D, A, H):
    return int(_load().oracle_param_count(int(N), int(D), int(A), int(H)))


def S(v):
    """One SplitMix64 output for state v (v + golden gamma, then the mixer)."""
    return int(_load().oracle_S(ctypes.c_uint64(v & 0xFFFFFFFFFFFFFFFF)))


def rng_draw(seed, e, n, t):
    r1, r2 = ctypes.c_uint64(), ctypes.c_uint64()
    _load().oracle_rng_draw(ctypes.c_uint64(seed), ctypes.c_uint32(e), ctypes.c_uint32(n),
                            ctypes.c_uint32(t), ctypes.byref(r1), ctypes.byref(r2))
    return r1.value, r2.value


def round_bf16(w):
    w = _c(w, np.float32)
    out = np.empty_like(w)
    _load().oracle_round_bf16(_p(w), _p(out), ctypes.c_long(w.size))
    return out


def act_step(dims, weights, obs, avail, h_in, reset, step_t, epsilon, seed, nthreads=None):
    """dims = (N, D, A, H).  Returns dict(h_out f64, action i32, q f64, greedy i32, explored u8)."""
    N, D, A, H = (int(v) for v in dims)
    weights = _c(weights, np.float32)
    assert weights.size == param_count(N, D, A, H)
    obs = _c(obs, np.float32)
    E = obs.shape[0]
    assert obs.shape == (E, N, D)
    avail = _c(avail, np.uint8); assert avail.shape == (E, N, A)
    h_in = _c(h_in, np.float64); assert h_in.shape == (E, N, H)
    reset = None if reset is None else _c(reset, np.uint8)
    step_t = _c(step_t, np.int32); assert step_t.shape == (E,)
    out = dict(h_out=np.empty((E, N, H), np.float64), action=np.empty((E, N), np.int32),
               q=np.empty((E, N, A), np.float64), greedy=np.empty((E, N), np.int32),
               explored=np.empty((E, N), np.uint8))
    _load().oracle_act_step(
        N, D, A, H, _p(weights), E, _p(obs), _p(avail), _p(h_in), _p(reset), _p(step_t),
        ctypes.c_float(float(np.float32(epsilon))), ctypes.c_uint64(int(seed)),
        _p(out["h_out"]), _p(out["action"]), _p(out["q"]), _p(out["greedy"]), _p(out["explored"]),
        int(nthreads or default_threads()))
    return out


def unroll_td(dims, w_online, w_target, obs, avail, actions, reward, terminated, filled, gamma,
              want_q_all=True, rows=None, nthreads=None):
    """Returns dict(q_taken, next_max, td_target [B,T,N] f64, q_all [B,T+1,N,A] f64 or None).

    w_target=None means target == online.  rows: optional int array of b*N+n
    pairs to evaluate; other output entries are NaN.
    """
    N, D, A, H = (int(v) for v in dims)
    w_online = _c(w_online, np.float32)
    w_target = w_online if w_target is None else _c(w_target, np.float32)
    assert w_online.size == w_target.size == param_count(N, D, A, H)
    obs = _c(obs, np.float32)
    B, S1 = obs.shape[0], obs.shape[1]
    T = S1 - 1
    assert obs.shape == (B, T + 1, N, D)
    avail = _c(avail, np.uint8); assert avail.shape == (B, T + 1, N, A)
    actions = _c(actions, np.int32); assert actions.shape == (B, T, N)
    reward = _c(reward, np.float32); assert reward.shape == (B, T)
    terminated = _c(terminated, np.uint8); assert terminated.shape == (B, T)
    filled = _c(filled, np.uint8); assert filled.shape == (B, T)
    fill = np.nan if rows is not None else 0.0
    out = dict(q_taken=np.full((B, T, N), fill), next_max=np.full((B, T, N), fill),
               td_target=np.full((B, T, N), fill),
               q_all=np.full((B, T + 1, N, A), fill) if want_q_all else None)
    rows_a = None if rows is None else _c(rows, np.int32)
    _load().oracle_unroll_td(
        N, D, A, H, _p(w_online), _p(w_target), B, T, _p(obs), _p(avail), _p(actions), _p(reward),
        _p(terminated), _p(filled), ctypes.c_float(float(np.float32(gamma))),
        _p(out["q_taken"]), _p(out["next_max"]), _p(out["td_target"]), _p(out["q_all"]),
        _p(rows_a), 0 if rows_a is None else int(rows_a.size), int(nthreads or default_threads()))
    return out


def unroll_td_double(dims, w_online, w_target, obs, avail, actions, reward, terminated, filled, gamma,
                     want_q_all=True, nthreads=None):
    """The double-estimator TD target: the online network picks the next action, the target values it.

    Returns dict(q_taken, next_max, td_target [B,T,N] f64, next_action [B,T,N] i32,
    q_all [B,T+1,N,A] f64 or None (online network)).
    """
    N, D, A, H = (int(v) for v in dims)
    w_online = _c(w_online, np.float32)
    w_target = w_online if w_target is None else _c(w_target, np.float32)
    assert w_online.size == w_target.size == param_count(N, D, A, H)
    obs = _c(obs, np.float32)
    B, T = obs.shape[0], obs.shape[1] - 1
    assert obs.shape == (B, T + 1, N, D)
    avail = _c(avail, np.uint8); assert avail.shape == (B, T + 1, N, A)
    actions = _c(actions, np.int32); assert actions.shape == (B, T, N)
    reward = _c(reward, np.float32); assert reward.shape == (B, T)
    terminated = _c(terminated, np.uint8); assert terminated.shape == (B, T)
    filled = _c(filled, np.uint8); assert filled.shape == (B, T)
    out = dict(q_taken=np.zeros((B, T, N)), next_max=np.zeros((B, T, N)), td_target=np.zeros((B, T, N)),
               next_action=np.zeros((B, T, N), np.int32),
               q_all=np.zeros((B, T + 1, N, A)) if want_q_all else None)
    _load().oracle_unroll_td_double(
        N, D, A, H, _p(w_online), _p(w_target), B, T, _p(obs), _p(avail), _p(actions), _p(reward),
        _p(terminated), _p(filled), ctypes.c_float(float(np.float32(gamma))),
        _p(out["q_taken"]), _p(out["next_max"]), _p(out["td_target"]), _p(out["q_all"]),
        _p(out["next_action"]), int(nthreads or default_threads()))
    return out
