"""Seeded synthetic inputs with the shapes of the paper's scenarios (Table 2).

The StarCraft scenarios the paper measures on (3m, 8m, 2s3z, 5m_vs_6m) need a
simulator; these generators stand in for them with arrays of the same shapes:
numbers of agents and actions, observation size and time-step limit from
Table 2, two unit types for the heterogeneous scenario from Table 1.  The fifth
workload is a scale-up with no counterpart in the paper.

This module is shared by the oracle's tests and by the GPU tests and bench.  It
holds no arithmetic of the method itself (no network evaluation, no action
selection rule, no TD target): only random draws and array layout.  It imports
neither the oracle nor the GPU binding.
"""
import numpy as np

BASE_SEED = 20220505

# E environments, N agents, D observation size, A actions, H hidden units,
# B episodes per learner batch, T transitions per episode (T+1 observation slots).
CONFIGS = [
    dict(name="cfg0_3m_tiny", E=8, N=3, D=30, A=9, H=64, B=4, T=60, dtype="fp32",
         epsilon=0.05, avail_p=0.7, lengths="uniform_all", hetero=False),
    dict(name="cfg1_8m", E=256, N=8, D=80, A=14, H=64, B=32, T=120, dtype="fp32",
         epsilon=0.05, avail_p=0.7, lengths="upper_half", hetero=False),
    dict(name="cfg2_2s3z_hetero", E=512, N=5, D=96, A=11, H=64, B=64, T=120, dtype="fp32",
         epsilon=0.05, avail_p=0.7, lengths="upper_half", hetero=True),
    dict(name="cfg3_5m_vs_6m_large_actor", E=4096, N=5, D=55, A=12, H=64, B=128, T=70, dtype="fp32",
         epsilon=0.1, avail_p=0.7, lengths="early20", hetero=False),
    dict(name="cfg4_scaleup_bf16", E=2048, N=32, D=300, A=40, H=128, B=64, T=200, dtype="bf16",
         epsilon=0.05, avail_p=0.5, lengths="upper_half", hetero=False),
]
GAMMA = 0.99


def config(i):
    c = dict(CONFIGS[i])
    c["index"] = i
    c["seed"] = BASE_SEED + i
    c["gamma"] = GAMMA
    return c


def dims(cfg):
    return (cfg["N"], cfg["D"], cfg["A"], cfg["H"])


def param_count(N, D, A, H):
    return (D + N) * H + H + 2 * 3 * H * H + 2 * 3 * H + A * H + A


def weight_slices(N, D, A, H):
    """Offsets of each tensor in the packed weight vector, in packing order."""
    shapes = [("W1", (H, D + N)), ("b1", (H,)), ("W_ih", (3 * H, H)), ("W_hh", (3 * H, H)),
              ("b_ih", (3 * H,)), ("b_hh", (3 * H,)), ("W2", (A, H)), ("b2", (A,))]
    out, off = {}, 0
    for name, shp in shapes:
        n = int(np.prod(shp))
        out[name] = (off, off + n, shp)
        off += n
    return out


def unpack_weights(dims_, w):
    sl = weight_slices(*dims_)
    return {k: np.asarray(w[a:b]).reshape(shp) for k, (a, b, shp) in sl.items()}


def pack_weights(dims_, parts):
    sl = weight_slices(*dims_)
    w = np.zeros(param_count(*dims_), np.float32)
    for k, (a, b, shp) in sl.items():
        w[a:b] = np.asarray(parts[k], np.float32).reshape(-1)
    return w


def make_weights(cfg, stream=0):
    """Xavier-uniform matrices (bound sqrt(6/(cols+rows))), biases U(-0.05, 0.05)."""
    rng = np.random.default_rng([cfg["seed"], 1000 + stream])
    parts = {}
    for name, (_, _, shp) in weight_slices(*dims(cfg)).items():
        if len(shp) == 2:
            bound = np.sqrt(6.0 / (shp[0] + shp[1]))
            parts[name] = rng.uniform(-bound, bound, shp)
        else:
            parts[name] = rng.uniform(-0.05, 0.05, shp)
    return pack_weights(dims(cfg), parts)


def _obs(rng, lead, cfg):
    N, D = cfg["N"], cfg["D"]
    obs = rng.random(lead + (N, D), dtype=np.float32)
    obs[rng.random(obs.shape, dtype=np.float32) < 0.3] = 0.0
    if cfg["hetero"]:
        type_a = np.arange(N) < 2                      # two units of the first type, rest of the second
        obs[..., D - 2] = type_a.astype(np.float32)
        obs[..., D - 1] = (~type_a).astype(np.float32)
    return obs


def _avail(rng, lead, cfg):
    N, A = cfg["N"], cfg["A"]
    p = np.full((N, A), cfg["avail_p"], np.float32)
    if cfg["hetero"]:
        p[:2, 6:A] = 0.5
    avail = (rng.random(lead + (N, A), dtype=np.float32) < p).astype(np.uint8)
    avail[..., 0] = 1
    return avail


def make_act_inputs(cfg, E=None, stream=0):
    """One decision step for E environments: obs, avail, h_in, reset, step_t."""
    E = cfg["E"] if E is None else E
    rng = np.random.default_rng([cfg["seed"], 2000 + stream])
    N, H = cfg["N"], cfg["H"]
    return dict(
        obs=_obs(rng, (E,), cfg),
        avail=_avail(rng, (E,), cfg),
        h_in=rng.uniform(-1.0, 1.0, (E, N, H)).astype(np.float32),
        reset=(rng.random(E) < 0.25).astype(np.uint8),
        step_t=rng.integers(0, cfg["T"] + 1, E).astype(np.int32),
        epsilon=float(cfg["epsilon"]),
        seed=int(cfg["seed"]) * 1000003 + stream,
    )


def _lengths(rng, cfg, B):
    T = cfg["T"]
    kind = cfg["lengths"]
    if kind == "uniform_all":
        L = rng.integers(1, T + 1, B)
        term = np.ones(B, bool)
    elif kind == "upper_half":
        L = rng.integers(T // 2, T + 1, B)
        term = L < T
    elif kind == "early20":
        early = rng.random(B) < 0.2
        L = np.where(early, rng.integers(1, T, B), T)
        term = early
    else:
        raise ValueError(kind)
    return L.astype(np.int64), term


def make_unroll_inputs(cfg, B=None, T=None, stream=0):
    """A batch of B whole trajectories of up to T transitions, padded to T."""
    cfg = dict(cfg)
    if T is not None:
        cfg["T"] = T
    B = cfg["B"] if B is None else B
    T, N, A = cfg["T"], cfg["N"], cfg["A"]
    rng = np.random.default_rng([cfg["seed"], 3000 + stream])
    L, term = _lengths(rng, cfg, B)
    obs = _obs(rng, (B, T + 1), cfg)
    avail = _avail(rng, (B, T + 1), cfg)
    slot = np.arange(T + 1)[None, :]
    pad = slot > L[:, None]                             # slots after the last observation
    obs[pad] = 0.0
    avail[pad] = 0
    avail[..., 0] = 1
    score = rng.random((B, T, N, A), dtype=np.float32)
    score[avail[:, :T] == 0] = -1.0
    actions = score.argmax(-1).astype(np.int32)         # uniform over the available actions
    step = np.arange(T)[None, :]
    filled = (step < L[:, None]).astype(np.uint8)
    terminated = ((step == (L[:, None] - 1)) & term[:, None]).astype(np.uint8)
    reward = rng.standard_normal((B, T)).astype(np.float32) * filled
    return dict(obs=obs, avail=avail, actions=actions, reward=reward, terminated=terminated,
                filled=filled, gamma=float(cfg["gamma"]), lengths=L)


# ------------------------------------------------------------------ mixing network (learner, Alg. 3)
# Global state sizes of Table 2 for the four scenarios; the scale-up workload has no counterpart.
STATE_DIMS = [48, 168, 120, 98, 512]
MIX_EMBED = 32


def mixer_dims(cfg):
    """(N agents, M hidden units of the mixer, S state size)."""
    return (cfg["N"], MIX_EMBED, STATE_DIMS[cfg["index"]] if "S" not in cfg else cfg["S"])


def mixer_param_count(N, M, S):
    return (N * M + 3 * M) * (S + 1) + M + 1


def mixer_slices(N, M, S):
    """Offsets of each tensor in the packed mixer parameter vector, in packing order."""
    shapes = [("Hw1", (N * M, S)), ("hb1", (N * M,)), ("Hb1", (M, S)), ("hbb1", (M,)), ("Hw2", (M, S)),
              ("hb2", (M,)), ("V1", (M, S)), ("c1", (M,)), ("v2", (M,)), ("c2", (1,))]
    out, off = {}, 0
    for name, shp in shapes:
        n = int(np.prod(shp))
        out[name] = (off, off + n, shp)
        off += n
    return out


def pack_mixer(dims_, parts):
    sl = mixer_slices(*dims_)
    w = np.zeros(mixer_param_count(*dims_), np.float32)
    for k, (a, b, shp) in sl.items():
        w[a:b] = np.asarray(parts[k], np.float32).reshape(-1)
    return w


def make_mixer_weights(cfg, stream=0):
    """Matrices uniform with the fan-in bound 1/sqrt(S) (1/sqrt(M) for v2), biases U(-0.05, 0.05)."""
    dims_ = mixer_dims(cfg)
    rng = np.random.default_rng([cfg["seed"], 4000 + stream])
    parts = {}
    for name, (_, _, shp) in mixer_slices(*dims_).items():
        if len(shp) == 2:
            bound = 1.0 / np.sqrt(shp[1])
            parts[name] = rng.uniform(-bound, bound, shp)
        elif name == "v2":
            parts[name] = rng.uniform(-1.0, 1.0, shp) / np.sqrt(shp[0])
        else:
            parts[name] = rng.uniform(-0.05, 0.05, shp)
    return pack_mixer(dims_, parts)


def make_mixer_inputs(cfg, B=None, T=None, stream=0):
    """The learner batch as the mixer sees it: global states of all T+1 slots, the agents' chosen
    values and bootstrap values per transition (values of the size the Q-network emits), and the
    batch's reward / terminated / filled arrays (same episode-length recipe as the unroll)."""
    cfg = dict(cfg)
    if T is not None:
        cfg["T"] = T
    B = cfg["B"] if B is None else B
    T, N = cfg["T"], cfg["N"]
    S = mixer_dims(cfg)[2]
    rng = np.random.default_rng([cfg["seed"], 5000 + stream])
    L, term = _lengths(rng, cfg, B)
    state = rng.random((B, T + 1, S), dtype=np.float32)
    state[rng.random(state.shape, dtype=np.float32) < 0.3] = 0.0
    state[np.arange(T + 1)[None, :] > L[:, None]] = 0.0
    q_taken = (rng.standard_normal((B, T, N)) * 0.5).astype(np.float32)
    next_max = (rng.standard_normal((B, T, N)) * 0.5 + 0.3).astype(np.float32)
    step = np.arange(T)[None, :]
    filled = (step < L[:, None]).astype(np.uint8)
    terminated = ((step == (L[:, None] - 1)) & term[:, None]).astype(np.uint8)
    reward = rng.standard_normal((B, T)).astype(np.float32) * filled
    return dict(state=state, q_taken=q_taken, next_max=next_max, reward=reward, terminated=terminated,
                filled=filled, gamma=float(cfg["gamma"]))
