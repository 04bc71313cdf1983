"""ctypes binding of libmarl_qnet.so (include/marl_qnet.h and include/marl_mixer.h), same
entry-point names.

Argument marshalling only: tensors are checked for dtype, shape, contiguity and
device, and their addresses handed to the C ABI together with torch's current
HIP stream.  Every step of the network, the action rule, the TD targets and the
mixing network run in the library's kernels.  There is no CPU fallback: if the library is not
built, or a call fails, an exception is raised.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmarl_qnet.so")

MARL_DTYPE_F32 = 0
MARL_DTYPE_BF16 = 1
DTYPES = {"fp32": MARL_DTYPE_F32, "bf16": MARL_DTYPE_BF16}

EXPORTS = ["marl_param_count", "marl_qnet_create", "marl_qnet_get_desc", "marl_act_step", "marl_act_step_indexed", "marl_unroll_td_indexed",
           "marl_unroll_td_double", "marl_qnet_grad_workspace_bytes", "marl_qnet_grad", "marl_qnet_grad_kept", "marl_unroll_td_keep", "marl_qnet_sgd_step", "marl_qnet_rmsprop_step", "marl_qnet_check_refresh_map",
           "marl_unroll_td", "marl_unroll_td_static", "marl_probe_stream", "marl_probe_mfma", "marl_qnet_reserve_unroll", "marl_destroy", "marl_strerror",
           "marl_last_device_error", "marl_qnet_set_timing", "marl_qnet_timing_read",
           "marl_qnet_set_kernels", "marl_qnet_kernels_in_use", "marl_qnet_set_weights"]
# include/marl_mixer.h
MIXER_EXPORTS = ["marl_mixer_param_count", "marl_mixer_create", "marl_mixer_destroy", "marl_mixer_td",
                 "marl_mixer_set_weights", "marl_mixer_grad_workspace_bytes", "marl_mixer_grad", "marl_mixer_sgd_step", "marl_mixer_rmsprop_step"]


class MarlError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"marl_qnet error {status}: {text}")
        self.status = status


class MixerDesc(ctypes.Structure):
    _fields_ = [("n_agents", ctypes.c_int32), ("embed", ctypes.c_int32), ("state_dim", ctypes.c_int32),
                ("weight_dtype", ctypes.c_int32), ("device", ctypes.c_int32)]


class Desc(ctypes.Structure):
    _fields_ = [("n_agents", ctypes.c_int32), ("obs_dim", ctypes.c_int32), ("n_actions", ctypes.c_int32),
                ("hidden", ctypes.c_int32), ("weight_dtype", ctypes.c_int32), ("device", ctypes.c_int32)]


_lib = None


def load():
    """Load the built library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2205_05248_amd.build` "
                "(there is no CPU fallback)")
        # The library must share one HIP runtime with torch, whose tensors and streams it is
        # handed: import torch first so that its libamdhip64 is the copy already in the process.
        import torch  # noqa: F401
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, f32, u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_uint64
        lib.marl_param_count.restype = ctypes.c_size_t
        lib.marl_param_count.argtypes = [ctypes.POINTER(Desc)]
        lib.marl_qnet_set_weights.restype = ctypes.c_int
        lib.marl_qnet_set_weights.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.marl_qnet_create.restype = ctypes.c_int
        lib.marl_qnet_create.argtypes = [ctypes.POINTER(Desc), vp, ctypes.c_size_t, ctypes.POINTER(vp)]
        lib.marl_qnet_get_desc.restype = ctypes.c_int
        lib.marl_qnet_get_desc.argtypes = [vp, ctypes.POINTER(Desc)]
        lib.marl_act_step.restype = ctypes.c_int
        lib.marl_act_step.argtypes = [vp, i32, vp, vp, vp, vp, vp, f32, u64, vp, vp, vp, vp]
        lib.marl_act_step_indexed.restype = ctypes.c_int
        lib.marl_act_step_indexed.argtypes = [vp, i32, vp, i32, vp, vp, vp, vp, vp, f32, u64, vp, vp, vp, vp]
        lib.marl_unroll_td.restype = ctypes.c_int
        lib.marl_unroll_td.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp]
        lib.marl_probe_stream.restype = ctypes.c_int
        lib.marl_probe_stream.argtypes = [vp, vp, ctypes.c_size_t, vp, vp]
        lib.marl_probe_mfma.restype = ctypes.c_int
        lib.marl_probe_mfma.argtypes = [i32, vp, ctypes.POINTER(ctypes.c_double), vp]
        lib.marl_unroll_td_static.restype = ctypes.c_int
        lib.marl_unroll_td_static.argtypes = lib.marl_unroll_td.argtypes
        lib.marl_unroll_td_indexed.restype = ctypes.c_int
        lib.marl_unroll_td_indexed.argtypes = [vp, vp, i32, vp, i32, i32, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp]
        lib.marl_unroll_td_double.restype = ctypes.c_int
        lib.marl_unroll_td_double.argtypes = [vp, vp, i32, vp, i32, i32, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp, vp]
        lib.marl_qnet_grad_workspace_bytes.restype = ctypes.c_int
        lib.marl_qnet_grad_workspace_bytes.argtypes = [vp, i32, i32, ctypes.POINTER(ctypes.c_size_t)]
        lib.marl_qnet_grad.restype = ctypes.c_int
        lib.marl_qnet_grad.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, ctypes.c_size_t, vp, vp]
        lib.marl_qnet_grad_kept.restype = ctypes.c_int
        lib.marl_qnet_grad_kept.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, ctypes.c_size_t, vp, vp]
        lib.marl_unroll_td_keep.restype = ctypes.c_int
        lib.marl_unroll_td_keep.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.marl_qnet_check_refresh_map.restype = ctypes.c_int
        lib.marl_qnet_check_refresh_map.argtypes = [ctypes.POINTER(Desc), vp, ctypes.c_size_t]
        lib.marl_qnet_rmsprop_step.restype = ctypes.c_int
        lib.marl_qnet_rmsprop_step.argtypes = [vp, vp, vp, vp, f32, f32, f32, vp]
        lib.marl_mixer_rmsprop_step.restype = ctypes.c_int
        lib.marl_mixer_rmsprop_step.argtypes = [vp, vp, vp, vp, f32, f32, f32, vp]
        lib.marl_qnet_sgd_step.restype = ctypes.c_int
        lib.marl_qnet_sgd_step.argtypes = [vp, vp, vp, f32, vp]
        lib.marl_qnet_reserve_unroll.restype = ctypes.c_int
        lib.marl_qnet_reserve_unroll.argtypes = [vp, i32, i32]
        lib.marl_qnet_kernels_in_use.restype = ctypes.c_int
        lib.marl_qnet_kernels_in_use.argtypes = [vp, i32]
        lib.marl_qnet_set_kernels.restype = ctypes.c_int
        lib.marl_qnet_set_kernels.argtypes = [vp, i32]
        lib.marl_qnet_set_timing.restype = ctypes.c_int
        lib.marl_qnet_set_timing.argtypes = [vp, i32]
        lib.marl_qnet_timing_read.restype = ctypes.c_int
        lib.marl_qnet_timing_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32),
                                              ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
        lib.marl_destroy.restype = ctypes.c_int
        lib.marl_destroy.argtypes = [vp]
        lib.marl_strerror.restype = ctypes.c_char_p
        lib.marl_strerror.argtypes = [ctypes.c_int]
        lib.marl_last_device_error.restype = ctypes.c_char_p
        lib.marl_last_device_error.argtypes = []
        lib.marl_mixer_param_count.restype = ctypes.c_size_t
        lib.marl_mixer_param_count.argtypes = [ctypes.POINTER(MixerDesc)]
        lib.marl_mixer_create.restype = ctypes.c_int
        lib.marl_mixer_create.argtypes = [ctypes.POINTER(MixerDesc), vp, ctypes.c_size_t, ctypes.POINTER(vp)]
        lib.marl_mixer_set_weights.restype = ctypes.c_int
        lib.marl_mixer_set_weights.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.marl_mixer_destroy.restype = None
        lib.marl_mixer_destroy.argtypes = [vp]
        lib.marl_mixer_grad_workspace_bytes.restype = ctypes.c_int
        lib.marl_mixer_grad_workspace_bytes.argtypes = [vp, i32, i32, ctypes.POINTER(ctypes.c_size_t)]
        lib.marl_mixer_grad.restype = ctypes.c_int
        lib.marl_mixer_grad.argtypes = [vp, i32, i32, vp, vp, vp, vp, ctypes.c_size_t, vp, vp, vp]
        lib.marl_mixer_sgd_step.restype = ctypes.c_int
        lib.marl_mixer_sgd_step.argtypes = [vp, vp, vp, f32, vp]
        lib.marl_mixer_td.restype = ctypes.c_int
        lib.marl_mixer_td.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp]
        _lib = lib
    return _lib


def check(status, detail=False):
    """detail: the call clears the thread's message on entry, so whatever is there afterwards is its own."""
    if status != 0:
        lib = load()
        text = lib.marl_strerror(status).decode()
        message = lib.marl_last_device_error().decode()
        if status == -6 or (detail and message):
            text += " (" + message + ")"
        raise MarlError(status, text)


def marl_param_count(n_agents, obs_dim, n_actions, hidden, weight_dtype=MARL_DTYPE_F32, device=0):
    d = Desc(n_agents, obs_dim, n_actions, hidden, weight_dtype, device)
    return int(load().marl_param_count(ctypes.byref(d)))


def marl_qnet_create(n_agents, obs_dim, n_actions, hidden, weight_dtype, device, host_weights):
    """Returns an opaque handle (int).  host_weights: packed fp32 numpy array."""
    w = np.ascontiguousarray(host_weights, dtype=np.float32)
    d = Desc(n_agents, obs_dim, n_actions, hidden, weight_dtype, device)
    out = ctypes.c_void_p()
    check(load().marl_qnet_create(ctypes.byref(d), w.ctypes.data_as(ctypes.c_void_p), w.size, ctypes.byref(out)))
    return out.value


def marl_qnet_set_weights(handle, host_weights):
    """Stream-ordered in-place weight refresh on torch's current stream."""
    w = np.ascontiguousarray(host_weights, dtype=np.float32)
    check(load().marl_qnet_set_weights(ctypes.c_void_p(handle), w.ctypes.data_as(ctypes.c_void_p), w.size, _stream()))


def marl_destroy(handle):
    check(load().marl_destroy(ctypes.c_void_p(handle)))


def _dev(t, dtype, shape, name, optional=False):
    import torch
    if t is None:
        if optional:
            return None
        raise ValueError(f"{name} is required")
    want = {"f32": torch.float32, "u8": torch.uint8, "i32": torch.int32}[dtype]
    if t.dtype != want or tuple(t.shape) != tuple(shape) or not t.is_contiguous() or not t.is_cuda:
        raise ValueError(f"{name}: expected contiguous device {dtype} tensor of shape {tuple(shape)}, "
                         f"got {t.dtype} {tuple(t.shape)} on {t.device}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def marl_act_step(handle, dims, obs, avail, h_in, reset, step_t, epsilon, seed, h_out, action, q_out=None):
    """dims = (N, D, A, H) of the handle; tensors live on the handle's device."""
    N, D, A, H = dims
    E = obs.shape[0]
    check(load().marl_act_step(
        ctypes.c_void_p(handle), E,
        _dev(obs, "f32", (E, N, D), "obs"), _dev(avail, "u8", (E, N, A), "avail"),
        _dev(h_in, "f32", (E, N, H), "h_in"), _dev(reset, "u8", (E,), "reset", optional=True),
        _dev(step_t, "i32", (E,), "step_t"), float(epsilon), int(seed) & 0xFFFFFFFFFFFFFFFF,
        _dev(h_out, "f32", (E, N, H), "h_out"), _dev(action, "i32", (E, N), "action"),
        _dev(q_out, "f32", (E, N, A), "q_out", optional=True), _stream()))


def marl_act_step_indexed(handle, dims, env_index, obs, avail, h_in, reset, step_t, epsilon, seed, h_out, action,
                          q_out=None):
    """Serves only the environments listed in env_index (device int32 vector); arrays as in marl_act_step."""
    N, D, A, H = dims
    E = obs.shape[0]
    n_listed = int(env_index.shape[0])
    check(load().marl_act_step_indexed(
        ctypes.c_void_p(handle), E, _dev(env_index, "i32", (n_listed,), "env_index"), n_listed,
        _dev(obs, "f32", (E, N, D), "obs"), _dev(avail, "u8", (E, N, A), "avail"),
        _dev(h_in, "f32", (E, N, H), "h_in"), _dev(reset, "u8", (E,), "reset", optional=True),
        _dev(step_t, "i32", (E,), "step_t"), float(epsilon), int(seed) & 0xFFFFFFFFFFFFFFFF,
        _dev(h_out, "f32", (E, N, H), "h_out"), _dev(action, "i32", (E, N), "action"),
        _dev(q_out, "f32", (E, N, A), "q_out", optional=True), _stream()))


def marl_probe_stream(src, dst, sink):
    """One streaming pass over src (a read, or a copy into dst when dst is given)."""
    nbytes = src.numel() * src.element_size()
    check(load().marl_probe_stream(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()) if dst is not None else None,
                                   nbytes, ctypes.c_void_p(sink.data_ptr()), _stream()))
    return nbytes * (2 if dst is not None else 1)


def marl_probe_mfma(iters, sink):
    """One launch of dependency-free bf16 matrix instructions; returns its floating-point operations."""
    flops = ctypes.c_double(0.0)
    check(load().marl_probe_mfma(int(iters), ctypes.c_void_p(sink.data_ptr()), ctypes.byref(flops), _stream()))
    return flops.value


STATIC_SCRATCH_BYTES = 64 << 20          # MARL_STATIC_SCRATCH_BYTES


def marl_unroll_td(online, target, dims, obs, avail, actions, reward, terminated, filled, gamma,
                   q_taken, next_max, td_target, q_all=None, static=False):
    """static: marl_unroll_td_static, the variant that allocates nothing (same arguments)."""
    N, D, A, H = dims
    B, T = obs.shape[0], obs.shape[1] - 1
    entry = load().marl_unroll_td_static if static else load().marl_unroll_td
    check(entry(
        ctypes.c_void_p(online), ctypes.c_void_p(target), B, T,
        _dev(obs, "f32", (B, T + 1, N, D), "obs"), _dev(avail, "u8", (B, T + 1, N, A), "avail"),
        _dev(actions, "i32", (B, T, N), "actions"), _dev(reward, "f32", (B, T), "reward"),
        _dev(terminated, "u8", (B, T), "terminated"), _dev(filled, "u8", (B, T), "filled"), float(gamma),
        _dev(q_taken, "f32", (B, T, N), "q_taken"), _dev(next_max, "f32", (B, T, N), "next_max"),
        _dev(td_target, "f32", (B, T, N), "td_target"), _dev(q_all, "f32", (B, T + 1, N, A), "q_all", optional=True),
        _stream()), detail=static)


def marl_qnet_reserve_unroll(handle, B, T):
    check(load().marl_qnet_reserve_unroll(ctypes.c_void_p(handle), B, T))


KERNELS_AUTO, KERNELS_TILE32, KERNELS_FUSED16, KERNELS_STREAM16 = 0, 1, 2, 3


def marl_qnet_set_kernels(handle, path):
    check(load().marl_qnet_set_kernels(ctypes.c_void_p(handle), int(path)))


ENTRY_ACT_STEP, ENTRY_UNROLL_TD = 0, 1


def marl_qnet_kernels_in_use(handle, entry):
    rc = load().marl_qnet_kernels_in_use(ctypes.c_void_p(handle), int(entry))
    if rc < 0:
        check(rc)
    return rc


def marl_qnet_set_timing(handle, enable):
    check(load().marl_qnet_set_timing(ctypes.c_void_p(handle), int(bool(enable))))


def marl_qnet_timing_read(handle):
    """Mean kernel durations (ms) over the calls recorded since timing was enabled / last read."""
    act, n_act, n_unroll = ctypes.c_float(), ctypes.c_int32(), ctypes.c_int32()
    unroll = (ctypes.c_float * 2)()
    check(load().marl_qnet_timing_read(ctypes.c_void_p(handle), ctypes.byref(act), ctypes.byref(n_act), unroll,
                                       ctypes.byref(n_unroll)))
    return dict(act_ms=act.value, act_calls=n_act.value, input_proj_ms=unroll[0], recurrent_ms=unroll[1],
                unroll_calls=n_unroll.value)


def marl_unroll_td_indexed(online, target, dims, episode_index, obs, avail, actions, reward, terminated, filled, gamma,
                           q_taken, next_max, td_target, q_all=None):
    """Inputs are pool arrays (leading dimension = pool size); episode_index (device int32 [B]) picks the batch."""
    N, D, A, H = dims
    pool, T = obs.shape[0], obs.shape[1] - 1
    B = int(episode_index.shape[0])
    check(load().marl_unroll_td_indexed(
        ctypes.c_void_p(online), ctypes.c_void_p(target), pool, _dev(episode_index, "i32", (B,), "episode_index"), B, T,
        _dev(obs, "f32", (pool, T + 1, N, D), "obs"), _dev(avail, "u8", (pool, T + 1, N, A), "avail"),
        _dev(actions, "i32", (pool, T, N), "actions"), _dev(reward, "f32", (pool, T), "reward"),
        _dev(terminated, "u8", (pool, T), "terminated"), _dev(filled, "u8", (pool, T), "filled"), float(gamma),
        _dev(q_taken, "f32", (B, T, N), "q_taken"), _dev(next_max, "f32", (B, T, N), "next_max"),
        _dev(td_target, "f32", (B, T, N), "td_target"), _dev(q_all, "f32", (B, T + 1, N, A), "q_all", optional=True),
        _stream()))


def marl_unroll_td_double(online, target, dims, obs, avail, actions, reward, terminated, filled, gamma,
                          q_taken, next_max, td_target, next_action, q_all=None, episode_index=None):
    """Double-estimator target; with episode_index the inputs are pool arrays as in marl_unroll_td_indexed."""
    N, D, A, H = dims
    pool, T = obs.shape[0], obs.shape[1] - 1
    B = pool if episode_index is None else int(episode_index.shape[0])
    check(load().marl_unroll_td_double(
        ctypes.c_void_p(online), ctypes.c_void_p(target), pool,
        _dev(episode_index, "i32", (B,), "episode_index", optional=True), B, T,
        _dev(obs, "f32", (pool, T + 1, N, D), "obs"), _dev(avail, "u8", (pool, T + 1, N, A), "avail"),
        _dev(actions, "i32", (pool, T, N), "actions"), _dev(reward, "f32", (pool, T), "reward"),
        _dev(terminated, "u8", (pool, T), "terminated"), _dev(filled, "u8", (pool, T), "filled"), float(gamma),
        _dev(q_taken, "f32", (B, T, N), "q_taken"), _dev(next_max, "f32", (B, T, N), "next_max"),
        _dev(td_target, "f32", (B, T, N), "td_target"), _dev(next_action, "i32", (B, T, N), "next_action"),
        _dev(q_all, "f32", (B, T + 1, N, A), "q_all", optional=True), _stream()))


def marl_qnet_grad_workspace_bytes(handle, B, T):
    n = ctypes.c_size_t(0)
    check(load().marl_qnet_grad_workspace_bytes(ctypes.c_void_p(handle), int(B), int(T), ctypes.byref(n)))
    return int(n.value)


def marl_qnet_grad(handle, dims, obs, actions, filled, grad_q_taken, workspace, grad_weights, kept=False):
    """workspace: a device uint8 tensor of at least marl_qnet_grad_workspace_bytes bytes.
    kept: the workspace holds the activations marl_unroll_td_keep left there."""
    N, D, A, H = dims
    B, T = obs.shape[0], obs.shape[1] - 1
    n_params = (D + N) * H + H + 6 * H * H + 6 * H + A * H + A
    fn = load().marl_qnet_grad_kept if kept else load().marl_qnet_grad
    check(fn(
        ctypes.c_void_p(handle), B, T, _dev(obs, "f32", (B, T + 1, N, D), "obs"),
        _dev(actions, "i32", (B, T, N), "actions"), _dev(filled, "u8", (B, T), "filled"),
        _dev(grad_q_taken, "f32", (B, T, N), "grad_q_taken"), _dev(workspace, "u8", (workspace.numel(),), "workspace"),
        int(workspace.numel()), _dev(grad_weights, "f32", (n_params,), "grad_weights"), _stream()))


class QNet:
    """Convenience owner of one handle (create on init, destroy on close)."""

    def __init__(self, dims, weights, dtype="fp32", device=0):
        self.dims = tuple(int(v) for v in dims)
        N, D, A, H = self.dims
        self.device = device
        self.handle = marl_qnet_create(N, D, A, H, DTYPES[dtype], device, weights)

    def act_step(self, obs, avail, h_in, reset, step_t, epsilon, seed, h_out, action, q_out=None):
        marl_act_step(self.handle, self.dims, obs, avail, h_in, reset, step_t, epsilon, seed, h_out, action, q_out)

    def unroll_td_indexed(self, target, episode_index, obs, avail, actions, reward, terminated, filled, gamma,
                          q_taken, next_max, td_target, q_all=None):
        tgt = self if target is None else target
        marl_unroll_td_indexed(self.handle, tgt.handle, self.dims, episode_index, obs, avail, actions, reward,
                               terminated, filled, gamma, q_taken, next_max, td_target, q_all)

    def unroll_td_double(self, target, obs, avail, actions, reward, terminated, filled, gamma,
                         q_taken, next_max, td_target, next_action, q_all=None, episode_index=None):
        tgt = self if target is None else target
        marl_unroll_td_double(self.handle, tgt.handle, self.dims, obs, avail, actions, reward, terminated, filled,
                              gamma, q_taken, next_max, td_target, next_action, q_all, episode_index)

    def rmsprop_step(self, weights, grad_weights, sq_avg, lr, alpha=0.99, eps=1e-5):
        n = weights.numel()
        check(load().marl_qnet_rmsprop_step(ctypes.c_void_p(self.handle), _dev(weights, "f32", (n,), "weights"),
                                            _dev(grad_weights, "f32", (n,), "grad_weights"), _dev(sq_avg, "f32", (n,), "sq_avg"),
                                            float(lr), float(alpha), float(eps), _stream()))

    def sgd_step(self, weights, grad_weights, lr):
        n = weights.numel()
        check(load().marl_qnet_sgd_step(ctypes.c_void_p(self.handle), _dev(weights, "f32", (n,), "weights"),
                                        _dev(grad_weights, "f32", (n,), "grad_weights"), float(lr), _stream()))

    def grad_workspace_bytes(self, B, T):
        return marl_qnet_grad_workspace_bytes(self.handle, B, T)

    def grad(self, obs, actions, filled, grad_q_taken, workspace, grad_weights, kept=False):
        marl_qnet_grad(self.handle, self.dims, obs, actions, filled, grad_q_taken, workspace, grad_weights, kept)

    def unroll_td_keep(self, target, obs, avail, actions, reward, terminated, filled, gamma,
                       q_taken, next_max, td_target, workspace, q_all=None):
        N, D, A, H = self.dims
        B, T = obs.shape[0], obs.shape[1] - 1
        tgt = self if target is None else target
        check(load().marl_unroll_td_keep(
            ctypes.c_void_p(self.handle), ctypes.c_void_p(tgt.handle), B, T, _dev(obs, "f32", (B, T + 1, N, D), "obs"),
            _dev(avail, "u8", (B, T + 1, N, A), "avail"), _dev(actions, "i32", (B, T, N), "actions"),
            _dev(reward, "f32", (B, T), "reward"), _dev(terminated, "u8", (B, T), "terminated"),
            _dev(filled, "u8", (B, T), "filled"), float(gamma), _dev(q_taken, "f32", (B, T, N), "q_taken"),
            _dev(next_max, "f32", (B, T, N), "next_max"), _dev(td_target, "f32", (B, T, N), "td_target"),
            _dev(q_all, "f32", (B, T + 1, N, A), "q_all", optional=True),
            _dev(workspace, "u8", (workspace.numel(),), "workspace"), int(workspace.numel()), _stream()))

    def act_step_indexed(self, env_index, obs, avail, h_in, reset, step_t, epsilon, seed, h_out, action, q_out=None):
        marl_act_step_indexed(self.handle, self.dims, env_index, obs, avail, h_in, reset, step_t, epsilon, seed,
                              h_out, action, q_out)

    def unroll_td(self, target, obs, avail, actions, reward, terminated, filled, gamma,
                  q_taken, next_max, td_target, q_all=None, static=False):
        tgt = self if target is None else target
        marl_unroll_td(self.handle, tgt.handle, self.dims, obs, avail, actions, reward, terminated, filled,
                       gamma, q_taken, next_max, td_target, q_all, static=static)

    def set_weights(self, weights):
        marl_qnet_set_weights(self.handle, weights)

    def set_kernels(self, path):
        marl_qnet_set_kernels(self.handle, path)

    def kernels_in_use(self, entry):
        return marl_qnet_kernels_in_use(self.handle, entry)

    def set_timing(self, enable):
        marl_qnet_set_timing(self.handle, enable)

    def timing_read(self):
        return marl_qnet_timing_read(self.handle)

    def close(self):
        if self.handle:
            marl_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ------------------------------------------------------------------ mixing network (include/marl_mixer.h)
def marl_mixer_param_count(n_agents, embed, state_dim, weight_dtype=MARL_DTYPE_F32, device=0):
    d = MixerDesc(n_agents, embed, state_dim, weight_dtype, device)
    return int(load().marl_mixer_param_count(ctypes.byref(d)))


def marl_mixer_create(n_agents, embed, state_dim, weight_dtype, device, host_weights):
    w = np.ascontiguousarray(host_weights, dtype=np.float32)
    d = MixerDesc(n_agents, embed, state_dim, weight_dtype, device)
    out = ctypes.c_void_p()
    check(load().marl_mixer_create(ctypes.byref(d), w.ctypes.data_as(ctypes.c_void_p), w.size, ctypes.byref(out)))
    return out.value


def marl_mixer_set_weights(handle, host_weights):
    """Stream-ordered in-place parameter refresh on torch's current stream."""
    w = np.ascontiguousarray(host_weights, dtype=np.float32)
    check(load().marl_mixer_set_weights(ctypes.c_void_p(handle), w.ctypes.data_as(ctypes.c_void_p), w.size, _stream()))


def marl_mixer_destroy(handle):
    load().marl_mixer_destroy(ctypes.c_void_p(handle))


def marl_mixer_td(online, target, dims, state, q_taken, next_max, reward, terminated, filled, gamma,
                  q_total, y_total, td_err, loss=None):
    N, M, S = dims
    B, T = int(state.shape[0]), int(state.shape[1]) - 1
    check(load().marl_mixer_td(
        ctypes.c_void_p(online), ctypes.c_void_p(target) if target else None, B, T,
        _dev(state, "f32", (B, T + 1, S), "state"), _dev(q_taken, "f32", (B, T, N), "q_taken"),
        _dev(next_max, "f32", (B, T, N), "next_max"), _dev(reward, "f32", (B, T), "reward"),
        _dev(terminated, "u8", (B, T), "terminated"), _dev(filled, "u8", (B, T), "filled"), float(gamma),
        _dev(q_total, "f32", (B, T), "q_total", optional=True), _dev(y_total, "f32", (B, T), "y_total", optional=True),
        _dev(td_err, "f32", (B, T), "td_err", optional=True), _dev(loss, "f32", (2,), "loss", optional=True), _stream()))


class Mixer:
    """Thin owner of a marl_mixer handle."""

    def __init__(self, dims, weights, dtype="fp32", device=0):
        self.dims = tuple(int(v) for v in dims)
        self.handle = marl_mixer_create(*self.dims, DTYPES[dtype], device, weights)

    def set_weights(self, weights):
        marl_mixer_set_weights(self.handle, weights)

    def rmsprop_step(self, weights, grad_weights, sq_avg, lr, alpha=0.99, eps=1e-5):
        n = weights.numel()
        check(load().marl_mixer_rmsprop_step(ctypes.c_void_p(self.handle), _dev(weights, "f32", (n,), "weights"),
                                             _dev(grad_weights, "f32", (n,), "grad_weights"), _dev(sq_avg, "f32", (n,), "sq_avg"),
                                             float(lr), float(alpha), float(eps), _stream()))

    def sgd_step(self, weights, grad_weights, lr):
        n = weights.numel()
        check(load().marl_mixer_sgd_step(ctypes.c_void_p(self.handle), _dev(weights, "f32", (n,), "weights"),
                                         _dev(grad_weights, "f32", (n,), "grad_weights"), float(lr), _stream()))

    def grad_workspace_bytes(self, B, T):
        n = ctypes.c_size_t(0)
        check(load().marl_mixer_grad_workspace_bytes(ctypes.c_void_p(self.handle), int(B), int(T), ctypes.byref(n)))
        return int(n.value)

    def grad(self, state, q_taken, grad_q_total, workspace, grad_q_taken, grad_weights):
        N, M, S = self.dims
        B, T = q_taken.shape[0], q_taken.shape[1]
        n_params = (N * M + 3 * M) * (S + 1) + M + 1
        check(load().marl_mixer_grad(
            ctypes.c_void_p(self.handle), B, T, _dev(state, "f32", (B, T + 1, S), "state"),
            _dev(q_taken, "f32", (B, T, N), "q_taken"), _dev(grad_q_total, "f32", (B, T), "grad_q_total"),
            _dev(workspace, "u8", (workspace.numel(),), "workspace"), int(workspace.numel()),
            _dev(grad_q_taken, "f32", (B, T, N), "grad_q_taken"), _dev(grad_weights, "f32", (n_params,), "grad_weights"),
            _stream()))

    def td(self, target, state, q_taken, next_max, reward, terminated, filled, gamma, q_total, y_total, td_err,
           loss=None):
        marl_mixer_td(self.handle, None if target is None else target.handle, self.dims, state, q_taken, next_max,
                      reward, terminated, filled, gamma, q_total, y_total, td_err, loss)

    def close(self):
        if self.handle:
            marl_mixer_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
