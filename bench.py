#!/usr/bin/env python3
"""One-GPU benchmark of the recurrent Q-network hot path.

A step is one pass of the whole path over one batch of synthetic input: one decision step
for E environments x N agents (marl_act_step, Q values written) followed by one unroll+TD over
B episodes x T transitions with a distinct target network (marl_unroll_td).  Inputs are
resident in HBM before timing starts; the act-step inputs rotate through a pool larger than
the 256 MB last-level cache so that they are read from HBM.

Prints ONE JSON line.  value = agent-steps/s of the whole step,
(E*N + B*T*N) / time per step; the act-step and unroll figures are reported separately next
to it, with a roofline object for the dominant kernel and the oracle's CPU timing.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"hbm_GBs": 8000.0, "fp32_TFs": 157.3, "bf16_TFs": 2500.0}
LLC_BYTES = 256 << 20
CALIBRATION_BYTES = 256 << 20        # size of the plain streaming kernel launched once for counter calibration


def csrc_digest():
    """SHA-256 over the kernel sources: a counter measurement is only quoted for the build it was taken on."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for p in sorted(glob.glob(os.path.join(ROOT, "paper_2205_05248_amd", "csrc", "*"))):
        h.update(os.path.basename(p).encode())
        h.update(open(p, "rb").read())
    return h.hexdigest()


def recorded_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` on `workload` from the rocprofv3 counter summary under
    profiles/, or None if there is none for the present kernel sources."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{kernel}_{workload}.txt")
    if not os.path.exists(path):
        return None
    kv = {}
    for line in open(path):
        if "=" in line and not line.lstrip().startswith("#"):
            k, v = line.split("=", 1)
            kv[k.strip()] = v.strip()
    if kv.get("csrc_sha256") != csrc_digest():
        return None
    return float(kv["hbm_bytes_per_launch"])


def flops_per_agent_step(N, D, A, H):
    # fc1 (the one-hot id is a column gather, not a multiply), two GRU products, fc2
    return 2 * D * H + 2 * (3 * H * H) * 2 + 2 * H * A


def act_bytes_per_agent_step(N, D, A, H, with_q=True):
    # obs + avail + h in + h out + action (+ Q)
    return 4 * D + A + 8 * H + 4 + (4 * A if with_q else 0)


def unroll_bytes_per_agent_step(N, D, A, H):
    # obs + avail + action + q_taken + next_max + td_target
    return 4 * D + A + 16


KERNELS = {"auto": 0, "tile32": 1, "fused16": 2, "stream16": 3}


class Bench:
    def __init__(self, ci, two_nets=True, kernels="auto"):
        import torch
        from paper_2205_05248_amd import binding, workloads as wl
        self.torch, self.wl = torch, wl
        self.cfg = cfg = wl.config(ci)
        self.dims = dims = wl.dims(cfg)
        N, D, A, H = dims
        self.w_on, self.w_tg = wl.make_weights(cfg, 0), wl.make_weights(cfg, 1)
        self.online = binding.QNet(dims, self.w_on, cfg["dtype"])
        self.target = binding.QNet(dims, self.w_tg, cfg["dtype"]) if two_nets else None
        self.online.set_kernels(KERNELS[kernels])
        self.fused = self.online.kernels_in_use(binding.ENTRY_UNROLL_TD) == binding.KERNELS_FUSED16
        self.act_fused = self.online.kernels_in_use(binding.ENTRY_ACT_STEP) == binding.KERNELS_FUSED16
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        E, B, T = cfg["E"], cfg["B"], cfg["T"]
        set_bytes = E * N * act_bytes_per_agent_step(*dims)
        self.pool = max(2, min(64, -(-2 * LLC_BYTES // set_bytes)))
        self.act_in = []
        for s in range(self.pool):
            inp = wl.make_act_inputs(cfg, stream=s % 4)
            self.act_in.append({k: dev(inp[k]) for k in ("obs", "avail", "h_in", "reset", "step_t")})
            self.act_meta = inp
        self.h_out = [torch.empty(E, N, H, device="cuda") for _ in range(self.pool)]
        self.action = torch.empty(E, N, dtype=torch.int32, device="cuda")
        self.q = [torch.empty(E, N, A, device="cuda") for _ in range(self.pool)]
        u = wl.make_unroll_inputs(cfg)
        self.u_host = u
        self.u = {k: dev(u[k]) for k in ("obs", "avail", "actions", "reward", "terminated", "filled")}
        self.u_out = [torch.empty(B, T, N, device="cuda") for _ in range(3)]
        self.n_act = 0
        torch.cuda.synchronize()

    def act(self):
        i = self.n_act % self.pool
        self.n_act += 1
        a = self.act_in[i]
        self.online.act_step(a["obs"], a["avail"], a["h_in"], a["reset"], a["step_t"], self.act_meta["epsilon"],
                             self.act_meta["seed"] + self.n_act, self.h_out[i], self.action, self.q[i])

    def unroll(self):
        u = self.u
        self.online.unroll_td(self.target, u["obs"], u["avail"], u["actions"], u["reward"], u["terminated"],
                              u["filled"], self.u_host["gamma"], *self.u_out)

    def run(self, steps, warmup):
        """K timed steps.  The library records HIP events around each of its kernels on the
        stream it launches on, so per-kernel means come from the same timed region."""
        torch = self.torch
        for _ in range(warmup):
            self.act(); self.unroll()
        # one plain streaming kernel of known size (reads and writes CALIBRATION_BYTES each), outside
        # the timed region: hardware byte counters collected over this run are scaled by what they
        # read for it
        src = torch.ones(CALIBRATION_BYTES // 4, device="cuda")
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)
        del src, dst
        torch.cuda.synchronize()
        self.online.set_timing(True)
        t0 = time.perf_counter()
        for _ in range(steps):
            self.act(); self.unroll()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        k = self.online.timing_read()
        self.online.set_timing(False)
        return wall, k

    def back_to_back_act(self, n=200):
        torch = self.torch
        for _ in range(5):
            self.act()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(n):
            self.act()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    def back_to_back_act_indexed(self, n=200):
        """The decision step through marl_act_step_indexed with every environment listed, in a random order."""
        torch = self.torch
        E = self.cfg["E"]
        order = torch.from_numpy(np.random.default_rng(0).permutation(E).astype(np.int32)).cuda()
        def call():
            i = self.n_act % self.pool
            self.n_act += 1
            a = self.act_in[i]
            self.online.act_step_indexed(order, a["obs"], a["avail"], a["h_in"], a["reset"], a["step_t"], self.act_meta["epsilon"],
                                         self.act_meta["seed"] + self.n_act, self.h_out[i], self.action, self.q[i])
        for _ in range(5):
            call()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(n):
            call()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    def cache_resident_act(self, n=100):
        """The same launch on one buffer over and over: inputs stay in the memory-side cache."""
        torch = self.torch
        a0 = self.act_in[0]
        call = lambda: self.online.act_step(a0["obs"], a0["avail"], a0["h_in"], a0["reset"], a0["step_t"],
                                            self.act_meta["epsilon"], self.act_meta["seed"], self.h_out[0], self.action, self.q[0])
        for _ in range(5):
            call()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(n):
            call()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    def single_net_unroll(self, n=10, double=False):
        """target == online: one network's unroll instead of two; double: the double-estimator
        target (the two networks one after the other, the second valuing the first's choice)."""
        torch = self.torch
        u = self.u
        if double:
            nxt = torch.empty(self.u_out[0].shape, dtype=torch.int32, device="cuda")
            call = lambda: self.online.unroll_td_double(self.target, u["obs"], u["avail"], u["actions"], u["reward"],
                                                        u["terminated"], u["filled"], self.u_host["gamma"],
                                                        *self.u_out, nxt)
        else:
            call = lambda: self.online.unroll_td(None, u["obs"], u["avail"], u["actions"], u["reward"],
                                                 u["terminated"], u["filled"], self.u_host["gamma"], *self.u_out)
        for _ in range(2):
            call()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(n):
            call()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    def act_outputs(self, seed):
        """The decision step on input set 0 (the one the oracle leg regenerates), copied to the host."""
        torch = self.torch
        a0 = self.act_in[0]
        self.online.act_step(a0["obs"], a0["avail"], a0["h_in"], a0["reset"], a0["step_t"], self.act_meta["epsilon"], seed,
                             self.h_out[0], self.action, self.q[0])
        torch.cuda.synchronize()
        return {"seed": seed, "h_out": self.h_out[0].cpu().numpy(), "action": self.action.cpu().numpy(),
                "q": self.q[0].cpu().numpy()}

    def unroll_outputs(self):
        """The unroll the timed region runs, with every slot's Q values as well, copied to the host."""
        torch = self.torch
        u = self.u
        B, T = self.cfg["B"], self.cfg["T"]
        N, D, A, H = self.dims
        q_all = torch.empty(B, T + 1, N, A, device="cuda")
        self.online.unroll_td(self.target, u["obs"], u["avail"], u["actions"], u["reward"], u["terminated"],
                              u["filled"], self.u_host["gamma"], *self.u_out, q_all)
        torch.cuda.synchronize()
        out = {k: v.cpu().numpy() for k, v in zip(("q_taken", "next_max", "td_target"), self.u_out)}
        out["q_all"] = q_all.cpu().numpy()
        return out

    def close(self):
        self.online.close()
        if self.target is not None:
            self.target.close()


def _median_time(fn, reps):
    times = []
    for _ in range(reps):
        t0 = time.perf_counter()
        fn()
        times.append(time.perf_counter() - t0)
    return float(np.median(times))


def cpu_baseline(ci, gpu_act=None, gpu_unroll=None):
    """The oracle as it stands, timed on this host's cores on a bounded sample of the workload: medians over
    repetitions, with all cores and with one thread.  Its outputs for the benchmarked inputs are also what the GPU
    results (gpu_act: the decision step on input set 0, gpu_unroll: the unroll's outputs) are compared with."""
    from oracle import marl_oracle as orc
    from paper_2205_05248_amd import workloads as wl
    cfg = wl.config(ci)
    dims = wl.dims(cfg)
    N, E, B, T = cfg["N"], cfg["E"], cfg["B"], cfg["T"]
    tol = 2e-2 if cfg["dtype"] == "bf16" else 1e-4
    rounded = lambda w: w if cfg["dtype"] != "bf16" else _bf16_matrices(orc, wl, dims, w)
    w_on, w_tg = rounded(wl.make_weights(cfg, 0)), rounded(wl.make_weights(cfg, 1))
    inp = wl.make_act_inputs(cfg, stream=0)
    threads = orc.default_threads()
    act = lambda n_env, nthreads, seed: orc.act_step(
        dims, w_on, inp["obs"][:n_env], inp["avail"][:n_env], inp["h_in"][:n_env], inp["reset"][:n_env],
        inp["step_t"][:n_env], inp["epsilon"], seed, nthreads=nthreads)
    act(min(E, 8), threads, 1)                                     # build / page in
    act_reps = 5
    t_act = _median_time(lambda: act(E, threads, inp["seed"]), act_reps)
    e_one = max(1, E // 16)
    t_act_one = _median_time(lambda: act(e_one, 1, inp["seed"]), act_reps) * E / e_one
    u = wl.make_unroll_inputs(cfg)
    rows_total = B * N
    unroll = lambda rows, nthreads, q_all: orc.unroll_td(
        dims, w_on, w_tg, u["obs"], u["avail"], u["actions"], u["reward"], u["terminated"], u["filled"], u["gamma"],
        want_q_all=q_all, rows=rows, nthreads=nthreads)
    unroll_reps = 3
    t_unroll = _median_time(lambda: unroll(None, threads, False), unroll_reps)
    rows_one = np.arange(min(rows_total, 64), dtype=np.int32)
    t_unroll_one = _median_time(lambda: unroll(rows_one, 1, False), unroll_reps) * rows_total / rows_one.size
    steps_act, steps_unroll = E * N, B * T * N
    out = {
        "value": (steps_act + steps_unroll) / (t_act + t_unroll), "unit": "agent-steps/s", "cores": threads,
        "kind": "oracle",
        "sample": f"act-step: all {steps_act} rows, median of {act_reps}; unroll+TD (two networks): all {rows_total} "
                  f"(episode, agent) rows over all T+1 slots, median of {unroll_reps}; single-thread figures: "
                  f"{e_one} environments / {rows_one.size} rows, scaled to the whole batch",
        "act_agent_steps_per_s": steps_act / t_act,
        "unroll_episode_steps_per_s": B * T / t_unroll,
        "single_thread": {"value": (steps_act + steps_unroll) / (t_act_one + t_unroll_one),
                          "act_agent_steps_per_s": steps_act / t_act_one,
                          "unroll_episode_steps_per_s": B * T / t_unroll_one},
        "seconds": {"act_all_cores": t_act, "unroll_all_cores": t_unroll, "act_one_thread_scaled": t_act_one,
                    "unroll_one_thread_scaled": t_unroll_one},
    }
    parity = {"tolerance": tol}
    if gpu_act is not None:
        ref = act(E, threads, gpu_act["seed"])
        # a near-tie: a greedy row whose two best available Q values lie within the tolerance of each other
        near = (ref["explored"] == 0) & (_top2_margin(ref["q"], inp["avail"]) <= tol)
        differ = gpu_act["action"] != ref["action"]
        parity["act_step"] = {
            "rows": steps_act, "max_abs_err_q": float(np.abs(gpu_act["q"] - ref["q"]).max()),
            "max_abs_err_h": float(np.abs(gpu_act["h_out"] - ref["h_out"]).max()),
            "near_ties": int(near.sum()),
            "actions_differing": int(differ.sum()),
            "actions_differing_outside_near_ties": int((differ & ~near).sum())}
    if gpu_unroll is not None:
        ref = unroll(None, threads, True)
        parity["unroll_td"] = {"rows": rows_total}
        for k in ("q_taken", "next_max", "td_target", "q_all"):
            if gpu_unroll.get(k) is not None:
                parity["unroll_td"]["max_abs_err_" + k] = float(np.abs(gpu_unroll[k] - ref[k]).max())
    return out, parity


def _bf16_matrices(orc, wl, dims, w):
    """A bf16 network's weights as the network holds them: the matrices rounded to bf16, the biases as given."""
    w = np.array(w, np.float32)
    for name, (a, b, shp) in wl.weight_slices(*dims).items():
        if len(shp) == 2:
            w[a:b] = orc.round_bf16(w[a:b])
    return w


def _top2_margin(q, avail):
    """Gap between the best and second-best available Q value of each row (inf with fewer than two)."""
    masked = np.where(avail != 0, q.astype(np.float64), -np.inf)
    top = np.sort(masked, axis=-1)[..., -2:]
    gap = top[..., 1] - top[..., 0]
    return np.where(np.isfinite(gap), gap, np.inf)


def measured_peaks():
    """What this GPU reaches on plain kernels, next to the nominal peaks: the library's streaming probe over 1 GiB
    (read only; copy, bytes read plus bytes written) and its probe of dependency-free bf16 matrix instructions."""
    import torch
    from paper_2205_05248_amd import binding

    def timed(fn, n):
        for _ in range(3):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / n
    src = torch.ones((1 << 30) // 4, device="cuda")
    dst = torch.empty_like(src)
    sink = torch.zeros(1, device="cuda")
    t_read = timed(lambda: binding.marl_probe_stream(src, None, sink), 20)
    t_copy = timed(lambda: binding.marl_probe_stream(src, dst, sink), 20)
    assert torch.equal(dst[-4096:], src[-4096:]) and float(sink) == 0.0
    del src, dst
    torch.cuda.empty_cache()
    flops = binding.marl_probe_mfma(20000, sink)
    t_mfma = timed(lambda: binding.marl_probe_mfma(20000, sink), 5)
    return {"stream_read_GBs": (1 << 30) / t_read / 1e9, "stream_copy_GBs": 2 * (1 << 30) / t_copy / 1e9,
            "mfma_bf16_TFLOPs": flops / t_mfma / 1e12,
            "nominal": {"hbm_GBs": PEAK["hbm_GBs"], "bf16_TFLOPs": PEAK["bf16_TFs"]}}


def mixer_section(ci, with_cpu, launches=20):
    """The mixing network on the same workload's batch (the row after the unroll in the learner
    step; not part of the timed step above): kernel time from events on the launch stream, and
    the mixer oracle on a bounded sample of transitions."""
    import torch
    from paper_2205_05248_amd import binding, workloads as wl
    cfg = wl.config(ci)
    dims = N, M, S = wl.mixer_dims(cfg)
    B, T = cfg["B"], cfg["T"]
    w_on, w_tg = wl.make_mixer_weights(cfg, 0), wl.make_mixer_weights(cfg, 1)
    online, target = binding.Mixer(dims, w_on, cfg["dtype"]), binding.Mixer(dims, w_tg, cfg["dtype"])
    m = wl.make_mixer_inputs(cfg)
    d = {k2: torch.from_numpy(np.ascontiguousarray(m[k2])).cuda()
         for k2 in ("state", "q_taken", "next_max", "reward", "terminated", "filled")}
    outs = [torch.empty(B, T, device="cuda") for _ in range(3)]
    call = lambda: online.td(target, d["state"], d["q_taken"], d["next_max"], d["reward"], d["terminated"],
                             d["filled"], m["gamma"], *outs)
    for _ in range(3):
        call()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(launches):
        call()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / launches
    # the mixer's backward pass on the same batch (parameter gradients and dL/dq_taken for an upstream dL/dQ_total)
    grad_ms = None
    try:
        need = online.grad_workspace_bytes(B, T)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        gq = torch.empty(B, T, N, device="cuda")
        gw = torch.empty(wl.mixer_param_count(*dims), device="cuda")
        gcall = lambda: online.grad(d["state"], d["q_taken"], outs[2], ws, gq, gw)
        for _ in range(2):
            gcall()
        torch.cuda.synchronize()
        a.record()
        for _ in range(launches):
            gcall()
        b.record()
        torch.cuda.synchronize()
        grad_ms = a.elapsed_time(b) / launches
    except binding.MarlError:
        pass
    online.close(); target.close()
    flops = 2 * B * T * 2 * (N * M + 3 * M) * S                  # two mixers, one multiply-add per generated quantity and state value
    io_bytes = B * (T + 1) * S * 4 + 2 * B * T * N * 4 + B * T * (4 + 2 + 12)
    out = {"kernel": "mixer_td", "ms": ms, "transitions_per_s": B * T / (ms * 1e-3), "bound": "mfma",
           "TFLOPs": flops / (ms * 1e-3) / 1e12, "mfma_frac": flops / (ms * 1e-3) / 1e12 / PEAK["bf16_TFs"],
           "GBs": io_bytes / (ms * 1e-3) / 1e9, "hbm_frac": io_bytes / (ms * 1e-3) / 1e9 / PEAK["hbm_GBs"],
           "grad_ms": grad_ms,
           "config": {"n_agents": N, "embed": M, "state_dim": S, "B": B, "T": T, "mixers": "online + target"}}
    if with_cpu:
        from oracle import mixer_oracle as mxo
        sample_b = max(1, min(B, 4096 // T))
        t0 = time.perf_counter()
        mxo.td(dims, w_on, w_tg, m["state"][:sample_b], m["q_taken"][:sample_b], m["next_max"][:sample_b],
               m["reward"][:sample_b], m["terminated"][:sample_b], m["filled"][:sample_b], m["gamma"])
        sec = time.perf_counter() - t0
        out["cpu_oracle"] = {"transitions_per_s": sample_b * T / sec, "cores": 1,
                             "sample": f"first {sample_b} of {B} episodes, all {T} transitions"}
        if grad_ms is not None:
            gb = max(1, min(B, 1024 // T))
            e = np.random.default_rng(2).normal(size=(gb, T))
            t0 = time.perf_counter()
            mxo.grad(dims, w_on, m["state"][:gb], m["q_taken"][:gb].astype(np.float64), e)
            sec = time.perf_counter() - t0
            out["grad_cpu_oracle"] = {"transitions_per_s": gb * T / sec, "cores": 1,
                                      "sample": f"first {gb} of {B} episodes, all {T} transitions"}
    return out


def grad_section(ci, with_cpu, launches=10):
    """The backward pass of the learner step on the same workload's batch (marl_qnet_grad: forward pass that
    keeps activations, time-reversed pass, weight-gradient products; not part of the timed step above):
    time per call from events on the launch stream, and the back-propagation oracle on a bounded sample."""
    import torch
    from paper_2205_05248_amd import binding, workloads as wl
    cfg = wl.config(ci)
    dims = N, D, A, H = wl.dims(cfg)
    B, T = cfg["B"], cfg["T"]
    w = wl.make_weights(cfg, 0)
    net = binding.QNet(dims, w, cfg["dtype"])
    u = wl.make_unroll_inputs(cfg)
    try:
        need = net.grad_workspace_bytes(B, T)
    except binding.MarlError:
        net.close()
        return {"kernel": "qnet_grad", "ms": None, "note": "the network does not fit the fused kernels the backward pass builds on"}
    d = {k: torch.from_numpy(np.ascontiguousarray(u[k])).cuda() for k in ("obs", "actions", "filled")}
    g_host = np.random.default_rng(1).normal(size=(B, T, N)).astype(np.float32)
    g = torch.from_numpy(g_host).cuda()
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    out_grad = torch.empty(wl.param_count(*dims), device="cuda")
    call = lambda: net.grad(d["obs"], d["actions"], d["filled"], g, ws, out_grad)
    for _ in range(2):
        call()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(launches):
        call()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / launches
    # the parameter update that follows it: weights -= lr * gradient, image rebuilt on the device
    master = torch.from_numpy(w.copy()).cuda()
    net.sgd_step(master, out_grad, 0.0)                   # the first call builds the map
    torch.cuda.synchronize()
    a.record()
    for _ in range(launches):
        net.sgd_step(master, out_grad, 0.0)
    b.record()
    torch.cuda.synchronize()
    sgd_ms = a.elapsed_time(b) / launches
    net.close()
    rows = B * N
    fwd = rows * (T + 1) * (2 * D * H + 12 * H * H + 2 * H * A)        # the forward pass again, activations kept
    back = rows * T * (12 * H * H + 12 * H * H)                        # the gates again + the two transposed products
    wgrad = rows * T * (2 * 2 * 3 * H * (H + 1) + 2 * H * (D + N) + 2 * A * (H + 1))
    flops = fwd + back + wgrad
    # bytes the four stages move by design (activations and adjoints kept in the workspace): the forward pass
    # reads the observations and writes x and h; the reverse pass reads x and h and writes the adjoints; each
    # product reads its two operands once
    a16 = (A + 15) // 16 * 16
    adj = 2 if cfg["dtype"] == "bf16" else 4                  # bytes per stored adjoint and per saved x (bf16 networks keep both as bf16)
    io_bytes = (rows * (T + 1) * (4 * D + 4 * H + adj * H) + rows * T * (4 * H + adj * H + adj * (5 * H + a16))
                + rows * T * ((adj * 3 * H + adj * H) + (adj * 3 * H + 4 * H) + (adj * H + 4 * D) + (adj * a16 + 4 * H)))
    out = {"kernel": "qnet_grad (4 kernels)", "ms": ms, "transitions_per_s": B * T / (ms * 1e-3), "bound": "hbm",
           "GBs": io_bytes / (ms * 1e-3) / 1e9, "hbm_frac": io_bytes / (ms * 1e-3) / 1e9 / PEAK["hbm_GBs"],
           "TFLOPs": flops / (ms * 1e-3) / 1e12, "mfma_frac": flops / (ms * 1e-3) / 1e12 / PEAK["bf16_TFs"],
           "sgd_step_ms": sgd_ms, "workspace_bytes": need,
           "config": {"B": B, "T": T, "rows": rows, "parameters": int(out_grad.numel())}}
    if with_cpu:
        from oracle import bptt_oracle as bpo
        sample_b = max(1, min(B, 2))
        t0 = time.perf_counter()
        bpo.qnet_grad(dims, w, u["obs"][:sample_b], u["actions"][:sample_b], u["filled"][:sample_b],
                      g_host[:sample_b].astype(np.float64))
        sec = time.perf_counter() - t0
        out["cpu_oracle"] = {"transitions_per_s": sample_b * T / sec, "cores": min(sample_b, bpo.default_threads()),
                             "sample": f"first {sample_b} of {B} episodes, all {T} transitions"}
    return out


def learner_section(ci, launches=10):
    """One whole learner iteration of Alg. 3 on the workload's batch, every stage in the library's kernels and
    chained on one stream with no host round trip: unroll (online + target), mixer forward with the TD loss, mixer
    backward, Q-network backward, both parameter updates (lr = 0: the weights stay put while timing).  The only
    work outside the library is one element-wise tensor operation, dL/dQ_total = -2 td_err / count."""
    import torch
    from paper_2205_05248_amd import binding, workloads as wl
    cfg = wl.config(ci)
    dims, mdims = wl.dims(cfg), wl.mixer_dims(cfg)
    N = dims[0]
    B, T = cfg["B"], cfg["T"]
    w, mw = wl.make_weights(cfg, 0), wl.make_mixer_weights(cfg, 0)
    online, target = binding.QNet(dims, w, cfg["dtype"]), binding.QNet(dims, wl.make_weights(cfg, 1), cfg["dtype"])
    mixer, mixer_tg = binding.Mixer(mdims, mw, cfg["dtype"]), binding.Mixer(mdims, wl.make_mixer_weights(cfg, 1), cfg["dtype"])
    try:
        need, mneed = online.grad_workspace_bytes(B, T), mixer.grad_workspace_bytes(B, T)
    except binding.MarlError:
        for h in (online, target, mixer, mixer_tg):
            h.close()
        return {"ms": None, "note": "the backward passes do not serve this shape"}
    u = wl.make_unroll_inputs(cfg)
    d = {k: torch.from_numpy(np.ascontiguousarray(u[k])).cuda()
         for k in ("obs", "avail", "actions", "reward", "terminated", "filled")}
    state = torch.from_numpy(wl.make_mixer_inputs(cfg)["state"]).cuda()
    q_taken, next_max, y = (torch.empty(B, T, N, device="cuda") for _ in range(3))
    q_total, y_total, td = (torch.empty(B, T, device="cuda") for _ in range(3))
    loss2 = torch.empty(2, device="cuda")
    master, grad = torch.from_numpy(w.copy()).cuda(), torch.empty(w.size, device="cuda")
    mmaster, mgrad = torch.from_numpy(mw.copy()).cuda(), torch.empty(mw.size, device="cuda")
    gq = torch.empty(B, T, N, device="cuda")
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    mws = torch.empty(mneed, dtype=torch.uint8, device="cuda")

    # dL/dQ_total = -2 td_err / count as one element-wise kernel: 0 + (-2) * td / count
    zero, e = torch.zeros(B, T, device="cuda"), torch.empty(B, T, device="cuda")

    def iteration():
        online.unroll_td_keep(target, d["obs"], d["avail"], d["actions"], d["reward"], d["terminated"], d["filled"],
                              u["gamma"], q_taken, next_max, y, ws)          # leaves x and h for the backward pass
        mixer.td(mixer_tg, state, q_taken, next_max, d["reward"], d["terminated"], d["filled"], u["gamma"],
                 q_total, y_total, td, loss2)
        torch.addcdiv(zero, td, loss2[1], value=-2.0, out=e)
        mixer.grad(state, q_taken, e, mws, gq, mgrad)
        online.grad(d["obs"], d["actions"], d["filled"], gq, ws, grad, kept=True)
        online.sgd_step(master, grad, 0.0)
        mixer.sgd_step(mmaster, mgrad, 0.0)

    for _ in range(2):
        iteration()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(launches):
        iteration()
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / launches
    # where the time goes: the same calls with an event after every stage
    stage_names = ["unroll_td_keep", "mixer_td", "dL/dQ_total (tensor op)", "mixer_grad", "qnet_grad_kept", "qnet_sgd_step", "mixer_sgd_step"]
    stage_ms = [0.0] * len(stage_names)

    def staged():
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(stage_names) + 1)]
        ev[0].record()
        online.unroll_td_keep(target, d["obs"], d["avail"], d["actions"], d["reward"], d["terminated"], d["filled"],
                              u["gamma"], q_taken, next_max, y, ws)
        ev[1].record()
        mixer.td(mixer_tg, state, q_taken, next_max, d["reward"], d["terminated"], d["filled"], u["gamma"],
                 q_total, y_total, td, loss2)
        ev[2].record()
        torch.addcdiv(zero, td, loss2[1], value=-2.0, out=e)
        ev[3].record()
        mixer.grad(state, q_taken, e, mws, gq, mgrad)
        ev[4].record()
        online.grad(d["obs"], d["actions"], d["filled"], gq, ws, grad, kept=True)
        ev[5].record()
        online.sgd_step(master, grad, 0.0)
        ev[6].record()
        mixer.sgd_step(mmaster, mgrad, 0.0)
        ev[7].record()
        torch.cuda.synchronize()
        for i in range(len(stage_names)):
            stage_ms[i] += ev[i].elapsed_time(ev[i + 1]) / launches

    for _ in range(launches):
        staged()
    # the same iteration replayed from a HIP graph (the calls allocate nothing and record no memset)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            iteration()
    torch.cuda.synchronize()
    for _ in range(2):
        graph.replay()
    torch.cuda.synchronize()
    a.record()
    for _ in range(launches):
        graph.replay()
    b.record()
    torch.cuda.synchronize()
    ms_graph = a.elapsed_time(b) / launches
    del graph
    for h in (online, target, mixer, mixer_tg):
        h.close()
    return {"ms": ms, "ms_graph_replay": ms_graph, "transitions_per_s": B * T / (ms * 1e-3),
            "agent_steps_per_s": B * T * N / (ms * 1e-3),
            "stage_ms": {k: round(v, 4) for k, v in zip(stage_names, stage_ms)},
            "stages": "unroll_td_keep (2 networks) + mixer_td + mixer_grad + qnet_grad_kept + qnet_sgd_step + mixer_sgd_step",
            "config": {"B": B, "T": T, "n_agents": N}}


def other_config(ci, kernels, steps=50, warmup=5):
    """(workload name, compact figures) of one of the paper-scenario configurations: the same step, timed the same way."""
    b = Bench(ci, kernels=kernels)
    cfg = b.cfg
    N, D, A, H = b.dims
    E, B, T = cfg["E"], cfg["B"], cfg["T"]
    wall, k = b.run(steps, warmup)
    act_b2b_ms = b.back_to_back_act()
    b.close()
    steps_act, steps_unroll, slots = E * N, B * T * N, B * (T + 1) * N
    act_s, unroll_s = k["act_ms"] * 1e-3, (k["input_proj_ms"] if not b.fused else 0.0) * 1e-3 + k["recurrent_ms"] * 1e-3
    return cfg["name"], {
        "ms_per_step": wall * 1e3 / steps, "agent_steps_per_s": (steps_act + steps_unroll) / (wall / steps),
        "act_step": {"kernel_ms": k["act_ms"], "kernel_ms_back_to_back": act_b2b_ms,
                     "agent_steps_per_s": steps_act / act_s,
                     "hbm_frac": steps_act * act_bytes_per_agent_step(*b.dims) / act_s / 1e9 / PEAK["hbm_GBs"]},
        "unroll_td": {"kernels_ms": unroll_s * 1e3, "episode_steps_per_s": B * T / unroll_s,
                      "mfma_frac": 2 * slots * flops_per_agent_step(*b.dims) / unroll_s / 1e12 / PEAK["bf16_TFs"]},
        "dtype": cfg["dtype"], "steps": steps}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="workload index 0..4")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle's timing and the comparison with it")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline step: no mixer / gradient / learner sections, no other configurations")
    ap.add_argument("--only-this-config", action="store_true", help="leave the other configurations' figures out")
    ap.add_argument("--single-net", action="store_true", help="target == online in the unroll")
    ap.add_argument("--kernels", choices=sorted(KERNELS), default="auto",
                    help="kernel family (auto: the library's choice)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU only: every (env, agent) row is independent, so more GPUs "
                 "would each run this same kernel on their own share; run with --gpus 1")
    import torch
    from paper_2205_05248_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    b = Bench(args.config, two_nets=not args.single_net, kernels=args.kernels)
    cfg, dims = b.cfg, b.dims
    N, D, A, H = dims
    E, B, T = cfg["E"], cfg["B"], cfg["T"]
    wall, k = b.run(args.steps, args.warmup)
    act_b2b_ms = b.back_to_back_act()
    act_indexed_ms = b.back_to_back_act_indexed()
    act_cached_ms = b.cache_resident_act()
    single_net_ms = b.single_net_unroll()
    double_ms = b.single_net_unroll(double=True)
    gpu_act = gpu_unroll = None
    if not args.no_cpu_baseline and not args.single_net:
        gpu_act, gpu_unroll = b.act_outputs(b.act_meta["seed"]), b.unroll_outputs()
    names = {binding.KERNELS_TILE32: "tile32", binding.KERNELS_FUSED16: "fused16", binding.KERNELS_STREAM16: "stream16"}
    kernel_names = {"act_step": names[b.online.kernels_in_use(binding.ENTRY_ACT_STEP)],
                    "unroll_td": names[b.online.kernels_in_use(binding.ENTRY_UNROLL_TD)]}
    b.close()

    ms_per_step = wall * 1e3 / args.steps
    steps_act, steps_unroll = E * N, B * T * N
    nets = 1 if args.single_net else 2
    slots = B * (T + 1) * N                                   # network evaluations per net in the unroll
    bf16 = cfg["dtype"] == "bf16"
    # every contraction runs on the bf16 MFMA pipe (fp32 networks as three bf16 products per
    # multiply), so the matrix peak is the bf16 one; flops counted are the algorithmic ones
    peak_tf = PEAK["bf16_TFs"]
    act_ms, proj_ms, rec_ms = k["act_ms"], k["input_proj_ms"], k["recurrent_ms"]
    kernels = {
        "act_step": {
            "ms": act_ms, "calls": k["act_calls"], "bound": "hbm",
            "bytes": steps_act * act_bytes_per_agent_step(*dims), "flops": steps_act * flops_per_agent_step(*dims)},
    }
    unroll_io_bytes = slots * (4 * D + A) + B * T * N * 16        # obs + avail once; action in, three outputs
    if b.fused:
        # one kernel does the whole unroll; nothing but its inputs and outputs touches HBM
        proj_ms = 0.0
        kernels["unroll_fused"] = {
            "ms": rec_ms, "calls": k["unroll_calls"], "bound": "mfma",
            "bytes": unroll_io_bytes, "flops": nets * slots * flops_per_agent_step(*dims)}
    else:
        gi_bytes = nets * slots * 3 * H * (2 if bf16 else 4)     # written by the projection, read by the recurrence
        kernels["input_proj"] = {
            "ms": proj_ms, "calls": k["unroll_calls"], "bound": "hbm",
            "bytes": slots * 4 * D + gi_bytes, "flops": nets * slots * (2 * D * H + 2 * 3 * H * H)}
        kernels["recurrent_td"] = {
            "ms": rec_ms, "calls": k["unroll_calls"], "bound": "mfma",
            "bytes": gi_bytes + slots * A + B * T * N * 16, "flops": nets * slots * (2 * 3 * H * H + 2 * H * A)}
    for v in kernels.values():
        sec = max(v["ms"], 1e-9) * 1e-3
        v["GBs"] = v["bytes"] / sec / 1e9
        v["TFLOPs"] = v["flops"] / sec / 1e12
        v["hbm_frac"] = v["GBs"] / PEAK["hbm_GBs"]
        v["mfma_frac"] = v["TFLOPs"] / peak_tf
    dom_name = max(kernels, key=lambda n: kernels[n]["ms"])
    dom = kernels[dom_name]
    traffic = recorded_traffic(dom_name, cfg["name"])
    if dom["bound"] == "hbm":
        roofline = {"kernel": dom_name, "bound": "hbm", "achieved": dom["GBs"], "peak": PEAK["hbm_GBs"],
                    "unit": "GB/s", "frac": dom["hbm_frac"], "traffic": traffic}
    else:
        roofline = {"kernel": dom_name, "bound": "mfma", "achieved": dom["TFLOPs"], "peak": peak_tf,
                    "unit": "TFLOP/s", "frac": dom["mfma_frac"], "traffic": traffic,
                    "mfma_products_per_multiply": 1 if bf16 else 3}
    unroll_ms = proj_ms + rec_ms
    out = {
        "metric": "agent-steps/s (act-step) and episode-steps/s (unroll+TD); % HBM/MFMA peak",
        "value": (steps_act + steps_unroll) / (ms_per_step * 1e-3),
        "unit": "agent-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights, f32 accumulate" if bf16 else "f32 (bf16 hi/lo split MFMA, f32 accumulate)",
        "data": "synthetic",
        "config": {"workload": cfg["name"], "E": E, "N": N, "obs_dim": D, "n_actions": A, "hidden": H,
                   "B": B, "T": T, "target_network": "distinct" if nets == 2 else "same",
                   "kernels": kernel_names,
                   "step": "1 act-step call (E*N rows, Q written) + 1 unroll+TD call (B*T transitions)"},
        "act_step": {"agent_steps_per_s": steps_act / (act_ms * 1e-3), "kernel_ms": act_ms,
                     "kernel_ms_back_to_back": act_b2b_ms, "kernel_ms_back_to_back_indexed_all_envs_shuffled": act_indexed_ms,
                     "kernel_ms_cache_resident_inputs": act_cached_ms, "hbm_GBs": kernels["act_step"]["GBs"],
                     "hbm_frac": kernels["act_step"]["hbm_frac"], "mfma_frac": kernels["act_step"]["mfma_frac"],
                     "input_pool_bytes": b.pool * kernels["act_step"]["bytes"]},
        "unroll_td": {"episode_steps_per_s": B * T / (unroll_ms * 1e-3), "episodes_per_s": B / (unroll_ms * 1e-3),
                      "agent_steps_per_s": steps_unroll / (unroll_ms * 1e-3), "kernels_ms": unroll_ms,
                      "single_network_ms": single_net_ms,
                      "double_estimator_target_ms": double_ms,
                      "kernels": {n: {"ms": v["ms"], "TFLOPs": v["TFLOPs"], "mfma_frac": v["mfma_frac"],
                                      "GBs": v["GBs"], "hbm_frac": v["hbm_frac"]}
                                  for n, v in kernels.items() if n != "act_step"}},
        "roofline": roofline,
    }
    out["measured_peaks"] = measured_peaks()
    if not args.no_extras:
        out["mixer_td"] = mixer_section(args.config, not args.no_cpu_baseline)
        out["qnet_grad"] = grad_section(args.config, not args.no_cpu_baseline)
        out["learner_iteration"] = learner_section(args.config)
        if not args.only_this_config:
            out["all_configs"] = {wl_name: v for wl_name, v in (other_config(ci, args.kernels) for ci in range(4) if ci != args.config)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["parity_vs_oracle"] = cpu_baseline(args.config, gpu_act, gpu_unroll)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
