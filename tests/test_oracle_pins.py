"""Pins of the CPU oracle against things other than itself (CPU only).

Expected values here come from closed forms, a library routine (torch CPU
GRUCell / Linear in float64), published SplitMix64 outputs, invariants, and
brute force written out in the test; none come from the oracle or from the
GPU path.
"""
import os

import numpy as np
import pytest
import torch

from oracle import marl_oracle as orc
from paper_2205_05248_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
M64 = (1 << 64) - 1
GAMMA64 = 0x9E3779B97F4A7C15


def small_cfg(N=3, D=5, A=6, H=8, seed=7, **kw):
    c = dict(name="t", E=4, N=N, D=D, A=A, H=H, B=2, T=5, dtype="fp32", epsilon=0.0, avail_p=0.7,
             lengths="uniform_all", hetero=False, seed=seed, gamma=0.99, index=0)
    c.update(kw)
    return c


def zero_parts(dims):
    return {k: np.zeros(shp) for k, (_, _, shp) in wl.weight_slices(*dims).items()}


def run_act(cfg, w, inp, **over):
    a = dict(inp)
    a.update(over)
    return orc.act_step(wl.dims(cfg), w, a["obs"], a["avail"], a["h_in"], a["reset"], a["step_t"],
                        a["epsilon"], a["seed"])


# ---------------------------------------------------------------- RNG bits
def test_splitmix64_published_vectors():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "splitmix64_vectors.txt")) if l[0] != "#"]
    assert len(rows) >= 8
    for seed, idx, val in rows:
        state = (int(seed) + int(idx) * GAMMA64) & M64
        assert orc.S(state) == int(val)


def test_rng_draw_is_keyed_chain_of_published_generator():
    # key = S(S(S(S(seed) ^ e) ^ n) ^ t); r1, r2 = first two outputs of the stream started at key.
    # Built here only from single S() outputs, each of which is pinned above.
    for seed, e, n, t in [(0, 0, 0, 0), (1234567, 3, 1, 59), (2**63 + 5, 4095, 31, 200)]:
        k = orc.S(orc.S(orc.S(orc.S(seed) ^ e) ^ n) ^ t)
        assert orc.rng_draw(seed, e, n, t) == (orc.S(k), orc.S((k + GAMMA64) & M64))
    # different counters give different draws
    draws = {orc.rng_draw(9, e, n, t) for e in range(4) for n in range(3) for t in range(5)}
    assert len(draws) == 60


# ---------------------------------------------------------------- bf16 rounding
def test_round_bf16_matches_library_and_ties_to_even():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(5000).astype(np.float32) * 0.2,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, 1e-40, -2.5],
                                 np.float32)])
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(orc.round_bf16(x), ref)
    # 1 + 2^-8 is halfway between 1 and 1 + 2^-7: ties to even -> 1.0;
    # 1 + 3*2^-8 is halfway between 1+2^-7 and 1+2^-6 -> 1 + 2^-6.
    np.testing.assert_array_equal(orc.round_bf16(np.array([1.00390625, 1.01171875], np.float32)),
                                  np.array([1.0, 1.015625], np.float32))


# ---------------------------------------------------------------- network: library cross-check
def torch_net(dims, w):
    N, D, A, H = dims
    p = {k: torch.from_numpy(np.array(v, np.float64)) for k, v in wl.unpack_weights(dims, w).items()}
    cell = torch.nn.GRUCell(H, H).double()
    with torch.no_grad():
        cell.weight_ih.copy_(p["W_ih"]); cell.weight_hh.copy_(p["W_hh"])
        cell.bias_ih.copy_(p["b_ih"]); cell.bias_hh.copy_(p["b_hh"])

    def step(obs, h):                       # obs [R,N,D], h [R,N,H]
        R = obs.shape[0]
        eye = torch.eye(N, dtype=torch.float64).expand(R, N, N)
        x_in = torch.cat([torch.from_numpy(obs.astype(np.float64)), eye], -1).reshape(R * N, D + N)
        x = torch.relu(torch.nn.functional.linear(x_in, p["W1"], p["b1"]))
        with torch.no_grad():
            hn = cell(x, h.reshape(R * N, H))
        q = torch.nn.functional.linear(hn, p["W2"], p["b2"])
        return hn.reshape(R, N, H), q.reshape(R, N, A)
    return step


@pytest.mark.parametrize("ci", [0, 1])
def test_act_step_matches_library_grucell(ci):
    cfg = wl.config(ci)
    w = wl.make_weights(cfg)
    inp = wl.make_act_inputs(cfg, E=6)
    out = run_act(cfg, w, inp, epsilon=0.0)
    h = torch.from_numpy(inp["h_in"].astype(np.float64))
    h = h * torch.from_numpy(1.0 - inp["reset"].astype(np.float64))[:, None, None]
    hn, q = torch_net(wl.dims(cfg), w)(inp["obs"], h)
    np.testing.assert_allclose(out["h_out"], hn.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["q"], q.numpy(), rtol=0, atol=1e-12)
    # greedy action = lowest-index maximum over available actions of the library's Q
    masked = np.where(inp["avail"] != 0, q.numpy(), -np.inf)
    np.testing.assert_array_equal(out["action"], masked.argmax(-1))
    np.testing.assert_array_equal(out["greedy"], masked.argmax(-1))
    assert not out["explored"].any()


def test_unroll_td_matches_library_unroll_and_brute_force_targets():
    cfg = wl.config(0)
    dims = wl.dims(cfg)
    N, D, A, H = dims
    w_on, w_tg = wl.make_weights(cfg, 0), wl.make_weights(cfg, 1)
    inp = wl.make_unroll_inputs(cfg, B=3, T=12)
    B, T = 3, 12
    out = orc.unroll_td(dims, w_on, w_tg, inp["obs"], inp["avail"], inp["actions"], inp["reward"],
                        inp["terminated"], inp["filled"], inp["gamma"])
    qs = {}
    for key, w in (("on", w_on), ("tg", w_tg)):
        step = torch_net(dims, w)
        h = torch.zeros(B, N, H, dtype=torch.float64)
        q_t = []
        for t in range(T + 1):
            h, q = step(inp["obs"][:, t], h)
            q_t.append(q.numpy())
        qs[key] = np.stack(q_t, 1)                                   # [B,T+1,N,A]
    np.testing.assert_allclose(out["q_all"], qs["on"], rtol=0, atol=1e-12)
    g = float(np.float32(inp["gamma"]))
    for b in range(B):
        for t in range(T):
            for n in range(N):
                f = float(inp["filled"][b, t])
                u = inp["actions"][b, t, n]
                cand = [qs["tg"][b, t + 1, n, a] for a in range(A) if inp["avail"][b, t + 1, n, a]]
                nm = max(cand)
                y = float(inp["reward"][b, t]) + g * (1.0 - float(inp["terminated"][b, t])) * nm
                assert abs(out["q_taken"][b, t, n] - f * qs["on"][b, t, n, u]) < 1e-12
                assert abs(out["next_max"][b, t, n] - f * nm) < 1e-12
                assert abs(out["td_target"][b, t, n] - f * y) < 1e-12
    # target == online: bootstrap comes from the online network's own Q
    same = orc.unroll_td(dims, w_on, None, inp["obs"], inp["avail"], inp["actions"], inp["reward"],
                         inp["terminated"], inp["filled"], inp["gamma"])
    np.testing.assert_array_equal(same["q_taken"], out["q_taken"])
    b, t, n = 0, 0, 1
    cand = [qs["on"][b, t + 1, n, a] for a in range(A) if inp["avail"][b, t + 1, n, a]]
    assert abs(same["next_max"][b, t, n] - inp["filled"][b, t] * max(cand)) < 1e-12


# ---------------------------------------------------------------- network: closed forms
def test_gru_all_zero_halves_hidden_state():
    cfg = small_cfg()
    dims = wl.dims(cfg)
    parts = zero_parts(dims)
    parts["W1"] = np.random.default_rng(0).normal(size=parts["W1"].shape)  # x is irrelevant when W_ih = 0
    parts["b2"] = np.arange(cfg["A"]) * 0.1
    w = wl.pack_weights(dims, parts)
    inp = wl.make_act_inputs(cfg)
    inp["reset"][:] = 0
    out = run_act(cfg, w, inp)
    np.testing.assert_array_equal(out["h_out"], inp["h_in"].astype(np.float64) * 0.5)  # r=z=1/2, n=0
    np.testing.assert_allclose(out["q"], np.broadcast_to(parts["b2"], out["q"].shape), atol=1e-7)
    # T+1 halvings from h_0 = 0 stay 0; Q = b2 at every slot
    u = wl.make_unroll_inputs(cfg)
    o = orc.unroll_td(dims, w, None, u["obs"], u["avail"], u["actions"], u["reward"], u["terminated"],
                      u["filled"], u["gamma"])
    np.testing.assert_allclose(o["q_all"], np.broadcast_to(parts["b2"], o["q_all"].shape), atol=1e-7)


def test_gru_update_gate_saturated_carries_or_replaces():
    cfg = small_cfg(D=8, H=8)
    dims = wl.dims(cfg)
    N, D, A, H = dims
    inp = wl.make_act_inputs(cfg)
    inp["reset"][:] = 0
    rnd = wl.unpack_weights(dims, wl.make_weights(cfg))
    # z = 1: h' = h whatever the rest of the weights are
    parts = {k: np.array(v) for k, v in rnd.items()}
    parts["b_ih"][H:2 * H] = 40.0
    out = run_act(cfg, wl.pack_weights(dims, parts), inp)
    np.testing.assert_allclose(out["h_out"], inp["h_in"], atol=1e-15)
    # z = 0, W_in = I, W1 = [I | 0], everything else 0: h' = tanh(relu(obs))
    parts = zero_parts(dims)
    parts["W1"][:, :D] = np.eye(H, D)
    parts["W_ih"][2 * H:3 * H] = np.eye(H)
    parts["b_ih"][H:2 * H] = -40.0
    out = run_act(cfg, wl.pack_weights(dims, parts), inp)
    np.testing.assert_allclose(out["h_out"], np.tanh(np.maximum(inp["obs"].astype(np.float64), 0)),
                               atol=1e-15)


def test_gru_reset_gate_paths():
    cfg = small_cfg(D=8, H=8)
    dims = wl.dims(cfg)
    N, D, A, H = dims
    inp = wl.make_act_inputs(cfg)
    inp["reset"][:] = 0
    parts = zero_parts(dims)
    parts["W1"][:, :D] = np.eye(H, D)                  # x = relu(obs) = obs
    parts["W_ih"][2 * H:] = 0.5 * np.eye(H)            # gi_n = x / 2
    parts["W_hh"][2 * H:] = 2.0 * np.eye(H)            # gh_n = 2 h + 0.25
    parts["b_hh"][2 * H:] = 0.25
    parts["b_ih"][H:2 * H] = -40.0                     # z = 0 -> h' = n
    x = inp["obs"].astype(np.float64)
    h = inp["h_in"].astype(np.float64)
    parts["b_ih"][:H] = -40.0                          # r = 0: the hidden term drops out
    out = run_act(cfg, wl.pack_weights(dims, parts), inp)
    np.testing.assert_allclose(out["h_out"], np.tanh(0.5 * x), atol=1e-15)
    parts["b_ih"][:H] = 40.0                           # r = 1: full hidden term, including b_hn
    out = run_act(cfg, wl.pack_weights(dims, parts), inp)
    np.testing.assert_allclose(out["h_out"], np.tanh(0.5 * x + 2.0 * h + 0.25), atol=1e-14)
    parts["b_ih"][:H] = 0.0                            # r = sigma(W_hr h): uses the hidden state, not x
    parts["W_hh"][:H] = 3.0 * np.eye(H)
    r = 1.0 / (1.0 + np.exp(-3.0 * h))
    out = run_act(cfg, wl.pack_weights(dims, parts), inp)
    np.testing.assert_allclose(out["h_out"], np.tanh(0.5 * x + r * (2.0 * h + 0.25)), atol=1e-14)


def test_scalar_gru_by_hand():
    # H = 1, D = 1, N = 1, A = 1: every weight is a scalar, evaluated by the textbook formulas.
    dims = (1, 1, 1, 1)
    vals = dict(W1=[[0.7, -0.2]], b1=[0.1], W_ih=[[0.3], [-0.4], [0.9]], W_hh=[[0.5], [0.6], [-0.8]],
                b_ih=[0.01, 0.02, 0.03], b_hh=[-0.04, 0.05, -0.06], W2=[[1.5]], b2=[-0.25])
    w = wl.pack_weights(dims, {k: np.array(v) for k, v in vals.items()})
    obs, h = 0.8, -0.3
    out = orc.act_step(dims, w, np.full((1, 1, 1), obs, np.float32), np.ones((1, 1, 1), np.uint8),
                       np.full((1, 1, 1), h), None, np.zeros(1, np.int32), 0.0, 1)
    f = lambda v: float(np.float32(v))
    x = max(0.0, f(0.7) * f(obs) + f(-0.2) * 1.0 + f(0.1))
    sg = lambda v: 1.0 / (1.0 + np.exp(-v))
    r = sg(f(0.3) * x + f(0.01) + f(0.5) * h + f(-0.04))
    z = sg(f(-0.4) * x + f(0.02) + f(0.6) * h + f(0.05))
    n = np.tanh(f(0.9) * x + f(0.03) + r * (f(-0.8) * h + f(-0.06)))
    hn = (1 - z) * n + z * h
    assert abs(out["h_out"][0, 0, 0] - hn) < 1e-15
    assert abs(out["q"][0, 0, 0] - (f(1.5) * hn + f(-0.25))) < 1e-15


def test_fc1_agent_id_column_and_reset_flag():
    cfg = small_cfg(D=8, H=8)
    dims = wl.dims(cfg)
    N, D, A, H = dims
    inp = wl.make_act_inputs(cfg)
    parts = zero_parts(dims)
    parts["W1"][:, D:] = np.arange(H * N).reshape(H, N) / 10.0 - 0.6   # only the id columns
    parts["b1"][:] = 0.05
    parts["W_ih"][2 * H:] = np.eye(H)
    parts["b_ih"][H:2 * H] = -40.0                                      # h' = tanh(x)
    out = run_act(cfg, wl.pack_weights(dims, parts), inp)
    for n in range(N):
        x = np.maximum(np.float32(parts["W1"][:, D + n]).astype(np.float64) + float(np.float32(0.05)), 0)
        np.testing.assert_allclose(out["h_out"][:, n], np.broadcast_to(np.tanh(x), (cfg["E"], H)), atol=1e-15)
    # reset[e] = 1 means h_in is treated as zero: with z = 1 (carry) the output is h or 0
    parts = zero_parts(dims)
    parts["b_ih"][H:2 * H] = 40.0
    inp["reset"][:] = [1, 0, 1, 0]
    out = run_act(cfg, wl.pack_weights(dims, parts), inp)
    keep = (1 - inp["reset"])[:, None, None]
    np.testing.assert_allclose(out["h_out"], inp["h_in"] * keep, atol=1e-15)


# ---------------------------------------------------------------- mask / argmax / epsilon-greedy
def q_equals_b2_net(cfg, b2):
    parts = zero_parts(wl.dims(cfg))
    parts["b2"] = np.asarray(b2, np.float64)
    return wl.pack_weights(wl.dims(cfg), parts)


def test_masked_argmax_lowest_index_on_ties_and_never_unavailable():
    cfg = small_cfg(A=6)
    w = q_equals_b2_net(cfg, [0.1, 0.9, 0.3, 0.9, -1.0, 0.9])
    inp = wl.make_act_inputs(cfg, E=64)
    for eps in (0.0, 0.3, 1.0):
        out = run_act(cfg, w, inp, epsilon=eps)
        chosen_avail = np.take_along_axis(inp["avail"], out["action"][..., None].astype(np.int64), -1)
        assert chosen_avail.all()
    out = run_act(cfg, w, inp, epsilon=0.0)
    av = inp["avail"].astype(bool)
    expect = np.where(av[..., 1], 1, np.where(av[..., 3], 3, np.where(av[..., 5], 5,
             np.where(av[..., 2], 2, 0))))                                 # action 0 is always available
    np.testing.assert_array_equal(out["action"], expect)
    # permuting the action columns permutes the choice (no ties)
    b2 = np.array([0.1, 0.9, 0.3, 0.7, -1.0, 0.5])
    perm = np.array([3, 0, 5, 1, 4, 2])
    a0 = run_act(cfg, q_equals_b2_net(cfg, b2), inp, epsilon=0.0)["action"]
    a1 = run_act(cfg, q_equals_b2_net(cfg, b2[perm]), inp, epsilon=0.0,
                 avail=inp["avail"][..., perm])["action"]
    np.testing.assert_array_equal(perm[a1], a0)
    # no action available: defined fallback is action 0
    none = np.zeros_like(inp["avail"])
    for eps in (0.0, 1.0):
        assert (run_act(cfg, w, inp, epsilon=eps, avail=none)["action"] == 0).all()


def test_epsilon_greedy_statistics_and_determinism():
    cfg = small_cfg(N=4, D=2, A=6, H=2)
    w = q_equals_b2_net(cfg, [0.0, 0.1, 0.2, 0.3, 0.4, 0.5])
    E = 50000
    inp = wl.make_act_inputs(cfg, E=E)
    inp["step_t"][:] = np.arange(E) % 7
    # epsilon = 1: uniform over the available actions, for every count c of available actions
    out = run_act(cfg, w, inp, epsilon=1.0)
    assert out["explored"].all()
    av = inp["avail"].reshape(-1, 6)
    act = out["action"].reshape(-1)
    assert av[np.arange(act.size), act].all()
    cnt = av.sum(-1)
    rank = (np.cumsum(av, -1) - 1)[np.arange(act.size), act]            # which of the c available ones
    for c in range(2, 7):
        sel = cnt == c
        hist = np.bincount(rank[sel], minlength=c).astype(np.float64)
        n = hist.sum()
        assert n > 2000
        chi2 = ((hist - n / c) ** 2 / (n / c)).sum()
        assert chi2 < 30.0, (c, hist)                                    # p < 1e-4 for up to 5 dof
    # epsilon = 0.05: explore rate inside a 5-sigma binomial band; greedy otherwise
    out = run_act(cfg, w, inp, epsilon=0.05)
    n = out["explored"].size
    rate = out["explored"].mean()
    assert abs(rate - 0.05) < 5 * np.sqrt(0.05 * 0.95 / n)
    keep = out["explored"] == 0
    np.testing.assert_array_equal(out["action"][keep], out["greedy"][keep])
    assert (out["greedy"] == np.where(inp["avail"] != 0, np.arange(6), -1).max(-1)).all()
    # the draw depends only on (seed, env, agent, step): a sub-batch of the first envs agrees
    sub = {k: (v[:100] if isinstance(v, np.ndarray) else v) for k, v in inp.items()}
    out_sub = run_act(cfg, w, sub, epsilon=0.5)
    out_all = run_act(cfg, w, inp, epsilon=0.5)
    np.testing.assert_array_equal(out_sub["action"], out_all["action"][:100])
    # and changes with seed and with step
    assert (run_act(cfg, w, inp, epsilon=1.0, seed=inp["seed"] + 1)["action"] != out_all["action"]).any()
    other_t = run_act(cfg, w, inp, epsilon=1.0, step_t=inp["step_t"] + 1)["action"]
    assert (other_t != run_act(cfg, w, inp, epsilon=1.0)["action"]).any()


def test_uniform_threshold_is_24_bit_fp32():
    # explore iff (r1 >> 40) * 2^-24 < epsilon, compared in fp32
    cfg = small_cfg(N=2, D=2, A=4, H=2)
    w = q_equals_b2_net(cfg, [0.0, 0.1, 0.2, 0.3])
    inp = wl.make_act_inputs(cfg, E=2000)
    eps = 0.37
    out = run_act(cfg, w, inp, epsilon=eps)
    for e in range(0, 2000, 97):
        for n in range(2):
            r1, _ = orc.rng_draw(inp["seed"], e, n, int(inp["step_t"][e]))
            u = np.float32(r1 >> 40) * np.float32(2.0 ** -24)
            assert bool(out["explored"][e, n]) == bool(u < np.float32(eps))


# ---------------------------------------------------------------- TD targets on hand-set Q
def test_td_brute_force_tiny_hand_set_q():
    cfg = small_cfg(N=2, D=3, A=3, H=4)
    dims = wl.dims(cfg)
    b2 = np.array([0.5, -1.0, 2.0])
    w = q_equals_b2_net(cfg, b2)
    B, T, N, A = 2, 3, 2, 3
    obs = np.zeros((B, T + 1, N, 3), np.float32)
    avail = np.array([[[[1, 1, 1], [1, 1, 0]], [[1, 0, 0], [1, 1, 1]], [[1, 1, 0], [0, 1, 0]], [[1, 0, 1], [1, 1, 0]]],
                      [[[1, 1, 1], [1, 1, 1]], [[0, 1, 0], [1, 0, 1]], [[1, 1, 1], [1, 0, 0]], [[1, 0, 0], [1, 0, 0]]]],
                     np.uint8)
    actions = np.array([[[2, 1], [0, 2], [1, 1]], [[0, 0], [1, 2], [2, 0]]], np.int32)
    reward = np.array([[1.0, -2.0, 0.5], [0.25, 3.0, 7.0]], np.float32)
    terminated = np.array([[0, 0, 1], [0, 1, 0]], np.uint8)
    filled = np.array([[1, 1, 1], [1, 1, 0]], np.uint8)
    g = np.float32(0.9)
    o = orc.unroll_td(dims, w, None, obs, avail, actions, reward, terminated, filled, g)
    gd = float(g)
    # next-step maxima over available actions, written out by hand from avail[:, t+1] and b2
    nm = np.array([[[0.5, 2.0], [0.5, -1.0], [2.0, 0.5]], [[-1.0, 2.0], [2.0, 0.5], [0.5, 0.5]]])
    exp_q = b2[actions].astype(np.float64)
    exp_y = reward[..., None].astype(np.float64) + gd * (1.0 - terminated[..., None]) * nm
    f = filled[..., None].astype(np.float64)
    np.testing.assert_allclose(o["q_taken"], f * exp_q, atol=1e-12)
    np.testing.assert_allclose(o["next_max"], f * nm, atol=1e-12)
    np.testing.assert_allclose(o["td_target"], f * exp_y, atol=1e-12)
    assert (o["td_target"][1, 2] == 0.0).all() and (o["q_taken"][1, 2] == 0.0).all()   # padded step
    np.testing.assert_allclose(o["td_target"][0, 2], reward[0, 2], atol=1e-12)          # terminated: y = r
    o0 = orc.unroll_td(dims, w, None, obs, avail, actions, reward, terminated, filled, 0.0)
    np.testing.assert_allclose(o0["td_target"], np.broadcast_to(f * reward[..., None], (B, T, N)), atol=1e-12)       # gamma = 0: y = r
    # nothing available at t+1: bootstrap value defined as 0
    avail2 = avail.copy(); avail2[0, 1, 0] = 0
    o2 = orc.unroll_td(dims, w, None, obs, avail2, actions, reward, terminated, filled, g)
    assert o2["next_max"][0, 0, 0] == 0.0 and abs(o2["td_target"][0, 0, 0] - 1.0) < 1e-12


# ---------------------------------------------------------------- structure
def test_act_iterated_equals_unroll():
    cfg = wl.config(0)
    dims = wl.dims(cfg)
    w = wl.make_weights(cfg)
    u = wl.make_unroll_inputs(cfg, B=3, T=10)
    o = orc.unroll_td(dims, w, None, u["obs"], u["avail"], u["actions"], u["reward"], u["terminated"],
                      u["filled"], u["gamma"])
    h = np.zeros((3, cfg["N"], cfg["H"]))
    for t in range(11):
        a = orc.act_step(dims, w, u["obs"][:, t], u["avail"][:, t], h, np.full(3, t == 0, np.uint8),
                         np.full(3, t, np.int32), 0.0, 5)
        h = a["h_out"]
        np.testing.assert_allclose(a["q"], o["q_all"][:, t], atol=1e-13)


def test_environments_and_agents_are_isolated():
    cfg = wl.config(0)
    w = wl.make_weights(cfg)
    inp = wl.make_act_inputs(cfg)
    base = run_act(cfg, w, inp)
    mod = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in inp.items()}
    mod["obs"][2] += 1.0
    mod["h_in"][2] *= -1.0
    mod["reset"][2] = 0
    out = run_act(cfg, w, mod)
    others = [e for e in range(cfg["E"]) if e != 2]
    for k in ("h_out", "q", "action"):
        np.testing.assert_array_equal(out[k][others], base[k][others])
    assert (out["q"][2] != base["q"][2]).any()
    # permuting environments permutes Q and hidden state
    perm = np.random.default_rng(3).permutation(cfg["E"])
    pin = {k: (v[perm] if isinstance(v, np.ndarray) else v) for k, v in inp.items()}
    pout = run_act(cfg, w, pin)
    np.testing.assert_array_equal(pout["q"], base["q"][perm])
    np.testing.assert_array_equal(pout["h_out"], base["h_out"][perm])


def test_row_subset_and_thread_count_do_not_change_values():
    cfg = wl.config(0)
    dims = wl.dims(cfg)
    w0, w1 = wl.make_weights(cfg, 0), wl.make_weights(cfg, 1)
    u = wl.make_unroll_inputs(cfg, B=4, T=9)
    args = (dims, w0, w1, u["obs"], u["avail"], u["actions"], u["reward"], u["terminated"], u["filled"], u["gamma"])
    full = orc.unroll_td(*args, nthreads=1)
    par = orc.unroll_td(*args, nthreads=4)
    rows = np.array([1, 7, 10], np.int32)
    part = orc.unroll_td(*args, rows=rows)
    N = cfg["N"]
    for k in ("q_taken", "next_max", "td_target"):
        np.testing.assert_array_equal(full[k], par[k])
        for r in rows:
            np.testing.assert_array_equal(part[k][r // N, :, r % N], full[k][r // N, :, r % N])
        assert np.isnan(part[k][0, :, 0]).all()


def test_generator_shapes_match_scenario_table():
    # Table 2: (actions, agents, obs, limit) = 3m (9,3,30,60), 8m (14,8,80,120), 5m_vs_6m (12,5,55,70)
    for ci, (A, N, D, T) in {0: (9, 3, 30, 60), 1: (14, 8, 80, 120), 3: (12, 5, 55, 70)}.items():
        c = wl.config(ci)
        assert (c["A"], c["N"], c["D"], c["T"]) == (A, N, D, T)
    c = wl.config(2)
    assert (c["A"], c["N"], c["T"]) == (11, 5, 120)
    for ci in range(3):
        c = wl.config(ci)
        u = wl.make_unroll_inputs(c, B=5)
        assert u["avail"][..., 0].all()
        L = u["lengths"]
        assert (u["filled"].sum(1) == L).all()
        assert (np.take_along_axis(u["avail"][:, :c["T"]], u["actions"][..., None].astype(np.int64), -1) == 1).all()
        assert orc.param_count(*wl.dims(c)) == wl.param_count(*wl.dims(c)) == wl.make_weights(c).size


# ---------------------------------------------------------------- double-estimator target
def _double(cfg, w_on, w_tg, inp):
    return orc.unroll_td_double(wl.dims(cfg), w_on, w_tg, inp["obs"], inp["avail"], inp["actions"], inp["reward"],
                                inp["terminated"], inp["filled"], inp["gamma"])


def test_double_target_brute_force_from_library_q():
    """Pick with the online network's library Q, value with the target's, written out in loops."""
    cfg = wl.config(0)
    dims = wl.dims(cfg)
    N, D, A, H = dims
    w_on, w_tg = wl.make_weights(cfg, 0), wl.make_weights(cfg, 1)
    B, T = 3, 12
    inp = wl.make_unroll_inputs(cfg, B=B, T=T)
    out = _double(cfg, w_on, w_tg, inp)
    qs = {}
    for key, w in (("on", w_on), ("tg", w_tg)):
        step = torch_net(dims, w)
        h = torch.zeros(B, N, H, dtype=torch.float64)
        q_t = []
        for t in range(T + 1):
            h, q = step(inp["obs"][:, t], h)
            q_t.append(q.numpy())
        qs[key] = np.stack(q_t, 1)
    g = float(np.float32(inp["gamma"]))
    differs = 0
    for b in range(B):
        for t in range(T):
            for n in range(N):
                f = float(inp["filled"][b, t])
                allowed = [a for a in range(A) if inp["avail"][b, t + 1, n, a]]
                pick = max(allowed, key=lambda a: (qs["on"][b, t + 1, n, a], -a))
                value = qs["tg"][b, t + 1, n, pick]
                differs += value != max(qs["tg"][b, t + 1, n, a] for a in allowed)
                y = float(inp["reward"][b, t]) + g * (1.0 - float(inp["terminated"][b, t])) * value
                assert out["next_action"][b, t, n] == pick
                assert abs(out["next_max"][b, t, n] - f * value) < 1e-12
                assert abs(out["td_target"][b, t, n] - f * y) < 1e-12
                assert abs(out["q_taken"][b, t, n] - f * qs["on"][b, t, n, inp["actions"][b, t, n]]) < 1e-12
    assert differs > 0, "the case must tell the two estimators apart"
    np.testing.assert_allclose(out["q_all"], qs["on"], rtol=0, atol=1e-12)


def test_double_target_reduces_to_plain_target_when_networks_coincide():
    cfg = wl.config(1)
    dims = wl.dims(cfg)
    w = wl.make_weights(cfg, 0)
    inp = wl.make_unroll_inputs(cfg, B=2, T=9)
    plain = orc.unroll_td(dims, w, None, inp["obs"], inp["avail"], inp["actions"], inp["reward"],
                          inp["terminated"], inp["filled"], inp["gamma"])
    both = _double(cfg, w, None, inp)
    for k in ("q_taken", "next_max", "td_target"):
        np.testing.assert_array_equal(both[k], plain[k])
    # and never above the plain target's bootstrap when the networks differ (max is an upper bound)
    w2 = wl.make_weights(cfg, 1)
    plain2 = orc.unroll_td(dims, w, w2, inp["obs"], inp["avail"], inp["actions"], inp["reward"],
                           inp["terminated"], inp["filled"], inp["gamma"])
    both2 = _double(cfg, w, w2, inp)
    assert (both2["next_max"] <= plain2["next_max"] + 1e-15).all()
    assert (both2["next_max"] < plain2["next_max"]).any()


def test_double_target_hand_set_q_ties_and_masks():
    """Q = b2 for both networks: the online b2 decides the index, the target b2 gives the value."""
    cfg = small_cfg(N=2, D=3, A=4, H=4)
    dims = wl.dims(cfg)
    parts_on, parts_tg = zero_parts(dims), zero_parts(dims)
    parts_on["b2"] = np.array([1.0, 3.0, 3.0, 2.0])          # tie between actions 1 and 2: lowest index
    parts_tg["b2"] = np.array([10.0, 20.0, 30.0, 40.0])
    w_on, w_tg = wl.pack_weights(dims, parts_on), wl.pack_weights(dims, parts_tg)
    B, T = 1, 3
    inp = wl.make_unroll_inputs(cfg, B=B, T=T)
    inp["avail"][:] = 1
    inp["avail"][0, 2, 0, 1] = 0                             # agent 0 at slot 2: action 1 unavailable -> 2
    inp["avail"][0, 3, 1, 1:3] = 0                           # agent 1 at slot 3: only {0, 3} -> 3
    inp["filled"][:] = 1
    inp["terminated"][:] = 0
    inp["terminated"][0, 2] = 1
    inp["reward"][:] = np.array([[0.5, -1.0, 2.0]], np.float32)
    out = _double(cfg, w_on, w_tg, inp)
    np.testing.assert_array_equal(out["next_action"][0], [[1, 1], [2, 1], [1, 3]])
    np.testing.assert_array_equal(out["next_max"][0], [[20.0, 20.0], [30.0, 20.0], [20.0, 40.0]])
    g = float(np.float32(inp["gamma"]))
    expect = np.array([[0.5 + g * 20, 0.5 + g * 20], [-1 + g * 30, -1 + g * 20], [2.0, 2.0]])
    np.testing.assert_allclose(out["td_target"][0], expect, rtol=0, atol=1e-12)
