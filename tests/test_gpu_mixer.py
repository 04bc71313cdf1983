"""GPU parity of the mixing network (include/marl_mixer.h) against its oracle, through the C ABI,
element by element on the same seeded inputs.

Tolerance: Q_total is a sum of M products w2 * elu(.) whose magnitude grows with the number of
agents (values up to a few tens on the scale-up workload), so the bound is stated relative to
the largest reference value of the case: max |gpu - oracle| <= tol * max(1, max |oracle|), with
tol = 1e-4 for fp32 parameters (bf16 value + remainder products, fp32 accumulation) and 2e-2 for
bf16 parameters, the same figures the Q-network is held to."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from oracle import marl_oracle as orc, mixer_oracle as mxo
from paper_2205_05248_amd import binding, workloads as wl

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def oracle_mixer_weights(dims, w, dtype):
    """bf16 mixers compute on the four state matrices rounded to bf16 (by the oracle's own rounding)."""
    if dtype != "bf16":
        return w
    out = np.array(w, np.float32)
    for name, (a, b, shp) in wl.mixer_slices(*dims).items():
        if len(shp) == 2:
            out[a:b] = orc.round_bf16(out[a:b])
    return out


def gpu_td(online, target, m, outputs=("q_total", "y_total", "td_err")):
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    B, T = m["reward"].shape
    out = {k: (torch.full((B, T), float("nan"), device="cuda") if k in outputs else None)
           for k in ("q_total", "y_total", "td_err")}
    out["loss"] = torch.full((2,), float("nan"), device="cuda") if "td_err" in outputs else None
    online.td(target, dev(m["state"]), dev(m["q_taken"]), dev(m["next_max"]), dev(m["reward"]), dev(m["terminated"]),
              dev(m["filled"]), m["gamma"], out["q_total"], out["y_total"], out["td_err"], out["loss"])
    torch.cuda.synchronize()
    return {k: (None if v is None else v.cpu().numpy()) for k, v in out.items()}


def check(got, ref, tol):
    worst = 0.0
    for k in ("q_total", "y_total", "td_err"):
        if got[k] is None:
            continue
        assert np.isfinite(got[k]).all(), k
        scale = max(1.0, float(np.abs(ref[k]).max()))
        err = float(np.abs(got[k] - ref[k]).max()) / scale
        assert err <= tol, f"{k}: max error {err:.3g} of scale {scale:.3g}"
        worst = max(worst, err)
    if got.get("loss") is not None and "loss" in ref:
        # sum of squares: each term carries twice the relative error of its td_err, fp32 summation on top
        scale = max(1.0, float(np.abs(ref["td_err"]).max()))
        assert got["loss"][1] == ref["loss"][1], "filled count"
        assert abs(got["loss"][0] - ref["loss"][0]) <= 4 * tol * scale * max(1.0, float(np.abs(ref["td_err"]).sum())), "loss sum"
    return worst


def run_case(cfg, dtype, B=None, T=None, distinct=True, stream=0):
    dims = wl.mixer_dims(cfg)
    w_on, w_tg = wl.make_mixer_weights(cfg, 0), wl.make_mixer_weights(cfg, 1)
    online = binding.Mixer(dims, w_on, dtype)
    target = binding.Mixer(dims, w_tg, dtype) if distinct else None
    m = wl.make_mixer_inputs(cfg, B=B, T=T, stream=stream)
    got = gpu_td(online, target, m)
    ref = mxo.td(dims, oracle_mixer_weights(dims, w_on, dtype), oracle_mixer_weights(dims, w_tg, dtype) if distinct else None,
                 m["state"], m["q_taken"], m["next_max"], m["reward"], m["terminated"], m["filled"], m["gamma"])
    worst = check(got, ref, TOL[dtype])
    online.close()
    if target is not None:
        target.close()
    return worst


@pytest.mark.parametrize("ci", [0, 1, 2, 3])
def test_mixer_paper_scenarios(ci):
    """The four scenarios' agent counts, state sizes (Table 2) and time-step limits, whole batch."""
    cfg = wl.config(ci)
    run_case(cfg, cfg["dtype"], B=min(cfg["B"], 32))


def test_mixer_scaleup_reduced_batch_both_dtypes():
    cfg = wl.config(4)
    run_case(cfg, "bf16", B=6)
    run_case(dict(cfg, S=512), "fp32", B=3)


def test_mixer_scaleup_full_size_every_transition():
    """The bench's launch configuration (B = 64, T = 200, 32 agents, state 512, bf16): all 12,800 transitions
    against the oracle (which takes them one by one), plus the identities that tie the outputs together."""
    cfg = wl.config(4)
    dims = wl.mixer_dims(cfg)
    w_on, w_tg = wl.make_mixer_weights(cfg, 0), wl.make_mixer_weights(cfg, 1)
    online, target = binding.Mixer(dims, w_on, "bf16"), binding.Mixer(dims, w_tg, "bf16")
    m = wl.make_mixer_inputs(cfg)
    got = gpu_td(online, target, m)
    ref = mxo.td(dims, oracle_mixer_weights(dims, w_on, "bf16"), oracle_mixer_weights(dims, w_tg, "bf16"), m["state"],
                 m["q_taken"], m["next_max"], m["reward"], m["terminated"], m["filled"], m["gamma"])
    scale = max(1.0, np.abs(ref["q_total"]).max(), np.abs(ref["y_total"]).max())
    for k in ("q_total", "y_total", "td_err"):
        assert np.isfinite(got[k]).all()
        err = np.abs(got[k] - ref[k]).max()
        assert err <= TOL["bf16"] * scale, f"max |{k} - oracle| = {err} against scale {scale}"
    assert (got["td_err"][m["filled"] == 0] == 0).all()
    np.testing.assert_array_equal(got["y_total"][m["terminated"] != 0], m["reward"][m["terminated"] != 0])
    np.testing.assert_allclose(got["td_err"], (got["y_total"] - got["q_total"]) * m["filled"], atol=1e-5)
    online.close(); target.close()


SHAPES = [
    # N, M, S, dtype, B, T
    (1, 16, 1, "fp32", 1, 1),            # the smallest of everything: one transition
    (2, 16, 31, "fp32", 3, 5),           # one partial k-step, 15 transitions: less than a tile
    (3, 32, 32, "bf16", 1, 16),          # exactly one tile, one full k-step
    (5, 64, 33, "fp32", 13, 5),          # one value past a k-step, 65 transitions: one past a workgroup
    (64, 32, 98, "bf16", 2, 40),         # the most agents
    (4, 32, 512, "fp32", 2, 9),          # the largest fp32 state
    (4, 16, 1024, "bf16", 2, 9),         # the largest bf16 state
    (7, 64, 257, "bf16", 5, 27),
    (3, 32, 256, "fp32", 129, 64),       # 8256 transitions of two-plane operands: workgroups of eight waves, the last one ragged
    (6, 16, 300, "bf16", 70, 120),       # the same with one plane and a padded state
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "N%d_M%d_S%d_%s_B%d_T%d" % s)
def test_mixer_shapes_at_the_edges(shape):
    N, M, S, dtype, B, T = shape
    cfg = dict(wl.config(0), N=N, S=S, B=B, T=T, lengths="uniform_all")
    dims = (N, M, S)
    w_on, w_tg = (wl.pack_mixer(dims, {k: np.random.default_rng([9, s, i]).uniform(-1, 1, shp) / np.sqrt(max(shp[-1], 1) if len(shp) == 2 else 4)
                                      for i, (k, (_, _, shp)) in enumerate(wl.mixer_slices(*dims).items())}) for s in (0, 1))
    online, target = binding.Mixer(dims, w_on, dtype), binding.Mixer(dims, w_tg, dtype)
    m = wl.make_mixer_inputs(cfg)
    got = gpu_td(online, target, m)
    ref = mxo.td(dims, oracle_mixer_weights(dims, w_on, dtype), oracle_mixer_weights(dims, w_tg, dtype), m["state"],
                 m["q_taken"], m["next_max"], m["reward"], m["terminated"], m["filled"], m["gamma"])
    check(got, ref, TOL[dtype])
    online.close(); target.close()


def test_mixer_target_defaults_to_online_and_outputs_are_optional():
    cfg = dict(wl.config(1), B=4, T=11)
    run_case(cfg, "fp32", distinct=False)
    dims = wl.mixer_dims(cfg)
    w = wl.make_mixer_weights(cfg)
    mixer = binding.Mixer(dims, w, "fp32")
    m = wl.make_mixer_inputs(cfg)
    only = gpu_td(mixer, None, m, outputs=("td_err",))
    full = gpu_td(mixer, mixer, m)
    np.testing.assert_array_equal(only["td_err"], full["td_err"])
    assert only["q_total"] is None
    other = binding.Mixer((dims[0], 16, dims[2]), wl.pack_mixer((dims[0], 16, dims[2]), {k: np.zeros(s) for k, (_, _, s) in wl.mixer_slices(dims[0], 16, dims[2]).items()}), "fp32")
    with pytest.raises(binding.MarlError) as err:
        gpu_td(mixer, other, m)
    assert err.value.status == -4                     # MARL_ERR_MISMATCH
    mixer.close(); other.close()


def test_mixer_is_monotone_on_the_device():
    """The defining property, checked on the kernel's own outputs: raising one agent's value never
    lowers Q_total (beyond rounding)."""
    cfg = dict(wl.config(3), B=8, T=20)
    dims = wl.mixer_dims(cfg)
    mixer = binding.Mixer(dims, wl.make_mixer_weights(cfg), "fp32")
    m = wl.make_mixer_inputs(cfg)
    base = gpu_td(mixer, None, m)["q_total"]
    for n in range(dims[0]):
        up = dict(m, q_taken=m["q_taken"].copy())
        up["q_taken"][..., n] += 1.5
        assert (gpu_td(mixer, None, up)["q_total"] >= base - 1e-4).all()
    mixer.close()


def test_mixer_set_weights_is_ordered_on_the_stream():
    """Parameters replaced in place, with no synchronisation in between: a call enqueued before the
    refresh sees the old mixer, calls after it the new one (the offset constant included, which is
    part of the uploaded image); a second refresh right behind the first does not disturb it."""
    cfg = dict(wl.config(2), B=6, T=13)
    dims = wl.mixer_dims(cfg)
    w0, w1, w2 = (wl.make_mixer_weights(cfg, s) for s in (0, 1, 2))
    for w in (w1, w2):
        w[-1] += 3.0                                # c2: a visible change of the constant
    mixer = binding.Mixer(dims, w0, "fp32")
    m = wl.make_mixer_inputs(cfg)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    d = {k: dev(m[k]) for k in ("state", "q_taken", "next_max", "reward", "terminated", "filled")}
    outs = []
    for w in (None, w1, w2):
        if w is not None:
            mixer.set_weights(w)
        o = [torch.empty(cfg["B"], cfg["T"], device="cuda") for _ in range(3)]
        mixer.td(None, d["state"], d["q_taken"], d["next_max"], d["reward"], d["terminated"], d["filled"], m["gamma"], *o)
        outs.append(o)
    torch.cuda.synchronize()
    for o, w in zip(outs, (w0, w1, w2)):
        ref = mxo.td(dims, w, None, m["state"], m["q_taken"], m["next_max"], m["reward"], m["terminated"], m["filled"], m["gamma"])
        check({k: t.cpu().numpy() for k, t in zip(("q_total", "y_total", "td_err"), o)}, ref, TOL["fp32"])
    with pytest.raises(binding.MarlError):
        mixer.set_weights(w0[:-1])
    mixer.close()


# ------------------------------------------------------------------ backward pass
GRAD_REL = {"fp32": 1e-3, "bf16": 3e-2}
# Half-width of the band of generated quantities in which the two sides may set a switch (an absolute value, the
# offset's relu) differently: the forward error of such a quantity against fp64.  A bf16 mixer rounds every state
# entry to bf16 before its products; the switches are decisions, and both sides take a decision on the same
# values: the oracle runs in its bf16-input mode (its own rounding routine, pinned against a library cast).  What
# is left is rounding in sums over up to 512 state entries: products of two bf16 values are exact in fp32 and their
# fp32 sum is off by about 1e-6 at values of order one; fp32 mixers split each operand into two bf16 planes and
# drop the low-by-low product, 2^-17 of each product, up to 1e-5 over the sum.
SWITCH_BAND = {"fp32": 2e-5, "bf16": 3e-6}
# The ambiguity budget that band may claim, as a share of the tensor's largest reference value: a band wide
# enough to hide an error fails here.
BUDGET_CAP = 0.02


def _gpu_mixer_grad(mixer, dims, m, e):
    N, M, S = dims
    B, T = m["q_taken"].shape[:2]
    d = {k: torch.from_numpy(np.ascontiguousarray(m[k])).cuda() for k in ("state", "q_taken")}
    ws = torch.empty(mixer.grad_workspace_bytes(B, T), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    gq = torch.full((B, T, N), float("nan"), device="cuda")
    gw = torch.full((wl.mixer_param_count(*dims),), float("nan"), device="cuda")
    mixer.grad(d["state"], d["q_taken"], torch.from_numpy(e.astype(np.float32)).cuda(), ws, gq, gw)
    torch.cuda.synchronize()
    return gq.cpu().numpy(), gw.cpu().numpy()


@pytest.mark.parametrize("ci,B,T,dtype", [(0, 3, 7, "fp32"), (1, 5, 9, "fp32"), (2, 7, 12, "fp32"), (3, 33, 5, "fp32"),
                                          (4, 3, 11, "bf16"), (4, 2, 5, "fp32"), (1, 6, 8, "bf16"), (3, 1, 2, "fp32"), (2, 40, 33, "bf16")])
def test_mixer_gradient_matches_the_oracle(ci, B, T, dtype):
    """Every entry of every parameter tensor, and dL/dq, within REL of the tensor's largest reference value.
    The absolute values and the offset's relu are switches set by forward values: where a generated weight or an
    offset unit is within the forward error of zero (SWITCH_BAND) the two sides may set them differently, and the
    oracle's ambiguity budget for exactly those terms is added to the bar of the entries they reach (zero for
    dL/dq, v2, c2, Hb1, hbb1, which the test checks)."""
    cfg = dict(wl.config(ci), dtype=dtype)
    dims = wl.mixer_dims(cfg)
    w = wl.make_mixer_weights(cfg)
    m = wl.make_mixer_inputs(cfg, B=B, T=T)
    # dL/dQ_total as the loss hands it over: zero on padding transitions (whose state rows are all zero)
    e = np.random.default_rng(ci).normal(size=(B, T)).astype(np.float32) * m["filled"]
    _compare_mixer_gradient(cfg["name"], dims, w, dtype, m, e)


GRAD_SHAPES = [
    # N, M, S, dtype, B, T
    (1, 16, 1, "fp32", 1, 1),            # the smallest of everything: one transition
    (5, 64, 33, "fp32", 13, 5),          # one value past a k-step, 65 transitions: one past a workgroup of four waves
    (40, 64, 40, "bf16", 3, 30),         # 2752 generated quantities per transition
    (64, 16, 98, "fp32", 2, 40),         # the most agents
    (4, 32, 512, "fp32", 2, 9),          # the largest fp32 state: fragments of a block read as they are used
    (4, 16, 1024, "bf16", 2, 9),         # the largest bf16 state
    (6, 32, 300, "bf16", 70, 120),       # 8400 transitions: workgroups of eight waves, the last one ragged
    (3, 32, 256, "fp32", 129, 64),       # the same with two-plane operands, 8256 transitions
]


@pytest.mark.parametrize("shape", GRAD_SHAPES, ids=lambda s: "N%d_M%d_S%d_%s_B%d_T%d" % s)
def test_mixer_gradient_shapes_at_the_edges(shape):
    """The same comparison on shapes chosen for the kernel's own limits and workgroup shapes."""
    N, M, S, dtype, B, T = shape
    cfg = dict(wl.config(0), N=N, S=S, B=B, T=T)
    dims = (N, M, S)
    w = wl.pack_mixer(dims, {k: np.random.default_rng([11, i]).uniform(-1, 1, shp) / np.sqrt(max(shp[-1], 1) if len(shp) == 2 else 4)
                             for i, (k, (_, _, shp)) in enumerate(wl.mixer_slices(*dims).items())})
    m = wl.make_mixer_inputs(cfg)
    # an upstream gradient of one sign: the sums then grow with the number of transitions as the switches'
    # ambiguity budget does, and the budget stays a small share of them on the large batches too
    e = np.abs(np.random.default_rng([12, N, S]).normal(size=(B, T))).astype(np.float32) * m["filled"]
    _compare_mixer_gradient("N%d M%d S%d" % dims, dims, w, dtype, m, e)


def _compare_mixer_gradient(label, dims, w, dtype, m, e):
    mixer = binding.Mixer(dims, w, dtype)
    got_q, got_w = _gpu_mixer_grad(mixer, dims, m, e)
    w_ref = w
    if dtype == "bf16":
        from oracle import marl_oracle as orc
        w_ref = np.array(w, np.float32)
        for name, (a, b, shp) in wl.mixer_slices(*dims).items():
            if len(shp) == 2:
                w_ref[a:b] = orc.round_bf16(w_ref[a:b])
    want_q, want_w, amb = mxo.grad(dims, w_ref, m["state"], m["q_taken"].astype(np.float64), e.astype(np.float64),
                                   switch_band=SWITCH_BAND[dtype], inputs_as_bf16=dtype == "bf16")
    rel = GRAD_REL[dtype]
    assert np.isfinite(got_q).all() and np.isfinite(got_w).all()
    bad, worst = [], {}
    err_q = np.abs(got_q - want_q).max() / np.abs(want_q).max()
    worst["dq"] = err_q
    if err_q > rel:
        bad.append(("dq", err_q))
    for name, (a, b, _) in wl.mixer_slices(*dims).items():
        scale = np.abs(want_w[a:b]).max()
        diff = np.abs(got_w[a:b] - want_w[a:b])
        worst[name] = diff.max() / max(scale, 1e-30)
        if name in ("Hb1", "hbb1", "v2", "c2"):
            assert amb[a:b].max() == 0
        assert amb[a:b].max() <= BUDGET_CAP * max(scale, 1e-30), (name, amb[a:b].max() / max(scale, 1e-30))
        if (diff - (rel * scale + 1e-6 + amb[a:b])).max() > 0:
            bad.append((name, worst[name], amb[a:b].max() / max(scale, 1e-30)))
    print(label, dtype, {k: f"{v:.1e}" for k, v in worst.items()})
    assert not bad, bad
    again_q, again_w = _gpu_mixer_grad(mixer, dims, m, e)
    np.testing.assert_array_equal(again_w, got_w)
    np.testing.assert_array_equal(again_q, got_q)
    mixer.close()
