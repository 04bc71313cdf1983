"""Pins of the back-propagation oracle against things other than itself (CPU only): a tensor
library's automatic differentiation of a forward pass written here, central finite differences of
the forward oracle, closed forms, linearity."""
import numpy as np
import pytest
import torch

from oracle import bptt_oracle as bpo
from oracle import marl_oracle as orc
from paper_2205_05248_amd import workloads as wl


def case(ci=0, B=3, T=7, seed=3):
    cfg = wl.config(ci)
    dims = wl.dims(cfg)
    w = wl.make_weights(cfg, 0)
    u = wl.make_unroll_inputs(cfg, B=B, T=T)
    g = np.random.default_rng(seed).normal(size=(B, T, dims[0]))
    return cfg, dims, w, u, g


def autograd_grad(dims, w, u, g, relu_band=None):
    """sum(g * q_taken) differentiated by the library; the forward pass is written with its ops.
    relu_band: also the ambiguity budget of W1 and b1, from the library's adjoint of x."""
    N, D, A, H = dims
    wt = torch.tensor(np.asarray(w, np.float64), requires_grad=True)
    sl = wl.weight_slices(*dims)
    p = {k: wt[a:b].reshape(shp) for k, (a, b, shp) in sl.items()}
    obs = torch.from_numpy(u["obs"].astype(np.float64))
    B, T = u["actions"].shape[:2]
    eye = torch.eye(N, dtype=torch.float64).expand(B, N, N)
    h = torch.zeros(B, N, H, dtype=torch.float64)
    total = torch.zeros((), dtype=torch.float64)
    act = torch.from_numpy(u["actions"].astype(np.int64))
    f = torch.from_numpy(u["filled"].astype(np.float64))
    gt = torch.from_numpy(g)
    kept = []
    for t in range(T):
        x_in = torch.cat([obs[:, t], eye], -1)
        pre = x_in @ p["W1"].T + p["b1"]
        x = torch.relu(pre)
        x.retain_grad()
        kept.append((x_in, pre, x))
        gi = x @ p["W_ih"].T + p["b_ih"]
        gh = h @ p["W_hh"].T + p["b_hh"]
        r = torch.sigmoid(gi[..., :H] + gh[..., :H])
        z = torch.sigmoid(gi[..., H:2 * H] + gh[..., H:2 * H])
        nn = torch.tanh(gi[..., 2 * H:] + r * gh[..., 2 * H:])
        h = (1 - z) * nn + z * h
        q = h @ p["W2"].T + p["b2"]
        total = total + (gt[:, t] * f[:, t, None] * q.gather(-1, act[:, t, :, None])[..., 0]).sum()
    total.backward()
    if relu_band is None:
        return wt.grad.numpy()
    amb = np.zeros(wt.numel())
    a1, b1_, shp = sl["W1"]
    ab, bb, _ = sl["b1"]
    for x_in, pre, x in kept:
        near = (pre.detach().abs() <= relu_band).double()
        dx = x.grad.abs() * near                                       # [B, N, H]
        amb[ab:bb] += dx.sum((0, 1)).numpy()
        amb[a1:b1_] += torch.einsum("bnj,bnd->jd", dx, x_in.abs()).reshape(-1).numpy()
    return wt.grad.numpy(), amb


def test_bf16_input_mode_is_the_gradient_on_library_cast_observations():
    """The diagnostic mode rounds the observation entries, and nothing else, the way a library's bfloat16 cast
    does: its result is the library's gradient at the cast observations, not the one at the raw ones."""
    cfg, dims, w, u, g = case(1, B=2, T=5)
    cast = dict(u, obs=torch.from_numpy(u["obs"]).to(torch.bfloat16).to(torch.float32).numpy())
    assert (cast["obs"] != u["obs"]).any()
    got = bpo.qnet_grad(dims, w, u["obs"], u["actions"], u["filled"], g, inputs_as_bf16=True)
    want = autograd_grad(dims, w, cast, g)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-10 * max(1.0, np.abs(want).max()))
    raw = bpo.qnet_grad(dims, w, u["obs"], u["actions"], u["filled"], g)
    assert np.abs(raw - got).max() > 1e-6 * np.abs(raw).max()


@pytest.mark.parametrize("ci", [0, 1])
def test_gradient_matches_library_autodiff(ci):
    cfg, dims, w, u, g = case(ci)
    got = bpo.qnet_grad(dims, w, u["obs"], u["actions"], u["filled"], g)
    want = autograd_grad(dims, w, u, g)
    scale = np.abs(want).max()
    assert scale > 0
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-11 * max(1.0, scale))
    # every tensor of the network receives a gradient in this case
    for name, (a, b, _) in wl.weight_slices(*dims).items():
        assert np.abs(want[a:b]).max() > 0, name


def test_gradient_matches_finite_differences_of_the_forward_oracle():
    cfg, dims, w, u, g = case(0, B=2, T=5)
    got = bpo.qnet_grad(dims, w, u["obs"], u["actions"], u["filled"], g)

    def objective(wv):
        out = orc.unroll_td(dims, wv, None, u["obs"], u["avail"], u["actions"], u["reward"], u["terminated"],
                            u["filled"], u["gamma"], want_q_all=False)
        return float((g * out["q_taken"]).sum())

    rng = np.random.default_rng(0)
    for name, (a, b, _) in wl.weight_slices(*dims).items():
        for p in rng.choice(np.arange(a, b), size=3, replace=False):
            lo, hi = np.array(w), np.array(w)
            lo[p] = np.float32(w[p] - 2e-3)
            hi[p] = np.float32(w[p] + 2e-3)
            slope = (objective(hi) - objective(lo)) / (float(hi[p]) - float(lo[p]))
            assert abs(slope - got[p]) <= 1e-4 * max(1.0, abs(got[p])), (name, p, slope, got[p])


def test_closed_forms_output_layer_and_linearity():
    cfg, dims, w, u, g = case(1, B=2, T=6)
    N, D, A, H = dims
    sl = wl.weight_slices(*dims)
    got = bpo.qnet_grad(dims, w, u["obs"], u["actions"], u["filled"], g)
    # d/db2[a] = sum of g over the filled transitions whose action is a
    f = (u["filled"] != 0)[..., None]
    want_b2 = np.array([(g * f * (u["actions"] == a)).sum() for a in range(A)])
    a0, b0, _ = sl["b2"]
    np.testing.assert_allclose(got[a0:b0], want_b2, rtol=0, atol=1e-12)
    # linear in g, and unfilled transitions carry nothing
    other = np.random.default_rng(9).normal(size=g.shape)
    both = bpo.qnet_grad(dims, w, u["obs"], u["actions"], u["filled"], 2.0 * g - 3.0 * other)
    sep = 2.0 * got - 3.0 * bpo.qnet_grad(dims, w, u["obs"], u["actions"], u["filled"], other)
    np.testing.assert_allclose(both, sep, rtol=0, atol=1e-10 * max(1.0, np.abs(sep).max()))
    masked = np.where(f, g, 1e6)
    np.testing.assert_array_equal(bpo.qnet_grad(dims, w, u["obs"], u["actions"], u["filled"], masked), got)
    # thread count does not change the rows' values, only the order of the final sum
    one = bpo.qnet_grad(dims, w, u["obs"], u["actions"], u["filled"], g, nthreads=1)
    np.testing.assert_allclose(one, got, rtol=0, atol=1e-12 * max(1.0, np.abs(got).max()))


def test_one_step_scalar_network_by_hand():
    """N = 1, D = 1, A = 1, H = 1, T = 1: every derivative written out."""
    dims = (1, 1, 1, 1)
    # W1 = [w_o, w_id], b1, W_ih = [wr, wz, wn], W_hh = [ur, uz, un], b_ih, b_hh, W2, b2
    w = np.array([0.7, 0.2, 0.1, 0.5, -0.4, 0.9, 0.3, 0.6, -0.8, 0.05, -0.1, 0.2, 0.15, 0.25, -0.3, 1.3, 0.4], np.float32)
    assert w.size == bpo._load().bptt_param_count(1, 1, 1, 1)
    o = np.float32(1.5)
    obs = np.array([o, 0.0], np.float32).reshape(1, 2, 1, 1)
    got = bpo.qnet_grad(dims, w, obs, np.zeros((1, 1, 1), np.int32), np.ones((1, 1), np.uint8), np.full((1, 1, 1), 2.0))
    W = [float(v) for v in w]
    x = max(0.0, W[0] * float(o) + W[1] + W[2])
    sig = lambda v: 1.0 / (1.0 + np.exp(-v))
    r = sig(W[3] * x + W[9] + W[12]); z = sig(W[4] * x + W[10] + W[13])
    ghn = W[14]                                    # h = 0: the hidden side of the candidate is its bias
    nn = np.tanh(W[5] * x + W[11] + r * ghn)
    h = (1 - z) * nn
    gq = 2.0
    dh = gq * W[15]
    dan = dh * (1 - z) * (1 - nn * nn)
    daz = dh * (0.0 - nn) * z * (1 - z)
    dar = dan * ghn * r * (1 - r)
    dx = dar * W[3] + daz * W[4] + dan * W[5]
    want = np.array([dx * float(o), dx, dx,                       # W1 (x > 0 here), b1
                     dar * x, daz * x, dan * x,                   # W_ih
                     0.0, 0.0, 0.0,                               # W_hh: h = 0
                     dar, daz, dan,                               # b_ih
                     dar, daz, dan * r,                           # b_hh
                     gq * h, gq])                                 # W2, b2
    assert x > 0
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_relu_ambiguity_budget_matches_the_library_adjoints():
    cfg, dims, w, u, g = case(1, B=2, T=6)
    band = 0.05
    got, amb = bpo.qnet_grad(dims, w, u["obs"], u["actions"], u["filled"], g, relu_band=band)
    want, want_amb = autograd_grad(dims, w, u, g, relu_band=band)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-11 * max(1.0, np.abs(want).max()))
    np.testing.assert_allclose(amb, want_amb, rtol=0, atol=1e-11 * max(1.0, want_amb.max()))
    sl = wl.weight_slices(*dims)
    assert amb[sl["W1"][0]:sl["W1"][1]].max() > 0 and amb[sl["b1"][1]:].max() == 0        # only the first layer
    # an empty band has an empty budget; a band that holds everything bounds the gradient itself
    _, none = bpo.qnet_grad(dims, w, u["obs"], u["actions"], u["filled"], g, relu_band=-1.0)
    assert none.max() == 0
    _, all_of_it = bpo.qnet_grad(dims, w, u["obs"], u["actions"], u["filled"], g, relu_band=1e9)
    a, b, _ = sl["W1"]
    assert (np.abs(got[a:b]) <= all_of_it[a:b] + 1e-12).all()
