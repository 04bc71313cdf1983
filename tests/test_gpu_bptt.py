"""GPU parity of the backward pass: marl_qnet_grad through the C ABI against the fp64 oracle, tensor by
tensor of the packed gradient.  Bar: every entry within REL * max |oracle tensor| (plus a small absolute
floor) of the oracle; REL = 1e-3 for fp32 networks (split-bf16 products, fp32 sums over all samples), 3e-2
for bf16 networks (weights, activations and the recurrent adjoints rounded to bf16).  The first layer's
ReLU is a yes/no decision taken on forward values: where the oracle's pre-activation is within the
forward tolerance of zero the two sides may decide differently, so the entries of W1 and b1 get, on top,
the oracle's ambiguity budget for that band (the summed magnitude of exactly those samples' terms)."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import bptt_oracle as bpo
from paper_2205_05248_amd import binding, workloads as wl
import parity_util as pu

pytestmark = pytest.mark.gpu
REL = {"fp32": 1e-3, "bf16": 3e-2}
# Half-width of the band of first-layer pre-activations in which the two sides may switch a unit differently:
# the forward error of that pre-activation.  fp32 networks: the forward tolerance.  bf16 networks: the kernel
# rounds every observation entry to bf16 (relative 2^-9) before the product, the oracle does not; with
# pre-activations of order one that is a few times 1e-3.
RELU_BAND = {"fp32": 1e-4, "bf16": 5e-3}


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    binding.load()
    if not torch.cuda.is_available():
        pytest.skip("no GPU in this container")


def gpu_grad(net, cfg, u, g, workspace=None):
    d = pu.to_dev(u, ["obs", "actions", "filled"])
    B, T = u["actions"].shape[:2]
    need = net.grad_workspace_bytes(B, T)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda") if workspace is None else workspace
    ws.fill_(0xFF)                                   # NaN patterns: nothing may be read before it is written
    n_params = wl.param_count(*wl.dims(cfg))
    out = torch.full((n_params,), float("nan"), device="cuda")
    net.grad(d["obs"], d["actions"], d["filled"], torch.from_numpy(g.astype(np.float32)).cuda(), ws, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def compare(cfg, got, want, amb):
    rel = REL[cfg["dtype"]]
    assert np.isfinite(got).all()
    worst, bad = {}, []
    for name, (a, b, _) in wl.weight_slices(*wl.dims(cfg)).items():
        scale = np.abs(want[a:b]).max()
        err = np.abs(got[a:b] - want[a:b])
        worst[name] = err.max() / max(scale, 1e-30)
        if name not in ("W1", "b1"):
            assert amb[a:b].max() == 0
        over = err - (rel * scale + 1e-6 + amb[a:b])
        if over.max() > 0:
            bad.append(f"{name}: max err {err.max():.3e} against scale {scale:.3e}, budget up to {amb[a:b].max():.3e}")
    print(cfg["name"], {k: f"{v:.1e}" for k, v in worst.items()}, "budget/scale W1 %.1e" % (
        amb[:wl.weight_slices(*wl.dims(cfg))["W1"][1]].max() / np.abs(want[:wl.weight_slices(*wl.dims(cfg))["W1"][1]]).max()))
    assert not bad, bad
    return worst


CASES = [(0, 4, 6, {}), (0, 32, 25, {}), (1, 5, 9, {}), (2, 7, 12, {}), (3, 33, 5, {}), (4, 3, 11, {}),
         # the widest first layer and more than sixteen agents with fp32 weights; a bf16 network with H = 64
         (4, 3, 7, dict(H=64, D=150, dtype="fp32")), (1, 6, 8, dict(dtype="bf16"))]


@pytest.mark.parametrize("ci,B,T,over", CASES, ids=lambda v: str(v).replace(" ", ""))
def test_gradient_matches_the_oracle(ci, B, T, over):
    cfg = dict(wl.config(ci), B=B, T=T, **over)
    dims = wl.dims(cfg)
    w = wl.make_weights(cfg, 0)
    net = binding.QNet(dims, w, cfg["dtype"])
    u = wl.make_unroll_inputs(cfg, B=B, T=T)
    g = np.random.default_rng(ci).normal(size=(B, T, dims[0])).astype(np.float32)
    got = gpu_grad(net, cfg, u, g)
    want, amb = bpo.qnet_grad(dims, pu.oracle_weights(cfg, w), u["obs"], u["actions"], u["filled"], g.astype(np.float64),
                              relu_band=RELU_BAND[cfg["dtype"]])
    compare(cfg, got, want, amb)
    # the same call again: identical bits (fixed summation order)
    again = gpu_grad(net, cfg, u, g)
    np.testing.assert_array_equal(again, got)
    net.close()
