"""marl_unroll_td_static, the unroll for callers that cannot allocate: through the C ABI against marl_unroll_td on
the same kernels (bit for bit) and against the oracle (the forward tolerance), on two calls in a row of which the
second is smaller, so that it runs over what the first left in the static buffer."""
import numpy as np
import pytest
import torch

from oracle import marl_oracle as orc
from paper_2205_05248_amd import binding, workloads as wl
import parity_util as pu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    binding.load()
    if not torch.cuda.is_available():
        pytest.skip("no GPU in this container")


def nets(cfg):
    w_on, w_tg = wl.make_weights(cfg, 0), wl.make_weights(cfg, 1)
    online = binding.QNet(wl.dims(cfg), w_on, cfg["dtype"])
    target = binding.QNet(wl.dims(cfg), w_tg, cfg["dtype"])
    return online, target, pu.oracle_weights(cfg, w_on), pu.oracle_weights(cfg, w_tg)


def oracle_unroll(cfg, w_on, w_tg, u):
    return orc.unroll_td(wl.dims(cfg), w_on, w_tg, u["obs"], u["avail"], u["actions"], u["reward"], u["terminated"],
                         u["filled"], u["gamma"])


def scratch_bytes(cfg, B, T, two=True):
    N, D, A, H = wl.dims(cfg)
    per_net = -(-B * N // 32) * (T + 1) * 3 * (H // 32) * (2048 if cfg["dtype"] == "bf16" else 4096)
    return (2 if two else 1) * (-(-per_net // 256) * 256)


# (configuration, first call's B and T, second call's B and T): the first one of each pair is the larger
CASES = [(1, (32, 120), (5, 9)),          # a paper scenario at full size: 46 MiB of the 64, fp32 weights, 64 hidden units
         (4, (5, 40), (2, 7)),            # the scale-up network (bf16, 128 hidden units, which left alone takes the fused kernels)
         (0, (4, 60), (4, 59))]


@pytest.mark.parametrize("ci,first,second", CASES, ids=lambda v: str(v).replace(" ", ""))
def test_static_unroll_matches_the_allocating_one_twice_in_a_row(ci, first, second):
    cfg = wl.config(ci)
    tol = pu.TOL[cfg["dtype"]]
    online, target, w_on, w_tg = nets(cfg)
    plain_on, plain_tg, _, _ = nets(cfg)                  # the allocating entry point runs on handles of its own
    plain_on.set_kernels(binding.KERNELS_TILE32)
    for stream, (B, T) in enumerate((first, second)):
        assert scratch_bytes(cfg, B, T) <= binding.STATIC_SCRATCH_BYTES
        u = wl.make_unroll_inputs(cfg, B=B, T=T, stream=stream)
        got = pu.gpu_unroll(online, target, cfg, u, static=True)
        same = pu.gpu_unroll(plain_on, plain_tg, cfg, u)
        for k in got:
            np.testing.assert_array_equal(got[k], same[k], err_msg=k)
        worst = pu.compare_unroll(got, oracle_unroll(cfg, w_on, w_tg, u), tol)
        print(f"cfg{ci} B={B} T={T}: static == allocating, max |. - oracle| = {worst:.2e}")
    # one network as its own target: one projection
    u = wl.make_unroll_inputs(cfg, B=second[0], T=second[1], stream=2)
    got = pu.gpu_unroll(online, None, cfg, u, static=True)
    pu.compare_unroll(got, oracle_unroll(cfg, w_on, None, u), tol)
    for net in (online, target, plain_on, plain_tg):
        net.close()


def test_static_unroll_takes_no_device_memory_and_refuses_what_does_not_fit():
    cfg = wl.config(4)
    online, target, _, _ = nets(cfg)
    N, D, A, H = wl.dims(cfg)
    # the benchmark's batch needs several hundred MiB: refused, with both sizes in the message, nothing launched
    B, T = cfg["B"], cfg["T"]
    assert scratch_bytes(cfg, B, T) > binding.STATIC_SCRATCH_BYTES
    z = lambda *shape, dtype=torch.float32: torch.zeros(*shape, dtype=dtype, device="cuda")
    args = (z(B, T + 1, N, D), z(B, T + 1, N, A, dtype=torch.uint8), z(B, T, N, dtype=torch.int32), z(B, T), z(B, T, dtype=torch.uint8),
            z(B, T, dtype=torch.uint8), 0.99, z(B, T, N), z(B, T, N), z(B, T, N))
    with pytest.raises(binding.MarlError) as err:
        online.unroll_td(target, *args, static=True)
    assert err.value.status == -2                                  # MARL_ERR_BAD_DIM
    assert str(scratch_bytes(cfg, B, T)) in str(err.value) and str(binding.STATIC_SCRATCH_BYTES) in str(err.value)
    del args
    # the largest batch of this shape that fits, by the documented formula, is accepted; one more slot is not
    B = 8
    T = max(t for t in range(1, 400) if scratch_bytes(cfg, B, t) <= binding.STATIC_SCRATCH_BYTES)
    u = wl.make_unroll_inputs(cfg, B=B, T=T)
    d = pu.to_dev(u, ["obs", "avail", "actions", "reward", "terminated", "filled"])
    outs = [torch.empty(B, T, N, device="cuda") for _ in range(3)]
    run = lambda: online.unroll_td(target, d["obs"], d["avail"], d["actions"], d["reward"], d["terminated"], d["filled"],
                                   u["gamma"], *outs, static=True)
    run()                                                          # first launch of these kernels in the process
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    for _ in range(3):
        run()
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before              # the device's free memory did not move
    assert all(torch.isfinite(o).all() for o in outs)
    u1 = wl.make_unroll_inputs(cfg, B=B, T=T + 1)
    d1 = pu.to_dev(u1, ["obs", "avail", "actions", "reward", "terminated", "filled"])
    outs1 = [torch.empty(B, T + 1, N, device="cuda") for _ in range(3)]
    with pytest.raises(binding.MarlError) as err:
        online.unroll_td(target, d1["obs"], d1["avail"], d1["actions"], d1["reward"], d1["terminated"], d1["filled"],
                         u1["gamma"], *outs1, static=True)
    assert err.value.status == -2
    online.close(); target.close()


def test_static_unroll_replays_from_a_hip_graph():
    """What the entry point is for: captured into a HIP graph (after one eager call, so that the kernels are loaded)
    and replayed on fresh input values with eager work between the replays; every replay equals the eager call."""
    cfg = dict(wl.config(1), B=6, T=11)
    N, D, A, H = wl.dims(cfg)
    online, target, w_on, w_tg = nets(cfg)
    keys = ["obs", "avail", "actions", "reward", "terminated", "filled"]
    batches = [wl.make_unroll_inputs(cfg, stream=s) for s in range(3)]
    u = pu.to_dev(batches[0], keys)
    B, T = cfg["B"], cfg["T"]
    outs = [torch.empty(B, T, N, device="cuda") for _ in range(3)]
    call = lambda: online.unroll_td(target, u["obs"], u["avail"], u["actions"], u["reward"], u["terminated"], u["filled"],
                                    batches[0]["gamma"], *outs, static=True)
    call()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            call()
    torch.cuda.synchronize()
    for r, batch in enumerate(batches):
        for k in keys:
            u[k].copy_(torch.from_numpy(np.ascontiguousarray(batch[k])))
        call()
        torch.cuda.synchronize()
        eager = [o.clone() for o in outs]
        for o in outs:
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for e, o in zip(eager, outs):
            assert torch.equal(e, o), f"replay {r} differs from the eager call"
        if r == 0:
            got = dict(zip(("q_taken", "next_max", "td_target"), (o.cpu().numpy() for o in outs)), q_all=None)
            pu.compare_unroll(got, oracle_unroll(cfg, w_on, w_tg, batch), pu.TOL[cfg["dtype"]])
    online.close(); target.close()
