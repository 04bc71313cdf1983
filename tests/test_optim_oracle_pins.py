"""Pins of the parameter-update oracle (CPU only): values worked by hand on numbers fp32 holds exactly, cases where
the order of the fp32 roundings decides the result, and a tensor library's optimisers."""
import numpy as np
import torch

from oracle import optim_oracle as opo

f32 = lambda *v: np.array(v, np.float32)


def test_sgd_by_hand():
    # 1 - 0.25 * 2 = 0.5 ;  -3 - 0.25 * (-4) = -2 ;  a zero gradient leaves the weight alone
    np.testing.assert_array_equal(opo.sgd_step(f32(1.0, -3.0, 7.5), f32(2.0, -4.0, 0.0), 0.25), f32(0.5, -2.0, 7.5))
    # the difference is rounded to fp32: 1 - 2^-25 lies halfway between 1 - 2^-24 and 1, and the tie goes to the
    # even neighbour, 1;  1 - 2^-24 is a float and stays
    np.testing.assert_array_equal(opo.sgd_step(f32(1.0, 1.0), f32(2.0 ** -25, 2.0 ** -24), 1.0), f32(1.0, 1.0 - 2.0 ** -24))
    # the product is rounded before the difference: lr = g = 1 + 2^-12 gives 1 + 2^-11 + 2^-24, whose tail is
    # exactly half a unit in the last place (2^-23): the tie goes to the even neighbour, 1 + 2^-11;
    # w = 1 + 2^-11 then yields exactly 0, where an unrounded product would have left -2^-24
    x = np.float32(1.0 + 2.0 ** -12)
    np.testing.assert_array_equal(opo.sgd_step(f32(1.0 + 2.0 ** -11), f32(x), x), f32(0.0))


def test_rmsprop_by_hand():
    # alpha = 0.75, eps = 2, lr = 0.5, w = 3, v = 0:
    # step 1, g = 4:  v = 0.75 * 0 + 0.25 * 16 = 4;  w = 3 - 0.5 * 4 / (2 + 2) = 2.5
    # step 2, g = 2:  v = 0.75 * 4 + 0.25 * 4 = 4;   w = 2.5 - 0.5 * 2 / (2 + 2) = 2.25
    # step 3, g = -2: v = 3 + 0.25 * 4 = 4 again;  w = 2.25 + 0.5 * 2 / 4 = 2.5
    w, v = f32(3.0), f32(0.0)
    w, v = opo.rmsprop_step(w, f32(4.0), v, 0.5, 0.75, 2.0)
    np.testing.assert_array_equal((w, v), (f32(2.5), f32(4.0)))
    w, v = opo.rmsprop_step(w, f32(2.0), v, 0.5, 0.75, 2.0)
    np.testing.assert_array_equal((w, v), (f32(2.25), f32(4.0)))
    w, v = opo.rmsprop_step(w, f32(-2.0), v, 0.5, 0.75, 2.0)
    np.testing.assert_array_equal((w, v), (f32(2.5), f32(4.0)))
    # a zero gradient decays the running square and leaves the weight: v = 0.75 * 4 = 3
    w, v = opo.rmsprop_step(w, f32(0.0), v, 0.5, 0.75, 2.0)
    np.testing.assert_array_equal((w, v), (f32(2.5), f32(3.0)))
    # alpha = 1 freezes the running square at zero: the step is lr * g / eps
    w, v = opo.rmsprop_step(f32(1.0), f32(8.0), f32(0.0), 0.5, 1.0, 4.0)
    np.testing.assert_array_equal((w, v), (f32(0.0), f32(0.0)))
    # alpha = 0: v = g^2, the step is lr * g / (|g| + eps) = 0.5 * 3 / (3 + 1)
    w, v = opo.rmsprop_step(f32(1.0), f32(3.0), f32(100.0), 0.5, 0.0, 1.0)
    np.testing.assert_array_equal((w, v), (f32(0.625), f32(9.0)))


def test_rmsprop_rounds_the_running_square_before_the_root():
    # g = 1 + 2^-12: g^2 = 1 + 2^-11 + 2^-24 rounds to 1 + 2^-11 in fp32; alpha = 0, so v is that value
    g = np.float32(1.0 + 2.0 ** -12)
    _, v = opo.rmsprop_step(f32(0.0), f32(g), f32(0.0), 1.0, 0.0, 1.0)
    np.testing.assert_array_equal(v, f32(1.0 + 2.0 ** -11))


def test_against_a_tensor_library():
    rng = np.random.default_rng(0)
    w0 = rng.normal(size=4096).astype(np.float32)
    grads = [(rng.normal(size=4096) * 10.0 ** (k - 1)).astype(np.float32) for k in range(4)]
    # plain descent: the library may fuse the product into the difference (one rounding instead of two): equal
    # within a unit in the last place of the largest step taken (0.03 * 100 * a few sigma)
    p = torch.nn.Parameter(torch.from_numpy(w0.copy()))
    opt = torch.optim.SGD([p], lr=0.03)
    w = w0.copy()
    for g in grads:
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        w = opo.sgd_step(w, g, 0.03)
    np.testing.assert_allclose(w, p.detach().numpy(), rtol=3e-7, atol=4e-6)
    # RMSprop (no momentum, not centred): the library's default form, eps outside the root
    p = torch.nn.Parameter(torch.from_numpy(w0.copy()))
    opt = torch.optim.RMSprop([p], lr=0.01, alpha=0.99, eps=1e-5)
    w, v = w0.copy(), np.zeros_like(w0)
    for g in grads:
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        w, v = opo.rmsprop_step(w, g, v, 0.01, 0.99, 1e-5)
    # (the library forms 1 - alpha in double precision, the definition here in fp32: 1e-6 relative on that factor)
    np.testing.assert_allclose(v, opt.state[p]["square_avg"].numpy(), rtol=3e-6)
    np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-5, atol=1e-6)
