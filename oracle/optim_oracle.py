"""CPU oracle of the learner's parameter update (Alg. 3, "update the parameters theta with the gradient").

TEST INFRASTRUCTURE ONLY: imported by tests/.  The GPU library never imports or calls it, and this module never
imports the GPU package.

The paper names the step and leaves the optimiser to its base algorithms (plain gradient descent; RMSprop in the
QMIX family).  Unlike the rest of the oracle this one computes in fp32, one rounding per operation in the order
written: the update is elementwise, so the order of operations is the whole definition, and an implementation
that follows it is reproducible bit for bit.  Each operation below is a single numpy float32 operation, so each
is rounded once (nearest, ties to even) and nothing is fused.
"""
import numpy as np

F = np.float32


def _f32(a):
    a = np.asarray(a)
    assert a.dtype == np.float32, "the update is defined on fp32 values"
    return a


def sgd_step(weights, grad, lr):
    """weights - lr * grad: the product rounded to fp32, then the difference rounded to fp32."""
    w, g = _f32(weights), _f32(grad)
    step = F(lr) * g
    return w - step


def rmsprop_step(weights, grad, sq_avg, lr, alpha, eps):
    """(weights', sq_avg'):
        sq_avg'  = alpha * sq_avg + (1 - alpha) * grad^2
        weights' = weights - lr * grad / (sqrt(sq_avg') + eps)
    evaluated left to right, products before sums, every operation rounded to fp32 on its own."""
    w, g, v = _f32(weights), _f32(grad), _f32(sq_avg)
    lr, alpha, eps = F(lr), F(alpha), F(eps)
    decayed = alpha * v
    squared = g * g
    fresh = (F(1.0) - alpha) * squared
    v_new = decayed + fresh
    root = np.sqrt(v_new)
    denom = root + eps
    ratio = g / denom
    step = lr * ratio
    return w - step, v_new
