"""Seeded synthetic inputs shared by the tests and the benchmark.  Holds none of the method's
arithmetic: only plain pseudo-random arrays of the documented shapes and value ranges.

The workloads draw their own randomness (actions, serves, initial states) from Philox inside the
step; the arrays below exercise the *external-action* entry of the boundary and hand-picked states.
"""
import numpy as np


def pong_actions(T, n, seed):
    """uint8 [T, n]: uniform over {0 stay, 1 up, 2 down}, plus a sprinkle of out-of-range codes
    (which the boundary defines as 'stay')."""
    rng = np.random.default_rng(seed)
    a = rng.integers(0, 3, size=(T, n), dtype=np.uint8)
    odd = rng.random((T, n)) < 0.01
    a[odd] = rng.integers(3, 256, size=int(odd.sum()), dtype=np.uint8)
    return a


def body_actions(T, n, seed, scale=1.2):
    """float32 [T, n, 6]: uniform in [-scale, scale]; scale > 1 exercises the clip to [-1, 1]."""
    rng = np.random.default_rng(seed)
    return rng.uniform(-scale, scale, size=(T, n, 6)).astype(np.float32)


def pong_positions(count, seed):
    """float32 [count, 4] = (ball x, ball y, agent y, opponent y) anywhere legal in the field."""
    rng = np.random.default_rng(seed)
    return np.stack([rng.uniform(0, 158, count), rng.uniform(0, 208, count),
                     rng.uniform(0, 194, count), rng.uniform(0, 194, count)], 1).astype(np.float32)


def cartpole_actions(T, n, seed):
    """uint8 [T, n]: uniform over {0 push left, 1 push right}, plus a sprinkle of other codes
    (which the boundary defines as 'push left')."""
    rng = np.random.default_rng(seed)
    a = rng.integers(0, 2, size=(T, n), dtype=np.uint8)
    odd = rng.random((T, n)) < 0.01
    a[odd] = rng.integers(2, 256, size=int(odd.sum()), dtype=np.uint8)
    return a
