"""Shared helpers of the GPU parity tests (marshalling only)."""
import numpy as np


def bits(a):
    """View float32 data as uint32 so comparisons are bit for bit (distinguishes -0.0, NaN)."""
    a = np.ascontiguousarray(a)
    return a.view(np.uint32) if a.dtype == np.float32 else a


def assert_bit_equal(got, want, what=""):
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    g, w = bits(got), bits(want)
    if not np.array_equal(g, w):
        bad = np.argwhere(g != w)
        first = tuple(bad[0])
        raise AssertionError("%s: %d of %d elements differ, first at %s: got %r want %r" % (
            what, len(bad), g.size, first, got[first], want[first]))


def split_state(blob, n, fields):
    """State blob -> (step counter, uint32 array [fields, n])."""
    step = int(np.frombuffer(blob[:8].tobytes(), np.uint64)[0])
    arr = np.frombuffer(blob[8:].tobytes(), np.uint32).reshape(fields, n)
    return step, arr


def pong_state_fields(envs):
    """Oracle Pong records -> uint32 [10, n] in the boundary's field order."""
    names = ["bx", "by", "vx", "vy", "pa", "po", "sa", "so", "ep_ret", "ep_len"]
    return np.stack([np.ascontiguousarray(envs[k]).view(np.uint32) for k in names])


def pong_blob(step, fields_u32):
    return np.concatenate([np.array([step], np.uint64).view(np.uint8),
                           np.ascontiguousarray(fields_u32).view(np.uint8).ravel()])


def tost_p(diff, se, margin):
    """p-value of the two one-sided tests for |true difference| < margin (the equivalence procedure
    of the paper's section 4.3, "Cross-backend policy transfer"), normal approximation (thousands
    of samples per side): the larger of the two one-sided p-values."""
    from scipy.stats import norm
    return float(max(norm.sf((diff + margin) / se), norm.sf((margin - diff) / se)))
