"""Pins for the oracle's Philox4x32-10 and its word -> draw mappings (CPU only)."""
import math
import os

import numpy as np

from oracle import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat_rows():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        v = [int(x, 16) for x in line.split()]
        rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def test_known_answer_vectors():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert orc.philox(ctr, key) == want


def _philox_bigint(ctr, key):
    """Independent implementation on Python integers: the bijection written as a 128-bit
    permutation network (multiply, split, xor, permute), no shared helper with the oracle."""
    M0, M1 = 0xD2511F53, 0xCD9E8D57
    c = list(ctr)
    k = list(key)
    for r in range(10):
        kr0 = (k[0] + r * 0x9E3779B9) % (1 << 32)
        kr1 = (k[1] + r * 0xBB67AE85) % (1 << 32)
        p0, p1 = M0 * c[0], M1 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ kr0, p1 % (1 << 32), (p0 >> 32) ^ c[3] ^ kr1, p0 % (1 << 32)]
    return c


def test_bigint_cross_check_random_inputs():
    assert _philox_bigint([0] * 4, [0] * 2) == [0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8]
    rng = np.random.default_rng(12345)
    vals = rng.integers(0, 1 << 32, size=(10000, 6), dtype=np.uint64)
    for row in vals:
        ctr = [int(x) for x in row[:4]]
        key = [int(x) for x in row[4:]]
        assert orc.philox(ctr, key) == _philox_bigint(ctr, key)


def test_bijection_on_counter_for_fixed_key():
    # Philox is a permutation of the counter space for a fixed key: distinct counters -> distinct
    # outputs.  A dropped xor or a swapped word would produce collisions on structured inputs.
    seen = set()
    for env in range(64):
        for step in range(64):
            seen.add(tuple(orc.philox([env, step, 0, 0], [7, 0])))
    assert len(seen) == 64 * 64


def test_draw_block_keying():
    # counter = (env, step_lo, step_hi, stream); key = (seed_lo, seed_hi)
    seed = 0x123456789ABCDEF0
    step = 0x0000000500000007
    assert orc.draw_block(seed, 42, step, 16) == orc.philox([42, 7, 5, 16],
                                                            [0x9ABCDEF0, 0x12345678])
    # each of the four coordinates matters
    base = orc.draw_block(1, 2, 3, 0)
    assert orc.draw_block(2, 2, 3, 0) != base
    assert orc.draw_block(1, 3, 3, 0) != base
    assert orc.draw_block(1, 2, 4, 0) != base
    assert orc.draw_block(1, 2, 3, 1) != base
    assert orc.draw_block(1, 2, 3 + (1 << 32), 0) != base
    assert orc.draw_block(1 + (1 << 32), 2, 3, 0) != base


def test_action_mapping_edges():
    L = orc.lib()
    # floor(3 w / 2^32): thresholds at ceil(2^32/3) and ceil(2^33/3)
    assert L.oracle_pong_action(0) == 0
    assert L.oracle_pong_action(0x55555555) == 0
    assert L.oracle_pong_action(0x55555556) == 1
    assert L.oracle_pong_action(0xAAAAAAAA) == 1
    assert L.oracle_pong_action(0xAAAAAAAB) == 2
    assert L.oracle_pong_action(0xFFFFFFFF) == 2
    for w in np.random.default_rng(1).integers(0, 1 << 32, 1000, dtype=np.uint64):
        assert L.oracle_pong_action(int(w)) == (3 * int(w)) // (1 << 32)


def test_uniform_and_serve_mappings_exact():
    L = orc.lib()
    assert L.oracle_u01(0) == 0.0
    assert L.oracle_u01(0xFF) == 0.0                       # low 8 bits are discarded
    assert L.oracle_u01(0x100) == 2.0 ** -24
    assert L.oracle_u01(0xFFFFFFFF) == (2 ** 24 - 1) / 2 ** 24
    assert L.oracle_u01_open0(0) == 2.0 ** -24
    assert L.oracle_u01_open0(0xFFFFFFFF) == 1.0
    assert L.oracle_pong_serve_vx(0x80000000) == 3.0
    assert L.oracle_pong_serve_vx(0x7FFFFFFF) == -3.0
    assert L.oracle_pong_serve_vy(0) == -2.0
    assert L.oracle_pong_serve_vy(0x80000000) == 0.0
    assert L.oracle_pong_serve_vy(0xFFFFFFFF) == 2.0 - 2.0 ** -22
    for w in np.random.default_rng(2).integers(0, 1 << 32, 1000, dtype=np.uint64):
        w = int(w)
        exact = -2.0 + 4.0 * ((w >> 8) / 2 ** 24)          # exact in binary64
        assert L.oracle_pong_serve_vy(w) == exact           # and the float32 result has no rounding
        assert L.oracle_uniform(w, -0.1, 0.1) == np.float32(-0.1) + (
            np.float32(0.1) - np.float32(-0.1)) * np.float32((w >> 8) / 2 ** 24)


def _blocks(seed, n_env, n_step, stream=0):
    out = np.empty((n_env, n_step, 4), np.uint64)
    for e in range(n_env):
        for s in range(n_step):
            out[e, s] = orc.draw_block(seed, e, s, stream)
    return out


def test_action_distribution_chi_square():
    L = orc.lib()
    w = _blocks(0, 64, 500)[:, :, 0].ravel()
    a = np.array([L.oracle_pong_action(int(x)) for x in w])
    n = a.size
    counts = np.bincount(a, minlength=3)
    chi2 = float(((counts - n / 3) ** 2 / (n / 3)).sum())
    # 2 degrees of freedom: P(chi2 > 18.4) = 1e-4
    assert chi2 < 18.4, (counts, chi2)


def test_serve_distribution_moments():
    L = orc.lib()
    blk = _blocks(5, 64, 500)
    vy = np.array([L.oracle_pong_serve_vy(int(x)) for x in blk[:, :, 2].ravel()], np.float64)
    vx = np.array([L.oracle_pong_serve_vx(int(x)) for x in blk[:, :, 1].ravel()], np.float64)
    n = vy.size
    # uniform on [-2,2): mean 0, variance 4/3; 4.5 standard errors
    assert abs(vy.mean()) < 4.5 * math.sqrt(4 / 3 / n)
    # var of the sample variance of a uniform: (mu4 - sigma^4)/n with mu4 = 16/5
    assert abs(vy.var() - 4 / 3) < 4.5 * math.sqrt((16 / 5 - 16 / 9) / n)
    assert abs((vx > 0).mean() - 0.5) < 4.5 * math.sqrt(0.25 / n)
    assert set(np.unique(vx)) == {-3.0, 3.0}


def test_normal_pair_matches_box_muller_and_moments():
    import ctypes as C
    L = orc.lib()
    out = (C.c_float * 2)()
    blk = _blocks(9, 32, 250, stream=17)
    xs = []
    for row in blk.reshape(-1, 4):
        wa, wb = int(row[0]), int(row[1])
        L.oracle_normal_pair(wa, wb, out)
        u1 = ((wa >> 8) + 1) / 2 ** 24
        u2 = (wb >> 8) / 2 ** 24
        r = math.sqrt(-2.0 * math.log(u1))
        assert abs(out[0] - r * math.cos(2 * math.pi * u2)) < 2e-6 * max(1.0, r)
        assert abs(out[1] - r * math.sin(2 * math.pi * u2)) < 2e-6 * max(1.0, r)
        xs += [out[0], out[1]]
    xs = np.array(xs, np.float64)
    n = xs.size
    assert abs(xs.mean()) < 4.5 / math.sqrt(n)
    assert abs(xs.var() - 1.0) < 4.5 * math.sqrt(2.0 / n)
