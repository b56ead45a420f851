"""Pins for the oracle's random numbers, dist() and sample() -- CPU only.

Each expectation here comes from something other than the oracle: published known-answer
vectors, closed forms evaluated with Python integers / fp64, numpy's sort, or brute force.
"""
import math
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- Philox4x32-10
def _kat_rows():
    rows = []
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert oracle.philox(key, ctr).tolist() == out


def _philox_py(key, ctr):
    """Independent restatement with Python integers (multiply-high/low, key schedule)."""
    k0, k1 = key
    c = list(ctr)
    M = 0xFFFFFFFF
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k0) & M, p1 & M, ((p0 >> 32) ^ c[3] ^ k1) & M, p0 & M]
        k0 = (k0 + 0x9E3779B9) & M
        k1 = (k1 + 0xBB67AE85) & M
    return c


def test_philox_python_restatement_matches_kat_and_oracle():
    for ctr, key, out in _kat_rows():
        assert _philox_py(key, ctr) == out
    rng = np.random.default_rng(0)
    for _ in range(200):
        key = [int(x) for x in rng.integers(0, 2**32, 2)]
        ctr = [int(x) for x in rng.integers(0, 2**32, 4)]
        assert oracle.philox(key, ctr).tolist() == _philox_py(key, ctr)


def test_draw_counter_layout():
    # key = (seed lo, seed hi); counter = (c lo, c hi, window index, 0)
    seed, c, i = 0x1234567890ABCDEF, 0x0000000700000005, 9
    exp = _philox_py([seed & 0xFFFFFFFF, seed >> 32], [c & 0xFFFFFFFF, c >> 32, i, 0])
    assert oracle.draw(seed, c, i).tolist() == exp


def test_u_acc_range():
    assert oracle.u_acc(0) == 0.0
    assert oracle.u_acc(0xFFFFFFFF) == 1.0 - 2.0**-24
    assert oracle.u_acc(0x80000000) == 0.5
    assert oracle.u_acc(0x000000FF) == 0.0          # low 8 bits are dropped


# ---------------------------------------------------------------- exp recipe
def test_exp_against_libm():
    xs = np.concatenate([np.linspace(-60, 0, 20001), -np.logspace(-8, 1.7, 3000)]).astype(np.float32)
    xs = xs[xs >= -60]
    worst = 0.0
    for x in xs:
        got = oracle.exp(x)
        want = math.exp(float(x))
        worst = max(worst, abs(got - want) / want)
    assert worst < 3 * 2.0**-24, worst          # within ~1.5 ulp of the exact value
    assert oracle.exp(0.0) == 1.0
    assert oracle.exp(-60.5) == 0.0
    assert oracle.exp(np.float32(-60.0)) > 0.0


# ---------------------------------------------------------------- dist()
def _softmax64(z, T=1.0):
    z = z.astype(np.float64) / T
    e = np.exp(z - z.max())
    return e / e.sum()


def test_dist_full_support_is_softmax():
    rng = np.random.default_rng(1)
    for V, T in [(8, 1.0), (1024, 1.0), (8192, 0.7), (100, 2.5)]:
        z = (rng.standard_normal(V) * 1.3).astype(np.float32)
        q = oracle.dist(z, V + 5, T)
        ref = _softmax64(z, np.float32(T).astype(np.float64))
        assert np.max(np.abs(q - ref) / ref) < 2e-6
        assert abs(q.astype(np.float64).sum() - 1.0) < 1e-6


def test_dist_topk_support_and_values():
    rng = np.random.default_rng(2)
    V, K = 4096, 500
    z = (rng.standard_normal(V) * 1.3).astype(np.float32)
    q = oracle.dist(z, K, 1.0)
    order = np.argsort(-z.astype(np.float64), kind="stable")      # value desc, index asc
    keep = np.zeros(V, bool); keep[order[:K]] = True
    assert np.array_equal(q > 0, keep)
    ref = np.zeros(V); ref[keep] = _softmax64(z[keep])
    assert np.max(np.abs(q - ref)) < 1e-8
    assert abs(q.astype(np.float64).sum() - 1.0) < 1e-6


def test_dist_ties_keep_exactly_k_lowest_index_first():
    z = np.array([1.0, 3.0, 2.0, 2.0, 2.0, 0.5, 2.0, 3.0], np.float32)
    q = oracle.dist(z, 4, 1.0)
    # 3.0 at {1,7}; then 2.0 at {2,3,4,6}: the two lowest indices survive
    assert np.nonzero(q)[0].tolist() == [1, 2, 3, 7]
    e = np.exp(np.array([0.0, -1.0, -1.0, 0.0]))
    assert np.allclose(q[[1, 2, 3, 7]], e / e.sum(), rtol=1e-6)
    q = oracle.dist(np.zeros(16, np.float32), 5, 1.0)
    assert np.nonzero(q)[0].tolist() == [0, 1, 2, 3, 4]
    assert np.allclose(q[:5], 0.2, rtol=1e-6)


def test_dist_negative_and_signed_zero_ordering():
    z = np.array([-1.0, -0.0, 0.0, -2.0, -1.0], np.float32)
    q = oracle.dist(z, 2, 1.0)
    assert np.nonzero(q)[0].tolist() == [1, 2]           # the two zeros beat the negatives
    q = oracle.dist(np.array([-3.0, -1.0, -2.0], np.float32), 1, 1.0)
    assert q.tolist() == [0.0, 1.0, 0.0]


def test_dist_greedy_modes_and_forced():
    rng = np.random.default_rng(3)
    z = rng.standard_normal(300).astype(np.float32)
    z[17] = z[200] = z.max() + 1.0                        # tie for the maximum
    for K, T in [(1, 1.0), (50, 0.0)]:
        q = oracle.dist(z, K, T)
        assert q[17] == 1.0 and q.sum() == 1.0
    q = oracle.dist(z, 50, 1.0, forced=123)
    assert q[123] == 1.0 and q.sum() == 1.0


def test_dist_temperature_sharpens():
    z = np.array([0.0, 1.0, 2.0, 3.0], np.float32)
    for T in (0.5, 1.0, 4.0):
        q = oracle.dist(z, 4, T)
        assert np.allclose(q, _softmax64(z, T), rtol=2e-6)


# ---------------------------------------------------------------- sample()
def _fixed40(w):
    return [int(math.floor(float(x) * 2**40)) if x > 0 else 0 for x in w]


def test_sample_closed_form_boundaries():
    w = np.array([0.1, 0.0, 0.25, 0.4, 0.05], np.float32)
    c = _fixed40(w); C = sum(c)
    pref = np.cumsum(c).tolist()
    rng = np.random.default_rng(4)
    ks = list(rng.integers(0, 2**32, 2000)) + [0, 1, 2**32 - 1, 2**31]
    # boundaries: smallest k32 whose tau reaches each prefix sum
    for p in pref[:-1]:
        k = (p << 32) // C
        ks += [max(k - 1, 0), k, min(k + 1, 2**32 - 1)]
    for k in ks:
        k = int(k)
        tau = (k * C) >> 32
        want = next(t for t, p in enumerate(pref) if p > tau)
        assert oracle.sample(w, k) == want
    assert oracle.sample(np.zeros(5, np.float32), 12345) == -1
    assert oracle.sample(np.array([0, 0, 1e-13, 0], np.float32), 7) == -1      # below 2^-40


def test_sample_brute_force_counts_and_monotone():
    w = np.array([0.3, 0.2, 0.0, 0.5], np.float32)
    c = _fixed40(w); C = sum(c)
    n = 1 << 16
    ks = (np.arange(n, dtype=np.uint64) << np.uint64(16)).astype(np.uint64)
    ids = np.array([oracle.sample(w, int(k)) for k in ks])
    assert np.all(np.diff(ids) >= 0)                      # monotone in k32
    counts = np.bincount(ids, minlength=4)
    assert counts[2] == 0
    for t in range(4):
        assert abs(counts[t] - n * c[t] / C) <= 1.0
    # unnormalised weights give the same proportions
    ids2 = np.array([oracle.sample(w * np.float32(0.125), int(k)) for k in ks[::16]])
    assert np.array_equal(ids2, ids[::16])


def test_sample_onehot_is_deterministic():
    w = np.zeros(64, np.float32); w[37] = 1.0
    for k in (0, 1, 2**31, 2**32 - 1):
        assert oracle.sample(w, k) == 37


def test_guidance_combination():
    """z = z_u + w (z_c - z_u): exact special cases and the fp64 value within the rounding of three fp32
    operations; applied to distributions it moves mass towards the conditional one"""
    rng = np.random.default_rng(11)
    zc = (rng.standard_normal(4096) * 1.3).astype(np.float32)
    zu = (rng.standard_normal(4096) * 1.3).astype(np.float32)
    assert np.array_equal(oracle.guide(zc, zu, 0.0), zu)                  # no guidance: unconditional
    assert np.array_equal(oracle.guide(zc, zc, 3.0), zc)                  # identical contexts: unchanged
    for w in (1.0, 3.0, 7.5, -0.5):
        got = oracle.guide(zc, zu, w).astype(np.float64)
        ref = zu.astype(np.float64) + w * (zc.astype(np.float64) - zu.astype(np.float64))
        scale = np.abs(zu) + abs(w) * np.abs(zc.astype(np.float64) - zu) + np.abs(ref)
        assert np.all(np.abs(got - ref) <= 2.0 ** -22 * scale)
    # w = 1 is the conditional logits up to that rounding; w > 1 extrapolates past them
    assert np.max(np.abs(oracle.guide(zc, zu, 1.0) - zc)) < 1e-6
    j = int(np.argmax(zc - zu))
    p1 = oracle.dist(oracle.guide(zc, zu, 1.0), 4096, 1.0)
    p3 = oracle.dist(oracle.guide(zc, zu, 3.0), 4096, 1.0)
    assert p3[j] > p1[j]
