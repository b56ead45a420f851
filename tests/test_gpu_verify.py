"""GPU parity: sampling distribution, verification and window slide vs the CPU oracle.

Bar: bit-exact (accepted count, token ids, and every fp32 probability), because every decision
in this part of the path is an integer comparison or one correctly rounded fp32 operation.
"""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import oracle  # noqa: E402
from paper_2410_01699_amd import synth  # noqa: E402


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2410_01699_amd import binding
    return binding


def _say(msg):
    print(msg, flush=True, file=sys.stderr)


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _gpu_dist(B, z, K, T, forced=None):
    rows, V = z.shape
    q = torch.empty((rows, V), dtype=torch.float32, device="cuda")
    f = None if forced is None else _dev(np.asarray(forced, np.int32))
    B.sjd_dist(_dev(z), rows, V, B.sjd_sampler(K, T), f, q)
    torch.cuda.synchronize()
    return q.cpu().numpy()


@pytest.mark.parametrize("V,K,T", [(8, 6, 1.0), (1024, 64, 1.0), (8192, 2000, 1.0), (16384, 2000, 1.0), (16384, 16384, 0.7),
                                   (1000, 999, 1.3), (4099, 1, 1.0), (777, 50, 0.0), (32768, 2000, 1.0), (64, 100, 1.0)])
def test_dist_bit_exact(B, V, K, T):
    _say(f"dist V={V} K={K} T={T}")
    z = synth.random_logits(5, V, seed=V + K)
    got = _gpu_dist(B, z, K, T)
    for r in range(z.shape[0]):
        want = oracle.dist(z[r], K, T)
        assert np.array_equal(got[r].view(np.uint32), want.view(np.uint32)), (r, np.abs(got[r] - want).max())


@pytest.mark.parametrize("V,K,T", [(8192, 2000, 1.0), (16384, 2000, 1.0), (3000, 429, 0.8), (8192, 8192, 1.0), (5000, 1, 1.0),
                                   (12000, 300, 0.0), (20000, 2000, 1.0), (64, 10, 1.0)])
def test_dist_many_rows_bit_exact(B, V, K, T):
    """hundreds of independent rows in one launch take the 256- or 512-thread variant of the distribution kernel
    (several rows per CU in flight; vocabularies above 16384 stay on the 1024-thread one): every row must come out
    bit for bit as the oracle's, ties at the K-th value, all-equal rows and forced rows included"""
    _say(f"dist, 700 rows: V={V} K={K} T={T}")
    rows = 700
    z = synth.random_logits(rows, V, seed=V + K + 1)
    z[0, ::7] = 0.25                      # many equal values around the K-th
    z[1] = 0.0                            # everything ties
    z[2, 10:40] = z[2].max() + 1          # ties at the top
    z[3] = np.round(z[3] * 4) / 4         # coarse grid: ties everywhere
    forced = np.full(rows, -1, np.int32)
    forced[5] = V - 1; forced[699] = 0
    got = _gpu_dist(B, z, K, T, forced=forced)
    for r in range(rows):
        want = oracle.dist(z[r], K, T, forced=int(forced[r]))
        assert np.array_equal(got[r].view(np.uint32), want.view(np.uint32)), (r, np.abs(got[r] - want).max())


def test_dist_ties_and_forced(B):
    _say("dist ties/forced")
    V = 3000
    z = synth.random_logits(4, V, seed=9)
    z[0, ::7] = 0.25                      # many equal values around the K-th
    z[1] = 0.0                            # everything ties
    z[2, 100:200] = z[2].max() + 1        # ties at the top
    z[3] = np.round(z[3] * 4) / 4         # coarse grid: ties everywhere
    for K in (1, 10, 429, 2000):
        got = _gpu_dist(B, z, K, 1.0)
        for r in range(4):
            want = oracle.dist(z[r], K, 1.0)
            assert np.array_equal(got[r].view(np.uint32), want.view(np.uint32)), (K, r)
            assert (got[r] > 0).sum() == min(K, V)
    got = _gpu_dist(B, z, 50, 1.0, forced=[5, -1, 2999, -1])
    assert got[0, 5] == 1.0 and got[0].sum() == 1.0 and got[2, 2999] == 1.0
    assert np.array_equal(got[1], oracle.dist(z[1], 50, 1.0))


def _rand_rows(rng, rows, V, support):
    out = np.zeros((rows, V), np.float32)
    for r in range(rows):
        idx = rng.choice(V, support, replace=False)
        e = np.exp(rng.standard_normal(support) * 1.3)
        out[r, idx] = (e / e.sum()).astype(np.float32)
    return out


def _run_verify_probs(B, q, p_old, draft, lo, init, img_pos0, hist, seed, counter, ring=None, alias=False):
    """ring (numpy [row_stride, V], sample-above only) is updated in place like the oracle's; alias: the
    next window is written over the current one, as the device-resident loop does"""
    L, V = p_old.shape
    dring = None if ring is None else _dev(ring)
    if alias:
        na = torch.zeros(1, dtype=torch.int32, device="cuda")
        nd = _dev(np.asarray(draft, np.int32)); pn = _dev(p_old)
        h = None if hist is None or len(hist) == 0 else _dev(np.asarray(hist, np.int32))
        B.sjd_verify_probs(_dev(q), pn, nd, L, V, lo, B.sjd_init(init.mode, init.row_stride, init.eol_id, init.flags),
                           img_pos0, h, seed, counter, na, nd, pn, ring=dring)
        torch.cuda.synchronize()
        if ring is not None:
            ring[...] = dring.cpu().numpy()
        return int(na.item()), nd.cpu().numpy(), pn.cpu().numpy()
    na = torch.zeros(1, dtype=torch.int32, device="cuda")
    nd = torch.zeros(L, dtype=torch.int32, device="cuda")
    pn = torch.zeros((L, V), dtype=torch.float32, device="cuda")
    h = None if hist is None or len(hist) == 0 else _dev(np.asarray(hist, np.int32))
    B.sjd_verify_probs(_dev(q), _dev(p_old), _dev(np.asarray(draft, np.int32)), L, V, lo,
                       B.sjd_init(init.mode, init.row_stride, init.eol_id, init.flags), img_pos0, h, seed, counter, na, nd, pn,
                       ring=dring)
    torch.cuda.synchronize()
    if ring is not None:
        ring[...] = dring.cpu().numpy()
    return int(na.item()), nd.cpu().numpy(), pn.cpu().numpy()


@pytest.mark.parametrize("L,V,support", [(2, 8, 6), (8, 1024, 64), (16, 8192, 2000), (32, 8192, 2000), (16, 16384, 2000),
                                         (5, 1000, 37), (32, 100, 100), (64, 8192, 2000), (64, 1000, 37), (47, 2048, 300)])
def test_verify_probs_bit_exact(B, L, V, support):
    rng = np.random.default_rng(L * 1000 + V)
    lo = 57344 if V == 8192 else 3
    accepted = []
    for case in range(6):
        _say(f"verify_probs L={L} V={V} case={case}")
        p_old = _rand_rows(rng, L, V, support)
        q = _rand_rows(rng, L + 1, V, support)
        # make several leading rows close to p_old so that the scan gets somewhere
        close = rng.integers(0, L)
        for i in range(1, close + 1):
            mix = np.float32(0.9) * p_old[i] + np.float32(0.1) * q[i]
            q[i] = mix
        if case == 5:
            q[:L] = p_old                                  # everything accepted
        draft = np.array([lo + rng.choice(V, p=p_old[i].astype(np.float64) / p_old[i].astype(np.float64).sum())
                          for i in range(L)], np.int32)
        init = oracle.Init(0, 0, -1)
        want = oracle.verify_probs(q, p_old, draft, lo, init, 11, None, 1234 + case, 40 + case)
        got = _run_verify_probs(B, q, p_old, draft, lo, init, 11, None, 1234 + case, 40 + case)
        assert got[0] == want[0]
        assert np.array_equal(got[1], want[1])
        assert np.array_equal(got[2].view(np.uint32), want[2].view(np.uint32))
        accepted.append(got[0])
    assert accepted[5] == L
    assert len(set(accepted)) > 1 or L == 2               # the cases do exercise different stopping points


@pytest.mark.parametrize("mode,stride,eol,flags", [(1, 8, -1, 0), (1, 3, -1, 0), (0, 7, 13, 0), (1, 5, 13, 0), (1, 1, -1, 0),
                                                   (2, 8, -1, 0), (2, 5, 13, 0), (0, 8, -1, 1), (2, 5, 13, 1), (1, 3, -1, 1),
                                                   (3, 8, -1, 0), (3, 5, 13, 0), (3, 4, 13, 1), (3, 2, 13, 0),
                                                   (4, 8, -1, 0), (4, 3, -1, 0), (4, 5, 13, 0), (4, 1, -1, 0),
                                                   (4, 3, -1, 1), (4, 16, -1, 0), (4, 2, 13, 1)])
def test_verify_probs_init_strategies(B, mode, stride, eol, flags):
    rng = np.random.default_rng(mode * 100 + stride)
    L, V, lo = 12, 64, 10
    for case in range(5):
        _say(f"verify init mode={mode} stride={stride} eol={eol} case={case}")
        img_pos0 = [0, 2, 9, 30, 31][case]
        hist = rng.integers(lo, lo + V, img_pos0).astype(np.int32)
        p_old = _rand_rows(rng, L, V, 20)
        q = _rand_rows(rng, L + 1, V, 20)
        for i in range(1, 1 + case * 2):
            q[i] = p_old[i]
        draft = np.array([lo + int(np.argmax(p_old[i])) for i in range(L)], np.int32)
        init = oracle.Init(mode, stride, eol, flags)
        ring_o = ring_g = None
        if mode == 4:                                      # distributions on record for earlier positions
            ring_o = _rand_rows(rng, stride, V, 20); ring_g = ring_o.copy()
        want = oracle.verify_probs(q, p_old, draft, lo, init, img_pos0, hist, 77, 5 + case, ring=ring_o)
        got = _run_verify_probs(B, q, p_old, draft, lo, init, img_pos0, hist, 77, 5 + case, ring=ring_g)
        assert got[0] == want[0]
        assert np.array_equal(got[1], want[1])
        assert np.array_equal(got[2].view(np.uint32), want[2].view(np.uint32))
        if mode == 4:
            assert np.array_equal(ring_g.view(np.uint32), ring_o.view(np.uint32))
        if mode >= 3:                                      # in place: index 0's carried row is recorded first
            ring_a = None if mode == 3 else _rand_rows(np.random.default_rng(mode * 100 + stride + 1000 * case), stride, V, 20)
            ring_b = None if ring_a is None else ring_a.copy()
            want = oracle.verify_probs(q, p_old, draft, lo, init, img_pos0, hist, 77, 5 + case, ring=ring_a)
            got = _run_verify_probs(B, q, p_old, draft, lo, init, img_pos0, hist, 77, 5 + case, ring=ring_b, alias=True)
            assert got[0] == want[0] and np.array_equal(got[1], want[1])
            assert np.array_equal(got[2].view(np.uint32), want[2].view(np.uint32))
            if mode == 4:
                assert np.array_equal(ring_b.view(np.uint32), ring_a.view(np.uint32))


@pytest.mark.parametrize("L,V,K", [(8, 1024, 64), (16, 8192, 2000), (32, 8192, 2000), (16, 16384, 2000), (64, 8192, 2000)])
def test_verify_from_logits_bit_exact(B, L, V, K):
    """the launch configuration of the real workloads (window x sampling vocabulary x top-K)"""
    rng = np.random.default_rng(V + L)
    lo = 57344 if V == 8192 else 0
    smp = oracle.Sampler(K, 1.0)
    for case in range(4):
        _say(f"verify logits L={L} V={V} K={K} case={case}")
        logits_prev = synth.random_logits(L, V, seed=100 + case)
        # p_old: what an earlier iteration would have carried = dist of slightly different logits
        p_old = np.stack([oracle.dist(logits_prev[i], K, 1.0) for i in range(L)])
        noise = synth.random_logits(L, V, seed=200 + case, std=0.05 * (case + 1))
        logits = np.concatenate([logits_prev[1:], synth.random_logits(1, V, seed=300 + case)]) + 0
        logits[:L - 1] += noise[:L - 1]
        draft = np.array([lo + oracle.sample(p_old[i], int(rng.integers(0, 2**32))) for i in range(L)], np.int32)
        init = oracle.Init(0, 32, -1)
        want = oracle.verify(logits, p_old, draft, lo, smp, init, 40, None, 99, 7 + case)
        na = torch.zeros(1, dtype=torch.int32, device="cuda")
        nd = torch.zeros(L, dtype=torch.int32, device="cuda")
        pn = torch.zeros((L, V), dtype=torch.float32, device="cuda")
        B.sjd_verify(_dev(logits), _dev(p_old), _dev(draft), L, V, lo, B.sjd_sampler(K, 1.0), B.sjd_init(0, 32, -1),
                     40, None, 99, 7 + case, na, nd, pn)
        torch.cuda.synchronize()
        assert int(na.item()) == want[0]
        assert np.array_equal(nd.cpu().numpy(), want[1])
        assert np.array_equal(pn.cpu().numpy().view(np.uint32), want[2].view(np.uint32))


def test_verify_aliasing_and_determinism(B):
    _say("verify alias")
    rng = np.random.default_rng(3)
    L, V, lo = 16, 2048, 0
    p_old = _rand_rows(rng, L, V, 300)
    q = _rand_rows(rng, L + 1, V, 300)
    q[1:4] = p_old[1:4]
    draft = np.array([int(np.argmax(p_old[i])) for i in range(L)], np.int32)
    init = oracle.Init(0, 0, -1)
    want = oracle.verify_probs(q, p_old, draft, lo, init, 0, None, 5, 6)
    # in place: new_draft aliases draft, p_new aliases p_old
    d = _dev(draft); p = _dev(p_old); na = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.sjd_verify_probs(_dev(q), p, d, L, V, lo, B.sjd_init(0, 0, -1), 0, None, 5, 6, na, d, p)
    torch.cuda.synchronize()
    assert int(na.item()) == want[0]
    assert np.array_equal(d.cpu().numpy(), want[1])
    assert np.array_equal(p.cpu().numpy().view(np.uint32), want[2].view(np.uint32))


def test_first_window(B):
    _say("first window")
    shape = synth.WORKLOADS["tiny"].shape
    blob = synth.make_weights(shape, seed=0)
    m = B.sjd_init_model(B.config_from_shape(shape), blob)
    try:
        V, lo = shape.v_s, shape.samp_lo
        q0 = oracle.dist(synth.random_logits(1, V, seed=1)[0], 64, 1.0)
        for mode, stride, eol, L in [(0, 8, -1, 8), (1, 3, -1, 8), (1, 4, 1000, 16), (0, 5, 7, 32), (2, 8, -1, 8), (2, 4, 1000, 16),
                                     (3, 8, -1, 8), (3, 4, 1000, 16), (3, 1, 1000, 4), (4, 3, -1, 8), (4, 4, 1000, 16),
                                     (4, 40, -1, 16), (4, 1, -1, 8)]:
            init = oracle.Init(mode, stride, eol)
            wd, wp = oracle.first_window(q0, L, lo, init, 31)
            d = torch.zeros(L, dtype=torch.int32, device="cuda")
            p = torch.zeros((L, V), dtype=torch.float32, device="cuda")
            B.sjd_first_window(m, _dev(q0), L, B.sjd_init(mode, stride, eol), 31, d, p)
            torch.cuda.synchronize()
            assert np.array_equal(d.cpu().numpy(), wd)
            assert np.array_equal(p.cpu().numpy().view(np.uint32), wp.view(np.uint32))
    finally:
        B.sjd_free_model(m)


def test_argument_errors(B):
    _say("verify arg errors")
    L, V = 4, 64
    z = torch.zeros((L, V), device="cuda"); d = torch.zeros(L, dtype=torch.int32, device="cuda")
    na = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(B.SjdError) as e:
        B.sjd_verify(z, z, d, 0, V, 0, B.sjd_sampler(5, 1.0), B.sjd_init(0, 0, -1), 0, None, 1, 1, na, d, z)
    assert e.value.code == B.SJD_EINVAL
    with pytest.raises(B.SjdError):
        B.sjd_verify(z, z, d, L, V, 0, B.sjd_sampler(0, 1.0), B.sjd_init(0, 0, -1), 0, None, 1, 1, na, d, z)
    with pytest.raises(B.SjdError):
        B.sjd_verify(z, z, d, L, B.SJD_MAX_SAMP_VOCAB + 1, 0, B.sjd_sampler(5, 1.0), B.sjd_init(0, 0, -1), 0, None, 1, 1,
                     na, d, z)
    with pytest.raises(B.SjdError):                       # sample-above needs the ring
        B.sjd_verify(z, z, d, L, V, 0, B.sjd_sampler(5, 1.0), B.sjd_init(4, 8, -1), 0, None, 1, 1, na, d, z)
    with pytest.raises(B.SjdError):                       # unknown initialiser
        B.sjd_verify(z, z, d, L, V, 0, B.sjd_sampler(5, 1.0), B.sjd_init(5, 8, -1), 0, None, 1, 1, na, d, z)
    with pytest.raises(B.SjdError):                       # repeat-above needs the history
        B.sjd_verify(z, z, d, L, V, 0, B.sjd_sampler(5, 1.0), B.sjd_init(1, 8, -1), 9, None, 1, 1, na, d, z)
