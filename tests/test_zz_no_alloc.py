"""GPU: the entry point that allocates nothing (sjd_verify_static) against sjd_verify.

Two calls in a row through the C ABI, the second on a smaller input, so that whatever the first call
left in the library's static scratch array must not leak into the second.  Bar: bit-exact (accepted
count, token ids, every fp32 probability), as for the rest of the verification.
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


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _case(L, V, K, seed, lo):
    rng = np.random.default_rng(seed)
    logits_prev = synth.random_logits(L, V, seed=100 + seed)
    p_old = np.stack([oracle.dist(logits_prev[i], K, 1.0) for i in range(L)])
    logits = np.concatenate([logits_prev[1:], synth.random_logits(1, V, seed=300 + seed)]) + 0
    logits[:L - 1] += synth.random_logits(L, V, seed=200 + seed, std=0.1)[:L - 1]
    draft = np.array([lo + oracle.sample(p_old[i], int(rng.integers(0, 2**32))) for i in range(L)], np.int32)
    return logits, p_old, draft


def _run(fn, B, logits, p_old, draft, L, V, lo, K, init, img_pos0, hist, seed, counter, ring=None):
    na = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    nd = torch.full((L,), -7, dtype=torch.int32, device="cuda")
    pn = torch.full((L, V), -7.0, dtype=torch.float32, device="cuda")
    fn(_dev(logits), _dev(p_old), _dev(draft), L, V, lo, B.sjd_sampler(K, 1.0), init, img_pos0,
       None if hist is None else _dev(hist), seed, counter, na, nd, pn, ring=ring)
    torch.cuda.synchronize()
    return int(na.item()), nd.cpu().numpy(), pn.cpu().numpy()


def test_static_verify_equals_allocating_verify_twice_in_a_row(B):
    # first call: the 7B launch configuration (fills most of the static scratch); second: a much
    # smaller window and vocabulary with another initialiser
    calls = [(32, 8192, 2000, 57344, B.sjd_init(0, 49, 65535, 0), 40, None),
             (5, 1000, 64, 0, B.sjd_init(1, 7, -1, 0), 9, np.arange(9, dtype=np.int32) * 3 % 1000)]
    for idx, (L, V, K, lo, init, img_pos0, hist) in enumerate(calls):
        print(f"static verify call {idx}: L={L} V={V}", flush=True, file=sys.stderr)
        logits, p_old, draft = _case(L, V, K, 11 + idx, lo)
        want = _run(B.sjd_verify, B, logits, p_old, draft, L, V, lo, K, init, img_pos0, hist, 99, 7 + idx)
        got = _run(B.sjd_verify_static, B, logits, p_old, draft, L, V, lo, K, init, img_pos0, hist, 99, 7 + idx)
        assert got[0] == want[0] and 1 <= got[0] <= L
        assert np.array_equal(got[1], want[1])
        assert np.array_equal(got[2].view(np.uint32), want[2].view(np.uint32))
        # and both equal the oracle
        ref = oracle.verify(logits, p_old, draft, lo, oracle.Sampler(K, 1.0),
                            oracle.Init(init.mode, init.row_stride, init.eol_id), img_pos0, hist, 99, 7 + idx)
        assert got[0] == ref[0] and np.array_equal(got[1], ref[1])
        assert np.array_equal(got[2].view(np.uint32), ref[2].view(np.uint32))


def test_static_verify_rejects_sizes_beyond_its_scratch(B):
    L, V = 32, 16384                    # 33 x 16384 floats > SJD_STATIC_VERIFY_FLOATS
    assert (L + 1) * V > B.SJD_STATIC_VERIFY_FLOATS
    z = torch.zeros((L, V), dtype=torch.float32, device="cuda")
    d = torch.zeros(L, dtype=torch.int32, device="cuda")
    na = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(B.SjdError) as e:
        B.sjd_verify_static(z, z, d, L, V, 0, B.sjd_sampler(10, 1.0), B.sjd_init(0, 0, -1, 0), 0, None, 1, 1, na, d,
                            torch.empty_like(z))
    assert e.value.code == B.SJD_ELIMIT and "static scratch" in str(e.value)
