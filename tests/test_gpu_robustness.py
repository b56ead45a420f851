"""GPU: bad device-side input ends in an error code (every kernel still exits normally), and a
generation resumes bit-exactly from its persisted state (sjd_step is a pure function of the cache,
the window, its distributions, the seed and the step counter)."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import oracle  # noqa: E402,F401  (the checker is built with the rest; these tests compare GPU runs with each other)
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


@pytest.mark.parametrize("dtype", [synth.DTYPE_F32, synth.DTYPE_BF16])
def test_token_id_outside_the_vocabulary_is_an_error_not_a_fault(B, dtype):
    _say(f"bad token id dtype={dtype}")
    shape = synth.ModelShape(2, 128, 4, 256, 512, 0, 512, 96, dtype)
    blob = synth.make_weights(shape, seed=3)
    m = B.sjd_init_model(B.config_from_shape(shape), blob)
    kv = B.sjd_kv_create(m)
    try:
        smp, init = B.sjd_sampler(50, 1.0), B.sjd_init(0, 8, -1)
        q = torch.empty(shape.v_s, dtype=torch.float32, device="cuda")
        prompt = synth.random_tokens(9, 0, 512, seed=1)
        B.sjd_prefill(m, kv, prompt, None, smp, init, q)
        L = 8
        out = torch.empty((L, shape.v_s), dtype=torch.float32, device="cuda")
        good = synth.random_tokens(L, 0, 512, seed=2)
        B.sjd_forward_logits(m, kv, _dev(good), L, out)
        assert B.sjd_kv_len(kv) == 9
        ref = out.cpu().numpy().copy()
        for bad_id in (512, -1, 2**30):
            bad = good.copy(); bad[3] = bad_id
            B.sjd_forward_logits(m, kv, _dev(bad), L, out)      # enqueues fine: the ids live on the device
            torch.cuda.synchronize()                            # ... and every kernel finishes
            with pytest.raises(B.SjdError) as e:
                B.sjd_kv_len(kv)
            assert e.value.code == B.SJD_EINVAL
            # rows in front of the bad one are untouched by it (causal), and nothing is NaN-poisoned there
            assert np.array_equal(out.cpu().numpy()[:3], ref[:3])
            # the handle works again after a new prefill
            B.sjd_prefill(m, kv, prompt, None, smp, init, q)
            B.sjd_forward_logits(m, kv, _dev(good), L, out)
            assert B.sjd_kv_len(kv) == 9
            assert np.array_equal(out.cpu().numpy(), ref)
    finally:
        B.sjd_kv_free(kv); B.sjd_free_model(m)


def test_step_with_image_position_beyond_the_cache_is_refused(B):
    _say("img_pos0 beyond the cache")
    shape = synth.ModelShape(2, 128, 4, 256, 512, 0, 512, 96, synth.DTYPE_F32)
    blob = synth.make_weights(shape, seed=3)
    m = B.sjd_init_model(B.config_from_shape(shape), blob)
    kv = B.sjd_kv_create(m)
    try:
        smp, init = B.sjd_sampler(50, 1.0), B.sjd_init(1, 8, -1)      # repeat-above reads earlier image tokens
        V, L = shape.v_s, 8
        q = torch.empty(V, dtype=torch.float32, device="cuda")
        B.sjd_prefill(m, kv, synth.random_tokens(9, 0, 512, seed=1), None, smp, init, q)
        draft = torch.zeros(L, dtype=torch.int32, device="cuda")
        p_old = torch.zeros((L, V), dtype=torch.float32, device="cuda")
        B.sjd_first_window(m, q, L, init, 5, draft, p_old)
        na = torch.full((1,), -3, dtype=torch.int32, device="cuda")
        nd = torch.zeros_like(draft); pn = torch.zeros_like(p_old)
        # far beyond anything the cache can hold: refused on the host
        with pytest.raises(B.SjdError) as e:
            B.sjd_step(m, kv, draft, p_old, L, smp, init, 10_000, 5, 1, na, nd, pn)
        assert e.value.code == B.SJD_EINVAL
        # the host only keeps an upper bound of the device-resident length: after a step it is n + L, so
        # a position between the true length and the bound is caught by the kernels
        B.sjd_step(m, kv, draft, p_old, L, smp, init, 0, 5, 1, na, nd, pn)
        torch.cuda.synchronize()
        a = int(na.item())
        assert 1 <= a <= L
        if a == L:
            pytest.skip("the whole window was accepted: the host bound equals the true length")
        # the host now believes n <= 9 + L while n = 9 + a: position 9 + a + 1 passes the host check
        na.fill_(-3)
        B.sjd_step(m, kv, nd, pn, L, smp, init, 9 + a + 1, 5, 2, na, draft, p_old)
        torch.cuda.synchronize()
        assert int(na.item()) == -3                                   # the step was not executed
        with pytest.raises(B.SjdError) as e:
            B.sjd_kv_len(kv)
        assert e.value.code == B.SJD_EINVAL
    finally:
        B.sjd_kv_free(kv); B.sjd_free_model(m)


def _run_steps(B, m, kv, draft, p_old, L, smp, init, img_pos0, seed, c0, n_steps, V):
    """n_steps iterations of sjd_step; returns per-step (accepted, new window ids, new distributions' bits)"""
    na = torch.zeros(1, dtype=torch.int32, device="cuda")
    d = draft.clone(); p = p_old.clone()
    nd = torch.zeros_like(d); pn = torch.zeros_like(p)
    trace, fixed = [], []
    for c in range(c0, c0 + n_steps):
        B.sjd_step(m, kv, d, p, L, smp, init, img_pos0, seed, c, na, nd, pn)
        torch.cuda.synchronize()
        a = int(na.item())
        fixed += d.cpu().numpy()[:a].tolist()
        img_pos0 += a
        trace.append((a, nd.cpu().numpy().copy(), pn.cpu().numpy().view(np.uint32).copy()))
        d, nd = nd, d; p, pn = pn, p
    return trace, fixed, d, p, img_pos0


@pytest.mark.parametrize("dtype,mode", [(synth.DTYPE_BF16, 0), (synth.DTYPE_BF16, 1), (synth.DTYPE_F32, 2)])
def test_resume_from_persisted_state_is_bit_exact(B, dtype, mode):
    """Persist (cache length, window ids, their distributions, step counter, image position) in the
    middle of a generation; roll the same handle back to it, and rebuild it in a NEW handle by
    pre-filling prompt + accepted tokens: both continue with exactly the iterations the first run
    made (accepted counts, ids, and every bit of the distributions)."""
    _say(f"resume dtype={dtype} mode={mode}")
    shape = synth.ModelShape(2, 256, 4, 512, 2048, 1024, 2048, 200, dtype)
    blob = synth.make_weights(shape, seed=8)
    m = B.sjd_init_model(B.config_from_shape(shape), blob)
    kv = B.sjd_kv_create(m)
    kv2 = B.sjd_kv_create(m)
    try:
        V, lo, L, seed = shape.v_s, shape.samp_lo, 8, 42
        smp, init = B.sjd_sampler(300, 1.0), B.sjd_init(mode, 8, -1)
        prompt = synth.random_tokens(20, 0, 1024, seed=1)
        q = torch.empty(V, dtype=torch.float32, device="cuda")
        B.sjd_prefill(m, kv, prompt, None, smp, init, q)
        draft = torch.zeros(L, dtype=torch.int32, device="cuda")
        p_old = torch.zeros((L, V), dtype=torch.float32, device="cuda")
        B.sjd_first_window(m, q, L, init, seed, draft, p_old)
        # 5 iterations, persist, 6 more
        _, fixed, d5, p5, pos5 = _run_steps(B, m, kv, draft, p_old, L, smp, init, 0, seed, 1, 5, V)
        n5 = B.sjd_kv_len(kv)
        assert n5 == 20 + pos5 == 20 + len(fixed)
        saved = (d5.cpu().numpy().copy(), p5.cpu().numpy().copy())
        want, _, _, _, _ = _run_steps(B, m, kv, d5, p5, L, smp, init, pos5, seed, 6, 6, V)

        # (1) the same handle rolled back
        B.sjd_kv_set_len(kv, n5)
        got, _, _, _, _ = _run_steps(B, m, kv, _dev(saved[0]), _dev(saved[1]), L, smp, init, pos5, seed, 6, 6, V)
        for (a, nd, pn), (a2, nd2, pn2) in zip(want, got):
            assert a == a2 and np.array_equal(nd, nd2) and np.array_equal(pn, pn2)

        # (2) a new handle: the cache is rebuilt from the ids (prompt + accepted image tokens)
        B.sjd_prefill(m, kv2, np.concatenate([prompt, np.array(fixed, np.int32)]), None, smp, init, q)
        assert B.sjd_kv_len(kv2) == n5
        got, _, _, _, _ = _run_steps(B, m, kv2, _dev(saved[0]), _dev(saved[1]), L, smp, init, pos5, seed, 6, 6, V)
        for (a, nd, pn), (a2, nd2, pn2) in zip(want, got):
            assert a == a2 and np.array_equal(nd, nd2)
            # the rebuilt cache rows come from prompt-sized row chunks instead of windows: equal values up to
            # summation order, so the distributions agree to rounding rather than bit for bit
            assert np.abs(pn.view(np.float32) - pn2.view(np.float32)).max() < (1e-5 if dtype == synth.DTYPE_F32 else 2e-3)
    finally:
        B.sjd_kv_free(kv); B.sjd_kv_free(kv2); B.sjd_free_model(m)


@pytest.mark.parametrize("use_graph", [True, False])
def test_two_handles_on_two_streams_from_two_host_threads(B, use_graph):
    """Handles of one model are independent: two host threads, each decoding an image on its own handle and its
    own stream at the same time (prefill, the device-resident loop in pieces, status polls in between), get exactly
    the tokens each gets when it runs alone."""
    import threading
    _say(f"two threads, two streams, graph={use_graph}")
    shape = synth.ModelShape(3, 256, 4, 512, 2048, 1024, 2048, 260, synth.DTYPE_BF16)
    blob = synth.make_weights(shape, seed=8)
    m = B.sjd_init_model(B.config_from_shape(shape), blob)
    kvs = [B.sjd_kv_create(m) for _ in range(2)]
    try:
        V, L, N = shape.v_s, 16, 150
        smp, init = B.sjd_sampler(300, 1.0), B.sjd_init(1, 10, 2047)
        prompts = [synth.random_tokens(20 + 30 * i, 0, 1024, seed=3 + i) for i in range(2)]

        def decode(i, stream, out, errs):
            try:
                q = qs[i]
                B.sjd_kv_use_graph(kvs[i], use_graph)
                B.sjd_prefill(m, kvs[i], prompts[i], None, smp, init, q, stream=stream)
                B.sjd_decode_begin(m, kvs[i], q, N, L, smp, init, 100 + i, stream=stream)
                done, guard = False, 0
                while not done:
                    B.sjd_decode_steps(m, kvs[i], 3, stream=stream)
                    _, _, done = B.sjd_decode_status(kvs[i])
                    guard += 1
                    assert guard < 4 * N
                toks, st = B.sjd_decode_result(kvs[i], N)
                out[i] = (toks.copy(), st.steps)
            except Exception as e:                      # noqa: BLE001  (reported by the main thread)
                errs.append((i, repr(e)))

        streams = [torch.cuda.Stream() for _ in range(2)]
        qs = [torch.empty(V, dtype=torch.float32, device="cuda") for _ in range(2)]     # (allocated up front)
        torch.cuda.synchronize()
        alone, errs = {}, []
        for i in range(2):
            decode(i, streams[i], alone, errs)
        assert not errs, errs
        for rep in range(2):
            both = {}
            th = [threading.Thread(target=decode, args=(i, streams[i], both, errs)) for i in range(2)]
            for t in th:
                t.start()
            for t in th:
                t.join(timeout=120)
            assert not errs, errs
            for i in range(2):
                assert i in both, "a thread did not finish"
                assert np.array_equal(both[i][0], alone[i][0]) and both[i][1] == alone[i][1], (rep, i)
    finally:
        torch.cuda.synchronize()
        for kv in kvs:
            B.sjd_kv_free(kv)
        B.sjd_free_model(m)
