"""GPU parity of classifier-free guidance: two contexts share every window forward, Step 3 works on
z = z_u + w (z_c - z_u)  (Sec. 5.1 gives the weight; logit-space guidance is the assumed mechanism).

The oracle side is two independent transformer oracles (one per context) whose logits are combined by
oracle.guide.  Bars as elsewhere: the guided logits themselves stay within 1e-4 (fp32 models) / 2e-2 (bf16
models) of the oracle's, although the combination amplifies the error of each forward by up to |w| + |1 - w|.
"""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import oracle  # noqa: E402
from paper_2410_01699_amd import synth  # noqa: E402

TOL_F32 = 1e-4
TOL_BF16 = 2e-2


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


class Pair:
    """GPU handle with both contexts pre-filled + one oracle model per context"""

    def __init__(self, B, shape, blob, prompt_c, prompt_u, w, smp, init, emb_c=None):
        self.B, self.shape, self.w = B, shape, w
        self.m = B.sjd_init_model(B.config_from_shape(shape), blob)
        self.kv = B.sjd_kv_create(self.m)
        self.oc, self.ou = oracle.Model(shape, blob), oracle.Model(shape, blob)
        self.q_last = torch.empty(shape.v_s, dtype=torch.float32, device="cuda")
        B.sjd_prefill(self.m, self.kv, prompt_c, emb_c, smp, init, self.q_last)
        B.sjd_prefill_uncond(self.m, self.kv, prompt_u, None, w, smp, init, self.q_last)
        torch.cuda.synchronize()
        self.Pc = len(prompt_c) + (0 if emb_c is None else len(emb_c))
        self.Pu = len(prompt_u)
        self.lp = oracle.guide(self.oc.prefill(prompt_c, emb_c), self.ou.prefill(prompt_u), w)

    def close(self):
        self.B.sjd_kv_free(self.kv); self.B.sjd_free_model(self.m)
        self.oc.close(); self.ou.close()

    def gpu_logits(self, tokens):
        L = len(tokens)
        out = torch.empty((L, self.shape.v_s), dtype=torch.float32, device="cuda")
        self.B.sjd_forward_logits(self.m, self.kv, _dev(np.asarray(tokens, np.int32)), L, out)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def ref_logits(self, n_img, tokens):
        """guided logits with n_img image tokens fixed behind both prompts"""
        zc = self.oc.forward_tokens(self.Pc + n_img, tokens)
        zu = self.ou.forward_tokens(self.Pu + n_img, tokens)
        return oracle.guide(zc, zu, self.w)


@pytest.mark.parametrize("case", ["tiny_fp32", "small_bf16", "hd128_bf16", "7b_dims_bf16", "7b_full_bf16"])
def test_guided_window_logits(B, case):
    if case == "tiny_fp32":
        shape = synth.WORKLOADS["tiny"].shape
        blob = synth.make_weights(shape, seed=0)
        pc = synth.random_tokens(9, 0, shape.samp_lo or 1024, seed=1)
        pu = synth.random_tokens(3, 0, shape.samp_lo or 1024, seed=2)
        tol, w = TOL_F32, 3.0
    elif case == "small_bf16":
        shape = synth.ModelShape(4, 256, 4, 512, 2048, 1024, 2048, 200, synth.DTYPE_BF16)
        blob = synth.make_weights(shape, seed=7)
        pc = synth.random_tokens(45, 0, 1024, seed=1)
        pu = synth.random_tokens(7, 0, 1024, seed=2)
        tol, w = TOL_BF16, 3.0
    elif case == "hd128_bf16":
        # a long conditional prompt (many key splits) against a one-token unconditional one
        shape = synth.ModelShape(2, 512, 4, 1024, 4096, 2048, 4096, 800, synth.DTYPE_BF16)
        blob = synth.make_weights(shape, seed=11)
        pc = synth.random_tokens(600, 0, 2048, seed=1)
        pu = synth.random_tokens(1, 0, 2048, seed=2)
        tol, w = TOL_BF16, 7.5
    elif case == "7b_full_bf16":
        # the paper's guided setup at its real shape (Sec. 5.1: 7B model, guidance weight 3, window 32): two
        # contexts x 32 rows = a 64-row forward through all 32 layers
        shape = synth.WORKLOADS["7b_48x48"].shape
        blob = synth.make_weights(shape, seed=0, threads=16)
        pc = synth.random_tokens(40, 0, shape.samp_lo, seed=1)
        pu = synth.random_tokens(9, 0, shape.samp_lo, seed=2)
        tol, w = TOL_BF16, 3.0
    else:
        shape = synth.ModelShape(2, 4096, 32, 11008, 65536, 57344, 65536, 200, synth.DTYPE_BF16)
        blob = synth.make_weights(shape, seed=0, threads=16)
        pc = synth.random_tokens(70, 0, 57344, seed=1)
        pu = synth.random_tokens(33, 0, 57344, seed=2)
        tol, w = TOL_BF16, 3.0
    smp = B.sjd_sampler(8, 1.0); init = B.sjd_init(0, 0, -1)
    _say(f"guided logits {case}")
    p = Pair(B, shape, blob, pc, pu, w, smp, init)
    try:
        assert B.sjd_kv_len(p.kv) == p.Pc
        if tol <= TOL_F32:
            q_ref = oracle.dist(p.lp, 8, 1.0)
            assert np.max(np.abs(p.q_last.cpu().numpy() - q_ref)) < 1e-5
        toks = synth.random_tokens(64, shape.samp_lo, shape.samp_hi, seed=3)
        n_img, worst = 0, 0.0
        windows = [(0, 16, 5), (16, 21, 5), (21, 22, 1), (22, 38, 16), (38, 47, 2)]
        if shape.dtype == synth.DTYPE_BF16:
            # two contexts of 32, 17 and 64 rows: the wide projection kernel, attention in groups of 32 queries
            windows += [(0, 32, 3), (32, 49, 17), (0, 64, 1)]
        if case == "7b_full_bf16":
            windows = [(0, 32, 3), (32, 48, 5)]          # (two fp64 oracles of 32 layers: keep it to two windows)
        for lo_, hi_, keep in windows:
            t = toks[lo_:hi_]
            _say(f"  window at image position {n_img} L={len(t)}")
            got = p.gpu_logits(t)
            ref = p.ref_logits(n_img, t)
            err = float(np.max(np.abs(got - ref)))
            worst = max(worst, err)
            assert err < tol, (n_img, err)
            n_img += keep
            B.sjd_kv_set_len(p.kv, p.Pc + n_img)       # moves both caches
        _say(f"  worst guided-logit error {worst:.3e} (bar {tol:.1e})")
    finally:
        p.close()


def test_guided_logits_with_embedding_row_prompts(B):
    """class-conditional style contexts: one id + raw embedding rows on the conditional side (crossing a
    32-position chunk boundary), a single id on the unconditional side"""
    shape = synth.ModelShape(3, 384, 6, 1024, 4096, 0, 4096, 140, synth.DTYPE_BF16)
    blob = synth.make_weights(shape, seed=3)
    rng = np.random.default_rng(4)
    emb = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits((rng.standard_normal((40, 384)) * 0.02).astype(np.float32))).reshape(40, 384)
    pc = np.array([7], np.int32); pu = np.array([9], np.int32)
    smp = B.sjd_sampler(8, 1.0); init = B.sjd_init(0, 0, -1)
    w = 3.0
    p = Pair(B, shape, blob, pc, pu, w, smp, init, emb_c=emb)
    try:
        assert p.Pc == 41 and B.sjd_kv_len(p.kv) == 41
        toks = synth.random_tokens(32, 0, 4096, seed=5)
        n_img = 0
        for lo_, hi_, keep in ((0, 16, 16), (16, 27, 4), (27, 32, 5)):
            got = p.gpu_logits(toks[lo_:hi_])
            ref = p.ref_logits(n_img, toks[lo_:hi_])
            err = float(np.max(np.abs(got - ref)))
            assert err < TOL_BF16, (n_img, err)
            n_img += keep
            B.sjd_kv_set_len(p.kv, p.Pc + n_img)
    finally:
        p.close()


def test_guidance_weight_zero_and_one(B):
    """w = 0 gives the unconditional context's logits (an ordinary one-context forward of the second
    prompt), w = 1 the conditional one's"""
    shape = synth.ModelShape(2, 256, 4, 512, 2048, 1024, 2048, 120, synth.DTYPE_BF16)
    blob = synth.make_weights(shape, seed=7)
    pc = synth.random_tokens(30, 0, 1024, seed=1); pu = synth.random_tokens(11, 0, 1024, seed=2)
    toks = synth.random_tokens(16, 1024, 2048, seed=3)
    smp = B.sjd_sampler(8, 1.0); init = B.sjd_init(0, 0, -1)
    m = B.sjd_init_model(B.config_from_shape(shape), blob)
    kv = B.sjd_kv_create(m)
    try:
        q = torch.empty(shape.v_s, dtype=torch.float32, device="cuda")
        out = torch.empty((16, shape.v_s), dtype=torch.float32, device="cuda")
        single = {}
        for name, prompt in (("c", pc), ("u", pu)):
            B.sjd_prefill(m, kv, prompt, None, smp, init, q)
            B.sjd_forward_logits(m, kv, _dev(toks), 16, out)
            torch.cuda.synchronize()
            single[name] = out.cpu().numpy().copy()
        for w in (0.0, 1.0):
            B.sjd_prefill(m, kv, pc, None, smp, init, q)
            B.sjd_prefill_uncond(m, kv, pu, None, w, smp, init, q)
            B.sjd_forward_logits(m, kv, _dev(toks), 16, out)
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            # each stream of the two-stream forward is an ordinary forward of its context up to the
            # summation order of the projections (32-row launches split K over more waves): far inside
            # the bf16 bar, so a stream reading the wrong cache, length or rows cannot hide
            ref = oracle.guide(single["c"], single["u"], w)
            assert np.max(np.abs(got - ref)) < 1e-3, w
            if w == 0.0:
                assert np.max(np.abs(got - single["u"])) < 1e-3
            else:
                assert np.max(np.abs(got - single["c"])) < 1e-3
    finally:
        B.sjd_kv_free(kv); B.sjd_free_model(m)


@pytest.mark.parametrize("L", [16, 32, 64])
def test_cfg_step_bit_exact_given_gpu_logits(B, L):
    """sjd_step under guidance: verification of the guided logits is bit-exact, and both caches advance
    by the accepted count (the next window's guided logits stay on the oracle's).  Windows of 32 and 64
    make forwards of 64 and 128 rows."""
    shape = synth.ModelShape(2, 256, 4, 512, 2048, 1024, 2048, 600, synth.DTYPE_BF16)
    blob = synth.make_weights(shape, seed=8)
    V, lo, K, w = shape.v_s, shape.samp_lo, 300, 3.0
    smp = B.sjd_sampler(K, 1.0); init = B.sjd_init(1, 16, 2047)
    osmp = oracle.Sampler(K, 1.0); oinit = oracle.Init(1, 16, 2047)
    p = Pair(B, shape, blob, synth.random_tokens(20, 0, 1024, seed=1), synth.random_tokens(6, 0, 1024, seed=2), w,
             smp, init)
    try:
        draft = torch.zeros(L, dtype=torch.int32, device="cuda")
        p_old = torch.zeros((L, V), dtype=torch.float32, device="cuda")
        B.sjd_first_window(p.m, p.q_last, L, init, 42, draft, p_old)
        na = torch.zeros(1, dtype=torch.int32, device="cuda")
        nd = torch.zeros(L, dtype=torch.int32, device="cuda"); pn = torch.zeros_like(p_old)
        hist = []
        for c in range(1, 9):
            _say(f"  guided step {c} fixed={len(hist)}")
            d_h, p_h = draft.cpu().numpy(), p_old.cpu().numpy()
            logits = p.gpu_logits(d_h)                          # guided logits of the same forward
            err = float(np.max(np.abs(logits - p.ref_logits(len(hist), d_h))))
            assert err < TOL_BF16, (c, err)
            want = oracle.verify(logits, p_h, d_h, lo, osmp, oinit, len(hist), np.array(hist, np.int32), 42, c)
            B.sjd_step(p.m, p.kv, draft, p_old, L, smp, init, len(hist), 42, c, na, nd, pn)
            torch.cuda.synchronize()
            a = int(na.item())
            assert a == want[0]
            assert np.array_equal(nd.cpu().numpy(), want[1])
            assert np.array_equal(pn.cpu().numpy().view(np.uint32), want[2].view(np.uint32))
            hist += d_h[:a].tolist()
            assert B.sjd_kv_len(p.kv) == p.Pc + len(hist)
            draft, nd = nd, draft; p_old, pn = pn, p_old
    finally:
        p.close()


@pytest.mark.parametrize("L,w,mode", [(8, 3.0, 0), (16, 3.0, 1), (1, 3.0, 0), (5, 0.0, 2), (16, 7.5, 0)])
def test_generate_cfg_tiny_fp32_token_identity(B, L, w, mode):
    wl = synth.WORKLOADS["tiny"]
    shape = wl.shape
    blob = synth.make_weights(shape, seed=0)
    pc, _ = synth.make_prompt(wl)
    pu = synth.random_tokens(2, 0, 1024, seed=9)
    oc, ou = oracle.Model(shape, blob), oracle.Model(shape, blob)
    m = B.sjd_init_model(B.config_from_shape(shape), blob)
    kv = B.sjd_kv_create(m)
    try:
        N = wl.n_image_tokens
        osmp = oracle.Sampler(wl.top_k, wl.temperature); oinit = oracle.Init(mode, wl.row_stride, -1, 0)
        Pc, Pu = len(pc), len(pu)

        def fwd(n_fixed, toks):
            k = n_fixed - Pc
            return oracle.guide(oc.forward_tokens(n_fixed, toks), ou.forward_tokens(Pu + k, toks), w)

        for seed in range(2):
            _say(f"generate cfg tiny L={L} w={w} mode={mode} seed={seed}")
            lp = oracle.guide(oc.prefill(pc), ou.prefill(pu), w)
            want, wst = oracle.generate_sjd_callback(fwd, Pc, lp, shape.v_s, shape.samp_lo, N, L, osmp, oinit, seed)
            got, st = B.sjd_generate_cfg(m, kv, pc, None, pu, None, w, N, L, B.sjd_sampler(wl.top_k, wl.temperature),
                                         B.sjd_init(mode, wl.row_stride, -1, 0), seed)
            assert np.array_equal(got, want), (seed, np.nonzero(got != want)[0][:5])
            assert st.steps == wst.steps
            assert list(st.accept_hist) == list(wst.accept_hist)
        if w == 0.0:
            # no weight on the condition: the same tokens as an unguided run from the second prompt
            plain, _ = B.sjd_generate(m, kv, pu, None, N, L, B.sjd_sampler(wl.top_k, wl.temperature),
                                      B.sjd_init(mode, wl.row_stride, -1, 0), 1)
            assert np.array_equal(plain, got)
    finally:
        B.sjd_kv_free(kv); B.sjd_free_model(m); oc.close(); ou.close()


def test_cfg_graph_replay_and_switching_off(B):
    """guided loop: captured iteration == kernel-by-kernel path; an unguided generation on the same
    handle before and after a guided one gives the same tokens (guidance state does not leak)"""
    shape = synth.ModelShape(3, 512, 8, 1024, 4096, 2048, 4096, 400, synth.DTYPE_BF16)
    blob = synth.make_weights(shape, seed=9)
    m = B.sjd_init_model(B.config_from_shape(shape), blob)
    kv = B.sjd_kv_create(m)
    try:
        pc = synth.random_tokens(40, 0, 2048, seed=1); pu = synth.random_tokens(5, 0, 2048, seed=2)
        smp = B.sjd_sampler(500, 1.0); init = B.sjd_init(0, 16, -1)
        B.sjd_kv_use_graph(kv, True)
        plain0, s0 = B.sjd_generate(m, kv, pc, None, 150, 16, smp, init, 1)
        outs = []
        for use_graph in (True, False, True):
            B.sjd_kv_use_graph(kv, use_graph)
            for w in (3.0, 1.5):
                _say(f"cfg graph={use_graph} w={w}")
                t, st = B.sjd_generate_cfg(m, kv, pc, None, pu, None, w, 150, 16, smp, init, 1)
                outs.append((use_graph, w, t, st.steps))
        ref = {w: (t, n) for ug, w, t, n in outs if not ug}
        for ug, w, t, n in outs:
            assert np.array_equal(t, ref[w][0]) and n == ref[w][1], (ug, w)
            assert t.min() >= 2048 and t.max() < 4096
        assert not np.array_equal(ref[3.0][0], ref[1.5][0])          # the weight matters
        assert not np.array_equal(ref[3.0][0], plain0)
        plain1, s1 = B.sjd_generate(m, kv, pc, None, 150, 16, smp, init, 1)
        assert np.array_equal(plain0, plain1) and s0.steps == s1.steps
    finally:
        B.sjd_kv_free(kv); B.sjd_free_model(m)


def test_cfg_errors(B):
    wl = synth.WORKLOADS["tiny"]
    shape = wl.shape
    blob = synth.make_weights(shape, seed=0)
    m = B.sjd_init_model(B.config_from_shape(shape), blob)
    kv = B.sjd_kv_create(m)
    try:
        V = shape.v_s
        smp = B.sjd_sampler(64, 1.0); init = B.sjd_init(0, 8, -1)
        q = torch.empty(V, dtype=torch.float32, device="cuda")
        pc = synth.random_tokens(4, 0, 1024, seed=1)
        with pytest.raises(B.SjdError) as e:              # no conditional prompt yet
            B.sjd_prefill_uncond(m, kv, pc, None, 3.0, smp, init, q)
        assert e.value.code == B.SJD_EINVAL
        B.sjd_prefill(m, kv, pc, None, smp, init, q)
        B.sjd_prefill_uncond(m, kv, pc, None, 3.0, smp, init, q)
        with pytest.raises(B.SjdError) as e:              # a second unconditional prompt
            B.sjd_prefill_uncond(m, kv, pc, None, 3.0, smp, init, q)
        assert e.value.code == B.SJD_EINVAL
        d = torch.zeros(32, dtype=torch.int32, device="cuda"); p = torch.zeros((32, V), device="cuda")
        na = torch.zeros(1, dtype=torch.int32, device="cuda")
        with pytest.raises(B.SjdError) as e:              # windows above 16 tokens under guidance
            B.sjd_step(m, kv, d, p, 17, smp, init, 0, 1, 1, na, d, p)
        assert e.value.code == B.SJD_EINVAL
        with pytest.raises(B.SjdError) as e:
            B.sjd_generate_cfg(m, kv, pc, None, pc, None, 3.0, 64, 32, smp, init, 0)
        assert e.value.code == B.SJD_EINVAL
        with pytest.raises(B.SjdError) as e:              # NaN weight
            B.sjd_prefill(m, kv, pc, None, smp, init, q)
            B.sjd_prefill_uncond(m, kv, pc, None, float("nan"), smp, init, q)
        assert e.value.code == B.SJD_EINVAL
        with pytest.raises(B.SjdError) as e:              # unconditional prompt + image does not fit
            B.sjd_generate_cfg(m, kv, pc, None, np.arange(shape.max_seq - 30, dtype=np.int32) % 1024, None, 3.0, 64, 8,
                               smp, init, 0)
        assert e.value.code == B.SJD_ESEQ
    finally:
        B.sjd_kv_free(kv); B.sjd_free_model(m)
