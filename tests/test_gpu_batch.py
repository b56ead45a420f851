"""GPU parity of batched decoding: B independent images share every window forward (Sec. 4.1 Step 2 for
B windows at once), Steps 3 and 4 run per image.

The oracle side is one transformer oracle per image (images are independent).  bf16 models only, so whole
token streams cannot be compared with the fp64 oracle; what is checked instead:
  * every image's logits of the shared forward against its own oracle forward (2e-2 bar);
  * the whole batched loop, iteration by iteration, against oracle verifications fed with the GPU's own
    batched logits: accepted counts and every fixed token bit-exact, for every image;
  * graph replay == kernel-by-kernel, images of different lengths of prompt, images that finish early.
"""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import oracle  # noqa: E402
from paper_2410_01699_amd import synth  # noqa: E402

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


SHAPE = synth.ModelShape(3, 256, 4, 512, 2048, 1024, 2048, 260, synth.DTYPE_BF16)


def _setup(B, nb, shape=SHAPE):
    blob = synth.make_weights(shape, seed=8, threads=16)
    m = B.sjd_init_model(B.config_from_shape(shape), blob)
    kvs = [B.sjd_kv_create(m) for _ in range(nb)]
    prompts = [synth.random_tokens(5 + 13 * b, 0, 1024, seed=10 + b) for b in range(nb)]
    return blob, m, kvs, prompts


def _teardown(B, m, kvs):
    for kv in kvs:
        B.sjd_kv_free(kv)
    B.sjd_free_model(m)


@pytest.mark.parametrize("nb,L", [(2, 16), (4, 8), (8, 4), (3, 7), (2, 9), (1, 32), (5, 1),
                                  (8, 16), (4, 32), (2, 64), (6, 13), (2, 40), (3, 32)])
def test_batched_forward_logits(B, nb, L):
    _say(f"batched forward B={nb} L={L}")
    blob, m, kvs, prompts = _setup(B, nb)
    oms = [oracle.Model(SHAPE, blob) for _ in range(nb)]
    try:
        V = SHAPE.v_s
        smp = B.sjd_sampler(8, 1.0); init = B.sjd_init(0, 0, -1)
        q = torch.empty(V, dtype=torch.float32, device="cuda")
        for b in range(nb):
            B.sjd_prefill(m, kvs[b], prompts[b], None, smp, init, q)
            oms[b].prefill(prompts[b])
        fixed = [0] * nb
        out = torch.empty((nb, L, V), dtype=torch.float32, device="cuda")
        for it in range(3):
            toks = np.stack([synth.random_tokens(L, 1024, 2048, seed=100 * it + b) for b in range(nb)])
            B.sjd_forward_logits_batch(m, kvs, _dev(toks), L, out)
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            for b in range(nb):
                ref = oms[b].forward_tokens(len(prompts[b]) + fixed[b], toks[b])
                err = float(np.max(np.abs(got[b] - ref)))
                assert err < TOL_BF16, (it, b, err)
                keep = 1 + (it + b) % L                    # every image keeps a different number of tokens
                fixed[b] += keep
                B.sjd_kv_set_len(kvs[b], len(prompts[b]) + fixed[b])
    finally:
        _teardown(B, m, kvs)
        for om in oms:
            om.close()


def test_batched_forward_7b_layer_shapes(B):
    """the 7B layer shapes (d 4096, 32 heads of 128, FFN 11008, 8192 sampled codes of 65536), two layers:
    two windows of 16 and four of 8 in one forward (32 rows), then eight of 16 and four of 32 (128 rows)"""
    shape = synth.ModelShape(2, 4096, 32, 11008, 65536, 57344, 65536, 200, synth.DTYPE_BF16)
    blob, m, kvs, _ = _setup(B, 8, shape)
    oms = [oracle.Model(shape, blob) for _ in range(8)]
    try:
        V = shape.v_s
        smp = B.sjd_sampler(8, 1.0); init = B.sjd_init(0, 0, -1)
        q = torch.empty(V, dtype=torch.float32, device="cuda")
        prompts = [synth.random_tokens(20 + 17 * b, 0, 57344, seed=10 + b) for b in range(8)]
        for b in range(8):
            B.sjd_prefill(m, kvs[b], prompts[b], None, smp, init, q)
            oms[b].prefill(prompts[b])
        for nb, L in ((2, 16), (4, 8), (8, 16), (4, 32)):
            _say(f"7b shapes: batched forward B={nb} L={L}")
            toks = np.stack([synth.random_tokens(L, 57344, 65536, seed=nb * 10 + b) for b in range(nb)])
            out = torch.empty((nb, L, V), dtype=torch.float32, device="cuda")
            B.sjd_forward_logits_batch(m, kvs[:nb], _dev(toks), L, out)
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            for b in range(nb):
                ref = oms[b].forward_tokens(len(prompts[b]), toks[b])
                err = float(np.max(np.abs(got[b] - ref)))
                _say(f"  image {b}: worst logit error {err:.3e}")
                assert err < TOL_BF16, (nb, b, err)
    finally:
        _teardown(B, m, kvs)
        for om in oms:
            om.close()


def test_batched_forward_and_steps_7b_full_size(B):
    """Eight images x 16 drafts on the full 7B model (32 layers; forwards of 128 rows on the wide projection
    kernel, Steps 3-4 of the eight images in shared launches), in the configuration `bench.py --batch 8` times:
    the logits of three of the images against the fp64 oracle (each image on its own prompt and cache), then
    three iterations of the captured batched loop whose verification must be bit-exact per image given the
    GPU's own logits."""
    w = synth.WORKLOADS["7b_32x32"]
    shape, nb, L = w.shape, 8, 16
    _say("7b batch: generating weights")
    blob = synth.make_weights(shape, seed=0, threads=16)
    m = B.sjd_init_model(B.config_from_shape(shape), blob)
    kvs = [B.sjd_kv_create(m) for _ in range(nb)]
    om = oracle.Model(shape, blob)
    try:
        V, lo = shape.v_s, shape.samp_lo
        smp = B.sjd_sampler(w.top_k, w.temperature); init = B.sjd_init(w.init_mode, w.row_stride, w.eol_id)
        osmp = oracle.Sampler(w.top_k, w.temperature); oinit = oracle.Init(w.init_mode, w.row_stride, w.eol_id)
        prompts = [synth.random_tokens(12 + 7 * b, 0, lo, seed=10 + b) for b in range(nb)]
        q = torch.empty(V, dtype=torch.float32, device="cuda")
        N = 40
        st = []
        B.sjd_kv_use_graph(kvs[0], True)
        for b in range(nb):
            B.sjd_prefill(m, kvs[b], prompts[b], None, smp, init, q)
            B.sjd_decode_begin(m, kvs[b], q, N, L, smp, init, 70 + b)
            torch.cuda.synchronize()
            d, p = oracle.first_window(q.cpu().numpy(), L, lo, oinit, 70 + b)
            st.append({"draft": d, "p": p, "hist": [], "c": 0})
        logits = torch.empty((nb, L, V), dtype=torch.float32, device="cuda")
        for it in range(3):
            toks = np.stack([s["draft"] for s in st]).astype(np.int32)
            B.sjd_forward_logits_batch(m, kvs, _dev(toks), L, logits)
            torch.cuda.synchronize()
            lg = logits.cpu().numpy()
            if it == 0:
                for b in (0, 3, 7):
                    _say(f"7b batch: oracle prefill + window of image {b} (fp64 on the host)")
                    om.prefill(prompts[b])
                    ref = om.forward_tokens(len(prompts[b]), toks[b])
                    err = float(np.max(np.abs(lg[b] - ref)))
                    _say(f"7b batch: image {b} worst logit error {err:.3e}")
                    assert err < TOL_BF16, (b, err)
            for b, s in enumerate(st):
                s["c"] += 1
                a, nd, pn = oracle.verify(lg[b], s["p"], s["draft"], lo, osmp, oinit, len(s["hist"]),
                                          np.array(s["hist"], np.int32), 70 + b, s["c"])
                s["hist"] += [int(t) for t in s["draft"][:a]]
                s["draft"] = np.concatenate([nd, s["draft"][L:]]).astype(np.int32)
                s["p"] = np.concatenate([pn, s["p"][L:]])
            _say(f"7b batch: loop iteration {it + 1}")
            B.sjd_decode_steps_batch(m, kvs, 1)
            torch.cuda.synchronize()
            for b, s in enumerate(st):
                fixed, steps, done = B.sjd_decode_status(kvs[b])
                assert fixed == len(s["hist"]) and steps == s["c"] and not done, (it, b, fixed, len(s["hist"]))
    finally:
        _teardown(B, m, kvs)
        om.close()


@pytest.mark.parametrize("nb,L,mode,use_graph", [(2, 16, 0, True), (4, 8, 1, True), (3, 5, 4, False), (8, 4, 3, True),
                                                 (8, 16, 0, True), (2, 64, 1, True), (4, 32, 4, False)])
def test_batched_loop_bit_exact_given_gpu_logits(B, nb, L, mode, use_graph):
    """every iteration of the batched loop == the oracle's verification of the same logits, per image"""
    _say(f"batched loop B={nb} L={L} mode={mode} graph={use_graph}")
    blob, m, kvs, prompts = _setup(B, nb)
    try:
        V, lo = SHAPE.v_s, SHAPE.samp_lo
        stride, eol, K = 6, 2047, 300
        N = [stride * (9 - 4 * (b % 3)) for b in range(nb)]     # images of different lengths: some finish early
        smp = B.sjd_sampler(K, 1.0); init = B.sjd_init(mode, stride, eol)
        osmp = oracle.Sampler(K, 1.0); oinit = oracle.Init(mode, stride, eol)
        q = torch.empty(V, dtype=torch.float32, device="cuda")
        B.sjd_kv_use_graph(kvs[0], use_graph)
        st = []
        for b in range(nb):
            B.sjd_prefill(m, kvs[b], prompts[b], None, smp, init, q)
            B.sjd_decode_begin(m, kvs[b], q, N[b], L, smp, init, 50 + b)
            torch.cuda.synchronize()
            d, p = oracle.first_window(q.cpu().numpy(), L, lo, oinit, 50 + b)
            st.append({"draft": d, "p": p, "hist": [], "c": 0, "done": False,
                       "ring": np.zeros((stride, V), np.float32) if mode == 4 else None})
        logits = torch.empty((nb, L, V), dtype=torch.float32, device="cuda")
        outs = [np.zeros(N[b], np.int32) for b in range(nb)]
        for it in range(4 * max(N)):
            if all(s["done"] for s in st):
                break
            # the logits the next iteration will see (same forward, deterministic; the cache rows it writes
            # are written again, alike, by the iteration itself)
            toks = np.stack([s["draft"] for s in st]).astype(np.int32)
            B.sjd_forward_logits_batch(m, kvs, _dev(toks), L, logits)
            torch.cuda.synchronize()
            lg = logits.cpu().numpy()
            for b, s in enumerate(st):
                if s["done"]:
                    continue
                s["c"] += 1
                n_acc = len(s["hist"])
                Le = min(L, N[b] - n_acc)
                a, nd, pn = oracle.verify(lg[b][:Le], s["p"][:Le], s["draft"][:Le], lo, osmp, oinit, n_acc,
                                          np.array(s["hist"], np.int32), 50 + b, s["c"], ring=s["ring"])
                s["hist"] += [int(t) for t in s["draft"][:a]]
                s["draft"] = np.concatenate([nd, s["draft"][Le:]]).astype(np.int32)
                s["p"] = np.concatenate([pn, s["p"][Le:]])
                s["done"] = len(s["hist"]) >= N[b] - 1
            B.sjd_decode_steps_batch(m, kvs, 1)
            torch.cuda.synchronize()
            for b, s in enumerate(st):
                fixed, steps, done = B.sjd_decode_status(kvs[b])
                assert fixed == len(s["hist"]), (it, b, fixed, len(s["hist"]))
                assert steps == s["c"] and bool(done) == s["done"], (it, b)
        assert all(s["done"] for s in st)
        assert len({s["c"] for s in st}) > 1                   # the images did finish at different iterations
        for b, s in enumerate(st):
            want = np.array(s["hist"][:N[b]], np.int32)
            if len(want) < N[b]:
                want = np.append(want, s["draft"][0]).astype(np.int32)    # the pending exact index-0 token
            got, stats = B.sjd_decode_result(kvs[b], N[b])
            assert np.array_equal(got, want), (b, np.nonzero(got != want)[0][:5])
            assert stats.steps == s["c"]
            assert np.all(got[stride - 1::stride] == eol)
    finally:
        _teardown(B, m, kvs)


def test_generate_batch_graph_equals_eager_and_images_are_independent(B):
    """sjd_generate_batch: replayed graph == kernel-by-kernel; an image's tokens do not depend on which
    other images share its forwards (same batch shape, different neighbours)"""
    blob, m, kvs, prompts = _setup(B, 4)
    try:
        smp = B.sjd_sampler(300, 1.0); init = B.sjd_init(1, 9, 2047)
        N, L = 9 * 12, 8
        res = {}
        for use_graph in (True, False, True):
            B.sjd_kv_use_graph(kvs[0], use_graph)
            _say(f"generate batch graph={use_graph}")
            toks, stats = B.sjd_generate_batch(m, kvs, prompts, None, N, L, smp, init, [3, 4, 5, 6])
            assert toks.shape == (4, N) and toks.min() >= 1024 and toks.max() < 2048
            assert np.all(toks[:, 8::9] == 2047)
            for b in range(4):
                hist = np.array(stats[b].accept_hist[:])
                assert hist.sum() == stats[b].steps and int((hist * np.arange(65)).sum()) in (N - 1, N)
            res.setdefault("ref", (toks, [s.steps for s in stats]))
            assert np.array_equal(toks, res["ref"][0]) and [s.steps for s in stats] == res["ref"][1]
        assert len({tuple(t) for t in res["ref"][0]}) == 4          # four different images
        # image 0 with other neighbours (prompts and seeds of the others changed): same tokens
        other = [prompts[0]] + [synth.random_tokens(7 + b, 0, 1024, seed=70 + b) for b in range(3)]
        toks2, _ = B.sjd_generate_batch(m, kvs, other, None, N, L, smp, init, [3, 40, 50, 60])
        assert np.array_equal(toks2[0], res["ref"][0][0])
        assert not np.array_equal(toks2[1], res["ref"][0][1])
    finally:
        _teardown(B, m, kvs)


def test_batch_errors(B):
    blob, m, kvs, prompts = _setup(B, 3)
    try:
        smp = B.sjd_sampler(300, 1.0); init = B.sjd_init(0, 9, -1)
        with pytest.raises(B.SjdError) as e:              # three windows of 64 do not fit 128 rows
            B.sjd_generate_batch(m, kvs, prompts, None, 32, 64, smp, init, [1, 2, 3])
        assert e.value.code == B.SJD_EINVAL
        with pytest.raises(B.SjdError) as e:              # the same handle twice
            B.sjd_generate_batch(m, [kvs[0], kvs[0]], prompts[:2], None, 32, 8, smp, init, [1, 2])
        assert e.value.code == B.SJD_EINVAL
        with pytest.raises(B.SjdError) as e:              # not begun
            B.sjd_decode_steps_batch(m, kvs[:2], 1)
        assert e.value.code == B.SJD_EINVAL
        q = torch.empty(SHAPE.v_s, dtype=torch.float32, device="cuda")
        for b, L in ((0, 8), (1, 4)):                     # begun with different windows
            B.sjd_prefill(m, kvs[b], prompts[b], None, smp, init, q)
            B.sjd_decode_begin(m, kvs[b], q, 20, L, smp, init, 1)
        with pytest.raises(B.SjdError) as e:
            B.sjd_decode_steps_batch(m, kvs[:2], 1)
        assert e.value.code == B.SJD_EINVAL
        with pytest.raises(B.SjdError) as e:              # image does not fit the cache
            B.sjd_generate_batch(m, kvs[:2], prompts[:2], None, 1000, 8, smp, init, [1, 2])
        assert e.value.code == B.SJD_ESEQ
        # fp32 models are not batched
        w = synth.WORKLOADS["tiny"]
        m32 = B.sjd_init_model(B.config_from_shape(w.shape), synth.make_weights(w.shape, seed=0))
        k32 = [B.sjd_kv_create(m32) for _ in range(2)]
        try:
            with pytest.raises(B.SjdError) as e:
                B.sjd_generate_batch(m32, k32, [np.arange(4, dtype=np.int32)] * 2, None, 16, 8, B.sjd_sampler(8, 1.0),
                                     B.sjd_init(0, 8, -1), [1, 2])
            assert e.value.code == B.SJD_EINVAL
        finally:
            _teardown(B, m32, k32)
    finally:
        _teardown(B, m, kvs)


# ------------------------------------------------------------------ guided batches (two contexts per image)
@pytest.mark.parametrize("nb,L,mode,use_graph", [(2, 16, 0, True), (4, 16, 1, True), (3, 7, 4, False), (2, 32, 3, True), (4, 9, 0, False)])
def test_guided_batch_logits_and_loop(B, nb, L, mode, use_graph):
    """Batched decoding under classifier-free guidance: every image brings a conditional and an unconditional
    context (2 x nb streams in one forward, its rows 2b and 2b + 1), each image with its own guidance weight.
    Guided logits of every image against two oracles per image (oracle.guide of their logits); then the whole
    batched loop, iteration by iteration, against oracle verifications fed the GPU's guided logits: accepted
    counts and tokens bit-exact per image, both caches of every image advancing together."""
    _say(f"guided batch B={nb} L={L} mode={mode} graph={use_graph}")
    blob, m, kvs, prompts = _setup(B, nb)
    ocs = [oracle.Model(SHAPE, blob) for _ in range(nb)]
    ous = [oracle.Model(SHAPE, blob) for _ in range(nb)]
    try:
        V, lo = SHAPE.v_s, SHAPE.samp_lo
        stride, eol, K = 6, 2047, 300
        N = [stride * (8 - 3 * (b % 2)) for b in range(nb)]
        ws = [3.0, 1.5, 7.5, 2.0][:nb]
        uprompts = [synth.random_tokens(3 + 4 * b, 0, 1024, seed=40 + b) for b in range(nb)]
        smp = B.sjd_sampler(K, 1.0); init = B.sjd_init(mode, stride, eol)
        osmp = oracle.Sampler(K, 1.0); oinit = oracle.Init(mode, stride, eol)
        q = torch.empty(V, dtype=torch.float32, device="cuda")
        B.sjd_kv_use_graph(kvs[0], use_graph)
        st = []
        for b in range(nb):
            B.sjd_prefill(m, kvs[b], prompts[b], None, smp, init, q)
            B.sjd_prefill_uncond(m, kvs[b], uprompts[b], None, ws[b], smp, init, q)
            B.sjd_decode_begin(m, kvs[b], q, N[b], L, smp, init, 90 + b)
            torch.cuda.synchronize()
            ocs[b].prefill(prompts[b]); ous[b].prefill(uprompts[b])
            d, p = oracle.first_window(q.cpu().numpy(), L, lo, oinit, 90 + b)
            st.append({"draft": d, "p": p, "hist": [], "c": 0, "done": False,
                       "ring": np.zeros((stride, V), np.float32) if mode == 4 else None})
        logits = torch.empty((nb, L, V), dtype=torch.float32, device="cuda")
        for it in range(4 * max(N)):
            if all(s["done"] for s in st):
                break
            toks = np.stack([s["draft"] for s in st]).astype(np.int32)
            B.sjd_forward_logits_batch(m, kvs, _dev(toks), L, logits)
            torch.cuda.synchronize()
            lg = logits.cpu().numpy()
            for b, s in enumerate(st):
                if s["done"]:
                    continue
                n_acc = len(s["hist"])
                if it < 3:
                    zc = ocs[b].forward_tokens(len(prompts[b]) + n_acc, toks[b])
                    zu = ous[b].forward_tokens(len(uprompts[b]) + n_acc, toks[b])
                    err = float(np.max(np.abs(lg[b] - oracle.guide(zc, zu, ws[b]))))
                    assert err < TOL_BF16, (it, b, err)
                s["c"] += 1
                Le = min(L, N[b] - n_acc)
                a, nd, pn = oracle.verify(lg[b][:Le], s["p"][:Le], s["draft"][:Le], lo, osmp, oinit, n_acc,
                                          np.array(s["hist"], np.int32), 90 + b, s["c"], ring=s["ring"])
                if it < 3:
                    # (the oracles' caches take the accepted tokens too: positions behind both prompts)
                    ocs[b].forward_tokens(len(prompts[b]) + n_acc, toks[b]); ocs[b].kv_set_len(len(prompts[b]) + n_acc + a)
                    ous[b].forward_tokens(len(uprompts[b]) + n_acc, toks[b]); ous[b].kv_set_len(len(uprompts[b]) + n_acc + a)
                s["hist"] += [int(t) for t in s["draft"][:a]]
                s["draft"] = np.concatenate([nd, s["draft"][Le:]]).astype(np.int32)
                s["p"] = np.concatenate([pn, s["p"][Le:]])
                s["done"] = len(s["hist"]) >= N[b] - 1
            B.sjd_decode_steps_batch(m, kvs, 1)
            torch.cuda.synchronize()
            for b, s in enumerate(st):
                fixed, steps, done = B.sjd_decode_status(kvs[b])
                assert fixed == len(s["hist"]), (it, b, fixed, len(s["hist"]))
                assert steps == s["c"] and bool(done) == s["done"], (it, b)
                assert B.sjd_kv_len(kvs[b]) == len(prompts[b]) + fixed
        assert all(s["done"] for s in st)
        for b, s in enumerate(st):
            want = np.array(s["hist"][:N[b]], np.int32)
            if len(want) < N[b]:
                want = np.append(want, s["draft"][0]).astype(np.int32)
            got, stats = B.sjd_decode_result(kvs[b], N[b])
            assert np.array_equal(got, want), (b, np.nonzero(got != want)[0][:5])
            assert np.all(got[stride - 1::stride] == eol)
    finally:
        _teardown(B, m, kvs)
        for om in ocs + ous:
            om.close()


def test_guided_batch_refuses_mixed_and_oversized_sets(B):
    """all handles of a batch are guided or none is; two contexts per image count against the eight streams and the
    128 rows of a forward"""
    blob, m, kvs, prompts = _setup(B, 5)
    try:
        V = SHAPE.v_s
        smp = B.sjd_sampler(8, 1.0); init = B.sjd_init(0, 0, -1)
        q = torch.empty(V, dtype=torch.float32, device="cuda")
        for b in range(5):
            B.sjd_prefill(m, kvs[b], prompts[b], None, smp, init, q)
            if b != 1:
                B.sjd_prefill_uncond(m, kvs[b], prompts[b][:2], None, 3.0, smp, init, q)
        out = torch.empty((5, 16, V), dtype=torch.float32, device="cuda")
        toks = _dev(np.zeros((5, 16), np.int32) + 1500)
        with pytest.raises(B.SjdError):                 # mixed
            B.sjd_forward_logits_batch(m, kvs[:2], toks, 16, out)
        B.sjd_prefill_uncond(m, kvs[1], prompts[1][:2], None, 3.0, smp, init, q)
        B.sjd_forward_logits_batch(m, kvs[:4], toks, 16, out)          # 8 streams x 16 rows: fits
        with pytest.raises(B.SjdError):                 # 10 streams
            B.sjd_forward_logits_batch(m, kvs, toks, 16, out)
        with pytest.raises(B.SjdError):                 # 8 streams x 32 rows
            B.sjd_forward_logits_batch(m, kvs[:4], _dev(np.zeros((4, 32), np.int32) + 1500), 32,
                                       torch.empty((4, 32, V), dtype=torch.float32, device="cuda"))
        torch.cuda.synchronize()
    finally:
        _teardown(B, m, kvs)
