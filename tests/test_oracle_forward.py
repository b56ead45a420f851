"""Pins for the oracle's transformer forward -- CPU only.

The paper gives no architecture beyond "auto-regressive transformer with a softmax
classifier" (Sec. 3.1); the workload configurations fix a Llama-style decoder.  The oracle is
pinned against the Hugging Face `LlamaForCausalLM` library implementation in fp64 (an
independent code base), and its KV-cached window path against its own full-sequence path.
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2410_01699_amd import synth


def _small_shape(dtype=synth.DTYPE_F32):
    return synth.ModelShape(n_layers=3, d_model=64, n_heads=4, d_ffn=96, vocab_total=200, samp_lo=40, samp_hi=200,
                            max_seq=48, dtype=dtype)


def _random_blob(shape, seed, std=0.25):
    """weights with O(1) activations and non-unit gains, so every term matters"""
    blob = synth.make_weights(shape, seed=seed, std=std).astype(np.float32) if shape.dtype == 0 else None
    assert blob is not None
    rng = np.random.default_rng(seed)
    for name, (off, shp) in synth.tensor_offsets(shape).items():
        if len(shp) == 1:
            blob[off:off + shp[0]] = rng.uniform(0.5, 1.5, shp[0]).astype(np.float32)
    return blob


def _hf_model(shape, blob):
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg = LlamaConfig(vocab_size=shape.vocab_total, hidden_size=shape.d_model, intermediate_size=shape.d_ffn,
                      num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_heads,
                      num_key_value_heads=shape.n_heads, max_position_embeddings=shape.max_seq,
                      rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_theta, attention_bias=False,
                      mlp_bias=False, tie_word_embeddings=False, hidden_act="silu")
    try:
        cfg._attn_implementation = "eager"
    except Exception:
        pass
    m = LlamaForCausalLM(cfg).double().eval()
    offs = synth.tensor_offsets(shape)

    def t(name):
        off, shp = offs[name]
        return torch.from_numpy(blob[off:off + int(np.prod(shp))].astype(np.float64).reshape(shp))

    sd = {"model.embed_tokens.weight": t("E"), "model.norm.weight": t("gf"), "lm_head.weight": t("Wlm")}
    for l in range(shape.n_layers):
        p = f"model.layers.{l}."
        sd[p + "input_layernorm.weight"] = t(f"l{l}.g1")
        sd[p + "self_attn.q_proj.weight"] = t(f"l{l}.Wq")
        sd[p + "self_attn.k_proj.weight"] = t(f"l{l}.Wk")
        sd[p + "self_attn.v_proj.weight"] = t(f"l{l}.Wv")
        sd[p + "self_attn.o_proj.weight"] = t(f"l{l}.Wo")
        sd[p + "post_attention_layernorm.weight"] = t(f"l{l}.g2")
        sd[p + "mlp.gate_proj.weight"] = t(f"l{l}.Wg")
        sd[p + "mlp.up_proj.weight"] = t(f"l{l}.Wu")
        sd[p + "mlp.down_proj.weight"] = t(f"l{l}.Wd")
    missing, unexpected = m.load_state_dict(sd, strict=False)
    assert not unexpected
    assert all("rotary" in k or "inv_freq" in k for k in missing), missing
    return m


@pytest.mark.parametrize("theta,eps", [(10000.0, 1e-5), (500000.0, 2e-2)])
def test_forward_matches_library_llama(theta, eps):
    # (the second case: a RoPE base and a normalisation epsilon that are not the defaults; the epsilon is
    # of the order of mean(x^2), so that dropping it or misplacing it shows)
    shape = dataclasses.replace(_small_shape(), rope_theta=theta, rms_eps=eps)
    blob = _random_blob(shape, seed=11)
    ids = synth.random_tokens(21, 0, shape.vocab_total, seed=5)
    om = oracle.Model(shape, blob)
    got = om.forward_full(om.embed(ids))
    hf = _hf_model(shape, blob)
    with torch.no_grad():
        ref = hf(torch.from_numpy(ids.astype(np.int64))[None]).logits[0].numpy()
    ref = ref[:, shape.samp_lo:shape.samp_hi]
    assert got.shape == ref.shape
    scale = np.abs(ref).max()
    assert scale > 0.5                                   # the case is not degenerate
    assert np.max(np.abs(got - ref)) < 1e-6 * max(1.0, scale)


def test_window_forward_equals_full_forward():
    shape = _small_shape()
    blob = _random_blob(shape, seed=12)
    ids = synth.random_tokens(30, 0, shape.vocab_total, seed=6)
    om = oracle.Model(shape, blob)
    full = om.forward_full(om.embed(ids))
    # prefill 9, then windows of 8, 1, 12 tokens, advancing by hand
    pos = 0
    for n in (9, 8, 1, 12):
        om.kv_set_len(pos)
        part = om.forward_window(om.embed(ids[pos:pos + n]))
        assert np.max(np.abs(part - full[pos:pos + n])) < 1e-6
        pos += n


def test_window_overwrite_after_partial_accept():
    """Rows written for rejected drafts must not leak: re-running from a shorter length
    with different tokens equals the full forward on the new sequence."""
    shape = _small_shape()
    blob = _random_blob(shape, seed=13)
    om = oracle.Model(shape, blob)
    a = synth.random_tokens(20, 0, shape.vocab_total, seed=7)
    b = a.copy(); b[12:] = synth.random_tokens(8, 0, shape.vocab_total, seed=8)
    om.kv_set_len(0); om.forward_window(om.embed(a[:10]))
    om.kv_set_len(10); om.forward_window(om.embed(a[10:20]))       # drafts 10..19
    om.kv_set_len(12)                                              # only two accepted
    got = om.forward_window(om.embed(b[12:20]))
    ref = om.forward_full(om.embed(b))[12:20]
    assert np.max(np.abs(got - ref)) < 1e-6


def test_causality_later_tokens_do_not_change_earlier_rows():
    shape = _small_shape()
    blob = _random_blob(shape, seed=14)
    om = oracle.Model(shape, blob)
    a = synth.random_tokens(16, 0, shape.vocab_total, seed=9)
    b = a.copy(); b[11] = (b[11] + 1) % shape.vocab_total
    la = om.forward_full(om.embed(a)); lb = om.forward_full(om.embed(b))
    assert np.array_equal(la[:11], lb[:11])
    assert not np.array_equal(la[11:], lb[11:])


def test_bf16_blob_is_read_exactly():
    shape = _small_shape(synth.DTYPE_BF16)
    blob16 = synth.make_weights(shape, seed=3, std=0.25)
    blob32 = synth.bf16_bits_to_f32(blob16)
    shape32 = _small_shape(synth.DTYPE_F32)
    ids = synth.random_tokens(12, 0, shape.vocab_total, seed=10)
    m16 = oracle.Model(shape, blob16); m32 = oracle.Model(shape32, blob32)
    assert np.array_equal(m16.forward_full(m16.embed(ids)), m32.forward_full(m32.embed(ids)))


def test_prefill_with_embedding_rows():
    shape = _small_shape()
    blob = _random_blob(shape, seed=15)
    om = oracle.Model(shape, blob)
    ids = synth.random_tokens(3, 0, shape.vocab_total, seed=11)
    emb = np.random.default_rng(0).standard_normal((5, shape.d_model)).astype(np.float32) * 0.3
    last = om.prefill(ids, emb)
    x = np.concatenate([om.embed(ids), emb.astype(np.float64)])
    ref = om.forward_full(x)[-1]
    assert np.max(np.abs(last - ref)) < 1e-6
    assert oracle.lib().orc_kv_len(om.kv) == 8
