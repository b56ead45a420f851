"""Seeded synthetic inputs: model shapes, random-init weight blobs, prompts.

This module is the only code shared by the CPU oracle's tests and the HIP
path.  It holds shapes and random-number plumbing only: none of the decoding
method's arithmetic lives here, and it imports neither the oracle nor the HIP
binding.

The paper runs third-party pretrained 7B models on caption prompts; neither
the weights nor the prompts exist here, so random-init decoders of the same
shapes and random token prompts of the same lengths stand in for them.

Weight blob layout (one flat array, element type fp32 or bf16-as-uint16, every
matrix row-major as [out_features][in_features], i.e. y = W x):

    E      [vocab_total, d]        token embedding table
    for each layer l = 0 .. n_layers-1:
        g1 [d]                     RMSNorm gain before attention
        Wq [d, d]   Wk [d, d]   Wv [d, d]   Wo [d, d]
        g2 [d]                     RMSNorm gain before the FFN
        Wg [F, d]   Wu [F, d]   Wd [d, F]
    gf     [d]                     final RMSNorm gain
    Wlm    [vocab_total, d]        LM head (untied)
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np

DTYPE_F32 = 0
DTYPE_BF16 = 1

INIT_UNIFORM = 0
INIT_REPEAT_ABOVE = 1


@dataclasses.dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    d_ffn: int
    vocab_total: int
    samp_lo: int          # sampling vocabulary = ids [samp_lo, samp_hi)
    samp_hi: int
    max_seq: int
    dtype: int            # DTYPE_F32 or DTYPE_BF16
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5

    @property
    def head_dim(self) -> int:
        return self.d_model // self.n_heads

    @property
    def v_s(self) -> int:
        return self.samp_hi - self.samp_lo

    def tensor_list(self):
        """(name, shape, kind) in blob order; kind is 'gain' or 'matrix'."""
        d, f, v = self.d_model, self.d_ffn, self.vocab_total
        out = [("E", (v, d), "matrix")]
        for l in range(self.n_layers):
            out += [
                (f"l{l}.g1", (d,), "gain"),
                (f"l{l}.Wq", (d, d), "matrix"), (f"l{l}.Wk", (d, d), "matrix"),
                (f"l{l}.Wv", (d, d), "matrix"), (f"l{l}.Wo", (d, d), "matrix"),
                (f"l{l}.g2", (d,), "gain"),
                (f"l{l}.Wg", (f, d), "matrix"), (f"l{l}.Wu", (f, d), "matrix"),
                (f"l{l}.Wd", (d, f), "matrix"),
            ]
        out += [("gf", (d,), "gain"), ("Wlm", (v, d), "matrix")]
        return out

    def n_params(self) -> int:
        return sum(int(np.prod(s)) for _, s, _ in self.tensor_list())

    def layer_param_count(self) -> int:
        d, f = self.d_model, self.d_ffn
        return self.n_layers * (4 * d * d + 3 * d * f)


@dataclasses.dataclass(frozen=True)
class Workload:
    """One benchmark configuration: a model shape plus the decoding set-up."""
    name: str
    shape: ModelShape
    n_prompt_ids: int     # prompt token ids fed first
    n_prompt_embeds: int  # raw embedding rows fed after the ids
    n_image_tokens: int   # N
    window: int           # L (the paper's W)
    top_k: int
    temperature: float
    init_mode: int
    row_stride: int       # image tokens per grid row incl. a row-end token
    eol_id: int           # forced row-end token id, -1 = none


def _shape(layers, d, heads, ffn, vocab, lo, hi, max_seq, dtype):
    return ModelShape(layers, d, heads, ffn, vocab, lo, hi, max_seq, dtype)


_SHAPE_7B_SHORT = _shape(32, 4096, 32, 11008, 65536, 57344, 65536, 64 + 1024 + 32, DTYPE_BF16)
_SHAPE_7B_LONG = _shape(32, 4096, 32, 11008, 65536, 57344, 65536, 64 + 2352 + 32, DTYPE_BF16)
_SHAPE_7B_1024 = _shape(32, 4096, 32, 11008, 65536, 57344, 65536, 64 + 4160 + 32, DTYPE_BF16)

WORKLOADS = {
    # Tiny: 2 layers, d=128, vocab 1024 all image codes, 8x8 grid.
    "tiny": Workload("tiny", _shape(2, 128, 4, 512, 1024, 0, 1024, 16 + 64 + 32, DTYPE_F32),
                     16, 0, 64, 8, 64, 1.0, INIT_UNIFORM, 8, -1),
    # ~775M class-conditional style: 1 condition id + 120 embedding rows.
    "775m": Workload("775m", _shape(24, 1536, 24, 4096, 16384, 0, 16384, 121 + 1024 + 16, DTYPE_BF16),
                     1, 120, 1024, 16, 2000, 1.0, INIT_UNIFORM, 32, -1),
    # 7B, 32x32 grid, sampling masked to the 8192 image codes at the top of the vocabulary.
    "7b_32x32": Workload("7b_32x32", _SHAPE_7B_SHORT, 64, 0, 1024, 16, 2000, 1.0, INIT_UNIFORM, 32, -1),
    # 7B, 48x48 grid + one forced row-end token per row (last image code id).
    "7b_48x48": Workload("7b_48x48", _SHAPE_7B_LONG, 64, 0, 2352, 32, 2000, 1.0, INIT_UNIFORM, 49, 65535),
    # same with drafts initialised from the token one grid row above.
    "7b_48x48_above": Workload("7b_48x48_above", _SHAPE_7B_LONG, 64, 0, 2352, 32, 2000, 1.0,
                               INIT_REPEAT_ABOVE, 49, 65535),
    # 7B, 64x64 grid (a 1024 x 1024 image at 16 x 16 pixels per code) + row-end tokens: 4160 tokens.
    "7b_64x64": Workload("7b_64x64", _SHAPE_7B_1024, 64, 0, 4160, 16, 2000, 1.0, INIT_UNIFORM, 65, 65535),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


_CHUNK = 1 << 22


def _fill_normal(dst: np.ndarray, seed: int, tensor_id: int, std: float, threads: int) -> None:
    """dst (1-D fp32 or uint16 view) <- i.i.d. N(0, std^2), chunk-seeded so the
    result does not depend on the thread count."""
    n = dst.size
    n_chunks = (n + _CHUNK - 1) // _CHUNK

    def work(c):
        lo, hi = c * _CHUNK, min(n, (c + 1) * _CHUNK)
        g = np.random.Generator(np.random.SFC64([seed, tensor_id, c]))
        x = g.standard_normal(hi - lo, dtype=np.float32)
        x *= np.float32(std)
        if dst.dtype == np.float32:
            dst[lo:hi] = x
        else:
            dst[lo:hi] = f32_to_bf16_bits(x)

    if threads <= 1 or n_chunks == 1:
        for c in range(n_chunks):
            work(c)
    else:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(work, range(n_chunks)))


def make_weights(shape: ModelShape, seed: int = 0, std: float = 0.02, threads: int = 8) -> np.ndarray:
    """Flat weight blob in the documented order: matrices i.i.d. N(0, std^2), gains 1.
    fp32 blob for DTYPE_F32; uint16 bf16 bit patterns for DTYPE_BF16."""
    np_dtype = np.float32 if shape.dtype == DTYPE_F32 else np.uint16
    blob = np.empty(shape.n_params(), dtype=np_dtype)
    one = np.float32(1.0) if shape.dtype == DTYPE_F32 else np.uint16(0x3F80)
    off = 0
    for tid, (_, shp, kind) in enumerate(shape.tensor_list()):
        n = int(np.prod(shp))
        if kind == "gain":
            blob[off:off + n] = one
        else:
            _fill_normal(blob[off:off + n], seed, tid, std, threads)
        off += n
    return blob


def tensor_offsets(shape: ModelShape) -> dict:
    """name -> (element offset, shape) into the blob."""
    out, off = {}, 0
    for name, shp, _ in shape.tensor_list():
        out[name] = (off, shp)
        off += int(np.prod(shp))
    return out


def make_prompt(w: Workload, seed: int = 1):
    """Prompt ids (int32) uniform over the non-image id range when there is one,
    else over the whole vocabulary; embedding rows (fp32 [n, d]) ~ N(0, 0.02^2)."""
    s = w.shape
    g = np.random.Generator(np.random.SFC64([seed, 0xABCD]))
    if s.samp_lo > 0:
        ids = g.integers(0, s.samp_lo, size=w.n_prompt_ids, dtype=np.int32)
    else:
        ids = g.integers(0, s.vocab_total, size=w.n_prompt_ids, dtype=np.int32)
    emb = (g.standard_normal((w.n_prompt_embeds, s.d_model), dtype=np.float32) * np.float32(0.02))
    if s.dtype == DTYPE_BF16:
        emb = bf16_bits_to_f32(f32_to_bf16_bits(emb)).reshape(emb.shape)
    return ids, emb


def random_logits(rows: int, v: int, seed: int, std: float = 1.28) -> np.ndarray:
    """fp32 logits with the scale a random-init LM head produces (std ~ 0.02*sqrt(d))."""
    g = np.random.Generator(np.random.SFC64([seed, 0x106175]))
    return g.standard_normal((rows, v), dtype=np.float32) * np.float32(std)


def random_tokens(n: int, lo: int, hi: int, seed: int) -> np.ndarray:
    g = np.random.Generator(np.random.SFC64([seed, 0x70C]))
    return g.integers(lo, hi, size=n, dtype=np.int32)
