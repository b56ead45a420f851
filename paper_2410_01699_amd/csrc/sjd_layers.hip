// Element-wise pieces of the window forward (paper Sec. 4.1 Step 2; the decoder itself is the
// Llama-style stack the workloads name): embedding gather for every model, and for the fp32 models
// RMSNorm fused with the residual add, RoPE + KV-cache write and SiLU(gate)*up (bf16 models do all of
// these inside their projection kernel).  All of them are bandwidth-trivial (rows <= 32).
#include "sjd_internal.h"

template <typename T> struct Act;
template <> struct Act<float> {
    __device__ static float load(const float *p, size_t i) { return p[i]; }
    __device__ static void store(float *p, size_t i, float v) { p[i] = v; }
};
template <> struct Act<bf16_t> {
    __device__ static float load(const bf16_t *p, size_t i) { return bf16_to_f32(p[i]); }
};

// x[row][:] = E[id][:]  (or the given raw embedding row); bf16 models keep x in act_off order and leave
// what the first projection reads: the hi / lo planes of x * gain (first layer's attention norm) in
// x24 and the sums of squares of x per 16 features in ssq.  Stream
// blockIdx.z takes its ids from ids.p[stream] and writes rows (stream << shift)..; one thread per 4
// consecutive features; grid (rows per stream, d / 1024, streams).
struct EmbedIds { const int32_t *p[SJD_MAX_STREAMS]; int32_t *err[SJD_MAX_STREAMS]; };
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T *E, EmbedIds ids, const float *emb_rows, int d, int shift,
                                                    float *x, void *x24, const bf16_t *gain, float *ssq, int vocab, int lo16)
{
    const int stream = blockIdx.z;
    const int r = blockIdx.x;
    const int j = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (j >= d) return;       // (d is a multiple of 32 in bf16 models: whole groups of 4 threads leave)
    float4 v;
    // an id outside the vocabulary (the ids come from caller-supplied device memory) reads nothing: its
    // row is zero and the error flag of the handle's state is raised
    const int id = emb_rows ? 0 : ids.p[stream][r];
    if (id < 0 || id >= vocab) {
        v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (j == 0 && ids.err[stream]) *ids.err[stream] = SJD_DEVERR_TOKEN_ID;
    } else if (emb_rows) {
        v = *reinterpret_cast<const float4 *>(emb_rows + (size_t)r * d + j);
    } else if (sizeof(T) == 2) {
        const uint2 u = *reinterpret_cast<const uint2 *>(reinterpret_cast<const bf16_t *>(E) + (size_t)id * d + j);
        v = make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u), __uint_as_float(u.y << 16),
                        __uint_as_float(u.y & 0xFFFF0000u));
    } else {
        v = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(E) + (size_t)id * d + j);
    }
    const int row = (stream << shift) + r;
    float *dst = sizeof(T) == 2 ? x + act_off(row, j, d / 32) : x + (size_t)row * d + j;
    *reinterpret_cast<float4 *>(dst) = v;
    if (sizeof(T) == 2) {
        const uint2 gn = *reinterpret_cast<const uint2 *>(gain + j);
        act24_store4(x24, row, j, d / 32, v.x * __uint_as_float(gn.x << 16), v.y * __uint_as_float(gn.x & 0xFFFF0000u),
                     v.z * __uint_as_float(gn.y << 16), v.w * __uint_as_float(gn.y & 0xFFFF0000u), lo16 != 0);
        float sq = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, v.w * v.w)));
        sq += __shfl_xor(sq, 1);                      // 4 consecutive threads hold 16 consecutive features
        sq += __shfl_xor(sq, 2);
        if ((threadIdx.x & 3) == 0) ssq[(size_t)row * ssq_stride(d) + (j >> 4)] = sq;
    }
}

// x[r] += sum_p part[p][r]  (skipped when part == NULL);  h[r] = x[r] * rsqrt(mean(x[r]^2) + eps) * g
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(float *x, const float *part, int n_part, size_t part_stride,
                                                      const T *gain, int d, float eps, T *h,
                                                      const SjdState *st)
{
    if (st->done) return;
    __shared__ float red[4];
    const int r = blockIdx.x;
    float *xr = x + (size_t)r * d;
    float ss = 0.f;
    for (int j = threadIdx.x; j < d; j += 256) {
        float v = xr[j];
        for (int p = 0; p < n_part; ++p) v += part[(size_t)p * part_stride + (size_t)r * d + j];
        if (n_part) xr[j] = v;
        ss += v * v;
    }
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    ss = red[0] + red[1] + red[2] + red[3];
    const float inv = rsqrtf(ss / (float)d + eps);
    for (int j = threadIdx.x; j < d; j += 256) Act<T>::store(h, (size_t)r * d + j, xr[j] * inv * Act<T>::load(gain, j));
}

// qkv[r][0:3d] = sum_p part[p][r][:];  rotate q and k (pairs j, j+hd/2) at position n+r;
// q -> qact[r][d];  k -> K cache row n+r;  v -> V cache (bf16: transposed [head][hd][pos]).
template <typename T>
__global__ __launch_bounds__(256) void rope_kv_kernel(const float *part, int n_part, size_t part_stride, int d, int hd,
                                                      int max_seq, const float *cosT, const float *sinT, float *qact,
                                                      T *kc, T *vc, int v_transposed, int rows_valid,
                                                      int stream, const SjdState *st)
{
    if (st->done) return;
    const int r = blockIdx.x;
    const int pos = state_n(st, stream) + r;
    const int half = hd / 2;
    const size_t row = (size_t)r * 3 * d;
    for (int e = threadIdx.x; e < d / 2; e += 256) {
        const int head = e / half, j = e % half;
        const int c0 = head * hd + j, c1 = c0 + half;
        float q0 = 0, q1 = 0, k0 = 0, k1 = 0, v0 = 0, v1 = 0;
        for (int p = 0; p < n_part; ++p) {
            const float *src = part + (size_t)p * part_stride + row;
            q0 += src[c0]; q1 += src[c1];
            k0 += src[d + c0]; k1 += src[d + c1];
            v0 += src[2 * d + c0]; v1 += src[2 * d + c1];
        }
        const float c = cosT[(size_t)pos * half + j], s = sinT[(size_t)pos * half + j];
        qact[(size_t)r * d + c0] = q0 * c - q1 * s;
        qact[(size_t)r * d + c1] = q1 * c + q0 * s;
        if (r < rows_valid) {
            Act<T>::store(kc, (size_t)pos * d + c0, k0 * c - k1 * s);
            Act<T>::store(kc, (size_t)pos * d + c1, k1 * c + k0 * s);
            if (v_transposed) {
                Act<T>::store(vc, (size_t)c0 * max_seq + pos, v0);
                Act<T>::store(vc, (size_t)c1 * max_seq + pos, v1);
            } else {
                Act<T>::store(vc, (size_t)pos * d + c0, v0);
                Act<T>::store(vc, (size_t)pos * d + c1, v1);
            }
        }
    }
}

// ffn[r][f] = SiLU(g) * u with g = sum_p part[p][r][f], u = sum_p part[p][r][F + f]
template <typename T>
__global__ __launch_bounds__(256) void silu_mul_kernel(const float *part, int n_part, size_t part_stride, int F, T *ffn,
                                                       const SjdState *st)
{
    if (st->done) return;
    const int r = blockIdx.y;
    const int f = blockIdx.x * 256 + threadIdx.x;
    if (f >= F) return;
    float g = 0, u = 0;
    for (int p = 0; p < n_part; ++p) {
        const float *src = part + (size_t)p * part_stride + (size_t)r * 2 * F;
        g += src[f]; u += src[F + f];
    }
    Act<T>::store(ffn, (size_t)r * F + f, g / (1.0f + expf(-g)) * u);
}

// out[r][c] = sum_p part[p][r][c]
__global__ __launch_bounds__(256) void reduce_rows_kernel(const float *part, int n_part, size_t part_stride, int cols,
                                                          float *out, const SjdState *st)
{
    if (st && st->done) return;
    const int r = blockIdx.y;
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= cols) return;
    float v = 0;
    for (int p = 0; p < n_part; ++p) v += part[(size_t)p * part_stride + (size_t)r * cols + c];
    out[(size_t)r * cols + c] = v;
}

// ---------------------------------------------------------------------------------------------
#define LAUNCH_CHECK() HIP_TRY(hipGetLastError())

int sjd_launch_embed(const sjd_model *m, const int32_t *const *ids, const float *emb_rows, int32_t rows,
                     const SjdStreams &sm, float *x, void *x24, float *ssq, int32_t *const *err, bool lo16, hipStream_t s)
{
    if (sm.count < 1 || sm.count > SJD_MAX_STREAMS || rows < 1 || rows > (1 << sm.shift) ||
        (sm.count << sm.shift) > SJD_ROWS_MAX)
        return SJD_EINVAL;
    if (m->cfg.dtype == 0 && sm.count != 1) return SJD_EINVAL;
    if (m->cfg.dtype == 1 && (!x24 || !ssq)) return SJD_EINVAL;
    const int d = m->cfg.d_model;
    EmbedIds e;
    for (int i = 0; i < SJD_MAX_STREAMS; ++i) {
        e.p[i] = (ids && i < sm.count) ? ids[i] : nullptr;
        e.err[i] = (err && i < sm.count) ? err[i] : nullptr;
    }
    const dim3 grid(rows, (d + 1023) / 1024, sm.count);
    if (m->cfg.dtype == 0)
        SJD_LAUNCH(embed_kernel<float>, grid, dim3(256), 0, s, (const float *)m->E, e, emb_rows, d, sm.shift, x, x24, (const bf16_t *)nullptr, ssq, m->cfg.vocab_total, lo16 ? 1 : 0);
    else
        SJD_LAUNCH(embed_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t *)m->E, e, emb_rows, d, sm.shift, x, x24, (const bf16_t *)m->layers[0].g1, ssq, m->cfg.vocab_total, lo16 ? 1 : 0);
    LAUNCH_CHECK();
    return SJD_OK;
}

int sjd_launch_rmsnorm(const sjd_model *m, float *x, const float *part, int32_t n_part, size_t part_stride,
                       const void *gain, int32_t rows, void *h, const SjdState *st, hipStream_t s)
{
    const int d = m->cfg.d_model;
    if (m->cfg.dtype != 0) return SJD_EINVAL;   // bf16 models normalise inside the projection kernel
    SJD_LAUNCH(rmsnorm_kernel<float>, dim3(rows), dim3(256), 0, s, x, part, n_part, part_stride,
                       (const float *)gain, d, m->cfg.rms_eps, (float *)h, st);
    LAUNCH_CHECK();
    return SJD_OK;
}

int sjd_launch_rope_kv(const sjd_model *m, sjd_kv *kv, int32_t layer, int32_t stream, const float *part, int32_t n_part,
                       size_t part_stride, int32_t rows, int32_t rows_valid, hipStream_t s)
{
    const int d = m->cfg.d_model, ms = m->cfg.max_seq;
    if (m->cfg.dtype != 0) return SJD_EINVAL;   // bf16 models do this in the QKV GEMM epilogue
    float *kc = (float *)(stream ? kv->k_u : kv->k), *vc = (float *)(stream ? kv->v_u : kv->v);
    SJD_LAUNCH(rope_kv_kernel<float>, dim3(rows), dim3(256), 0, s, part, n_part, part_stride, d, m->hd, ms,
                       m->rope_cos, m->rope_sin, kv->qact, kc + (size_t)layer * kv->k_layer_stride,
                       vc + (size_t)layer * kv->v_layer_stride, 0, rows_valid, stream, kv->state);
    LAUNCH_CHECK();
    return SJD_OK;
}

int sjd_launch_silu_mul(const sjd_model *m, const float *part, int32_t n_part, size_t part_stride, int32_t rows,
                        void *ffn, const SjdState *st, hipStream_t s)
{
    const int F = m->cfg.d_ffn;
    if (m->cfg.dtype != 0) return SJD_EINVAL;   // bf16 models do this in the gate/up epilogue
    dim3 grid((F + 255) / 256, rows);
    SJD_LAUNCH(silu_mul_kernel<float>, grid, dim3(256), 0, s, part, n_part, part_stride, F, (float *)ffn, st);
    LAUNCH_CHECK();
    return SJD_OK;
}

int sjd_launch_reduce_rows(const float *part, int32_t n_part, size_t part_stride, int32_t rows, int32_t cols,
                           float *out, const SjdState *st, hipStream_t s)
{
    dim3 grid((cols + 255) / 256, rows);
    SJD_LAUNCH(reduce_rows_kernel, grid, dim3(256), 0, s, part, n_part, part_stride, cols, out, st);
    LAUNCH_CHECK();
    return SJD_OK;
}
