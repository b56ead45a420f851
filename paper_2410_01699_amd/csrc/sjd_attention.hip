// Window attention (paper Sec. 4.1 Step 2 "forward pass ... with a causal mask"): the `rows` window
// queries attend the n cached positions plus the window positions up to their own.  The key range
// is cut into `splits` chunks so that heads x splits workgroups cover the chip; every workgroup keeps
// an online-softmax state (running max, denominator, unnormalised output) for its chunk and a small
// second kernel merges the chunks in a fixed order.
//
// Two kernels: a generic one for the fp32 models (key/value tiles of 64 positions staged in LDS as
// fp32, plain FMA arithmetic) and an MFMA one for bf16 caches.
#include "sjd_internal.h"

#define ATT_TILE 64
#define ATT_THREADS 256

template <typename T> __device__ __forceinline__ float ld(const T *p, size_t i);
template <> __device__ __forceinline__ float ld<float>(const float *p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float ld<bf16_t>(const bf16_t *p, size_t i) { return bf16_to_f32(p[i]); }
// attention output feeds the O projection: bf16 models store it as hi/lo bf16 planes
template <typename T> __device__ __forceinline__ void st_act(T *p, int r, int c, int d, float v);
template <> __device__ __forceinline__ void st_act<float>(float *p, int r, int c, int d, float v) { p[(size_t)r * d + c] = v; }
template <> __device__ __forceinline__ void st_act<bf16_t>(bf16_t *p, int r, int c, int d, float v)
{
    const bf16_t hi = f32_to_bf16(v);
    const size_t o = act_off(r, c, d / 32);
    p[o] = hi;
    p[(size_t)SJD_ROWS_MAX * d + o] = f32_to_bf16(v - bf16_to_f32(hi));
}

// part layout per (head, split): [rows][hd] unnormalised output, then m[rows], then l[rows]
template <typename T, int HD>
__global__ __launch_bounds__(ATT_THREADS) void attn_partial_kernel(const float *__restrict__ qact, const T *__restrict__ kc,
                                                                   const T *__restrict__ vc, int d, int max_seq,
                                                                   int rows, int v_transposed, int splits,
                                                                   float *__restrict__ part, const SjdState *st)
{
    if (st->done) return;
    constexpr int ROWS = SJD_ROWS_MAX;
    constexpr int RG = ATT_THREADS / HD;          // row groups in the PV phase
    constexpr int RPT = (ROWS + RG - 1) / RG;     // rows per thread there
    __shared__ float qs[ROWS][HD + 1];
    __shared__ float ks[ATT_TILE][HD + 1];        // reused for V
    __shared__ float sc[ROWS][ATT_TILE];
    __shared__ float m_run[ROWS], l_run[ROWS], scale_old[ROWS];

    const int head = blockIdx.x, split = blockIdx.y, tid = threadIdx.x;
    const int n = st->n;
    const int total = n + rows;
    int chunk = (total + splits - 1) / splits;
    chunk = (chunk + ATT_TILE - 1) / ATT_TILE * ATT_TILE;
    const int k_beg = split * chunk, k_end = min(total, k_beg + chunk);
    const float inv_sqrt = rsqrtf((float)HD);

    for (int e = tid; e < ROWS * HD; e += ATT_THREADS) {
        int r = e / HD, j = e % HD;
        qs[r][j] = r < rows ? qact[(size_t)r * d + head * HD + j] * inv_sqrt : 0.f;
    }
    if (tid < ROWS) { m_run[tid] = -INFINITY; l_run[tid] = 0.f; }
    float acc[RPT];
#pragma unroll
    for (int i = 0; i < RPT; ++i) acc[i] = 0.f;
    const int pv_j = tid % HD, pv_g = tid / HD;
    __syncthreads();

    for (int t0 = k_beg; t0 < k_end; t0 += ATT_TILE) {
        const int tl = min(ATT_TILE, k_end - t0);
        for (int e = tid; e < ATT_TILE * HD; e += ATT_THREADS) {
            int kk = e / HD, j = e % HD;
            ks[kk][j] = kk < tl ? ld<T>(kc, (size_t)(t0 + kk) * d + head * HD + j) : 0.f;
        }
        __syncthreads();
        for (int e = tid; e < ROWS * ATT_TILE; e += ATT_THREADS) {
            int r = e / ATT_TILE, kk = e % ATT_TILE;
            float s = -INFINITY;
            if (r < rows && kk < tl && t0 + kk <= n + r) {     // causal inside the window
                s = 0.f;
#pragma unroll 8
                for (int j = 0; j < HD; ++j) s = fmaf(qs[r][j], ks[kk][j], s);
            }
            sc[r][kk] = s;
        }
        __syncthreads();
        // online softmax bookkeeping: one thread per row
        if (tid < ROWS) {
            const int r = tid;
            float mx = m_run[r];
            for (int kk = 0; kk < ATT_TILE; ++kk) mx = fmaxf(mx, sc[r][kk]);
            float so = (mx == -INFINITY) ? 1.f : expf(m_run[r] - mx);
            float sum = 0.f;
            for (int kk = 0; kk < ATT_TILE; ++kk) {
                float p = (sc[r][kk] == -INFINITY) ? 0.f : expf(sc[r][kk] - mx);
                sc[r][kk] = p;
                sum += p;
            }
            l_run[r] = l_run[r] * so + sum;
            m_run[r] = mx;
            scale_old[r] = so;
        }
        // V tile into ks
        for (int e = tid; e < ATT_TILE * HD; e += ATT_THREADS) {
            int kk, j;
            if (v_transposed) { j = e / ATT_TILE; kk = e % ATT_TILE; } else { kk = e / HD; j = e % HD; }
            float v = 0.f;
            if (kk < tl)
                v = v_transposed ? ld<T>(vc, (size_t)(head * HD + j) * max_seq + t0 + kk)
                                 : ld<T>(vc, (size_t)(t0 + kk) * d + head * HD + j);
            ks[kk][j] = v;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
            const int r = pv_g + i * RG;
            if (r < ROWS) {
                float a = acc[i] * scale_old[r];
                for (int kk = 0; kk < ATT_TILE; ++kk) a = fmaf(sc[r][kk], ks[kk][pv_j], a);
                acc[i] = a;
            }
        }
        __syncthreads();
    }
    float *dst = part + (size_t)(head * splits + split) * (ROWS * HD + 2 * ROWS);
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        const int r = pv_g + i * RG;
        if (r < ROWS) dst[r * HD + pv_j] = acc[i];
    }
    if (tid < ROWS) { dst[ROWS * HD + tid] = m_run[tid]; dst[ROWS * HD + ROWS + tid] = l_run[tid]; }
}

template <typename T, int HD>
__global__ void attn_combine_kernel(const float *__restrict__ part, int splits, int d, int rows, T *__restrict__ out,
                                    const SjdState *st)
{
    if (st->done) return;
    constexpr int ROWS = SJD_ROWS_MAX;
    const int head = blockIdx.x;
    for (int e = threadIdx.x; e < rows * HD; e += blockDim.x) {
        const int r = e / HD, j = e % HD;
        float mx = -INFINITY;
        for (int s = 0; s < splits; ++s)
            mx = fmaxf(mx, part[(size_t)(head * splits + s) * (ROWS * HD + 2 * ROWS) + ROWS * HD + r]);
        float num = 0.f, den = 0.f;
        for (int s = 0; s < splits; ++s) {
            const float *p = part + (size_t)(head * splits + s) * (ROWS * HD + 2 * ROWS);
            const float ms = p[ROWS * HD + r];
            if (ms == -INFINITY) continue;
            const float w = expf(ms - mx);
            num += w * p[r * HD + j];
            den += w * p[ROWS * HD + ROWS + r];
        }
        st_act<T>(out, r, head * HD + j, d, num / den);
    }
}

// ---------------------------------------------------------------------------------------------
// bf16 caches: MFMA kernel.  One wave per (head, key chunk); per block of 32 keys
//   S^T[key][query] = K[key][:] . Q[query][:]      A = K tile (16 keys x 32 dims, straight from the
//                                                   row-major K cache), B = Q (hi + lo bf16 planes)
//   O^T[dim][query] += V^T[dim][key] * P[key][query] A = V^T tile from the transposed V cache, B = P
// The two 16-key score tiles of a block leave lane l (query l%16, group g = l/16) with the keys
// {4g..4g+3} and {16+4g..16+4g+3}; using the same key order for the V^T operand makes the
// probabilities the B operand of the second product without any cross-lane movement.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ void split8(const float (&x)[8], bf16x8 &hi, bf16x8 &lo)
{
    union { bf16x8 v; bf16_t s[8]; } h, l;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        h.s[e] = f32_to_bf16(x[e]);
        l.s[e] = f32_to_bf16(x[e] - bf16_to_f32(h.s[e]));
    }
    hi = h.v; lo = l.v;
}

template <int HD, int MT>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const float *__restrict__ qact, const bf16_t *__restrict__ kc,
                                                        const bf16_t *__restrict__ vc, int d, int vstride, int rows,
                                                        int splits, float *__restrict__ part, const SjdState *st)
{
    if (st->done) return;
    constexpr int ROWS = SJD_ROWS_MAX;
    constexpr int KS = HD / 32;      // k-steps of the score product
    constexpr int DT = HD / 16;      // output dim tiles
    const int lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
    const int head = blockIdx.x;
    const int split = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (split >= splits) return;
    const int n = st->n;
    const int total = n + rows;
    int chunk = (total + splits - 1) / splits;
    chunk = (chunk + 31) / 32 * 32;
    const int k_beg = split * chunk, k_end = min(total, k_beg + chunk);
    const float scale = rsqrtf((float)HD);

    // Q as B operand: lane holds Q[query c (+16 mt)][32 ks + 8 g .. +8], scaled, hi/lo
    bf16x8 qh[MT][KS], ql[MT][KS];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            float x[8];
            const float *src = qact + (size_t)(mt * 16 + c) * d + head * HD + ks * 32 + g * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = src[e] * scale;
            split8(x, qh[mt][ks], ql[mt][ks]);
        }

    f32x4 o[MT][DT];
    float m_run[MT], l_run[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        m_run[mt] = -INFINITY; l_run[mt] = 0.f;
#pragma unroll
        for (int t = 0; t < DT; ++t) o[mt][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }

    for (int k0 = k_beg; k0 < k_end; k0 += 32) {
        // K tiles: keys k0 + c and k0 + 16 + c
        bf16x8 ka[2][KS];
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                ka[h][ks] = *reinterpret_cast<const bf16x8 *>(kc + (size_t)(k0 + h * 16 + c) * d + head * HD + ks * 32 + g * 8);
        // V^T tiles: dims 16 t + c, keys (k0 + 4g .. +4) and (k0 + 16 + 4g .. +4)
        bf16x8 va[DT];
#pragma unroll
        for (int t = 0; t < DT; ++t) {
            const bf16_t *vp = vc + (size_t)(head * HD + t * 16 + c) * vstride + k0 + g * 4;
            union { bf16x8 v; uint2 u[2]; } w;
            w.u[0] = *reinterpret_cast<const uint2 *>(vp);
            w.u[1] = *reinterpret_cast<const uint2 *>(vp + 16);
            va[t] = w.v;
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            f32x4 s[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                s[h] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    s[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[h][ks], qh[mt][ks], s[h], 0, 0, 0);
                    s[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[h][ks], ql[mt][ks], s[h], 0, 0, 0);
                }
            }
            // mask: key position <= n + query row; keys past the chunk end are masked too
            const int qrow = mt * 16 + c;
            float p[8];
            float mx = m_run[mt];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int key = k0 + (e >> 2) * 16 + g * 4 + (e & 3);
                const bool ok = key < k_end && key <= n + qrow && qrow < rows;
                p[e] = ok ? s[e >> 2][e & 3] : -INFINITY;
                mx = fmaxf(mx, p[e]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float so = (mx == -INFINITY) ? 1.f : __expf(m_run[mt] - mx);
            float sum = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                p[e] = (p[e] == -INFINITY) ? 0.f : __expf(p[e] - mx);
                sum += p[e];
            }
            sum += __shfl_xor(sum, 16);
            sum += __shfl_xor(sum, 32);
            l_run[mt] = l_run[mt] * so + sum;
            m_run[mt] = mx;
            bf16x8 ph, pl;
            split8(p, ph, pl);
#pragma unroll
            for (int t = 0; t < DT; ++t) {
                o[mt][t] *= so;
                o[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[t], ph, o[mt][t], 0, 0, 0);
                o[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[t], pl, o[mt][t], 0, 0, 0);
            }
        }
    }
    // partial: [rows][HD] unnormalised output, m[rows], l[rows]; lane holds dims 16t + 4g .. +4 of query c
    float *dst = part + (size_t)(head * splits + split) * (ROWS * HD + 2 * ROWS);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int t = 0; t < DT; ++t)
            *reinterpret_cast<f32x4 *>(dst + (size_t)(mt * 16 + c) * HD + t * 16 + g * 4) = o[mt][t];
        if (g == 0) { dst[ROWS * HD + mt * 16 + c] = m_run[mt]; dst[ROWS * HD + ROWS + mt * 16 + c] = l_run[mt]; }
    }
}

// merge of the key chunks, bf16 models: one workgroup per head; weights exp(m_s - M) per (row, chunk)
// are computed once into LDS, empty chunks are skipped, output goes out as hi/lo bf16 planes
template <int HD>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float *__restrict__ part, int splits, int d, int rows,
                                                         bf16_t *__restrict__ out, const SjdState *st)
{
    if (st->done) return;
    constexpr int ROWS = SJD_ROWS_MAX;
    constexpr int MAXS = 64;
    __shared__ float w[ROWS][MAXS];
    __shared__ float inv_den[ROWS];
    const int head = blockIdx.x;
    const size_t stride = ROWS * HD + 2 * ROWS;
    const float *base = part + (size_t)head * splits * stride;
    if (threadIdx.x < rows) {
        const int r = threadIdx.x;
        float mx = -INFINITY;
        for (int s = 0; s < splits; ++s) mx = fmaxf(mx, base[s * stride + ROWS * HD + r]);
        float den = 0.f;
        for (int s = 0; s < splits; ++s) {
            const float ms = base[s * stride + ROWS * HD + r];
            const float ww = (ms == -INFINITY) ? 0.f : __expf(ms - mx);
            w[r][s] = ww;
            den += ww * base[s * stride + ROWS * HD + ROWS + r];
        }
        inv_den[r] = 1.0f / den;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < rows * (HD / 4); e += 256) {
        const int r = e / (HD / 4), j = (e % (HD / 4)) * 4;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < splits; ++s) {
            const float ww = w[r][s];
            if (ww != 0.f) acc += ww * *reinterpret_cast<const f32x4 *>(base + s * stride + (size_t)r * HD + j);
        }
        acc *= inv_den[r];
        const size_t o = act_off(r, head * HD + j, d / 32);
        bf16_t hi[4], lo[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) { hi[q] = f32_to_bf16(acc[q]); lo[q] = f32_to_bf16(acc[q] - bf16_to_f32(hi[q])); }
        uint2 ph, pl;
        ph.x = (uint32_t)hi[0] | ((uint32_t)hi[1] << 16); ph.y = (uint32_t)hi[2] | ((uint32_t)hi[3] << 16);
        pl.x = (uint32_t)lo[0] | ((uint32_t)lo[1] << 16); pl.y = (uint32_t)lo[2] | ((uint32_t)lo[3] << 16);
        *reinterpret_cast<uint2 *>(out + o) = ph;
        *reinterpret_cast<uint2 *>(out + (size_t)ROWS * d + o) = pl;
    }
}

int32_t sjd_attention_splits(const sjd_model *m)
{
    if (m->cfg.dtype == 1) {
        // MFMA kernel: one wave per chunk, about 512 waves in all, chunks of at least 32 keys
        int s = (512 + m->cfg.n_heads - 1) / m->cfg.n_heads;
        s = (s + 3) / 4 * 4;
        if (s > 64) s = 64;
        int max_s = (m->cfg.max_seq + 31) / 32;
        max_s = (max_s + 3) / 4 * 4;
        if (s > max_s) s = max_s;
        return s < 4 ? 4 : s;
    }
    int s = (512 + m->cfg.n_heads - 1) / m->cfg.n_heads;   // about two workgroups per CU
    int max_s = (m->cfg.max_seq + ATT_TILE - 1) / ATT_TILE;
    if (s > max_s) s = max_s;
    return s < 1 ? 1 : s;
}

size_t sjd_attention_part_elems(const sjd_model *m)
{
    return (size_t)m->cfg.n_heads * sjd_attention_splits(m) * (SJD_ROWS_MAX * m->hd + 2 * SJD_ROWS_MAX);
}

template <typename T, int HD>
static int launch_t(const sjd_model *m, sjd_kv *kv, int32_t layer, int32_t rows, hipStream_t s)
{
    const int d = m->cfg.d_model, ms = m->cfg.max_seq, H = m->cfg.n_heads;
    hipLaunchKernelGGL((attn_partial_kernel<T, HD>), dim3(H, kv->att_splits), dim3(ATT_THREADS), 0, s,
                       kv->qact, (const T *)kv->k + (size_t)layer * kv->k_layer_stride,
                       (const T *)kv->v + (size_t)layer * kv->v_layer_stride, d, ms, rows, 0, kv->att_splits,
                       kv->att_part, kv->state);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL((attn_combine_kernel<T, HD>), dim3(H), dim3(256), 0, s, kv->att_part, kv->att_splits, d, rows,
                       (T *)kv->att_out, kv->state);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

template <int HD>
static int launch_mfma(const sjd_model *m, sjd_kv *kv, int32_t layer, int32_t rows, hipStream_t s)
{
    const int d = m->cfg.d_model, H = m->cfg.n_heads, splits = kv->att_splits;
    const bf16_t *kc = (const bf16_t *)kv->k + (size_t)layer * kv->k_layer_stride;
    const bf16_t *vc = (const bf16_t *)kv->v + (size_t)layer * kv->v_layer_stride;
    dim3 grid(H, splits / 4), block(256);
    if (rows <= 16)
        hipLaunchKernelGGL((attn_mfma_kernel<HD, 1>), grid, block, 0, s, kv->qact, kc, vc, d, kv->v_stride, rows, splits,
                           kv->att_part, kv->state);
    else
        hipLaunchKernelGGL((attn_mfma_kernel<HD, 2>), grid, block, 0, s, kv->qact, kc, vc, d, kv->v_stride, rows, splits,
                           kv->att_part, kv->state);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL((attn_merge_kernel<HD>), dim3(H), dim3(256), 0, s, kv->att_part, splits, d, rows,
                       (bf16_t *)kv->att_out, kv->state);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_launch_attention(const sjd_model *m, sjd_kv *kv, int32_t layer, int32_t rows, hipStream_t s)
{
    const int hd = m->hd;
    if (m->cfg.dtype == 1) {
        if (hd == 32) return launch_mfma<32>(m, kv, layer, rows, s);
        if (hd == 64) return launch_mfma<64>(m, kv, layer, rows, s);
        if (hd == 128) return launch_mfma<128>(m, kv, layer, rows, s);
        return SJD_EINVAL;
    }
    if (m->cfg.dtype == 0) {
        if (hd == 16) return launch_t<float, 16>(m, kv, layer, rows, s);
        if (hd == 32) return launch_t<float, 32>(m, kv, layer, rows, s);
        if (hd == 64) return launch_t<float, 64>(m, kv, layer, rows, s);
        if (hd == 128) return launch_t<float, 128>(m, kv, layer, rows, s);
    }
    return SJD_EINVAL;
}
