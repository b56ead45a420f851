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

// One workgroup of AW waves per head.  Wave w takes the 32-key blocks w, w+AW, ... of the range
// [0, n+rows), prefetching the next block's K/V tiles while it works on the current one, and keeps
// an online-softmax state (running max, denominator, unnormalised O^T) per query.  The waves then
// agree on the per-query maximum through LDS, rescale, and their outputs are added AW/4... four
// waves at a time in wave order (fixed order -> deterministic); the result is written as hi/lo bf16
// planes in the layout the O projection streams.
#define AW 8
template <int HD, int MT>
__global__ __launch_bounds__(64 * AW) void attn_mfma_kernel(const float *__restrict__ qact,
                                                           const bf16_t *__restrict__ kc,
                                                           const bf16_t *__restrict__ vc, int d, int vstride,
                                                           int rows, bf16_t *__restrict__ out, const SjdState *st)
{
    if (st->done) return;
    constexpr int ROWS = SJD_ROWS_MAX;
    constexpr int KS = HD / 32;      // k-steps of the score product
    constexpr int DT = HD / 16;      // output dim tiles
    __shared__ float m_all[AW][MT * 16], l_all[AW][MT * 16];
    __shared__ f32x4 o_slot[4][DT][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
    const int head = blockIdx.x;
    const int n = st->n;
    const int total = n + rows;
    const float scale = rsqrtf((float)HD);

    __shared__ bf16x8 q_lds[MT][KS][2][64];
    f32x4 o[MT][DT];
    float m_run[MT], l_run[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        m_run[mt] = -INFINITY; l_run[mt] = 0.f;
#pragma unroll
        for (int t = 0; t < DT; ++t) o[mt][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }

    bf16x8 ka0[2][KS], ka1[2][KS], va0[DT], va1[DT];
    // K tiles: keys k0 + c and k0 + 16 + c (prefetched one block ahead); V^T tiles: dims 16 t + c,
    // keys (k0 + 4g .. +4), (k0 + 16 + 4g .. +4) (loaded when the block starts: their latency hides
    // behind the score product and the softmax)
#define LOAD_K(k0, ka)                                                                               \
    if ((k0) < total) {                                                                              \
        _Pragma("unroll") for (int h = 0; h < 2; ++h)                                                \
            _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                        \
                ka[h][ks] = *reinterpret_cast<const bf16x8 *>(kc + (size_t)((k0) + h * 16 + c) * d + head * HD + ks * 32 + g * 8); \
    }
#define LOAD_V(k0, va)                                                                               \
    if ((k0) < total) _Pragma("unroll") for (int t = 0; t < DT; ++t) {                                                 \
        const bf16_t *vp = vc + (size_t)(head * HD + t * 16 + c) * vstride + (k0) + g * 4;           \
        union { bf16x8 v; uint2 u[2]; } w_;                                                          \
        w_.u[0] = *reinterpret_cast<const uint2 *>(vp);                                              \
        w_.u[1] = *reinterpret_cast<const uint2 *>(vp + 16);                                         \
        va[t] = w_.v;                                                                                \
    }
#define COMPUTE_KV(k0, ka, va)                                                                       \
    _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) {                                              \
        f32x4 s_[2];                                                                                 \
        _Pragma("unroll") for (int h = 0; h < 2; ++h) {                                              \
            s_[h] = (f32x4){0.f, 0.f, 0.f, 0.f};                                                     \
            _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                      \
                s_[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[h][ks], q_lds[mt][ks][0][lane], s_[h], 0, 0, 0); \
                s_[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[h][ks], q_lds[mt][ks][1][lane], s_[h], 0, 0, 0); \
            }                                                                                        \
        }                                                                                            \
        const int qrow = mt * 16 + c;                                                                \
        float p_[8];                                                                                 \
        float mx = m_run[mt];                                                                        \
        _Pragma("unroll") for (int e = 0; e < 8; ++e) {                                              \
            const int key = (k0) + (e >> 2) * 16 + g * 4 + (e & 3);                                  \
            const bool ok = key <= n + qrow && qrow < rows;     /* causal inside the window */       \
            p_[e] = ok ? s_[e >> 2][e & 3] : -INFINITY;                                              \
            mx = fmaxf(mx, p_[e]);                                                                   \
        }                                                                                            \
        mx = fmaxf(mx, __shfl_xor(mx, 16));                                                          \
        mx = fmaxf(mx, __shfl_xor(mx, 32));                                                          \
        const float so = (mx == -INFINITY) ? 1.f : __expf(m_run[mt] - mx);                           \
        float sum = 0.f;                                                                             \
        _Pragma("unroll") for (int e = 0; e < 8; ++e) {                                              \
            p_[e] = (p_[e] == -INFINITY) ? 0.f : __expf(p_[e] - mx);                                 \
            sum += p_[e];                                                                            \
        }                                                                                            \
        sum += __shfl_xor(sum, 16);                                                                  \
        sum += __shfl_xor(sum, 32);                                                                  \
        l_run[mt] = l_run[mt] * so + sum;                                                            \
        m_run[mt] = mx;                                                                              \
        bf16x8 ph, pl;                                                                               \
        split8(p_, ph, pl);                                                                          \
        _Pragma("unroll") for (int t = 0; t < DT; ++t) {                                             \
            o[mt][t] *= so;                                                                          \
            o[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[t], ph, o[mt][t], 0, 0, 0);        \
            o[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[t], pl, o[mt][t], 0, 0, 0);        \
        }                                                                                            \
    }

    constexpr bool PREFETCH = (MT * HD <= 128);   // the biggest variant has no registers to spare
    int k0 = wave * 32;
    LOAD_K(k0, ka0) LOAD_V(k0, va0)               // in flight while Q is staged
    // Q as B operand, kept in LDS (all waves use the same tiles): entry [mt][ks][plane][lane] holds
    // Q[query c (+16 mt)][32 ks + 8 g .. +8], scaled by 1/sqrt(HD), as hi and lo bf16 planes
    for (int u = threadIdx.x; u < MT * KS * 64; u += 64 * AW) {
        const int l = u & 63, ks = (u >> 6) % KS, mt = (u >> 6) / KS;
        float x[8];
        const float4 *src = reinterpret_cast<const float4 *>(qact + (size_t)(mt * 16 + (l & 15)) * d + head * HD + ks * 32 + (l >> 4) * 8);
        const float4 x0 = src[0], x1 = src[1];
        x[0] = x0.x * scale; x[1] = x0.y * scale; x[2] = x0.z * scale; x[3] = x0.w * scale;
        x[4] = x1.x * scale; x[5] = x1.y * scale; x[6] = x1.z * scale; x[7] = x1.w * scale;
        bf16x8 hi, lo;
        split8(x, hi, lo);
        q_lds[mt][ks][0][l] = hi; q_lds[mt][ks][1][l] = lo;
    }

    __syncthreads();                              // q_lds ready
    if constexpr (PREFETCH) {
        while (k0 < total) {
            LOAD_K(k0 + AW * 32, ka1) LOAD_V(k0 + AW * 32, va1)
            COMPUTE_KV(k0, ka0, va0)
            k0 += AW * 32;
            if (k0 >= total) break;
            LOAD_K(k0 + AW * 32, ka0) LOAD_V(k0 + AW * 32, va0)
            COMPUTE_KV(k0, ka1, va1)
            k0 += AW * 32;
        }
    } else {
        while (k0 < total) {
            COMPUTE_KV(k0, ka0, va0)
            k0 += AW * 32;
            LOAD_K(k0, ka0) LOAD_V(k0, va0)
        }
        (void)ka1; (void)va1;
    }
#undef LOAD_K
#undef LOAD_V
#undef COMPUTE_KV

    // ---- merge the AW waves -------------------------------------------------------------------
    if (g == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) { m_all[wave][mt * 16 + c] = m_run[mt]; l_all[wave][mt * 16 + c] = l_run[mt]; }
    }
    __syncthreads();
    float inv_den[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        float M = -INFINITY;
        for (int w = 0; w < AW; ++w) M = fmaxf(M, m_all[w][mt * 16 + c]);
        float den = 0.f;
        for (int w = 0; w < AW; ++w) {
            const float mw = m_all[w][mt * 16 + c];
            den += (mw == -INFINITY) ? 0.f : __expf(mw - M) * l_all[w][mt * 16 + c];
        }
        inv_den[mt] = 1.0f / den;
        const float mine = (m_run[mt] == -INFINITY) ? 0.f : __expf(m_run[mt] - M);
#pragma unroll
        for (int t = 0; t < DT; ++t) o[mt][t] *= mine;
    }
    // add the rescaled outputs four waves at a time; waves 0..3 keep the running sums
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        for (int r = 1; r < AW / 4; ++r) {
            __syncthreads();
            if ((wave >> 2) == r) {
#pragma unroll
                for (int t = 0; t < DT; ++t) o_slot[wave & 3][t][lane] = o[mt][t];
            }
            __syncthreads();
            if (wave < 4) {
#pragma unroll
                for (int t = 0; t < DT; ++t) o[mt][t] += o_slot[wave][t][lane];
            }
        }
        // waves 0..3 -> slots, then wave 0 adds slots 1..3 in order and writes the head's output
        __syncthreads();
        if (wave < 4) {
#pragma unroll
            for (int t = 0; t < DT; ++t) o_slot[wave][t][lane] = o[mt][t];
        }
        __syncthreads();
        // 256 result fragments (DT x 64) per query tile: spread them over the workgroup
        for (int u = threadIdx.x; u < DT * 64; u += 64 * AW) {
            const int t = u >> 6, l = u & 63;
            f32x4 v = o_slot[0][t][l];
            v += o_slot[1][t][l]; v += o_slot[2][t][l]; v += o_slot[3][t][l];
            const int q = mt * 16 + (l & 15);
            if (q >= rows) continue;
            // per-query denominator lives with lane c == q of any wave: recompute from LDS
            float M = -INFINITY;
            for (int w = 0; w < AW; ++w) M = fmaxf(M, m_all[w][q]);
            float den = 0.f;
            for (int w = 0; w < AW; ++w) {
                const float mw = m_all[w][q];
                den += (mw == -INFINITY) ? 0.f : __expf(mw - M) * l_all[w][q];
            }
            v *= 1.0f / den;
            const size_t off = act_off(q, head * HD + t * 16 + (l >> 4) * 4, d / 32);
            bf16_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) { hi[e] = f32_to_bf16(v[e]); lo[e] = f32_to_bf16(v[e] - bf16_to_f32(hi[e])); }
            uint2 ph, pl;
            ph.x = (uint32_t)hi[0] | ((uint32_t)hi[1] << 16); ph.y = (uint32_t)hi[2] | ((uint32_t)hi[3] << 16);
            pl.x = (uint32_t)lo[0] | ((uint32_t)lo[1] << 16); pl.y = (uint32_t)lo[2] | ((uint32_t)lo[3] << 16);
            *reinterpret_cast<uint2 *>(out + off) = ph;
            *reinterpret_cast<uint2 *>(out + (size_t)ROWS * d + off) = pl;
        }
    }
    (void)inv_den;
}

int32_t sjd_attention_splits(const sjd_model *m)
{
    if (m->cfg.dtype == 1) return 1;   // the MFMA kernel merges its key chunks inside the workgroup
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
    const int d = m->cfg.d_model, H = m->cfg.n_heads;
    const bf16_t *kc = (const bf16_t *)kv->k + (size_t)layer * kv->k_layer_stride;
    const bf16_t *vc = (const bf16_t *)kv->v + (size_t)layer * kv->v_layer_stride;
    if (rows <= 16)
        hipLaunchKernelGGL((attn_mfma_kernel<HD, 1>), dim3(H), dim3(64 * AW), 0, s, kv->qact, kc, vc, d, kv->v_stride, rows,
                           (bf16_t *)kv->att_out, kv->state);
    else
        hipLaunchKernelGGL((attn_mfma_kernel<HD, 2>), dim3(H), dim3(64 * AW), 0, s, kv->qact, kc, vc, d, kv->v_stride, rows,
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
