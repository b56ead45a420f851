// Window attention (paper Sec. 4.1 Step 2 "forward pass ... with a causal mask"): the `rows` window
// queries attend the n cached positions plus the window positions up to their own.  The key range
// is cut into `splits` chunks so that heads x splits workgroups cover the chip; every workgroup keeps
// an online-softmax state (running max, denominator, unnormalised output) for its chunk and a small
// second kernel merges the chunks in a fixed order.
//
// This is the generic kernel (fp32 and bf16 caches, any head size up to 128): key/value tiles of 64
// positions are staged in LDS as fp32.
#include "sjd_internal.h"

#define ATT_TILE 64
#define ATT_THREADS 256

template <typename T> __device__ __forceinline__ float ld(const T *p, size_t i);
template <> __device__ __forceinline__ float ld<float>(const float *p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float ld<bf16_t>(const bf16_t *p, size_t i) { return bf16_to_f32(p[i]); }
// attention output feeds the O projection: bf16 models store it as hi/lo bf16 planes
template <typename T> __device__ __forceinline__ void st_act(T *p, size_t plane, size_t i, float v);
template <> __device__ __forceinline__ void st_act<float>(float *p, size_t, size_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void st_act<bf16_t>(bf16_t *p, size_t plane, size_t i, float v)
{
    const bf16_t hi = f32_to_bf16(v);
    p[i] = hi;
    p[plane + i] = f32_to_bf16(v - bf16_to_f32(hi));
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
        st_act<T>(out, (size_t)ROWS * d, (size_t)r * d + head * HD + j, num / den);
    }
}

int32_t sjd_attention_splits(const sjd_model *m)
{
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
    const size_t per_layer = (size_t)ms * d;
    const int vt = m->cfg.dtype == 1;
    hipLaunchKernelGGL((attn_partial_kernel<T, HD>), dim3(H, kv->att_splits), dim3(ATT_THREADS), 0, s,
                       kv->qact, (const T *)kv->k + layer * per_layer, (const T *)kv->v + layer * per_layer,
                       d, ms, rows, vt, kv->att_splits, kv->att_part, kv->state);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL((attn_combine_kernel<T, HD>), dim3(H), dim3(256), 0, s, kv->att_part, kv->att_splits, d, rows,
                       (T *)kv->att_out, kv->state);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_launch_attention(const sjd_model *m, sjd_kv *kv, int32_t layer, int32_t rows, hipStream_t s)
{
    const int hd = m->hd;
    if (m->cfg.dtype == 0) {
        if (hd == 16) return launch_t<float, 16>(m, kv, layer, rows, s);
        if (hd == 32) return launch_t<float, 32>(m, kv, layer, rows, s);
        if (hd == 64) return launch_t<float, 64>(m, kv, layer, rows, s);
        if (hd == 128) return launch_t<float, 128>(m, kv, layer, rows, s);
    } else {
        if (hd == 16) return launch_t<bf16_t, 16>(m, kv, layer, rows, s);
        if (hd == 32) return launch_t<bf16_t, 32>(m, kv, layer, rows, s);
        if (hd == 64) return launch_t<bf16_t, 64>(m, kv, layer, rows, s);
        if (hd == 128) return launch_t<bf16_t, 128>(m, kv, layer, rows, s);
    }
    return SJD_EINVAL;
}
