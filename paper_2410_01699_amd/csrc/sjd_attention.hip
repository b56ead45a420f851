// Window attention (paper Sec. 4.1 Step 2 "forward pass ... with a causal mask"): the `rows` window
// queries attend the n cached positions plus the window positions up to their own.  The key range
// is cut into `splits` chunks so that heads x splits workgroups cover the chip; every workgroup keeps
// an online-softmax state (running max, denominator, unnormalised output) for its chunk and a small
// second kernel merges the chunks in a fixed order.
//
// Two implementations: a generic one for the fp32 models (key/value tiles of 64 positions staged in
// LDS as fp32, plain FMA arithmetic) and an MFMA one for the blocked hi/lo cache of bf16 models.
#include "sjd_internal.h"

#include <algorithm>

#define ATT_TILE 64
#define ATT_THREADS 256

template <typename T> __device__ __forceinline__ float ld(const T *p, size_t i);
template <> __device__ __forceinline__ float ld<float>(const float *p, size_t i) { return p[i]; }
template <typename T> __device__ __forceinline__ void st_act(T *p, int r, int c, int d, float v);
template <> __device__ __forceinline__ void st_act<float>(float *p, int r, int c, int d, float v) { p[(size_t)r * d + c] = v; }

// part layout per (head, split): [rows][hd] unnormalised output, then m[rows], then l[rows]
template <typename T, int HD>
__global__ __launch_bounds__(ATT_THREADS) void attn_partial_kernel(const float *__restrict__ qact, const T *__restrict__ kc,
                                                                   const T *__restrict__ vc, int d, int max_seq,
                                                                   int rows, int v_transposed, int splits,
                                                                   float *__restrict__ part, int stream,
                                                                   const SjdState *st)
{
    if (st->done) return;
    constexpr int ROWS = SJD_ROWS_F32;
    constexpr int RG = ATT_THREADS / HD;          // row groups in the PV phase
    constexpr int RPT = (ROWS + RG - 1) / RG;     // rows per thread there
    __shared__ float qs[ROWS][HD + 1];
    __shared__ float ks[ATT_TILE][HD + 1];        // reused for V
    __shared__ float sc[ROWS][ATT_TILE];
    __shared__ float m_run[ROWS], l_run[ROWS], scale_old[ROWS];

    const int head = blockIdx.x, split = blockIdx.y, tid = threadIdx.x;
    const int n = state_n(st, stream);
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
    constexpr int ROWS = SJD_ROWS_F32;
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
// bf16 models: MFMA kernels over the blocked hi/lo cache.  Per block of 32 positions
//   S^T[key][query] = K[key][:] . Q[query][:]       A = K tile (16 keys x 32 dims), B = Q
//   O^T[dim][query] += V^T[dim][key] * P[key][query] A = V^T tile (16 dims x 32 keys), B = P
// Both cache operands are stored exactly as the lanes consume them, so a wave fetches a block's K and
// V tiles as contiguous 1 KiB loads.  Every operand is a hi + lo bf16 pair; a product keeps the
// three leading terms hi*hi + hi*lo + lo*hi (about 16 significant bits).  The two 16-key score tiles
// of a block leave lane l (query l%16, group g = l/16) with the keys {4g..4g+3} and {16+4g..16+4g+3};
// the V^T tiles use the same key order, which makes the probabilities the B operand of the second
// product without any cross-lane movement.
//
// attn_split_kernel: workgroup (head, split) of AW waves takes a contiguous range of blocks; wave w
// handles every AW-th block of it with an online softmax (running max, denominator, unnormalised
// O^T per query); the waves are merged through LDS in wave order and the workgroup writes one
// partial result.  attn_merge_kernel combines the splits of a head in split order.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ void split8(const float (&x)[8], bf16x8 &hi, bf16x8 &lo)
{
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const __bf16 h = (__bf16)x[e];
        hi[e] = h;
        lo[e] = (__bf16)(x[e] - (float)h);
    }
}

#define AW 4
// partial record of (head, split): O[MT*16][HD] unnormalised, then m[MT*16], then l[MT*16]
template <int HD, int MT>
__global__ __launch_bounds__(64 * AW) void attn_split_kernel(const float *__restrict__ qact, SjdStreams sm,
                                                            size_t layer_off, int d, int nblk_cache, int rows,
                                                            int splits, int qgroups, float *__restrict__ part)
{
    // blockIdx.z = (stream, query group): the stream has its own cache and cache length and its queries in
    // rows (stream << shift)..; a stream with more than MT * 16 rows is covered by several groups of
    // MT * 16 consecutive queries, each walking the keys on its own
    const int stream = blockIdx.z / qgroups, qbase = (blockIdx.z % qgroups) * (MT * 16);
    const SjdStreamEntry ent = stream_entry(sm, stream);
    if (*ent.done) return;
    const int n = *ent.n;
    const bf16_t *__restrict__ kvc = ent.kvc + layer_off;
    const int row0 = (stream << sm.shift) + qbase;
    part += (size_t)blockIdx.z * gridDim.x * splits * (MT * 16 * HD + 2 * MT * 16);
    constexpr int KS = HD / 32;      // k-steps of the score product
    constexpr int DT = HD / 16;      // output dim tiles
    constexpr int REC = MT * 16 * HD + 2 * MT * 16;
    __shared__ float m_all[AW][MT * 16], l_all[AW][MT * 16];
    __shared__ f32x4 o_slot[AW][DT][64];
    __shared__ bf16x8 q_lds[MT][KS][2][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
    const int head = blockIdx.x, split = blockIdx.y;
    const int total = n + rows;
    const int nblk = (total + 31) >> 5;
    const int bps = (nblk + splits - 1) / splits;
    const int b_beg = split * bps, b_end = min(nblk, b_beg + bps);
    const float scale = rsqrtf((float)HD);

    // the first block's K and V tiles are requested before anything else, so that their latency
    // overlaps the staging of Q
    bf16x8 ka[2][KS][2], va[DT][2];
    auto load_block = [&](int blk) {
        const bf16x8 *rec = reinterpret_cast<const bf16x8 *>(kvc + kv_block_off(head, blk, nblk_cache, HD)) + lane;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int pl = 0; pl < 2; ++pl) ka[h][ks][pl] = rec[((h * KS + ks) * 2 + pl) * 64];
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int pl = 0; pl < 2; ++pl) va[t][pl] = rec[(2 * KS * 2 + t * 2 + pl) * 64];
    };
    int blk = b_beg + wave;
    if (blk < b_end) load_block(blk);

    // Q as B operand, shared by the waves: entry [mt][ks][plane][lane] holds
    // Q[query c (+16 mt)][32 ks + 8 g .. +8], scaled by 1/sqrt(HD), as hi and lo bf16 planes
    for (int u = threadIdx.x; u < MT * KS * 64; u += 64 * AW) {
        const int l = u & 63, ks = (u >> 6) % KS, mt = (u >> 6) / KS;
        float x[8];
        // (query rows past the stream's `rows` are masked below; the clamp keeps their loads inside qact)
        const int qr = min(row0 + mt * 16 + (l & 15), SJD_ROWS_MAX - 1);
        const float4 *src = reinterpret_cast<const float4 *>(qact + (size_t)qr * d + head * HD + ks * 32 + (l >> 4) * 8);
        const float4 x0 = src[0], x1 = src[1];
        x[0] = x0.x * scale; x[1] = x0.y * scale; x[2] = x0.z * scale; x[3] = x0.w * scale;
        x[4] = x1.x * scale; x[5] = x1.y * scale; x[6] = x1.z * scale; x[7] = x1.w * scale;
        bf16x8 hi, lo;
        split8(x, hi, lo);
        q_lds[mt][ks][0][l] = hi; q_lds[mt][ks][1][l] = lo;
    }

    f32x4 o[MT][DT];
    float m_run[MT], l_run[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        m_run[mt] = -INFINITY; l_run[mt] = 0.f;
#pragma unroll
        for (int t = 0; t < DT; ++t) o[mt][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    __syncthreads();                              // q_lds ready

    while (blk < b_end) {
        const int k0 = blk * 32;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            f32x4 s_[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                s_[h] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 qh = q_lds[mt][ks][0][lane], ql = q_lds[mt][ks][1][lane];
                    s_[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[h][ks][1], qh, s_[h], 0, 0, 0);
                    s_[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[h][ks][0], ql, s_[h], 0, 0, 0);
                    s_[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[h][ks][0], qh, s_[h], 0, 0, 0);
                }
            }
            const int qrow = qbase + mt * 16 + c;    // row inside the stream's window
            float p_[8];
            float mx = m_run[mt];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int key = k0 + (e >> 2) * 16 + g * 4 + (e & 3);
                const bool ok = key <= n + qrow && qrow < rows;     // causal inside the window
                p_[e] = ok ? s_[e >> 2][e & 3] : -INFINITY;
                mx = fmaxf(mx, p_[e]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float so = (mx == -INFINITY) ? 1.f : __expf(m_run[mt] - mx);
            float sum = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                p_[e] = (p_[e] == -INFINITY) ? 0.f : __expf(p_[e] - mx);
                sum += p_[e];
            }
            sum += __shfl_xor(sum, 16);
            sum += __shfl_xor(sum, 32);
            l_run[mt] = l_run[mt] * so + sum;
            m_run[mt] = mx;
            bf16x8 ph, pl;
            split8(p_, ph, pl);
#pragma unroll
            for (int t = 0; t < DT; ++t) {
                o[mt][t] *= so;
                o[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[t][1], ph, o[mt][t], 0, 0, 0);
                o[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[t][0], pl, o[mt][t], 0, 0, 0);
                o[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[t][0], ph, o[mt][t], 0, 0, 0);
            }
        }
        blk += AW;
        if (blk < b_end) load_block(blk);
    }

    // ---- merge the AW waves (wave order) and write the partial record -----------------------------
    if (g == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) { m_all[wave][mt * 16 + c] = m_run[mt]; l_all[wave][mt * 16 + c] = l_run[mt]; }
    }
    __syncthreads();
    float *dst = part + (size_t)(head * splits + split) * REC;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < AW; ++w) M = fmaxf(M, m_all[w][mt * 16 + c]);
        const float mine = (m_run[mt] == -INFINITY) ? 0.f : __expf(m_run[mt] - M);
        if (mt) __syncthreads();                  // o_slot is reused
#pragma unroll
        for (int t = 0; t < DT; ++t) o_slot[wave][t][lane] = o[mt][t] * mine;
        __syncthreads();
        for (int u = threadIdx.x; u < DT * 64; u += 64 * AW) {
            const int t = u >> 6, l = u & 63;
            f32x4 v = o_slot[0][t][l];
#pragma unroll
            for (int w = 1; w < AW; ++w) v += o_slot[w][t][l];
            // lane l holds dims 16 t + 4 (l/16) .. +4 of query l%16
            *reinterpret_cast<f32x4 *>(dst + (size_t)(mt * 16 + (l & 15)) * HD + t * 16 + (l >> 4) * 4) = v;
        }
        if (wave == 0 && g == 0) {
            float den = 0.f;
#pragma unroll
            for (int w = 0; w < AW; ++w) {
                const float mw = m_all[w][mt * 16 + c];
                den += (mw == -INFINITY) ? 0.f : __expf(mw - M) * l_all[w][mt * 16 + c];
            }
            dst[MT * 16 * HD + mt * 16 + c] = M;
            dst[MT * 16 * HD + MT * 16 + mt * 16 + c] = den;
        }
    }
}

// out[q][head*HD + :] = sum_s w_s O_s[q][:] / sum_s w_s l_s,  w_s = exp(m_s - max_s m_s), written as
// the hi / lo operand planes the O projection streams (act24_idx).  All loads of a thread are issued before anything
// depends on them (splits <= ATT_MAX_SPLITS).
#define ATT_MAX_SPLITS 16
template <int HD, int MT>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float *__restrict__ part, int splits, int d, int rows,
                                                        void *__restrict__ out, int shift, int qgroups, int lo16)
{
    constexpr int REC = MT * 16 * HD + 2 * MT * 16;
    constexpr int Q4 = HD / 4;
    const int head = blockIdx.x, stream = blockIdx.z / qgroups, qbase = (blockIdx.z % qgroups) * (MT * 16);
    const float *base = part + ((size_t)blockIdx.z * gridDim.x + head) * splits * REC;
    const int u = blockIdx.y * 256 + threadIdx.x;
    if (u >= min(rows - qbase, MT * 16) * Q4) return;
    const int q = u / Q4, j4 = u % Q4;
    float ms[ATT_MAX_SPLITS], ls[ATT_MAX_SPLITS];
    f32x4 os[ATT_MAX_SPLITS];
#pragma unroll
    for (int s = 0; s < ATT_MAX_SPLITS; ++s) {
        const float *p = base + (size_t)(s < splits ? s : 0) * REC;
        ms[s] = p[MT * 16 * HD + q];
        ls[s] = p[MT * 16 * HD + MT * 16 + q];
        os[s] = *reinterpret_cast<const f32x4 *>(p + (size_t)q * HD + j4 * 4);
    }
    float M = -INFINITY;
#pragma unroll
    for (int s = 0; s < ATT_MAX_SPLITS; ++s) if (s < splits) M = fmaxf(M, ms[s]);
    f32x4 num = {0.f, 0.f, 0.f, 0.f};
    float den = 0.f;
#pragma unroll
    for (int s = 0; s < ATT_MAX_SPLITS; ++s) {
        const float w = (s < splits && ms[s] != -INFINITY) ? __expf(ms[s] - M) : 0.f;   // an empty split holds zeros
        num += w * os[s];
        den += w * ls[s];
    }
    const f32x4 o = num * (1.0f / den);
    act24_store4(out, (stream << shift) + qbase + q, head * HD + j4 * 4, d / 32, o[0], o[1], o[2], o[3], lo16 != 0);
}

int32_t sjd_attention_splits(const sjd_model *m)
{
    const int H = m->cfg.n_heads;
    if (m->cfg.dtype == 1) {
        // about two workgroups per CU, but at least four 32-position blocks per split at full length
        int s = (512 + H - 1) / H;
        int max_s = ((m->cfg.max_seq + 31) / 32 + 3) / 4;
        if (s > max_s) s = max_s;
        if (s > 16) s = 16;              // ATT_MAX_SPLITS of the merge kernel
        return s < 1 ? 1 : s;
    }
    int s = (512 + H - 1) / H;   // about two workgroups per CU
    int max_s = (m->cfg.max_seq + ATT_TILE - 1) / ATT_TILE;
    if (s > max_s) s = max_s;
    return s < 1 ? 1 : s;
}

size_t sjd_attention_part_elems(const sjd_model *m)
{
    if (m->cfg.dtype == 0) return (size_t)m->cfg.n_heads * sjd_attention_splits(m) * (SJD_ROWS_F32 * m->hd + 2 * SJD_ROWS_F32);
    // (stream, query group) pairs of up to 32 rows each: one or two of them run at the full number of key
    // splits, more of them (up to SJD_MAX_STREAMS) split their keys less finely (never below one split
    // each), so that pairs x splits stays within 2 x the full number
    const int splits = std::max(sjd_attention_splits(m), SJD_MAX_STREAMS / 2);
    return (size_t)m->cfg.n_heads * 2 * splits * (32 * m->hd + 2 * 32);
}

template <typename T, int HD>
static int launch_t(const sjd_model *m, sjd_kv *kv, int32_t layer, int32_t rows, int32_t stream, hipStream_t s)
{
    const int d = m->cfg.d_model, ms = m->cfg.max_seq, H = m->cfg.n_heads;
    const T *kc = (const T *)(stream ? kv->k_u : kv->k), *vc = (const T *)(stream ? kv->v_u : kv->v);
    SJD_LAUNCH((attn_partial_kernel<T, HD>), dim3(H, kv->att_splits), dim3(ATT_THREADS), 0, s,
                       kv->qact, kc + (size_t)layer * kv->k_layer_stride,
                       vc + (size_t)layer * kv->v_layer_stride, d, ms, rows, 0, kv->att_splits,
                       kv->att_part, stream, kv->state);
    HIP_TRY(hipGetLastError());
    SJD_LAUNCH((attn_combine_kernel<T, HD>), dim3(H), dim3(256), 0, s, kv->att_part, kv->att_splits, d, rows,
                       (T *)kv->att_out, kv->state);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

template <int HD, int MT>
static int launch_mfma_t(const sjd_model *m, sjd_kv *kv, int32_t layer, int32_t rows, const SjdStreams &sm, bool lo16,
                         hipStream_t s)
{
    const int d = m->cfg.d_model, H = m->cfg.n_heads;
    const size_t off = (size_t)layer * kv->k_layer_stride;
    // (stream, query group) pairs: the partial-record buffer holds two of them at att_splits key splits;
    // more of them share it by splitting their keys less finely
    const int qgroups = (rows + MT * 16 - 1) / (MT * 16), pairs = sm.count * qgroups;
    const int splits = pairs <= 2 ? kv->att_splits : std::max(1, 2 * kv->att_splits / pairs);
    if (pairs * splits > 2 * std::max(kv->att_splits, SJD_MAX_STREAMS / 2)) return SJD_EINVAL;    // (what att_part holds)
    const int grows = std::min(rows, MT * 16);
    SJD_LAUNCH((attn_split_kernel<HD, MT>), dim3(H, splits, pairs), dim3(64 * AW), 0, s, kv->qact, sm, off, d,
                       kv->nblk, rows, splits, qgroups, kv->att_part);
    HIP_TRY(hipGetLastError());
    SJD_LAUNCH((attn_merge_kernel<HD, MT>), dim3(H, (grows * (HD / 4) + 255) / 256, pairs), dim3(256), 0, s, kv->att_part,
                       splits, d, rows, kv->att_out, sm.shift, qgroups, lo16 ? 1 : 0);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

template <int HD>
static int launch_mfma(const sjd_model *m, sjd_kv *kv, int32_t layer, int32_t rows, const SjdStreams &sm, bool lo16,
                       hipStream_t s)
{
    if (sm.count < 1 || sm.count > SJD_MAX_STREAMS || rows > (1 << sm.shift) || (sm.count << sm.shift) > SJD_ROWS_MAX)
        return SJD_EINVAL;
    if (rows <= 16) return launch_mfma_t<HD, 1>(m, kv, layer, rows, sm, lo16, s);
    return launch_mfma_t<HD, 2>(m, kv, layer, rows, sm, lo16, s);     // 32 queries per (stream, query group)
}

int sjd_launch_attention(const sjd_model *m, sjd_kv *kv, int32_t layer, int32_t rows, const SjdStreams &sm, bool lo16,
                         hipStream_t s)
{
    const int hd = m->hd;
    if (m->cfg.dtype != 1) return SJD_EINVAL;
    if (hd == 32) return launch_mfma<32>(m, kv, layer, rows, sm, lo16, s);
    if (hd == 64) return launch_mfma<64>(m, kv, layer, rows, sm, lo16, s);
    if (hd == 128) return launch_mfma<128>(m, kv, layer, rows, sm, lo16, s);
    return SJD_EINVAL;
}

int sjd_launch_attention_f32(const sjd_model *m, sjd_kv *kv, int32_t layer, int32_t rows, int32_t stream, hipStream_t s)
{
    const int hd = m->hd;
    if (m->cfg.dtype != 0 || stream < 0 || stream > 1) return SJD_EINVAL;
    if (hd == 16) return launch_t<float, 16>(m, kv, layer, rows, stream, s);
    if (hd == 32) return launch_t<float, 32>(m, kv, layer, rows, stream, s);
    if (hd == 64) return launch_t<float, 64>(m, kv, layer, rows, stream, s);
    if (hd == 128) return launch_t<float, 128>(m, kv, layer, rows, stream, s);
    return SJD_EINVAL;
}
