// bf16 skinny-M projections of the window forward (paper Sec. 4.1 Step 2) with fused prologue and
// epilogues.
//
// C[M x N] = A[M x K] * W^T, M = window size (16 or 32 rows), is a pure weight stream: every weight
// is read from HBM once and used for M multiply-adds (about M flop per byte, far left of the MFMA
// ridge), so the design goal is HBM bandwidth, not matrix-core throughput.
//
//  - W is pre-packed (sjd_repack_bf16) into 16x32 tiles in the exact A-operand register order of
//    v_mfma_f32_16x16x32_bf16: one 16-byte load per lane fetches 1 KiB of contiguous HBM per wave.
//  - The activations are the B operand (tokens on the 16 columns), multiplied as a pair of bf16
//    operands hi + lo: ~16 significant bits.  Inside the model they arrive from L2 in 3 bytes per
//    value, stored by their producers in B-operand order (act24_idx): the bf16 hi plane is the first
//    operand as stored, the second is rebuilt from the byte plane.  The test hook can also pass fp32
//    values in the same order (act_off), split on the fly into hi = bf16(x) and lo = bf16(x - hi).
//    A wave reuses each activation tile for its TN weight tiles, so TN sets the ratio of L2 to HBM
//    traffic.
//  - RMSNorm in front of a projection is folded in and costs the streaming loop nothing: whoever
//    writes the residual stream (the residual epilogue, the embedding kernel) leaves the planes of
//    x * gain of the NEXT normalisation, plus the sum of squares of x over its 16 features per
//    token; the projection behind the normalisation adds those partial sums (every workgroup in the
//    same order, so they agree bit for bit) and applies rsqrt(mean(x^2) + eps) of each token to its
//    final sums (the factor is constant along the reduction).
//  - One workgroup owns TN output tiles (16*TN features) for the WHOLE reduction; its WK waves
//    split K between them and add their fp32 accumulators through LDS in wave order.  No global
//    partial sums, no atomics: results are deterministic and the epilogue sees final values.
//    (A stream-K variant that balanced work across waves through global partial tiles and a ticket
//    counter was measured 2-4x slower here: the device-scope fences it needs write back L2.)
//  - Each wave keeps U k-steps of loads in flight ahead of the MFMAs (register double buffering);
//    U = 2, or 4 for long walks over 16 rows.
//  - Epilogues see final fp32 values: plain store (LM head logits), residual add into the fp32
//    stream (O and down projections), SiLU(gate)*up (gate and up rows are interleaved inside each
//    tile when packed, so a lane holds both), RoPE + KV-cache write (Q/K rows of a head are packed
//    as (j, j+hd/2) pairs, so the rotation is lane-local).
#include "sjd_gemm_epi.h"

// ---------------------------------------------------------------------------------------------
// in-workgroup split-K
// ---------------------------------------------------------------------------------------------
template <int MT, int TN, int WK, int U, int EPI, int PRO>
__global__ __launch_bounds__(64 * WK) void gemm_fused_kernel(const bf16_t *__restrict__ Wp,
                                                            const void *__restrict__ Xv,
                                                            const float *__restrict__ ssq_in, float eps, int N, int K,
                                                            SjdGemmEpi ep)
{
    static_assert(MT * TN * 64 <= 64 * WK, "one epilogue fragment per thread");
    __shared__ f32x4 red[WK][MT * TN][64];
    __shared__ float ssq[WK][MT * 16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
    const int tile0 = blockIdx.x * TN;
    const int KT = K / 32;
    const int kps = (KT + WK - 1) / WK;
    const int kt0 = wave * kps;
    const int kt1 = min(KT, kt0 + kps);
    // Workgroups walk their k-range from different starting points (and wrap around): all workgroups
    // of a launch read the same activation tiles, and in lockstep they would all want the same few
    // cache lines at the same moment.  The starting point depends on the workgroup index only, so the
    // summation order of a given output is the same in every launch.
    const int klen = max(kt1 - kt0, 1);
    // (short walks gain nothing from it)
    const int rot = klen >= 16 ? (int)((((blockIdx.x >> 3) & 31u) * (unsigned)klen) >> 5) : 0;   // in [0, klen)

    f32x4 acc[MT][TN];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) acc[mt][tn] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // weights: the TN tiles of a k-step are adjacent (in 16-byte units)
    const bf16x8 *wp = reinterpret_cast<const bf16x8 *>(Wp) + (size_t)blockIdx.x * KT * TN * 64 + lane;
    // this lane's activation values: token c (+16 mt), columns 32 kt + 8 g .. +8, as two float4, or as
    // 8 bf16 of the hi plane and 8 bytes of the lo plane
    constexpr bool A24 = PRO != SJD_PRO_PLAIN;                                  // operand planes (3 or 4 bytes per value)
    constexpr bool L16 = PRO == SJD_PRO_NORM16 || PRO == SJD_PRO_A16;           // the lo plane holds bf16 values
    constexpr bool NORM = PRO == SJD_PRO_NORM || PRO == SJD_PRO_NORM16;
    const f32x4 *xp = reinterpret_cast<const f32x4 *>(Xv) + lane;
    const uint2 *xl = reinterpret_cast<const uint2 *>(reinterpret_cast<const char *>(Xv) + act24_lo_base(KT)) + lane;
    const f32x4 *xp16 = reinterpret_cast<const f32x4 *>(reinterpret_cast<const char *>(Xv) + act24_lo_base(KT)) + lane;
    // an all-zero weight tile: the tile behind the activations (fp32: tile SJD_MTILES * KT of 2 KiB;
    // planes: tile SJD_MTILES * KT of the hi plane, 1 KiB)
    const bf16x8 *zw = reinterpret_cast<const bf16x8 *>(xp + (size_t)SJD_MTILES * KT * (A24 ? 64 : 128));

    bf16x8 a0[U][TN], a1[U][TN];
    f32x4 b0[U][MT][2], b1[U][MT][2];

    // Loads are unconditional (no branch between issue and use, so that the compiler can count
    // exactly which loads must have landed before a stage is consumed).  A k-step past this wave's
    // range fetches the all-zero tile that follows every activation matrix, for both operands.
#define LOAD_STAGE(kbase, a, b)                                                                   \
    _Pragma("unroll") for (int u = 0; u < U; ++u) {                                               \
        const int ki_ = (kbase) + u;              /* position in this wave's walk */              \
        const bool ok_ = ki_ < kt1;                                                               \
        const int kr_ = ki_ + rot;                                                                \
        const int kq_ = kr_ >= kt1 ? kr_ - klen : kr_;                                            \
        _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) {   /* L2 hits first: they return first */ \
            const size_t tix_ = ok_ ? (size_t)mt * KT + kq_ : (size_t)SJD_MTILES * KT;            \
            if (L16) {                                                                            \
                b[u][mt][0] = xp[tix_ * 64];                          /* 8 bf16 of either plane */ \
                b[u][mt][1] = xp16[tix_ * 64];                                                    \
            } else if (A24) {                                                                     \
                b[u][mt][0] = xp[tix_ * 64];                          /* 8 bf16 of the hi plane */ \
                const uint2 l_ = xl[tix_ * 64];                                                   \
                b[u][mt][1][0] = __uint_as_float(l_.x); b[u][mt][1][1] = __uint_as_float(l_.y);   \
            } else {                                                                              \
                b[u][mt][0] = xp[tix_ * 128];                                                     \
                b[u][mt][1] = xp[tix_ * 128 + 64];                                                \
            }                                                                                     \
        }                                                                                         \
        _Pragma("unroll") for (int tn = 0; tn < TN; ++tn)                                         \
            a[u][tn] = __builtin_nontemporal_load(ok_ ? wp + ((size_t)kq_ * TN + tn) * 64 : zw);  \
    }
#define MMA_STAGE(a, b)                                                                           \
    _Pragma("unroll") for (int u = 0; u < U; ++u)                                                 \
        _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) {                                       \
            bf16x8 bh_, bl_;                                                                      \
            if (L16) {                                                                            \
                bh_ = __builtin_bit_cast(bf16x8, b[u][mt][0]);                                    \
                bl_ = __builtin_bit_cast(bf16x8, b[u][mt][1]);                                    \
            } else if (A24) {                                                                     \
                /* value = hi bits | lo byte << 8 (as fp32); second operand = value - hi, exact */ \
                bh_ = __builtin_bit_cast(bf16x8, b[u][mt][0]);                                    \
                _Pragma("unroll") for (int e = 0; e < 8; ++e) {                                   \
                    const uint32_t hw_ = __float_as_uint(b[u][mt][0][e >> 1]);                    \
                    const uint32_t lw_ = __float_as_uint(b[u][mt][1][e >> 2]);                    \
                    const uint32_t hb_ = (e & 1) ? (hw_ & 0xFFFF0000u) : (hw_ << 16);             \
                    const uint32_t lb_ = ((lw_ >> (8 * (e & 3))) & 0xFFu) << 8;                   \
                    bl_[e] = (__bf16)(__uint_as_float(hb_ | lb_) - __uint_as_float(hb_));         \
                }                                                                                 \
            } else {                                                                              \
                float x_[8];                                                                      \
                _Pragma("unroll") for (int e = 0; e < 8; ++e) x_[e] = b[u][mt][e >> 2][e & 3];    \
                split8(x_, bh_, bl_);                                                             \
            }                                                                                     \
            _Pragma("unroll") for (int tn = 0; tn < TN; ++tn) {                                   \
                acc[mt][tn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u][tn], bh_, acc[mt][tn], 0, 0, 0); \
                acc[mt][tn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u][tn], bl_, acc[mt][tn], 0, 0, 0); \
            }                                                                                     \
        }

    // (An iteration enqueued after its generation has finished is not skipped here: it recomputes rows
    // nobody reads, inside the buffers and the cache, and the verification that follows leaves the
    // loop state alone.  Reading a finished flag first would put a dependent scalar load in front of
    // every launch's first weight loads.)
    // sum(x^2) of token c (+16 mt): K/16 partial sums left by whoever wrote x (rows of ssq_stride(K)
    // floats, zero padded).  Wave w, lane group g fetch every (4 WK)-th float4 of the row before the
    // first weights are requested (loads return in order: they have landed by the time the first
    // stage has, without a wait of their own) and add them up after the main loop; groups and waves
    // are added below in a fixed order.
    constexpr int PJ = 4;
    f32x4 pr[MT][PJ];
    const int NQ = ssq_stride(K) / 4, slice = wave * 4 + g;
    if (NORM) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const f32x4 *pp = reinterpret_cast<const f32x4 *>(ssq_in + (size_t)(mt * 16 + c) * (NQ * 4));
#pragma unroll
            for (int j = 0; j < PJ; ++j)
                pr[mt][j] = pp[min(slice + j * 4 * WK, NQ - 1)];    // (past the row's end: a duplicate, dropped below)
        }
    }
    LOAD_STAGE(kt0, a0, b0)
    // epilogue fragment of this thread (threads past MT*TN*64 have none and fetch a duplicate): D
    // layout of tile mtn puts features 4*(l/16) .. +4 of token l%16 in lane l
    const bool has_frag = threadIdx.x < MT * TN * 64;
    const int f_mtn = min((int)(threadIdx.x >> 6), MT * TN - 1);
    const int f_m = (f_mtn / TN) * 16 + c, f_n0 = (tile0 + f_mtn % TN) * 16 + g * 4;
    EpiPre pre;
    preload_epilogue<EPI>(ep, N, f_m, f_n0, pre);
    int kt = kt0;
    // (the scheduling barriers keep the compiler from starting on the previous stage before the next
    // one's loads are issued, which would drain the memory pipeline once per iteration)
    for (; kt + 2 * U < kt1; kt += 2 * U) {      // the stage loaded last still lies inside the range
        LOAD_STAGE(kt + U, a1, b1)
        __builtin_amdgcn_sched_barrier(0);
        MMA_STAGE(a0, b0)
        __builtin_amdgcn_sched_barrier(0);
        LOAD_STAGE(kt + 2 * U, a0, b0)
        __builtin_amdgcn_sched_barrier(0);
        MMA_STAGE(a1, b1)
        __builtin_amdgcn_sched_barrier(0);
    }
    LOAD_STAGE(kt + U, a1, b1)
    __builtin_amdgcn_sched_barrier(0);
    MMA_STAGE(a0, b0)
    MMA_STAGE(a1, b1)
#undef LOAD_STAGE
#undef MMA_STAGE

    // add the WK accumulators in wave order (fixed order -> deterministic)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) red[wave][mt * TN + tn][lane] = acc[mt][tn];
    if (NORM) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float t = 0.f;
#pragma unroll
            for (int j = 0; j < PJ; ++j)
                t += slice + j * 4 * WK < NQ ? (pr[mt][j][0] + pr[mt][j][1]) + (pr[mt][j][2] + pr[mt][j][3]) : 0.f;
            // (rows longer than 4 * PJ * 4 WK partial sums: the rest, latency exposed)
            const f32x4 *pp = reinterpret_cast<const f32x4 *>(ssq_in + (size_t)(mt * 16 + c) * (NQ * 4));
            for (int i = slice + PJ * 4 * WK; i < NQ; i += 4 * WK) { const f32x4 v = pp[i]; t += (v[0] + v[1]) + (v[2] + v[3]); }
            t += __shfl_xor(t, 16);
            t += __shfl_xor(t, 32);
            if (g == 0) ssq[wave][mt * 16 + c] = t;
        }
    }
    __syncthreads();
    if (has_frag) {
        f32x4 v = red[0][f_mtn][lane];
#pragma unroll
        for (int w = 1; w < WK; ++w) v += red[w][f_mtn][lane];
        if (NORM) {
            float sq = ssq[0][f_m];
#pragma unroll
            for (int w = 1; w < WK; ++w) sq += ssq[w][f_m];
            v *= rsqrtf(sq / (float)K + eps);
        }
        apply_epilogue<EPI>(ep, N, f_m, f_n0, v, pre);
    }
}

// ---------------------------------------------------------------------------------------------
// weight and activation packing
// ---------------------------------------------------------------------------------------------
// row-major [N][K] bf16 -> MFMA streaming order (tn tiles interleaved along k), packed row n' taken
// from source row perm(n')
//   perm 0: identity
//   perm 1: rows [0, 2d) (Q then K) reordered inside each head to (j, j+hd/2) pairs; rest identity
//   perm 2: N = 2F, packed (gate f, up f) interleaved: n' even -> row n'/2, odd -> row F + n'/2
__global__ void repack_bf16_kernel(const bf16_t *__restrict__ src, bf16_t *__restrict__ dst, int N, int K, int tn,
                                   int perm, int d, int hd)
{
    const int KT = K / 32;
    const size_t total = (size_t)N * K / 8;   // 16-byte groups
    for (size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (size_t)gridDim.x * blockDim.x) {
        const int l = (int)(g & 63);
        const size_t tile = g >> 6;
        const int t = (int)(tile % tn);
        const int kt = (int)((tile / tn) % KT);
        const size_t nt = tile / ((size_t)tn * KT) * tn + t;
        size_t np = nt * 16 + (l & 15), row = np;
        if (perm == 1 && np < (size_t)2 * d) {
            const size_t region = np / d * d, c = np % d;
            const size_t head = c / hd, p = c % hd;
            row = region + head * hd + (p >> 1) + ((p & 1) ? hd / 2 : 0);
        } else if (perm == 2) {
            row = (np >> 1) + ((np & 1) ? (size_t)N / 2 : 0);
        }
        const bf16_t *s = src + row * (size_t)K + (size_t)kt * 32 + (l >> 4) * 8;
        reinterpret_cast<uint4 *>(dst)[g] = *reinterpret_cast<const uint4 *>(s);
    }
}

int sjd_repack_bf16(const bf16_t *src_dev, bf16_t *dst_dev, int32_t N, int32_t K, int32_t tn, int32_t perm, int32_t d,
                    int32_t hd, hipStream_t s)
{
    if (N % 16 || K % 32 || tn < 1 || (N / 16) % tn) return SJD_EINVAL;
    if (perm == 1 && (hd % 8 || d % hd || N < 2 * d)) return SJD_EINVAL;
    if (perm == 2 && N % 32) return SJD_EINVAL;
    SJD_LAUNCH(repack_bf16_kernel, dim3(2048), dim3(256), 0, s, src_dev, dst_dev, N, K, tn, perm, d, hd);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

// row-major bf16 [rows][K] -> fp32 in act_off order (test hook)
__global__ void bf16_rows_to_f32_kernel(const bf16_t *__restrict__ src, size_t n, int K, float *__restrict__ dst)
{
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (size_t)gridDim.x * blockDim.x)
        dst[act_off((int)(e / K), (int)(e % K), K / 32)] = bf16_to_f32(src[e]);
}

// row-major fp32 [rows][K] -> hi / lo planes (test hook)
__global__ void f32_rows_to_act24_kernel(const float *__restrict__ src, size_t n, int K, void *__restrict__ dst, int lo16)
{
    const int KT = K / 32;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (size_t)gridDim.x * blockDim.x) {
        const uint32_t v = f32_to_act24(src[e]);
        const size_t i = act24_idx((int)(e / K), (int)(e % K), KT);
        ((bf16_t *)dst)[i] = (bf16_t)(v >> 16);
        if (lo16) *reinterpret_cast<bf16_t *>((uint8_t *)dst + act24_lo_base(KT) + 2 * i) = (bf16_t)act24_lo16(v);
        else ((uint8_t *)dst)[act24_lo_base(KT) + i] = (uint8_t)(v >> 8);
    }
}

// row-major bf16 [rows][K] -> hi / lo planes (test hook; exact: the byte plane is zero)
__global__ void bf16_rows_to_act24_kernel(const bf16_t *__restrict__ src, size_t n, int K, void *__restrict__ dst)
{
    const int KT = K / 32;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (size_t)gridDim.x * blockDim.x) {
        const size_t i = act24_idx((int)(e / K), (int)(e % K), KT);
        ((bf16_t *)dst)[i] = src[e];       // (the lo plane stays as allocated: zero in either form)
    }
}

int sjd_bf16_rows_to_act24(const bf16_t *src, int32_t rows, int32_t K, void *dst, hipStream_t s)
{
    if (rows < 1 || rows > SJD_ROWS_MAX || K < 32 || K % 32) return SJD_EINVAL;
    SJD_LAUNCH(bf16_rows_to_act24_kernel, dim3(256), dim3(256), 0, s, src, (size_t)rows * K, K, dst);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_f32_rows_to_act24(const float *src, int32_t rows, int32_t K, void *dst, bool lo16, hipStream_t s)
{
    if (rows < 1 || rows > SJD_ROWS_MAX || K < 32 || K % 32) return SJD_EINVAL;
    SJD_LAUNCH(f32_rows_to_act24_kernel, dim3(256), dim3(256), 0, s, src, (size_t)rows * K, K, dst, lo16 ? 1 : 0);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_bf16_rows_to_f32(const bf16_t *src, int32_t rows, int32_t K, float *dst, hipStream_t s)
{
    if (rows < 1 || rows > SJD_ROWS_MAX || K < 32 || K % 32) return SJD_EINVAL;
    SJD_LAUNCH(bf16_rows_to_f32_kernel, dim3(256), dim3(256), 0, s, src, (size_t)rows * K, K, dst);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

// ---------------------------------------------------------------------------------------------
// configuration and launch
// ---------------------------------------------------------------------------------------------
// Tiles per workgroup: fill the 256 CUs evenly.  Among tilings that waste about the same share of
// the last round of workgroups, prefer the largest TN (fewest re-reads of the activations).
void sjd_choose_tiles(SjdLinear *lin)
{
    const int tiles = lin->N / 16;
    int best_tn = 1;
    double best_eff = -1.0;
    for (int t = 1; t <= 3; ++t) {
        if (tiles % t) continue;
        const int blocks = tiles / t;
        if (blocks < 128 && t > 1) continue;
        const double eff = (double)blocks / (256.0 * ((blocks + 255) / 256));
        if (eff > best_eff + 0.02 || (eff > best_eff - 0.02 && t > best_tn)) {
            if (eff > best_eff) best_eff = eff;
            best_tn = t;
        }
    }
    lin->tn = best_tn; lin->wk = 0; lin->u = 0; lin->wg = 0; lin->wks = 0; lin->wide_from = 0;
    // two-tile groups, at least 512 of them (N >= 16384): three per workgroup still give one workgroup to most CUs
    lin->whole_k_rows = (best_tn == 2 && tiles / 2 >= 512) ? 32 : 0;
}

template <int MT, int TN, int WK, int U, int PRO>
static int launch_epi(const SjdLinear *lin, const void *act, const float *ssq_in, float eps, const SjdGemmEpi &ep,
                      hipStream_t s)
{
    if constexpr (WK * MT * TN * 1024 + WK * MT * 64 <= 65536) {
        dim3 grid(lin->N / (16 * TN)), block(64 * WK);
        const bf16_t *W = (const bf16_t *)lin->w;
#define GO(EPI) SJD_LAUNCH((gemm_fused_kernel<MT, TN, WK, U, EPI, PRO>), grid, block, 0, s, W, act, ssq_in, eps, lin->N, lin->K, ep)
        if constexpr (PRO == SJD_PRO_A24 || PRO == SJD_PRO_A16) {
            // (the plane activations feed the residual projections; the plain store serves the test hook)
            switch (ep.kind) {
                case SJD_EPI_STORE: GO(SJD_EPI_STORE); break;
                case SJD_EPI_RESID: GO(SJD_EPI_RESID); break;
                default: return SJD_EINVAL;
            }
        } else {
            switch (ep.kind) {
                case SJD_EPI_STORE: GO(SJD_EPI_STORE); break;
                case SJD_EPI_RESID: GO(SJD_EPI_RESID); break;
                case SJD_EPI_SILU: GO(SJD_EPI_SILU); break;
                case SJD_EPI_QKV: GO(SJD_EPI_QKV); break;
                default: return SJD_EINVAL;
            }
        }
#undef GO
        HIP_TRY(hipGetLastError());
        return SJD_OK;
    } else {
        return SJD_EINVAL;
    }
}

int sjd_launch_gemm_bf16(const SjdLinear *lin, const void *act, int form, const float *ssq_in, float eps, int32_t rows,
                         const SjdGemmEpi &ep, float *part, size_t part_elems, hipStream_t s)
{
    const bool act24 = form != SJD_ACT_F32, lo16 = form == SJD_ACT_P4;
    if (rows < 1 || rows > SJD_ROWS_MAX || (ssq_in && !act24) || form < 0 || form > 2) return SJD_EINVAL;
    // the wide kernel: above SJD_ROWS_SKINNY rows, or from lin->wide_from rows on; it reads the 4-byte planes
    const bool wide = rows > SJD_ROWS_SKINNY || (lin->wide_from > 0 && rows >= lin->wide_from && lo16 && part);
    if (wide) {
        if (!lo16) return SJD_EINVAL;
        return sjd_launch_gemm_wide(lin, act, ssq_in, eps, rows, ep, part, part_elems, s);
    }
    // the wide kernel's whole-K variant (shapes whose N alone fills the chip; activations in the 3-byte form)
    // (measured inside 7B iterations: 5 % of an iteration at 32 rows; at 16 rows the skinny kernel is 2 % ahead)
    if (rows > 16 && rows <= lin->whole_k_rows && form == SJD_ACT_P3 &&
        (ep.kind == SJD_EPI_SILU || ep.kind == SJD_EPI_STORE) && (ssq_in || ep.kind == SJD_EPI_STORE))
        return sjd_launch_gemm_wide3(lin, act, ssq_in, eps, rows, ep, s);
    if (ep.kind == SJD_EPI_RESID && ep.out24 && (!ep.gain_next || !ep.ssq_out)) return SJD_EINVAL;
    if (lin->tn < 1 || lin->N % (16 * lin->tn) || lin->K % 32) return SJD_EINVAL;
    const int mt = rows <= 16 ? 1 : 2;
    const int tn = lin->tn;               // fixed when the weights were packed
    // waves per workgroup: 0 = automatic.  Four waves (longer k-range per wave, more workgroups per CU, one
    // of which can run its epilogue while another streams) measured 2-8 % faster inside a 7B iteration
    // than eight where a workgroup holds at most three accumulator fragments; eight with four or more.
    int wk = lin->wk;
    // (four fragments over a short reduction -- eight waves would walk fewer than 16 k-steps each -- also run
    // better on four waves: 12-21 % on the 775M shapes at 32 rows)
    if (wk == 0) wk = (mt * tn <= 3 || (mt * tn == 4 && lin->K / 32 / 8 < 16)) ? 4 : 8;
    if (wk != 8 && wk != 4) return SJD_EINVAL;
    // k-steps per prefetch stage: 0 = automatic.  Four instead of two: 1 % of a 7B iteration and 1.4 % of a
    // 775M one, for 16 rows and four waves that each walk at least 32 k-steps (alone on cold weights
    // only the single-tile shapes gain, 6-7 %, and two-tile ones lose as much; inside an iteration none
    // loses); shorter walks and 32 rows are 6-29 % slower with four.
    int u = lin->u;
    if (u == 0) u = (mt == 1 && wk == 4 && lin->K / 32 / wk >= 32) ? 4 : 2;
    if (u == 4) {
        if (mt != 1 || wk != 4) return SJD_EINVAL;       // (the only deep variants built)
#define DEEP(TN)                                                                                      \
        if (tn == TN) {                                                                               \
            if (lo16 && ssq_in) return launch_epi<1, TN, 4, 4, SJD_PRO_NORM16>(lin, act, ssq_in, eps, ep, s); \
            if (lo16) return launch_epi<1, TN, 4, 4, SJD_PRO_A16>(lin, act, ssq_in, eps, ep, s);      \
            if (ssq_in) return launch_epi<1, TN, 4, 4, SJD_PRO_NORM>(lin, act, ssq_in, eps, ep, s);   \
            if (act24) return launch_epi<1, TN, 4, 4, SJD_PRO_A24>(lin, act, ssq_in, eps, ep, s);     \
            return launch_epi<1, TN, 4, 4, SJD_PRO_PLAIN>(lin, act, ssq_in, eps, ep, s);              \
        }
        DEEP(1) DEEP(2) DEEP(3)
#undef DEEP
        return SJD_EINVAL;
    }
    if (u != 2) return SJD_EINVAL;
#define CASE(MT, TN)                                                                                      \
    if (mt == MT && tn == TN) {                                                                           \
        if constexpr (MT * TN <= 4) {                                                                     \
            if (wk == 4) {                                                                                \
                if (lo16 && ssq_in) return launch_epi<MT, TN, 4, 2, SJD_PRO_NORM16>(lin, act, ssq_in, eps, ep, s); \
                if (lo16) return launch_epi<MT, TN, 4, 2, SJD_PRO_A16>(lin, act, ssq_in, eps, ep, s);         \
                if (ssq_in) return launch_epi<MT, TN, 4, 2, SJD_PRO_NORM>(lin, act, ssq_in, eps, ep, s);      \
                if (act24) return launch_epi<MT, TN, 4, 2, SJD_PRO_A24>(lin, act, ssq_in, eps, ep, s);      \
                return launch_epi<MT, TN, 4, 2, SJD_PRO_PLAIN>(lin, act, ssq_in, eps, ep, s);               \
            }                                                                                             \
        } else if (wk == 4) return SJD_EINVAL;                                                            \
        if (lo16 && ssq_in) return launch_epi<MT, TN, 8, 2, SJD_PRO_NORM16>(lin, act, ssq_in, eps, ep, s);    \
        if (lo16) return launch_epi<MT, TN, 8, 2, SJD_PRO_A16>(lin, act, ssq_in, eps, ep, s);                 \
        if (ssq_in) return launch_epi<MT, TN, 8, 2, SJD_PRO_NORM>(lin, act, ssq_in, eps, ep, s);              \
        if (act24) return launch_epi<MT, TN, 8, 2, SJD_PRO_A24>(lin, act, ssq_in, eps, ep, s);              \
        return launch_epi<MT, TN, 8, 2, SJD_PRO_PLAIN>(lin, act, ssq_in, eps, ep, s);                       \
    }
    CASE(1, 1) CASE(1, 2) CASE(1, 3)
    CASE(2, 1) CASE(2, 2) CASE(2, 3)
#undef CASE
    return SJD_EINVAL;
}
