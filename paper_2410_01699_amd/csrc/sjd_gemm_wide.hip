// bf16 projections of a window forward with MORE than 32 rows (paper Sec. 4.1 Step 2 for windows of 64
// tokens, for guided windows of 32 -- two contexts -- and for batches of images that share one pass
// over the weights): C[M x N] = A[M x K] * W^T, M = 33 .. 128; also the down projection from 17 rows on and,
// in a whole-K variant, the gate/up projection at 17 .. 32 rows.
//
// With this many rows a workgroup can no longer afford a private copy of the activations per wave (M
// rows cost M * 96 bytes of activations per KiB of weights), so the roles inside a workgroup change
// with respect to the skinny kernel:
//  - the waves of a workgroup (four; three in the whole-K variant) split N: each streams its own packed
//    weight groups (the same layout the skinny kernel reads: every weight byte still leaves HBM once and
//    goes straight into the registers of the one wave that uses it);
//  - all of them walk the SAME k-steps, and the activation tiles of a stage of k-steps are staged in LDS by
//    the workgroup and read from there by every wave: L2 -> CU activation traffic drops by the number of
//    waves.  The producers of a wide forward's activations write the second operand ready made (2-byte lo
//    plane), so staging is a copy; the whole-K variant reads the 3-byte form and rebuilds the second operand
//    once per workgroup while it parks a tile;
//  - K is split across workgroups (grid.y) wherever N alone gives too few of them; every workgroup
//    writes its fp32 sums as whole accumulator fragments, and a second kernel adds the K-slices in
//    slice order (deterministic), applies the token factors of a folded RMSNorm and runs the same
//    epilogues as the skinny kernel (residual, SiLU * up, RoPE + cache write, plain store).  (Adding the
//    slices in the last workgroup to arrive instead was measured 3x slower: the device-scope fences around
//    its arrival counter write back and invalidate the L2 of the XCD.)
// At M = 128 the two MFMAs per weight tile and M-tile price the matrix cores at about 9.8 TB/s of
// weights; measured, the kernel runs at about a third of the bf16 MFMA peak there, bound by what a CU pulls
// through its L1 (2 bytes of activations per byte of weights at four waves per workgroup): the one regime
// of this path where matrix-core utilisation is a meaningful number.
#include "sjd_gemm_epi.h"

#include <algorithm>
#include <mutex>

// one pipeline stage = KU k-steps; LDS holds two stages of MT activation tiles as hi and lo operands
#define WIDE_WAVES 4

// The whole-K variant (FUSED: grid.y = 1, NW = 3 waves): for a projection with so many output features that N
// alone fills the chip (gate/up of the 7B model: 688 weight groups = 230 workgroups of three), up to 32 rows.
// The workgroup holds final sums, so it runs the epilogue itself (no partial sums, no second kernel), and it
// reads the activations in the 3-byte form the skinny kernel's other consumers of the same buffer read (P3:
// the second operand is rebuilt once per workgroup while a tile is parked in LDS).
template <int EPI, bool NORM, int MT, int TNE>
__device__ __forceinline__ void wide_fused_tail(const f32x4 (&acc)[MT][TNE], int TN, const int *grp, int groups, int N,
                                                const float *rs, const SjdGemmEpi &ep)
{
    const int lane = threadIdx.x & 63, g4 = lane >> 4, c = lane & 15;
#pragma unroll
    for (int t = 0; t < TNE; ++t) {
        const int j = t / TN;
        if (grp[j] >= groups) continue;
        const int ntile = grp[j] * TN + t % TN;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int f_m = mt * 16 + c, f_n0 = ntile * 16 + g4 * 4;
            EpiPre pre;
            preload_epilogue<EPI>(ep, N, f_m, f_n0, pre);
            f32x4 v = acc[mt][t];
            if (NORM) v *= rs[f_m];
            apply_epilogue<EPI>(ep, N, f_m, f_n0, v, pre);
        }
    }
}

template <int MT, int TN, int G, int KU, int NW, bool P3, bool FUSED>
__global__ __launch_bounds__(64 * NW, 2) void gemm_wide_kernel(const bf16_t *__restrict__ Wp,
                                                            const void *__restrict__ Xv, int N, int K, int kps,
                                                            f32x4 *__restrict__ part, const float *__restrict__ ssq_in,
                                                            float eps, SjdGemmEpi ep)
{
    constexpr int TNE = TN * G;               // 16-feature tiles per wave
    constexpr int TPS = KU * MT;              // activation tiles per stage
    constexpr int APT = TPS / NW;             // of which each wave fetches
    static_assert(TPS % NW == 0 && APT >= 1, "the waves share the staging of a stage evenly");
    extern __shared__ bf16x8 act_lds[];       // [2 stages][KU][MT][plane][64 lanes]
    __shared__ float rs_s[MT * 16];           // FUSED: token factors of a folded RMSNorm
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int KT = K / 32, NT = N / 16, groups = NT / TN;
    const int k0 = blockIdx.y * kps, k1 = min(KT, k0 + kps);

    const bf16x8 *xp = reinterpret_cast<const bf16x8 *>(Xv) + lane;
    const bf16x8 *xl = reinterpret_cast<const bf16x8 *>(reinterpret_cast<const char *>(Xv) + act24_lo_base(KT)) + lane;   // 2-byte lo plane
    const uint2 *xl8 = reinterpret_cast<const uint2 *>(reinterpret_cast<const char *>(Xv) + act24_lo_base(KT)) + lane;     // 1-byte lo plane (P3)
    const size_t ztile = (size_t)SJD_MTILES * KT;        // the all-zero tile behind every activation matrix
    const bf16x8 *zw = xp + ztile * 64;
    // this wave's packed weight groups (a group past the end reads the zero tile and stores nothing)
    const bf16x8 *wp[G];
    int grp[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
        grp[j] = (blockIdx.x * NW + wave) * G + j;
        wp[j] = grp[j] < groups ? reinterpret_cast<const bf16x8 *>(Wp) + (size_t)grp[j] * KT * TN * 64 + lane : nullptr;
    }

    f32x4 acc[MT][TNE];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < TNE; ++t) acc[mt][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // Weights: a ring of WD stages in registers, requested WD - 1 stages ahead of their use (a stage is
    // KU k-steps; HBM latency under load is several stages long).  Activations: both operand planes come
    // ready made (the forward's producers write the 2-byte lo plane), so a stage is requested from L2 one
    // stage ahead into registers and parked in LDS, tile by tile, between the products of the stage before.
    // stages of weights in registers: four, three or two, at most 32 weight tiles (128 registers) in all
    constexpr int WD = KU * TNE <= 4 ? 4 : KU * TNE <= 8 ? 3 : 2;
    bf16x8 a_[WD][KU][TNE];
    bf16x8 sh_[APT], sl_[APT];
    uint2 s8_[APT];                           // (P3: the byte plane entries instead of sl_)

    // All loads are unconditional: a k-step past this workgroup's slice fetches the zero tile.
#define LOAD_ACT(kbase)                                                                               \
    _Pragma("unroll") for (int i = 0; i < APT; ++i) {                                                 \
        const int ti_ = i * NW + wave, u_ = ti_ / MT, mt_ = ti_ % MT, kk_ = (kbase) + u_;             \
        const size_t tix_ = kk_ < k1 ? (size_t)mt_ * KT + kk_ : ztile;                                \
        sh_[i] = xp[tix_ * 64];                                                                       \
        if constexpr (P3) s8_[i] = xl8[tix_ * 64];                                                    \
        else sl_[i] = xl[tix_ * 64];                                                                  \
    }
#define PARK_TILE(buf, i)                                                                             \
    {                                                                                                 \
        const int ti_ = (i) * NW + wave, u_ = ti_ / MT, mt_ = ti_ % MT;                               \
        bf16x8 *dst_ = act_lds + ((((buf) * KU + u_) * MT + mt_) * 2) * 64 + lane;                    \
        dst_[0] = sh_[i];                                                                             \
        if constexpr (P3) dst_[64] = lo_from_byte_plane(sh_[i], s8_[i]);                              \
        else dst_[64] = sl_[i];                                                                       \
    }
#define STORE_ACT(buf) _Pragma("unroll") for (int i = 0; i < APT; ++i) PARK_TILE(buf, i)
#define LOAD_W(a, kbase)                                                                              \
    _Pragma("unroll") for (int u = 0; u < KU; ++u) {                                                  \
        const int kk_ = (kbase) + u;                                                                  \
        _Pragma("unroll") for (int j = 0; j < G; ++j)                                                 \
            _Pragma("unroll") for (int tn = 0; tn < TN; ++tn)                                         \
                a[u][j * TN + tn] = __builtin_nontemporal_load(                                       \
                    (kk_ < k1 && wp[j]) ? wp[j] + ((size_t)kk_ * TN + tn) * 64 : zw);                 \
    }
    // One stage of products.  The operand pairs of the STEPS = KU * MT (k-step, M-tile) steps are fetched from
    // LDS PD steps ahead of the MFMAs that use them, through a ring of PD + 1 register pairs, and the parking
    // of the next stage's activations is spread over the last steps (by then its loads have landed): a
    // scheduling barrier after every step keeps this order in the instruction stream (left to itself the
    // compiler reuses one register pair and waits for every LDS read in turn).
#define COMPUTE_AND_PARK(a, buf, buf_store)                                                           \
    {                                                                                                 \
        constexpr int STEPS = KU * MT, PD = STEPS < 3 ? STEPS : 3;                                    \
        bf16x8 bq_[PD + 1][2];                                                                        \
        const bf16x8 *base_ = act_lds + (size_t)(buf) * STEPS * 128 + lane;                           \
        _Pragma("unroll") for (int p = 0; p < PD; ++p) { bq_[p][0] = base_[p * 128]; bq_[p][1] = base_[p * 128 + 64]; } \
        _Pragma("unroll") for (int st = 0; st < STEPS; ++st) {                                        \
            if (st + PD < STEPS) {                                                                    \
                bq_[(st + PD) % (PD + 1)][0] = base_[(st + PD) * 128];                                \
                bq_[(st + PD) % (PD + 1)][1] = base_[(st + PD) * 128 + 64];                           \
            }                                                                                         \
            const int u = st / MT, mt = st % MT;                                                      \
            _Pragma("unroll") for (int t = 0; t < TNE; ++t) {                                         \
                acc[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u][t], bq_[st % (PD + 1)][0], acc[mt][t], 0, 0, 0); \
                acc[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u][t], bq_[st % (PD + 1)][1], acc[mt][t], 0, 0, 0); \
            }                                                                                         \
            if (st >= STEPS - APT) PARK_TILE(buf_store, st - (STEPS - APT))                           \
            __builtin_amdgcn_sched_barrier(0);                                                        \
        }                                                                                             \
    }
    // Round r (stage r at k-steps kt .. kt + KU): request stage r + 1's activations and stage r + WD - 1's
    // weights, multiply stage r from LDS buffer r % 2 and park stage r + 1's activations in the other
    // buffer.  The barrier at the end of a round orders "every wave has read buffer b" before "buffer b is
    // overwritten" one round later, and "buffer b ^ 1 is written" before it is read in the next round.
    // prologue: stage 0 of the activations, stages 0 .. WD - 2 of the weights; stage 0 into buffer 0
    LOAD_ACT(k0)
#pragma unroll
    for (int r = 0; r < WD - 1; ++r) LOAD_W(a_[r], k0 + r * KU)
    if constexpr (FUSED) {
        // sum(x^2) of every token from the partial sums its writer left (four threads per token, fixed order)
        if (ssq_in && threadIdx.x < MT * 64) {
            const int tok = threadIdx.x >> 2, sl = threadIdx.x & 3;
            const int NQ = ssq_stride(K) / 4;
            const f32x4 *pp = reinterpret_cast<const f32x4 *>(ssq_in + (size_t)tok * (NQ * 4));
            float t = 0.f;
#pragma unroll 8
            for (int i = sl; i < NQ; i += 4) { const f32x4 v = pp[i]; t += (v[0] + v[1]) + (v[2] + v[3]); }
            t += __shfl_xor(t, 1);
            t += __shfl_xor(t, 2);
            if (sl == 0) rs_s[tok] = rsqrtf(t / (float)K + eps);
        }
    }
    STORE_ACT(0)
    __syncthreads();
    constexpr int PERIOD = WD % 2 ? 2 * WD : WD;      // rounds after which both ring positions repeat
    for (int kt = k0; kt < k1;) {
#pragma unroll
        for (int r = 0; r < PERIOD; ++r) {
            LOAD_ACT(kt + KU)
            LOAD_W(a_[(r + WD - 1) % WD], kt + (WD - 1) * KU)
            __builtin_amdgcn_sched_barrier(0);
            COMPUTE_AND_PARK(a_[r % WD], r & 1, (r + 1) & 1)
            __syncthreads();
            kt += KU;
            if (kt >= k1) break;
        }
    }
#undef LOAD_ACT
#undef STORE_ACT
#undef PARK_TILE
#undef LOAD_W
#undef COMPUTE_AND_PARK

    if constexpr (FUSED) {
        // the whole reduction was this workgroup's: final sums, epilogue here
        switch (ep.kind) {
            case SJD_EPI_SILU: wide_fused_tail<SJD_EPI_SILU, true, MT, TNE>(acc, TN, grp, groups, N, rs_s, ep); break;
            default:
                if (ssq_in) wide_fused_tail<SJD_EPI_STORE, true, MT, TNE>(acc, TN, grp, groups, N, rs_s, ep);
                else wide_fused_tail<SJD_EPI_STORE, false, MT, TNE>(acc, TN, grp, groups, N, rs_s, ep);
                break;
        }
        return;
    }
    // fp32 sums of this K-slice, as whole accumulator fragments: [slice][m tile][n tile][lane]
#pragma unroll
    for (int j = 0; j < G; ++j) {
        if (grp[j] >= groups) continue;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int ntile = grp[j] * TN + tn;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                part[(((size_t)blockIdx.y * MT + mt) * NT + ntile) * 64 + lane] = acc[mt][j * TN + tn];
        }
    }
}

// Second kernel: adds the K-slices of every accumulator fragment in slice order, applies
// rsqrt(mean(x^2) + eps) of each token when an RMSNorm is folded into the projection (PRO_NORM: the
// planes held x * gain and ssq_in the per-16-feature sums of squares of x), and runs the epilogue.
// Workgroup (x, mt): M-tile mt, EPI_TILES consecutive n tiles; lane l of a wave holds features
// 16 ntile + 4 (l / 16) .. + 4 of token 16 mt + l % 16, exactly as the MFMA left them.
#define EPI_TILES 8
template <int EPI, int PRO>
__global__ __launch_bounds__(256) void gemm_wide_epilogue_kernel(const f32x4 *__restrict__ part, int KS, int MT, int NT,
                                                                 const float *__restrict__ ssq_in, float eps, int N, int K,
                                                                 SjdGemmEpi ep)
{
    __shared__ float rs[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
    const int mt = blockIdx.y;
    if (PRO == SJD_PRO_NORM) {
        // 16 threads per token add every 16th float4 of its row of partial sums, then fold
        const int tok = threadIdx.x >> 4, sl = threadIdx.x & 15;
        const int NQ = ssq_stride(K) / 4;
        const f32x4 *pp = reinterpret_cast<const f32x4 *>(ssq_in + (size_t)(mt * 16 + tok) * (NQ * 4));
        float t = 0.f;
        for (int i = sl; i < NQ; i += 16) { const f32x4 v = pp[i]; t += (v[0] + v[1]) + (v[2] + v[3]); }
        t += __shfl_xor(t, 8);
        t += __shfl_xor(t, 4);
        t += __shfl_xor(t, 2);
        t += __shfl_xor(t, 1);
        if (sl == 0) rs[tok] = rsqrtf(t / (float)K + eps);
        __syncthreads();
    }
    const float scale = PRO == SJD_PRO_NORM ? rs[c] : 1.0f;
    for (int i = wave; i < EPI_TILES; i += 4) {
        const int ntile = blockIdx.x * EPI_TILES + i;
        if (ntile >= NT) break;
        const int f_m = mt * 16 + c, f_n0 = ntile * 16 + g * 4;
        EpiPre pre;
        preload_epilogue<EPI>(ep, N, f_m, f_n0, pre);
        f32x4 v = part[((size_t)mt * NT + ntile) * 64 + lane];
        for (int y = 1; y < KS; ++y) v += part[(((size_t)y * MT + mt) * NT + ntile) * 64 + lane];
        if (PRO == SJD_PRO_NORM) v *= scale;
        apply_epilogue<EPI>(ep, N, f_m, f_n0, v, pre);
    }
}

// ---------------------------------------------------------------------------------------------
// launch
// ---------------------------------------------------------------------------------------------
static std::mutex g_wide_mutex;
static size_t g_wide_lds[5][4][3] = {};      // dynamic LDS already enabled per (MT/2, TN, G) instantiation

// k-steps per stage: 16 (k-step, M-tile) products between two workgroup barriers whatever the row count (a
// stage of few products would spend its time in the barrier); half of that where a wave holds 3 or 4 weight
// tiles per k-step
constexpr int wide_ku(int MT, int TNE) { return MT == 2 ? (TNE >= 3 ? 4 : 8) : MT == 4 ? (TNE >= 3 ? 2 : 4) : 2; }
#define WIDE_KU wide_ku(MT, TN * G)
template <int MT, int TN, int G>
static int enable_lds_t()
{
    const size_t lds = (size_t)2 * WIDE_KU * MT * 2 * 1024;
    if (lds <= 48 * 1024) return SJD_OK;
    std::lock_guard<std::mutex> lock(g_wide_mutex);
    if (g_wide_lds[MT / 2][TN][G] < lds) {
        HIP_TRY(hipFuncSetAttribute((const void *)gemm_wide_kernel<MT, TN, G, WIDE_KU, WIDE_WAVES, false, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
        g_wide_lds[MT / 2][TN][G] = lds;
    }
    return SJD_OK;
}

// Dynamic LDS above the default limit has to be enabled per kernel; done when a cache handle is created,
// so that launches recorded during graph capture never touch function attributes.
int sjd_gemm_wide_setup()
{
    SJD_TRY((enable_lds_t<8, 1, 1>())); SJD_TRY((enable_lds_t<8, 1, 2>())); SJD_TRY((enable_lds_t<8, 2, 1>()));
    SJD_TRY((enable_lds_t<8, 2, 2>())); SJD_TRY((enable_lds_t<8, 3, 1>()));
    SJD_TRY((enable_lds_t<4, 1, 1>())); SJD_TRY((enable_lds_t<4, 1, 2>())); SJD_TRY((enable_lds_t<4, 2, 1>()));
    SJD_TRY((enable_lds_t<2, 1, 1>())); SJD_TRY((enable_lds_t<2, 1, 2>())); SJD_TRY((enable_lds_t<2, 2, 1>()));
    return SJD_OK;
}

template <int MT, int TN, int G>
static int launch_wide_t(const SjdLinear *lin, const void *act, int ks, int kps, f32x4 *part, hipStream_t s)
{
    constexpr int KU = WIDE_KU;
    const size_t lds = (size_t)2 * KU * MT * 2 * 1024;
    SJD_TRY((enable_lds_t<MT, TN, G>()));
    const int groups = lin->N / 16 / TN;
    dim3 grid((groups + WIDE_WAVES * G - 1) / (WIDE_WAVES * G), ks);
    SJD_LAUNCH((gemm_wide_kernel<MT, TN, G, KU, WIDE_WAVES, false, false>), grid, dim3(64 * WIDE_WAVES), lds, s,
               (const bf16_t *)lin->w, act, lin->N, lin->K, kps, part, (const float *)nullptr, 0.f, SjdGemmEpi{});
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

template <int MT>
static int launch_wide_mt(const SjdLinear *lin, const void *act, int g, int ks, int kps, f32x4 *part, hipStream_t s)
{
    const int tn = lin->tn;
    if (tn == 1 && g == 1) return launch_wide_t<MT, 1, 1>(lin, act, ks, kps, part, s);
    if (tn == 1 && g == 2) return launch_wide_t<MT, 1, 2>(lin, act, ks, kps, part, s);
    if (tn == 2 && g == 1) return launch_wide_t<MT, 2, 1>(lin, act, ks, kps, part, s);
    if (tn == 2 && g == 2) return launch_wide_t<MT, 2, 2>(lin, act, ks, kps, part, s);
    if (tn == 3 && g == 1) return launch_wide_t<MT, 3, 1>(lin, act, ks, kps, part, s);
    return SJD_EINVAL;
}

// Workgroups and K-slices: every slice at least 8 k-steps long, and the partial sums of all slices inside
// `part_elems` floats.
void sjd_wide_plan(const SjdLinear *lin, int mt, size_t part_elems, int *g_out, int *ks_out, int *kps_out)
{
    const int KT = lin->K / 32, groups = lin->N / 16 / lin->tn;
    // two weight groups per wave: one-tile groups, and two-tile groups of a long N up to 64 rows (at more rows
    // the accumulators of four tiles per M-tile no longer fit the registers)
    int g = lin->wg > 0 ? lin->wg : (lin->tn == 1 || (lin->tn == 2 && mt <= 4 && groups >= 512) ? 2 : 1);
    if (lin->tn == 3) g = 1;
    if (g > 2) g = 2;
    const int wgx = (groups + WIDE_WAVES * g - 1) / (WIDE_WAVES * g);
    // K-slices (measured on the 7B shapes at 64 and 128 rows): about 256 workgroups where N alone gives at
    // most 128 of them; 4 slices up to 256, 2 up to 512 (more slices cost more partial-sum traffic than the
    // extra workgroups win), none above
    int ks = lin->wks > 0 ? lin->wks : wgx >= 512 ? 1 : wgx >= 256 ? 2 : wgx > 128 ? 4 : (256 + wgx - 1) / wgx;
    if (lin->wks <= 0 && lin->tn == 2 && g == 2) ks = 2;      // (measured: 86 wide workgroups x 2 beat x 3 and x 4)
    ks = std::max(1, std::min(ks, KT / 8 > 0 ? KT / 8 : 1));
    const size_t per_slice = (size_t)mt * 16 * lin->N;
    while (ks > 1 && per_slice * ks > part_elems) --ks;
    const int ku = wide_ku(mt, lin->tn * g);
    int kps = (KT + ks - 1) / ks;
    kps = (kps + ku - 1) / ku * ku;             // whole stages
    ks = (KT + kps - 1) / kps;
    *g_out = g; *ks_out = ks; *kps_out = kps;
}

// The whole-K variant: three waves per workgroup, two-tile weight groups, activations in the 3-byte form, up to 32
// rows, epilogue in the kernel.  Stages of 6 k-steps (12 activation tiles, four per wave).
#define WIDE3_KU 6
template <int MT>
static int launch_wide3_t(const SjdLinear *lin, const void *act, const float *ssq_in, float eps, const SjdGemmEpi &ep,
                          hipStream_t s)
{
    const size_t lds = (size_t)2 * WIDE3_KU * MT * 2 * 1024;          // 24 or 48 KB
    const int groups = lin->N / 16 / 2, KT = lin->K / 32;
    dim3 grid((groups + 2) / 3, 1);
    SJD_LAUNCH((gemm_wide_kernel<MT, 2, 1, WIDE3_KU, 3, true, true>), grid, dim3(192), lds, s, (const bf16_t *)lin->w, act, lin->N,
               lin->K, KT, (f32x4 *)nullptr, ssq_in, eps, ep);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_launch_gemm_wide3(const SjdLinear *lin, const void *act, const float *ssq_in, float eps, int32_t rows,
                          const SjdGemmEpi &ep, hipStream_t s)
{
    if (rows < 1 || rows > 32 || lin->tn != 2 || lin->N % 32 || lin->K % 32) return SJD_EINVAL;
    // (plain store with or without a folded RMSNorm, SiLU(gate) * up behind one: what the shapes that come here use)
    const bool ok = ssq_in ? (ep.kind == SJD_EPI_STORE || ep.kind == SJD_EPI_SILU) : ep.kind == SJD_EPI_STORE;
    if (!ok) return SJD_EINVAL;
    return launch_wide3_t<2>(lin, act, ssq_in, eps, ep, s);       // (two M-tiles whatever the row count)
}

int sjd_launch_gemm_wide(const SjdLinear *lin, const void *act, const float *ssq_in, float eps, int32_t rows,
                         const SjdGemmEpi &ep, float *part, size_t part_elems, hipStream_t s)
{
    if (rows < 1 || rows > SJD_ROWS_MAX || !part) return SJD_EINVAL;
    if (lin->tn < 1 || lin->tn > 3 || lin->N % (16 * lin->tn) || lin->K % 32) return SJD_EINVAL;
    if (ep.kind == SJD_EPI_RESID && ep.out24 && (!ep.gain_next || !ep.ssq_out)) return SJD_EINVAL;
    int mt = (rows + 15) / 16;
    mt = (mt + 1) & ~1;                          // variants for 32, 64, 96 and 128 rows
    if ((size_t)mt * 16 * lin->N > part_elems) return SJD_EINVAL;
    int g, ks, kps;
    sjd_wide_plan(lin, mt, part_elems, &g, &ks, &kps);
    f32x4 *p4 = reinterpret_cast<f32x4 *>(part);
    int rc;
    switch (mt) {
        case 2: rc = launch_wide_mt<2>(lin, act, g, ks, kps, p4, s); break;
        case 4: rc = launch_wide_mt<4>(lin, act, g, ks, kps, p4, s); break;
        case 6: rc = launch_wide_mt<6>(lin, act, g, ks, kps, p4, s); break;
        default: rc = launch_wide_mt<8>(lin, act, g, ks, kps, p4, s); break;
    }
    SJD_TRY(rc);
    const int NT = lin->N / 16;
    dim3 grid((NT + EPI_TILES - 1) / EPI_TILES, mt);
#define GO(EPI, PRO) SJD_LAUNCH((gemm_wide_epilogue_kernel<EPI, PRO>), grid, dim3(256), 0, s, p4, ks, mt, NT, ssq_in, eps, lin->N, lin->K, ep)
    if (ssq_in) {
        switch (ep.kind) {
            case SJD_EPI_STORE: GO(SJD_EPI_STORE, SJD_PRO_NORM); break;
            case SJD_EPI_SILU: GO(SJD_EPI_SILU, SJD_PRO_NORM); break;
            case SJD_EPI_QKV: GO(SJD_EPI_QKV, SJD_PRO_NORM); break;
            default: return SJD_EINVAL;
        }
    } else {
        switch (ep.kind) {
            case SJD_EPI_STORE: GO(SJD_EPI_STORE, SJD_PRO_A24); break;
            case SJD_EPI_RESID: GO(SJD_EPI_RESID, SJD_PRO_A24); break;
            default: return SJD_EINVAL;
        }
    }
#undef GO
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}
