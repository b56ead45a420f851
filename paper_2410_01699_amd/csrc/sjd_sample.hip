// Sampling distribution, probabilistic verification and window slide for SJD on gfx950.
//
// Paper Sec. 3.1 (softmax classifier + top-K sampling), Sec. 4.1 Step 3 (Eqs. 1-3) and Step 4,
// Sec. 4.2 (initialisation of new slots).  Two kernels per iteration:
//   sjd_rows_kernel      one workgroup per window index i = 1..L: top-K select (radix select on
//                        order-preserving keys held in LDS), softmax, the accept test of Eq. 1 for
//                        its own draft, a candidate sample from q_i (Eq. 3) and a candidate sample
//                        from max(0, q_i - p_old_i) (Eq. 2).  Nothing here depends on where the scan
//                        stops, so all rows run concurrently.
//   sjd_finalize_kernel  a few workgroups per slot of the NEXT window: finds the first rejection, picks
//                        the candidates that apply, copies the distributions into next-window order,
//                        initialises the tail slots and advances the device-resident state.
//
// Every data-dependent decision is an integer comparison or one correctly rounded fp32 operation
// (this file is compiled with floating-point contraction off), so results do not depend on
// reduction order: sums that decide anything are taken in 40-bit fixed point.
#include "sjd_internal.h"

#include <cstring>
#include <mutex>

#define DIST_THREADS 1024
#define DIST_WAVES (DIST_THREADS / 64)

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  key = seed, counter = (step counter, window index, 0).
// Output words in order: accept test, residual resample, plain sample, slot initialisation.
// ---------------------------------------------------------------------------------------------
struct U4 { uint32_t w[4]; };

__device__ __forceinline__ U4 philox_draw(uint64_t seed, uint64_t c, uint32_t i)
{
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    uint32_t c0 = (uint32_t)c, c1 = (uint32_t)(c >> 32), c2 = i, c3 = 0u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
        uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
        c0 = h1 ^ c1 ^ k0; c1 = l1; c2 = h0 ^ c3 ^ k1; c3 = l0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    U4 o; o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
    return o;
}

__device__ __forceinline__ float u_from_word(uint32_t w) { return __fmul_rn((float)(w >> 8), 0x1p-24f); }

// exp(x), x <= 0, as a fixed sequence of correctly rounded fp32 operations (Cody-Waite reduction,
// degree-7 Taylor polynomial); exactly 0 below -60.
__device__ __forceinline__ float exp_fixed(float x)
{
    if (!(x >= -60.0f)) return 0.0f;
    float n = rintf(__fmul_rn(x, 1.44269504088896341f));
    float r = __fmaf_rn(n, -0.693145751953125f, x);
    r = __fmaf_rn(n, -1.42860682030941723e-6f, r);
    float p = 1.0f / 5040.0f;
    p = __fmaf_rn(p, r, 1.0f / 720.0f);
    p = __fmaf_rn(p, r, 1.0f / 120.0f);
    p = __fmaf_rn(p, r, 1.0f / 24.0f);
    p = __fmaf_rn(p, r, 1.0f / 6.0f);
    p = __fmaf_rn(p, r, 0.5f);
    p = __fmaf_rn(p, r, 1.0f);
    p = __fmaf_rn(p, r, 1.0f);
    return ldexpf(p, (int)n);
}

// fp32 bits -> unsigned key whose integer order is the order of the floats
__device__ __forceinline__ uint32_t order_key(float z)
{
    uint32_t b = __float_as_uint(z);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// floor(w * 2^40) for a non-negative fp32 below 2^23, by shifting the significand (exact)
__device__ __forceinline__ uint64_t fixed40(float w)
{
    uint32_t b = __float_as_uint(w);
    if ((int32_t)b <= 0) return 0;              // zero, negative (sign bit) -> 0
    int e = (int)(b >> 23);
    if (e == 0) return 0;                       // subnormal: far below 2^-40
    uint64_t mant = (uint64_t)((b & 0x7FFFFFu) | 0x800000u);
    int sh = e - 110;                           // (e - 127) + 40 - 23
    if (sh >= 0) return mant << sh;
    if (sh > -24) return mant >> (-sh);
    return 0;
}

// ---------------------------------------------------------------------------------------------
// workgroup-wide helpers (DIST_THREADS threads)
// ---------------------------------------------------------------------------------------------
// Wave-wide scans and reductions without LDS traffic: a Hillis-Steele scan inside each row of 16
// lanes with DPP row shifts (a lane whose source falls outside its row receives the identity), then
// the four row totals are read from lanes 15/31/47/63 and folded in.
template <int N>
__device__ __forceinline__ uint32_t dpp_row_shr(uint32_t identity, uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)x, 0x110 + N, 0xf, 0xf, false);
}
__device__ __forceinline__ uint64_t readlane_u64(uint64_t v, int l)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l);
    return ((uint64_t)hi << 32) | lo;
}
// inclusive prefix sums over the 64 lanes; `total` is the wave's sum (the same in every lane)
__device__ __forceinline__ uint64_t wave_scan_u64(uint64_t v, uint64_t &total)
{
#define SJD_STEP(N)                                                              \
    {                                                                            \
        const uint32_t tl = dpp_row_shr<N>(0u, (uint32_t)v);                     \
        const uint32_t th = dpp_row_shr<N>(0u, (uint32_t)(v >> 32));             \
        v += ((uint64_t)th << 32) | tl;                                          \
    }
    SJD_STEP(1) SJD_STEP(2) SJD_STEP(4) SJD_STEP(8)
#undef SJD_STEP
    const uint64_t r0 = readlane_u64(v, 15), r1 = readlane_u64(v, 31), r2 = readlane_u64(v, 47), r3 = readlane_u64(v, 63);
    const int row = (threadIdx.x & 63) >> 4;
    total = r0 + r1 + r2 + r3;
    return v + (row == 0 ? 0 : row == 1 ? r0 : row == 2 ? r0 + r1 : r0 + r1 + r2);
}
__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v)
{
    uint64_t total;
    (void)wave_scan_u64(v, total);
    return total;
}
__device__ __forceinline__ int wave_scan_i32(int v, int &total)
{
    uint32_t x = (uint32_t)v;
    x += dpp_row_shr<1>(0u, x); x += dpp_row_shr<2>(0u, x); x += dpp_row_shr<4>(0u, x); x += dpp_row_shr<8>(0u, x);
    const int r0 = __builtin_amdgcn_readlane((int)x, 15), r1 = __builtin_amdgcn_readlane((int)x, 31);
    const int r2 = __builtin_amdgcn_readlane((int)x, 47), r3 = __builtin_amdgcn_readlane((int)x, 63);
    const int row = (threadIdx.x & 63) >> 4;
    total = r0 + r1 + r2 + r3;
    return (int)x + (row == 0 ? 0 : row == 1 ? r0 : row == 2 ? r0 + r1 : r0 + r1 + r2);
}
__device__ __forceinline__ int wave_sum_i32(int v)
{
    int total;
    (void)wave_scan_i32(v, total);
    return total;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
#define SJD_STEP(N) { const uint32_t t = dpp_row_shr<N>(0u, v); v = t > v ? t : v; }
    SJD_STEP(1) SJD_STEP(2) SJD_STEP(4) SJD_STEP(8)
#undef SJD_STEP
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 15), r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 31);
    const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 47), r3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
    const uint32_t a = r0 > r1 ? r0 : r1, b2 = r2 > r3 ? r2 : r3;
    return a > b2 ? a : b2;
}
__device__ __forceinline__ int wave_min_i32(int v)
{
#define SJD_STEP(N) { const int t = (int)dpp_row_shr<N>(0x7FFFFFFFu, (uint32_t)v); v = t < v ? t : v; }
    SJD_STEP(1) SJD_STEP(2) SJD_STEP(4) SJD_STEP(8)
#undef SJD_STEP
    const int r0 = __builtin_amdgcn_readlane(v, 15), r1 = __builtin_amdgcn_readlane(v, 31);
    const int r2 = __builtin_amdgcn_readlane(v, 47), r3 = __builtin_amdgcn_readlane(v, 63);
    return min(min(r0, r1), min(r2, r3));
}

template <int NWV>                   // NWV = waves per workgroup
struct DistSharedT {
    uint64_t wave_tot[NWV];
    uint64_t wave_tot2[NWV];         // second draw of block_sample2
    int result2;
    uint32_t wave_u32[NWV];
    int hist[256];
    int whist[NWV][256];          // per-wave digit counts (keeps same-bin LDS atomics inside one wave)
    uint32_t sel_prefix[2];       // result of a radix pass, double-buffered by pass parity
    int sel_rank[2];
    int top4[NWV][2];             // per-wave counts of the four highest top bytes (two 16-bit fields each)
    int ncand;                    // keys sharing the 16 resolved bits, and the low halves of the first 64
    uint32_t cand[64];
    int result;
};
typedef DistSharedT<DIST_WAVES> DistShared;


// Categorical draw from non-negative weights by inverse CDF over 40-bit fixed-point values taken
// in index order: tau = floor(k32 * C / 2^32), result = first index whose inclusive prefix sum
// exceeds tau.  Wave w owns the contiguous index range [w*span, (w+1)*span), span = 64 * ceil(V/1024);
// inside it lane l owns the indices w*span + 64 j + l, j < EPT (EPT >= ceil(V/1024) at compile time, so
// that per-thread values can live in registers).  The weight of index t, the j-th of its thread, is
// weight(j, t).  Returns -1 when C == 0.  All threads get the result.
template <int EPT, class WeightFn>
__device__ int block_sample(WeightFn weight, int V, uint32_t k32, DistShared *sh)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int span = ((V + DIST_WAVES * 64 - 1) / (DIST_WAVES * 64)) * 64;  // multiple of 64
    const int beg = wave * span;
    const int end = min(V, beg + span);
    uint64_t cj[EPT];
    uint64_t local = 0;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int t = beg + j * 64 + lane;
        cj[j] = t < end ? fixed40(weight(j, t)) : 0;
        local += cj[j];
    }
    local = wave_sum_u64(local);
    __syncthreads();                       // protects sh->wave_tot / result from the previous use
    if (lane == 0) sh->wave_tot[wave] = local;
    if (threadIdx.x == 0) sh->result = -1;
    __syncthreads();
    uint64_t C = 0, mine = 0;
    for (int w = 0; w < DIST_WAVES; ++w) { if (w == wave) mine = C; C += sh->wave_tot[w]; }
    if (C != 0) {
        uint64_t tau = __umul64hi((uint64_t)k32 << 32, C);    // (k32 * C) >> 32
        if (tau >= mine && tau < mine + local) {               // exactly one wave
            uint64_t base = mine;
            bool found = false;
#pragma unroll
            for (int j = 0; j < EPT; ++j) {
                if (!found && beg + j * 64 < end) {
                    uint64_t group_total;
                    const uint64_t incl = wave_scan_u64(cj[j], group_total);
                    unsigned long long hit = __ballot(base + incl > tau);
                    if (hit) {
                        if (lane == 0) sh->result = beg + j * 64 + __ffsll(hit) - 1;
                        found = true;
                    }
                    base += group_total;
                }
            }
        }
    }
    __syncthreads();
    return sh->result;
}

// Two draws at once from two weight functions over the same index range (one pass over the row, one
// pair of barriers): results as block_sample would give them for (w1, k1) and (w2, k2).
template <int EPT, class W1, class W2>
__device__ void block_sample2(W1 w1, W2 w2, int V, uint32_t k1, uint32_t k2, DistShared *sh, int &r1, int &r2)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int span = ((V + DIST_WAVES * 64 - 1) / (DIST_WAVES * 64)) * 64;
    const int beg = wave * span;
    const int end = min(V, beg + span);
    uint64_t c1[EPT], c2[EPT];
    uint64_t loc1 = 0, loc2 = 0;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int t = beg + j * 64 + lane;
        c1[j] = t < end ? fixed40(w1(j, t)) : 0;
        c2[j] = t < end ? fixed40(w2(j, t)) : 0;
        loc1 += c1[j];
        loc2 += c2[j];
    }
    loc1 = wave_sum_u64(loc1);
    loc2 = wave_sum_u64(loc2);
    __syncthreads();                       // protects the shared fields from the previous use
    if (lane == 0) { sh->wave_tot[wave] = loc1; sh->wave_tot2[wave] = loc2; }
    if (threadIdx.x == 0) { sh->result = -1; sh->result2 = -1; }
    __syncthreads();
    uint64_t C1 = 0, C2 = 0, mine1 = 0, mine2 = 0;
    for (int w = 0; w < DIST_WAVES; ++w) {
        if (w == wave) { mine1 = C1; mine2 = C2; }
        C1 += sh->wave_tot[w];
        C2 += sh->wave_tot2[w];
    }
    auto find = [&](const uint64_t (&cj)[EPT], uint64_t C, uint64_t mine, uint64_t local, uint32_t k32, int *out) {
        if (C == 0) return;
        const uint64_t tau = __umul64hi((uint64_t)k32 << 32, C);    // (k32 * C) >> 32
        if (tau >= mine && tau < mine + local) {                   // exactly one wave
            uint64_t base = mine;
            bool found = false;
#pragma unroll
            for (int j = 0; j < EPT; ++j) {
                if (!found && beg + j * 64 < end) {
                    uint64_t group_total;
                    const uint64_t incl = wave_scan_u64(cj[j], group_total);
                    unsigned long long hit = __ballot(base + incl > tau);
                    if (hit) {
                        if (lane == 0) *out = beg + j * 64 + __ffsll(hit) - 1;
                        found = true;
                    }
                    base += group_total;
                }
            }
        }
    };
    find(c1, C1, mine1, loc1, k1, &sh->result);
    find(c2, C2, mine2, loc2, k2, &sh->result2);
    __syncthreads();
    r1 = sh->result;
    r2 = sh->result2;
}

// The sampling distribution of one logits row, left in `buf` (LDS, V floats) and returned to the
// caller for writing.  Steps: (1) forced -> one-hot; (2) keep exactly K entries by (value
// descending, index ascending); (3) e = exp((z - max)/T), Z = sum of e in fixed point,
// q = e / Z; (4) K == 1 or T == 0 -> one-hot at the arg-max, lowest index on ties.
// Classifier-free guidance (the paper's Sec. 5.1 names the weight, not the mechanism; the usual
// logit-space form is used): z = z_u + w * (z_c - z_u), three separately rounded fp32 operations.
__device__ __forceinline__ float guide(float zc, float zu, float w) { return __fadd_rn(zu, __fmul_rn(w, __fsub_rn(zc, zu))); }

// NT threads per workgroup: 1024 for the rows of a decoding iteration (shortest time per row); fewer where
// many independent rows run at once (more rows per CU in flight).  Results do not depend on NT: every sum that
// decides anything is an integer.
template <int EPT, int NT = DIST_THREADS>
__device__ void block_dist(const float *__restrict__ z, const float *__restrict__ z_u, float cfg_scale, int V, int top_k,
                           float T, int forced, uint32_t *buf, DistSharedT<NT / 64> *sh)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float *qb = reinterpret_cast<float *>(buf);
    if (forced >= 0) {
        for (int t = tid; t < V; t += NT) qb[t] = (t == forced) ? 1.0f : 0.0f;
        __syncthreads();
        return;
    }
    // keys into LDS, block max (all loads of a thread are issued before any is used)
    uint32_t kmax = 0;
    float zr[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int t = tid + j * NT;
        zr[j] = t < V ? z[t] : 0.0f;
    }
    if (z_u) {
        float zu[EPT];
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const int t = tid + j * NT;
            zu[j] = t < V ? z_u[t] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < EPT; ++j) zr[j] = guide(zr[j], zu[j], cfg_scale);
    }
    // every thread keeps the keys of its own elements (t = tid + j * NT) in registers; the
    // copy in LDS serves the steps that walk the row in a different order
    uint32_t kr[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int t = tid + j * NT;
        kr[j] = 0;
        if (t < V) {
            uint32_t k = order_key(zr[j]);
            kr[j] = k;
            buf[t] = k;
            kmax = k > kmax ? k : kmax;
        }
    }
    kmax = wave_max_u32(kmax);
    if (lane == 0) sh->wave_u32[wave] = kmax;
    if (tid == 0) sh->ncand = 0;
    __syncthreads();
    kmax = 0;
    for (int w = 0; w < (NT / 64); ++w) kmax = sh->wave_u32[w] > kmax ? sh->wave_u32[w] : kmax;

    if (top_k == 1 || T == 0.0f) {
        // lowest index holding the maximum
        int best = 0x7FFFFFFF;
        for (int t = tid; t < V; t += NT) if (buf[t] == kmax) best = min(best, t);
        best = wave_min_i32(best);
        __syncthreads();
        if (lane == 0) sh->hist[wave] = best;
        __syncthreads();
        best = 0x7FFFFFFF;
        for (int w = 0; w < (NT / 64); ++w) best = min(best, sh->hist[w]);
        __syncthreads();
        for (int t = tid; t < V; t += NT) qb[t] = (t == best) ? 1.0f : 0.0f;
        __syncthreads();
        return;
    }

    // ---- radix select of the K-th largest key: 4 passes of 8 bits, most significant first ----
    uint32_t kth = 0;
    int room = 0x7FFFFFFF;     // how many entries equal to kth survive
    bool cut = top_k < V;
    if (cut) {
        uint32_t prefix = 0, mask = 0;
        int rank = top_k;      // we look for the rank-th largest among keys matching the prefix
        int first_shift = 24;
        {
            // Top byte (sign and high exponent bits): the keys crowd into the few highest values that
            // occur, which is the worst case for a histogram in LDS (every lane on the same counter) and
            // the best for counting in registers: the four highest top bytes, four 8-bit counters per
            // thread (at most EPT <= 32 each), widened to 16-bit fields for the sums (at most V <= 32768).
            const uint32_t dmax = kmax >> 24;
            uint32_t cnt = 0;
#pragma unroll
            for (int j = 0; j < EPT; ++j) {
                const int t = tid + j * NT;
                if (t < V) {
                    const uint32_t diff = dmax - (kr[j] >> 24);
                    if (diff < 4u) cnt += 1u << (8 * diff);
                }
            }
            int lo = (int)((cnt & 0xFFu) | ((cnt & 0xFF00u) << 8));               // counts of dmax, dmax - 1
            int hi = (int)(((cnt >> 16) & 0xFFu) | ((cnt >> 24) << 16));         // counts of dmax - 2, dmax - 3
            lo = wave_sum_i32(lo);
            hi = wave_sum_i32(hi);
            if (lane == 0) { sh->top4[wave][0] = lo; sh->top4[wave][1] = hi; }
            __syncthreads();
            lo = 0; hi = 0;
            for (int w = 0; w < (NT / 64); ++w) { lo += sh->top4[w][0]; hi += sh->top4[w][1]; }
            const int c0 = lo & 0xFFFF, c1 = (lo >> 16) & 0xFFFF, c2 = hi & 0xFFFF, c3 = (hi >> 16) & 0xFFFF;
            int digit = -1, before = 0;
            if (rank <= c0) { digit = (int)dmax; }
            else if (rank <= c0 + c1) { digit = (int)dmax - 1; before = c0; }
            else if (rank <= c0 + c1 + c2) { digit = (int)dmax - 2; before = c0 + c1; }
            else if (rank <= c0 + c1 + c2 + c3) { digit = (int)dmax - 3; before = c0 + c1 + c2; }
            if (digit >= 0) {          // (the same decision in every thread)
                prefix = (uint32_t)digit << 24;
                rank -= before;
                mask = 255u << 24;
                first_shift = 16;
            }
        }
        for (int shift = first_shift; shift >= 0; shift -= 8) {
            const int par = (shift >> 3) & 1;
            if (shift == 8) {
                // 16 bits are resolved: the keys that share them are few (a sliver of the value range).
                // Up to 64 of them are finished by one wave, each lane ranking its key against the rest.
#pragma unroll
                for (int j = 0; j < EPT; ++j) {
                    const uint32_t k = kr[j];
                    if (tid + j * NT < V && (k & mask) == prefix) {
                        const int pos = atomicAdd(&sh->ncand, 1);
                        if (pos < 64) sh->cand[pos] = k & 0xFFFFu;
                    }
                }
                __syncthreads();
                const int n = sh->ncand;
                if (n <= 64) {
                    if (wave == 0) {
                        const uint32_t mine = lane < n ? sh->cand[lane] : 0u;
                        int gt = 0, ge = 0;
                        for (int i = 0; i < n; ++i) {
                            const uint32_t other = (uint32_t)__builtin_amdgcn_readlane((int)mine, i);
                            gt += other > mine;
                            ge += other >= mine;
                        }
                        if (lane < n && gt < rank && rank <= ge) {       // every lane holding that value agrees
                            sh->sel_prefix[par] = prefix | mine;
                            sh->sel_rank[par] = rank - gt;
                        }
                    }
                    __syncthreads();
                    prefix = sh->sel_prefix[par];
                    rank = sh->sel_rank[par];
                    mask = 0xFFFFFFFFu;
                    break;
                }
            }
            // a wave clears and fills its own histogram: no workgroup barrier in between (the readers of
            // the previous pass are behind that pass's barriers)
            for (int b = lane; b < 256; b += 64) sh->whist[wave][b] = 0;
#pragma unroll
            for (int j = 0; j < EPT; ++j) {
                const uint32_t k = kr[j];
                if (tid + j * NT < V && (k & mask) == prefix) atomicAdd(&sh->whist[wave][(k >> shift) & 255u], 1);
            }
            __syncthreads();
            if (tid < 256) {
                int c = 0;
#pragma unroll
                for (int w = 0; w < (NT / 64); ++w) c += sh->whist[w][tid];
                sh->hist[tid] = c;
            }
            __syncthreads();
            if (wave == 0) {
                // lane l covers digits 255-4l .. 252-4l (descending)
                int d0 = 255 - 4 * lane;
                int h0 = sh->hist[d0], h1 = sh->hist[d0 - 1], h2 = sh->hist[d0 - 2], h3 = sh->hist[d0 - 3];
                int tot = h0 + h1 + h2 + h3, all_;
                const int incl = wave_scan_i32(tot, all_);
                int excl = incl - tot;
                if (excl < rank && rank <= incl) {           // exactly one lane
                    int digit, before;
                    if (rank <= excl + h0) { digit = d0; before = excl; }
                    else if (rank <= excl + h0 + h1) { digit = d0 - 1; before = excl + h0; }
                    else if (rank <= excl + h0 + h1 + h2) { digit = d0 - 2; before = excl + h0 + h1; }
                    else { digit = d0 - 3; before = excl + h0 + h1 + h2; }
                    sh->sel_prefix[par] = prefix | ((uint32_t)digit << shift);
                    sh->sel_rank[par] = rank - before;
                }
            }
            __syncthreads();
            prefix = sh->sel_prefix[par];
            rank = sh->sel_rank[par];
            mask |= 255u << shift;
        }
        kth = prefix;
        room = rank;           // = K - #(keys > kth)
        // entries equal to kth: do they all fit?
        int eq = 0;
#pragma unroll
        for (int j = 0; j < EPT; ++j) eq += (tid + j * NT < V) && kr[j] == kth;
        eq = wave_sum_i32(eq);
        if (lane == 0) sh->hist[wave] = eq;
        __syncthreads();
        eq = 0;
        for (int w = 0; w < (NT / 64); ++w) eq += sh->hist[w];
        __syncthreads();
        if (eq > room) {
            // ties cut the K-th value: keep the `room` lowest indices.  Wave w scans its contiguous
            // index range; a tie that loses gets its key lowered to kth - 1 so that the test
            // `key >= kth` below drops it (kth == 0 only arises from NaN logits, which are
            // outside the contract).
            const int span = ((V + (NT / 64) * 64 - 1) / ((NT / 64) * 64)) * 64;
            const int beg = wave * span, end = min(V, beg + span);
            int cnt = 0;
            for (int t = beg + lane; t < end; t += 64) cnt += buf[t] == kth;
            cnt = wave_sum_i32(cnt);
            if (lane == 0) sh->hist[wave] = cnt;
            __syncthreads();
            int base = 0;
            for (int w = 0; w < wave; ++w) base += sh->hist[w];
            for (int g = beg; g < end; g += 64) {
                int t = g + lane;
                int f = (t < end && buf[t] == kth) ? 1 : 0;
                int group_total;
                const int incl = wave_scan_i32(f, group_total);
                if (f && base + incl > room && kth > 0) buf[t] = kth - 1;
                base += group_total;
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < EPT; ++j) {           // the keys of lost ties changed: take them again
                const int t = tid + j * NT;
                if (t < V) kr[j] = buf[t];
            }
        }
    }

    // ---- softmax over the survivors ----------------------------------------------------------
    const float m = key_to_float(kmax);
    uint64_t csum = 0;
    float er[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const uint32_t k = kr[j];
        const bool keep = tid + j * NT < V && (!cut || k >= kth);
        float e = 0.0f;
        if (keep) {
            float x = __fdiv_rn(__fsub_rn(key_to_float(k), m), T);   // the key still holds the logit's bits
            e = exp_fixed(x);
        }
        er[j] = e;
        csum += fixed40(e);
    }
    csum = wave_sum_u64(csum);
    if (lane == 0) sh->wave_tot[wave] = csum;
    __syncthreads();
    uint64_t C = 0;
    for (int w = 0; w < (NT / 64); ++w) C += sh->wave_tot[w];
    const float Z = __fmul_rn(__ull2float_rn(C), 0x1p-40f);
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int t = tid + j * NT;
        if (t < V) qb[t] = (er[j] != 0.0f) ? __fdiv_rn(er[j], Z) : 0.0f;     // (over the keys: same storage)
    }
    __syncthreads();
}

__device__ __forceinline__ int forced_index(const sjd_init &init, int img_pos, int lo)
{
    if (init.eol_id >= 0 && init.row_stride > 0 && (img_pos + 1) % init.row_stride == 0) return init.eol_id - lo;
    return -1;
}

// ---------------------------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------------------------
struct StepSnap {       // per-step scalars frozen by the rows kernel for the finalize kernel
    int32_t n, img_pos0, L_eff, active;
    uint64_t counter;
};

struct RowsArgs {
    const float *logits, *logits_u, *q_in, *p_old;
    float cfg_scale;
    const int32_t *draft;
    int32_t L, V, lo;
    sjd_sampler smp;
    sjd_init init;
    uint64_t seed;
    const SjdState *state;
    int32_t img_pos0;
    uint64_t counter;
    float *q;
    int32_t *tok_smp, *tok_res, *acc_flag, *draft_snap;
    StepSnap *snap;
};

template <int EPT>
__device__ __forceinline__ void rows_body(const RowsArgs &a)
{
    extern __shared__ uint32_t buf[];
    __shared__ DistShared sh;
    const int i = blockIdx.x + 1;          // window index 1..L
    int img_pos0 = a.img_pos0, L = a.L, n = 0, active = 1;
    uint64_t counter = a.counter;
    if (a.state) {
        img_pos0 = a.state->img_pos0; L = a.state->L_eff; counter = a.state->counter; n = a.state->n;
        active = !a.state->done;
    }
    if (blockIdx.x == 0) {
        if (threadIdx.x == 0) {
            a.snap->n = n; a.snap->img_pos0 = img_pos0; a.snap->L_eff = L; a.snap->counter = counter;
            a.snap->active = active;
        }
        for (int j = threadIdx.x; j < a.L; j += DIST_THREADS) a.draft_snap[j] = a.draft[j];
    }
    if (!active || i > L) return;
    const int V = a.V;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int span = ((V + DIST_WAVES * 64 - 1) / (DIST_WAVES * 64)) * 64;
    const int beg = wave * span, end = min(V, beg + span);
    // everything this workgroup needs from p_old is requested now and used after the distribution
    // is done: the thread's share of the row (in block_sample's index order) and, in thread 0, the
    // entry of the draft token for the accept test
    const float *po = a.p_old + (size_t)(i < L ? i : 0) * V;
    float por[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int t = beg + j * 64 + lane;
        por[j] = (i < L && t < end) ? po[t] : 0.0f;
    }
    int x_draft = -1;
    float po_x = 0.0f;
    if (threadIdx.x == 0 && i < L) {
        x_draft = a.draft[i] - a.lo;
        if (x_draft >= 0 && x_draft < V) po_x = po[x_draft];
    }

    float *qrow = a.q + (size_t)i * V;
    float *qb = reinterpret_cast<float *>(buf);
    if (a.q_in) {
        const float *src = a.q_in + (size_t)i * V;
        float tmp[EPT];
#pragma unroll
        for (int j = 0; j < EPT; ++j) { const int t = threadIdx.x + j * DIST_THREADS; tmp[j] = t < V ? src[t] : 0.0f; }
#pragma unroll
        for (int j = 0; j < EPT; ++j) { const int t = threadIdx.x + j * DIST_THREADS; if (t < V) qb[t] = tmp[j]; }
        __syncthreads();
    } else {
        block_dist<EPT>(a.logits + (size_t)(i - 1) * V, a.logits_u ? a.logits_u + (size_t)(i - 1) * V : nullptr, a.cfg_scale,
                        V, a.smp.top_k, a.smp.temperature, forced_index(a.init, img_pos0 + i, a.lo), buf, &sh);
    }
    for (int t = threadIdx.x; t < V; t += DIST_THREADS) qrow[t] = qb[t];

    const U4 rnd = philox_draw(a.seed, counter, (uint32_t)i);
    // candidate for Eq. 3 (and for the bonus index L): a plain sample from q_i; candidate for Eq. 2: a
    // sample from max(0, q_i - p_old_i), or, if that vanishes, from q_i with the same random word
    int s, rs = -1;
    auto w_q = [&](int, int t) { return qb[t]; };
    auto w_res = [&](int j, int t) { float d = __fsub_rn(qb[t], por[j]); return d > 0.0f ? d : 0.0f; };
    if constexpr (EPT <= 8) {            // both draws in one pass where their fixed-point values fit the registers
        if (i < L) block_sample2<EPT>(w_q, w_res, V, rnd.w[2], rnd.w[1], &sh, s, rs);
        else s = block_sample<EPT>(w_q, V, rnd.w[2], &sh);
    } else {
        s = block_sample<EPT>(w_q, V, rnd.w[2], &sh);
        if (i < L) rs = block_sample<EPT>(w_res, V, rnd.w[1], &sh);
    }
    if (threadIdx.x == 0) a.tok_smp[i] = s;
    if (i < L) {
        if (threadIdx.x == 0) {
            // Eq. 1: accept iff r < min(1, q_i(x_i) / p_old_i(x_i)); a NaN ratio rejects
            int ok = 0;
            if (x_draft >= 0 && x_draft < V) {
                float ratio = __fdiv_rn(qb[x_draft], po_x);
                float r = u_from_word(rnd.w[0]);
                ok = (ratio >= 1.0f) || (r < ratio);
            }
            a.acc_flag[i] = ok;
        }
        if (rs < 0) rs = block_sample<EPT>([&](int, int t) { return qb[t]; }, V, rnd.w[1], &sh);
        if (threadIdx.x == 0) a.tok_res[i] = rs;
    }
}

template <int EPT>
__global__ __launch_bounds__(DIST_THREADS) void sjd_rows_kernel(RowsArgs a) { rows_body<EPT>(a); }

// The images of a batch verified side by side: blockIdx.y picks the image's arguments.
template <class Args>
struct ArgsBatch { Args a[SJD_MAX_STREAMS]; };
template <int EPT>
__global__ __launch_bounds__(DIST_THREADS) void sjd_rows_batch_kernel(ArgsBatch<RowsArgs> ab) { rows_body<EPT>(ab.a[blockIdx.y]); }

struct FinalArgs {
    int32_t L, V, lo;
    sjd_init init;
    uint64_t seed;
    const int32_t *hist;          // image-position-indexed ids, or NULL
    SjdState *state;              // advanced by workgroup 0 when non-NULL
    int32_t *kv_tokens;           // cache-position-indexed ids (with state), or NULL
    const float *q;
    const float *p_old;           // row 0 = the distribution index 0 carried (may alias p_new)
    float *ring;                  // initialiser (d): [row_stride][V] distributions of accepted positions
    const int32_t *tok_smp, *tok_res, *acc_flag, *draft_snap;
    const StepSnap *snap;
    int32_t *n_accepted, *new_draft;
    float *p_new;
};

#define FIN_PARTS 8     // workgroups sharing the copy of one distribution row
__device__ __forceinline__ void finalize_body(const FinalArgs &a)
{
    const StepSnap sn = *a.snap;
    if (!sn.active) return;
    const int L = sn.L_eff, V = a.V, lo = a.lo;
    const int j = blockIdx.x, part = blockIdx.y;
    // this workgroup's slice of row j
    const int per = (V + FIN_PARTS - 1) / FIN_PARTS;
    const int t_beg = part * per, t_end = min(V, t_beg + per);
    // Eq. 1 scan: index 0 is exact by construction; stop at the first rejection.  Every wave loads
    // all flags at once (lane i holds flag i) and counts the leading run of accepts.
    const int lane_ = threadIdx.x & 63;
    const int flag_ = lane_ == 0 ? 1 : (lane_ < L ? a.acc_flag[lane_] : 0);
    const unsigned long long run_ = __ballot(flag_ != 0);
    const int acc = ~run_ ? __ffsll((long long)~run_) - 1 : 64;     // (a window of 64 accepted whole leaves no zero bit)
    const int n_model = (a.init.flags & SJD_INIT_NO_REFINE) ? 1 : L - acc + 1;
    const int n_hist = sn.img_pos0 + acc;
    const int back = a.init.mode == 1 ? a.init.row_stride : a.init.mode == 2 ? 1 : 0;   // repeat-above / -left
    const int32_t *hist = a.hist;
    if (a.kv_tokens) hist = a.kv_tokens + (sn.n - sn.img_pos0);

    // initialiser (d): put the distribution of accepted index j on record (entry position % row_stride;
    // of several accepted positions sharing an entry the last one writes).  Index 0 records the row it
    // carried, read here before the next window's row 0 may overwrite it (p_new may be p_old).
    if (a.init.mode == 4 && j < acc && j + a.init.row_stride >= acc) {
        const float *src = j == 0 ? a.p_old : a.q + (size_t)j * V;
        float *dst = a.ring + (size_t)((sn.img_pos0 + j) % a.init.row_stride) * V;
        for (int t = t_beg + threadIdx.x; t < t_end; t += 256) dst[t] = src[t];
        __syncthreads();
    }

    if (j < L) {
        auto model_tok = [&](int slot) {   // token of next-window slot < n_model (local index)
            int src = acc + slot;
            if (slot == 0) return acc < L ? a.tok_res[acc] : a.tok_smp[L];
            return a.tok_smp[src];
        };
        if (j < n_model) {
            if (threadIdx.x == 0 && part == 0) a.new_draft[j] = model_tok(j) + lo;
            const float *src = a.q + (size_t)(acc + j) * V;
            float *dst = a.p_new + (size_t)j * V;
            for (int t0 = t_beg + threadIdx.x; t0 < t_end; t0 += 8 * 256) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) { const int t = t0 + u * 256; v[u] = t < t_end ? src[t] : 0.0f; }
#pragma unroll
                for (int u = 0; u < 8; ++u) { const int t = t0 + u * 256; if (t < t_end) dst[t] = v[u]; }
            }
        } else {
            // Sec. 4.2 initialisation of image position n_hist + j
            int pos = n_hist + j;
            bool onehot = forced_index(a.init, pos, lo) >= 0 || (back > 0 && pos - back >= 0);
            int tok;
            for (;;) {
                int f = forced_index(a.init, pos, lo);
                if (f >= 0) { tok = f; break; }
                if (back > 0 && pos - back >= 0) {
                    pos -= back;
                    if (pos < sn.img_pos0) { tok = hist[pos] - lo; break; }
                    if (pos < n_hist) { tok = a.draft_snap[pos - sn.img_pos0] - lo; break; }
                    int slot = pos - n_hist;
                    if (slot < n_model) { tok = model_tok(slot); break; }
                    continue;      // the slot above is itself newly initialised: resolve it
                }
                U4 rnd = philox_draw(a.seed, sn.counter, (uint32_t)(L + 1 + (pos - n_hist - n_model)));
                tok = (int)(((uint64_t)rnd.w[3] * (uint64_t)V) >> 32);
                break;
            }
            if (threadIdx.x == 0 && part == 0) a.new_draft[j] = tok + lo;
            float *dst = a.p_new + (size_t)j * V;
            const float u = __fdiv_rn(1.0f, (float)V);
            for (int t = t_beg + threadIdx.x; t < t_end; t += 256) dst[t] = onehot ? (t == tok ? 1.0f : 0.0f) : u;
        }
    }
    if (j == 0 && part == 0 && threadIdx.x == 0) {
        if (a.n_accepted) a.n_accepted[0] = acc;
        if (a.state) {
            SjdState *st = a.state;
            if (a.kv_tokens) for (int i = 0; i < acc; ++i) a.kv_tokens[sn.n + i] = a.draft_snap[i];
            st->n = sn.n + acc;
            st->n_u += acc;              // the unconditional stream (if any) takes the same tokens
            st->img_pos0 = sn.img_pos0 + acc;
            st->counter = sn.counter + 1;
            st->steps += 1;
            st->accept_hist[acc < 64 ? acc : 64] += 1;
            if (st->n_image > 0) {
                int left = st->n_image - st->img_pos0;
                st->L_eff = left < a.L ? left : a.L;
                if (st->img_pos0 >= st->n_image - 1) st->done = 1;
            }
        }
    }
}

__global__ __launch_bounds__(256) void sjd_finalize_kernel(FinalArgs a) { finalize_body(a); }
__global__ __launch_bounds__(256) void sjd_finalize_batch_kernel(ArgsBatch<FinalArgs> ab) { finalize_body(ab.a[blockIdx.z]); }

// Initialisers (c) and (d) of Sec. 4.2, run after the finalize kernel (which has given every new slot
// the uniform initialisation): a new slot that finds a recorded distribution becomes a fresh draw from
// it and carries that row.
//   (c) the nearest slot to the left in the next window that is neither a forced row end nor itself
//       new (a run of new slots all draw from the last model row, each with its own random word);
//   (d) the position one grid row up: accepted (before or in this iteration) -> ring[pos % row_stride],
//       which the finalize kernel has brought up to date; in the next window -> that slot's row, or,
//       if that slot is new as well, whatever it resolves to.
// No source (first grid row, only forced slots to the left) leaves the uniform initialisation.
struct TailArgs {
    int32_t V, lo;
    sjd_init init;
    uint64_t seed;
    const float *q;
    const float *ring;
    const int32_t *acc_flag;
    const StepSnap *snap;
    int32_t *new_draft;
    float *p_new;
};

template <int EPT>
__device__ __forceinline__ void tail_body(const TailArgs &a)
{
    __shared__ DistShared sh;
    const StepSnap sn = *a.snap;
    if (!sn.active) return;
    const int L = sn.L_eff, V = a.V, lo = a.lo, j = blockIdx.x;
    if (j >= L) return;
    const int lane_ = threadIdx.x & 63;
    const int flag_ = lane_ == 0 ? 1 : (lane_ < L ? a.acc_flag[lane_] : 0);
    const unsigned long long run_ = __ballot(flag_ != 0);
    const int acc = ~run_ ? __ffsll((long long)~run_) - 1 : 64;     // (a window of 64 accepted whole leaves no zero bit)
    const int n_model = (a.init.flags & SJD_INIT_NO_REFINE) ? 1 : L - acc + 1;
    const int n_hist = sn.img_pos0 + acc;
    const int stride = a.init.row_stride;
    if (j < n_model) return;
    const int pos = n_hist + j;
    if (forced_index(a.init, pos, lo) >= 0) return;
    const float *src = nullptr;
    if (a.init.mode == 3) {
        for (int p = pos - 1; p >= n_hist; --p) {
            if (forced_index(a.init, p, lo) >= 0) continue;
            const int slot = p - n_hist;
            if (slot < n_model) { src = a.q + (size_t)(acc + slot) * V; break; }
        }
    } else {
        for (int p = pos - stride; p >= 0; p -= stride) {
            if (p < n_hist) { src = a.ring + (size_t)(p % stride) * V; break; }
            const int slot = p - n_hist;
            if (slot < n_model) { src = a.q + (size_t)(acc + slot) * V; break; }
        }
    }
    if (!src) return;
    const U4 rnd = philox_draw(a.seed, sn.counter, (uint32_t)(L + 1 + (j - n_model)));
    const int tok = block_sample<EPT>([&](int, int t) { return src[t]; }, V, rnd.w[3], &sh);
    if (tok < 0) return;
    if (threadIdx.x == 0) a.new_draft[j] = tok + lo;
    float *dst = a.p_new + (size_t)j * V;
    for (int t = threadIdx.x; t < V; t += DIST_THREADS) dst[t] = src[t];
}

template <int EPT>
__global__ __launch_bounds__(DIST_THREADS) void sjd_tail_kernel(TailArgs a) { tail_body<EPT>(a); }
template <int EPT>
__global__ __launch_bounds__(DIST_THREADS) void sjd_tail_batch_kernel(ArgsBatch<TailArgs> ab) { tail_body<EPT>(ab.a[blockIdx.y]); }

template <int EPT, int NT = DIST_THREADS>
__global__ __launch_bounds__(NT) void sjd_dist_kernel(const float *logits, const float *logits_u, float cfg_scale,
                                                      int V, sjd_sampler smp, const int32_t *forced, float *q)
{
    extern __shared__ uint32_t buf[];
    __shared__ DistSharedT<NT / 64> sh;
    const int row = blockIdx.x;
    block_dist<EPT, NT>(logits + (size_t)row * V, logits_u ? logits_u + (size_t)row * V : nullptr, cfg_scale, V, smp.top_k,
                        smp.temperature, forced ? forced[row] : -1, buf, &sh);
    const float *qb = reinterpret_cast<const float *>(buf);
    for (int t = threadIdx.x; t < V; t += NT) q[(size_t)row * V + t] = qb[t];
}

// First window (step counter 0): slot 0 ~ q_first, slots 1..L-1 by the init strategy.
template <int EPT>
__global__ __launch_bounds__(DIST_THREADS) void sjd_first_window_kernel(const float *q_first, int L, int V, int lo,
                                                                        sjd_init init, uint64_t seed,
                                                                        int32_t *draft, float *p_old)
{
    extern __shared__ uint32_t buf[];
    __shared__ DistShared sh;
    __shared__ int tok0;
    const int j = blockIdx.x;
    if (j > 0 && (init.mode == 3 || init.mode == 4) && forced_index(init, j, lo) < 0) {
        // sampled initialisers: the only recorded distribution in the first window is slot 0's
        // (every other slot is new and looked through): (c) reaches it unless it is a forced row end,
        // (d) when the chain of positions above ends at 0
        const bool from_first = init.mode == 3 ? forced_index(init, 0, lo) < 0
                                               : (init.row_stride > 0 && j % init.row_stride == 0);
        if (from_first) {
            const U4 rnd = philox_draw(seed, 0, (uint32_t)j);
            const int tok = block_sample<EPT>([&](int, int t) { return q_first[t]; }, V, rnd.w[3], &sh);
            if (tok >= 0) {
                if (threadIdx.x == 0) draft[j] = tok + lo;
                float *dst = p_old + (size_t)j * V;
                for (int t = threadIdx.x; t < V; t += DIST_THREADS) dst[t] = q_first[t];
                return;
            }
        }
    }
    if (j == 0 || init.mode == 1 || init.mode == 2) {
        // slot 0's token (every workgroup that may copy from it recomputes it: same inputs, same bits)
        float *qb = reinterpret_cast<float *>(buf);
        for (int t = threadIdx.x; t < V; t += DIST_THREADS) qb[t] = q_first[t];
        __syncthreads();
        U4 rnd = philox_draw(seed, 0, 0);
        int s = block_sample<EPT>([&](int, int t) { return qb[t]; }, V, rnd.w[2], &sh);
        if (threadIdx.x == 0) tok0 = s;
        __syncthreads();
    }
    if (j == 0) {
        if (threadIdx.x == 0) draft[0] = tok0 + lo;
        for (int t = threadIdx.x; t < V; t += DIST_THREADS) p_old[t] = q_first[t];
        return;
    }
    int pos = j;
    const int back = init.mode == 1 ? init.row_stride : init.mode == 2 ? 1 : 0;
    bool onehot = forced_index(init, pos, lo) >= 0 || (back > 0 && pos - back >= 0);
    int tok;
    for (;;) {
        int f = forced_index(init, pos, lo);
        if (f >= 0) { tok = f; break; }
        if (back > 0 && pos - back >= 0) {
            pos -= back;
            if (pos == 0) { tok = tok0; break; }
            continue;
        }
        U4 rnd = philox_draw(seed, 0, (uint32_t)pos);
        tok = (int)(((uint64_t)rnd.w[3] * (uint64_t)V) >> 32);
        break;
    }
    if (threadIdx.x == 0) draft[j] = tok + lo;
    float *dst = p_old + (size_t)j * V;
    const float u = __fdiv_rn(1.0f, (float)V);
    for (int t = threadIdx.x; t < V; t += DIST_THREADS) dst[t] = onehot ? (t == tok ? 1.0f : 0.0f) : u;
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
// Dynamic LDS above the default limit has to be enabled per kernel.  The limit is only ever
// raised, and sjd_sample_setup() raises it when a cache is created, so that launches recorded
// during graph capture never need to touch function attributes.
// Elements per thread are a compile-time bound (per-thread values live in registers): 4, 8, 16 or 32
// for vocabularies up to 4096, 8192, 16384, 32768.
static int ept_class(int V) { const int e = (V + DIST_THREADS - 1) / DIST_THREADS; return e <= 4 ? 0 : e <= 8 ? 1 : e <= 16 ? 2 : 3; }
#define EPT_SWITCH(cls, STMT)                  \
    switch (cls) {                             \
        case 0: { constexpr int EPT = 4; STMT; } break;  \
        case 1: { constexpr int EPT = 8; STMT; } break;  \
        case 2: { constexpr int EPT = 16; STMT; } break; \
        default: { constexpr int EPT = 32; STMT; } break; \
    }
static size_t g_lds_set[4][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
static std::mutex g_lds_mutex;      // (handles may be created from several host threads)
static int ensure_lds(int which, int cls, size_t bytes)
{
    if (bytes <= 48 * 1024) return SJD_OK;
    std::lock_guard<std::mutex> lock(g_lds_mutex);
    if (bytes <= g_lds_set[which][cls]) return SJD_OK;
    const void *fn = nullptr;
    EPT_SWITCH(cls, fn = which == 0 ? (const void *)sjd_rows_kernel<EPT>
                       : which == 1 ? (const void *)sjd_dist_kernel<EPT>
                       : which == 2 ? (const void *)sjd_first_window_kernel<EPT> : (const void *)sjd_rows_batch_kernel<EPT>)
    HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    g_lds_set[which][cls] = bytes;
    return SJD_OK;
}

template <int NT> static int ensure_lds_many(size_t lds);
int sjd_sample_setup(int32_t V)
{
    const size_t lds = (size_t)V * 4;
    for (int which = 0; which < 4; ++which) SJD_TRY(ensure_lds(which, ept_class(V), lds));
    if (V > 256 * 32 && V <= 512 * 32) SJD_TRY(ensure_lds_many<512>(lds));      // (the many-rows variant of sjd_dist)
    return SJD_OK;
}

static void fill_verify_args(const SjdVerifyArgs *v, RowsArgs &r, FinalArgs &f, TailArgs &t)
{
    r.logits = v->logits; r.logits_u = v->logits_u; r.cfg_scale = v->cfg_scale; r.q_in = v->q_in; r.p_old = v->p_old;
    r.draft = v->draft;
    r.L = v->L; r.V = v->V; r.lo = v->lo; r.smp = v->smp; r.init = v->init; r.seed = v->seed;
    r.state = v->state; r.img_pos0 = v->img_pos0; r.counter = v->counter;
    r.q = v->q; r.tok_smp = v->tok_smp; r.tok_res = v->tok_res; r.acc_flag = v->acc_flag;
    r.draft_snap = v->draft_snap; r.snap = reinterpret_cast<StepSnap *>(v->snap);
    f.L = v->L; f.V = v->V; f.lo = v->lo; f.init = v->init; f.seed = v->seed; f.hist = v->hist;
    f.state = v->state; f.kv_tokens = v->kv_tokens; f.q = v->q; f.tok_smp = v->tok_smp; f.tok_res = v->tok_res;
    f.acc_flag = v->acc_flag; f.draft_snap = v->draft_snap; f.snap = reinterpret_cast<const StepSnap *>(v->snap);
    f.n_accepted = v->n_accepted; f.new_draft = v->new_draft; f.p_new = v->p_new;
    f.p_old = v->p_old; f.ring = v->ring;
    t.V = v->V; t.lo = v->lo; t.init = v->init; t.seed = v->seed; t.q = v->q; t.ring = v->ring;
    t.acc_flag = v->acc_flag; t.snap = reinterpret_cast<const StepSnap *>(v->snap); t.new_draft = v->new_draft;
    t.p_new = v->p_new;
}

int sjd_launch_verify(const SjdVerifyArgs *v, hipStream_t s)
{
    if (v->V < 1 || v->V > SJD_MAX_SAMP_VOCAB || v->L < 1 || v->L > SJD_MAX_WINDOW) return SJD_EINVAL;
    if (v->init.mode == 4 && (!v->ring || v->init.row_stride < 1)) return SJD_EINVAL;
    size_t lds = (size_t)v->V * 4;
    SJD_TRY(ensure_lds(0, ept_class(v->V), lds));
    RowsArgs r; FinalArgs f; TailArgs t;
    fill_verify_args(v, r, f, t);
    EPT_SWITCH(ept_class(v->V), SJD_LAUNCH(sjd_rows_kernel<EPT>, dim3(v->L), dim3(DIST_THREADS), lds, s, r))
    HIP_TRY(hipGetLastError());
    SJD_LAUNCH(sjd_finalize_kernel, dim3(v->L, FIN_PARTS), dim3(256), 0, s, f);
    HIP_TRY(hipGetLastError());
    if (v->init.mode == 3 || v->init.mode == 4) {
        EPT_SWITCH(ept_class(v->V), SJD_LAUNCH(sjd_tail_kernel<EPT>, dim3(v->L), dim3(DIST_THREADS), 0, s, t))
        HIP_TRY(hipGetLastError());
    }
    return SJD_OK;
}

// Steps 3-4 of B images in the same two or three launches (the images are independent: every workgroup works on
// one image's rows with that image's arguments).  All B share window size, vocabulary and initialiser mode.
int sjd_launch_verify_batch(const SjdVerifyArgs *v, int32_t B, hipStream_t s)
{
    if (B < 1 || B > SJD_MAX_STREAMS) return SJD_EINVAL;
    if (B == 1) return sjd_launch_verify(v, s);
    ArgsBatch<RowsArgs> rb; ArgsBatch<FinalArgs> fb; ArgsBatch<TailArgs> tb;
    std::memset(&rb, 0, sizeof(rb)); std::memset(&fb, 0, sizeof(fb)); std::memset(&tb, 0, sizeof(tb));
    for (int b = 0; b < B; ++b) {
        if (v[b].V != v[0].V || v[b].L != v[0].L || v[b].init.mode != v[0].init.mode) return SJD_EINVAL;
        if (v[b].V < 1 || v[b].V > SJD_MAX_SAMP_VOCAB || v[b].L < 1 || v[b].L > SJD_MAX_WINDOW) return SJD_EINVAL;
        if (v[b].init.mode == 4 && (!v[b].ring || v[b].init.row_stride < 1)) return SJD_EINVAL;
        fill_verify_args(&v[b], rb.a[b], fb.a[b], tb.a[b]);
    }
    const int L = v[0].L, V = v[0].V;
    size_t lds = (size_t)V * 4;
    SJD_TRY(ensure_lds(3, ept_class(V), lds));
    EPT_SWITCH(ept_class(V), SJD_LAUNCH(sjd_rows_batch_kernel<EPT>, dim3(L, B), dim3(DIST_THREADS), lds, s, rb))
    HIP_TRY(hipGetLastError());
    SJD_LAUNCH(sjd_finalize_batch_kernel, dim3(L, FIN_PARTS, B), dim3(256), 0, s, fb);
    HIP_TRY(hipGetLastError());
    if (v[0].init.mode == 3 || v[0].init.mode == 4) {
        EPT_SWITCH(ept_class(V), SJD_LAUNCH(sjd_tail_batch_kernel<EPT>, dim3(L, B), dim3(DIST_THREADS), 0, s, tb))
        HIP_TRY(hipGetLastError());
    }
    return SJD_OK;
}

// Many independent rows in one launch (far more than the chip has CUs): workgroups of 256 or 512 threads with 32
// values per thread, so that a CU has four or two rows in flight instead of one; same results bit for bit.
#define DIST_MANY_ROWS 512
template <int NT>
static int ensure_lds_many(size_t lds)
{
    static std::mutex mu;
    static size_t lds_set = 0;
    if (lds <= 48 * 1024) return SJD_OK;
    std::lock_guard<std::mutex> lock(mu);
    if (lds > lds_set) {
        HIP_TRY(hipFuncSetAttribute((const void *)sjd_dist_kernel<32, NT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        lds_set = lds;
    }
    return SJD_OK;
}

template <int NT>
static int launch_dist_many(const float *logits, const float *logits_u, float cfg_scale, int32_t rows, int32_t V,
                            const sjd_sampler *smp, const int32_t *forced, float *q, hipStream_t s)
{
    const size_t lds = (size_t)V * 4;
    SJD_TRY(ensure_lds_many<NT>(lds));
    SJD_LAUNCH((sjd_dist_kernel<32, NT>), dim3(rows), dim3(NT), lds, s, logits, logits_u, cfg_scale, V, *smp, forced, q);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_launch_dist(const float *logits, const float *logits_u, float cfg_scale, int32_t rows, int32_t V,
                    const sjd_sampler *smp, const int32_t *forced, float *q, hipStream_t s)
{
    if (V < 1 || V > SJD_MAX_SAMP_VOCAB || rows < 1) return SJD_EINVAL;
    if (rows >= DIST_MANY_ROWS && V <= 256 * 32) return launch_dist_many<256>(logits, logits_u, cfg_scale, rows, V, smp, forced, q, s);
    if (rows >= DIST_MANY_ROWS && V <= 512 * 32) return launch_dist_many<512>(logits, logits_u, cfg_scale, rows, V, smp, forced, q, s);
    size_t lds = (size_t)V * 4;
    SJD_TRY(ensure_lds(1, ept_class(V), lds));
    EPT_SWITCH(ept_class(V), SJD_LAUNCH(sjd_dist_kernel<EPT>, dim3(rows), dim3(DIST_THREADS), lds, s, logits, logits_u, cfg_scale, V, *smp, forced, q))
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_launch_first_window(const float *q_first, int32_t L, int32_t V, int32_t lo, const sjd_init *init,
                            uint64_t seed, int32_t *draft, float *p_old, hipStream_t s)
{
    if (V < 1 || V > SJD_MAX_SAMP_VOCAB || L < 1 || L > SJD_MAX_WINDOW) return SJD_EINVAL;
    size_t lds = (size_t)V * 4;
    SJD_TRY(ensure_lds(2, ept_class(V), lds));
    EPT_SWITCH(ept_class(V), SJD_LAUNCH(sjd_first_window_kernel<EPT>, dim3(L), dim3(DIST_THREADS), lds, s, q_first, L, V, lo,
                                        *init, seed, draft, p_old))
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

// out[e] = guided logits of two rows sets (parity hook of the two-stream forward)
__global__ void sjd_guide_kernel(const float *zc, const float *zu, float w, size_t n, float *out)
{
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (size_t)gridDim.x * blockDim.x)
        out[e] = guide(zc[e], zu[e], w);
}

int sjd_launch_guide(const float *logits, const float *logits_u, float cfg_scale, size_t n, float *out, hipStream_t s)
{
    SJD_LAUNCH(sjd_guide_kernel, dim3(256), dim3(256), 0, s, logits, logits_u, cfg_scale, n, out);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}
