// Sampling distribution, probabilistic verification and window slide for SJD on gfx950.
//
// Paper Sec. 3.1 (softmax classifier + top-K sampling), Sec. 4.1 Step 3 (Eqs. 1-3) and Step 4,
// Sec. 4.2 (initialisation of new slots).  Two kernels per iteration:
//   sjd_rows_kernel      one workgroup per window index i = 1..L: top-K select (radix select on
//                        order-preserving keys held in LDS), softmax, the accept test of Eq. 1 for
//                        its own draft, a candidate sample from q_i (Eq. 3) and a candidate sample
//                        from max(0, q_i - p_old_i) (Eq. 2).  Nothing here depends on where the scan
//                        stops, so all rows run concurrently.
//   sjd_finalize_kernel  one workgroup per slot of the NEXT window: finds the first rejection, picks
//                        the candidates that apply, copies the distributions into next-window order,
//                        initialises the tail slots and advances the device-resident state.
//
// Every data-dependent decision is an integer comparison or one correctly rounded fp32 operation
// (this file is compiled with floating-point contraction off), so results do not depend on
// reduction order: sums that decide anything are taken in 40-bit fixed point.
#include "sjd_internal.h"

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
__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        uint32_t lo = __shfl_xor((uint32_t)v, o), hi = __shfl_xor((uint32_t)(v >> 32), o);
        v += ((uint64_t)hi << 32) | lo;
    }
    return v;
}
__device__ __forceinline__ uint64_t shfl_up_u64(uint64_t v, int o)
{
    uint32_t lo = __shfl_up((uint32_t)v, o), hi = __shfl_up((uint32_t)(v >> 32), o);
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t shfl_u64(uint64_t v, int src)
{
    uint32_t lo = __shfl((uint32_t)v, src), hi = __shfl((uint32_t)(v >> 32), src);
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { uint32_t t = __shfl_xor(v, o); v = t > v ? t : v; }
    return v;
}
__device__ __forceinline__ int wave_sum_i32(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

struct DistShared {
    uint64_t wave_tot[DIST_WAVES];
    uint32_t wave_u32[DIST_WAVES];
    int hist[256];
    uint32_t sel_prefix;
    int sel_rank;
    int result;
};

// Categorical draw from non-negative weights by inverse CDF over 40-bit fixed-point values taken
// in index order: tau = floor(k32 * C / 2^32), result = first index whose inclusive prefix sum
// exceeds tau.  The weight of index t is WeightFn(t).  Wave w owns the contiguous index range
// [w*span, (w+1)*span).  Returns -1 when C == 0.  All threads get the result.
template <class WeightFn>
__device__ int block_sample(WeightFn weight, int V, uint32_t k32, DistShared *sh)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int span = ((V + DIST_WAVES * 64 - 1) / (DIST_WAVES * 64)) * 64;  // multiple of 64
    const int beg = wave * span;
    const int end = min(V, beg + span);
    uint64_t local = 0;
    for (int t = beg + lane; t < end; t += 64) local += fixed40(weight(t));
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
            for (int g = beg; g < end; g += 64) {
                int t = g + lane;
                uint64_t c = t < end ? fixed40(weight(t)) : 0;
                uint64_t incl = c;
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) { uint64_t up = shfl_up_u64(incl, o); if (lane >= o) incl += up; }
                unsigned long long hit = __ballot(base + incl > tau);
                if (hit) {
                    if (lane == 0) sh->result = g + __ffsll(hit) - 1;
                    break;
                }
                base += shfl_u64(incl, 63);
            }
        }
    }
    __syncthreads();
    return sh->result;
}

// The sampling distribution of one logits row, left in `buf` (LDS, V floats) and returned to the
// caller for writing.  Steps: (1) forced -> one-hot; (2) keep exactly K entries by (value
// descending, index ascending); (3) e = exp((z - max)/T), Z = sum of e in fixed point,
// q = e / Z; (4) K == 1 or T == 0 -> one-hot at the arg-max, lowest index on ties.
__device__ void block_dist(const float *__restrict__ z, int V, int top_k, float T, int forced, uint32_t *buf,
                           DistShared *sh)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float *qb = reinterpret_cast<float *>(buf);
    if (forced >= 0) {
        for (int t = tid; t < V; t += DIST_THREADS) qb[t] = (t == forced) ? 1.0f : 0.0f;
        __syncthreads();
        return;
    }
    // keys into LDS, block max
    uint32_t kmax = 0;
    for (int t = tid; t < V; t += DIST_THREADS) {
        uint32_t k = order_key(z[t]);
        buf[t] = k;
        kmax = k > kmax ? k : kmax;
    }
    kmax = wave_max_u32(kmax);
    if (lane == 0) sh->wave_u32[wave] = kmax;
    __syncthreads();
    kmax = 0;
    for (int w = 0; w < DIST_WAVES; ++w) kmax = sh->wave_u32[w] > kmax ? sh->wave_u32[w] : kmax;

    if (top_k == 1 || T == 0.0f) {
        // lowest index holding the maximum
        int best = 0x7FFFFFFF;
        for (int t = tid; t < V; t += DIST_THREADS) if (buf[t] == kmax) best = min(best, t);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) best = min(best, __shfl_xor(best, o));
        __syncthreads();
        if (lane == 0) sh->hist[wave] = best;
        __syncthreads();
        best = 0x7FFFFFFF;
        for (int w = 0; w < DIST_WAVES; ++w) best = min(best, sh->hist[w]);
        __syncthreads();
        for (int t = tid; t < V; t += DIST_THREADS) qb[t] = (t == best) ? 1.0f : 0.0f;
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
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256) sh->hist[tid] = 0;
            __syncthreads();
            for (int t = tid; t < V; t += DIST_THREADS) {
                uint32_t k = buf[t];
                if ((k & mask) == prefix) atomicAdd(&sh->hist[(k >> shift) & 255u], 1);
            }
            __syncthreads();
            if (wave == 0) {
                // lane l covers digits 255-4l .. 252-4l (descending)
                int d0 = 255 - 4 * lane;
                int h0 = sh->hist[d0], h1 = sh->hist[d0 - 1], h2 = sh->hist[d0 - 2], h3 = sh->hist[d0 - 3];
                int tot = h0 + h1 + h2 + h3, incl = tot;
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) { int up = __shfl_up(incl, o); if (lane >= o) incl += up; }
                int excl = incl - tot;
                if (excl < rank && rank <= incl) {           // exactly one lane
                    int digit, before;
                    if (rank <= excl + h0) { digit = d0; before = excl; }
                    else if (rank <= excl + h0 + h1) { digit = d0 - 1; before = excl + h0; }
                    else if (rank <= excl + h0 + h1 + h2) { digit = d0 - 2; before = excl + h0 + h1; }
                    else { digit = d0 - 3; before = excl + h0 + h1 + h2; }
                    sh->sel_prefix = prefix | ((uint32_t)digit << shift);
                    sh->sel_rank = rank - before;
                }
            }
            __syncthreads();
            prefix = sh->sel_prefix;
            rank = sh->sel_rank;
            mask |= 255u << shift;
            __syncthreads();
        }
        kth = prefix;
        room = rank;           // = K - #(keys > kth)
        // entries equal to kth: do they all fit?
        int eq = 0;
        for (int t = tid; t < V; t += DIST_THREADS) eq += buf[t] == kth;
        eq = wave_sum_i32(eq);
        if (lane == 0) sh->hist[wave] = eq;
        __syncthreads();
        eq = 0;
        for (int w = 0; w < DIST_WAVES; ++w) eq += sh->hist[w];
        __syncthreads();
        if (eq > room) {
            // ties cut the K-th value: keep the `room` lowest indices.  Wave w scans its contiguous
            // index range; a tie that loses gets its key lowered to kth - 1 so that the test
            // `key >= kth` below drops it (kth == 0 only arises from NaN logits, which are
            // outside the contract).
            const int span = ((V + DIST_WAVES * 64 - 1) / (DIST_WAVES * 64)) * 64;
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
                int incl = f;
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) { int up = __shfl_up(incl, o); if (lane >= o) incl += up; }
                if (f && base + incl > room && kth > 0) buf[t] = kth - 1;
                base += __shfl(incl, 63);
            }
            __syncthreads();
        }
    }

    // ---- softmax over the survivors ----------------------------------------------------------
    const float m = key_to_float(kmax);
    uint64_t csum = 0;
    for (int t = tid; t < V; t += DIST_THREADS) {
        uint32_t k = buf[t];
        bool keep = !cut || k >= kth;
        float e = 0.0f;
        if (keep) {
            float x = __fdiv_rn(__fsub_rn(z[t], m), T);
            e = exp_fixed(x);
        }
        qb[t] = e;
        csum += fixed40(e);
    }
    csum = wave_sum_u64(csum);
    if (lane == 0) sh->wave_tot[wave] = csum;
    __syncthreads();
    uint64_t C = 0;
    for (int w = 0; w < DIST_WAVES; ++w) C += sh->wave_tot[w];
    const float Z = __fmul_rn(__ull2float_rn(C), 0x1p-40f);
    for (int t = tid; t < V; t += DIST_THREADS) {
        float e = qb[t];
        qb[t] = (e != 0.0f) ? __fdiv_rn(e, Z) : 0.0f;
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
    const float *logits, *q_in, *p_old;
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

__global__ __launch_bounds__(DIST_THREADS) void sjd_rows_kernel(RowsArgs a)
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
    float *qrow = a.q + (size_t)i * V;
    float *qb = reinterpret_cast<float *>(buf);
    if (a.q_in) {
        const float *src = a.q_in + (size_t)i * V;
        for (int t = threadIdx.x; t < V; t += DIST_THREADS) qb[t] = src[t];
        __syncthreads();
    } else {
        block_dist(a.logits + (size_t)(i - 1) * V, V, a.smp.top_k, a.smp.temperature,
                   forced_index(a.init, img_pos0 + i, a.lo), buf, &sh);
    }
    for (int t = threadIdx.x; t < V; t += DIST_THREADS) qrow[t] = qb[t];

    const U4 rnd = philox_draw(a.seed, counter, (uint32_t)i);
    // candidate for Eq. 3 (and for the bonus index L): a plain sample from q_i
    int s = block_sample([&](int t) { return qb[t]; }, V, rnd.w[2], &sh);
    if (threadIdx.x == 0) a.tok_smp[i] = s;
    if (i < L) {
        const float *po = a.p_old + (size_t)i * V;
        if (threadIdx.x == 0) {
            // Eq. 1: accept iff r < min(1, q_i(x_i) / p_old_i(x_i)); a NaN ratio rejects
            int x = a.draft[i] - a.lo;
            int ok = 0;
            if (x >= 0 && x < V) {
                float ratio = __fdiv_rn(qb[x], po[x]);
                float r = u_from_word(rnd.w[0]);
                ok = (ratio >= 1.0f) || (r < ratio);
            }
            a.acc_flag[i] = ok;
        }
        // candidate for Eq. 2: sample from max(0, q_i - p_old_i); if that vanishes, from q_i
        int rs = block_sample([&](int t) { float d = __fsub_rn(qb[t], po[t]); return d > 0.0f ? d : 0.0f; }, V,
                              rnd.w[1], &sh);
        if (rs < 0) rs = block_sample([&](int t) { return qb[t]; }, V, rnd.w[1], &sh);
        if (threadIdx.x == 0) a.tok_res[i] = rs;
    }
}

struct FinalArgs {
    int32_t L, V, lo;
    sjd_init init;
    uint64_t seed;
    const int32_t *hist;          // image-position-indexed ids, or NULL
    SjdState *state;              // advanced by workgroup 0 when non-NULL
    int32_t *kv_tokens;           // cache-position-indexed ids (with state), or NULL
    const float *q;
    const int32_t *tok_smp, *tok_res, *acc_flag, *draft_snap;
    const StepSnap *snap;
    int32_t *n_accepted, *new_draft;
    float *p_new;
};

__global__ __launch_bounds__(256) void sjd_finalize_kernel(FinalArgs a)
{
    const StepSnap sn = *a.snap;
    if (!sn.active) return;
    const int L = sn.L_eff, V = a.V, lo = a.lo;
    const int j = blockIdx.x;
    // Eq. 1 scan: index 0 is exact by construction; stop at the first rejection
    int acc = 1;
    while (acc < L && a.acc_flag[acc]) ++acc;
    const int n_model = L - acc + 1;
    const int n_hist = sn.img_pos0 + acc;
    const int32_t *hist = a.hist;
    if (a.kv_tokens) hist = a.kv_tokens + (sn.n - sn.img_pos0);

    if (j < L) {
        auto model_tok = [&](int slot) {   // token of next-window slot < n_model (local index)
            int src = acc + slot;
            if (slot == 0) return acc < L ? a.tok_res[acc] : a.tok_smp[L];
            return a.tok_smp[src];
        };
        if (j < n_model) {
            if (threadIdx.x == 0) a.new_draft[j] = model_tok(j) + lo;
            const float *src = a.q + (size_t)(acc + j) * V;
            float *dst = a.p_new + (size_t)j * V;
            for (int t = threadIdx.x; t < V; t += 256) dst[t] = src[t];
        } else {
            // Sec. 4.2 initialisation of image position n_hist + j
            int pos = n_hist + j;
            bool onehot = forced_index(a.init, pos, lo) >= 0 || (a.init.mode == 1 && pos - a.init.row_stride >= 0);
            int tok;
            for (;;) {
                int f = forced_index(a.init, pos, lo);
                if (f >= 0) { tok = f; break; }
                if (a.init.mode == 1 && pos - a.init.row_stride >= 0) {
                    pos -= a.init.row_stride;
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
            if (threadIdx.x == 0) a.new_draft[j] = tok + lo;
            float *dst = a.p_new + (size_t)j * V;
            const float u = __fdiv_rn(1.0f, (float)V);
            for (int t = threadIdx.x; t < V; t += 256) dst[t] = onehot ? (t == tok ? 1.0f : 0.0f) : u;
        }
    }
    if (j == 0 && threadIdx.x == 0) {
        if (a.n_accepted) a.n_accepted[0] = acc;
        if (a.state) {
            SjdState *st = a.state;
            if (a.kv_tokens) for (int i = 0; i < acc; ++i) a.kv_tokens[sn.n + i] = a.draft_snap[i];
            st->n = sn.n + acc;
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

__global__ __launch_bounds__(DIST_THREADS) void sjd_dist_kernel(const float *logits, int V, sjd_sampler smp,
                                                                const int32_t *forced, float *q)
{
    extern __shared__ uint32_t buf[];
    __shared__ DistShared sh;
    const int row = blockIdx.x;
    block_dist(logits + (size_t)row * V, V, smp.top_k, smp.temperature, forced ? forced[row] : -1, buf, &sh);
    const float *qb = reinterpret_cast<const float *>(buf);
    for (int t = threadIdx.x; t < V; t += DIST_THREADS) q[(size_t)row * V + t] = qb[t];
}

// First window (step counter 0): slot 0 ~ q_first, slots 1..L-1 by the init strategy.
__global__ __launch_bounds__(DIST_THREADS) void sjd_first_window_kernel(const float *q_first, int L, int V, int lo,
                                                                        sjd_init init, uint64_t seed,
                                                                        int32_t *draft, float *p_old)
{
    extern __shared__ uint32_t buf[];
    __shared__ DistShared sh;
    __shared__ int tok0;
    const int j = blockIdx.x;
    if (j == 0 || init.mode == 1) {
        // slot 0's token (every workgroup that may copy from it recomputes it: same inputs, same bits)
        float *qb = reinterpret_cast<float *>(buf);
        for (int t = threadIdx.x; t < V; t += DIST_THREADS) qb[t] = q_first[t];
        __syncthreads();
        U4 rnd = philox_draw(seed, 0, 0);
        int s = block_sample([&](int t) { return qb[t]; }, V, rnd.w[2], &sh);
        if (threadIdx.x == 0) tok0 = s;
        __syncthreads();
    }
    if (j == 0) {
        if (threadIdx.x == 0) draft[0] = tok0 + lo;
        for (int t = threadIdx.x; t < V; t += DIST_THREADS) p_old[t] = q_first[t];
        return;
    }
    int pos = j;
    bool onehot = forced_index(init, pos, lo) >= 0 || (init.mode == 1 && pos - init.row_stride >= 0);
    int tok;
    for (;;) {
        int f = forced_index(init, pos, lo);
        if (f >= 0) { tok = f; break; }
        if (init.mode == 1 && pos - init.row_stride >= 0) {
            pos -= init.row_stride;
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
static size_t g_lds_set[3] = {0, 0, 0};
static int ensure_lds(int which, const void *fn, size_t bytes)
{
    if (bytes <= 48 * 1024 || bytes <= g_lds_set[which]) return SJD_OK;
    HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    g_lds_set[which] = bytes;
    return SJD_OK;
}

int sjd_sample_setup(int32_t V)
{
    const size_t lds = (size_t)V * 4;
    SJD_TRY(ensure_lds(0, (const void *)sjd_rows_kernel, lds));
    SJD_TRY(ensure_lds(1, (const void *)sjd_dist_kernel, lds));
    SJD_TRY(ensure_lds(2, (const void *)sjd_first_window_kernel, lds));
    return SJD_OK;
}

int sjd_launch_verify(const SjdVerifyArgs *v, hipStream_t s)
{
    if (v->V < 1 || v->V > SJD_MAX_SAMP_VOCAB || v->L < 1 || v->L > SJD_ROWS_MAX) return SJD_EINVAL;
    size_t lds = (size_t)v->V * 4;
    SJD_TRY(ensure_lds(0, (const void *)sjd_rows_kernel, lds));
    RowsArgs r;
    r.logits = v->logits; r.q_in = v->q_in; r.p_old = v->p_old; r.draft = v->draft;
    r.L = v->L; r.V = v->V; r.lo = v->lo; r.smp = v->smp; r.init = v->init; r.seed = v->seed;
    r.state = v->state; r.img_pos0 = v->img_pos0; r.counter = v->counter;
    r.q = v->q; r.tok_smp = v->tok_smp; r.tok_res = v->tok_res; r.acc_flag = v->acc_flag;
    r.draft_snap = v->draft_snap; r.snap = reinterpret_cast<StepSnap *>(v->snap);
    SJD_LAUNCH(sjd_rows_kernel, dim3(v->L), dim3(DIST_THREADS), lds, s, r);
    HIP_TRY(hipGetLastError());
    FinalArgs f;
    f.L = v->L; f.V = v->V; f.lo = v->lo; f.init = v->init; f.seed = v->seed; f.hist = v->hist;
    f.state = v->state; f.kv_tokens = v->kv_tokens; f.q = v->q; f.tok_smp = v->tok_smp; f.tok_res = v->tok_res;
    f.acc_flag = v->acc_flag; f.draft_snap = v->draft_snap; f.snap = reinterpret_cast<const StepSnap *>(v->snap);
    f.n_accepted = v->n_accepted; f.new_draft = v->new_draft; f.p_new = v->p_new;
    SJD_LAUNCH(sjd_finalize_kernel, dim3(v->L), dim3(256), 0, s, f);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_launch_dist(const float *logits, int32_t rows, int32_t V, const sjd_sampler *smp, const int32_t *forced,
                    float *q, hipStream_t s)
{
    if (V < 1 || V > SJD_MAX_SAMP_VOCAB || rows < 1) return SJD_EINVAL;
    size_t lds = (size_t)V * 4;
    SJD_TRY(ensure_lds(1, (const void *)sjd_dist_kernel, lds));
    SJD_LAUNCH(sjd_dist_kernel, dim3(rows), dim3(DIST_THREADS), lds, s, logits, V, *smp, forced, q);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

int sjd_launch_first_window(const float *q_first, int32_t L, int32_t V, int32_t lo, const sjd_init *init,
                            uint64_t seed, int32_t *draft, float *p_old, hipStream_t s)
{
    if (V < 1 || V > SJD_MAX_SAMP_VOCAB || L < 1 || L > SJD_ROWS_MAX) return SJD_EINVAL;
    size_t lds = (size_t)V * 4;
    SJD_TRY(ensure_lds(2, (const void *)sjd_first_window_kernel, lds));
    SJD_LAUNCH(sjd_first_window_kernel, dim3(L), dim3(DIST_THREADS), lds, s, q_first, L, V, lo, *init, seed,
                       draft, p_old);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}
