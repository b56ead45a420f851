/* CPU oracle for Speculative Jacobi Decoding -- TEST INFRASTRUCTURE ONLY (see sjd_oracle.h).
 *
 * Written from the paper's Sec. 3.1 (auto-regressive sampling), Sec. 3.2 (Jacobi decoding),
 * Sec. 4.1 (Steps 1-4, Eqs. 1-3), Sec. 4.2 (initialisation) and Appendix A (Theorem 1).
 * Plain loops, fp64 for the transformer, no blocking or fusion.  Every function is pinned by
 * tests that do not call it to produce their own expectation (closed forms, brute force,
 * the L=1 == AR and K=1 == greedy reductions, a chi-square against the exact AR joint).
 */
#include "sjd_oracle.h"

#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* threads the fp64 matrix products use (for reporting timings) */
int32_t orc_num_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}

/* ===================================================================================== */
/* Philox4x32-10: the published counter-based generator (Salmon et al., SC'11).          */
/* ===================================================================================== */
void orc_philox4x32_10(const uint32_t key[2], const uint32_t ctr[4], uint32_t out[4])
{
    uint32_t k0 = key[0], k1 = key[1];
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Reading: key = 64-bit seed, counter = (step counter c, window index i, 0); the four output
 * words are used, in order, for: acceptance test, residual resample, plain sample, init.   */
void orc_draw(uint64_t seed, uint64_t c, uint32_t i, uint32_t out[4])
{
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t ctr[4] = {(uint32_t)c, (uint32_t)(c >> 32), i, 0u};
    orc_philox4x32_10(key, ctr, out);
}

/* r ~ U[0,1) of Eq. 1 with 24 random bits, so that r < 1 always holds. */
float orc_u_acc(uint32_t word)
{
    return (float)(word >> 8) * 0x1p-24f;
}

/* ===================================================================================== */
/* exp for the softmax, as a fixed recipe of correctly-rounded fp32 operations (Cody-Waite */
/* range reduction + degree-7 Taylor polynomial), so that any IEEE machine gives the same  */
/* bits.  Domain x <= 0; x < -60 returns exactly 0.                                         */
/* ===================================================================================== */
float orc_exp(float x)
{
    if (!(x >= -60.0f)) return 0.0f;
    float n = rintf(x * 1.44269504088896341f);
    float r = fmaf(n, -0.693145751953125f, x);          /* ln2 high part: 0x1.62e3p-1      */
    r = fmaf(n, -1.42860682030941723e-6f, r);           /* ln2 low part                    */
    float p = 1.0f / 5040.0f;
    p = fmaf(p, r, 1.0f / 720.0f);
    p = fmaf(p, r, 1.0f / 120.0f);
    p = fmaf(p, r, 1.0f / 24.0f);
    p = fmaf(p, r, 1.0f / 6.0f);
    p = fmaf(p, r, 0.5f);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    return ldexpf(p, (int)n);                           /* exact: result stays normal      */
}

/* total order on fp32 bit patterns that agrees with < on ordinary floats */
static uint32_t order_key(float z)
{
    uint32_t b;
    memcpy(&b, &z, 4);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

/* weight -> 40-bit fixed point, truncated (exact: power-of-two scaling of an fp32) */
static uint64_t fixed40(float w)
{
    if (!(w > 0.0f)) return 0;
    return (uint64_t)((double)w * 0x1p40);
}

/* ===================================================================================== */
/* dist(): the distribution the sampler really draws from (Sec. 3.1: softmax + top-K).     */
/*  1. forced >= 0: one-hot.                                                               */
/*  2. keep the K largest logits, ties at the K-th value resolved towards the lower index. */
/*  3. e_t = exp((z_t - max)/T); Z = sum of the e_t in 40-bit fixed point (order-free);    */
/*     q_t = e_t / Z.                                                                      */
/*  4. K == 1 or T == 0: one-hot at the arg-max (lowest index on ties).                    */
/* ===================================================================================== */
void orc_dist(const float *z, int32_t V, int32_t top_k, float temperature, int32_t forced, float *q)
{
    for (int32_t t = 0; t < V; ++t) q[t] = 0.0f;
    if (forced >= 0) { q[forced] = 1.0f; return; }

    /* arg-max by (key desc, index asc) */
    int32_t best = 0;
    for (int32_t t = 1; t < V; ++t)
        if (order_key(z[t]) > order_key(z[best])) best = t;
    if (top_k == 1 || temperature == 0.0f) { q[best] = 1.0f; return; }

    /* keep[t] = 1 iff fewer than K entries precede t in the order (key desc, index asc) */
    int32_t K = top_k < V ? top_k : V;
    unsigned char *keep = (unsigned char *)malloc((size_t)V);
    if (K >= V) {
        memset(keep, 1, (size_t)V);
    } else {
        /* K-th largest key by counting: smallest key value kth such that #(key > kth) < K */
        uint32_t *keys = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)V);
        for (int32_t t = 0; t < V; ++t) keys[t] = order_key(z[t]);
        uint32_t kth = 0; /* binary search over the 32-bit key space */
        {
            uint32_t lo = 0, hi = 0xFFFFFFFFu;
            while (lo < hi) {
                uint32_t mid = lo + (hi - lo) / 2;
                int32_t above = 0;
                for (int32_t t = 0; t < V; ++t) above += keys[t] > mid;
                if (above < K) hi = mid; else lo = mid + 1;
            }
            kth = lo;
        }
        int32_t above = 0;
        for (int32_t t = 0; t < V; ++t) above += keys[t] > kth;
        int32_t room = K - above; /* how many entries equal to kth survive, lowest index first */
        for (int32_t t = 0; t < V; ++t) {
            if (keys[t] > kth) keep[t] = 1;
            else if (keys[t] == kth && room > 0) { keep[t] = 1; --room; }
            else keep[t] = 0;
        }
        free(keys);
    }

    float m = z[best];
    uint64_t C = 0;
    for (int32_t t = 0; t < V; ++t) {
        if (!keep[t]) continue;
        float x = (z[t] - m) / temperature;
        q[t] = orc_exp(x);
        C += fixed40(q[t]);
    }
    float Z = (float)C * 0x1p-40f;
    for (int32_t t = 0; t < V; ++t)
        if (keep[t]) q[t] = q[t] / Z;
    free(keep);
}

/* ===================================================================================== */
/* sample(): categorical draw by inverse CDF over 40-bit fixed-point weights.               */
/* tau = floor(k32 * C / 2^32); result = first index whose inclusive prefix sum exceeds it. */
/* ===================================================================================== */
int32_t orc_sample(const float *w, int32_t V, uint32_t k32)
{
    uint64_t C = 0;
    for (int32_t t = 0; t < V; ++t) C += fixed40(w[t]);
    if (C == 0) return -1;
    uint64_t tau = (uint64_t)(((unsigned __int128)k32 * (unsigned __int128)C) >> 32);
    uint64_t prefix = 0;
    for (int32_t t = 0; t < V; ++t) {
        prefix += fixed40(w[t]);
        if (prefix > tau) return t;
    }
    return -1; /* unreachable: tau < C */
}

/* Classifier-free guidance (Sec. 5.1 gives the weight, the usual logit-space mechanism is assumed):
 * z = z_uncond + w * (z_cond - z_uncond), three separately rounded fp32 operations.             */
void orc_guide(const float *z_cond, const float *z_uncond, float w, int64_t n, float *out)
{
    for (int64_t i = 0; i < n; ++i) {
        float diff = z_cond[i] - z_uncond[i];
        float scaled = w * diff;
        out[i] = z_uncond[i] + scaled;
    }
}

/* position-dependent allowed set: the last position of every grid row is the row-end token */
static int32_t forced_index(const orc_init *init, int32_t img_pos, int32_t lo)
{
    if (init->eol_id >= 0 && init->row_stride > 0 && (img_pos + 1) % init->row_stride == 0)
        return init->eol_id - lo;
    return -1;
}

/* Sec. 4.2: a newly initialised slot.  Returns the token (local index) and writes the
 * distribution it was really drawn from (so that Eq. 1's denominator is truthful):
 *   uniform           -> uniform row
 *   repeat-above (b)  -> copy of the current token one grid row up, one-hot row; the first
 *                        grid row falls back to uniform.
 *   repeat-left (a)   -> copy of the current token at the previous raster position, one-hot row
 *                        (the first column takes the last token of the row before).
 *   sample-left (c)   -> a fresh draw from the distribution recorded for the nearest slot to the left
 *                        in the window being built that is not a forced row-end slot; that row is
 *                        the new slot's row too.  No such slot -> uniform.
 *   sample-above (d)  -> a fresh draw from the distribution recorded for the position one grid row up:
 *                        `ring` for an accepted position, the window's row otherwise; first grid row
 *                        -> uniform.
 * `cur(pos)` = current token at image position pos: accepted history or the window being built.
 * `rows` = distributions of the window being built (slot s at rows + s*V; slots left of this one are
 * final), `ring` = [row_stride x V] distributions of accepted positions, entry pos % row_stride.  */
static int32_t init_slot(const orc_init *init, int32_t V, int32_t lo, int32_t img_pos, uint32_t word,
                         const int32_t *hist, int32_t n_hist, const int32_t *window, const float *rows,
                         const float *ring, float *row)
{
    int32_t forced = forced_index(init, img_pos, lo);
    int32_t tok = -1;
    int onehot = 0;
    if (forced >= 0) {
        tok = forced; onehot = 1;
    } else if ((init->mode == 1 && img_pos - init->row_stride >= 0) || (init->mode == 2 && img_pos - 1 >= 0)) {
        int32_t src = img_pos - (init->mode == 1 ? init->row_stride : 1);
        int32_t id = src < n_hist ? hist[src] : window[src - n_hist];
        tok = id - lo; onehot = 1;
    } else if (init->mode == 3 || init->mode == 4) {
        const float *src = NULL;
        if (init->mode == 3) {
            int32_t s = img_pos - n_hist - 1;                       /* slot to the left */
            while (s >= 0 && forced_index(init, n_hist + s, lo) >= 0) --s;
            if (s >= 0) src = rows + (size_t)s * V;
        } else {
            int32_t up = img_pos - init->row_stride;
            if (up >= n_hist) src = rows + (size_t)(up - n_hist) * V;
            else if (up >= 0) src = ring + (size_t)(up % init->row_stride) * V;
        }
        if (src) {
            tok = orc_sample(src, V, word);
            if (tok >= 0) {
                memcpy(row, src, sizeof(float) * (size_t)V);
                return tok;
            }
        }
    }
    if (tok < 0) tok = (int32_t)(((uint64_t)word * (uint64_t)V) >> 32);
    if (onehot) {
        for (int32_t t = 0; t < V; ++t) row[t] = 0.0f;
        row[tok] = 1.0f;
    } else {
        float u = 1.0f / (float)V;
        for (int32_t t = 0; t < V; ++t) row[t] = u;
    }
    return tok;
}

/* ===================================================================================== */
/* One verification (Sec. 4.1, Step 3 and Step 4).                                          */
/* ===================================================================================== */
int32_t orc_verify_probs(const float *q, const float *p_old, const int32_t *draft, int32_t L, int32_t V,
                         int32_t lo, const orc_init *init, int32_t img_pos0, const int32_t *hist,
                         uint64_t seed, uint64_t counter, float *ring, int32_t *new_draft, float *p_new)
{
    if (init->mode == 4 && !ring) { fprintf(stderr, "orc_verify: sample-above needs the ring\n"); abort(); }
    uint32_t w4[4];

    /* Eq. 1: scan left to right.  Window index 0 follows an all-accepted prefix, so its
     * distribution is unchanged from the last iteration (ratio 1): accepted by construction. */
    int32_t a = 1;
    for (int32_t i = 1; i < L; ++i) {
        int32_t x = draft[i] - lo;
        float ratio = q[(size_t)i * V + x] / p_old[(size_t)i * V + x];
        orc_draw(seed, counter, (uint32_t)i, w4);
        float r = orc_u_acc(w4[0]);
        int accept = (ratio >= 1.0f) || (r < ratio);     /* r < min(1, ratio); NaN rejects */
        if (!accept) break;
        ++a;
    }

    /* tokens for window indices a..L of this iteration's window */
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)(L + 1));
    if (a < L) {
        /* Eq. 2: resample the rejected index from normalize(max(0, p_new - p_old)) */
        float *w = (float *)malloc(sizeof(float) * (size_t)V);
        for (int32_t t = 0; t < V; ++t) {
            float diff = q[(size_t)a * V + t] - p_old[(size_t)a * V + t];
            w[t] = diff > 0.0f ? diff : 0.0f;
        }
        orc_draw(seed, counter, (uint32_t)a, w4);
        int32_t s = orc_sample(w, V, w4[1]);
        if (s < 0) s = orc_sample(q + (size_t)a * V, V, w4[1]);   /* residual vanished numerically */
        tok[a] = s;
        free(w);
    } else {
        /* every draft accepted: the last forward row is an exact distribution for index L */
        orc_draw(seed, counter, (uint32_t)L, w4);
        tok[L] = orc_sample(q + (size_t)L * V, V, w4[2]);
    }
    /* Eq. 3: every later index is sampled afresh from this iteration's distribution */
    for (int32_t i = a + 1; i <= L; ++i) {
        orc_draw(seed, counter, (uint32_t)i, w4);
        tok[i] = orc_sample(q + (size_t)i * V, V, w4[2]);
    }

    /* Step 4: next window = unaccepted indices a..L followed by a-1 newly initialised slots.
     * With refinement switched off (the ablation of App. "refinement"), only the resampled index a
     * survives and every later slot is newly initialised. */
    int32_t n_model = (init->flags & 1) ? 1 : L - a + 1;
    for (int32_t j = 0; j < n_model; ++j) {
        new_draft[j] = tok[a + j] + lo;
        memcpy(p_new + (size_t)j * V, q + (size_t)(a + j) * V, sizeof(float) * (size_t)V);
    }
    /* sample-above: record the distribution of every accepted position, in position order.  Index 0
     * carries its (exact) row from the last iteration, the others this iteration's rows. */
    if (init->mode == 4)
        for (int32_t i = 0; i < a; ++i)
            memcpy(ring + (size_t)((img_pos0 + i) % init->row_stride) * V, i == 0 ? p_old : q + (size_t)i * V,
                   sizeof(float) * (size_t)V);
    /* accepted history seen by repeat-above: hist[0..img_pos0) then draft[0..a) */
    int32_t n_hist = img_pos0 + a;
    int32_t *h2 = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_hist > 0 ? n_hist : 1));
    for (int32_t p = 0; p < img_pos0; ++p) h2[p] = hist ? hist[p] : 0;
    for (int32_t p = 0; p < a; ++p) h2[img_pos0 + p] = draft[p];
    for (int32_t j = n_model; j < L; ++j) {
        orc_draw(seed, counter, (uint32_t)(L + 1 + (j - n_model)), w4);
        int32_t t = init_slot(init, V, lo, n_hist + j, w4[3], h2, n_hist, new_draft, p_new, ring,
                              p_new + (size_t)j * V);
        new_draft[j] = t + lo;
    }
    free(h2);
    free(tok);
    return a;
}

int32_t orc_verify(const float *logits, const float *p_old, const int32_t *draft, int32_t L, int32_t V,
                   int32_t lo, const orc_sampler *smp, const orc_init *init, int32_t img_pos0,
                   const int32_t *hist, uint64_t seed, uint64_t counter, float *ring, int32_t *new_draft,
                   float *p_new)
{
    float *q = (float *)malloc(sizeof(float) * (size_t)(L + 1) * V);
    memcpy(q, p_old, sizeof(float) * (size_t)V);
    for (int32_t i = 1; i <= L; ++i)
        orc_dist(logits + (size_t)(i - 1) * V, V, smp->top_k, smp->temperature,
                 forced_index(init, img_pos0 + i, lo), q + (size_t)i * V);
    int32_t a = orc_verify_probs(q, p_old, draft, L, V, lo, init, img_pos0, hist, seed, counter, ring, new_draft,
                                 p_new);
    free(q);
    return a;
}

void orc_first_window(const float *q_first, int32_t L, int32_t V, int32_t lo, const orc_init *init,
                      uint64_t seed, int32_t *draft, float *p_old)
{
    uint32_t w4[4];
    orc_draw(seed, 0, 0, w4);
    draft[0] = orc_sample(q_first, V, w4[2]) + lo;
    memcpy(p_old, q_first, sizeof(float) * (size_t)V);
    for (int32_t j = 1; j < L; ++j) {
        orc_draw(seed, 0, (uint32_t)j, w4);
        int32_t t = init_slot(init, V, lo, j, w4[3], NULL, 0, draft, p_old, NULL, p_old + (size_t)j * V);
        draft[j] = t + lo;
    }
}

/* ===================================================================================== */
/* Llama-style decoder in fp64.  Per layer:                                                 */
/*   h = RMSNorm(x; g1); q,k,v = Wq h, Wk h, Wv h; RoPE(q,k; pos);                          */
/*   x += Wo * softmax(q k^T / sqrt(hd) + causal) v;                                        */
/*   h = RMSNorm(x; g2); x += Wd (SiLU(Wg h) * (Wu h)).                                     */
/* logits = Wlm[lo:hi] RMSNorm(x; gf).  RoPE rotates dimension j with j + hd/2 by           */
/* pos * theta^(-2j/hd).                                                                    */
/* ===================================================================================== */
struct orc_model {
    orc_config cfg;
    const void *blob;
};

struct orc_kv {
    int32_t n_layers, d, max_seq, len;
    double *k, *v; /* [layer][pos][d] */
};

static double wval(const orc_model *m, size_t idx)
{
    if (m->cfg.dtype == 0) return (double)((const float *)m->blob)[idx];
    uint32_t b = (uint32_t)((const uint16_t *)m->blob)[idx] << 16;
    float f;
    memcpy(&f, &b, 4);
    return (double)f;
}

/* element offsets of the tensors in the blob (order documented with the weight generator) */
typedef struct {
    size_t E, gf, Wlm;
    size_t per_layer, g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd; /* layer l: base + l*per_layer */
    size_t layer0;
} offsets;

static offsets blob_offsets(const orc_config *c)
{
    offsets o;
    size_t d = (size_t)c->d_model, f = (size_t)c->d_ffn, v = (size_t)c->vocab_total;
    o.E = 0;
    o.layer0 = v * d;
    o.g1 = 0;
    o.Wq = d;
    o.Wk = o.Wq + d * d;
    o.Wv = o.Wk + d * d;
    o.Wo = o.Wv + d * d;
    o.g2 = o.Wo + d * d;
    o.Wg = o.g2 + d;
    o.Wu = o.Wg + f * d;
    o.Wd = o.Wu + f * d;
    o.per_layer = o.Wd + d * f;
    o.gf = o.layer0 + (size_t)c->n_layers * o.per_layer;
    o.Wlm = o.gf + d;
    return o;
}

orc_model *orc_model_create(const orc_config *cfg, const void *blob)
{
    orc_model *m = (orc_model *)malloc(sizeof(orc_model));
    m->cfg = *cfg;
    m->blob = blob;
    return m;
}
void orc_model_free(orc_model *m) { free(m); }

orc_kv *orc_kv_create(const orc_model *m)
{
    orc_kv *kv = (orc_kv *)malloc(sizeof(orc_kv));
    kv->n_layers = m->cfg.n_layers;
    kv->d = m->cfg.d_model;
    kv->max_seq = m->cfg.max_seq;
    kv->len = 0;
    size_t n = (size_t)kv->n_layers * kv->max_seq * kv->d;
    kv->k = (double *)calloc(n, sizeof(double));
    kv->v = (double *)calloc(n, sizeof(double));
    return kv;
}
void orc_kv_free(orc_kv *kv) { if (kv) { free(kv->k); free(kv->v); free(kv); } }
void orc_kv_set_len(orc_kv *kv, int32_t n) { kv->len = n; }
int32_t orc_kv_len(const orc_kv *kv) { return kv->len; }

void orc_embed(const orc_model *m, const int32_t *ids, int32_t n, double *x)
{
    size_t d = (size_t)m->cfg.d_model;
    for (int32_t t = 0; t < n; ++t)
        for (size_t j = 0; j < d; ++j) x[t * d + j] = wval(m, (size_t)ids[t] * d + j);
}

/* y[T x n_out] = x[T x n_in] * W^T, W stored [n_out][n_in] at element offset w_off */
static void linear(const orc_model *m, size_t w_off, const double *x, int32_t T, int32_t n_in, int32_t n_out,
                   double *y)
{
#pragma omp parallel for schedule(static)
    for (int32_t o = 0; o < n_out; ++o) {
        for (int32_t t = 0; t < T; ++t) {
            double acc = 0.0;
            for (int32_t i = 0; i < n_in; ++i)
                acc += wval(m, w_off + (size_t)o * n_in + i) * x[(size_t)t * n_in + i];
            y[(size_t)t * n_out + o] = acc;
        }
    }
}

static void rmsnorm(const orc_model *m, size_t g_off, const double *x, int32_t T, int32_t d, double *h)
{
    for (int32_t t = 0; t < T; ++t) {
        double ss = 0.0;
        for (int32_t j = 0; j < d; ++j) ss += x[(size_t)t * d + j] * x[(size_t)t * d + j];
        double inv = 1.0 / sqrt(ss / d + (double)m->cfg.rms_eps);
        for (int32_t j = 0; j < d; ++j) h[(size_t)t * d + j] = x[(size_t)t * d + j] * inv * wval(m, g_off + j);
    }
}

static void rope(const orc_model *m, double *v, int32_t T, int32_t pos0)
{
    int32_t H = m->cfg.n_heads, hd = m->cfg.d_model / H, half = hd / 2;
    for (int32_t t = 0; t < T; ++t)
        for (int32_t h = 0; h < H; ++h)
            for (int32_t j = 0; j < half; ++j) {
                double ang = (double)(pos0 + t) * pow((double)m->cfg.rope_theta, -2.0 * j / hd);
                double c = cos(ang), s = sin(ang);
                double *p = v + (size_t)t * m->cfg.d_model + (size_t)h * hd;
                double a = p[j], b = p[j + half];
                p[j] = a * c - b * s;
                p[j + half] = b * c + a * s;
            }
}

/* The shared layer stack.  Keys/values for positions pos0..pos0+T-1 are written to
 * (kc, vc) rows of each layer; query t attends positions 0..pos0+t.                     */
static void decoder_stack(const orc_model *m, double *kc, double *vc, int32_t kv_stride_layer, int32_t pos0,
                          const double *x_in, int32_t T, float *logits)
{
    const orc_config *c = &m->cfg;
    offsets o = blob_offsets(c);
    int32_t d = c->d_model, F = c->d_ffn, H = c->n_heads, hd = d / H;
    size_t Td = (size_t)T * d;
    double *x = (double *)malloc(sizeof(double) * Td);
    double *h = (double *)malloc(sizeof(double) * Td);
    double *q = (double *)malloc(sizeof(double) * Td);
    double *k = (double *)malloc(sizeof(double) * Td);
    double *v = (double *)malloc(sizeof(double) * Td);
    double *att = (double *)malloc(sizeof(double) * Td);
    double *proj = (double *)malloc(sizeof(double) * Td);
    double *gate = (double *)malloc(sizeof(double) * (size_t)T * F);
    double *up = (double *)malloc(sizeof(double) * (size_t)T * F);
    double *sc = (double *)malloc(sizeof(double) * (size_t)(pos0 + T));
    memcpy(x, x_in, sizeof(double) * Td);

    for (int32_t l = 0; l < c->n_layers; ++l) {
        size_t base = o.layer0 + (size_t)l * o.per_layer;
        double *kl = kc + (size_t)l * kv_stride_layer, *vl = vc + (size_t)l * kv_stride_layer;

        rmsnorm(m, base + o.g1, x, T, d, h);
        linear(m, base + o.Wq, h, T, d, d, q);
        linear(m, base + o.Wk, h, T, d, d, k);
        linear(m, base + o.Wv, h, T, d, d, v);
        rope(m, q, T, pos0);
        rope(m, k, T, pos0);
        memcpy(kl + (size_t)pos0 * d, k, sizeof(double) * Td);
        memcpy(vl + (size_t)pos0 * d, v, sizeof(double) * Td);

        for (int32_t t = 0; t < T; ++t)
            for (int32_t hh = 0; hh < H; ++hh) {
                int32_t n_keys = pos0 + t + 1; /* causal: positions 0..pos0+t */
                const double *qv = q + (size_t)t * d + (size_t)hh * hd;
                double mx = -INFINITY;
                for (int32_t s = 0; s < n_keys; ++s) {
                    const double *kv = kl + (size_t)s * d + (size_t)hh * hd;
                    double dot = 0.0;
                    for (int32_t j = 0; j < hd; ++j) dot += qv[j] * kv[j];
                    sc[s] = dot / sqrt((double)hd);
                    if (sc[s] > mx) mx = sc[s];
                }
                double den = 0.0;
                for (int32_t s = 0; s < n_keys; ++s) { sc[s] = exp(sc[s] - mx); den += sc[s]; }
                double *out = att + (size_t)t * d + (size_t)hh * hd;
                for (int32_t j = 0; j < hd; ++j) out[j] = 0.0;
                for (int32_t s = 0; s < n_keys; ++s) {
                    const double *vv = vl + (size_t)s * d + (size_t)hh * hd;
                    double p = sc[s] / den;
                    for (int32_t j = 0; j < hd; ++j) out[j] += p * vv[j];
                }
            }
        linear(m, base + o.Wo, att, T, d, d, proj);
        for (size_t e = 0; e < Td; ++e) x[e] += proj[e];

        rmsnorm(m, base + o.g2, x, T, d, h);
        linear(m, base + o.Wg, h, T, d, F, gate);
        linear(m, base + o.Wu, h, T, d, F, up);
        for (size_t e = 0; e < (size_t)T * F; ++e) {
            double g = gate[e];
            gate[e] = g / (1.0 + exp(-g)) * up[e];       /* SiLU(g) * u */
        }
        linear(m, base + o.Wd, gate, T, F, d, proj);
        for (size_t e = 0; e < Td; ++e) x[e] += proj[e];
    }

    rmsnorm(m, o.gf, x, T, d, h);
    int32_t V = c->samp_hi - c->samp_lo;
    double *lg = (double *)malloc(sizeof(double) * (size_t)T * V);
    linear(m, o.Wlm + (size_t)c->samp_lo * d, h, T, d, V, lg);
    for (size_t e = 0; e < (size_t)T * V; ++e) logits[e] = (float)lg[e];

    free(lg); free(sc); free(up); free(gate); free(proj); free(att);
    free(v); free(k); free(q); free(h); free(x);
}

void orc_forward_full(const orc_model *m, const double *x_in, int32_t T, float *logits)
{
    size_t n = (size_t)m->cfg.n_layers * T * m->cfg.d_model;
    double *kc = (double *)calloc(n, sizeof(double)), *vc = (double *)calloc(n, sizeof(double));
    decoder_stack(m, kc, vc, T * m->cfg.d_model, 0, x_in, T, logits);
    free(kc); free(vc);
}

void orc_forward_window(const orc_model *m, orc_kv *kv, const double *x_in, int32_t L, float *logits)
{
    decoder_stack(m, kv->k, kv->v, kv->max_seq * kv->d, kv->len, x_in, L, logits);
}

/* ===================================================================================== */
/* Decoding loops.                                                                          */
/* ===================================================================================== */
void orc_generate_sjd(orc_forward_fn fwd, void *ctx, int32_t n_prompt, const float *logits_prompt, int32_t V,
                      int32_t lo, int32_t N, int32_t L, const orc_sampler *smp, const orc_init *init,
                      uint64_t seed, int32_t *out, orc_stats *stats)
{
    int32_t *draft = (int32_t *)malloc(sizeof(int32_t) * (size_t)L);
    int32_t *next = (int32_t *)malloc(sizeof(int32_t) * (size_t)L);
    float *p_old = (float *)malloc(sizeof(float) * (size_t)L * V);
    float *p_new = (float *)malloc(sizeof(float) * (size_t)L * V);
    float *logits = (float *)malloc(sizeof(float) * (size_t)L * V);
    float *q0 = (float *)malloc(sizeof(float) * (size_t)V);
    float *ring = init->mode == 4 ? (float *)calloc((size_t)init->row_stride * V, sizeof(float)) : NULL;
    if (stats) memset(stats, 0, sizeof(*stats));

    /* Step 1 for the very first window: index 0 from the prompt's exact distribution */
    orc_dist(logits_prompt, V, smp->top_k, smp->temperature, forced_index(init, 0, lo), q0);
    orc_first_window(q0, L, V, lo, init, seed, draft, p_old);

    int32_t n_acc = 0;
    uint64_t c = 0;
    while (n_acc < N - 1) {
        ++c;
        int32_t Le = L < N - n_acc ? L : N - n_acc;      /* window clipped at the image end */
        fwd(ctx, n_prompt + n_acc, draft, Le, logits);   /* Step 2 */
        int32_t a = orc_verify(logits, p_old, draft, Le, V, lo, smp, init, n_acc, out, seed, c, ring, next, p_new);
        for (int32_t i = 0; i < a; ++i) out[n_acc + i] = draft[i];
        n_acc += a;
        memcpy(draft, next, sizeof(int32_t) * (size_t)Le);
        memcpy(p_old, p_new, sizeof(float) * (size_t)Le * V);
        if (stats) { stats->steps++; if (a <= 64) stats->accept_hist[a]++; }
    }
    if (n_acc == N - 1) out[N - 1] = draft[0];           /* pending index 0 is exact */

    free(ring); free(q0); free(logits); free(p_new); free(p_old); free(next); free(draft);
}

void orc_generate_ar(orc_forward_fn fwd, void *ctx, int32_t n_prompt, const float *logits_prompt, int32_t V,
                     int32_t lo, int32_t N, const orc_sampler *smp, const orc_init *init, uint64_t seed,
                     int32_t *out)
{
    float *q = (float *)malloc(sizeof(float) * (size_t)V);
    float *logits = (float *)malloc(sizeof(float) * (size_t)V);
    uint32_t w4[4];
    orc_dist(logits_prompt, V, smp->top_k, smp->temperature, forced_index(init, 0, lo), q);
    orc_draw(seed, 0, 0, w4);
    out[0] = orc_sample(q, V, w4[2]) + lo;
    for (int32_t c = 1; c < N; ++c) {
        fwd(ctx, n_prompt + c - 1, &out[c - 1], 1, logits);
        orc_dist(logits, V, smp->top_k, smp->temperature, forced_index(init, c, lo), q);
        orc_draw(seed, (uint64_t)c, 1, w4);
        out[c] = orc_sample(q, V, w4[2]) + lo;
    }
    free(logits); free(q);
}

/* transformer-backed model callback */
void orc_tf_forward(void *vctx, int32_t n_fixed, const int32_t *tokens, int32_t L, float *logits)
{
    orc_tf_ctx *c = (orc_tf_ctx *)vctx;
    double *x = (double *)malloc(sizeof(double) * (size_t)L * c->m->cfg.d_model);
    orc_embed(c->m, tokens, L, x);
    orc_kv_set_len(c->kv, n_fixed);
    orc_forward_window(c->m, c->kv, x, L, logits);
    free(x);
}

void orc_tf_prefill(orc_tf_ctx *c, const int32_t *ids, int32_t n_ids, const float *embeds, int32_t n_embeds,
                    float *logits_last)
{
    int32_t P = n_ids + n_embeds, d = c->m->cfg.d_model, V = c->m->cfg.samp_hi - c->m->cfg.samp_lo;
    double *x = (double *)malloc(sizeof(double) * (size_t)P * d);
    float *lg = (float *)malloc(sizeof(float) * (size_t)P * V);
    orc_embed(c->m, ids, n_ids, x);
    for (size_t e = 0; e < (size_t)n_embeds * d; ++e) x[(size_t)n_ids * d + e] = (double)embeds[e];
    orc_kv_set_len(c->kv, 0);
    orc_forward_window(c->m, c->kv, x, P, lg);
    orc_kv_set_len(c->kv, P);
    memcpy(logits_last, lg + (size_t)(P - 1) * V, sizeof(float) * (size_t)V);
    free(lg); free(x);
}

/* toy table model: logits of the next token are looked up by the whole prefix */
void orc_toy_forward(void *vctx, int32_t n_fixed, const int32_t *tokens, int32_t L, float *logits)
{
    orc_toy_ctx *c = (orc_toy_ctx *)vctx;
    for (int32_t s = 0; s < L; ++s) {
        if (n_fixed + s < 16) c->fixed[n_fixed + s] = tokens[s];
        int32_t len = n_fixed + s + 1; /* prefix length that conditions row s */
        float *row = logits + (size_t)s * c->V;
        if (len >= c->depth) { for (int32_t t = 0; t < c->V; ++t) row[t] = 0.0f; continue; }
        size_t off = 0, pw = 1, idx = 0;
        for (int32_t k = 0; k < len; ++k) { off += pw; pw *= (size_t)c->V; }
        for (int32_t k = 0; k < len; ++k) idx = idx * (size_t)c->V + (size_t)c->fixed[k];
        memcpy(row, c->table + (off + idx) * (size_t)c->V, sizeof(float) * (size_t)c->V);
    }
}

void orc_toy_histogram(const float *table, int32_t V, int32_t depth, int32_t L, const orc_sampler *smp,
                       const orc_init *init, uint64_t seed0, int64_t runs, int32_t use_ar, int64_t *hist,
                       int64_t *total_steps)
{
    int64_t cells = 1;
    for (int32_t k = 0; k < depth; ++k) cells *= V;
    for (int64_t i = 0; i < cells; ++i) hist[i] = 0;
    int64_t steps = 0;
    for (int64_t r = 0; r < runs; ++r) {
        orc_toy_ctx ctx;
        ctx.V = V; ctx.depth = depth; ctx.table = table;
        int32_t out[16];
        orc_stats st;
        if (use_ar) orc_generate_ar(orc_toy_forward, &ctx, 0, table, V, 0, depth, smp, init, seed0 + (uint64_t)r, out);
        else {
            orc_generate_sjd(orc_toy_forward, &ctx, 0, table, V, 0, depth, L, smp, init, seed0 + (uint64_t)r, out, &st);
            steps += st.steps;
        }
        int64_t idx = 0;
        for (int32_t k = 0; k < depth; ++k) idx = idx * V + out[k];
        hist[idx]++;
    }
    if (total_steps) *total_steps = steps;
}
