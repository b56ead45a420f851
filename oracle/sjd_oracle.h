/* CPU oracle for Speculative Jacobi Decoding (SJD) -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of what the GPU hot path
 * computes: a Llama-style decoder forward in fp64 and the SJD iteration
 * (Sec. 4.1, Steps 1-4; Eqs. 1-3).  It shares no code with the HIP library
 * and must never be linked, imported or called from the product path; only
 * the tests, the smoke check and the CPU-baseline leg of the benchmark use it.
 *
 * Where the paper is silent (sampler mechanics, random numbers, tie-breaks,
 * the arithmetic of the softmax) the oracle takes one fixed reading, stated at
 * each function, chosen so that every data-dependent decision is an integer
 * comparison or a single correctly-rounded fp32 operation.
 */
#ifndef SJD_ORACLE_H
#define SJD_ORACLE_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int32_t orc_num_threads(void);

/* ---- random numbers: Philox4x32-10 (Salmon et al., SC'11) ------------------------- */
void orc_philox4x32_10(const uint32_t key[2], const uint32_t ctr[4], uint32_t out[4]);
/* the four words drawn for (seed, step counter c, window index i): acc, res, smp, init */
void orc_draw(uint64_t seed, uint64_t c, uint32_t i, uint32_t out[4]);
float orc_u_acc(uint32_t word);                 /* top 24 bits -> [0, 1-2^-24] */

/* guided logits of classifier-free guidance: out = z_uncond + w * (z_cond - z_uncond) */
void orc_guide(const float *z_cond, const float *z_uncond, float w, int64_t n, float *out);

/* ---- sampler pieces ---------------------------------------------------------------- */
float orc_exp(float x);                         /* the fixed fp32 exp recipe, x <= 0 */

/* dist(): logits row over the sampling vocabulary -> probabilities q[V]  (Sec. 3.1:
 * softmax classifier + top-K sampling).  forced >= 0 makes q one-hot at that index.   */
void orc_dist(const float *z, int32_t V, int32_t top_k, float temperature, int32_t forced, float *q);

/* fixed-point inverse-CDF sample from non-negative weights w[V]; returns the index, or
 * -1 when every weight quantises to zero.                                               */
int32_t orc_sample(const float *w, int32_t V, uint32_t k32);

typedef struct {
    int32_t top_k;
    float temperature;
} orc_sampler;

typedef struct {
    int32_t mode;        /* 0 uniform, 1 repeat the token one grid row above, 2 repeat the left token,
                            3 sample from the left slot's distribution, 4 from the one a grid row above */
    int32_t row_stride;  /* image tokens per grid row (incl. a row-end token) */
    int32_t eol_id;      /* token id forced at the last position of a row, -1 = none */
    int32_t flags;       /* bit 0: no refinement (unaccepted drafts are replaced by new slots) */
} orc_init;

/* One SJD verification (Sec. 4.1 Step 3 + Step 4) from precomputed distributions.
 *   q      [(L+1) x V]  row i = distribution of window index i from THIS iteration
 *                       (row 0 is ignored: index 0 is exact by construction; row L = bonus)
 *   p_old  [L x V]      distributions the drafts were drawn from
 *   draft  [L]          token ids (global ids, lo <= id < lo+V)
 *   hist   [img_pos0]   image tokens accepted so far (needed by repeat-above init)
 *   ring   [row_stride x V]  mode 4 only (else may be NULL), in/out: distribution recorded for the
 *                       accepted position p at entry p % row_stride; this call adds its accepted ones
 * Outputs: new_draft[L], p_new[L x V] in next-window layout; returns n_accepted in [1, L]. */
int32_t orc_verify_probs(const float *q, const float *p_old, const int32_t *draft, int32_t L, int32_t V,
                         int32_t lo, const orc_init *init, int32_t img_pos0, const int32_t *hist,
                         uint64_t seed, uint64_t counter, float *ring, int32_t *new_draft, float *p_new);

/* Same from logits: logits[L x V], row s belongs to window index s+1. */
int32_t orc_verify(const float *logits, const float *p_old, const int32_t *draft, int32_t L, int32_t V,
                   int32_t lo, const orc_sampler *smp, const orc_init *init, int32_t img_pos0,
                   const int32_t *hist, uint64_t seed, uint64_t counter, float *ring, int32_t *new_draft,
                   float *p_new);

/* Initial window (step counter 0): slot 0 ~ q_first, slots 1.. by the init strategy. */
void orc_first_window(const float *q_first, int32_t L, int32_t V, int32_t lo, const orc_init *init,
                      uint64_t seed, int32_t *draft, float *p_old);

/* ---- the model: Llama-style decoder, fp64 arithmetic ----------------------------- */
typedef struct {
    int32_t n_layers, d_model, n_heads, d_ffn;
    int32_t vocab_total, samp_lo, samp_hi;
    int32_t max_seq;
    int32_t dtype;                 /* 0: blob is fp32, 1: blob is bf16 bit patterns */
    float rope_theta, rms_eps;
} orc_config;

typedef struct orc_model orc_model;  /* config + borrowed pointer to the weight blob */
typedef struct orc_kv orc_kv;        /* fp64 K/V rows [layer][pos][d] + length        */

orc_model *orc_model_create(const orc_config *cfg, const void *blob);
void orc_model_free(orc_model *m);
orc_kv *orc_kv_create(const orc_model *m);
void orc_kv_free(orc_kv *kv);
void orc_kv_set_len(orc_kv *kv, int32_t n);
int32_t orc_kv_len(const orc_kv *kv);

/* Plain definition: causal forward over a whole sequence, no cache.  x_in [T x d] fp64
 * input embeddings (see orc_embed); logits [T x V_s] fp32.                             */
void orc_forward_full(const orc_model *m, const double *x_in, int32_t T, float *logits);

/* Window forward against the cache: rows at positions n..n+L-1 (n = cache length), their
 * K/V written to the cache; the length is NOT advanced.  logits [L x V_s].             */
void orc_forward_window(const orc_model *m, orc_kv *kv, const double *x_in, int32_t L, float *logits);

/* rows of the embedding table for ids -> x [n x d] fp64 */
void orc_embed(const orc_model *m, const int32_t *ids, int32_t n, double *x);

/* ---- decoding loops ----------------------------------------------------------------- */
/* model callback: forward `L` tokens at positions n..n+L-1 where n = tokens already fixed
 * (prompt + accepted); must leave the first n positions' state intact; logits [L x V].   */
typedef void (*orc_forward_fn)(void *ctx, int32_t n_fixed, const int32_t *tokens, int32_t L, float *logits);

typedef struct {
    int32_t steps;            /* window forwards */
    int32_t accept_hist[65];  /* accept_hist[a] = #steps that accepted a tokens */
} orc_stats;

/* SJD generation of N image tokens after a prompt of n_prompt fixed positions whose last
 * logits row is logits_prompt[V].  out[N].                                             */
void orc_generate_sjd(orc_forward_fn fwd, void *ctx, int32_t n_prompt, const float *logits_prompt, int32_t V,
                      int32_t lo, int32_t N, int32_t L, const orc_sampler *smp, const orc_init *init,
                      uint64_t seed, int32_t *out, orc_stats *stats);

/* Independent ordinary autoregressive sampling with the same random words. */
void orc_generate_ar(orc_forward_fn fwd, void *ctx, int32_t n_prompt, const float *logits_prompt, int32_t V,
                     int32_t lo, int32_t N, const orc_sampler *smp, const orc_init *init, uint64_t seed,
                     int32_t *out);

/* transformer-backed callback context */
typedef struct {
    const orc_model *m;
    orc_kv *kv;
} orc_tf_ctx;
void orc_tf_forward(void *ctx, int32_t n_fixed, const int32_t *tokens, int32_t L, float *logits);
/* prefill ids then embedding rows; returns logits of the last position in logits_last[V_s] */
void orc_tf_prefill(orc_tf_ctx *c, const int32_t *ids, int32_t n_ids, const float *embeds, int32_t n_embeds,
                    float *logits_last);

/* toy table model: vocab V, logits depend on the whole token prefix (max length depth) */
typedef struct {
    int32_t V, depth;
    const float *table;     /* [sum_{k=0..depth-1} V^k][V] logits, prefix-major          */
    int32_t fixed[16];      /* tokens fixed so far (image tokens only; prompt is empty)   */
} orc_toy_ctx;
void orc_toy_forward(void *ctx, int32_t n_fixed, const int32_t *tokens, int32_t L, float *logits);

/* Monte-Carlo over seeds seed0..seed0+runs-1 on the toy model: histogram of complete
 * length-`depth` outputs (V^depth cells), SJD with window L (use_ar != 0: the AR loop). */
void orc_toy_histogram(const float *table, int32_t V, int32_t depth, int32_t L, const orc_sampler *smp,
                       const orc_init *init, uint64_t seed0, int64_t runs, int32_t use_ar, int64_t *hist,
                       int64_t *total_steps);

#ifdef __cplusplus
}
#endif
#endif
