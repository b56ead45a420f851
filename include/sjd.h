/* sjd.h -- C ABI of the MI355X (gfx950) hot path of Speculative Jacobi Decoding (SJD).
 *
 * The problem (paper Sec. 4.1, first paragraph): after the prompt has been pre-filled, decode the
 * image tokens W at a time.  Each iteration runs ONE causal forward of the auto-regressive
 * transformer over the W draft tokens (Step 2), accepts a prefix of them with the probabilistic
 * criterion of Eq. 1, resamples the first rejected position from the calibrated distribution of
 * Eq. 2, re-draws every later position from this iteration's distributions (Eq. 3), and slides the
 * window (Step 4).  By Theorem 1 every produced token is distributed exactly as under ordinary
 * auto-regressive sampling.  W is called L here.
 *
 * Conventions
 *  - Every function returns SJD_OK (0) or a negative SJD_E* code; nothing aborts or throws.
 *  - "dev" pointers are device (HBM) addresses on the current HIP device, "host" pointers are
 *    ordinary host memory.  The caller owns every buffer it passes; the library owns only its
 *    opaque handles.  Buffers must not overlap unless stated.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device work is
 *    enqueued on it and is asynchronous; outputs are valid once the caller has synchronised.
 *  - Probabilities and logits are fp32 rows over the SAMPLING vocabulary: column t stands for
 *    token id samp_lo + t, V_s = samp_hi - samp_lo columns per row.
 *  - All decisions are deterministic functions of the inputs: identical calls give identical bits.
 *  - Threads: a model is read-only once built; a cache handle (sjd_kv) is used by one host thread at a
 *    time.  Different handles of one model may be driven from different host threads on different streams
 *    at the same time (the handles of one batched call belong to that call).
 */
#ifndef SJD_H
#define SJD_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SJD_OK 0
#define SJD_EINVAL (-1) /* bad argument (null pointer, size out of range, unsupported shape)   */
#define SJD_ENOMEM (-2) /* device or host allocation failed                                    */
#define SJD_ESEQ (-3)   /* the call would run past max_seq                                     */
#define SJD_EHIP (-4)   /* a HIP runtime call failed; sjd_strerror() reports the last message  */
#define SJD_ELIMIT (-5) /* a size exceeds a fixed limit of the entry point; sjd_strerror() says which */

#define SJD_MAX_WINDOW 64     /* largest L accepted by sjd_step / sjd_generate                 */
#define SJD_MAX_ROWS 128      /* rows one window forward computes: L x contexts (2 under guidance) x
                                 images of a batch, each image's rows rounded up to a power of two  */
#define SJD_MAX_SAMP_VOCAB 32768 /* largest V_s the verification kernels hold in LDS          */

typedef struct sjd_model sjd_model; /* repacked device weights + tables; immutable after init  */
typedef struct sjd_kv sjd_kv;       /* KV cache, its length n, ids of the cached tokens, scratch */

/* Llama-style decoder (the paper fixes no architecture; Sec. 3.1 only requires an
 * auto-regressive transformer with a softmax classifier over the token vocabulary).          */
typedef struct {
    int32_t n_layers, d_model, n_heads, d_ffn;
    int32_t vocab_total, samp_lo, samp_hi; /* sampling ids = [samp_lo, samp_hi)                */
    int32_t max_seq;                       /* KV rows; needs prompt + N + L                    */
    int32_t dtype;                         /* 0 = fp32 throughout; 1 = bf16 weights, activations
                                              and cache as bf16 operand pairs hi + lo (about 16
                                              significant bits), fp32 accumulation             */
    float rope_theta, rms_eps;
} sjd_config;

/* top-K sampling (Sec. 3.1).  temperature == 0 or top_k == 1 selects greedy decoding, which
 * turns SJD into the deterministic Jacobi iteration of Sec. 3.2.                              */
typedef struct {
    int32_t top_k;
    float temperature;
} sjd_sampler;

/* Initialisation of new window slots (Sec. 4.2).  mode 0: uniform over the sampling ids;
 * mode 1: strategy (b), repeat the token one grid row above (uniform in the first grid row);
 * mode 2: strategy (a), repeat the token at the previous raster position;
 * mode 3: strategy (c), a fresh draw from the distribution on record for the nearest slot to the left
 *         that is not a forced row end (a run of new slots all draw from the last model row);
 * mode 4: strategy (d), a fresh draw from the distribution on record for the position one grid row
 *         up (the cache handle keeps the distributions of the last row_stride accepted positions;
 *         uniform in the first grid row).  The row drawn from is the slot's row in Eq. 1.
 * eol_id >= 0 forces that id at the last position of every grid row.
 * flags bit 0 (SJD_INIT_NO_REFINE): the ablation without refinement (App. "acceleration originates
 * from the refinement"): only the resampled position survives an iteration, every later slot of the
 * next window is newly initialised instead of re-drawn by Eq. 3.                                */
#define SJD_INIT_NO_REFINE 1
typedef struct {
    int32_t mode;
    int32_t row_stride; /* image tokens per grid row, a row-end token included                 */
    int32_t eol_id;
    int32_t flags;
} sjd_init;

typedef struct {
    int32_t steps;           /* window forwards (the paper's "decoding steps", Sec. 5.1)        */
    int32_t accept_hist[65]; /* accept_hist[a] = number of steps that accepted a tokens         */
    float ms_prefill;        /* host wall-clock of the prefill, milliseconds                    */
    float ms_decode;         /* host wall-clock of the decoding loop (all steps), milliseconds  */
} sjd_stats;

/* ---- model and cache ---------------------------------------------------------------------- */
/* host_weights: flat blob, element type per cfg->dtype (fp32, or bf16 bit patterns), tensors in
 * the order E[vocab,d]; per layer g1[d] Wq Wk Wv Wo [d,d] g2[d] Wg Wu [F,d] Wd [d,F]; gf[d];
 * Wlm[vocab,d]; every matrix row-major [out][in].  The blob is copied and repacked; the pointer
 * is not retained.  nbytes must match the configuration exactly (else SJD_EINVAL).            */
int sjd_init_model(const sjd_config *cfg, const void *host_weights, size_t nbytes, sjd_model **out);
void sjd_free_model(sjd_model *m);

int sjd_kv_create(const sjd_model *m, sjd_kv **out);
void sjd_kv_free(sjd_kv *kv);
int sjd_kv_reset(sjd_kv *kv);                     /* n = 0                                       */
int sjd_kv_len(const sjd_kv *kv, int32_t *n);     /* synchronises the device, then reads n       */
int sjd_kv_set_len(sjd_kv *kv, int32_t n);        /* roll the cache back/forward to n rows (resume) */

/* ---- the path ----------------------------------------------------------------------------- */
/* Pre-fill the prompt (Sec. 4.1 "after pre-filling the tokens of text prompts"): n_ids token ids
 * (host) followed by n_embeds raw embedding rows (host fp32 [n_embeds x d_model]); either may be
 * empty, not both.  Resets the cache, leaves n = n_ids + n_embeds, and writes
 * q_last (dev [V_s]) = the sampling distribution of the first image token.                     */
int sjd_prefill(sjd_model *m, sjd_kv *kv, const int32_t *ids, int32_t n_ids, const float *embeds,
                int32_t n_embeds, const sjd_sampler *smp, const sjd_init *init, float *q_last, void *stream);

/* Classifier-free guidance (Sec. 5.1 runs its text-to-image models with guidance weight 3; the
 * mechanism is the usual one in logit space): right after sjd_prefill, pre-fill a second,
 * unconditional prompt into a second cache of the same handle.  From then on every window forward
 * runs both contexts on the same draft tokens (one pass over the weights, 2 x L rows) and Step 3
 * works on z = z_uncond + guidance * (z_cond - z_uncond); both caches advance by the accepted
 * count.  q_last is overwritten with the guided distribution of the first image token.  Windows go
 * up to SJD_MAX_WINDOW tokens with guidance on as well (two contexts x 64 rows = SJD_MAX_ROWS; fp32
 * models: 32); the next sjd_prefill switches it off.                                             */
int sjd_prefill_uncond(sjd_model *m, sjd_kv *kv, const int32_t *ids, int32_t n_ids, const float *embeds,
                       int32_t n_embeds, float guidance, const sjd_sampler *smp, const sjd_init *init, float *q_last,
                       void *stream);

/* First Jacobi window (Sec. 4.1 "starts with a sequence of initialized candidate tokens"):
 * slot 0 is sampled from q_first (dev [V_s]) and carries it as its distribution; slots 1..L-1
 * follow `init`.  Uses step counter 0.  draft dev [L], p_old dev [L x V_s].                   */
int sjd_first_window(const sjd_model *m, const float *q_first, int32_t L, const sjd_init *init,
                     uint64_t philox_seed, int32_t *draft, float *p_old, void *stream);

/* One SJD iteration (Sec. 4.1 Steps 1-4) on the window that starts at cache length n:
 *   draft   dev [L]        token ids of the window (Step 1)
 *   p_old   dev [L x V_s]  the distribution each draft was drawn from; row 0 must be the exact
 *                          conditional of draft[0] (it is never re-verified)
 *   img_pos0               image index of draft[0] (decides row ends and the row above)
 *   philox_seed, counter   random stream: Philox4x32-10 keyed by the seed, counter = (counter,
 *                          window index); counter 0 belongs to sjd_first_window
 * Outputs (dev): n_accepted[1] in [1, L]; new_draft[L] and p_new[L x V_s] already in the layout
 * of the next window (unaccepted positions first, then newly initialised slots).  new_draft may
 * alias draft and p_new may alias p_old.  The cache length advances by n_accepted and the ids of
 * the accepted tokens are recorded in the cache.  SJD_ESEQ if n + L > max_seq.                 */
int sjd_step(sjd_model *m, sjd_kv *kv, const int32_t *draft, const float *p_old, int32_t L,
             const sjd_sampler *smp, const sjd_init *init, int32_t img_pos0, uint64_t philox_seed,
             uint64_t counter, int32_t *n_accepted, int32_t *new_draft, float *p_new, void *stream);

/* Whole generation: prefill, first window, then iterations until N image tokens are fixed.
 * out_tokens host [N]; stats may be NULL.  Runs on the default stream and synchronises.        */
int sjd_generate(sjd_model *m, sjd_kv *kv, const int32_t *ids, int32_t n_ids, const float *embeds,
                 int32_t n_embeds, int32_t N, int32_t L, const sjd_sampler *smp, const sjd_init *init,
                 uint64_t philox_seed, int32_t *out_tokens, sjd_stats *stats);

/* sjd_generate with classifier-free guidance: both prompts, then the guided loop.                */
int sjd_generate_cfg(sjd_model *m, sjd_kv *kv, const int32_t *ids, int32_t n_ids, const float *embeds,
                     int32_t n_embeds, const int32_t *uncond_ids, int32_t n_uncond_ids, const float *uncond_embeds,
                     int32_t n_uncond_embeds, float guidance, int32_t N, int32_t L, const sjd_sampler *smp,
                     const sjd_init *init, uint64_t philox_seed, int32_t *out_tokens, sjd_stats *stats);

/* The same loop in pieces, with the loop state (cache length, image position, Philox counter,
 * window, its distributions) resident on the device so that iterations can be enqueued without
 * waiting for the outcome of the previous one (Sec. 4.1: the accepted count of Step 3 decides
 * where the next window starts, which is a data dependence, not a host decision).
 *   sjd_decode_begin   after sjd_prefill: first window from q_first (dev [V_s]), counters reset.
 *   sjd_decode_steps   enqueue n_steps iterations on `stream` (one HIP-graph replay each);
 *                      an iteration that starts after the N-th token is fixed changes nothing
 *                      (its forward still runs, on rows nobody reads: do not enqueue far past
 *                      the end; an iteration fixes at most L tokens).
 *   sjd_decode_status  synchronise; image tokens fixed so far, iterations run, finished flag.
 *   sjd_decode_result  after `done`: the N tokens (host) and the step statistics.
 *   sjd_kv_use_graph   0: launch kernels one by one instead of replaying a captured graph.     */
int sjd_decode_begin(sjd_model *m, sjd_kv *kv, const float *q_first, int32_t N, int32_t L,
                     const sjd_sampler *smp, const sjd_init *init, uint64_t philox_seed, void *stream);
int sjd_decode_steps(sjd_model *m, sjd_kv *kv, int32_t n_steps, void *stream);
int sjd_decode_status(sjd_kv *kv, int32_t *n_fixed, int32_t *steps, int32_t *done);
int sjd_decode_result(sjd_kv *kv, int32_t *out_tokens, sjd_stats *stats);
int sjd_kv_use_graph(sjd_kv *kv, int32_t on);

/* Per-kernel-class timing: runs n_steps iterations of the loop above kernel by kernel, every launch
 * carrying a start/stop HIP event pair that the runtime stamps with the kernel's own begin and end
 * (on `stream`), and adds up milliseconds, launch counts and HBM bytes (weights for the
 * projections; for attention the K/V records, as stored -- hi and lo halves, twice the bf16 size --
 * of the positions each profiled step really attended over; logits + both probability windows for
 * the verification) per class.  The per-launch intervals include a few microseconds of dispatch latency each, so the
 * projections (the dominant class) are timed a second time: the projection launches of n_steps
 * iterations alone, back to back in one event interval (ms_gemm_back_to_back; the same number of
 * launches and bytes as in the per-launch pass).  Synchronises.                                */
#define SJD_PROF_GEMM 0        /* QKV / O / gate-up / down projections and the LM head           */
#define SJD_PROF_ATTENTION 1   /* window attention incl. the merge of its key chunks             */
#define SJD_PROF_ELEMENTWISE 2 /* embedding, RMSNorm, RoPE + cache write, SiLU*up, reductions    */
#define SJD_PROF_VERIFY 3      /* Sec. 4.1 Step 3 + Step 4 kernels                               */
typedef struct {
    double ms[4];
    double bytes[4];
    int64_t launches[4];
    int32_t steps;
    double ms_gemm_back_to_back;
} sjd_profile;
int sjd_profile_steps(sjd_model *m, sjd_kv *kv, int32_t n_steps, sjd_profile *out, void *stream);
/* the same for iterations of sjd_decode_steps_batch */
int sjd_profile_steps_batch(sjd_model *m, sjd_kv *const *kvs, int32_t B, int32_t n_steps, sjd_profile *out,
                            void *stream);

/* ---- batched decoding --------------------------------------------------------------------------
 * B independent images share every window forward (Sec. 4.1 Step 2 for B windows at once): one pass
 * over the weights serves B x L rows, so an iteration costs little more than for one image and the
 * throughput grows almost B-fold.  Each image keeps its own handle (cache, loop state, random
 * stream); Steps 3 and 4 run per image exactly as in sjd_decode_steps.  bf16 models.  Guidance: all
 * handles guided (each after its own sjd_prefill_uncond, each with its own weight) or none; a guided
 * image brings two contexts.  The contexts' windows (each rounded up to a power of two of rows) must
 * fit the SJD_MAX_ROWS rows of one forward, at most 8 contexts: L <= 64 for 2 contexts, L <= 32 for
 * up to 4, L <= 16 for up to 8.  The first handle lends its activation buffers and, with graphs on,
 * holds the captured iteration (re-captured when the set of handles or their settings change).
 *
 * sjd_decode_steps_batch: every handle has been through sjd_prefill (+ sjd_prefill_uncond) +
 * sjd_decode_begin with the same L, sampler and initialiser (seeds may differ); poll and collect per handle with
 * sjd_decode_status / sjd_decode_result.  A handle whose image is complete sits out further
 * iterations.  kvs: host array of B distinct handles.                                          */
int sjd_decode_steps_batch(sjd_model *m, sjd_kv *const *kvs, int32_t B, int32_t n_steps, void *stream);

/* Prompts to images for B handles, without guidance (it pre-fills every handle anew; guided batches go
 * through the pieces above).  ids / embeds: host arrays of B host pointers (embeds and
 * n_embeds may be NULL), out_tokens host [B x N], stats host [B] or NULL (times are the batch's). */
int sjd_generate_batch(sjd_model *m, sjd_kv *const *kvs, int32_t B, const int32_t *const *ids, const int32_t *n_ids,
                       const float *const *embeds, const int32_t *n_embeds, int32_t N, int32_t L,
                       const sjd_sampler *smp, const sjd_init *init, const uint64_t *philox_seeds, int32_t *out_tokens,
                       sjd_stats *stats);

/* ---- pieces of the step, exported for parity tests and profiling --------------------------- */
/* Step 2 alone: forward `L` tokens (dev ids) at positions n..n+L-1, write their K/V rows, return
 * logits dev [L x V_s] fp32 (the guided logits while guidance is on).  Does not advance n.     */
int sjd_forward_logits(sjd_model *m, sjd_kv *kv, const int32_t *tokens, int32_t L, float *logits, void *stream);

/* The same for B handles in one forward: tokens dev [B x L], logits dev [B x L x V_s] (of guided handles:
 * the guided logits).  A handle
 * inside a generation (sjd_decode_begin) whose image is complete is skipped: its rows of `logits`
 * are left as they are.                                                                          */
int sjd_forward_logits_batch(sjd_model *m, sjd_kv *const *kvs, int32_t B, const int32_t *tokens, int32_t L,
                             float *logits, void *stream);

/* Step 3 + Step 4 alone, from logits (row s belongs to window index s+1).  hist: dev ids of the
 * image tokens fixed so far [img_pos0] (may be NULL when init->mode is 0 or 3, or img_pos0 == 0).
 * ring: dev [row_stride x V_s], in/out, init->mode == 4 only (else may be NULL): entry p % row_stride
 * holds the distribution on record for accepted image position p; the call adds the positions it
 * accepts.  V_s <= SJD_MAX_SAMP_VOCAB.                                                          */
int sjd_verify(const float *logits, const float *p_old, const int32_t *draft, int32_t L, int32_t V_s,
               int32_t samp_lo, const sjd_sampler *smp, const sjd_init *init, int32_t img_pos0,
               const int32_t *hist, float *ring, uint64_t philox_seed, uint64_t counter, int32_t *n_accepted,
               int32_t *new_draft, float *p_new, void *stream);

/* Same from precomputed distributions q dev [(L+1) x V_s] (row 0 ignored, row L = the bonus
 * distribution of the position just past the window).                                          */
int sjd_verify_probs(const float *q, const float *p_old, const int32_t *draft, int32_t L, int32_t V_s,
                     int32_t samp_lo, const sjd_init *init, int32_t img_pos0, const int32_t *hist, float *ring,
                     uint64_t philox_seed, uint64_t counter, int32_t *n_accepted, int32_t *new_draft,
                     float *p_new, void *stream);

/* sjd_verify for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, same outputs, but the scratch that
 * sjd_verify allocates per call (the distributions of the L + 1 window indices, candidates, flags)
 * lives in a static device array of the library, SJD_STATIC_VERIFY_FLOATS floats (1.06 MiB, held on
 * every GPU the library runs on until the process ends).  The call allocates nothing, frees nothing
 * and does not synchronise: outputs are valid once `stream` has been synchronised.  SJD_ELIMIT when
 * (L + 1) * V_s exceeds SJD_STATIC_VERIFY_FLOATS (the 7B and 775M workloads fit: 33 x 8192 and
 * 17 x 16384).  Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two
 * streams, two threads) race; run them one after the other.                                      */
#define SJD_STATIC_VERIFY_FLOATS (17 * 16384)
int sjd_verify_static(const float *logits, const float *p_old, const int32_t *draft, int32_t L, int32_t V_s,
                      int32_t samp_lo, const sjd_sampler *smp, const sjd_init *init, int32_t img_pos0,
                      const int32_t *hist, float *ring, uint64_t philox_seed, uint64_t counter, int32_t *n_accepted,
                      int32_t *new_draft, float *p_new, void *stream);

/* The sampling distribution of Sec. 3.1 for `rows` logits rows: top-K, temperature, softmax.
 * forced: dev [rows] column index to make one-hot, or -1; may be NULL.  q dev [rows x V_s].     */
int sjd_dist(const float *logits, int32_t rows, int32_t V_s, const sjd_sampler *smp, const int32_t *forced,
             float *q, void *stream);

/* C[M x N] (fp32, dev) = A[M x K] * W[N x K]^T with the kernel the model uses for its projections.
 * dtype as in sjd_config; A and W are dev, row-major, element type per dtype; W is repacked into
 * the library's streaming layout first (not timed separately).  dtype 2: W bf16 and A fp32, A taken
 * through the 3-byte form (16 significant bits) in which bf16 models hand the attention output and
 * the FFN hidden to their projections.  For kernel-level parity tests.                            */
int sjd_gemm_test(int32_t dtype, const void *A, const void *W, int32_t M, int32_t N, int32_t K, float *C,
                  void *stream);

/* Tuning aid: average microseconds per launch of the bf16 projection kernel (plain-store epilogue) at
 * shape M x N x K over `iters` back-to-back launches on zero-filled operands (activations in the
 * 3-byte form the model's projections read).  `tn` = output tiles
 * per workgroup (1..3), wk = waves splitting K (8 or 4; 0 = the choice the model makes), u = k-steps per
 * prefetch stage (2; 4 for wk = 4, M <= 16; 0 = the choice the model makes).
 * More than 32 rows run the wide kernel (waves split N and share the activations through LDS, K split
 * across workgroups, a second kernel adds the slices): then wk = K-slices and u = weight groups per wave
 * (0 = automatic); wk >= 100 asks for the wide kernel at any row count, with wk - 100 K-slices.  M above
 * SJD_MAX_ROWS is an off-path measurement of the wide kernel's matrix-core rate: the rows are cut into
 * chunks of SJD_MAX_ROWS, one launch pair each over the same weights.
 * A negative `iters` times |iters| launches that rotate through more than 1 GiB of weight copies,
 * so that no launch finds its weights in the last-level cache (the situation inside a step).
 * tn = 0 measures the floor instead of the projection: a kernel that only reads the same N x K x 2 bytes
 * (wk workgroups of 256 threads, 0 = 256, four 16-byte loads per lane in flight; u = 0: every workgroup a
 * contiguous share, as the projection kernels read their packed weights; u = 1: all workgroups sweep the bytes
 * together, 4 KiB per wave and round).
 * SJD_EINVAL for an unsupported combination.                                                     */
int sjd_gemm_bench(int32_t M, int32_t N, int32_t K, int32_t tn, int32_t wk, int32_t u, int32_t iters,
                   float *us_per_launch);

const char *sjd_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif
