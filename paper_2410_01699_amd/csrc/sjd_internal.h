// Internal declarations of the SJD HIP library (gfx950 only).  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "sjd.h"

#define SJD_ROWS_MAX SJD_MAX_ROWS       // rows (window slots of all streams, or a prefill chunk) one forward pass handles
#define SJD_MTILES (SJD_ROWS_MAX / 16)  // 16-row tiles of an activation matrix
#define SJD_ROWS_SKINNY 32              // up to here the skinny projection kernel runs, above it the wide one
#define SJD_LO16_FROM_ROWS 33           // forwards with at least this many rows keep the 2-byte lo plane (see sjd_api.hip)
#define SJD_ROWS_F32 32                 // fp32 models (launch-bound toys): rows per forward, largest window

typedef unsigned short bf16_t;  // raw bf16 bit pattern

// ---- error plumbing ------------------------------------------------------------------------
void sjd_set_hip_error(hipError_t e, const char *what);
#define HIP_TRY(expr)                              \
    do {                                           \
        hipError_t e_ = (expr);                    \
        if (e_ != hipSuccess) {                    \
            sjd_set_hip_error(e_, #expr);          \
            return SJD_EHIP;                       \
        }                                          \
    } while (0)
#define SJD_TRY(expr)                \
    do {                             \
        int rc_ = (expr);            \
        if (rc_ != SJD_OK) return rc_; \
    } while (0)

// ---- kernel launches -------------------------------------------------------------------------
// Every kernel of the path is launched through SJD_LAUNCH.  While sjd_profile_steps() runs, a hook
// hands each launch a start/stop event pair, or lets only the launches of one kernel class through
// (the others are skipped, so that one class can be timed back to back); otherwise it is a plain
// launch.
struct SjdLaunchHook {
    int (*next)(void *self, hipEvent_t *start, hipEvent_t *stop);   // NULL: no per-launch events
    void *self;
    int cur_kind;       // class of the launches being issued (set by the orchestration)
    int only_kind;      // >= 0: skip every launch of another class
};
extern thread_local SjdLaunchHook *sjd_launch_hook;
#define SJD_LAUNCH(kernel, grid, block, lds, stream, ...)                                            \
    do {                                                                                             \
        hipEvent_t ps_ = nullptr, pe_ = nullptr;                                                     \
        if (sjd_launch_hook) {                                                                       \
            if (sjd_launch_hook->only_kind >= 0 && sjd_launch_hook->only_kind != sjd_launch_hook->cur_kind) break; \
            if (sjd_launch_hook->next) (void)sjd_launch_hook->next(sjd_launch_hook->self, &ps_, &pe_); \
        }                                                                                            \
        if (ps_) hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, ps_, pe_, 0, __VA_ARGS__);  \
        else hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                      \
    } while (0)

// ---- device helpers shared by kernels ------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (bf16_t)((u >> 16) | 0x40);  // NaN stays NaN
    u += 0x7FFFu + ((u >> 16) & 1u);                                         // round to nearest even
    return (bf16_t)(u >> 16);
}

// Device-resident decoding state: everything that changes from step to step, so that a step can
// be enqueued (or replayed from a graph) without the host knowing the outcome of the last one.
struct SjdState {
    int32_t n;          // cache length (prompt + accepted tokens)
    int32_t img_pos0;   // image index of window slot 0
    int32_t L_eff;      // slots of the window in use this step
    int32_t reserved0;
    uint64_t counter;   // Philox step counter
    int32_t n_image;    // N, image tokens to produce (generate loop; 0 = unbounded single steps)
    int32_t done;       // generation finished: later steps leave the state and the tokens alone
    int32_t steps;      // window forwards executed
    int32_t accept_hist[65];
    int32_t n_u;        // length of the second (unconditional) cache when guidance is on
    int32_t err;        // set by a kernel that was handed bad device-side input (SJD_DEVERR_*); the calls that
                        // read the state report it as SJD_EINVAL, sjd_kv_reset / sjd_prefill clear it
};
#define SJD_DEVERR_TOKEN_ID 1   // a token id outside [0, vocab_total) reached the embedding (its row was taken as zero)
#define SJD_DEVERR_IMG_POS 2    // sjd_step with img_pos0 beyond the cache length (the step was not executed)
// Two token streams share one window forward when classifier-free guidance is on: stream 0 is the
// conditional context (cache length n), stream 1 the unconditional one (cache length n_u).
__device__ __forceinline__ int state_n(const SjdState *st, int stream) { return stream ? st->n_u : st->n; }

// Token streams that share one window forward of a bf16 model: the two contexts of one image under
// classifier-free guidance, or one context per image in batched decoding.  Stream s owns rows
// [s << shift, (s + 1) << shift) of every activation matrix (count << shift <= SJD_ROWS_MAX), has its own cache
// and its own cache length; the weights are streamed once for all of them.
#define SJD_MAX_STREAMS 8
struct SjdStreamEntry {
    const int32_t *n;       // device: the stream's cache length
    const int32_t *done;    // device: its generation has finished (attention skips the stream)
    bf16_t *kvc;            // its cache, layer 0 (kernels add the layer offset)
};
// Passed to kernels by value, so it is kept small (every kernel waits for its arguments): stream 0
// travels inside, the others are looked up in a table in device memory.
struct SjdStreams {
    int32_t count;                  // 0 (no device state: kernel test hooks) .. SJD_MAX_STREAMS
    int32_t shift;                  // log2 of the rows reserved per stream
    SjdStreamEntry first;           // stream 0
    const SjdStreamEntry *table;    // device [count]: every stream (entry 0 repeats `first`); unused when count <= 1
};
// entry of stream s, s uniform across the wave
__device__ __forceinline__ SjdStreamEntry stream_entry(const SjdStreams &sm, int s)
{
    if (s == 0) return sm.first;
    return sm.table[s];
}

// Activations of bf16 models are laid out in the B-operand order of v_mfma_f32_16x16x32_bf16, so that a
// wave fetches the 16 x 32 tile of a k-step with contiguous loads.  As fp32 (the residual stream, which
// is accumulated at full precision and read and written by the residual epilogues only; the operands of
// the hooks that run the projection kernel alone): element (row m, column k) of a [SJD_ROWS_MAX x K]
// matrix lives at act_off(m, k, K/32) floats: tile (m/16, k/32) of 512 floats, inside it two halves
// (k%8 < 4, >= 4) of 64 lanes x 4 floats, lane = 16 * ((k%32)/8) + m%16.
__host__ __device__ __forceinline__ size_t act_off(int m, int k, int KT)
{
    return (((size_t)(m >> 4) * KT + (k >> 5)) * 2 + ((k >> 2) & 1)) * 256 + ((((k & 31) >> 3) * 16 + (m & 15)) << 2) + (k & 3);
}
//
// What the projections of the decoder stack stream is a 3-byte form: the fp32 value rounded to 16
// significant bits (the precision the hi + lo operand pair carries anyway), its upper 16 bits in a
// bf16 "hi" plane that IS the first MFMA operand, the next 8 bits in a byte "lo" plane from which the
// projection rebuilds the second operand.  The attention output and the FFN hidden exist in this form
// only; every writer of the residual stream also leaves the planes of x * gain of the normalisation
// that follows, plus per-token sums of squares (ssq_stride).  Every byte a projection reads passes
// through its CU's vector memory pipeline at the same cost, whether it comes from HBM or from L2, so
// a quarter less activation traffic is time saved on the shapes whose workgroups read more activation
// than weight bytes.  Plane layout for a [SJD_ROWS_MAX x K] matrix: tiles (m/16, k/32) of 512 values,
// value index act24_idx(); the hi plane holds SJD_MTILES * K/32 tiles plus one all-zero tile, the lo
// plane follows it.
__host__ __device__ __forceinline__ size_t act24_idx(int m, int k, int KT)
{
    return (((size_t)(m >> 4) * KT + (k >> 5)) << 9) + ((((k & 31) >> 3) * 16 + (m & 15)) << 3) + (k & 7);
}
__host__ __device__ __forceinline__ size_t act24_lo_base(int KT) { return (size_t)(SJD_MTILES * KT + 1) * 1024; }   // bytes
// Forwards of more than SJD_ROWS_SKINNY rows (the wide projection kernel) keep the second operand ready
// made: the lo plane then holds bf16(value - hi) (exact: 8 significant bits), 2 bytes per value in the
// same index order, so that a tile of either plane goes from L2 straight into LDS.  Same numbers, 4
// bytes per value instead of 3.  A buffer is allocated for the larger form.
__host__ __device__ __forceinline__ size_t act24_bytes(int KT) { return (size_t)(SJD_MTILES * KT + 1) * 2048; }
// fp32 -> 16 significant bits (round to nearest even), returned in fp32 position: bits 31..16 are the
// hi plane entry, bits 15..8 the lo plane entry
__device__ __forceinline__ uint32_t f32_to_act24(float x)
{
    uint32_t u = __float_as_uint(x);
    u += 0x7Fu + ((u >> 8) & 1u);
    return u & 0xFFFFFF00u;
}
// the second operand of a value in that form, as bf16 bits: value - hi (exact)
__device__ __forceinline__ uint32_t act24_lo16(uint32_t u)
{
    return __float_as_uint(__uint_as_float(u) - __uint_as_float(u & 0xFFFF0000u)) >> 16;
}
// Row length (floats) of the per-token partial sums of squares a writer of a residual matrix
// leaves, one per 16 features; padded (with zeros nobody writes) to whole float4.
__host__ __device__ __forceinline__ int ssq_stride(int K) { return (K / 16 + 3) & ~3; }
// planes of 4 consecutive values (k a multiple of 4) / of 2 (k even) of row m; lo16: the 2-byte lo plane
__device__ __forceinline__ void act24_store4(void *base, int m, int k, int KT, float v0, float v1, float v2, float v3,
                                             bool lo16)
{
    const uint32_t a = f32_to_act24(v0), b = f32_to_act24(v1), c = f32_to_act24(v2), d = f32_to_act24(v3);
    const size_t i = act24_idx(m, k, KT);
    *reinterpret_cast<uint2 *>((bf16_t *)base + i) = make_uint2((a >> 16) | (b & 0xFFFF0000u), (c >> 16) | (d & 0xFFFF0000u));
    if (lo16)
        *reinterpret_cast<uint2 *>((uint8_t *)base + act24_lo_base(KT) + 2 * i) =
            make_uint2(act24_lo16(a) | (act24_lo16(b) << 16), act24_lo16(c) | (act24_lo16(d) << 16));
    else
        *reinterpret_cast<uint32_t *>((uint8_t *)base + act24_lo_base(KT) + i) =
            ((a >> 8) & 0xFFu) | (b & 0xFF00u) | ((c << 8) & 0xFF0000u) | ((d << 16) & 0xFF000000u);
}
__device__ __forceinline__ void act24_store2(void *base, int m, int k, int KT, float v0, float v1, bool lo16)
{
    const uint32_t a = f32_to_act24(v0), b = f32_to_act24(v1);
    const size_t i = act24_idx(m, k, KT);
    *reinterpret_cast<uint32_t *>((bf16_t *)base + i) = (a >> 16) | (b & 0xFFFF0000u);
    if (lo16)
        *reinterpret_cast<uint32_t *>((uint8_t *)base + act24_lo_base(KT) + 2 * i) = act24_lo16(a) | (act24_lo16(b) << 16);
    else
        *reinterpret_cast<uint16_t *>((uint8_t *)base + act24_lo_base(KT) + i) = (uint16_t)(((a >> 8) & 0xFFu) | (b & 0xFF00u));
}
//
// KV cache of bf16 models: per layer, per head, per block of 32 positions one contiguous record of
// 128*hd bf16 values, laid out as the MFMA operands the attention kernel consumes, each value kept
// as hi = bf16(v) and lo = bf16(v - hi) (two "planes"):
//   K tiles  [h = 0,1][ks = 0..hd/32)[plane]  512 values: lane l = 16 g + c, element e holds
//            K[position 32 blk + 16 h + c][dim 32 ks + 8 g + e]             (A operand of S^T = K Q^T)
//   V tiles  [t = 0..hd/16)[plane]            512 values: lane l = 16 g + c, element e holds
//            V[position 32 blk + 16 (e/4) + 4 g + e%4][dim 16 t + c]        (A operand of O^T = V^T P)
__host__ __device__ __forceinline__ size_t kv_block_off(int head, int blk, int nblk, int hd)
{
    return ((size_t)head * nblk + blk) * (size_t)(128 * hd);
}
__host__ __device__ __forceinline__ int kv_k_off(int kk, int dim, int hd, int plane)   // kk = position % 32
{
    const int h = kk >> 4, c = kk & 15, ks = dim >> 5, g = (dim & 31) >> 3, e = dim & 7;
    return (((h * (hd >> 5) + ks) * 2 + plane) << 9) + ((g * 16 + c) << 3) + e;
}
__host__ __device__ __forceinline__ int kv_v_off(int kk, int dim, int hd, int plane)
{
    const int t = dim >> 4, c = dim & 15, g = (kk & 15) >> 2, e = ((kk >> 4) << 2) + (kk & 3);
    return 64 * hd + (((t * 2 + plane)) << 9) + ((g * 16 + c) << 3) + e;
}

// ---- one linear layer's weights ------------------------------------------------------------
// fp32 models keep W as given ([N][K] row-major).  bf16 models hold W in MFMA streaming order:
// tiles of 16 output features x 32 input features; the tn tiles a workgroup owns are interleaved
// along k, tile (nt, kt) at (((nt/tn) * K/32 + kt) * tn + nt%tn) * 512 elements, so that each wave
// reads one contiguous stream; inside a tile lane l (0..63) owns the 8 consecutive elements
// W[nt*16 + l%16][kt*32 + (l/16)*8 .. +8].
struct SjdLinear {
    const void *w;
    int32_t N, K;
    int32_t tn;       // bf16: 16-wide output tiles per workgroup
    int32_t wk;       // bf16: waves per workgroup splitting K (0 = chosen at launch)
    int32_t u;        // bf16: k-steps per prefetch stage (0 = chosen at launch)
    int32_t wg, wks;  // bf16, wide kernel (more than 32 rows): weight groups per wave, K-slices (0 = chosen at launch)
    int32_t wide_from;   // bf16: rows from which the wide kernel runs (0 = above SJD_ROWS_SKINNY)
    int32_t whole_k_rows;   // bf16: from 17 up to this many rows (at most 32) the wide kernel's whole-K variant runs (0 = never)
};

// what the bf16 GEMM does with its final fp32 values
#define SJD_EPI_STORE 0   // out[m][n] = v
#define SJD_EPI_RESID 1   // out[m][n] += v                       (residual stream)
#define SJD_EPI_SILU 2    // ffn[m][f] = SiLU(gate) * up          (rows packed gate/up interleaved)
#define SJD_EPI_QKV 3     // RoPE on q,k at position n+m; q -> qact, k,v -> cache
struct SjdGemmEpi {
    int32_t kind;
    SjdStreams sm;               // QKV: who owns which rows
    size_t layer_off;            // QKV: element offset of this layer inside every stream's cache
    float *out;                  // STORE / RESID: [rows][N]
    void *out24;                 // RESID: planes of (updated rows) * gain_next, or NULL: none of the three
    const bf16_t *gain_next;     // RESID: [N] gain of the normalisation that follows
    float *ssq_out;              // RESID: [rows][ssq_stride(N)] sum of squares of the updated rows per 16 features
    void *ffn; int32_t F;                                         // SILU: [rows][F] in act24 planes
    int32_t lo16;                // RESID, SILU: the planes they write carry the 2-byte lo plane (wide forwards)
    float *qact; const float *cosT, *sinT;                        // QKV
    int32_t d, hd, nblk, rows_valid, max_seq;                     // rows_valid: rows per stream whose K/V are stored
};

struct SjdLayer {
    const void *g1, *g2;
    SjdLinear qkv, o, gu, down;  // qkv: rows [Wq; Wk; Wv]; gu: rows [Wg; Wu]
};

struct sjd_model {
    sjd_config cfg;
    int32_t hd, V_s;
    void *weights;        // one device allocation holding everything below
    const void *E;        // embedding table [vocab][d], element type per dtype, row-major
    const void *gf;
    SjdLinear lm;         // rows samp_lo..samp_hi of the LM head
    SjdLayer *layers;     // host array
    float *rope_cos, *rope_sin;  // [max_seq][hd/2]
};

struct sjd_kv {
    const sjd_model *m;
    void *k, *v;          // fp32 models: K and V as [layer][pos][d]; bf16 models: k holds the blocked
                          // hi/lo cache described above ([layer][head][block][128*hd]), v is unused
    void *k_u, *v_u;      // the same for the unconditional stream (allocated when guidance is first used)
    int32_t cfg_on;       // a second stream is pre-filled: forwards run both, logits are guided
    float cfg_scale;
    int32_t n_upper_u;    // host-side upper bound of n_u
    float *logits_last;   // [V_s] raw logits of the last prompt position (stream 0), for guidance
    size_t k_layer_stride, v_layer_stride;   // elements
    int32_t nblk;         // bf16 models: 32-position blocks per head
    int32_t *tokens;      // [max_seq] ids of cached positions (-1 for raw-embedding rows)
    SjdState *state;      // device
    // ---- scratch for one forward over <= SJD_ROWS_MAX rows ----
    float *x;             // [rows][d] residual stream
    void *x24;            // bf16 models: hi / lo planes of x * (gain of the next normalisation)
    float *ssq;           // bf16 models: [rows][ssq_stride(d)] partial sums of squares of x
    void *h;              // fp32 models: [rows][d] normalised activations
    float *part;          // fp32 models: GEMM output
    size_t part_elems;
    float *qact;          // [rows][d] rotated queries (fp32)
    float *att_part;      // attention partials per (head, split): [rows][hd] + m,l
    int32_t att_splits;
    void *att_out;        // [rows][d] fp32; bf16 models: hi / lo planes
    void *ffn;            // [rows][F] fp32; bf16 models: hi / lo planes
    float *logits;        // [rows][V_s]
    // ---- scratch for verification ----
    float *q;             // [(rows+1)][V_s]
    int32_t *tok_smp, *tok_res, *acc_flag, *draft_snap;  // [rows+1] each
    void *snap;
    int32_t *forced;      // [rows+1]
    int32_t *ids_stage;   // [rows] device copy of prompt ids chunk
    float *emb_stage;     // [rows][d]
    // generate loop buffers
    int32_t *g_draft;     // [rows]
    float *g_p;           // [rows][V_s]
    int32_t *g_nacc;      // [1]
    float *q_first;       // [V_s]
    int32_t n_upper;      // host-side upper bound of the device-resident n
    SjdState *state_host; // pinned host copy the state is read into
    hipStream_t last_stream;   // stream of the handle's most recent enqueue: reading the state waits for it only
    // device-resident decoding loop (sjd_decode_*)
    int32_t dec_active, dec_N, dec_L;
    sjd_sampler dec_smp;
    sjd_init dec_init;
    uint64_t dec_seed;
    int32_t use_graph;
    hipGraph_t graph;
    hipGraphExec_t graph_exec;
    // batched decoding led by this handle: one captured iteration for a fixed set of handles
    hipGraph_t bgraph;
    hipGraphExec_t bgraph_exec;
    struct BatchKey {
        int32_t B, L;
        sjd_sampler smp;
        sjd_init init;
        const void *kv[SJD_MAX_STREAMS], *state[SJD_MAX_STREAMS], *cache[SJD_MAX_STREAMS], *ring[SJD_MAX_STREAMS];
        const void *cache_u[SJD_MAX_STREAMS];      // guided batches: the handles' second caches ...
        float cfg_scale[SJD_MAX_STREAMS];          // ... and their guidance weights
        int32_t cfg_on;
        uint64_t seed[SJD_MAX_STREAMS];
    } bkey;
    SjdStreamEntry *cfg_tab;                   // device [2]: the two contexts of this handle under guidance
    SjdStreamEntry *btab;                      // device [SJD_MAX_STREAMS]: handles of the batch this one leads
    SjdStreamEntry btab_host[SJD_MAX_STREAMS]; // what btab holds
    float *ring;          // [ring_rows][V_s] distributions of accepted image positions (initialiser (d))
    int32_t ring_rows;
    int32_t graph_cfg_on;   // stream mode and guidance weight the captured iteration was recorded with
    float graph_cfg_scale;
    void *prof;           // SjdProfiler* while sjd_profile_steps runs, else NULL
    double prof_kv_tokens;   // while profiling: cached positions (all streams) the next iteration's attention reads
};

// ---- kernel launchers (each returns SJD_OK or an SJD_E* code) --------------------------------
// `st` (device, fp32 models' kernels) lets a kernel skip its work once a generation has finished; NULL = always run.
// bf16 models: `rows` rows per stream, stream s from ids[s] (device ids; all streams share emb_rows when
// that is given instead), written at row s << sm.shift.  fp32 models: one stream, ids[0].
// err[s] (device, may be NULL): receives SJD_DEVERR_TOKEN_ID when an id of stream s lies outside the vocabulary
// lo16: x24 gets the 2-byte lo plane (the forward runs on the wide projection kernel)
int sjd_launch_embed(const sjd_model *m, const int32_t *const *ids, const float *emb_rows, int32_t rows,
                     const SjdStreams &sm, float *x, void *x24, float *ssq, int32_t *const *err, bool lo16, hipStream_t s);
int sjd_launch_rmsnorm(const sjd_model *m, float *x, const float *part, int32_t n_part, size_t part_stride,
                       const void *gain, int32_t rows, void *h, const SjdState *st, hipStream_t s);
int sjd_launch_rope_kv(const sjd_model *m, sjd_kv *kv, int32_t layer, int32_t stream, const float *part, int32_t n_part,
                       size_t part_stride, int32_t rows, int32_t rows_valid, hipStream_t s);
int sjd_launch_silu_mul(const sjd_model *m, const float *part, int32_t n_part, size_t part_stride, int32_t rows,
                        void *ffn, const SjdState *st, hipStream_t s);
int sjd_launch_reduce_rows(const float *part, int32_t n_part, size_t part_stride, int32_t rows, int32_t cols,
                           float *out, const SjdState *st, hipStream_t s);
int sjd_launch_gemm(int32_t dtype, const SjdLinear *lin, const void *act, int32_t rows, float *part,
                    const SjdState *st, hipStream_t s);
int sjd_repack_bf16(const bf16_t *src_dev, bf16_t *dst_dev, int32_t N, int32_t K, int32_t tn, int32_t perm, int32_t d,
                    int32_t hd, hipStream_t s);
void sjd_choose_tiles(SjdLinear *lin);
// bf16 projection: act = the 3-byte planes described at act24_idx() (act24 set) or fp32 [SJD_ROWS_MAX x K]
// in act_off order.  ssq_in != NULL (planes only): the planes hold x * gain and ssq_in the partial sums
// of squares of x ([rows][ssq_stride(K)]); the projection applies rsqrt(mean(x^2) + eps) per row.
// More than SJD_ROWS_SKINNY rows go to the wide kernel (planes only), which needs `part`: room for the fp32
// sums of its K-slices (part_elems floats, at least 16 * ceil(rows / 16) * N); NULL = skinny kernel only.
#define SJD_ACT_F32 0     // fp32 values in act_off order (test hook)
#define SJD_ACT_P3 1      // operand planes, 1-byte lo plane (3 bytes per value)
#define SJD_ACT_P4 2      // operand planes, 2-byte lo plane (4 bytes per value)
int sjd_launch_gemm_bf16(const SjdLinear *lin, const void *act, int form, const float *ssq_in, float eps, int32_t rows,
                         const SjdGemmEpi &ep, float *part, size_t part_elems, hipStream_t s);
int sjd_launch_gemm_wide(const SjdLinear *lin, const void *act, const float *ssq_in, float eps, int32_t rows,
                         const SjdGemmEpi &ep, float *part, size_t part_elems, hipStream_t s);
int sjd_launch_gemm_wide3(const SjdLinear *lin, const void *act, const float *ssq_in, float eps, int32_t rows,
                          const SjdGemmEpi &ep, hipStream_t s);
void sjd_wide_plan(const SjdLinear *lin, int mt, size_t part_elems, int *g_out, int *ks_out, int *kps_out);
int sjd_gemm_wide_setup();
int sjd_bf16_rows_to_f32(const bf16_t *src, int32_t rows, int32_t K, float *dst, hipStream_t s);
int sjd_f32_rows_to_act24(const float *src, int32_t rows, int32_t K, void *dst, bool lo16, hipStream_t s);
int sjd_bf16_rows_to_act24(const bf16_t *src, int32_t rows, int32_t K, void *dst, hipStream_t s);    // (either lo form: zeros)
// fp32 models: `stream` 0 / 1 selects the cache and length of the handle
int sjd_launch_attention_f32(const sjd_model *m, sjd_kv *kv, int32_t layer, int32_t rows, int32_t stream, hipStream_t s);
// bf16 models: `rows` query rows per stream of sm against that stream's cache
int sjd_launch_attention(const sjd_model *m, sjd_kv *kv, int32_t layer, int32_t rows, const SjdStreams &sm, bool lo16,
                         hipStream_t s);
int32_t sjd_attention_splits(const sjd_model *m);
size_t sjd_attention_part_elems(const sjd_model *m);
// sampling / verification
struct SjdVerifyArgs {
    const float *logits;     // [L][V] or NULL when q rows are given
    const float *logits_u;   // [L][V] unconditional logits, or NULL: z = z_u + cfg_scale * (z - z_u)
    float cfg_scale;
    const float *q_in;       // [(L+1)][V] precomputed distributions or NULL
    const float *p_old;      // [L][V]
    float *ring;             // [row_stride][V] distributions of accepted positions (init mode 4), else NULL
    const int32_t *draft;    // [L]
    int32_t L, V, lo;
    sjd_sampler smp;
    sjd_init init;
    const int32_t *hist;     // image tokens fixed so far (index = image position) or NULL
    uint64_t seed;
    // state: when `state` != NULL, img_pos0 / counter / L_eff come from it and it is advanced
    SjdState *state;
    int32_t *kv_tokens;      // record accepted ids at cache positions (with state) or NULL
    int32_t img_pos0;
    uint64_t counter;
    int32_t *n_accepted;     // [1]
    int32_t *new_draft;      // [L]
    float *p_new;            // [L][V]
    // scratch
    float *q;                // [(L+1)][V]
    int32_t *tok_smp, *tok_res, *acc_flag, *draft_snap;
    void *snap;              // 32 bytes: per-step scalars frozen for the second kernel
};
int sjd_launch_verify(const SjdVerifyArgs *a, hipStream_t s);
int sjd_launch_verify_batch(const SjdVerifyArgs *a, int32_t B, hipStream_t s);   // a[B]: one per image, same L, V, init mode
int sjd_sample_setup(int32_t V);   // raise the dynamic-LDS limit of the sampling kernels for vocabulary V
int sjd_launch_dist(const float *logits, const float *logits_u, float cfg_scale, int32_t rows, int32_t V,
                    const sjd_sampler *smp, const int32_t *forced, float *q, hipStream_t s);
int sjd_launch_guide(const float *logits, const float *logits_u, float cfg_scale, size_t n, float *out, hipStream_t s);
int sjd_launch_first_window(const float *q_first, int32_t L, int32_t V, int32_t lo, const sjd_init *init,
                            uint64_t seed, int32_t *draft, float *p_old, hipStream_t s);
