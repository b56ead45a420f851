// C-ABI entry points and step orchestration of the SJD library (see include/sjd.h).
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "sjd_internal.h"

// ---- errors ---------------------------------------------------------------------------------
static thread_local char g_hip_msg[256] = "no HIP error recorded";
static thread_local char g_limit_msg[256] = "a size exceeds a fixed limit of the entry point";
void sjd_set_hip_error(hipError_t e, const char *what)
{
    snprintf(g_hip_msg, sizeof(g_hip_msg), "HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
}

extern "C" const char *sjd_strerror(int code)
{
    switch (code) {
        case SJD_OK: return "ok";
        case SJD_EINVAL: return "invalid argument (host-side check, or a kernel met a token id outside the vocabulary "
                                "or an image position beyond the cache length)";
        case SJD_ENOMEM: return "out of memory";
        case SJD_ESEQ: return "sequence would exceed max_seq";
        case SJD_EHIP: return g_hip_msg;
        case SJD_ELIMIT: return g_limit_msg;
        default: return "unknown error code";
    }
}

static size_t elt_size(int dtype) { return dtype == 0 ? 4 : 2; }

static int dev_alloc(void **p, size_t bytes)
{
    hipError_t e = hipMalloc(p, bytes ? bytes : 16);
    if (e == hipErrorOutOfMemory) { *p = nullptr; (void)hipGetLastError(); return SJD_ENOMEM; }
    HIP_TRY(e);
    HIP_TRY(hipMemset(*p, 0, bytes ? bytes : 16));
    return SJD_OK;
}

// ---- model ----------------------------------------------------------------------------------
static int check_config(const sjd_config *c)
{
    if (!c) return SJD_EINVAL;
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->d_ffn < 1 || c->vocab_total < 1) return SJD_EINVAL;
    if (c->d_model % c->n_heads) return SJD_EINVAL;
    const int hd = c->d_model / c->n_heads;
    if (hd != 16 && hd != 32 && hd != 64 && hd != 128) return SJD_EINVAL;
    if (c->samp_lo < 0 || c->samp_hi > c->vocab_total || c->samp_lo >= c->samp_hi) return SJD_EINVAL;
    if (c->samp_hi - c->samp_lo > SJD_MAX_SAMP_VOCAB) return SJD_EINVAL;
    if (c->max_seq < 2) return SJD_EINVAL;
    if (c->dtype != 0 && c->dtype != 1) return SJD_EINVAL;
    if (c->dtype == 0 && (c->d_model % 4 || c->d_ffn % 4)) return SJD_EINVAL;
    if (c->dtype == 1 && (c->d_model % 32 || c->d_ffn % 32 || (c->samp_hi - c->samp_lo) % 16 || c->d_model > 8192 || hd < 32))
        return SJD_EINVAL;
    if (!(c->rope_theta > 0.f) || !(c->rms_eps >= 0.f)) return SJD_EINVAL;
    return SJD_OK;
}

static size_t blob_elems(const sjd_config *c)
{
    const size_t d = c->d_model, f = c->d_ffn, v = c->vocab_total;
    return v * d + (size_t)c->n_layers * (2 * d + 4 * d * d + 3 * d * f) + d + v * d;
}

extern "C" void sjd_free_model(sjd_model *m)
{
    if (!m) return;
    if (m->weights) (void)hipFree(m->weights);
    if (m->rope_cos) (void)hipFree(m->rope_cos);
    if (m->rope_sin) (void)hipFree(m->rope_sin);
    delete[] m->layers;
    delete m;
}

extern "C" int sjd_init_model(const sjd_config *cfg, const void *host_weights, size_t nbytes, sjd_model **out)
{
    if (!out) return SJD_EINVAL;
    *out = nullptr;
    SJD_TRY(check_config(cfg));
    if (!host_weights) return SJD_EINVAL;
    const size_t es = elt_size(cfg->dtype);
    const size_t total = blob_elems(cfg);
    if (nbytes != total * es) return SJD_EINVAL;

    sjd_model *m = new (std::nothrow) sjd_model();
    if (!m) return SJD_ENOMEM;
    m->cfg = *cfg;
    m->hd = cfg->d_model / cfg->n_heads;
    m->V_s = cfg->samp_hi - cfg->samp_lo;
    m->layers = new (std::nothrow) SjdLayer[cfg->n_layers];
    if (!m->layers) { sjd_free_model(m); return SJD_ENOMEM; }

    int rc = dev_alloc(&m->weights, total * es);
    if (rc != SJD_OK) { sjd_free_model(m); return rc; }
    const size_t d = cfg->d_model, f = cfg->d_ffn, v = cfg->vocab_total;
    const char *hb = (const char *)host_weights;
    char *db = (char *)m->weights;

    // staging buffer for the largest matrix that needs repacking (bf16 only)
    void *stage = nullptr;
    size_t stage_elems = 0;
    if (cfg->dtype == 1) {
        stage_elems = std::max<size_t>({3 * d * d, 2 * f * d, d * f, (size_t)m->V_s * d});
        rc = dev_alloc(&stage, stage_elems * es);
        if (rc != SJD_OK) { sjd_free_model(m); return rc; }
    }
    auto fail = [&](int code) { if (stage) (void)hipFree(stage); sjd_free_model(m); return code; };
#define UP_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) { sjd_set_hip_error(e_, #expr); return fail(SJD_EHIP); } } while (0)

    // copy a tensor as is; returns its device pointer
    auto plain = [&](size_t off, size_t n) -> const void * {
        const hipError_t e = hipMemcpy(db + off * es, hb + off * es, n * es, hipMemcpyHostToDevice);
        if (e != hipSuccess) { sjd_set_hip_error(e, "weight upload"); return nullptr; }
        return db + off * es;
    };
    // a linear layer [N][K] starting at element `off`: fp32 as is, bf16 repacked
    auto linear = [&](size_t off, int N, int K, int perm, SjdLinear *lin) -> int {
        memset(lin, 0, sizeof(*lin));
        lin->N = N; lin->K = K; lin->tn = 1;
        lin->w = db + off * es;
        const size_t n = (size_t)N * K;
        if (cfg->dtype == 0) {
            HIP_TRY(hipMemcpy(db + off * es, hb + off * es, n * es, hipMemcpyHostToDevice));
            return SJD_OK;
        }
        HIP_TRY(hipMemcpy(stage, hb + off * es, n * es, hipMemcpyHostToDevice));
        sjd_choose_tiles(lin);           // the packed order depends on the tiles per workgroup
        SJD_TRY(sjd_repack_bf16((const bf16_t *)stage, (bf16_t *)(db + off * es), N, K, lin->tn, perm, (int)d, m->hd, 0));
        HIP_TRY(hipDeviceSynchronize());
        return SJD_OK;
    };

    size_t off = 0;
    m->E = plain(off, v * d); if (!m->E) return fail(SJD_EHIP);
    off += v * d;
    for (int l = 0; l < cfg->n_layers; ++l) {
        SjdLayer *L = &m->layers[l];
        L->g1 = plain(off, d); if (!L->g1) return fail(SJD_EHIP);
        off += d;
        rc = linear(off, (int)(3 * d), (int)d, 1, &L->qkv); if (rc) return fail(rc);
        off += 3 * d * d;
        rc = linear(off, (int)d, (int)d, 0, &L->o); if (rc) return fail(rc);
        off += d * d;
        L->g2 = plain(off, d); if (!L->g2) return fail(SJD_EHIP);
        off += d;
        rc = linear(off, (int)(2 * f), (int)d, 2, &L->gu); if (rc) return fail(rc);
        off += 2 * f * d;
        rc = linear(off, (int)d, (int)f, 0, &L->down); if (rc) return fail(rc);
        off += d * f;
        // From 17 rows on the skinny kernel reads two M-tiles of activations per weight tile in every wave; a
        // projection with one weight tile per workgroup and a long reduction (the 7B down projection: 256
        // workgroups, each re-reading 32 x 11008 activations) is then faster on the wide kernel, whose waves
        // share the activations through LDS (measured alone on cold weights: 23.6 against 29.9 us).
        if (cfg->dtype == 1 && L->down.tn == 1 && L->down.N >= 4096 && L->down.K >= 2 * L->down.N) L->down.wide_from = 17;
    }
    m->gf = plain(off, d); if (!m->gf) return fail(SJD_EHIP);
    off += d;
    rc = linear(off + (size_t)cfg->samp_lo * d, m->V_s, (int)d, 0, &m->lm); if (rc) return fail(rc);
    if (stage) { (void)hipFree(stage); stage = nullptr; }

    // RoPE tables in fp64 on the host, rounded once to fp32: angle = pos * theta^(-2j/hd)
    const int half = m->hd / 2;
    std::vector<float> c((size_t)cfg->max_seq * half), s((size_t)cfg->max_seq * half);
    for (int p = 0; p < cfg->max_seq; ++p)
        for (int j = 0; j < half; ++j) {
            double ang = (double)p * std::pow((double)cfg->rope_theta, -2.0 * j / m->hd);
            c[(size_t)p * half + j] = (float)std::cos(ang);
            s[(size_t)p * half + j] = (float)std::sin(ang);
        }
    rc = dev_alloc((void **)&m->rope_cos, c.size() * 4); if (rc) return fail(rc);
    rc = dev_alloc((void **)&m->rope_sin, s.size() * 4); if (rc) return fail(rc);
    UP_TRY(hipMemcpy(m->rope_cos, c.data(), c.size() * 4, hipMemcpyHostToDevice));
    UP_TRY(hipMemcpy(m->rope_sin, s.data(), s.size() * 4, hipMemcpyHostToDevice));
    UP_TRY(hipDeviceSynchronize());
#undef UP_TRY
    *out = m;
    return SJD_OK;
}

// ---- cache + scratch ------------------------------------------------------------------------
#define SJD_RING_ROWS_DEFAULT 128   // rows of the distribution ring a handle is created with (initialiser (d))
extern "C" void sjd_kv_free(sjd_kv *kv)
{
    if (!kv) return;
    void *ptrs[] = {kv->k, kv->v, kv->k_u, kv->v_u, kv->logits_last, kv->ring, kv->cfg_tab, kv->btab, kv->tokens, kv->state, kv->x, kv->x24, kv->ssq, kv->h, kv->part, kv->qact, kv->att_part, kv->att_out,
                    kv->ffn, kv->logits, kv->q, kv->tok_smp, kv->tok_res, kv->acc_flag, kv->draft_snap, kv->snap,
                    kv->forced, kv->ids_stage, kv->emb_stage, kv->g_draft, kv->g_p, kv->g_nacc, kv->q_first};
    for (void *p : ptrs) if (p) (void)hipFree(p);
    if (kv->state_host) (void)hipHostFree(kv->state_host);
    if (kv->graph_exec) (void)hipGraphExecDestroy(kv->graph_exec);
    if (kv->graph) (void)hipGraphDestroy(kv->graph);
    if (kv->bgraph_exec) (void)hipGraphExecDestroy(kv->bgraph_exec);
    if (kv->bgraph) (void)hipGraphDestroy(kv->bgraph);
    delete kv;
}

extern "C" int sjd_kv_create(const sjd_model *m, sjd_kv **out)
{
    if (!m || !out) return SJD_EINVAL;
    *out = nullptr;
    sjd_kv *kv = new (std::nothrow) sjd_kv();
    if (!kv) return SJD_ENOMEM;
    memset(kv, 0, sizeof(*kv));
    kv->m = m;
    kv->use_graph = 1;
    const sjd_config &c = m->cfg;
    const size_t d = c.d_model, F = c.d_ffn, V = m->V_s, R = SJD_ROWS_MAX;
    size_t part = 0;
    auto upd = [&](const SjdLinear &l) { part = std::max(part, (size_t)R * l.N); };
    for (int l = 0; l < c.n_layers; ++l) { upd(m->layers[l].qkv); upd(m->layers[l].o); upd(m->layers[l].gu); upd(m->layers[l].down); }
    upd(m->lm);
    kv->part_elems = part;
    kv->att_splits = sjd_attention_splits(m);
    int rc = SJD_OK;
#define A(ptr, bytes) if (rc == SJD_OK) rc = dev_alloc((void **)&(ptr), (bytes))
    if (c.dtype == 1) {
        // blocked hi/lo cache: [layer][head][block of 32 positions][128 * hd] bf16, K and V together
        kv->nblk = (c.max_seq + 31) / 32;
        kv->k_layer_stride = (size_t)kv->nblk * 128 * d;
        A(kv->k, (size_t)c.n_layers * kv->k_layer_stride * 2);
    } else {
        kv->k_layer_stride = kv->v_layer_stride = (size_t)c.max_seq * d;
        A(kv->k, (size_t)c.n_layers * kv->k_layer_stride * 4);
        A(kv->v, (size_t)c.n_layers * kv->v_layer_stride * 4);
    }
    A(kv->tokens, (size_t)c.max_seq * 4);
    A(kv->state, sizeof(SjdState));
    // bf16 models: every activation matrix is followed by one all-zero operand tile (2 KiB); the
    // attention output and the FFN hidden are hi / lo planes (3 bytes per value, zero tile included:
    // smaller than the fp32 matrices of the fp32 models these sizes are written for)
    A(kv->x, R * d * 4 + 2048);
    A(kv->x24, c.dtype == 1 ? act24_bytes((int)d / 32) : 16);
    A(kv->ssq, c.dtype == 1 ? R * ssq_stride((int)d) * 4 : 16);
    A(kv->h, c.dtype == 0 ? R * d * 4 : 16);
    // fp32 models: the output of a linear layer; bf16 models: the fp32 sums of the wide projection kernel's
    // K-slices (two full outputs' worth: shapes with few output features split K further)
    if (c.dtype == 1) kv->part_elems = 2 * part;
    A(kv->part, kv->part_elems * 4);
    A(kv->qact, R * d * 4);
    A(kv->att_part, sjd_attention_part_elems(m) * 4);
    A(kv->att_out, R * d * 4 + 2048);
    A(kv->ffn, R * F * 4 + 2048);
    A(kv->logits, R * V * 4);
    A(kv->q, (R + 1) * V * 4);
    A(kv->tok_smp, (R + 1) * 4);
    A(kv->tok_res, (R + 1) * 4);
    A(kv->acc_flag, (R + 1) * 4);
    A(kv->draft_snap, (R + 1) * 4);
    A(kv->snap, 64);
    A(kv->forced, (R + 1) * 4);
    A(kv->ids_stage, R * 4);
    A(kv->emb_stage, R * d * 4);
    A(kv->g_draft, R * 4);
    A(kv->g_p, R * V * 4);
    A(kv->g_nacc, 16);
    A(kv->q_first, V * 4);
    A(kv->logits_last, V * 4);
    A(kv->ring, (size_t)SJD_RING_ROWS_DEFAULT * V * 4);
    if (rc == SJD_OK) kv->ring_rows = SJD_RING_ROWS_DEFAULT;
    A(kv->cfg_tab, 2 * sizeof(SjdStreamEntry));
    A(kv->btab, SJD_MAX_STREAMS * sizeof(SjdStreamEntry));
#undef A
    if (rc == SJD_OK) rc = sjd_sample_setup(m->V_s);
    if (rc == SJD_OK && c.dtype == 1) rc = sjd_gemm_wide_setup();
    if (rc == SJD_OK) {
        const hipError_t e = hipHostMalloc((void **)&kv->state_host, sizeof(SjdState), hipHostMallocDefault);
        if (e != hipSuccess) { kv->state_host = nullptr; sjd_set_hip_error(e, "hipHostMalloc"); rc = e == hipErrorOutOfMemory ? SJD_ENOMEM : SJD_EHIP; }
    }
    if (rc != SJD_OK) { sjd_kv_free(kv); return rc; }
    *out = kv;
    return SJD_OK;
}

static int state_write(sjd_kv *kv, const SjdState &st, hipStream_t s)
{
    // small synchronous-with-respect-to-host copy (source is on the stack)
    HIP_TRY(hipMemcpyAsync(kv->state, &st, sizeof(SjdState), hipMemcpyHostToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));
    return SJD_OK;
}
// Waits for the stream the handle's work was last enqueued on (not for the device: other handles on
// other streams keep running) and copies the state into the handle's pinned host buffer.  A kernel
// that met bad device-side input has left a flag in the state: reported here as SJD_EINVAL.
static int state_read(const sjd_kv *kv, SjdState *st)
{
    HIP_TRY(hipMemcpyAsync(kv->state_host, kv->state, sizeof(SjdState), hipMemcpyDeviceToHost, kv->last_stream));
    HIP_TRY(hipStreamSynchronize(kv->last_stream));
    *st = *kv->state_host;
    return st->err ? SJD_EINVAL : SJD_OK;
}

extern "C" int sjd_kv_reset(sjd_kv *kv)
{
    if (!kv) return SJD_EINVAL;
    HIP_TRY(hipDeviceSynchronize());
    SjdState st;
    memset(&st, 0, sizeof(st));
    kv->n_upper = 0;
    kv->n_upper_u = 0;
    kv->dec_active = 0;
    kv->cfg_on = 0;
    return state_write(kv, st, 0);
}

extern "C" int sjd_kv_len(const sjd_kv *kv, int32_t *n)
{
    if (!kv || !n) return SJD_EINVAL;
    SjdState st;
    SJD_TRY(state_read(kv, &st));
    *n = st.n;
    const_cast<sjd_kv *>(kv)->n_upper = st.n;
    return SJD_OK;
}

extern "C" int sjd_kv_set_len(sjd_kv *kv, int32_t n)
{
    if (!kv || n < 0 || n > kv->m->cfg.max_seq) return SJD_EINVAL;
    SjdState st;
    SJD_TRY(state_read(kv, &st));
    if (kv->cfg_on) {                   // both streams hold the same image tokens: move them together
        const int n_u = st.n_u + (n - st.n);
        if (n_u < 0 || n_u > kv->m->cfg.max_seq) return SJD_EINVAL;
        st.n_u = n_u;
        kv->n_upper_u = n_u;
    }
    st.n = n;
    st.done = 0;
    kv->n_upper = n;
    return state_write(kv, st, 0);
}

static void drop_graph(sjd_kv *kv)
{
    if (kv->graph_exec) { (void)hipGraphExecDestroy(kv->graph_exec); kv->graph_exec = nullptr; }
    if (kv->graph) { (void)hipGraphDestroy(kv->graph); kv->graph = nullptr; }
}

static void drop_batch_graph(sjd_kv *kv)
{
    if (kv->bgraph_exec) { (void)hipGraphExecDestroy(kv->bgraph_exec); kv->bgraph_exec = nullptr; }
    if (kv->bgraph) { (void)hipGraphDestroy(kv->bgraph); kv->bgraph = nullptr; }
    memset(&kv->bkey, 0, sizeof(kv->bkey));
}

// ---- optional per-kernel timing -------------------------------------------------------------
thread_local SjdLaunchHook *sjd_launch_hook = nullptr;

struct SjdProfiler {
    std::vector<hipEvent_t> ev;      // pairs (start, stop), one per kernel launch
    std::vector<int> kind;           // per pair
    std::vector<double> bytes;       // per pair: algorithmic HBM bytes attributed to the launch
    size_t used = 0;
    int cur_kind = 0;
    double cur_bytes = 0;            // handed to the first launch of the current scope
    int rc = SJD_OK;
    SjdLaunchHook hook;
    void scope(int k, double b) { cur_kind = k; cur_bytes = b; hook.cur_kind = k; }
    static int next(void *self, hipEvent_t *start, hipEvent_t *stop)
    {
        SjdProfiler *p = (SjdProfiler *)self;
        if (p->used + 2 > p->ev.size()) {
            for (int i = 0; i < 2; ++i) {
                hipEvent_t e;
                if (hipEventCreate(&e) != hipSuccess) { p->rc = SJD_EHIP; return SJD_EHIP; }
                p->ev.push_back(e);
            }
            p->kind.push_back(0); p->bytes.push_back(0);
        }
        p->kind[p->used / 2] = p->cur_kind; p->bytes[p->used / 2] = p->cur_bytes;
        p->cur_bytes = 0;
        *start = p->ev[p->used]; *stop = p->ev[p->used + 1];
        p->used += 2;
        return SJD_OK;
    }
    int drain(sjd_profile *out, hipStream_t s)
    {
        HIP_TRY(hipStreamSynchronize(s));
        for (size_t i = 0; i < used; i += 2) {
            float ms = 0.f;
            HIP_TRY(hipEventElapsedTime(&ms, ev[i], ev[i + 1]));
            const int k = kind[i / 2];
            out->ms[k] += ms; out->launches[k] += 1; out->bytes[k] += bytes[i / 2];
        }
        used = 0;
        return rc;
    }
    void destroy() { for (hipEvent_t e : ev) (void)hipEventDestroy(e); ev.clear(); }
};
#define PROF(kv, k, b, call)                                             \
    do {                                                                 \
        if ((kv)->prof) ((SjdProfiler *)(kv)->prof)->scope((k), (b));    \
        SJD_TRY(call);                                                   \
    } while (0)

// rows one forward computes and the largest window: bf16 models SJD_MAX_ROWS / SJD_MAX_WINDOW, the fp32
// models (launch-bound toys on plain kernels) 32 / 32; under guidance two contexts share the rows
static int rows_max(const sjd_model *m) { return m->cfg.dtype == 1 ? SJD_ROWS_MAX : SJD_ROWS_F32; }
static int window_max(const sjd_model *m, bool guided)
{
    const int w = std::min(rows_max(m) / (guided ? 2 : 1), SJD_MAX_WINDOW);
    return m->cfg.dtype == 1 ? w : std::min(w, SJD_ROWS_F32);
}

// Which form the activations of a forward over `grows` rows take between its kernels: the 2-byte lo plane
// (second MFMA operand ready made, 4 bytes per value) from SJD_LO16_FROM_ROWS rows on, the 1-byte lo plane
// (3 bytes per value, second operand rebuilt by every wave) below.  One choice per forward: every producer
// and every consumer of a forward agree.
static int g_lo16_from_rows = SJD_LO16_FROM_ROWS;
static bool rows_use_lo16(int grows) { return grows >= g_lo16_from_rows; }

// ---- the window forward (Step 2) ------------------------------------------------------------
// rows = rows computed (<= 32), rows_valid = rows whose K/V are written.  Inputs already in kv->x.
static double lin_bytes(const sjd_model *m, const SjdLinear &l) { return (double)l.N * l.K * elt_size(m->cfg.dtype); }

// `stream` selects the cache and the cache length the rows are positioned with (0 conditional,
// 1 unconditional).
static int forward_rows_f32(sjd_model *m, sjd_kv *kv, int32_t rows, int32_t rows_valid, int32_t stream, float *logits,
                            hipStream_t s)
{
    const SjdState *st = kv->state;
    const SjdLinear *prev = nullptr;   // GEMM whose output still has to be added to x
    const double kv_bytes_layer = kv->prof ? 2.0 * kv->prof_kv_tokens * m->cfg.d_model * 4
                                           : 2.0 * ((stream ? kv->n_upper_u : kv->n_upper) + rows) * m->cfg.d_model * 4;
    for (int l = 0; l < m->cfg.n_layers; ++l) {
        const SjdLayer &L = m->layers[l];
        PROF(kv, SJD_PROF_ELEMENTWISE, 0, sjd_launch_rmsnorm(m, kv->x, prev ? kv->part : nullptr, prev ? 1 : 0, 0, L.g1, rows, kv->h, st, s));
        PROF(kv, SJD_PROF_GEMM, lin_bytes(m, L.qkv), sjd_launch_gemm(0, &L.qkv, kv->h, rows, kv->part, st, s));
        PROF(kv, SJD_PROF_ELEMENTWISE, 0, sjd_launch_rope_kv(m, kv, l, stream, kv->part, 1, 0, rows, rows_valid, s));
        PROF(kv, SJD_PROF_ATTENTION, kv_bytes_layer, sjd_launch_attention_f32(m, kv, l, rows, stream, s));
        PROF(kv, SJD_PROF_GEMM, lin_bytes(m, L.o), sjd_launch_gemm(0, &L.o, kv->att_out, rows, kv->part, st, s));
        PROF(kv, SJD_PROF_ELEMENTWISE, 0, sjd_launch_rmsnorm(m, kv->x, kv->part, 1, 0, L.g2, rows, kv->h, st, s));
        PROF(kv, SJD_PROF_GEMM, lin_bytes(m, L.gu), sjd_launch_gemm(0, &L.gu, kv->h, rows, kv->part, st, s));
        PROF(kv, SJD_PROF_ELEMENTWISE, 0, sjd_launch_silu_mul(m, kv->part, 1, 0, rows, kv->ffn, st, s));
        PROF(kv, SJD_PROF_GEMM, lin_bytes(m, L.down), sjd_launch_gemm(0, &L.down, kv->ffn, rows, kv->part, st, s));
        prev = &L.down;
    }
    PROF(kv, SJD_PROF_ELEMENTWISE, 0, sjd_launch_rmsnorm(m, kv->x, kv->part, 1, 0, m->gf, rows, kv->h, st, s));
    PROF(kv, SJD_PROF_GEMM, lin_bytes(m, m->lm), sjd_launch_gemm(0, &m->lm, kv->h, rows, logits, st, s));
    return SJD_OK;
}

// the streams of one handle: its conditional context alone (mode 0), its unconditional one alone (1),
// or both in rows 0.. and (1 << cfg_shift(rows)).. (2)
static SjdStreamEntry handle_entry(const sjd_kv *kv, bool uncond)
{
    const SjdState *st = kv->state;
    SjdStreamEntry e;
    e.n = uncond ? &st->n_u : &st->n;
    e.done = &st->done;
    e.kvc = (bf16_t *)(uncond ? kv->k_u : kv->k);
    return e;
}

// rows reserved per context in a two-context (guided) forward of `rows` window rows: the smallest
// power of two that holds them, at least one 16-row tile
static int cfg_shift(int32_t rows)
{
    int shift = 4;
    while ((1 << shift) < rows) ++shift;
    return shift;
}

static SjdStreams handle_streams(const sjd_kv *kv, int32_t stream_mode, int32_t rows)
{
    SjdStreams sm;
    memset(&sm, 0, sizeof(sm));
    sm.count = stream_mode == 2 ? 2 : 1;
    sm.shift = stream_mode == 2 ? cfg_shift(rows) : 7;
    sm.first = handle_entry(kv, stream_mode == 1);
    sm.table = stream_mode == 2 ? kv->cfg_tab : nullptr;     // filled when the second cache is allocated
    return sm;
}

// bf16: RMSNorm, residual adds, SiLU*up, RoPE and the cache write happen inside the projection kernel.
// `rows` rows per stream of `sm` (inputs already in kv->x, stream i at row i << sm.shift; the logits
// land in the same rows of `logits`).  The activation buffers are kv's; the caches are the streams'.
// kv_tokens_upper: upper bound of the cached positions all streams together read (profiling only).
static int forward_rows_bf16(sjd_model *m, sjd_kv *kv, const SjdStreams &sm, int32_t rows, int32_t rows_valid,
                             double kv_tokens_upper, float *logits, hipStream_t s)
{
    const int d = m->cfg.d_model, F = m->cfg.d_ffn;
    const float eps = m->cfg.rms_eps;
    const int grows = ((sm.count - 1) << sm.shift) + rows;      // rows the projections compute
    // Which kernel each projection runs on decides the form of the buffer it reads (its producer writes
    // that form): the residual stream's planes feed QKV, gate/up and the LM head, which go wide together
    // (above SJD_ROWS_SKINNY rows); the attention output feeds O and the FFN hidden feeds down, which may go
    // wide from fewer rows on (SjdLinear::wide_from).
    const bool lo16 = rows_use_lo16(grows);
    const int form = lo16 ? SJD_ACT_P4 : SJD_ACT_P3;
    auto goes_wide = [&](const SjdLinear &lin) { return lo16 || (lin.wide_from > 0 && grows >= lin.wide_from); };
    const bool o_wide = goes_wide(m->layers[0].o), down_wide = goes_wide(m->layers[0].down);
    // upper bound of the K/V bytes one layer's attention reads (hi + lo planes)
    const double kv_bytes_layer = 2.0 * kv_tokens_upper * d * 4;
    SjdGemmEpi e_qkv, e_res, e_silu, e_lm;
    memset(&e_qkv, 0, sizeof(e_qkv));
    e_qkv.sm = sm;
    e_res = e_qkv; e_silu = e_qkv; e_lm = e_qkv;
    e_qkv.kind = SJD_EPI_QKV; e_qkv.qact = kv->qact; e_qkv.cosT = m->rope_cos; e_qkv.sinT = m->rope_sin;
    e_qkv.d = d; e_qkv.hd = m->hd; e_qkv.nblk = kv->nblk; e_qkv.rows_valid = rows_valid; e_qkv.max_seq = m->cfg.max_seq;
    e_res.kind = SJD_EPI_RESID; e_res.out = kv->x; e_res.out24 = kv->x24; e_res.ssq_out = kv->ssq; e_res.lo16 = lo16;
    e_silu.kind = SJD_EPI_SILU; e_silu.ffn = kv->ffn; e_silu.F = F; e_silu.lo16 = down_wide;
    e_lm.kind = SJD_EPI_STORE; e_lm.out = logits;
    const void *x = kv->x24, *att = kv->att_out, *ffn = kv->ffn;     // hi / lo planes, 3 bytes per value
    // x24 holds x * (gain of the normalisation the next projection sits behind), kv->ssq its partial
    // sums of squares: written by the embedding kernel for the first layer, by each residual epilogue
    // for whatever follows it
    const float *ssq = kv->ssq;
    for (int l = 0; l < m->cfg.n_layers; ++l) {
        const SjdLayer &L = m->layers[l];
        e_qkv.layer_off = (size_t)l * kv->k_layer_stride;
        PROF(kv, SJD_PROF_GEMM, lin_bytes(m, L.qkv), sjd_launch_gemm_bf16(&L.qkv, x, form, ssq, eps, grows, e_qkv, kv->part, kv->part_elems, s));
        PROF(kv, SJD_PROF_ATTENTION, kv_bytes_layer, sjd_launch_attention(m, kv, l, rows, sm, o_wide, s));
        e_res.gain_next = (const bf16_t *)L.g2;
        PROF(kv, SJD_PROF_GEMM, lin_bytes(m, L.o), sjd_launch_gemm_bf16(&L.o, att, o_wide ? SJD_ACT_P4 : SJD_ACT_P3, nullptr, 0.f, grows, e_res, kv->part, kv->part_elems, s));
        PROF(kv, SJD_PROF_GEMM, lin_bytes(m, L.gu), sjd_launch_gemm_bf16(&L.gu, x, form, ssq, eps, grows, e_silu, kv->part, kv->part_elems, s));
        e_res.gain_next = (const bf16_t *)(l + 1 < m->cfg.n_layers ? m->layers[l + 1].g1 : m->gf);
        PROF(kv, SJD_PROF_GEMM, lin_bytes(m, L.down), sjd_launch_gemm_bf16(&L.down, ffn, down_wide ? SJD_ACT_P4 : SJD_ACT_P3, nullptr, 0.f, grows, e_res, kv->part, kv->part_elems, s));
    }
    PROF(kv, SJD_PROF_GEMM, lin_bytes(m, m->lm), sjd_launch_gemm_bf16(&m->lm, x, form, ssq, eps, grows, e_lm, kv->part, kv->part_elems, s));
    return SJD_OK;
}

// Embedding + decoder stack for one window or prompt chunk of one handle.  ids (device) or emb_rows
// (device fp32 rows), `rows` of them; stream_mode as in handle_streams.  Two streams see the same
// rows; their logits land in rows 0.. and (1 << cfg_shift(rows)).. of `logits`.
static int forward_window(sjd_model *m, sjd_kv *kv, const int32_t *ids, const float *emb_rows, int32_t rows,
                          int32_t rows_valid, int32_t stream_mode, float *logits, hipStream_t s)
{
    if (rows > rows_max(m) || (stream_mode == 2 && rows > rows_max(m) / 2)) return SJD_EINVAL;
    kv->last_stream = s;
    if (m->cfg.dtype == 1) {
        const SjdStreams sm = handle_streams(kv, stream_mode, rows);
        const int32_t *idv[SJD_MAX_STREAMS] = {ids, ids};
        int32_t *errv[SJD_MAX_STREAMS] = {&kv->state->err, &kv->state->err};
        const bool lo16 = rows_use_lo16(((sm.count - 1) << sm.shift) + rows);
        PROF(kv, SJD_PROF_ELEMENTWISE, 0, sjd_launch_embed(m, idv, emb_rows, rows, sm, kv->x, kv->x24, kv->ssq, errv, lo16, s));
        // (only the profiler uses the count: it has read the true lengths before the iteration)
        const double toks = kv->prof ? kv->prof_kv_tokens
                                     : (stream_mode == 1 ? 0 : kv->n_upper + rows) + (stream_mode == 0 ? 0 : kv->n_upper_u + rows);
        return forward_rows_bf16(m, kv, sm, rows, rows_valid, toks, logits, s);
    }
    // fp32 models are launch-bound toys: two streams are two forwards
    const SjdStreams one = handle_streams(kv, 0, rows);     // (only the finished flag is used by the embedding)
    const int32_t *idv[SJD_MAX_STREAMS] = {ids};
    int32_t *errv[SJD_MAX_STREAMS] = {&kv->state->err};
    for (int stream = (stream_mode == 1 ? 1 : 0); stream <= (stream_mode == 0 ? 0 : 1); ++stream) {
        PROF(kv, SJD_PROF_ELEMENTWISE, 0, sjd_launch_embed(m, idv, emb_rows, rows, one, kv->x, kv->x24, kv->ssq, errv, false, s));
        SJD_TRY(forward_rows_f32(m, kv, rows, rows_valid, stream,
                                 logits + (stream_mode == 2 && stream ? ((size_t)1 << cfg_shift(rows)) * m->V_s : 0), s));
    }
    return SJD_OK;
}

// n lives on the device; the host keeps an upper bound and only synchronises to refresh it when
// the bound (not necessarily n itself) would run past max_seq.
static int check_room(sjd_kv *kv, int32_t L)
{
    const int ms = kv->m->cfg.max_seq;
    if (kv->n_upper + L <= ms && (!kv->cfg_on || kv->n_upper_u + L <= ms)) return SJD_OK;
    SjdState st;
    SJD_TRY(state_read(kv, &st));
    kv->n_upper = st.n;
    kv->n_upper_u = st.n_u;
    if (st.n + L > ms || (kv->cfg_on && st.n_u + L > ms)) return SJD_ESEQ;
    return SJD_OK;
}

__global__ void clear_done_kernel(SjdState *st) { st->done = 0; }

extern "C" int sjd_forward_logits(sjd_model *m, sjd_kv *kv, const int32_t *tokens, int32_t L, float *logits, void *stream)
{
    if (!m || !kv || kv->m != m || !tokens || !logits || L < 1) return SJD_EINVAL;
    if (L > rows_max(m) / (kv->cfg_on ? 2 : 1)) return SJD_EINVAL;
    SJD_TRY(check_room(kv, L));
    hipStream_t s = (hipStream_t)stream;
    SJD_LAUNCH(clear_done_kernel, dim3(1), dim3(1), 0, s, kv->state);
    HIP_TRY(hipGetLastError());
    if (!kv->cfg_on) return forward_window(m, kv, tokens, nullptr, L, L, 0, logits, s);
    SJD_TRY(forward_window(m, kv, tokens, nullptr, L, L, 2, kv->logits, s));
    return sjd_launch_guide(kv->logits, kv->logits + ((size_t)1 << cfg_shift(L)) * m->V_s, kv->cfg_scale, (size_t)L * m->V_s,
                            logits, s);
}

// rows appended to stream `stream`; the ids of stream 0 are recorded for the repeat initialisers
__global__ void advance_n_kernel(SjdState *st, int32_t *tokens, const int32_t *ids, int rows, int stream)
{
    if (stream) {
        if (threadIdx.x == 0) st->n_u += rows;
        return;
    }
    const int n = st->n;
    for (int r = threadIdx.x; r < rows; r += blockDim.x) tokens[n + r] = ids ? ids[r] : -1;
    __syncthreads();
    if (threadIdx.x == 0) st->n = n + rows;
}

__global__ void forced_first_kernel(int32_t *forced, sjd_init init, int lo)
{
    forced[0] = (init.eol_id >= 0 && init.row_stride == 1) ? init.eol_id - lo : -1;
}

// the prompt of one stream, in chunks of up to SJD_ROWS_MAX positions; leaves the raw logits of the
// last position in kv->logits row *rows_last - 1
static int prefill_stream(sjd_model *m, sjd_kv *kv, int32_t stream_id, const int32_t *ids, int32_t n_ids,
                          const float *embeds, int32_t n_embeds, int *rows_last, hipStream_t s)
{
    const int P = n_ids + n_embeds, d = m->cfg.d_model;
    const int chunk = rows_max(m);
    for (int p0 = 0; p0 < P; p0 += chunk) {
        const int rows = std::min(chunk, P - p0);
        const int id_rows = std::max(0, std::min(rows, n_ids - p0));   // leading rows that are ids
        // a chunk is either all ids or all embedding rows; split mixed chunks
        int done_rows = 0;
        while (done_rows < rows) {
            int cnt; bool is_id = (p0 + done_rows) < n_ids;
            cnt = is_id ? (id_rows - done_rows) : (rows - done_rows);
            if (is_id) {
                HIP_TRY(hipMemcpyAsync(kv->ids_stage, ids + p0 + done_rows, (size_t)cnt * 4, hipMemcpyHostToDevice, s));
                HIP_TRY(hipStreamSynchronize(s));
                SJD_TRY(forward_window(m, kv, kv->ids_stage, nullptr, cnt, cnt, stream_id, kv->logits, s));
            } else {
                HIP_TRY(hipMemcpyAsync(kv->emb_stage, embeds + (size_t)(p0 + done_rows - n_ids) * d, (size_t)cnt * d * 4,
                                       hipMemcpyHostToDevice, s));
                HIP_TRY(hipStreamSynchronize(s));
                SJD_TRY(forward_window(m, kv, nullptr, kv->emb_stage, cnt, cnt, stream_id, kv->logits, s));
            }
            SJD_LAUNCH(advance_n_kernel, dim3(1), dim3(64), 0, s, kv->state, kv->tokens,
                               is_id ? kv->ids_stage : (const int32_t *)nullptr, cnt, stream_id);
            HIP_TRY(hipGetLastError());
            HIP_TRY(hipStreamSynchronize(s));   // staging buffers are reused by the next chunk
            if (stream_id) kv->n_upper_u += cnt; else kv->n_upper += cnt;
            done_rows += cnt;
            *rows_last = cnt;
        }
    }
    return SJD_OK;
}

static int check_prompt(const sjd_model *m, const int32_t *ids, int32_t n_ids, const float *embeds, int32_t n_embeds)
{
    if (n_ids < 0 || n_embeds < 0 || n_ids + n_embeds < 1) return SJD_EINVAL;
    if ((n_ids && !ids) || (n_embeds && !embeds)) return SJD_EINVAL;
    if (n_ids + n_embeds + 1 > m->cfg.max_seq) return SJD_ESEQ;
    for (int i = 0; i < n_ids; ++i) if (ids[i] < 0 || ids[i] >= m->cfg.vocab_total) return SJD_EINVAL;
    return SJD_OK;
}

extern "C" int sjd_prefill(sjd_model *m, sjd_kv *kv, const int32_t *ids, int32_t n_ids, const float *embeds,
                           int32_t n_embeds, const sjd_sampler *smp, const sjd_init *init, float *q_last, void *stream)
{
    if (!m || !kv || kv->m != m || !smp || !q_last) return SJD_EINVAL;
    if (smp->top_k < 1 || !(smp->temperature >= 0.f)) return SJD_EINVAL;
    SJD_TRY(check_prompt(m, ids, n_ids, embeds, n_embeds));
    hipStream_t s = (hipStream_t)stream;
    SJD_TRY(sjd_kv_reset(kv));          // also switches guidance off
    int rows_last = 0;
    SJD_TRY(prefill_stream(m, kv, 0, ids, n_ids, embeds, n_embeds, &rows_last, s));
    HIP_TRY(hipMemcpyAsync(kv->logits_last, kv->logits + (size_t)(rows_last - 1) * m->V_s, (size_t)m->V_s * 4,
                           hipMemcpyDeviceToDevice, s));
    // distribution of the first image token from the last prompt row
    sjd_init ini = init ? *init : sjd_init{0, 0, -1, 0};
    SJD_LAUNCH(forced_first_kernel, dim3(1), dim3(1), 0, s, kv->forced, ini, m->cfg.samp_lo);
    HIP_TRY(hipGetLastError());
    return sjd_launch_dist(kv->logits_last, nullptr, 0.f, 1, m->V_s, smp, kv->forced, q_last, s);
}

static int alloc_uncond_cache(sjd_kv *kv)
{
    const sjd_config &c = kv->m->cfg;
    // same layout as the first cache: bf16 K and V blocked together, fp32 K and V apart
    if (!kv->k_u) SJD_TRY(dev_alloc(&kv->k_u, (size_t)c.n_layers * kv->k_layer_stride * (c.dtype == 1 ? 2 : 4)));
    if (c.dtype == 0 && !kv->v_u) SJD_TRY(dev_alloc(&kv->v_u, (size_t)c.n_layers * kv->v_layer_stride * 4));
    // the table of the handle's two contexts, read by the kernels of a two-stream forward
    const SjdStreamEntry two[2] = {handle_entry(kv, false), handle_entry(kv, true)};
    HIP_TRY(hipMemcpy(kv->cfg_tab, two, sizeof(two), hipMemcpyHostToDevice));
    return SJD_OK;
}

extern "C" int sjd_prefill_uncond(sjd_model *m, sjd_kv *kv, const int32_t *ids, int32_t n_ids, const float *embeds,
                                  int32_t n_embeds, float guidance, const sjd_sampler *smp, const sjd_init *init,
                                  float *q_last, void *stream)
{
    if (!m || !kv || kv->m != m || !smp || !q_last || !(guidance == guidance)) return SJD_EINVAL;
    if (smp->top_k < 1 || !(smp->temperature >= 0.f)) return SJD_EINVAL;
    if (kv->n_upper < 1 || kv->cfg_on || kv->dec_active) return SJD_EINVAL;    // right after sjd_prefill only
    SJD_TRY(check_prompt(m, ids, n_ids, embeds, n_embeds));
    hipStream_t s = (hipStream_t)stream;
    SJD_TRY(alloc_uncond_cache(kv));
    int rows_last = 0;
    SJD_TRY(prefill_stream(m, kv, 1, ids, n_ids, embeds, n_embeds, &rows_last, s));
    kv->cfg_on = 1;
    kv->cfg_scale = guidance;
    sjd_init ini = init ? *init : sjd_init{0, 0, -1, 0};
    SJD_LAUNCH(forced_first_kernel, dim3(1), dim3(1), 0, s, kv->forced, ini, m->cfg.samp_lo);
    HIP_TRY(hipGetLastError());
    return sjd_launch_dist(kv->logits_last, kv->logits + (size_t)(rows_last - 1) * m->V_s, guidance, 1, m->V_s, smp,
                           kv->forced, q_last, s);
}

extern "C" int sjd_first_window(const sjd_model *m, const float *q_first, int32_t L, const sjd_init *init,
                                uint64_t philox_seed, int32_t *draft, float *p_old, void *stream)
{
    if (!m || !q_first || !init || !draft || !p_old || L < 1 || L > window_max(m, false)) return SJD_EINVAL;
    if (init->mode < 0 || init->mode > 4 || ((init->mode == 1 || init->mode == 4) && init->row_stride < 1)) return SJD_EINVAL;
    return sjd_launch_first_window(q_first, L, m->V_s, m->cfg.samp_lo, init, philox_seed, draft, p_old, (hipStream_t)stream);
}

static int check_sampling(const sjd_sampler *smp, const sjd_init *init, int lo, int hi)
{
    if (!smp || !init) return SJD_EINVAL;
    if (smp->top_k < 1 || !(smp->temperature >= 0.f)) return SJD_EINVAL;
    if (init->mode < 0 || init->mode > 4 || (init->flags & ~SJD_INIT_NO_REFINE)) return SJD_EINVAL;
    if ((init->mode == 1 || init->mode == 4) && init->row_stride < 1) return SJD_EINVAL;
    if (init->eol_id >= 0 && (init->eol_id < lo || init->eol_id >= hi || init->row_stride < 1)) return SJD_EINVAL;
    return SJD_OK;
}

__global__ void set_step_kernel(SjdState *st, int img_pos0, uint64_t counter, int L)
{
    st->img_pos0 = img_pos0; st->counter = counter; st->L_eff = L; st->n_image = 0; st->done = 0;
    // An image position beyond the cache length would make the repeat initialisers look for image
    // tokens in front of the cache's id record: the step is not executed (its verification kernels
    // see a finished generation and return) and the handle reports the error when its state is read.
    if (img_pos0 > st->n) { st->err = SJD_DEVERR_IMG_POS; st->done = 1; }
}

// initialiser (d) keeps the distributions of the last row_stride accepted image positions: a ring of
// SJD_RING_ROWS_DEFAULT rows comes with the handle; a wider grid makes sjd_decode_begin (which may
// allocate) replace it, while sjd_step (which never allocates) refuses with SJD_ELIMIT.
static int ensure_ring(sjd_kv *kv, const sjd_init *init, bool may_allocate)
{
    if (init->mode != 4 || kv->ring_rows >= init->row_stride) return SJD_OK;
    if (!may_allocate) {
        snprintf(g_limit_msg, sizeof(g_limit_msg), "sjd_step: initialiser (d) with row_stride %d needs a ring of that many rows, the "
                 "handle holds %d (sjd_decode_begin allocates a larger one)", init->row_stride, kv->ring_rows);
        return SJD_ELIMIT;
    }
    if (kv->ring) { HIP_TRY(hipDeviceSynchronize()); (void)hipFree(kv->ring); kv->ring = nullptr; kv->ring_rows = 0; }
    drop_graph(kv);                      // a captured iteration holds the old address
    SJD_TRY(dev_alloc((void **)&kv->ring, (size_t)init->row_stride * kv->m->V_s * 4));
    kv->ring_rows = init->row_stride;
    return SJD_OK;
}

// forward + verification of one window, everything stream-ordered, state device-resident
static int enqueue_step(sjd_model *m, sjd_kv *kv, const int32_t *draft, const float *p_old, int32_t L,
                        const sjd_sampler *smp, const sjd_init *init, uint64_t seed, int32_t *n_accepted,
                        int32_t *new_draft, float *p_new, hipStream_t s)
{
    SJD_TRY(forward_window(m, kv, draft, nullptr, L, L, kv->cfg_on ? 2 : 0, kv->logits, s));
    SjdVerifyArgs v;
    memset(&v, 0, sizeof(v));
    if (kv->cfg_on) { v.logits_u = kv->logits + ((size_t)1 << cfg_shift(L)) * m->V_s; v.cfg_scale = kv->cfg_scale; }
    v.logits = kv->logits; v.p_old = p_old; v.draft = draft; v.L = L; v.V = m->V_s; v.lo = m->cfg.samp_lo;
    v.smp = *smp; v.init = *init; v.seed = seed; v.state = kv->state; v.kv_tokens = kv->tokens;
    v.n_accepted = n_accepted; v.new_draft = new_draft; v.p_new = p_new; v.ring = kv->ring;
    v.q = kv->q; v.tok_smp = kv->tok_smp; v.tok_res = kv->tok_res; v.acc_flag = kv->acc_flag;
    v.draft_snap = kv->draft_snap; v.snap = kv->snap;
    PROF(kv, SJD_PROF_VERIFY, 3.0 * L * m->V_s * 4, sjd_launch_verify(&v, s));
    return SJD_OK;
}

extern "C" int sjd_step(sjd_model *m, sjd_kv *kv, const int32_t *draft, const float *p_old, int32_t L,
                        const sjd_sampler *smp, const sjd_init *init, int32_t img_pos0, uint64_t philox_seed,
                        uint64_t counter, int32_t *n_accepted, int32_t *new_draft, float *p_new, void *stream)
{
    if (!m || !kv || kv->m != m || !draft || !p_old || !n_accepted || !new_draft || !p_new) return SJD_EINVAL;
    if (L < 1 || L > window_max(m, kv->cfg_on) || img_pos0 < 0) return SJD_EINVAL;
    SJD_TRY(check_sampling(smp, init, m->cfg.samp_lo, m->cfg.samp_hi));
    if (img_pos0 > kv->n_upper) return SJD_EINVAL;       // (n_upper >= n: surely beyond the cache)
    SJD_TRY(check_room(kv, L));
    SJD_TRY(ensure_ring(kv, init, false));
    hipStream_t s = (hipStream_t)stream;
    kv->dec_active = 0;
    SJD_LAUNCH(set_step_kernel, dim3(1), dim3(1), 0, s, kv->state, img_pos0, counter, L);
    HIP_TRY(hipGetLastError());
    SJD_TRY(enqueue_step(m, kv, draft, p_old, L, smp, init, philox_seed, n_accepted, new_draft, p_new, s));
    kv->n_upper += L;
    kv->n_upper_u += L;
    return SJD_OK;
}

__global__ void begin_generate_kernel(SjdState *st, int N, int L)
{
    st->img_pos0 = 0; st->counter = 1; st->n_image = N; st->L_eff = L < N ? L : N; st->done = (N <= 1);
    st->steps = 0;
    for (int i = 0; i < 65; ++i) st->accept_hist[i] = 0;
}

// ---- device-resident decoding loop -----------------------------------------------------------
extern "C" int sjd_decode_begin(sjd_model *m, sjd_kv *kv, const float *q_first, int32_t N, int32_t L,
                                const sjd_sampler *smp, const sjd_init *init, uint64_t philox_seed, void *stream)
{
    if (!m || !kv || kv->m != m || !q_first || N < 1 || L < 1 || L > window_max(m, kv->cfg_on)) return SJD_EINVAL;
    SJD_TRY(check_sampling(smp, init, m->cfg.samp_lo, m->cfg.samp_hi));
    SJD_TRY(ensure_ring(kv, init, true));
    if (kv->n_upper + N + L > m->cfg.max_seq || (kv->cfg_on && kv->n_upper_u + N + L > m->cfg.max_seq)) {
        SjdState st;
        SJD_TRY(state_read(kv, &st));
        kv->n_upper = st.n; kv->n_upper_u = st.n_u;
        if (st.n + N + L > m->cfg.max_seq || (kv->cfg_on && st.n_u + N + L > m->cfg.max_seq)) return SJD_ESEQ;
    }
    hipStream_t s = (hipStream_t)stream;
    const bool same = kv->graph_exec && kv->dec_L == L && kv->dec_smp.top_k == smp->top_k &&
                      kv->dec_smp.temperature == smp->temperature && kv->dec_init.mode == init->mode &&
                      kv->dec_init.row_stride == init->row_stride && kv->dec_init.eol_id == init->eol_id &&
                      kv->dec_init.flags == init->flags && kv->dec_seed == philox_seed &&
                      kv->graph_cfg_on == kv->cfg_on && (!kv->cfg_on || kv->graph_cfg_scale == kv->cfg_scale);
    if (!same) drop_graph(kv);          // the captured step has these baked into its kernel arguments
    kv->dec_N = N; kv->dec_L = L; kv->dec_smp = *smp; kv->dec_init = *init; kv->dec_seed = philox_seed;
    kv->dec_active = 1;
    SJD_TRY(sjd_launch_first_window(q_first, L, m->V_s, m->cfg.samp_lo, init, philox_seed, kv->g_draft, kv->g_p, s));
    SJD_LAUNCH(begin_generate_kernel, dim3(1), dim3(1), 0, s, kv->state, N, L);
    HIP_TRY(hipGetLastError());
    kv->last_stream = s;
    kv->n_upper += N;                    // the loop never fixes more than N tokens
    kv->n_upper_u += N;
    return SJD_OK;
}

static int decode_one(sjd_model *m, sjd_kv *kv, hipStream_t s)
{
    return enqueue_step(m, kv, kv->g_draft, kv->g_p, kv->dec_L, &kv->dec_smp, &kv->dec_init, kv->dec_seed, kv->g_nacc,
                        kv->g_draft, kv->g_p, s);
}

extern "C" int sjd_decode_steps(sjd_model *m, sjd_kv *kv, int32_t n_steps, void *stream)
{
    if (!m || !kv || kv->m != m || n_steps < 0 || !kv->dec_active) return SJD_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    kv->last_stream = s;
    if (!kv->use_graph) {
        for (int i = 0; i < n_steps; ++i) SJD_TRY(decode_one(m, kv, s));
        return SJD_OK;
    }
    if (!kv->graph_exec) {
        // capture one iteration; everything that varies between iterations lives in device memory
        hipStream_t cs;
        HIP_TRY(hipStreamCreateWithFlags(&cs, hipStreamNonBlocking));
        hipError_t e = hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal);
        int rc = SJD_OK;
        if (e != hipSuccess) { sjd_set_hip_error(e, "hipStreamBeginCapture"); rc = SJD_EHIP; }
        if (rc == SJD_OK) rc = decode_one(m, kv, cs);
        hipGraph_t g = nullptr;
        e = hipStreamEndCapture(cs, &g);
        if (rc == SJD_OK && e != hipSuccess) { sjd_set_hip_error(e, "hipStreamEndCapture"); rc = SJD_EHIP; }
        (void)hipStreamDestroy(cs);
        kv->last_stream = s;
        if (rc != SJD_OK) { if (g) (void)hipGraphDestroy(g); return rc; }
        kv->graph = g;
        kv->graph_cfg_on = kv->cfg_on; kv->graph_cfg_scale = kv->cfg_scale;
        e = hipGraphInstantiate(&kv->graph_exec, g, nullptr, nullptr, 0);
        if (e != hipSuccess) { sjd_set_hip_error(e, "hipGraphInstantiate"); drop_graph(kv); return SJD_EHIP; }
    }
    kv->last_stream = s;                // (the capture above went through a stream of its own, gone by now)
    for (int i = 0; i < n_steps; ++i) HIP_TRY(hipGraphLaunch(kv->graph_exec, s));
    return SJD_OK;
}

// ---- batched decoding: B handles share every window forward --------------------------------------
// rows reserved per handle: the smallest power of two that holds the window, such that all fit in
// the 32 rows one projection launch computes
static int batch_shift(int32_t B, int32_t L)
{
    for (int shift = 0; shift <= 6; ++shift)
        if ((1 << shift) >= L) return (B << shift) <= SJD_ROWS_MAX ? shift : -1;
    return -1;
}

// streams of a batch: one per handle, two (conditional, unconditional) when the handles run guided
static int batch_stream_count(sjd_kv *const *kvs, int32_t B) { return kvs[0]->cfg_on ? 2 * B : B; }

// guided: 0 = the handles' guidance state does not matter (they are about to be pre-filled anew),
// 1 = all guided or none (with every guided handle's second cache in place)
static int check_batch(sjd_model *m, sjd_kv *const *kvs, int32_t B, int32_t L, bool decoding, int guided = 1)
{
    if (!m || !kvs || B < 1 || B > SJD_MAX_STREAMS || m->cfg.dtype != 1) return SJD_EINVAL;
    for (int b = 0; b < B; ++b) {
        sjd_kv *kv = kvs[b];
        if (!kv || kv->m != m) return SJD_EINVAL;
        if (guided && (kv->cfg_on != kvs[0]->cfg_on || (kv->cfg_on && !kv->k_u))) return SJD_EINVAL;
        for (int c = 0; c < b; ++c) if (kvs[c] == kv) return SJD_EINVAL;
        if (decoding) {
            const sjd_kv *k0 = kvs[0];
            if (!kv->dec_active || kv->dec_L != L) return SJD_EINVAL;
            if (kv->dec_smp.top_k != k0->dec_smp.top_k || kv->dec_smp.temperature != k0->dec_smp.temperature ||
                memcmp(&kv->dec_init, &k0->dec_init, sizeof(sjd_init)) != 0)
                return SJD_EINVAL;
        }
    }
    const int S = guided ? batch_stream_count(kvs, B) : B;
    if (S > SJD_MAX_STREAMS) return SJD_EINVAL;
    return batch_shift(S, L) < 0 ? SJD_EINVAL : SJD_OK;
}

// The table of the batch lives in the first handle; it is rewritten (after the stream has drained:
// kernels in flight may still read it) only when the set of handles changes.  Not to be called
// while a stream is being captured.
static int prepare_batch_table(sjd_kv *const *kvs, int32_t B, hipStream_t s)
{
    sjd_kv *kv0 = kvs[0];
    SjdStreamEntry want[SJD_MAX_STREAMS];
    memset(want, 0, sizeof(want));
    if (kv0->cfg_on) {
        for (int b = 0; b < B; ++b) { want[2 * b] = handle_entry(kvs[b], false); want[2 * b + 1] = handle_entry(kvs[b], true); }
    } else {
        for (int b = 0; b < B; ++b) want[b] = handle_entry(kvs[b], false);
    }
    if (memcmp(want, kv0->btab_host, sizeof(want)) == 0) return SJD_OK;
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipMemcpy(kv0->btab, want, sizeof(want), hipMemcpyHostToDevice));
    memcpy(kv0->btab_host, want, sizeof(want));
    return SJD_OK;
}

static SjdStreams batch_streams(sjd_kv *const *kvs, int32_t B, int32_t L)
{
    SjdStreams sm;
    memset(&sm, 0, sizeof(sm));
    sm.count = batch_stream_count(kvs, B); sm.shift = batch_shift(sm.count, L);
    sm.first = handle_entry(kvs[0], false);
    sm.table = kvs[0]->btab;
    return sm;
}

// one window forward for all handles: handle b's tokens ids[b] (device); its rows are rows b << shift of the
// first handle's activation buffers and of its logits buffer (guided: rows 2b << shift for the conditional
// context, (2b + 1) << shift for the unconditional one, both fed the same tokens)
static int forward_batch(sjd_model *m, sjd_kv *const *kvs, int32_t B, const int32_t *const *ids, int32_t L, hipStream_t s)
{
    sjd_kv *kv0 = kvs[0];
    const SjdStreams sm = batch_streams(kvs, B, L);
    const int per = kv0->cfg_on ? 2 : 1;
    const int32_t *ids_s[SJD_MAX_STREAMS] = {};
    int32_t *errv[SJD_MAX_STREAMS] = {};
    for (int b = 0; b < B; ++b) {
        for (int c = 0; c < per; ++c) { ids_s[per * b + c] = ids[b]; errv[per * b + c] = &kvs[b]->state->err; }
        kvs[b]->last_stream = s;
    }
    const bool lo16 = rows_use_lo16(((sm.count - 1) << sm.shift) + L);
    PROF(kv0, SJD_PROF_ELEMENTWISE, 0, sjd_launch_embed(m, ids_s, nullptr, L, sm, kv0->x, kv0->x24, kv0->ssq, errv, lo16, s));
    double toks = 0;
    for (int b = 0; b < B; ++b) toks += kvs[b]->n_upper + L + (kv0->cfg_on ? kvs[b]->n_upper_u + L : 0);
    if (kv0->prof) toks = kv0->prof_kv_tokens;
    return forward_rows_bf16(m, kv0, sm, L, L, toks, kv0->logits, s);
}

static int decode_one_batch(sjd_model *m, sjd_kv *const *kvs, int32_t B, hipStream_t s)
{
    sjd_kv *kv0 = kvs[0];
    const int L = kv0->dec_L, per = kv0->cfg_on ? 2 : 1, shift = batch_shift(per * B, L);
    const int32_t *ids[SJD_MAX_STREAMS] = {};
    for (int b = 0; b < B; ++b) ids[b] = kvs[b]->g_draft;
    SJD_TRY(forward_batch(m, kvs, B, ids, L, s));
    SjdVerifyArgs vs[SJD_MAX_STREAMS];
    memset(vs, 0, sizeof(vs));
    for (int b = 0; b < B; ++b) {
        sjd_kv *kv = kvs[b];
        SjdVerifyArgs &v = vs[b];
        v.logits = kv0->logits + ((size_t)(per * b) << shift) * m->V_s; v.p_old = kv->g_p; v.draft = kv->g_draft; v.L = L;
        if (per == 2) { v.logits_u = kv0->logits + ((size_t)(2 * b + 1) << shift) * m->V_s; v.cfg_scale = kv->cfg_scale; }
        v.V = m->V_s; v.lo = m->cfg.samp_lo; v.smp = kv->dec_smp; v.init = kv->dec_init; v.seed = kv->dec_seed;
        v.state = kv->state; v.kv_tokens = kv->tokens; v.n_accepted = kv->g_nacc; v.new_draft = kv->g_draft;
        v.p_new = kv->g_p; v.ring = kv->ring; v.q = kv->q; v.tok_smp = kv->tok_smp; v.tok_res = kv->tok_res;
        v.acc_flag = kv->acc_flag; v.draft_snap = kv->draft_snap; v.snap = kv->snap;
    }
    // Steps 3-4 of all B images side by side
    PROF(kv0, SJD_PROF_VERIFY, 3.0 * B * L * m->V_s * 4, sjd_launch_verify_batch(vs, B, s));
    return SJD_OK;
}

extern "C" int sjd_decode_steps_batch(sjd_model *m, sjd_kv *const *kvs, int32_t B, int32_t n_steps, void *stream)
{
    if (!kvs || B < 1 || !kvs[0] || n_steps < 0) return SJD_EINVAL;
    sjd_kv *kv0 = kvs[0];
    SJD_TRY(check_batch(m, kvs, B, kv0->dec_L, true));
    hipStream_t s = (hipStream_t)stream;
    SJD_TRY(prepare_batch_table(kvs, B, s));
    for (int b = 0; b < B; ++b) kvs[b]->last_stream = s;
    if (!kv0->use_graph) {
        for (int i = 0; i < n_steps; ++i) SJD_TRY(decode_one_batch(m, kvs, B, s));
        return SJD_OK;
    }
    sjd_kv::BatchKey key;
    memset(&key, 0, sizeof(key));
    key.B = B; key.L = kv0->dec_L; key.smp = kv0->dec_smp; key.init = kv0->dec_init;
    for (int b = 0; b < B; ++b) {
        key.kv[b] = kvs[b]; key.state[b] = kvs[b]->state; key.cache[b] = kvs[b]->k; key.ring[b] = kvs[b]->ring;
        key.seed[b] = kvs[b]->dec_seed;
        if (kv0->cfg_on) { key.cache_u[b] = kvs[b]->k_u; key.cfg_scale[b] = kvs[b]->cfg_scale; }
    }
    key.cfg_on = kv0->cfg_on;
    if (kv0->bgraph_exec && memcmp(&key, &kv0->bkey, sizeof(key)) != 0) drop_batch_graph(kv0);
    if (!kv0->bgraph_exec) {
        // one iteration of all handles; what varies between iterations lives in device memory
        hipStream_t cs;
        HIP_TRY(hipStreamCreateWithFlags(&cs, hipStreamNonBlocking));
        hipError_t e = hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal);
        int rc = SJD_OK;
        if (e != hipSuccess) { sjd_set_hip_error(e, "hipStreamBeginCapture"); rc = SJD_EHIP; }
        if (rc == SJD_OK) rc = decode_one_batch(m, kvs, B, cs);
        hipGraph_t g = nullptr;
        e = hipStreamEndCapture(cs, &g);
        if (rc == SJD_OK && e != hipSuccess) { sjd_set_hip_error(e, "hipStreamEndCapture"); rc = SJD_EHIP; }
        (void)hipStreamDestroy(cs);
        for (int b = 0; b < B; ++b) kvs[b]->last_stream = s;
        if (rc != SJD_OK) { if (g) (void)hipGraphDestroy(g); return rc; }
        kv0->bgraph = g;
        e = hipGraphInstantiate(&kv0->bgraph_exec, g, nullptr, nullptr, 0);
        if (e != hipSuccess) { sjd_set_hip_error(e, "hipGraphInstantiate"); drop_batch_graph(kv0); return SJD_EHIP; }
        memcpy(&kv0->bkey, &key, sizeof(key));    // byte copy: the comparison above is one too
    }
    for (int b = 0; b < B; ++b) kvs[b]->last_stream = s;     // (the capture above went through a stream of its own)
    for (int i = 0; i < n_steps; ++i) HIP_TRY(hipGraphLaunch(kv0->bgraph_exec, s));
    return SJD_OK;
}

struct DoneFlags { int32_t *p[SJD_MAX_STREAMS]; int32_t count; };
__global__ void clear_done_batch_kernel(DoneFlags f)
{
    if ((int)threadIdx.x < f.count) *f.p[threadIdx.x] = 0;
}

extern "C" int sjd_forward_logits_batch(sjd_model *m, sjd_kv *const *kvs, int32_t B, const int32_t *tokens, int32_t L,
                                        float *logits, void *stream)
{
    if (!tokens || !logits || L < 1) return SJD_EINVAL;
    SJD_TRY(check_batch(m, kvs, B, L, false));
    for (int b = 0; b < B; ++b) SJD_TRY(check_room(kvs[b], L));
    hipStream_t s = (hipStream_t)stream;
    SJD_TRY(prepare_batch_table(kvs, B, s));
    const SjdStreams sm = batch_streams(kvs, B, L);
    // a handle that is not inside a generation computes regardless of how its last one ended; one that
    // is keeps its finished flag (its rows are skipped once its image is complete)
    DoneFlags idle;
    memset(&idle, 0, sizeof(idle));
    for (int b = 0; b < B; ++b) if (!kvs[b]->dec_active) idle.p[idle.count++] = &kvs[b]->state->done;
    if (idle.count) {
        SJD_LAUNCH(clear_done_batch_kernel, dim3(1), dim3(64), 0, s, idle);
        HIP_TRY(hipGetLastError());
    }
    const int32_t *ids[SJD_MAX_STREAMS] = {};
    for (int b = 0; b < B; ++b) ids[b] = tokens + (size_t)b * L;
    SJD_TRY(forward_batch(m, kvs, B, ids, L, s));
    // rows b << shift .. of the shared logits buffer -> [B][L][V_s] (guided: the two contexts' rows combined)
    const size_t V = m->V_s;
    for (int b = 0; b < B; ++b) {
        if (kvs[0]->cfg_on) {
            SJD_TRY(sjd_launch_guide(kvs[0]->logits + ((size_t)(2 * b) << sm.shift) * V, kvs[0]->logits + ((size_t)(2 * b + 1) << sm.shift) * V,
                                     kvs[b]->cfg_scale, (size_t)L * V, logits + (size_t)b * L * V, s));
        } else {
            HIP_TRY(hipMemcpyAsync(logits + (size_t)b * L * V, kvs[0]->logits + ((size_t)b << sm.shift) * V, (size_t)L * V * 4,
                                   hipMemcpyDeviceToDevice, s));
        }
    }
    return SJD_OK;
}

extern "C" int sjd_generate_batch(sjd_model *m, sjd_kv *const *kvs, int32_t B, const int32_t *const *ids,
                                  const int32_t *n_ids, const float *const *embeds, const int32_t *n_embeds, int32_t N,
                                  int32_t L, const sjd_sampler *smp, const sjd_init *init, const uint64_t *philox_seeds,
                                  int32_t *out_tokens, sjd_stats *stats)
{
    if (!ids || !n_ids || !philox_seeds || !out_tokens || N < 1) return SJD_EINVAL;
    SJD_TRY(check_batch(m, kvs, B, L, false, 0));       // (every handle is pre-filled anew below, which ends guidance)
    SJD_TRY(check_sampling(smp, init, m->cfg.samp_lo, m->cfg.samp_hi));
    for (int b = 0; b < B; ++b)
        if (n_ids[b] + (n_embeds ? n_embeds[b] : 0) + N + L > m->cfg.max_seq) return SJD_ESEQ;
    hipStream_t s = 0;
    auto t0 = std::chrono::steady_clock::now();
    for (int b = 0; b < B; ++b) {
        sjd_kv *kv = kvs[b];
        SJD_TRY(sjd_prefill(m, kv, ids[b], n_ids[b], embeds ? embeds[b] : nullptr, n_embeds ? n_embeds[b] : 0, smp, init,
                            kv->q_first, s));
        SJD_TRY(sjd_decode_begin(m, kv, kv->q_first, N, L, smp, init, philox_seeds[b], s));
    }
    HIP_TRY(hipStreamSynchronize(s));
    auto t1 = std::chrono::steady_clock::now();
    // iterations are enqueued a few at a time, never more than the image furthest from its end can
    // still take; a handle whose image is complete sits out the rest (its rows are still computed, its
    // attention and verification kernels return at once)
    int enq = 0, all_done = 0, most_left = N - 1;
    while (!all_done) {
        const int k = std::max(1, std::min(8, (most_left + L - 1) / L));
        SJD_TRY(sjd_decode_steps_batch(m, kvs, B, k, s));
        enq += k;
        all_done = 1;
        most_left = 0;
        for (int b = 0; b < B; ++b) {
            int done = 0, fixed = 0;
            SJD_TRY(sjd_decode_status(kvs[b], &fixed, nullptr, &done));
            all_done &= done;
            if (!done) most_left = std::max(most_left, N - 1 - fixed);
        }
        if (enq > 4 * (N + 8)) {                  // cannot happen: every iteration fixes at least one token per image
            snprintf(g_hip_msg, sizeof(g_hip_msg), "sjd_generate_batch: %d iterations enqueued without finishing %d tokens", enq, N);
            return SJD_EHIP;
        }
    }
    auto t2 = std::chrono::steady_clock::now();
    for (int b = 0; b < B; ++b) {
        sjd_stats *st = stats ? stats + b : nullptr;
        SJD_TRY(sjd_decode_result(kvs[b], out_tokens + (size_t)b * N, st));
        if (st) {
            st->ms_prefill = std::chrono::duration<float, std::milli>(t1 - t0).count();
            st->ms_decode = std::chrono::duration<float, std::milli>(t2 - t1).count();
        }
    }
    return SJD_OK;
}

extern "C" int sjd_decode_status(sjd_kv *kv, int32_t *n_fixed, int32_t *steps, int32_t *done)
{
    if (!kv) return SJD_EINVAL;
    SjdState st;
    SJD_TRY(state_read(kv, &st));
    if (n_fixed) *n_fixed = st.img_pos0;
    if (steps) *steps = st.steps;
    if (done) *done = st.done;
    return SJD_OK;
}

extern "C" int sjd_decode_result(sjd_kv *kv, int32_t *out_tokens, sjd_stats *stats)
{
    if (!kv || !kv->dec_active || !out_tokens) return SJD_EINVAL;
    SjdState st;
    SJD_TRY(state_read(kv, &st));
    if (!st.done) return SJD_EINVAL;
    const int N = kv->dec_N, P = st.n - st.img_pos0;
    // image tokens = cache ids P .. ; when N-1 were fixed the pending exact slot 0 is the last one
    const int fixed = st.img_pos0 < N ? st.img_pos0 : N;
    HIP_TRY(hipMemcpy(out_tokens, kv->tokens + P, (size_t)fixed * 4, hipMemcpyDeviceToHost));
    if (fixed < N) HIP_TRY(hipMemcpy(out_tokens + fixed, kv->g_draft, 4, hipMemcpyDeviceToHost));
    if (stats) {
        stats->steps = st.steps;
        for (int i = 0; i < 65; ++i) stats->accept_hist[i] = st.accept_hist[i];
    }
    return SJD_OK;
}

extern "C" int sjd_kv_use_graph(sjd_kv *kv, int32_t on)
{
    if (!kv) return SJD_EINVAL;
    kv->use_graph = on ? 1 : 0;
    return SJD_OK;
}

static int generate_common(sjd_model *m, sjd_kv *kv, const int32_t *ids, int32_t n_ids, const float *embeds,
                           int32_t n_embeds, bool guided, const int32_t *u_ids, int32_t n_u_ids, const float *u_embeds,
                           int32_t n_u_embeds, float guidance, int32_t N, int32_t L, const sjd_sampler *smp,
                           const sjd_init *init, uint64_t philox_seed, int32_t *out_tokens, sjd_stats *stats)
{
    if (!m || !kv || kv->m != m || !out_tokens || N < 1 || L < 1 || L > window_max(m, guided)) return SJD_EINVAL;
    SJD_TRY(check_sampling(smp, init, m->cfg.samp_lo, m->cfg.samp_hi));
    if (n_ids + n_embeds + N + L > m->cfg.max_seq) return SJD_ESEQ;
    if (guided && n_u_ids + n_u_embeds + N + L > m->cfg.max_seq) return SJD_ESEQ;
    hipStream_t s = 0;
    auto t0 = std::chrono::steady_clock::now();
    SJD_TRY(sjd_prefill(m, kv, ids, n_ids, embeds, n_embeds, smp, init, kv->q_first, s));
    if (guided) SJD_TRY(sjd_prefill_uncond(m, kv, u_ids, n_u_ids, u_embeds, n_u_embeds, guidance, smp, init, kv->q_first, s));
    SJD_TRY(sjd_decode_begin(m, kv, kv->q_first, N, L, smp, init, philox_seed, s));
    HIP_TRY(hipStreamSynchronize(s));
    auto t1 = std::chrono::steady_clock::now();
    // Iterations are enqueued a few at a time, never more than the image can still take (an iteration
    // fixes at most L tokens): the forward of an iteration past the end would be wasted work.
    int enq = 0, done = 0, fixed = 0;
    while (!done) {
        const int k = std::max(1, std::min(8, (N - 1 - fixed + L - 1) / L));
        SJD_TRY(sjd_decode_steps(m, kv, k, s));
        enq += k;
        SJD_TRY(sjd_decode_status(kv, &fixed, nullptr, &done));
        if (enq > 4 * (N + 8)) {                  // cannot happen: every iteration fixes at least one token
            snprintf(g_hip_msg, sizeof(g_hip_msg), "sjd_generate: %d iterations enqueued without finishing %d tokens", enq, N);
            return SJD_EHIP;
        }
    }
    auto t2 = std::chrono::steady_clock::now();
    SJD_TRY(sjd_decode_result(kv, out_tokens, stats));
    if (stats) {
        stats->ms_prefill = std::chrono::duration<float, std::milli>(t1 - t0).count();
        stats->ms_decode = std::chrono::duration<float, std::milli>(t2 - t1).count();
    }
    return SJD_OK;
}

extern "C" int sjd_generate(sjd_model *m, sjd_kv *kv, const int32_t *ids, int32_t n_ids, const float *embeds,
                            int32_t n_embeds, int32_t N, int32_t L, const sjd_sampler *smp, const sjd_init *init,
                            uint64_t philox_seed, int32_t *out_tokens, sjd_stats *stats)
{
    return generate_common(m, kv, ids, n_ids, embeds, n_embeds, false, nullptr, 0, nullptr, 0, 0.f, N, L, smp, init,
                           philox_seed, out_tokens, stats);
}

extern "C" int sjd_generate_cfg(sjd_model *m, sjd_kv *kv, const int32_t *ids, int32_t n_ids, const float *embeds,
                                int32_t n_embeds, const int32_t *uncond_ids, int32_t n_uncond_ids,
                                const float *uncond_embeds, int32_t n_uncond_embeds, float guidance, int32_t N, int32_t L,
                                const sjd_sampler *smp, const sjd_init *init, uint64_t philox_seed, int32_t *out_tokens,
                                sjd_stats *stats)
{
    return generate_common(m, kv, ids, n_ids, embeds, n_embeds, true, uncond_ids, n_uncond_ids, uncond_embeds,
                           n_uncond_embeds, guidance, N, L, smp, init, philox_seed, out_tokens, stats);
}

// ---- per-kernel-class timing of eager iterations (HIP events on the launch stream) ------------
// kvs[0] carries the profiler; B == 0: the single-handle iteration of kvs[0]
static int profile_steps(sjd_model *m, sjd_kv *const *kvs, int32_t B, int32_t n_steps, sjd_profile *out, hipStream_t s)
{
    sjd_kv *kv = kvs[0];
    auto one = [&]() { return B ? decode_one_batch(m, kvs, B, s) : decode_one(m, kv, s); };
    memset(out, 0, sizeof(*out));
    SjdProfiler prof;
    prof.hook.next = SjdProfiler::next; prof.hook.self = &prof; prof.hook.cur_kind = 0; prof.hook.only_kind = -1;
    kv->prof = &prof;
    sjd_launch_hook = &prof.hook;
    int rc = SJD_OK;
    for (int i = 0; i < n_steps && rc == SJD_OK; ++i) {
        // cached positions this iteration's attention reads, from the device-resident lengths (every
        // stream: its cache plus the window rows; a finished image reads nothing)
        double toks = 0;
        for (int b = 0; b < (B ? B : 1) && rc == SJD_OK; ++b) {
            SjdState st;
            rc = state_read(kvs[b], &st);
            if (rc == SJD_OK && !st.done) toks += st.n + st.L_eff + (kvs[b]->cfg_on ? st.n_u + st.L_eff : 0);
        }
        kv->prof_kv_tokens = toks;
        if (rc == SJD_OK) rc = one();
        if (rc == SJD_OK) rc = prof.drain(out, s);
    }
    // second pass: the projections of n_steps iterations alone, back to back, inside one event pair
    // (the other kernels are skipped, so the loop state does not advance and the projections run on
    // whatever the buffers hold; the next real iteration overwrites all of it)
    if (rc == SJD_OK) {
        hipEvent_t e0 = nullptr, e1 = nullptr;
        prof.hook.next = nullptr; prof.hook.only_kind = SJD_PROF_GEMM;
        if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) rc = SJD_EHIP;
        if (rc == SJD_OK) rc = one();                                      // warm-up
        if (rc == SJD_OK && hipEventRecord(e0, s) != hipSuccess) rc = SJD_EHIP;
        for (int i = 0; i < n_steps && rc == SJD_OK; ++i) rc = one();
        if (rc == SJD_OK && hipEventRecord(e1, s) != hipSuccess) rc = SJD_EHIP;
        if (rc == SJD_OK && hipEventSynchronize(e1) != hipSuccess) rc = SJD_EHIP;
        float ms = 0.f;
        if (rc == SJD_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = SJD_EHIP;
        out->ms_gemm_back_to_back = ms;
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
    sjd_launch_hook = nullptr;
    kv->prof = nullptr;
    prof.destroy();
    out->steps = n_steps;
    return rc;
}

extern "C" int sjd_profile_steps(sjd_model *m, sjd_kv *kv, int32_t n_steps, sjd_profile *out, void *stream)
{
    if (!m || !kv || kv->m != m || n_steps < 1 || !out || !kv->dec_active) return SJD_EINVAL;
    sjd_kv *one[1] = {kv};
    return profile_steps(m, one, 0, n_steps, out, (hipStream_t)stream);
}

extern "C" int sjd_profile_steps_batch(sjd_model *m, sjd_kv *const *kvs, int32_t B, int32_t n_steps, sjd_profile *out,
                                       void *stream)
{
    if (!kvs || B < 1 || !kvs[0] || n_steps < 1 || !out) return SJD_EINVAL;
    SJD_TRY(check_batch(m, kvs, B, kvs[0]->dec_L, true));
    SJD_TRY(prepare_batch_table(kvs, B, (hipStream_t)stream));
    return profile_steps(m, kvs, B, n_steps, out, (hipStream_t)stream);
}

// ---- hooks ----------------------------------------------------------------------------------
struct Scratch {
    float *q = nullptr; int32_t *ints = nullptr; void *snap = nullptr;
    ~Scratch() { if (q) (void)hipFree(q); if (ints) (void)hipFree(ints); if (snap) (void)hipFree(snap); }
};

static int verify_common(const float *logits, const float *q_in, const float *p_old, const int32_t *draft, int32_t L,
                         int32_t V, int32_t lo, const sjd_sampler *smp, const sjd_init *init, int32_t img_pos0,
                         const int32_t *hist, float *ring, uint64_t seed, uint64_t counter, int32_t *n_accepted,
                         int32_t *new_draft, float *p_new, hipStream_t s)
{
    if (!p_old || !draft || !n_accepted || !new_draft || !p_new || !init) return SJD_EINVAL;
    if (init->mode == 4 && !ring) return SJD_EINVAL;
    if (L < 1 || L > SJD_MAX_WINDOW || V < 1 || V > SJD_MAX_SAMP_VOCAB || img_pos0 < 0) return SJD_EINVAL;
    sjd_sampler sm = smp ? *smp : sjd_sampler{1, 1.0f};
    SJD_TRY(check_sampling(&sm, init, lo, lo + V));
    if ((init->mode == 1 || init->mode == 2) && img_pos0 > 0 && !hist) return SJD_EINVAL;
    Scratch sc;
    SJD_TRY(dev_alloc((void **)&sc.q, (size_t)(L + 1) * V * 4));
    SJD_TRY(dev_alloc((void **)&sc.ints, (size_t)(L + 1) * 4 * 4));
    SJD_TRY(dev_alloc(&sc.snap, 64));
    SjdVerifyArgs v;
    memset(&v, 0, sizeof(v));
    v.logits = logits; v.q_in = q_in; v.p_old = p_old; v.draft = draft; v.L = L; v.V = V; v.lo = lo;
    v.smp = sm; v.init = *init; v.hist = hist; v.ring = ring; v.seed = seed; v.img_pos0 = img_pos0; v.counter = counter;
    v.n_accepted = n_accepted; v.new_draft = new_draft; v.p_new = p_new; v.q = sc.q;
    v.tok_smp = sc.ints; v.tok_res = sc.ints + (L + 1); v.acc_flag = sc.ints + 2 * (L + 1);
    v.draft_snap = sc.ints + 3 * (L + 1); v.snap = sc.snap;
    SJD_TRY(sjd_launch_verify(&v, s));
    HIP_TRY(hipStreamSynchronize(s));   // scratch is freed on return
    return SJD_OK;
}

extern "C" int sjd_verify(const float *logits, const float *p_old, const int32_t *draft, int32_t L, int32_t V_s,
                          int32_t samp_lo, const sjd_sampler *smp, const sjd_init *init, int32_t img_pos0,
                          const int32_t *hist, float *ring, uint64_t philox_seed, uint64_t counter,
                          int32_t *n_accepted, int32_t *new_draft, float *p_new, void *stream)
{
    if (!logits || !smp) return SJD_EINVAL;
    return verify_common(logits, nullptr, p_old, draft, L, V_s, samp_lo, smp, init, img_pos0, hist, ring, philox_seed, counter,
                         n_accepted, new_draft, p_new, (hipStream_t)stream);
}

extern "C" int sjd_verify_probs(const float *q, const float *p_old, const int32_t *draft, int32_t L, int32_t V_s,
                                int32_t samp_lo, const sjd_init *init, int32_t img_pos0, const int32_t *hist,
                                float *ring, uint64_t philox_seed, uint64_t counter, int32_t *n_accepted,
                                int32_t *new_draft, float *p_new, void *stream)
{
    if (!q) return SJD_EINVAL;
    return verify_common(nullptr, q, p_old, draft, L, V_s, samp_lo, nullptr, init, img_pos0, hist, ring, philox_seed, counter,
                         n_accepted, new_draft, p_new, (hipStream_t)stream);
}

// ---- Step 3 + Step 4 for callers that cannot allocate ------------------------------------------
// sjd_verify_static keeps what sjd_verify allocates per call (the distributions q[(L+1) x V_s], the
// per-index candidates and flags, the frozen step scalars) in one file-scope device array.  In host
// code the array's name is only a handle for the runtime: its device address is looked up once per
// device with hipGetSymbolAddress and that pointer is what the kernels are given.
struct VerifyStatic {
    float q[SJD_STATIC_VERIFY_FLOATS];
    int32_t ints[4 * (SJD_MAX_WINDOW + 1)];
    unsigned char snap[64];
};
static __device__ __align__(256) unsigned char scratch[sizeof(VerifyStatic)];
#define SJD_MAX_DEVICES 64
static VerifyStatic *g_scratch_ptr[SJD_MAX_DEVICES];     // per device: every GPU holds its own copy of the array
static std::mutex g_scratch_mutex;

static int static_scratch(VerifyStatic **out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= SJD_MAX_DEVICES) return SJD_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return SJD_EHIP;
        g_scratch_ptr[dev] = (VerifyStatic *)p;
    }
    *out = g_scratch_ptr[dev];
    return SJD_OK;
}

extern "C" int sjd_verify_static(const float *logits, const float *p_old, const int32_t *draft, int32_t L, int32_t V_s,
                                 int32_t samp_lo, const sjd_sampler *smp, const sjd_init *init, int32_t img_pos0,
                                 const int32_t *hist, float *ring, uint64_t philox_seed, uint64_t counter,
                                 int32_t *n_accepted, int32_t *new_draft, float *p_new, void *stream)
{
    if (!logits || !smp || !p_old || !draft || !n_accepted || !new_draft || !p_new || !init) return SJD_EINVAL;
    if (init->mode == 4 && !ring) return SJD_EINVAL;
    if (L < 1 || L > SJD_MAX_WINDOW || V_s < 1 || V_s > SJD_MAX_SAMP_VOCAB || img_pos0 < 0) return SJD_EINVAL;
    if ((size_t)(L + 1) * V_s > SJD_STATIC_VERIFY_FLOATS) {
        snprintf(g_limit_msg, sizeof(g_limit_msg), "sjd_verify_static: (L + 1) * V_s = %zu exceeds the static scratch of %d floats",
                 (size_t)(L + 1) * V_s, SJD_STATIC_VERIFY_FLOATS);
        return SJD_ELIMIT;
    }
    SJD_TRY(check_sampling(smp, init, samp_lo, samp_lo + V_s));
    if ((init->mode == 1 || init->mode == 2) && img_pos0 > 0 && !hist) return SJD_EINVAL;
    VerifyStatic *sc = nullptr;
    SJD_TRY(static_scratch(&sc));
    // Nothing in the scratch has to start at zero: the first kernel writes every row, candidate, flag
    // and scalar the second one reads.  Calls that overlap on one GPU would share it and race.
    SjdVerifyArgs v;
    memset(&v, 0, sizeof(v));
    v.logits = logits; v.p_old = p_old; v.draft = draft; v.L = L; v.V = V_s; v.lo = samp_lo;
    v.smp = *smp; v.init = *init; v.hist = hist; v.ring = ring; v.seed = philox_seed; v.img_pos0 = img_pos0; v.counter = counter;
    v.n_accepted = n_accepted; v.new_draft = new_draft; v.p_new = p_new; v.q = sc->q;
    v.tok_smp = sc->ints; v.tok_res = sc->ints + (L + 1); v.acc_flag = sc->ints + 2 * (L + 1);
    v.draft_snap = sc->ints + 3 * (L + 1); v.snap = sc->snap;
    return sjd_launch_verify(&v, (hipStream_t)stream);
}

extern "C" int sjd_dist(const float *logits, int32_t rows, int32_t V_s, const sjd_sampler *smp, const int32_t *forced,
                        float *q, void *stream)
{
    if (!logits || !smp || !q || rows < 1) return SJD_EINVAL;
    if (smp->top_k < 1 || !(smp->temperature >= 0.f)) return SJD_EINVAL;
    return sjd_launch_dist(logits, nullptr, 0.f, rows, V_s, smp, forced, q, (hipStream_t)stream);
}

struct GemmScratch {
    void *Ap = nullptr, *Wp = nullptr, *part = nullptr; float *out = nullptr;
    ~GemmScratch() { for (void *p : {Ap, Wp, part, (void *)out}) if (p) (void)hipFree(p); }
};

extern "C" int sjd_gemm_test(int32_t dtype, const void *A, const void *W, int32_t M, int32_t N, int32_t K, float *C,
                             void *stream)
{
    if (!A || !W || !C || M < 1 || M > (dtype == 0 ? SJD_ROWS_F32 : SJD_ROWS_MAX) || N < 1 || K < 1) return SJD_EINVAL;
    if (dtype < 0 || dtype > 2) return SJD_EINVAL;
    if (dtype >= 1 && (N % 16 || K % 32)) return SJD_EINVAL;
    if (dtype == 0 && K % 4) return SJD_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const size_t es = elt_size(dtype);
    const bool wide = dtype >= 1 && M > SJD_ROWS_SKINNY;
    GemmScratch g;
    SJD_TRY(dev_alloc(&g.Ap, (size_t)SJD_ROWS_MAX * K * 4 + 2048));   // rows past M and the tile behind stay zero
    SJD_TRY(dev_alloc((void **)&g.out, (size_t)SJD_ROWS_MAX * N * 4));
    const size_t part_elems = wide ? (size_t)8 * SJD_ROWS_MAX * N : 0;      // (room for up to 8 K-slices)
    if (wide) SJD_TRY(dev_alloc(&g.part, part_elems * 4));
    SjdLinear lin;
    memset(&lin, 0, sizeof(lin));
    lin.N = N; lin.K = K; lin.tn = 1; lin.w = W;
    if (dtype >= 1) {
        // the wide kernel reads the 3-byte planes only (exact for bf16 values: their low byte is zero)
        if (dtype == 1 && !wide) SJD_TRY(sjd_bf16_rows_to_f32((const bf16_t *)A, M, K, (float *)g.Ap, s));
        else if (dtype == 1) SJD_TRY(sjd_bf16_rows_to_act24((const bf16_t *)A, M, K, g.Ap, s));
        else SJD_TRY(sjd_f32_rows_to_act24((const float *)A, M, K, g.Ap, wide, s));     // hi / lo planes
        SJD_TRY(dev_alloc(&g.Wp, (size_t)N * K * es));
        sjd_choose_tiles(&lin);
        SJD_TRY(sjd_repack_bf16((const bf16_t *)W, (bf16_t *)g.Wp, N, K, lin.tn, 0, 0, 0, s));
        lin.w = g.Wp;
        SjdGemmEpi ep;
        memset(&ep, 0, sizeof(ep));
        ep.kind = SJD_EPI_STORE; ep.out = g.out;
        SJD_TRY(sjd_launch_gemm_bf16(&lin, g.Ap, wide ? SJD_ACT_P4 : dtype == 2 ? SJD_ACT_P3 : SJD_ACT_F32, nullptr, 0.f, M, ep,
                                     (float *)g.part, part_elems, s));
    } else {
        HIP_TRY(hipMemcpyAsync(g.Ap, A, (size_t)M * K * es, hipMemcpyDeviceToDevice, s));
        SJD_TRY(sjd_launch_gemm(0, &lin, g.Ap, M, g.out, nullptr, s));
    }
    HIP_TRY(hipMemcpyAsync(C, g.out, (size_t)M * N * 4, hipMemcpyDeviceToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));
    return SJD_OK;
}

// The floor for a kernel that has to read `bytes` of weights: a plain streaming read of them (workgroup b takes
// a contiguous share, its four waves a quarter each, four 16-byte loads per lane in flight), nothing else.
typedef __attribute__((ext_vector_type(4))) float stream_f32x4;
__global__ __launch_bounds__(256) void stream_read_kernel(const stream_f32x4 *__restrict__ p, size_t per16, float *out,
                                                          int interleaved)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t q = per16 / 4;                       // 16-byte units per wave (a multiple of 64)
    const stream_f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    stream_f32x4 acc = zero;
    if (interleaved) {
        // all workgroups sweep the buffer together: round r, workgroup b, wave w reads the 4 KiB chunk (r * grid + b) * 4 + w
        const size_t rounds = q / 256;
        for (size_t r = 0; r < rounds; ++r) {
            const stream_f32x4 *src = p + (((r * gridDim.x + blockIdx.x) * 4 + wave) * 256) + lane;
            const stream_f32x4 a = __builtin_nontemporal_load(src), b = __builtin_nontemporal_load(src + 64);
            const stream_f32x4 c = __builtin_nontemporal_load(src + 128), d = __builtin_nontemporal_load(src + 192);
            acc += (a + b) + (c + d);
        }
    } else {
        const stream_f32x4 *src = p + (size_t)blockIdx.x * per16 + (size_t)wave * q + lane;
        for (size_t i = 0; i + 64 <= q; i += 256) {
            const stream_f32x4 a = __builtin_nontemporal_load(src + i);
            const stream_f32x4 b = i + 128 <= q ? __builtin_nontemporal_load(src + i + 64) : zero;
            const stream_f32x4 c = i + 192 <= q ? __builtin_nontemporal_load(src + i + 128) : zero;
            const stream_f32x4 d = i + 256 <= q ? __builtin_nontemporal_load(src + i + 192) : zero;
            acc += (a + b) + (c + d);
        }
    }
    if ((acc[0] + acc[1]) + (acc[2] + acc[3]) == 1.2345e30f) out[blockIdx.x] = acc[0];      // (keeps the loads; never true on zeros)
}

static int stream_floor_bench(size_t bytes, int32_t wgs, int32_t interleaved, int32_t iters, float *us_per_launch)
{
    const bool cold = iters < 0;
    if (cold) iters = -iters;
    if (wgs <= 0) wgs = 256;
    if (wgs > 65536 || bytes < (size_t)wgs * 16384) return SJD_EINVAL;
    const size_t per16 = bytes / wgs / 16 / 1024 * 1024;            // 16-byte units per workgroup, a multiple of 4 waves x 4 KiB
    const size_t used = per16 * 16 * wgs;
    const int copies = cold ? (int)((((size_t)1 << 30) + used - 1) / used) + 1 : 1;
    GemmScratch g;
    SJD_TRY(dev_alloc(&g.Wp, used * copies));
    SJD_TRY(dev_alloc((void **)&g.out, (size_t)wgs * 4));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    HIP_TRY(hipEventCreate(&e0));
    if (hipError_t e = hipEventCreate(&e1); e != hipSuccess) { (void)hipEventDestroy(e0); sjd_set_hip_error(e, "hipEventCreate"); return SJD_EHIP; }
    for (int i = 0; i < 3; ++i)
        SJD_LAUNCH(stream_read_kernel, dim3(wgs), dim3(256), 0, 0, (const stream_f32x4 *)g.Wp, per16, g.out, interleaved);
    (void)hipEventRecord(e0, 0);
    for (int i = 0; i < iters; ++i)
        SJD_LAUNCH(stream_read_kernel, dim3(wgs), dim3(256), 0, 0,
                   (const stream_f32x4 *)((const char *)g.Wp + (size_t)(i % copies) * used), per16, g.out, interleaved);
    (void)hipEventRecord(e1, 0);
    (void)hipEventSynchronize(e1);
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    *us_per_launch = ms * 1e3f / iters;
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

extern "C" int sjd_gemm_bench(int32_t M, int32_t N, int32_t K, int32_t tn, int32_t wk, int32_t u, int32_t iters,
                              float *us_per_launch)
{
    if (M < 1 || N < 16 || K < 32 || N % 16 || K % 32 || iters == 0 || !us_per_launch) return SJD_EINVAL;
    // tn = 0: no product, the plain streaming read of the same weight bytes by wk workgroups
    if (tn == 0) return stream_floor_bench((size_t)N * K * 2, wk, u, iters, us_per_launch);
    // iters < 0: rotate through enough weight copies that none is still in the last-level cache
    const bool cold = iters < 0;
    if (cold) iters = -iters;
    if (tn < 1 || tn > 3 || N % (16 * tn)) return SJD_EINVAL;
    // More rows than one forward computes: an off-path measurement of the wide kernel's matrix-core rate.  The
    // rows are cut into chunks of SJD_ROWS_MAX, each a launch pair of its own over the same weights (which
    // then come from the last-level cache for every chunk after the first).
    const int chunks = (M + SJD_ROWS_MAX - 1) / SJD_ROWS_MAX, rows = chunks > 1 ? SJD_ROWS_MAX : M;
    // wk >= 100 asks for the wide kernel at any row count, with wk - 100 K-slices (0 = automatic) and u
    // weight groups per wave (0 = automatic)
    const bool force_wide = wk >= 100;
    if (force_wide) wk -= 100;
    const bool wide = rows > SJD_ROWS_SKINNY || force_wide;
    // skinny kernel: u + 10 reads the activations in their 4-byte form (2-byte lo plane) instead of 3 bytes
    int form = wide ? SJD_ACT_P4 : SJD_ACT_P3;
    if (!wide && u >= 10) { u -= 10; form = SJD_ACT_P4; }
    if (!wide && (u != 0 && u != 2 && u != 4)) return SJD_EINVAL;       // (0: the model's choice)
    const size_t wbytes = (size_t)N * K * 2;
    const int copies = cold ? (int)((((size_t)1 << 30) + wbytes - 1) / wbytes) + 1 : 1;
    GemmScratch g;
    SJD_TRY(dev_alloc(&g.Ap, (size_t)SJD_ROWS_MAX * K * 4 + 2048));
    SJD_TRY(dev_alloc(&g.Wp, wbytes * copies));
    SJD_TRY(dev_alloc((void **)&g.out, (size_t)SJD_ROWS_MAX * N * 4));
    const size_t part_elems = wide ? (size_t)8 * SJD_ROWS_MAX * N : 0;      // (room for up to 8 K-slices)
    if (wide) SJD_TRY(dev_alloc(&g.part, part_elems * 4));
    SjdLinear lin;
    memset(&lin, 0, sizeof(lin));
    lin.N = N; lin.K = K; lin.tn = tn; lin.w = g.Wp;
    if (force_wide && u == 7 && rows > 16 && rows <= 32 && tn == 2) { lin.whole_k_rows = 32; form = SJD_ACT_P3; }   // the wide kernel's whole-K variant
    else if (wide) { lin.wks = wk; lin.wg = u; lin.wide_from = 1; }      // wide kernel: K-slices and weight groups per wave (0 = automatic)
    else { lin.wk = wk; lin.u = u; }
    SjdGemmEpi ep;
    memset(&ep, 0, sizeof(ep));
    ep.kind = SJD_EPI_STORE; ep.out = g.out;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    HIP_TRY(hipEventCreate(&e0));
    if (hipError_t e = hipEventCreate(&e1); e != hipSuccess) { (void)hipEventDestroy(e0); sjd_set_hip_error(e, "hipEventCreate"); return SJD_EHIP; }
    int rc = SJD_OK;
    auto one = [&]() {
        int r = SJD_OK;
        for (int c = 0; c < chunks && r == SJD_OK; ++c)
            r = sjd_launch_gemm_bf16(&lin, g.Ap, form, nullptr, 0.f, rows, ep, (float *)g.part, part_elems, 0);
        return r;
    };
    for (int i = 0; i < 3 && rc == SJD_OK; ++i) rc = one();
    if (rc == SJD_OK) {
        (void)hipEventRecord(e0, 0);
        for (int i = 0; i < iters && rc == SJD_OK; ++i) {
            lin.w = (const char *)g.Wp + (size_t)(i % copies) * wbytes;
            rc = one();
        }
        (void)hipEventRecord(e1, 0);
        (void)hipEventSynchronize(e1);
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        *us_per_launch = ms * 1e3f / iters;
    }
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    return rc;
}
