/* Test-only driver: runs the CPU oracle end to end (transformer prefill, SJD generation with every
 * initialiser, the AR loop, the toy-model Monte-Carlo) on a tiny seeded model.  Built by
 * tests/test_oracle_sanitizers.py together with oracle/sjd_oracle.c under
 * -fsanitize=address,undefined: any out-of-bounds access, use after free, leak, signed overflow or
 * misaligned access in the oracle ends the process with a report.  Prints a checksum of the tokens. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "sjd_oracle.h"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static float frand(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return ((float)((rng_state >> 40) & 0xFFFF) / 65536.0f - 0.5f) * 0.2f;
}

int main(void)
{
    orc_config cfg = {2, 32, 2, 48, 96, 32, 96, 80, 0, 10000.0f, 1e-5f};
    const size_t d = cfg.d_model, f = cfg.d_ffn, v = cfg.vocab_total;
    const size_t n = v * d + (size_t)cfg.n_layers * (2 * d + 4 * d * d + 3 * d * f) + d + v * d;
    float *blob = malloc(n * sizeof(float));
    if (!blob) return 2;
    for (size_t i = 0; i < n; ++i) blob[i] = frand();
    /* gains = 1 (positions per the blob order: g1 at the start of a layer, g2 after the four d x d matrices) */
    size_t off = v * d;
    for (int l = 0; l < cfg.n_layers; ++l) {
        for (size_t j = 0; j < d; ++j) blob[off + j] = 1.0f;
        off += d + 4 * d * d;
        for (size_t j = 0; j < d; ++j) blob[off + j] = 1.0f;
        off += d + 3 * d * f;
    }
    for (size_t j = 0; j < d; ++j) blob[off + j] = 1.0f;

    orc_model *m = orc_model_create(&cfg, blob);
    if (!m) return 3;
    const int32_t V = cfg.samp_hi - cfg.samp_lo, N = 24;
    int32_t prompt[5] = {1, 7, 30, 2, 19};
    float embeds[3 * 32];
    for (int i = 0; i < 3 * 32; ++i) embeds[i] = frand();
    uint64_t sum = 0;
    for (int mode = 0; mode <= 4; ++mode) {
        for (int flags = 0; flags <= 1; ++flags) {
            orc_tf_ctx ctx = {m, orc_kv_create(m)};
            if (!ctx.kv) return 4;
            float *lp = malloc((size_t)V * sizeof(float));
            orc_tf_prefill(&ctx, prompt, 5, embeds, 3, lp);
            orc_sampler smp = {mode == 2 ? 1 : 20, 1.0f};
            orc_init init = {mode, 6, mode % 2 ? cfg.samp_hi - 1 : -1, flags};
            int32_t out[24];
            orc_stats st;
            const int L = mode == 3 ? 1 : 7 + mode;
            orc_generate_sjd(orc_tf_forward, &ctx, 8, lp, V, cfg.samp_lo, N, L, &smp, &init, 11 + mode, out, &st);
            for (int i = 0; i < N; ++i) sum = sum * 1315423911u + (uint64_t)out[i];
            sum += (uint64_t)st.steps;
            orc_kv_set_len(ctx.kv, 8);
            orc_generate_ar(orc_tf_forward, &ctx, 8, lp, V, cfg.samp_lo, N, &smp, &init, 11 + mode, out);
            for (int i = 0; i < N; ++i) sum = sum * 1315423911u + (uint64_t)out[i];
            free(lp);
            orc_kv_free(ctx.kv);
        }
    }
    orc_model_free(m);
    free(blob);

    /* toy table model: vocabulary 4, depth 3 */
    enum { TV = 4, DEPTH = 3, PREFIXES = 1 + 4 + 16 };
    float table[PREFIXES * TV];
    for (int i = 0; i < PREFIXES * TV; ++i) table[i] = frand() * 20.0f;
    int64_t hist[TV * TV * TV];
    int64_t steps = 0;
    orc_sampler smp = {3, 1.0f};
    orc_init init = {0, 2, -1, 0};
    orc_toy_histogram(table, TV, DEPTH, 3, &smp, &init, 5, 2000, 0, hist, &steps);
    for (int i = 0; i < TV * TV * TV; ++i) sum += (uint64_t)hist[i] * (uint64_t)(i + 1);
    printf("oracle sanitize run ok, checksum %llu\n", (unsigned long long)sum);
    return 0;
}
