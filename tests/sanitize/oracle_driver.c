/* Runs every C entry point of the oracle on a small head under AddressSanitizer and UndefinedBehaviorSanitizer
 * (host only; built and run by tests/test_sanitizers.py).  The inputs come from a private linear congruential
 * generator: the point is memory safety and defined behaviour, the values are checked elsewhere. */
#include "../../oracle/mtp_oracle.c"

#include <stdio.h>

static uint32_t lcg_state = 12345u;
static uint32_t lcg(void) { return lcg_state = lcg_state * 1664525u + 1013904223u; }
/* a bf16 bit pattern of a value in (-scale, scale) */
static uint16_t rnd_bf16(float scale) {
    float f = ((float)(lcg() >> 8) / 8388608.0f - 1.0f) * scale;
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}
static uint16_t *rnd_vec(size_t n, float scale, float offset) {
    uint16_t *p = (uint16_t *)malloc(n * sizeof(uint16_t));
    for (size_t i = 0; i < n; ++i) {
        if (offset != 0.0f) {
            float f = offset + ((float)(lcg() >> 8) / 8388608.0f - 1.0f) * scale;
            uint32_t u;
            memcpy(&u, &f, 4);
            p[i] = (uint16_t)(u >> 16);
        } else {
            p[i] = rnd_bf16(scale);
        }
    }
    return p;
}

int main(void) {
    orc_config cfg = {64, 4, 2, 16, 96, 50, 1e-6f, 10000.0f, 24, 0};
    const int32_t d = cfg.d_model, qd = cfg.n_q_heads * cfg.head_dim, kvd = cfg.n_kv_heads * cfg.head_dim, F = cfg.d_ffn,
                  V = cfg.vocab_size, cap = cfg.kv_capacity;
    orc_weights w;
    w.embed = rnd_vec((size_t)V * d, 0.05f, 0.f);
    w.lm_head = rnd_vec((size_t)V * d, 0.05f, 0.f);
    w.g_hnorm = rnd_vec(d, 0.02f, 1.f);
    w.g_enorm = rnd_vec(d, 0.02f, 1.f);
    w.g_attn_norm = rnd_vec(d, 0.02f, 1.f);
    w.g_mlp_norm = rnd_vec(d, 0.02f, 1.f);
    w.g_final_norm = rnd_vec(d, 0.02f, 1.f);
    w.w_proj = rnd_vec((size_t)d * 2 * d, 0.05f, 0.f);
    w.w_q = rnd_vec((size_t)qd * d, 0.05f, 0.f);
    w.w_k = rnd_vec((size_t)kvd * d, 0.05f, 0.f);
    w.w_v = rnd_vec((size_t)kvd * d, 0.05f, 0.f);
    w.b_q = rnd_vec(qd, 0.05f, 0.f);
    w.b_k = rnd_vec(kvd, 0.05f, 0.f);
    w.b_v = NULL; /* the optional bias, absent once */
    w.w_o = rnd_vec((size_t)d * qd, 0.05f, 0.f);
    w.w_gate = rnd_vec((size_t)F * d, 0.05f, 0.f);
    w.w_up = rnd_vec((size_t)F * d, 0.05f, 0.f);
    w.w_down = rnd_vec((size_t)d * F, 0.05f, 0.f);

    enum { B = 3, K = 3, M = 4, N = 11 };
    int32_t ids[N];
    for (int i = 0; i < N; ++i) ids[i] = i * 4 + (i & 1); /* ascending, below V */
    const size_t cache = (size_t)B * cfg.n_kv_heads * cap * cfg.head_dim;
    uint16_t *kc = rnd_vec(cache, 1.0f, 0.f), *vc = rnd_vec(cache, 1.0f, 0.f);
    uint16_t *hidden = rnd_vec((size_t)M * B * d, 1.0f, 0.f);
    int32_t kv_len[B] = {0, 7, cap - K}; /* empty context, ordinary, exactly full after K steps */
    int32_t token[M * B], forced[B * (K - 1)], draft[B * K], ext_len[B] = {4, 0, 2}, ext_draft[M * B];
    for (int i = 0; i < M * B; ++i) token[i] = (int32_t)(lcg() % (uint32_t)V);
    for (int i = 0; i < B * (K - 1); ++i) forced[i] = (int32_t)(lcg() % (uint32_t)V);
    real *logits = (real *)malloc(sizeof(real) * B * K * V), *hid_out = (real *)malloc(sizeof(real) * M * B * d),
         *margin = (real *)malloc(sizeof(real) * M * B);

    /* compressed head, free-running; then the full head with forced tokens */
    int rc = orc_chain(&cfg, &w, B, K, hidden, token, kc, vc, kv_len, NULL, ids, N, draft, logits, hid_out, margin);
    if (rc) return 10 + rc;
    for (int i = 0; i < B * K; ++i)
        if (draft[i] < 0 || draft[i] >= V) return 2;
    rc = orc_chain(&cfg, &w, B, K, hidden, token, kc, vc, kv_len, forced, NULL, V, draft, logits, NULL, NULL);
    if (rc) return 20 + rc;

    /* a sequence that does not fit must be refused, not written */
    int32_t kv_over[1] = {cap - K + 1};
    rc = orc_chain(&cfg, &w, 1, K, hidden, token, kc, vc, kv_over, NULL, ids, N, draft, NULL, NULL, NULL);
    if (rc == 0) return 3;

    /* acceptance, both modes, every accept length */
    int32_t target[B * (K + 1)], acc[B], out_tok[B * (K + 1)], pend[B], kv2[B];
    for (int a = 0; a <= K; ++a)
        for (int mode = 0; mode < 2; ++mode) {
            for (int b = 0; b < B; ++b) {
                kv2[b] = kv_len[b];
                for (int j = 0; j <= K; ++j)
                    target[b * (K + 1) + j] = (j < a && j < K) ? draft[b * K + j] : V + j; /* V+j never matches */
            }
            orc_accept(B, K, draft, target, mode, kv2, acc, out_tok, pend);
            for (int b = 0; b < B; ++b)
                if (acc[b] != a) return 4;
        }

    /* a block of new positions with ragged counts, one of them zero; then one that does not fit */
    int32_t kv3[B] = {0, 7, 3};
    rc = orc_extend(&cfg, &w, B, M, hidden, token, ext_len, kc, vc, kv3, ids, N, ext_draft, NULL, hid_out, margin);
    if (rc != 0 || kv3[0] != 4 || kv3[1] != 7 || kv3[2] != 5) return 5;
    int32_t kv4[B] = {cap - 1, 0, 0};
    rc = orc_extend(&cfg, &w, B, M, hidden, token, ext_len, kc, vc, kv4, NULL, V, ext_draft, NULL, NULL, NULL);
    if (rc != 1 || kv4[0] != cap - 1) return 6;

    free(logits); free(hid_out); free(margin); free(kc); free(vc); free(hidden);
    free((void *)w.embed); free((void *)w.lm_head); free((void *)w.g_hnorm); free((void *)w.g_enorm);
    free((void *)w.g_attn_norm); free((void *)w.g_mlp_norm); free((void *)w.g_final_norm); free((void *)w.w_proj);
    free((void *)w.w_q); free((void *)w.w_k); free((void *)w.w_v); free((void *)w.b_q); free((void *)w.b_k);
    free((void *)w.w_o); free((void *)w.w_gate); free((void *)w.w_up); free((void *)w.w_down);
    puts("oracle under sanitizers: ok");
    return 0;
}
