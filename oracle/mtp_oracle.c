/*
 * CPU oracle for the FastMTP draft path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the correctness reference the HIP library is compared with.  It
 * is deliberately plain: scalar loops, sums taken left to right, one sequence
 * at a time, no blocking, no fusion.  It shares no code with the HIP library
 * and must never be called from the product path; only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may load it.
 *
 * What it computes (citations are to the FastMTP paper, arXiv 2509.18362):
 *   - one MTP head with the DeepSeek-V3 module layout, a single weight set
 *     reused at every draft depth (Sec. 2.1 "Architecture Design");
 *   - the recursive drafting of Sec. 2.3 "Drafting phase": step 1 consumes the
 *     target model's hidden state and the embedding of the verified token,
 *     step k>1 consumes the head's own output hidden state and the embedding
 *     of the previously drafted token;
 *   - the compressed output head of Sec. 2.2, Eq. (3): logits only for the
 *     rows W[ids[i], :] of the main model's output head, greedy argmax
 *     (Sec. 3.1 "greedy decoding"), mapped back to the full-vocabulary id;
 *   - sequential acceptance up to the first mismatch (Sec. 2.3 "Verification
 *     phase") and the bookkeeping of the draft KV length after it.
 *
 * Precision: `real` is float by default (the reference precision named for this
 * build) and double when compiled with -DORC_F64; the double build bounds the
 * float build's own rounding error.  bf16 inputs are widened exactly.  The only
 * rounding to bf16 inside the method is the KV-cache append.
 *
 * Parity pins (tests/test_oracle_pins.py): every function below is pinned to
 * library routines, closed forms or invariants; none is "parity unpinned".
 * The paper prints no worked numeric example of a draft step.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifdef ORC_F64
typedef double real;
#define R_SQRT sqrt
#define R_EXP exp
#else
typedef float real;
#define R_SQRT sqrtf
#define R_EXP expf
#endif

typedef struct {
    int32_t d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab_size;
    float rms_eps;
    float rope_theta;
    int32_t kv_capacity;    /* tokens per (sequence, kv head) in the cache */
    int32_t recur_pre_norm; /* 0: the recurring hidden state is the final-norm output (default reading);
                               1: it is the residual stream before the final norm (alternative reading) */
} orc_config;

typedef struct { /* bf16 bit patterns, row-major [out][in] */
    const uint16_t *embed, *lm_head;
    const uint16_t *g_hnorm, *g_enorm, *g_attn_norm, *g_mlp_norm, *g_final_norm;
    const uint16_t *w_proj;
    const uint16_t *w_q, *w_k, *w_v;
    const uint16_t *b_q, *b_k, *b_v; /* may be NULL */
    const uint16_t *w_o;
    const uint16_t *w_gate, *w_up, *w_down;
} orc_weights;

typedef struct { /* optional per-step intermediates; any pointer may be NULL */
    real *c;    /* [2d]     concatenated normalised inputs       */
    real *x;    /* [d]      projection output                    */
    real *q;    /* [Hq*hd]  queries after RoPE                   */
    real *k;    /* [Hkv*hd] new key after RoPE, before rounding  */
    real *v;    /* [Hkv*hd] new value, before rounding           */
    real *attn; /* [Hq*hd]  attention output                     */
    real *x1;   /* [d]      after attention residual             */
    real *m;    /* [F]      SwiGLU product                       */
    real *x2;   /* [d]      after MLP residual                   */
} orc_trace;

int orc_real_bytes(void) { return (int)sizeof(real); }

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---- bf16 <-> real ---------------------------------------------------- */

static inline float bf16_widen(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static inline uint16_t f32_round_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40); /* NaN stays NaN */
    u += 0x7fffu + ((u >> 16) & 1u); /* nearest, ties to even */
    return (uint16_t)(u >> 16);
}

/* Round to the nearest bf16, ties to even, without double rounding in the double build. */
uint16_t orc_round_bf16(real x) {
#ifdef ORC_F64
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0xffffu) == 0x8000u && (double)f != x && isfinite(f)) {
        /* the float landed on a bf16 tie only because of the first rounding:
           decide by where the exact value lies */
        double fa = fabs((double)f), xa = fabs(x);
        u = (xa > fa) ? u + 1u : u - 1u;
        memcpy(&f, &u, 4);
    }
    return f32_round_bf16(f);
#else
    return f32_round_bf16(x);
#endif
}

float orc_widen_bf16(uint16_t b) { return bf16_widen(b); }

/* ---- building blocks --------------------------------------------------- */

/* RMSNorm(u; g)_i = g_i * u_i / sqrt(mean(u^2) + eps) */
void orc_rmsnorm(const real *u, const uint16_t *g, int32_t d, float eps, real *out) {
    real ss = 0;
    for (int32_t i = 0; i < d; ++i) ss += u[i] * u[i];
    real inv = (real)1 / R_SQRT(ss / (real)d + (real)eps);
    for (int32_t i = 0; i < d; ++i) out[i] = (real)bf16_widen(g[i]) * (u[i] * inv);
}

/* y = W x (+ bias), W is [n_out][n_in] bf16 */
void orc_linear(const uint16_t *W, const uint16_t *bias, const real *x, int32_t n_out, int32_t n_in, real *y) {
#pragma omp parallel for schedule(static)
    for (int32_t o = 0; o < n_out; ++o) {
        const uint16_t *row = W + (size_t)o * (size_t)n_in;
        real acc = 0;
        for (int32_t i = 0; i < n_in; ++i) acc += (real)bf16_widen(row[i]) * x[i];
        if (bias) acc += (real)bf16_widen(bias[o]);
        y[o] = acc;
    }
}

/* Rotary embedding at position pos on n_heads vectors of head_dim; pairs (j, j + head_dim/2). */
void orc_rope(real *u, int32_t n_heads, int32_t head_dim, int32_t pos, float theta) {
    int32_t half = head_dim / 2;
    for (int32_t h = 0; h < n_heads; ++h) {
        real *p = u + (size_t)h * head_dim;
        for (int32_t j = 0; j < half; ++j) {
            double ang = (double)pos * pow((double)theta, -2.0 * (double)j / (double)head_dim);
            real cs = (real)cos(ang), sn = (real)sin(ang);
            real a = p[j], b = p[j + half];
            p[j] = a * cs - b * sn;
            p[j + half] = b * cs + a * sn;
        }
    }
}

/* Grouped-query attention of one new token over cache slots 0..len-1 of one sequence.
 * q: [Hq][hd]; kc, vc: [Hkv][cap][hd] bf16; out: [Hq][hd].
 * Query head h reads KV head h / (Hq/Hkv). */
int orc_attention(const real *q, const uint16_t *kc, const uint16_t *vc, int32_t len, int32_t cap, int32_t Hq,
                  int32_t Hkv, int32_t hd, real *out) {
    if (len <= 0 || len > cap || Hq % Hkv != 0) return -1;
    int32_t group = Hq / Hkv;
    real scale = (real)1 / R_SQRT((real)hd);
    int fail = 0;
#pragma omp parallel for schedule(static)
    for (int32_t h = 0; h < Hq; ++h) {
        const uint16_t *K = kc + (size_t)(h / group) * cap * hd;
        const uint16_t *V = vc + (size_t)(h / group) * cap * hd;
        const real *qh = q + (size_t)h * hd;
        real *s = (real *)malloc((size_t)len * sizeof(real));
        if (!s) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        real mx = 0;
        for (int32_t t = 0; t < len; ++t) {
            real acc = 0;
            for (int32_t j = 0; j < hd; ++j) acc += qh[j] * (real)bf16_widen(K[(size_t)t * hd + j]);
            s[t] = acc * scale;
            if (t == 0 || s[t] > mx) mx = s[t];
        }
        real den = 0;
        for (int32_t t = 0; t < len; ++t) {
            s[t] = R_EXP(s[t] - mx);
            den += s[t];
        }
        for (int32_t j = 0; j < hd; ++j) {
            real acc = 0;
            for (int32_t t = 0; t < len; ++t) acc += (s[t] / den) * (real)bf16_widen(V[(size_t)t * hd + j]);
            out[(size_t)h * hd + j] = acc;
        }
        free(s);
    }
    return fail ? -2 : 0;
}

/* m = silu(W_g y) * (W_u y), silu(z) = z / (1 + exp(-z)) */
void orc_swiglu(const uint16_t *w_gate, const uint16_t *w_up, const real *y, int32_t F, int32_t d, real *m) {
#pragma omp parallel for schedule(static)
    for (int32_t o = 0; o < F; ++o) {
        const uint16_t *rg = w_gate + (size_t)o * d, *ru = w_up + (size_t)o * d;
        real g = 0, u = 0;
        for (int32_t i = 0; i < d; ++i) g += (real)bf16_widen(rg[i]) * y[i];
        for (int32_t i = 0; i < d; ++i) u += (real)bf16_widen(ru[i]) * y[i];
        m[o] = (g / ((real)1 + R_EXP(-g))) * u;
    }
}

/* Eq. (3): z_i = W[ids[i], :] . h for i < n (ids == NULL means ids[i] = i, the full head).
 * best_index = smallest i attaining the maximum; margin = top-1 minus top-2 logit (0 if n == 1).
 * logits may be NULL. */
int orc_lm_head(const uint16_t *W, int32_t V, const int32_t *ids, int32_t n, int32_t d, const real *h,
                real *logits, int32_t *best_index, real *margin) {
    if (n <= 0) return -1;
    real *z = logits ? logits : (real *)malloc((size_t)n * sizeof(real));
    if (!z) return -2;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < n; ++i) {
        int32_t r = ids ? ids[i] : i;
        if (r < 0 || r >= V) {
#pragma omp atomic write
            bad = 1;
            z[i] = 0;
            continue;
        }
        const uint16_t *row = W + (size_t)r * d;
        real acc = 0;
        for (int32_t j = 0; j < d; ++j) acc += (real)bf16_widen(row[j]) * h[j];
        z[i] = acc;
    }
    int32_t bi = 0;
    for (int32_t i = 1; i < n; ++i)
        if (z[i] > z[bi]) bi = i;
    real second = 0;
    int have = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (i == bi) continue;
        if (!have || z[i] > second) {
            second = z[i];
            have = 1;
        }
    }
    if (best_index) *best_index = bi;
    if (margin) *margin = have ? z[bi] - second : 0;
    if (!logits) free(z);
    return bad ? -3 : 0;
}

/* ---- one draft step ----------------------------------------------------- */

/* One application of the MTP head for one sequence.
 *   h      [d]   hidden state fed to the head (target's at step 1, own output afterwards)
 *   token        id whose embedding is paired with h
 *   kc, vc       this sequence's cache [Hkv][cap][hd]; slot `pos` is written (bf16), slots 0..pos are read
 *   pos          index of the new cache slot = number of entries already present
 * Outputs: hhat [d] (final-norm output), x2 via trace, logits [n] (optional), draft id, margin.
 */
int orc_step(const orc_config *cfg, const orc_weights *w, const real *h, int32_t token, uint16_t *kc, uint16_t *vc,
             int32_t pos, const int32_t *ids, int32_t n, real *hhat, real *logits, int32_t *draft_id,
             real *margin, const orc_trace *tr) {
    const int32_t d = cfg->d_model, Hq = cfg->n_q_heads, Hkv = cfg->n_kv_heads, hd = cfg->head_dim;
    const int32_t F = cfg->d_ffn, V = cfg->vocab_size, cap = cfg->kv_capacity;
    const int32_t qd = Hq * hd, kvd = Hkv * hd;
    if (token < 0 || token >= V) return -10;
    if (pos < 0 || pos >= cap) return -11;
    if (hd % 2 != 0 || Hq % Hkv != 0) return -12;

    size_t total = (size_t)d * 8 + (size_t)qd * 2 + (size_t)kvd * 2 + (size_t)F;
    real *buf = (real *)malloc(total * sizeof(real));
    if (!buf) return -13;
    real *e = buf, *c = e + d, *x = c + 2 * d, *y = x + d, *x1 = y + d, *y2 = x1 + d, *x2 = y2 + d;
    real *q = x2 + d, *attn = q + qd, *k = attn + qd, *v = k + kvd, *m = v + kvd;

    /* embedding of the paired token; dual RMSNorm; concatenation, hidden half first */
    for (int32_t i = 0; i < d; ++i) e[i] = (real)bf16_widen(w->embed[(size_t)token * d + i]);
    orc_rmsnorm(h, w->g_hnorm, d, cfg->rms_eps, c);
    orc_rmsnorm(e, w->g_enorm, d, cfg->rms_eps, c + d);
    /* 2d -> d projection */
    orc_linear(w->w_proj, NULL, c, d, 2 * d, x);
    /* decoder layer: pre-norm attention */
    orc_rmsnorm(x, w->g_attn_norm, d, cfg->rms_eps, y);
    orc_linear(w->w_q, w->b_q, y, qd, d, q);
    orc_linear(w->w_k, w->b_k, y, kvd, d, k);
    orc_linear(w->w_v, w->b_v, y, kvd, d, v);
    orc_rope(q, Hq, hd, pos, cfg->rope_theta);
    orc_rope(k, Hkv, hd, pos, cfg->rope_theta);
    if (tr && tr->k) memcpy(tr->k, k, (size_t)kvd * sizeof(real));
    if (tr && tr->v) memcpy(tr->v, v, (size_t)kvd * sizeof(real));
    /* append to the cache in its storage format; attention reads the stored values */
    for (int32_t g = 0; g < Hkv; ++g)
        for (int32_t j = 0; j < hd; ++j) {
            kc[((size_t)g * cap + pos) * hd + j] = orc_round_bf16(k[(size_t)g * hd + j]);
            vc[((size_t)g * cap + pos) * hd + j] = orc_round_bf16(v[(size_t)g * hd + j]);
        }
    int rc = orc_attention(q, kc, vc, pos + 1, cap, Hq, Hkv, hd, attn);
    if (rc) {
        free(buf);
        return rc;
    }
    orc_linear(w->w_o, NULL, attn, d, qd, x1);
    for (int32_t i = 0; i < d; ++i) x1[i] = x[i] + x1[i];
    /* pre-norm SwiGLU MLP */
    orc_rmsnorm(x1, w->g_mlp_norm, d, cfg->rms_eps, y2);
    orc_swiglu(w->w_gate, w->w_up, y2, F, d, m);
    orc_linear(w->w_down, NULL, m, d, F, x2);
    for (int32_t i = 0; i < d; ++i) x2[i] = x1[i] + x2[i];
    /* final norm: the head's output hidden state */
    orc_rmsnorm(x2, w->g_final_norm, d, cfg->rms_eps, hhat);
    /* compressed output head + greedy pick, mapped back to a full-vocabulary id */
    int32_t bi = 0;
    rc = orc_lm_head(w->lm_head, V, ids, n, d, hhat, logits, &bi, margin);
    if (draft_id) *draft_id = ids ? ids[bi] : bi;

    if (tr) {
        if (tr->c) memcpy(tr->c, c, (size_t)2 * d * sizeof(real));
        if (tr->x) memcpy(tr->x, x, (size_t)d * sizeof(real));
        if (tr->q) memcpy(tr->q, q, (size_t)qd * sizeof(real));
        if (tr->attn) memcpy(tr->attn, attn, (size_t)qd * sizeof(real));
        if (tr->x1) memcpy(tr->x1, x1, (size_t)d * sizeof(real));
        if (tr->m) memcpy(tr->m, m, (size_t)F * sizeof(real));
        if (tr->x2) memcpy(tr->x2, x2, (size_t)d * sizeof(real));
    }
    free(buf);
    return rc;
}

/* ---- K recursive steps for a batch --------------------------------------- */

/* Sequences are independent and processed one after another.
 *   hidden_in [B][d] bf16, token_in [B], kv_len [B] (entries present before drafting; not modified)
 *   k_cache, v_cache [B][Hkv][cap][hd] bf16: slots kv_len[b] .. kv_len[b]+K-1 are written
 *   forced [B][K-1] or NULL: tokens fed at steps 2..K instead of the previous draft (teacher forcing,
 *          Sec. 2.1 "Training Mechanism"; used by tests to keep chains aligned)
 *   draft_out [B][K]; logits_out [B][K][n] or NULL; hidden_out [B][K][d] or NULL; margin_out [B][K] or NULL
 */
int orc_chain(const orc_config *cfg, const orc_weights *w, int32_t B, int32_t K, const uint16_t *hidden_in,
              const int32_t *token_in, uint16_t *k_cache, uint16_t *v_cache, const int32_t *kv_len,
              const int32_t *forced, const int32_t *ids, int32_t n, int32_t *draft_out, real *logits_out,
              real *hidden_out, real *margin_out) {
    const int32_t d = cfg->d_model;
    const size_t seq_stride = (size_t)cfg->n_kv_heads * cfg->kv_capacity * cfg->head_dim;
    real *h = (real *)malloc((size_t)d * 3 * sizeof(real));
    if (!h) return -13;
    real *hhat = h + d, *x2 = hhat + d;
    orc_trace tr;
    memset(&tr, 0, sizeof tr);
    tr.x2 = x2;
    int rc = 0;
    for (int32_t b = 0; b < B && !rc; ++b) {
        for (int32_t i = 0; i < d; ++i) h[i] = (real)bf16_widen(hidden_in[(size_t)b * d + i]);
        int32_t tok = token_in[b];
        for (int32_t k = 0; k < K; ++k) {
            int32_t did = -1;
            real mg = 0;
            rc = orc_step(cfg, w, h, tok, k_cache + b * seq_stride, v_cache + b * seq_stride, kv_len[b] + k, ids, n,
                          hhat, logits_out ? logits_out + ((size_t)b * K + k) * n : NULL, &did, &mg, &tr);
            if (rc) break;
            draft_out[(size_t)b * K + k] = did;
            if (margin_out) margin_out[(size_t)b * K + k] = mg;
            if (hidden_out) memcpy(hidden_out + ((size_t)b * K + k) * d, hhat, (size_t)d * sizeof(real));
            memcpy(h, cfg->recur_pre_norm ? x2 : hhat, (size_t)d * sizeof(real));
            tok = (forced && k + 1 < K) ? forced[(size_t)b * (K - 1) + k] : did;
        }
    }
    free(h);
    return rc;
}

/* ---- first draft step over several new positions --------------------------- */

/* Sec. 2.3 "Drafting phase": the first draft step runs over the shifted prefix, i.e. the head is applied to every new
 * position with the TARGET model's hidden state of that position and the embedding of the token that follows it; the
 * last position yields the first draft token, the others only extend the head's KV cache.  Position j of sequence b
 * sits at cache slot kv_len[b] + j and attends slots 0 .. kv_len[b] + j (causal inside the new block).
 * Here that is the one-position routine applied to the positions in order, each finding its predecessors' entries
 * in the cache.
 *   Arrays with a position axis are position-major: hidden_in [m_max][B][d] bf16, tokens [m_max][B],
 *   draft_out [m_max][B], logits_out [m_max][B][n] or NULL, hidden_out [m_max][B][d] or NULL, margin_out
 *   [m_max][B] or NULL.  ext_len [B]: number of new positions of each sequence, 0 .. m_max.
 *   kv_len [B] is advanced by ext_len.  Positions at or beyond ext_len[b] report draft -1 and leave the other
 *   outputs untouched.  A sequence whose new positions do not fit the cache (or with a negative length) is left
 *   alone entirely (draft -1 everywhere, kv_len unchanged) and the function returns 1 after finishing the others.
 */
int orc_extend(const orc_config *cfg, const orc_weights *w, int32_t B, int32_t m_max, const uint16_t *hidden_in,
               const int32_t *tokens, const int32_t *ext_len, uint16_t *k_cache, uint16_t *v_cache, int32_t *kv_len,
               const int32_t *ids, int32_t n, int32_t *draft_out, real *logits_out, real *hidden_out,
               real *margin_out) {
    const int32_t d = cfg->d_model;
    const size_t seq_stride = (size_t)cfg->n_kv_heads * cfg->kv_capacity * cfg->head_dim;
    real *h = (real *)malloc((size_t)d * 2 * sizeof(real));
    if (!h) return -13;
    real *hhat = h + d;
    int overflow = 0;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t L = kv_len[b], m = ext_len[b];
        for (int32_t j = 0; j < m_max; ++j) draft_out[(size_t)j * B + b] = -1;
        if (L < 0 || m < 0 || m > m_max || L + m > cfg->kv_capacity) {
            overflow = 1;
            continue;
        }
        for (int32_t j = 0; j < m; ++j) {
            const size_t r = (size_t)j * B + b;
            for (int32_t i = 0; i < d; ++i) h[i] = (real)bf16_widen(hidden_in[r * d + i]);
            int32_t did = -1;
            real mg = 0;
            int rc = orc_step(cfg, w, h, tokens[r], k_cache + b * seq_stride, v_cache + b * seq_stride, L + j, ids, n,
                              hhat, logits_out ? logits_out + r * n : NULL, &did, &mg, NULL);
            if (rc) {
                free(h);
                return rc;
            }
            draft_out[r] = did;
            if (margin_out) margin_out[r] = mg;
            if (hidden_out) memcpy(hidden_out + r * d, hhat, (size_t)d * sizeof(real));
        }
        kv_len[b] = L + m;
    }
    free(h);
    return overflow;
}

/* ---- acceptance and cache bookkeeping ------------------------------------ */

/* draft [B][K] = d_1..d_K, target [B][K+1] = g_1..g_{K+1} (the target model's greedy tokens at the same
 * positions).  a = number of leading positions where d_j == g_j.  Emitted tokens: d_1..d_a, g_{a+1}, padded
 * with -1 to K+1.  Draft-cache slot L+j-1 was computed from input token x_j (x_1 verified, x_j = d_{j-1}).
 *   mode 0 (keep confirmed): kv_len <- L + min(a+1, K); pending = (a == K): the entry for d_K does not exist yet
 *   mode 1 (discard draft) : kv_len <- L; pending = 0
 */
void orc_accept(int32_t B, int32_t K, const int32_t *draft, const int32_t *target, int32_t mode, int32_t *kv_len,
                int32_t *accept_len, int32_t *out_tokens, int32_t *pending) {
    for (int32_t b = 0; b < B; ++b) {
        const int32_t *dr = draft + (size_t)b * K, *tg = target + (size_t)b * (K + 1);
        int32_t a = 0;
        while (a < K && dr[a] == tg[a]) ++a;
        for (int32_t j = 0; j <= K; ++j) out_tokens[(size_t)b * (K + 1) + j] = j < a ? dr[j] : (j == a ? tg[a] : -1);
        accept_len[b] = a;
        if (mode == 0) {
            kv_len[b] += (a + 1 < K) ? a + 1 : K;
            pending[b] = (a == K);
        } else {
            pending[b] = 0;
        }
    }
}
