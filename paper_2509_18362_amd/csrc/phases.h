// The phases of one FastMTP draft step as workgroup-level device functions (gfx950).
//
// Every phase is written for a "virtual grid": workgroup `vb` of `nvb` takes its share of the phase's work.
// Matrix-vector phases stream bf16 weight rows from HBM straight into the B operand of a 16x16x32 MFMA; the
// activation vector(s) sit in LDS as the sum of two bf16 numbers and form the A operand (row i = sequence i of
// the current batch chunk), so a 16-row weight tile costs no vector-ALU work besides address arithmetic.
#pragma once
#include "device_utils.h"

namespace mtp {

struct DraftParams {
    // shape (Sec. 3.1 "Model Configuration")
    int d, Hq, Hkv, hd, F, V, qd, kvd, qkv_dim, cap;
    float eps, theta;
    // call
    int B, K, n;
    const int *ids; // compressed vocabulary, nullptr = full vocabulary (Sec. 2.2, Eq. (3))
    // tensors of the head, bf16
    const uint16_t *embed, *lm_head, *g_h, *g_e, *g_attn, *g_mlp, *g_final, *w_proj, *w_q, *w_k, *w_v, *b_q, *b_k,
        *b_v, *w_o, *w_gate, *w_up, *w_down;
    // per-call inputs and outputs
    const uint16_t *hidden_in;
    const int *token_in, *kv_len, *forced;
    uint16_t *k_cache, *v_cache;
    int *draft_out;
    float *logits_out, *hidden_out;
    // workspace
    float *x, *qkv, *attn, *x1, *m, *x2, *hhat, *attn_part;
    unsigned long long *keys; // [max_draft_steps][max_batch] packed (logit, index) maxima
    int *err;                 // sticky error word
    int *attn_cnt;            // [max_batch][Hkv] arrival counters of the split-KV merge
    int max_batch;
    // launch plan
    int split_tokens, max_splits; // attention: tokens per split, splits per (sequence, KV head)
    int nb_proj, nb_d, nb_q, nb_down; // sequences staged in LDS per pass, by reduction length (2d, d, Hq*hd, F)
};

enum : int { kErrKvOverflow = 1, kErrTokenRange = 2 };

// ---------------------------------------------------------------------------------------------------
// per-sequence state helpers
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ bool seq_dead(const DraftParams &p, int b) {
    int L = p.kv_len[b];
    return L < 0 || L + p.K > p.cap;
}

// token whose embedding enters step `step` (0-based) for sequence b; out-of-range ids are reported and replaced by 0
__device__ __forceinline__ int step_token(const DraftParams &p, int b, int step) {
    int tok;
    if (step == 0)
        tok = p.token_in[b];
    else if (p.forced)
        tok = p.forced[(size_t)b * (p.K - 1) + step - 1];
    else {
        uint32_t i = key_index(p.keys[(size_t)(step - 1) * p.max_batch + b]);
        if (i >= (uint32_t)p.n) i = 0;
        tok = p.ids ? p.ids[i] : (int)i;
    }
    if (tok < 0 || tok >= p.V) {
        atomicOr(p.err, kErrTokenRange);
        tok = 0;
    }
    return tok;
}

// ---------------------------------------------------------------------------------------------------
// staging of activation vectors into LDS as bf16 hi + lo
// ---------------------------------------------------------------------------------------------------
constexpr int kMaxNormIter = 4; // d <= 4 * 4 * kBlock = 8192

// RMSNorm(u; g) of one vector of length d (Sec. 2.1: DeepSeek-V3 MTP module uses RMSNorm on both inputs), written to
// hi/lo (bf16) and optionally to out_f32.  SRC_BF16: u is bf16 bits, else float.  Contains barriers.
template <bool SRC_BF16>
__device__ void stage_rmsnorm(const void *src, const uint16_t *gain, int d, float eps, uint16_t *hi, uint16_t *lo,
                              float *red, float *out_f32, float *out2_f32 = nullptr) {
    float v[kMaxNormIter][4];
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < kMaxNormIter; ++it) {
        int e = (it * kBlock + threadIdx.x) * 4;
        if (e < d) {
            if (SRC_BF16) {
                u32x2 raw = *reinterpret_cast<const u32x2 *>(static_cast<const uint16_t *>(src) + e);
                v[it][0] = lo_half(raw.x);
                v[it][1] = hi_half(raw.x);
                v[it][2] = lo_half(raw.y);
                v[it][3] = hi_half(raw.y);
            } else {
                f32x4 raw = *reinterpret_cast<const f32x4 *>(static_cast<const float *>(src) + e);
                v[it][0] = raw.x;
                v[it][1] = raw.y;
                v[it][2] = raw.z;
                v[it][3] = raw.w;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) ss += v[it][q] * v[it][q];
        }
    }
    float tot = block_sum(ss, red);
    float inv = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
    for (int it = 0; it < kMaxNormIter; ++it) {
        int e = (it * kBlock + threadIdx.x) * 4;
        if (e < d) {
            u32x2 g = *reinterpret_cast<const u32x2 *>(gain + e);
            float o[4];
            o[0] = lo_half(g.x) * (v[it][0] * inv);
            o[1] = hi_half(g.x) * (v[it][1] * inv);
            o[2] = lo_half(g.y) * (v[it][2] * inv);
            o[3] = hi_half(g.y) * (v[it][3] * inv);
            uint16_t h[4], l[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) split_bf16(o[q], h[q], l[q]);
            u32x2 ph = {(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
            u32x2 pl = {(uint32_t)l[0] | ((uint32_t)l[1] << 16), (uint32_t)l[2] | ((uint32_t)l[3] << 16)};
            *reinterpret_cast<u32x2 *>(hi + e) = ph;
            *reinterpret_cast<u32x2 *>(lo + e) = pl;
            f32x4 w = {o[0], o[1], o[2], o[3]};
            if (out_f32) *reinterpret_cast<f32x4 *>(out_f32 + e) = w;
            if (out2_f32) *reinterpret_cast<f32x4 *>(out2_f32 + e) = w;
        }
    }
}

// plain copy of a float vector of length K (multiple of 4) into hi/lo, zero-padded to kpad
__device__ void stage_plain(const float *src, int K, int kpad, uint16_t *hi, uint16_t *lo) {
    for (int e = threadIdx.x * 4; e < kpad; e += kBlock * 4) {
        u32x2 ph = {0u, 0u}, pl = {0u, 0u};
        if (e < K) {
            f32x4 raw = *reinterpret_cast<const f32x4 *>(src + e);
            uint16_t h[4], l[4];
            split_bf16(raw.x, h[0], l[0]);
            split_bf16(raw.y, h[1], l[1]);
            split_bf16(raw.z, h[2], l[2]);
            split_bf16(raw.w, h[3], l[3]);
            ph.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
            ph.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
            pl.x = (uint32_t)l[0] | ((uint32_t)l[1] << 16);
            pl.y = (uint32_t)l[2] | ((uint32_t)l[3] << 16);
        }
        *reinterpret_cast<u32x2 *>(hi + e) = ph;
        *reinterpret_cast<u32x2 *>(lo + e) = pl;
    }
}

// ---------------------------------------------------------------------------------------------------
// weight-streaming core
// ---------------------------------------------------------------------------------------------------
// For rows [r0, r1) of NMAT matrices that share the input: out[mat][i][row] = sum_k W_mat[row][k] * act[i][k],
// i < nb sequences.  The rows are cut into 16-row tiles; the 8 waves split the reduction range of each tile and
// their partial sums meet in LDS.  Weight loads run one chunk (U MFMA k-steps) ahead of the MFMAs, across tile
// boundaries, so the HBM stream never drains inside a phase.
//   rowptr(mat, row) -> const uint16_t* : start of a weight row (K bf16, 16-byte aligned)
//   epi(i, row, sums[NMAT])             : called by one thread per (sequence, row)
// LDS: act_hi/act_lo [nb][kpad] bf16 (kpad = K rounded up to 32, zero padded); partial [2][kWaves][NMAT][nbmax][16].
template <int NMAT, int U, class RowPtr, class Epi>
__device__ void gemv_rows(RowPtr rowptr, int K, int r0, int r1, int nb, int nbmax, const uint16_t *act_hi,
                          const uint16_t *act_lo, int kpad, float *partial, Epi &epi) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int j = lane & 15, g = lane >> 4;
    const int nks = (K + 31) / 32;
    const int per = (nks + kWaves - 1) / kWaves;
    const int ks0 = min(wave * per, nks), ks1 = min(ks0 + per, nks);
    const int nch = (per + U - 1) / U;
    const int ntiles = (r1 - r0 + 15) / 16;
    if (ntiles <= 0) return;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    const uint16_t *base[NMAT];     // row start for the tile whose loads are being issued
    const uint16_t *base_nxt[NMAT]; // ... and for the tile after it (fetched early: a gather reads an index first)
    auto row_of = [&](int tile) { return min(r0 + tile * 16 + j, r1 - 1); };
#pragma unroll
    for (int mt = 0; mt < NMAT; ++mt) {
        base[mt] = rowptr(mt, row_of(0));
        base_nxt[mt] = rowptr(mt, row_of(min(1, ntiles - 1)));
    }

    auto load = [&](u32x4(&buf)[NMAT][U], int ch) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int ks = ks0 + ch * U + u;
            int k = ks * 32 + g * 8;
            bool ok = ks < ks1 && k < K;
#pragma unroll
            for (int mt = 0; mt < NMAT; ++mt) buf[mt][u] = ok ? ldg16(base[mt] + k) : zero4;
        }
    };

    f32x4 acc_h[NMAT], acc_l[NMAT];
    auto clear = [&]() {
#pragma unroll
        for (int mt = 0; mt < NMAT; ++mt) {
            acc_h[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
            acc_l[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };
    clear();

    auto compute = [&](u32x4(&buf)[NMAT][U], int ch) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int ks = ks0 + ch * U + u;
            if (ks < ks1) { // wave-uniform
                u32x4 ah = zero4, al = zero4;
                if (j < nb) {
                    ah = *reinterpret_cast<const u32x4 *>(act_hi + (size_t)j * kpad + ks * 32 + g * 8);
                    al = *reinterpret_cast<const u32x4 *>(act_lo + (size_t)j * kpad + ks * 32 + g * 8);
                }
#pragma unroll
                for (int mt = 0; mt < NMAT; ++mt) {
                    acc_h[mt] = mfma16(ah, buf[mt][u], acc_h[mt]);
                    acc_l[mt] = mfma16(al, buf[mt][u], acc_l[mt]);
                }
            }
        }
    };

    auto finish_tile = [&](int tile) {
        float *pb = partial + (size_t)(tile & 1) * kWaves * NMAT * nbmax * 16;
#pragma unroll
        for (int mt = 0; mt < NMAT; ++mt) {
            f32x4 s = acc_h[mt] + acc_l[mt];
            float sv[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                int i = g * 4 + v;
                if (i < nb) pb[((wave * NMAT + mt) * nbmax + i) * 16 + j] = sv[v];
            }
        }
        clear();
        __syncthreads();
        if ((int)threadIdx.x < 16 * nb) {
            int i = threadIdx.x >> 4, jj = threadIdx.x & 15;
            float sums[NMAT];
#pragma unroll
            for (int mt = 0; mt < NMAT; ++mt) {
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) s += pb[((w * NMAT + mt) * nbmax + i) * 16 + jj];
                sums[mt] = s;
            }
            int row = r0 + tile * 16 + jj;
            if (row < r1) epi(i, row, sums);
        }
    };

    u32x4 wb0[NMAT][U], wb1[NMAT][U];
    int tile = 0, ch = 0;       // position of the compute stream
    int ltile = 0, lch = 0;     // position of the load stream
    auto advance_load = [&]() { // move the load stream one chunk on; returns false past the end
        if (++lch == nch) {
            lch = 0;
            ++ltile;
            if (ltile >= ntiles) return false;
#pragma unroll
            for (int mt = 0; mt < NMAT; ++mt) {
                base[mt] = base_nxt[mt];
                base_nxt[mt] = rowptr(mt, row_of(min(ltile + 1, ntiles - 1)));
            }
        }
        return true;
    };
    auto step = [&](u32x4(&cur)[NMAT][U], u32x4(&nxt)[NMAT][U]) {
        if (advance_load()) load(nxt, lch);
        compute(cur, ch);
        if (++ch == nch) {
            finish_tile(tile);
            ch = 0;
            ++tile;
        }
    };
    load(wb0, 0);
    const int total = ntiles * nch;
    for (int it = 0; it < total; it += 2) {
        step(wb0, wb1);
        if (it + 1 < total) step(wb1, wb0);
    }
}

// carve-up of the dynamic LDS of a matrix-vector phase
struct GemvLds {
    uint16_t *hi, *lo;
    float *partial, *red;
    int kpad;
};
__host__ __device__ inline size_t gemv_lds_bytes(int K, int nb, int nmat) {
    size_t kpad = (size_t)((K + 31) / 32) * 32;
    return 2 * kpad * nb * sizeof(uint16_t) + (size_t)2 * kWaves * nmat * nb * 16 * sizeof(float) + 64;
}
__device__ inline GemvLds gemv_lds(char *smem, int K, int nb, int nmat) {
    GemvLds l;
    l.kpad = ((K + 31) / 32) * 32;
    l.hi = reinterpret_cast<uint16_t *>(smem);
    l.lo = l.hi + (size_t)l.kpad * nb;
    l.partial = reinterpret_cast<float *>(l.lo + (size_t)l.kpad * nb);
    l.red = l.partial + (size_t)2 * kWaves * nmat * nb * 16;
    return l;
}

// rows [r0, r1) of workgroup vb when `rows` rows are dealt out as evenly as possible
__device__ __forceinline__ void row_share(int rows, int vb, int nvb, int &r0, int &r1) {
    int q = rows / nvb, rem = rows % nvb;
    r0 = vb * q + min(vb, rem);
    r1 = r0 + q + (vb < rem ? 1 : 0);
}

// ---------------------------------------------------------------------------------------------------
// phase 1: embedding gather + dual RMSNorm + concat + 2d->d projection   (steps 1-3 of the draft step)
// ---------------------------------------------------------------------------------------------------
__device__ void phase_proj(const DraftParams &p, int step, int vb, int nvb, char *smem) {
    const int d = p.d;
    int r0, r1;
    row_share(d, vb, nvb, r0, r1);
    if (vb == 0 && (int)threadIdx.x < p.B) {
        int b = threadIdx.x;
        p.keys[(size_t)step * p.max_batch + b] = 0ull; // this step's argmax accumulator
        if (seq_dead(p, b)) atomicOr(p.err, kErrKvOverflow);
        if (step > 0) { // the previous step's winner is final now
            uint32_t i = key_index(p.keys[(size_t)(step - 1) * p.max_batch + b]);
            if (i >= (uint32_t)p.n) i = 0;
            p.draft_out[(size_t)b * p.K + step - 1] = seq_dead(p, b) ? -1 : (p.ids ? p.ids[i] : (int)i);
        }
    }
    const int nbmax = p.nb_proj;
    GemvLds l = gemv_lds(smem, 2 * d, nbmax, 1);
    for (int b0 = 0; b0 < p.B; b0 += nbmax) {
        int nb = min(nbmax, p.B - b0);
        __syncthreads();
        for (int i = 0; i < nb; ++i) {
            int b = b0 + i;
            int tok = step_token(p, b, step);
            uint16_t *hi = l.hi + (size_t)i * l.kpad, *lo = l.lo + (size_t)i * l.kpad;
            if (step == 0)
                stage_rmsnorm<true>(p.hidden_in + (size_t)b * d, p.g_h, d, p.eps, hi, lo, l.red, nullptr);
            else
                stage_rmsnorm<false>(p.hhat + (size_t)b * d, p.g_h, d, p.eps, hi, lo, l.red, nullptr);
            stage_rmsnorm<true>(p.embed + (size_t)tok * d, p.g_e, d, p.eps, hi + d, lo + d, l.red, nullptr);
        }
        __syncthreads();
        auto rowptr = [&](int, int row) { return p.w_proj + (size_t)row * 2 * d; };
        auto epi = [&](int i, int row, float(&s)[1]) { p.x[(size_t)(b0 + i) * d + row] = s[0]; };
        gemv_rows<1, 8>(rowptr, 2 * d, r0, r1, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, epi);
    }
}

// ---------------------------------------------------------------------------------------------------
// phase 2: attention-input RMSNorm + fused QKV projection (+bias)          (step 4)
// Rotary embedding and the cache append happen where q, k, v are consumed (phase_attn).
// ---------------------------------------------------------------------------------------------------
__device__ void phase_qkv(const DraftParams &p, int step, int vb, int nvb, char *smem) {
    const int d = p.d, rows = p.qkv_dim;
    int r0, r1;
    row_share(rows, vb, nvb, r0, r1);
    const int nbmax = p.nb_d;
    GemvLds l = gemv_lds(smem, d, nbmax, 1);
    for (int b0 = 0; b0 < p.B; b0 += nbmax) {
        int nb = min(nbmax, p.B - b0);
        __syncthreads();
        for (int i = 0; i < nb; ++i)
            stage_rmsnorm<false>(p.x + (size_t)(b0 + i) * d, p.g_attn, d, p.eps, l.hi + (size_t)i * l.kpad,
                                 l.lo + (size_t)i * l.kpad, l.red, nullptr);
        __syncthreads();
        auto rowptr = [&](int, int row) {
            if (row < p.qd) return p.w_q + (size_t)row * d;
            if (row < p.qd + p.kvd) return p.w_k + (size_t)(row - p.qd) * d;
            return p.w_v + (size_t)(row - p.qd - p.kvd) * d;
        };
        auto epi = [&](int i, int row, float(&s)[1]) {
            float bias = 0.f;
            if (row < p.qd) {
                if (p.b_q) bias = bf16_to_f32(p.b_q[row]);
            } else if (row < p.qd + p.kvd) {
                if (p.b_k) bias = bf16_to_f32(p.b_k[row - p.qd]);
            } else {
                if (p.b_v) bias = bf16_to_f32(p.b_v[row - p.qd - p.kvd]);
            }
            p.qkv[(size_t)(b0 + i) * rows + row] = s[0] + bias;
        };
        gemv_rows<1, 8>(rowptr, d, r0, r1, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, epi);
    }
}

// ---------------------------------------------------------------------------------------------------
// phase 3: rotary embedding, cache append, split-KV grouped-query decode attention, split merge   (steps 5-6)
// ---------------------------------------------------------------------------------------------------
// One work item = (sequence, KV head, split of `split_tokens` cache slots).  The G query heads of the group share
// every key/value they read.  A token's head vector is spread over HD/8 lanes (16 bytes each), so a wave-wide
// load covers 64/(HD/8) consecutive tokens = 1 KiB of contiguous cache.  Each lane group keeps its own online
// softmax state; the groups of all 8 waves are merged through LDS, the splits through a workspace in global
// memory by whichever workgroup arrives last at the (sequence, KV head) counter.
template <int G, int HD>
struct AttnLds {
    static constexpr int LPT = HD / 8;          // lanes per token
    static constexpr int TPI = kWave / LPT;     // tokens per wave-wide load
    static constexpr int NSTREAM = kWaves * TPI; // independent softmax streams per workgroup
    float q[G][HD];
    float cs[HD / 2], sn[HD / 2];
    float knew[HD], vnew[HD];
    float acc[NSTREAM][G][HD];
    float ml[NSTREAM][G][2];
    int is_last;
};

template <int G, int HD>
__device__ void phase_attn(const DraftParams &p, int step, int vb, int nvb, char *smem) {
    using L = AttnLds<G, HD>;
    constexpr int LPT = L::LPT, TPI = L::TPI, NSTREAM = L::NSTREAM, U = 4;
    L &s = *reinterpret_cast<L *>(smem);
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int c = lane % LPT, tq = lane / LPT;
    const int T = p.split_tokens, S = p.max_splits;
    const int n_items = p.B * p.Hkv * S;
    const float scale = 1.0f / sqrtf((float)HD);
    const int PW = HD + 2; // floats per (head, split) partial: acc[HD], max, sum

    for (int item = vb; item < n_items; item += nvb) {
        const int b = item / (p.Hkv * S), rem = item % (p.Hkv * S), kvh = rem / S, sp = rem % S;
        const bool dead = seq_dead(p, b);
        const int Lb = dead ? 0 : p.kv_len[b];
        const int len = Lb + step + 1, pnew = len - 1;
        const int nsplit = (len + T - 1) / T;
        if (sp >= nsplit) continue; // uniform for the workgroup
        const int t0 = sp * T, t1 = min(t0 + T, len);
        const bool last = (sp == nsplit - 1);
        const int ntok = last ? (t1 - 1 - t0) : (t1 - t0); // slots read from the cache; the new token comes from qkv
        const uint16_t *kc = p.k_cache + ((size_t)b * p.Hkv + kvh) * p.cap * HD;
        const uint16_t *vc = p.v_cache + ((size_t)b * p.Hkv + kvh) * p.cap * HD;
        const float *qkv = p.qkv + (size_t)b * p.qkv_dim;

        __syncthreads(); // LDS of the previous item is free
        if (tid < HD / 2) {
            // angle in double: positions reach 2^15 and the pair frequency spans six decades
            double inv = pow((double)p.theta, -2.0 * (double)tid / (double)HD);
            double sn, cs;
            sincos((double)pnew * inv, &sn, &cs);
            s.cs[tid] = (float)cs;
            s.sn[tid] = (float)sn;
        }
        __syncthreads();
        for (int idx = tid; idx < G * HD / 2; idx += kBlock) {
            int gq = idx / (HD / 2), jj = idx % (HD / 2);
            const float *src = qkv + (size_t)(kvh * G + gq) * HD;
            float a = src[jj], bb = src[jj + HD / 2], cs = s.cs[jj], sn = s.sn[jj];
            s.q[gq][jj] = (a * cs - bb * sn) * scale;
            s.q[gq][jj + HD / 2] = (bb * cs + a * sn) * scale;
        }
        if (last) {
            uint16_t *kdst = p.k_cache + (((size_t)b * p.Hkv + kvh) * p.cap + pnew) * HD;
            uint16_t *vdst = p.v_cache + (((size_t)b * p.Hkv + kvh) * p.cap + pnew) * HD;
            if (tid < HD / 2) {
                const float *src = qkv + p.qd + (size_t)kvh * HD;
                float a = src[tid], bb = src[tid + HD / 2], cs = s.cs[tid], sn = s.sn[tid];
                uint16_t r0 = f32_to_bf16(a * cs - bb * sn), r1 = f32_to_bf16(bb * cs + a * sn);
                s.knew[tid] = bf16_to_f32(r0);
                s.knew[tid + HD / 2] = bf16_to_f32(r1);
                if (!dead) {
                    kdst[tid] = r0;
                    kdst[tid + HD / 2] = r1;
                }
            } else if (tid >= kWave * 2 && tid < kWave * 2 + HD) {
                int e = tid - kWave * 2;
                uint16_t r = f32_to_bf16(qkv[p.qd + p.kvd + (size_t)kvh * HD + e]);
                s.vnew[e] = bf16_to_f32(r);
                if (!dead) vdst[e] = r;
            }
        }
        __syncthreads();

        float q[G][8];
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int e = 0; e < 8; ++e) q[g][e] = s.q[g][c * 8 + e];
        float mx[G], sum[G], acc[G][8];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            mx[g] = -INFINITY;
            sum[g] = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
        }

        auto absorb = [&](const float(&sc)[U][G], const float(&vv)[U][8], const bool(&ok)[U]) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float mb = mx[g];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (ok[u]) mb = fmaxf(mb, sc[u][g]);
                if (mb == -INFINITY) continue;
                float alpha = expf(mx[g] - mb); // 0 when nothing was absorbed before
                float sm = sum[g] * alpha;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[g][e] *= alpha;
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (ok[u]) {
                        float pr = expf(sc[u][g] - mb);
                        sm += pr;
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[g][e] += pr * vv[u][e];
                    }
                mx[g] = mb;
                sum[g] = sm;
            }
        };

        const int nblk = (ntok + TPI - 1) / TPI;
        for (int base = wave; base < nblk; base += kWaves * U) {
            u32x4 kr[U], vr[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int t = (base + u * kWaves) * TPI + tq;
                ok[u] = t < ntok;
                size_t off = (size_t)(t0 + t) * HD + c * 8;
                kr[u] = ok[u] ? ldg16(kc + off) : u32x4{0u, 0u, 0u, 0u};
                vr[u] = ok[u] ? ldg16(vc + off) : u32x4{0u, 0u, 0u, 0u};
            }
            float sc[U][G], vv[U][8];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float kf[8] = {lo_half(kr[u].x), hi_half(kr[u].x), lo_half(kr[u].y), hi_half(kr[u].y),
                               lo_half(kr[u].z), hi_half(kr[u].z), lo_half(kr[u].w), hi_half(kr[u].w)};
                vv[u][0] = lo_half(vr[u].x);
                vv[u][1] = hi_half(vr[u].x);
                vv[u][2] = lo_half(vr[u].y);
                vv[u][3] = hi_half(vr[u].y);
                vv[u][4] = lo_half(vr[u].z);
                vv[u][5] = hi_half(vr[u].z);
                vv[u][6] = lo_half(vr[u].w);
                vv[u][7] = hi_half(vr[u].w);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float a = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) a += q[g][e] * kf[e];
                    sc[u][g] = (LPT == 16) ? row16_sum(a) : oct_sum(a);
                }
            }
            absorb(sc, vv, ok);
        }
        if (last && wave == 0) { // the token being appended, from LDS; every lane group computes it, group 0 keeps it
            float sc[U][G], vv[U][8];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                ok[u] = (u == 0) && (tq == 0);
#pragma unroll
                for (int g = 0; g < G; ++g) sc[u][g] = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) vv[u][e] = 0.f;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) vv[0][e] = s.vnew[c * 8 + e];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float a = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) a += q[g][e] * s.knew[c * 8 + e];
                sc[0][g] = (LPT == 16) ? row16_sum(a) : oct_sum(a);
            }
            absorb(sc, vv, ok);
        }

        // merge the lane groups of the workgroup
        const int stream = wave * TPI + tq;
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s.acc[stream][g][c * 8 + e] = acc[g][e];
            if (c == 0) {
                s.ml[stream][g][0] = mx[g];
                s.ml[stream][g][1] = sum[g];
            }
        }
        __syncthreads();
        for (int o = tid; o < G * HD; o += kBlock) {
            int g = o / HD, dd = o % HD;
            float M = -INFINITY;
            for (int st = 0; st < NSTREAM; ++st) M = fmaxf(M, s.ml[st][g][0]);
            float Ls = 0.f, A = 0.f;
            for (int st = 0; st < NSTREAM; ++st) {
                float mm = s.ml[st][g][0];
                if (mm != -INFINITY) {
                    float w = expf(mm - M);
                    Ls += s.ml[st][g][1] * w;
                    A += s.acc[st][g][dd] * w;
                }
            }
            int hq = kvh * G + g;
            if (nsplit == 1) {
                p.attn[(size_t)b * p.qd + (size_t)hq * HD + dd] = A / Ls;
            } else {
                float *dst = p.attn_part + (((size_t)b * p.Hq + hq) * S + sp) * PW;
                dst[dd] = A;
                if (dd == 0) {
                    dst[HD] = M;
                    dst[HD + 1] = Ls;
                }
            }
        }
        if (nsplit > 1) {
            __threadfence();
            __syncthreads();
            if (tid == 0) {
                int old = __hip_atomic_fetch_add(&p.attn_cnt[b * p.Hkv + kvh], 1, __ATOMIC_ACQ_REL,
                                                 __HIP_MEMORY_SCOPE_AGENT);
                s.is_last = (old == nsplit - 1);
            }
            __syncthreads();
            if (s.is_last) {
                __threadfence();
                for (int o = tid; o < G * HD; o += kBlock) {
                    int g = o / HD, dd = o % HD, hq = kvh * G + g;
                    const float *src = p.attn_part + ((size_t)b * p.Hq + hq) * S * PW;
                    float M = -INFINITY;
                    for (int s2 = 0; s2 < nsplit; ++s2) M = fmaxf(M, src[(size_t)s2 * PW + HD]);
                    float Ls = 0.f, A = 0.f;
                    for (int s2 = 0; s2 < nsplit; ++s2) {
                        float w = expf(src[(size_t)s2 * PW + HD] - M);
                        Ls += src[(size_t)s2 * PW + HD + 1] * w;
                        A += src[(size_t)s2 * PW + dd] * w;
                    }
                    p.attn[(size_t)b * p.qd + (size_t)hq * HD + dd] = A / Ls;
                }
                if (tid == 0) p.attn_cnt[b * p.Hkv + kvh] = 0; // ready for the next step
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// phase 4: output projection + residual                                      (step 7)
// ---------------------------------------------------------------------------------------------------
__device__ void phase_oproj(const DraftParams &p, int, int vb, int nvb, char *smem) {
    const int d = p.d, K = p.qd;
    int r0, r1;
    row_share(d, vb, nvb, r0, r1);
    const int nbmax = p.nb_q;
    GemvLds l = gemv_lds(smem, K, nbmax, 1);
    for (int b0 = 0; b0 < p.B; b0 += nbmax) {
        int nb = min(nbmax, p.B - b0);
        __syncthreads();
        for (int i = 0; i < nb; ++i)
            stage_plain(p.attn + (size_t)(b0 + i) * K, K, l.kpad, l.hi + (size_t)i * l.kpad, l.lo + (size_t)i * l.kpad);
        __syncthreads();
        auto rowptr = [&](int, int row) { return p.w_o + (size_t)row * K; };
        auto epi = [&](int i, int row, float(&s)[1]) {
            size_t o = (size_t)(b0 + i) * d + row;
            p.x1[o] = p.x[o] + s[0];
        };
        gemv_rows<1, 8>(rowptr, K, r0, r1, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, epi);
    }
}

// ---------------------------------------------------------------------------------------------------
// phase 5: MLP-input RMSNorm + gate and up projections + SiLU(gate) * up       (step 8)
// ---------------------------------------------------------------------------------------------------
__device__ void phase_gateup(const DraftParams &p, int, int vb, int nvb, char *smem) {
    const int d = p.d, F = p.F;
    int r0, r1;
    row_share(F, vb, nvb, r0, r1);
    const int nbmax = p.nb_d;
    GemvLds l = gemv_lds(smem, d, nbmax, 2);
    for (int b0 = 0; b0 < p.B; b0 += nbmax) {
        int nb = min(nbmax, p.B - b0);
        __syncthreads();
        for (int i = 0; i < nb; ++i)
            stage_rmsnorm<false>(p.x1 + (size_t)(b0 + i) * d, p.g_mlp, d, p.eps, l.hi + (size_t)i * l.kpad,
                                 l.lo + (size_t)i * l.kpad, l.red, nullptr);
        __syncthreads();
        auto rowptr = [&](int mt, int row) { return (mt == 0 ? p.w_gate : p.w_up) + (size_t)row * d; };
        auto epi = [&](int i, int row, float(&s)[2]) {
            float gt = s[0];
            p.m[(size_t)(b0 + i) * F + row] = (gt / (1.0f + expf(-gt))) * s[1];
        };
        gemv_rows<2, 4>(rowptr, d, r0, r1, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, epi);
    }
}

// ---------------------------------------------------------------------------------------------------
// phase 6: down projection + residual                                         (step 9, first half)
// ---------------------------------------------------------------------------------------------------
__device__ void phase_down(const DraftParams &p, int, int vb, int nvb, char *smem) {
    const int d = p.d, K = p.F;
    int r0, r1;
    row_share(d, vb, nvb, r0, r1);
    const int nbmax = p.nb_down;
    GemvLds l = gemv_lds(smem, K, nbmax, 1);
    for (int b0 = 0; b0 < p.B; b0 += nbmax) {
        int nb = min(nbmax, p.B - b0);
        __syncthreads();
        for (int i = 0; i < nb; ++i)
            stage_plain(p.m + (size_t)(b0 + i) * K, K, l.kpad, l.hi + (size_t)i * l.kpad, l.lo + (size_t)i * l.kpad);
        __syncthreads();
        auto rowptr = [&](int, int row) { return p.w_down + (size_t)row * K; };
        auto epi = [&](int i, int row, float(&s)[1]) {
            size_t o = (size_t)(b0 + i) * d + row;
            p.x2[o] = p.x1[o] + s[0];
        };
        gemv_rows<1, 8>(rowptr, K, r0, r1, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, epi);
    }
}

// ---------------------------------------------------------------------------------------------------
// phase 7: final RMSNorm + compressed output head + argmax                       (steps 9-10; Eq. (3))
// ---------------------------------------------------------------------------------------------------
// Row i of the compressed head is lm_head[ids[i]]; rows are dealt out in subset order, so every workgroup scans a
// contiguous, ascending range of subset indices.  Each reducing thread keeps the best (logit, index) it has seen;
// the workgroup's winner per sequence goes into a 64-bit atomic max whose key orders by logit, then by lower index.
__device__ void phase_lmhead(const DraftParams &p, int step, int vb, int nvb, char *smem) {
    const int d = p.d, n = p.n;
    int r0, r1;
    row_share(n, vb, nvb, r0, r1);
    const int nbmax = p.nb_d;
    GemvLds l = gemv_lds(smem, d, nbmax, 1);
    for (int b0 = 0; b0 < p.B; b0 += nbmax) {
        int nb = min(nbmax, p.B - b0);
        __syncthreads();
        for (int i = 0; i < nb; ++i) {
            int b = b0 + i;
            // workgroup 0 also publishes the step's output hidden state: for the next step and for the caller
            float *hh = (vb == 0) ? p.hhat + (size_t)b * d : nullptr;
            float *ho = (vb == 0 && p.hidden_out) ? p.hidden_out + ((size_t)b * p.K + step) * d : nullptr;
            stage_rmsnorm<false>(p.x2 + (size_t)b * d, p.g_final, d, p.eps, l.hi + (size_t)i * l.kpad,
                                 l.lo + (size_t)i * l.kpad, l.red, hh, ho);
        }
        __syncthreads();
        unsigned long long best = 0ull;
        auto rowptr = [&](int, int row) {
            int r = p.ids ? p.ids[row] : row;
            return p.lm_head + (size_t)r * d;
        };
        auto epi = [&](int i, int row, float(&s)[1]) {
            if (p.logits_out) p.logits_out[((size_t)(b0 + i) * p.K + step) * n + row] = s[0];
            unsigned long long key = argmax_key(s[0], (uint32_t)row);
            best = key > best ? key : best;
        };
        gemv_rows<1, 8>(rowptr, d, r0, r1, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, epi);
        // threads 16*i .. 16*i+15 hold candidates of sequence i
        if ((int)threadIdx.x < 16 * nb) {
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) {
                unsigned long long o = __shfl_xor(best, off, kWave);
                best = o > best ? o : best;
            }
            if ((threadIdx.x & 15) == 0 && best != 0ull)
                atomicMax(&p.keys[(size_t)step * p.max_batch + b0 + (threadIdx.x >> 4)], best);
        }
    }
}

// after the last step: publish the last draft id
__device__ void phase_finalize(const DraftParams &p, int vb) {
    if (vb == 0 && (int)threadIdx.x < p.B) {
        int b = threadIdx.x;
        uint32_t i = key_index(p.keys[(size_t)(p.K - 1) * p.max_batch + b]);
        if (i >= (uint32_t)p.n) i = 0;
        p.draft_out[(size_t)b * p.K + p.K - 1] = seq_dead(p, b) ? -1 : (p.ids ? p.ids[i] : (int)i);
    }
}

} // namespace mtp
