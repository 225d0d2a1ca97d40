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
    float *x, *qkv, *attn, *o, *gu, *dn, *hhat, *attn_part; // o = w_o attn, gu = [w_gate y2; w_up y2], dn = w_down m
                                                            // (residuals and SiLU*mul are applied by the consumers)
    int *err;                 // sticky error word
    const double *rope_inv;   // [hd/2] rotary pair frequencies theta^(-2j/hd), computed on the host in double
    unsigned long long *cand; // [max_draft_steps][max_batch][head_grid] packed (logit, index) maximum of every
                              // workgroup of the output-head phase; the consumer takes the maximum over them
    int head_grid;            // workgroups of the output-head phase = candidates per sequence (their stride in cand)
    // One id list per sequence (several languages in one batch, Sec. 2.2): the output head is launched once per group
    // of adjacent sequences with ids/n of that group; whoever turns a winner into a token id looks the sequence up.
    const int *seq_list;             // [B] slot of each sequence's list in the tables below, or null: one list, ids/n
    const int *const *list_ids;      // per slot: the id list (null = the full vocabulary)
    const int *list_n;               // per slot: rows of the head
    const int *list_cands;           // per slot: candidates the head's launch leaves per sequence (<= head_grid)
    int seq_lo, seq_hi;              // output head, launch per phase: sequences of this launch (0, B if one list)
    int logit_stride;                // floats per (sequence, step) in logits_out: n, or the largest n of the lists
    int fused_gemv_bytes;     // single-launch kernel: bytes of LDS shared by the staged activations and the attention
    long long bar_timeout;    // wall-clock ticks a workgroup may wait for a hand-over before giving up
    long long *trace;         // optional wall-clock stamps (100 MHz) of every workgroup of the single-launch kernel
    int max_batch;
    // launch plan
    int split_tokens, max_splits; // attention: tokens per split, splits per (sequence, KV head)
    int mfma_attn;                // the splits are long enough for the matrix-core attention
    int own_hidden;               // step 1 of this call starts from hhat (fp32, put there by the host: the head's own
                                  // output of an earlier call) instead of hidden_in (bf16, the target model's)
    // Several new positions per sequence (first draft step over a block): every phase sees one row per (position,
    // sequence), row = position * sequences + sequence, B = rows, with a cache length per ROW in kv_len.  A small
    // kernel appends every row's key and value before the attention, which then runs once over all rows: a row's
    // cache is that of sequence row % ext_B, and its own position is read from the cache like the others.
    int kv_appended, ext_B;
    int nb_proj, nb_d, nb_q, nb_down; // sequences staged in LDS per pass, by reduction length (2d, d, Hq*hd, F)
    // batched path (two or more sequences): activations travel between the phases as bf16 hi + lo in global memory
    uint16_t *act[2];    // two [max_batch][a_stride] hi arrays, each followed (a_lo elements later) by its lo array
    size_t a_lo;
    int a_stride;
    uint16_t *attn_split; // where the attention phases also leave their result split (nullptr: they do not)
    float *ssq;          // [3][max_batch][d/16] sums of squares over 16-row tiles of x, x1, x2
    float *part;         // partial sums of the row groups, [KP][tiles][sequence tiles][64] x 4 floats
    int *ticket;         // arrival counters of the row groups (zero between launches)
    int *attn_ticket;    // [max_batch][Hkv] arrival counters of the attention splits (zero between phases): the
                         // workgroup that finishes last merges the splits
    int *attn_queue;     // two words (zero between launches): next item of the attention launch that hands its items
                         // out one by one, and the workgroups that have left it
    int b0, nb;          // sequences of this pass
    // Hand-over by tagged elements (single-launch kernel for one sequence without grid barriers): every element of
    // a vector that crosses from one phase to the next is a 64-bit word (float bits, tag in the upper half); the
    // tag names the (call, step, phase) that produced it, so a consumer that polls an element knows when it is there.
    unsigned long long *xt, *qkvt, *attnt, *ot, *gut, *dnt; // [d], [qkv_dim], [qd], [d], [2F], [d]
    unsigned long long *candt; // [max_draft_steps][head_grid][2]: (orderable logit, tag), (token id, tag)
    unsigned tag_base;         // tag of (step, section) = tag_base + 8 * step + section + 1; never 0
    int bg_rg[6], bg_kp[6]; // row groups and reduction parts of the six matrix phases
    int bg_sep[6];          // 1: the phase's epilogue runs as a kernel of its own
};

enum : int { kErrKvOverflow = 1, kErrTokenRange = 2, kErrBarrierTimeout = 4 };
// matrix phases of the batched path, and the vectors whose sums of squares travel with them
enum : int { BG_PROJ = 0, BG_QKV, BG_OPROJ, BG_GATEUP, BG_DOWN, BG_LMHEAD, BG_COUNT };
enum : int { SSQ_X = 0, SSQ_X1, SSQ_X2, SSQ_COUNT };

// ---------------------------------------------------------------------------------------------------
// tagged hand-over elements
// ---------------------------------------------------------------------------------------------------
// sections of a draft step whose results cross to other workgroups, in order; tag = tag_base + 8 * step + section + 1
enum : int { TS_X = 0, TS_QKV, TS_ATTN, TS_O, TS_GU, TS_DN, TS_CAND };
__device__ __forceinline__ unsigned step_tag(const DraftParams &p, int step, int section) {
    return p.tag_base + 8u * (unsigned)step + (unsigned)section + 1u;
}
__device__ __forceinline__ unsigned long long pack_tagged(float v, unsigned tag) {
    return ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(v);
}
__device__ __forceinline__ void st_tagged(unsigned long long *p, float v, unsigned tag) {
    __hip_atomic_store(p, pack_tagged(v, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Bounded wait shared by every poll loop of the barrier-free kernel: true once the time limit has passed (then the
// sticky error word is set and every later wait of every workgroup gives up at its first check, so the grid drains).
struct PollClock {
    long long t0;
    unsigned spins;
    __device__ __forceinline__ PollClock() : t0(wall_clock64()), spins(0) {}
    __device__ __forceinline__ bool expired(const DraftParams &p) {
        if ((++spins & 31u) != 0) return false;
        if (__hip_atomic_load(p.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kErrBarrierTimeout) return true;
        if (wall_clock64() - t0 > p.bar_timeout) {
            atomicOr(p.err, kErrBarrierTimeout);
            return true;
        }
        return false;
    }
};
// one element, polled until its tag is the wanted one
__device__ __forceinline__ float ld_tagged(const DraftParams &p, const unsigned long long *src, unsigned tag) {
    unsigned long long w = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((unsigned)(w >> 32) != tag) {
        PollClock clk;
        do {
            w = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } while ((unsigned)(w >> 32) != tag && !clk.expired(p));
    }
    return __uint_as_float((unsigned)w);
}

// two elements, polled together
__device__ __forceinline__ void ld_tagged2(const DraftParams &p, const unsigned long long *a, const unsigned long long *b,
                                           unsigned tag, float &va, float &vb) {
    unsigned long long wa = __hip_atomic_load(a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned long long wb = __hip_atomic_load(b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((unsigned)(wa >> 32) != tag || (unsigned)(wb >> 32) != tag) {
        PollClock clk;
        do {
            wa = __hip_atomic_load(a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            wb = __hip_atomic_load(b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } while (((unsigned)(wa >> 32) != tag || (unsigned)(wb >> 32) != tag) && !clk.expired(p));
    }
    va = __uint_as_float((unsigned)wa);
    vb = __uint_as_float((unsigned)wb);
}

// ---------------------------------------------------------------------------------------------------
// per-sequence state helpers
// ---------------------------------------------------------------------------------------------------
constexpr int kRowInactive = -0x40000000; // kv_len of a (position, sequence) row beyond the sequence's new positions
__device__ __forceinline__ bool seq_dead(const DraftParams &p, int b) {
    int L = p.kv_len[b];
    return L < 0 || L + p.K > p.cap;
}
// dead because its cache cannot take the new entries (or its length is invalid): reported; an inactive row is not
__device__ __forceinline__ bool seq_overflows(const DraftParams &p, int b) {
    return seq_dead(p, b) && p.kv_len[b] != kRowInactive;
}

// maximum of a 64-bit key over the workgroup; red64 holds kWaves words; contains two barriers
__device__ __forceinline__ unsigned long long block_max_u64(unsigned long long v, unsigned long long *red64) {
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        unsigned long long o = __shfl_xor(v, off, kWave);
        v = o > v ? o : v;
    }
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) red64[threadIdx.x / kWave] = v;
    __syncthreads();
    unsigned long long r = 0ull;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) r = red64[w] > r ? red64[w] : r;
    return r;
}

// Winner of the output head of `step` for sequence b: maximum over the candidates the head's workgroups left behind
// (larger logit first, then lower subset index).  Called by all threads of a workgroup; contains barriers.
// the output head as sequence b sees it: its id list, its row count, the candidates its launch left behind
struct SeqHead {
    const int *ids;
    int n, cands;
};
__device__ __forceinline__ SeqHead seq_head(const DraftParams &p, int b) {
    if (p.seq_list) {
        const int s = p.seq_list[b];
        return SeqHead{p.list_ids[s], p.list_n[s], p.list_cands[s]};
    }
    return SeqHead{p.ids, p.n, p.head_grid};
}

template <bool COH = false>
__device__ __forceinline__ unsigned long long winner_key(const DraftParams &p, int step, int b,
                                                         unsigned long long *red64) {
    const unsigned long long *cand = p.cand + ((size_t)step * p.max_batch + b) * p.head_grid;
    unsigned long long best = 0ull;
    const int ncand = seq_head(p, b).cands;
    for (int w = threadIdx.x; w < ncand; w += kBlock) {
        const unsigned long long c = ld_u64<COH>(cand + w);
        best = c > best ? c : best;
    }
    return block_max_u64(best, red64);
}
__device__ __forceinline__ int key_token(const DraftParams &p, int b, unsigned long long key) {
    const SeqHead h = seq_head(p, b);
    uint32_t i = key_index(key);
    if (i >= (uint32_t)h.n) i = 0;
    return h.ids ? h.ids[i] : (int)i;
}

// ---------------------------------------------------------------------------------------------------
// staging of activation vectors into LDS as bf16 hi + lo
// ---------------------------------------------------------------------------------------------------
constexpr int kMaxNormIter = 4; // d <= 4 * 4 * kBlock = 8192

// RMSNorm(u; g) of one vector of length d (Sec. 2.1: DeepSeek-V3 MTP module uses RMSNorm on both inputs), written to
// hi/lo (bf16) and optionally to out_f32.  SRC_BF16: u is bf16 bits, else float.  Contains barriers.
// add1/add2 (float, optional) are added to the source element-wise first, in that order: the residual stream is
// kept as its summands and put together where it is consumed.
// COH: the float source, add1, add2 are read and out_f32 is written with device-coherent accesses (out2_f32, an output
// of the call, is not).
template <bool SRC_BF16, bool COH = false>
__device__ __forceinline__ void stage_rmsnorm(const void *src, const uint16_t *gain, int d, float eps, uint16_t *hi, uint16_t *lo,
                              float *red, float *out_f32, float *out2_f32 = nullptr, const float *add1 = nullptr,
                              const float *add2 = nullptr) {
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
                f32x4 raw = ld_f32x4<COH>(static_cast<const float *>(src) + e);
                v[it][0] = raw.x;
                v[it][1] = raw.y;
                v[it][2] = raw.z;
                v[it][3] = raw.w;
            }
            if (add1) {
                f32x4 a = ld_f32x4<COH>(add1 + e);
                v[it][0] += a.x;
                v[it][1] += a.y;
                v[it][2] += a.z;
                v[it][3] += a.w;
            }
            if (add2) {
                f32x4 a = ld_f32x4<COH>(add2 + e);
                v[it][0] += a.x;
                v[it][1] += a.y;
                v[it][2] += a.z;
                v[it][3] += a.w;
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
            if (out_f32) st_f32x4<COH>(out_f32 + e, w);
            if (out2_f32) *reinterpret_cast<f32x4 *>(out2_f32 + e) = w;
        }
    }
}

// The same by ONE wave, in two passes over the source (the second pass hits L1/L2): used when a workgroup stages
// several sequences, one per wave, instead of one after the other.
template <bool SRC_BF16>
__device__ __forceinline__ void stage_rmsnorm_wave(const void *src, const uint16_t *gain, int d, float eps,
                                                   uint16_t *hi, uint16_t *lo, float *out_f32, float *out2_f32 = nullptr,
                                                   const float *add1 = nullptr, const float *add2 = nullptr) {
    const int lane = threadIdx.x & (kWave - 1);
    auto load4 = [&](int e, float(&v)[4]) {
        if (SRC_BF16) {
            u32x2 raw = *reinterpret_cast<const u32x2 *>(static_cast<const uint16_t *>(src) + e);
            v[0] = lo_half(raw.x);
            v[1] = hi_half(raw.x);
            v[2] = lo_half(raw.y);
            v[3] = hi_half(raw.y);
        } else {
            f32x4 raw = *reinterpret_cast<const f32x4 *>(static_cast<const float *>(src) + e);
            v[0] = raw.x;
            v[1] = raw.y;
            v[2] = raw.z;
            v[3] = raw.w;
        }
        if (add1) {
            f32x4 a = *reinterpret_cast<const f32x4 *>(add1 + e);
            v[0] += a.x;
            v[1] += a.y;
            v[2] += a.z;
            v[3] += a.w;
        }
        if (add2) {
            f32x4 a = *reinterpret_cast<const f32x4 *>(add2 + e);
            v[0] += a.x;
            v[1] += a.y;
            v[2] += a.z;
            v[3] += a.w;
        }
    };
    float ss = 0.f;
    for (int e = lane * 4; e < d; e += kWave * 4) {
        float v[4];
        load4(e, v);
#pragma unroll
        for (int q = 0; q < 4; ++q) ss += v[q] * v[q];
    }
    const float inv = 1.0f / sqrtf(wave_sum(ss) / (float)d + eps);
    for (int e = lane * 4; e < d; e += kWave * 4) {
        float v[4];
        load4(e, v);
        u32x2 g = *reinterpret_cast<const u32x2 *>(gain + e);
        float o[4] = {lo_half(g.x) * (v[0] * inv), hi_half(g.x) * (v[1] * inv), lo_half(g.y) * (v[2] * inv),
                      hi_half(g.y) * (v[3] * inv)};
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

// Staging of nb sequences: alone, a sequence gets the whole workgroup (shortest latency); several are dealt to the
// waves.  f(i, whole_workgroup) stages sequence i.  Ends with a barrier.
template <class F>
__device__ __forceinline__ void stage_sequences(int nb, F f) {
    __syncthreads();
    if (nb == 1) {
        f(0, true);
    } else {
        for (int i = threadIdx.x / kWave; i < nb; i += kWaves) f(i, false);
    }
    __syncthreads();
}

// winner_key by one wave
__device__ __forceinline__ unsigned long long winner_key_wave(const DraftParams &p, int step, int b) {
    const unsigned long long *cand = p.cand + ((size_t)step * p.max_batch + b) * p.head_grid;
    unsigned long long best = 0ull;
    const int ncand = seq_head(p, b).cands;
    for (int w = threadIdx.x & (kWave - 1); w < ncand; w += kWave) best = cand[w] > best ? cand[w] : best;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        unsigned long long o = __shfl_xor(best, off, kWave);
        best = o > best ? o : best;
    }
    return best;
}

// plain copy of a float vector of length K (multiple of 4) into hi/lo, zero-padded to kpad
template <bool COH = false>
__device__ __forceinline__ void stage_plain(const float *src, int K, int kpad, uint16_t *hi, uint16_t *lo) {
    for (int e = threadIdx.x * 4; e < kpad; e += kBlock * 4) {
        u32x2 ph = {0u, 0u}, pl = {0u, 0u};
        if (e < K) {
            f32x4 raw = ld_f32x4<COH>(src + e);
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

// m = silu(g) * u from the gate/up projection output gu = [g (F floats); u (F floats)], silu(z) = z / (1 + exp(-z)),
// into hi/lo, zero-padded to kpad
template <bool COH = false>
__device__ __forceinline__ void stage_swiglu(const float *gu, int F, int kpad, uint16_t *hi, uint16_t *lo) {
    for (int e = threadIdx.x * 4; e < kpad; e += kBlock * 4) {
        u32x2 ph = {0u, 0u}, pl = {0u, 0u};
        if (e < F) {
            f32x4 g = ld_f32x4<COH>(gu + e);
            f32x4 u = ld_f32x4<COH>(gu + F + e);
            float m[4] = {(g.x / (1.0f + expf(-g.x))) * u.x, (g.y / (1.0f + expf(-g.y))) * u.y,
                          (g.z / (1.0f + expf(-g.z))) * u.z, (g.w / (1.0f + expf(-g.w))) * u.w};
            uint16_t h[4], l[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) split_bf16(m[q], h[q], l[q]);
            ph.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
            ph.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
            pl.x = (uint32_t)l[0] | ((uint32_t)l[1] << 16);
            pl.y = (uint32_t)l[2] | ((uint32_t)l[3] << 16);
        }
        *reinterpret_cast<u32x2 *>(hi + e) = ph;
        *reinterpret_cast<u32x2 *>(lo + e) = pl;
    }
}

// rows [r0, r1) of workgroup vb when `rows` rows are dealt out as evenly as possible
__device__ __forceinline__ void row_share(int rows, int vb, int nvb, int &r0, int &r1) {
    int q = rows / nvb, rem = rows % nvb;
    r0 = vb * q + min(vb, rem);
    r1 = r0 + q + (vb < rem ? 1 : 0);
}

// ---------------------------------------------------------------------------------------------------
// weight-streaming core
// ---------------------------------------------------------------------------------------------------
// Barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding global load, which
// would drain the weight prefetch at each tile boundary.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// For rows [r0, r1) of NMAT matrices that share the input: out[mat][i][row] = sum_k W_mat[row][k] * act[i][k],
// i < nb sequences.  The rows are cut into 16-row tiles; the 8 waves split the reduction range of each tile and
// their partial sums meet in LDS.  A wave's work is a sequence of chunks (tile, part of its k-range); one chunk is
// eight 16-byte loads per lane = 8 KiB of weights.  A ring of kRingDepth chunks lives in registers: it is primed
// before the activations exist (so HBM is busy while they are staged, or while a grid barrier completes) and a
// slot is refilled as soon as its MFMAs have been issued, across tile boundaries.  The inner loop is branch-free:
// a chunk is always read from inside its row (shifted left at the end of the row) and lanes whose elements belong
// to another chunk, another wave or another sequence slot get a zero activation operand.
//   rowptr(mat, row) -> const uint16_t* : start of a weight row (K bf16, 16-byte aligned, finite values)
//   epi(i, row, sums[NMAT])             : called by one thread per (sequence, row)
// LDS: act_hi/act_lo [nb][kpad] bf16; partial [2][kWaves][NMAT][nbmax][16] float.
constexpr int kRingDepth = 3;  // weight chunks in flight per wave (3 x 8 KiB)
constexpr int kChunkLoads = 8; // 16-byte loads per lane per chunk
struct Ring {
    u32x4 b[kRingDepth][kChunkLoads];
};

struct GemvGeom {
    int K, r0, r1, ntiles, nks, ks0, ks1, nch, total; // total = ntiles * nch chunks for every wave of the workgroup
    int j, g, wave;
};

template <int NMAT>
__device__ __forceinline__ GemvGeom gemv_geom_rows(int K, int r0, int r1) {
    constexpr int U = kChunkLoads / NMAT;
    GemvGeom q;
    const int lane = threadIdx.x & (kWave - 1);
    q.wave = threadIdx.x / kWave;
    q.j = lane & 15;
    q.g = lane >> 4;
    q.K = K;
    q.r0 = r0;
    q.r1 = r1;
    q.nks = (K + 31) / 32;
    const int per = (q.nks + kWaves - 1) / kWaves;
    q.ks0 = min(q.wave * per, q.nks);
    q.ks1 = min(q.ks0 + per, q.nks);
    q.nch = (per + U - 1) / U;
    q.ntiles = max((r1 - r0 + 15) / 16, 0);
    q.total = q.ntiles * q.nch;
    return q;
}

// request chunk (tile, ch) of this wave into buf: per matrix one base address and immediate offsets
template <int NMAT, class RowPtr>
__device__ __forceinline__ void gemv_issue(const GemvGeom &q, RowPtr rowptr, u32x4 (&buf)[kChunkLoads], int tile,
                                           int ch) {
    constexpr int U = kChunkLoads / NMAT;
    const int row = min(q.r0 + tile * 16 + q.j, q.r1 - 1);
    const int kstart = min((q.ks0 + ch * U) * 32, q.K - U * 32); // the chunk never leaves its row
#pragma unroll
    for (int mt = 0; mt < NMAT; ++mt) {
        const uint16_t *base = rowptr(mt, row) + kstart + q.g * 8;
#pragma unroll
        for (int u = 0; u < U; ++u) buf[mt * U + u] = ldg16(base + u * 32);
    }
}

// fill the ring with the first kRingDepth chunks (fewer if the phase is shorter)
template <int NMAT, class RowPtr>
__device__ __forceinline__ void gemv_prime(const GemvGeom &q, RowPtr rowptr, Ring &ring) {
#pragma unroll
    for (int s = 0; s < kRingDepth; ++s)
        if (s < q.total) gemv_issue<NMAT>(q, rowptr, ring.b[s], s / q.nch, s % q.nch);
}

// consume the whole phase; the ring must have been primed and the activations staged
template <int NMAT, class RowPtr, class Epi>
__device__ __forceinline__ void gemv_run(const GemvGeom &q, RowPtr rowptr, Ring &ring, int nb, int nbmax,
                                         const uint16_t *act_hi, const uint16_t *act_lo, int kpad, float *partial,
                                         Epi &epi) {
    constexpr int U = kChunkLoads / NMAT;
    if (q.total <= 0) return;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    const int jact = min(q.j, nb - 1);
    const bool jok = q.j < nb;
    f32x4 acc_h[NMAT], acc_l[NMAT];
#pragma unroll
    for (int mt = 0; mt < NMAT; ++mt) {
        acc_h[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc_l[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    int ct = 0, cc = 0;                                   // chunk being consumed
    int it = kRingDepth / q.nch, ic = kRingDepth % q.nch; // chunk to request next
    for (int n0 = 0; n0 < q.total; n0 += kRingDepth) {
#pragma unroll
        for (int s = 0; s < kRingDepth; ++s) {
            if (n0 + s < q.total) { // uniform
                const int own_lo = (q.ks0 + cc * U) * 32;
                const int own_hi = min(q.ks0 + (cc + 1) * U, q.ks1) * 32;
                const int kstart = min(own_lo, q.K - U * 32);
                const int e0 = kstart + q.g * 8;
                const uint16_t *ah_p = act_hi + (size_t)jact * kpad + e0;
                const uint16_t *al_p = act_lo + (size_t)jact * kpad + e0;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const bool ok = jok && (e0 + u * 32 >= own_lo) && (e0 + u * 32 < own_hi);
                    u32x4 ah = *reinterpret_cast<const u32x4 *>(ah_p + u * 32);
                    u32x4 al = *reinterpret_cast<const u32x4 *>(al_p + u * 32);
                    ah = ok ? ah : zero4;
                    al = ok ? al : zero4;
#pragma unroll
                    for (int mt = 0; mt < NMAT; ++mt) {
                        acc_h[mt] = mfma16(ah, ring.b[s][mt * U + u], acc_h[mt]);
                        acc_l[mt] = mfma16(al, ring.b[s][mt * U + u], acc_l[mt]);
                    }
                    // keep the scheduler from hoisting all of the chunk's LDS reads (64 registers) above the MFMAs
                    if (u % 2 == 1) __builtin_amdgcn_sched_barrier(0);
                }
                if (n0 + s + kRingDepth < q.total) { // the slot is free again: request the chunk kRingDepth ahead
                    gemv_issue<NMAT>(q, rowptr, ring.b[s], it, ic);
                    if (++ic == q.nch) {
                        ic = 0;
                        ++it;
                    }
                }
                if (cc == q.nch - 1) { // tile complete: meet the other waves' partial sums in LDS
                    float *pb = partial + (size_t)(ct & 1) * kWaves * NMAT * nbmax * 16;
#pragma unroll
                    for (int mt = 0; mt < NMAT; ++mt) {
                        f32x4 sv = acc_h[mt] + acc_l[mt];
                        float e[4] = {sv.x, sv.y, sv.z, sv.w};
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            int i = q.g * 4 + v;
                            if (i < nb) pb[((q.wave * NMAT + mt) * nbmax + i) * 16 + q.j] = e[v];
                        }
                        acc_h[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
                        acc_l[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
                    lds_barrier();
                    if ((int)threadIdx.x < 16 * nb) {
                        int i = threadIdx.x >> 4, jj = threadIdx.x & 15;
                        float sums[NMAT];
#pragma unroll
                        for (int mt = 0; mt < NMAT; ++mt) {
                            float sacc = 0.f;
#pragma unroll
                            for (int w = 0; w < kWaves; ++w) sacc += pb[((w * NMAT + mt) * nbmax + i) * 16 + jj];
                            sums[mt] = sacc;
                        }
                        int row = q.r0 + ct * 16 + jj;
                        if (row < q.r1) epi(i, row, sums);
                    }
                    cc = 0;
                    ++ct;
                } else {
                    ++cc;
                }
            }
        }
    }
}

// one pass of a phase launched on its own: request the first chunks, stage the activations, stream the rest
template <int NMAT, int UNUSED, class RowPtr, class Stage, class Epi>
__device__ __forceinline__ void gemv_rows(RowPtr rowptr, int K, int r0, int r1, int nb, int nbmax,
                                          const uint16_t *act_hi, const uint16_t *act_lo, int kpad, float *partial,
                                          Stage stage, Epi &epi) {
    const GemvGeom q = gemv_geom_rows<NMAT>(K, r0, r1);
    Ring ring;
    gemv_prime<NMAT>(q, rowptr, ring);
    stage(); // ends with a barrier: the activations are visible to every wave
    gemv_run<NMAT>(q, rowptr, ring, nb, nbmax, act_hi, act_lo, kpad, partial, epi);
}

// ---------------------------------------------------------------------------------------------------
// row mode: the weight-streaming core for up to four sequences
// ---------------------------------------------------------------------------------------------------
// A wave owns whole weight rows and reads them front to back: every load instruction fetches 1 KiB of one row
// (lane l gets elements [512 b + 8 l, 512 b + 8 l + 8) of 512-element block b), and the activations are read from
// LDS in exactly the same lane order.  Fed to the 16x16x32 MFMA as they are, lane (i, g) of the A operand and lane
// (j, g) of the B operand hold elements (16 g + i) 8 .. +8 and (16 g + j) 8 .. +8 of the block, so the DIAGONAL of
// the 16x16 result holds sixteen partial dot products that together cover the block; accumulating over the blocks of
// a row and summing the diagonal at the end of the row gives the row's dot product.  15/16 of the MFMA work is
// thrown away, which is free here: the matrix cores idle at batch 1, while the vector ALUs (address arithmetic
// only), the row-contiguous access pattern and the absence of any cross-wave reduction are what a bandwidth-bound
// kernel wants.  Rows are dealt evenly to all waves of the grid, so phases whose row count is not a multiple of the
// 16-row MFMA tile (q/k/v, gate/up) stay balanced.  One MFMA pair (hi, lo) per sequence per block.
constexpr int kRowModeMaxSeq = 4;

// NB: compile-time number of sequence slots (1, 2 or 4); slots at or beyond nb compute on a zero operand.  The
// consume loop must stay straight-line code, or the compiler falls back to waiting for every outstanding load.
// DEPTH: chunks in flight per wave.  Two measure best (16 KiB per wave, 32 MiB over the chip); with three the phases
// run 3-5 % slower.
constexpr int kRowDepth = 2;
template <int NMAT, int NB, bool STREAM, int DEPTH = kRowDepth, class RowPtr, class Stage, class Epi>
__device__ __forceinline__ void gemv_rowmode(RowPtr rowptr, int K, int rows, int vb, int nvb, int nb,
                                             const uint16_t *act_hi, const uint16_t *act_lo, int kpad, Stage stage,
                                             Epi &epi) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    // Rows are interleaved over all waves of the grid (row r belongs to wave r mod #waves): at any moment the grid
    // reads a compact, advancing window of the matrix, like one linear sweep, instead of thousands of far-apart streams.
    const int stride = nvb * kWaves;
    const int wr0 = vb * kWaves + wave;
    const int nrows = wr0 < rows ? (rows - wr0 + stride - 1) / stride : 0;
    const int wr_last = wr0 + max(nrows - 1, 0) * stride;
    const int nblk = (K + 511) / 512;                          // 512-element blocks per row (the last may overlap)
    const int cpr = (nblk + kChunkLoads - 1) / kChunkLoads;    // chunks per (row, matrix): a chunk never straddles rows
    const int nchunks = nrows * NMAT * cpr;                    // uniform per wave
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    // load stream position: (row, matrix, chunk within the row), and the number of chunks requested so far.  A
    // request past the wave's last chunk goes to an empty buffer (row 0, zero bytes): it returns zeros and moves no
    // data, so the ring is filled and refilled without a branch.  After a conditional load the compiler no longer
    // knows how many loads are outstanding and waits for all of them at the next use of any.
    int l_row = wr0, l_mt = 0, l_c = 0, l_n = 0;
    auto issue_chunk = [&](u32x4(&buf)[kChunkLoads]) {
        const bool live = l_n < nchunks;
        ++l_n;
        const row_rsrc rs = make_row_rsrc(rowptr(l_mt, live ? min(l_row, wr_last) : 0), live ? K * 2 : 0); // uniform
#pragma unroll
        for (int u = 0; u < kChunkLoads; ++u) {
            const int blk = min(l_c * kChunkLoads + u, nblk - 1); // empty slots of a row's last chunk re-read its last block
            buf[u] = row_load16<STREAM>(rs, lane * 16, min(blk * 512, K - 512) * 2);
        }
        if (++l_c == cpr) {
            l_c = 0;
            if (++l_mt == NMAT) {
                l_mt = 0;
                l_row += stride;
            }
        }
    };

    u32x4 ring[DEPTH][kChunkLoads];
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) issue_chunk(ring[s]);
    stage(); // ends with a barrier: the activations are visible to every wave
    if (nchunks <= 0) return;

    f32x4 acc_h[NB], acc_l[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        acc_h[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc_l[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    float sums[NB][NMAT];
    const int dv = (lane & 15) - 4 * (lane >> 4); // which of this lane's four results lies on the diagonal, if any
    int c_row = wr0, c_mt = 0, c_c = 0;
    for (int n0 = 0; n0 < nchunks; n0 += DEPTH) {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            // No branch around the loads of this body: slots past the wave's last chunk hold zeros and are "consumed"
            // like the others, and every slot is refilled, so the number of loads in flight at each wait is known at
            // compile time and a wait covers exactly the chunk that is consumed.
            {
#pragma unroll
                for (int u = 0; u < kChunkLoads; ++u) {
                    const int blk = c_c * kChunkLoads + u;
                    const int e0 = min(min(blk, nblk - 1) * 512, K - 512) + lane * 8;
                    // slots past the row's last block contribute nothing; a last block that was shifted left to stay
                    // inside the row only contributes the elements the block before it did not cover
                    const bool own = blk < nblk && e0 >= blk * 512;
#pragma unroll
                    for (int i = 0; i < NB; ++i) {
                        const int ia = min(i, nb - 1); // slots beyond nb re-read a valid row and are zeroed
                        u32x4 ah = *reinterpret_cast<const u32x4 *>(act_hi + (size_t)ia * kpad + e0);
                        u32x4 al = *reinterpret_cast<const u32x4 *>(act_lo + (size_t)ia * kpad + e0);
                        const bool use = own && i < nb;
                        ah = use ? ah : zero4;
                        al = use ? al : zero4;
                        acc_h[i] = mfma16(ah, ring[s][u], acc_h[i]);
                        acc_l[i] = mfma16(al, ring[s][u], acc_l[i]);
                    }
                }
                issue_chunk(ring[s]); // the slot is free again
                if (n0 + s < nchunks && ++c_c == cpr) { // end of a row of matrix c_mt: sum the diagonal
                    c_c = 0;
#pragma unroll
                    for (int i = 0; i < NB; ++i) {
                        f32x4 t = acc_h[i] + acc_l[i];
                        float v = dv == 0 ? t.x : dv == 1 ? t.y : dv == 2 ? t.z : dv == 3 ? t.w : 0.f;
                        v = wave_sum(v);
#pragma unroll
                        for (int mt = 0; mt < NMAT; ++mt) sums[i][mt] = (mt == c_mt) ? v : sums[i][mt];
                        acc_h[i] = f32x4{0.f, 0.f, 0.f, 0.f};
                        acc_l[i] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
                    if (++c_mt == NMAT) {
                        c_mt = 0;
                        if (lane == 0) {
#pragma unroll
                            for (int i = 0; i < NB; ++i)
                                if (i < nb) epi(i, c_row, sums[i]);
                        }
                        c_row += stride;
                    }
                }
            }
        }
    }
}

__device__ __forceinline__ bool use_row_mode(int nb, int K) { return nb <= kRowModeMaxSeq && K >= 512; }

// picks the core by batch chunk and reduction length (both uniform for the launch)
template <int NMAT, bool STREAM, class RowPtr, class Stage, class Epi>
__device__ __forceinline__ void gemv_auto(RowPtr rowptr, int K, int rows, int vb, int nvb, int nb, int nbmax,
                                          const uint16_t *act_hi, const uint16_t *act_lo, int kpad, float *partial,
                                          Stage stage, Epi &epi) {
    int r0, r1;
    row_share(rows, vb, nvb, r0, r1); // tile mode: a contiguous share of the rows per workgroup
    if (use_row_mode(nb, K)) {
        if (nb == 1)
            gemv_rowmode<NMAT, 1, STREAM>(rowptr, K, rows, vb, nvb, nb, act_hi, act_lo, kpad, stage, epi);
        else if (nb == 2)
            gemv_rowmode<NMAT, 2, STREAM>(rowptr, K, rows, vb, nvb, nb, act_hi, act_lo, kpad, stage, epi);
        else
            gemv_rowmode<NMAT, 4, STREAM>(rowptr, K, rows, vb, nvb, nb, act_hi, act_lo, kpad, stage, epi);
    } else
        gemv_rows<NMAT, 0>(rowptr, K, r0, r1, nb, nbmax, act_hi, act_lo, kpad, partial, stage, epi);
}

// carve-up of the dynamic LDS of a matrix-vector phase
struct GemvLds {
    uint16_t *hi, *lo;
    float *partial, *red;
    int kpad;
};
// Row stride of the staged activations: K rounded up to the MFMA depth, plus 16 bytes.  The sixteen lanes that read
// the same 16-byte column of sixteen different sequences then hit sixteen different groups of four LDS banks; with a
// stride that is a multiple of 256 bytes they would all hit the same group.
__host__ __device__ inline int gemv_kpad(int K) { return (K + 31) / 32 * 32 + 8; }
__host__ __device__ inline size_t gemv_lds_bytes(int K, int nb, int nmat) {
    size_t kpad = (size_t)gemv_kpad(K);
    return 2 * kpad * nb * sizeof(uint16_t) + (size_t)2 * kWaves * nmat * nb * 16 * sizeof(float) + 64;
}
__device__ inline GemvLds gemv_lds(char *smem, int K, int nb, int nmat) {
    GemvLds l;
    l.kpad = gemv_kpad(K);
    l.hi = reinterpret_cast<uint16_t *>(smem);
    l.lo = l.hi + (size_t)l.kpad * nb;
    l.partial = reinterpret_cast<float *>(l.lo + (size_t)l.kpad * nb);
    l.red = l.partial + (size_t)2 * kWaves * nmat * nb * 16;
    return l;
}


// ---------------------------------------------------------------------------------------------------
// phase 1: embedding gather + dual RMSNorm + concat + 2d->d projection   (steps 1-3 of the draft step)
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ void phase_proj(const DraftParams &p, int step, int vb, int nvb, char *smem) {
    const int d = p.d;
    if (step == 0 && vb == 0 && (int)threadIdx.x < p.B && seq_overflows(p, threadIdx.x)) atomicOr(p.err, kErrKvOverflow);
    const int nbmax = p.nb_proj;
    GemvLds l = gemv_lds(smem, 2 * d, nbmax, 1);
    for (int b0 = 0; b0 < p.B; b0 += nbmax) {
        int nb = min(nbmax, p.B - b0);
        auto stage = [&]() {
            stage_sequences(nb, [&](int i, bool whole) {
                const int b = b0 + i;
                const bool lead = whole ? threadIdx.x == 0 : (threadIdx.x & (kWave - 1)) == 0;
                // x_1 is the verified token; afterwards the previous step's draft (or the forced token)
                int tok;
                if (step == 0) {
                    tok = p.token_in[b];
                } else {
                    unsigned long long key = whole ? winner_key(p, step - 1, b, reinterpret_cast<unsigned long long *>(l.red))
                                                   : winner_key_wave(p, step - 1, b);
                    int did = key_token(p, b, key);
                    if (vb == 0 && lead) p.draft_out[(size_t)b * p.K + step - 1] = seq_dead(p, b) ? -1 : did;
                    tok = p.forced ? p.forced[(size_t)b * (p.K - 1) + step - 1] : did;
                }
                if (tok < 0 || tok >= p.V) { // reported, and replaced by id 0 so that every access stays in bounds
                    if (lead) atomicOr(p.err, kErrTokenRange);
                    tok = 0;
                }
                uint16_t *hi = l.hi + (size_t)i * l.kpad, *lo = l.lo + (size_t)i * l.kpad;
                if (whole) {
                    if (step == 0 && !p.own_hidden)
                        stage_rmsnorm<true>(p.hidden_in + (size_t)b * d, p.g_h, d, p.eps, hi, lo, l.red, nullptr);
                    else
                        stage_rmsnorm<false>(p.hhat + (size_t)b * d, p.g_h, d, p.eps, hi, lo, l.red, nullptr);
                    stage_rmsnorm<true>(p.embed + (size_t)tok * d, p.g_e, d, p.eps, hi + d, lo + d, l.red, nullptr);
                } else {
                    if (step == 0 && !p.own_hidden)
                        stage_rmsnorm_wave<true>(p.hidden_in + (size_t)b * d, p.g_h, d, p.eps, hi, lo, nullptr);
                    else
                        stage_rmsnorm_wave<false>(p.hhat + (size_t)b * d, p.g_h, d, p.eps, hi, lo, nullptr);
                    stage_rmsnorm_wave<true>(p.embed + (size_t)tok * d, p.g_e, d, p.eps, hi + d, lo + d, nullptr);
                }
            });
        };
        auto rowptr = [&](int, int row) { return p.w_proj + (size_t)row * 2 * d; };
        auto epi = [&](int i, int row, float(&s)[1]) { p.x[(size_t)(b0 + i) * d + row] = s[0]; };
        gemv_auto<1, true>(rowptr, 2 * d, d, vb, nvb, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, stage, epi);
    }
}

// ---------------------------------------------------------------------------------------------------
// phase 2: attention-input RMSNorm + fused QKV projection                  (step 4)
// Bias, rotary embedding and the cache append happen where q, k, v are consumed (phase_attn).
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ void phase_qkv(const DraftParams &p, int step, int vb, int nvb, char *smem) {
    const int d = p.d, rows = p.qkv_dim;
    const int nbmax = p.nb_d;
    GemvLds l = gemv_lds(smem, d, nbmax, 1);
    for (int b0 = 0; b0 < p.B; b0 += nbmax) {
        int nb = min(nbmax, p.B - b0);
        auto stage = [&]() {
            stage_sequences(nb, [&](int i, bool whole) {
                const float *src = p.x + (size_t)(b0 + i) * d;
                uint16_t *hi = l.hi + (size_t)i * l.kpad, *lo = l.lo + (size_t)i * l.kpad;
                if (whole)
                    stage_rmsnorm<false>(src, p.g_attn, d, p.eps, hi, lo, l.red, nullptr);
                else
                    stage_rmsnorm_wave<false>(src, p.g_attn, d, p.eps, hi, lo, nullptr);
            });
        };
        auto rowptr = [&](int, int row) {
            if (row < p.qd) return p.w_q + (size_t)row * d;
            if (row < p.qd + p.kvd) return p.w_k + (size_t)(row - p.qd) * d;
            return p.w_v + (size_t)(row - p.qd - p.kvd) * d;
        };
        // biases are added where q, k, v are consumed: the epilogue stays free of loads
        auto epi = [&](int i, int row, float(&s)[1]) { p.qkv[(size_t)(b0 + i) * rows + row] = s[0]; };
        gemv_auto<1, true>(rowptr, d, rows, vb, nvb, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, stage, epi);
    }
}

// ---------------------------------------------------------------------------------------------------
// phase 3: bias, rotary embedding, cache append, split-KV grouped-query decode attention      (steps 5-6)
// ---------------------------------------------------------------------------------------------------
// One work item = (sequence, KV head, split of `split_tokens` cache slots).  The G query heads of the group share
// every key/value they read.  A token's head vector is spread over HD/8 lanes (16 bytes each), so a wave-wide
// load covers 64/(HD/8) consecutive tokens = 1 KiB of contiguous cache.  Each lane group keeps its own online
// softmax state; the groups of all 8 waves are merged through LDS.  A sequence that fits one split is finished
// here; otherwise the item leaves (sum of p*V, max, sum of p) per head in the workspace and the item of the same
// (sequence, KV head) that finishes last merges them (merge_head).
// At batch 1 the phase moves little data and is bound by its chain of dependent memory round trips, so the first
// cache loads are issued before anything else and the rotary table costs no double-precision transcendental.
template <int G, int HD>
struct AttnLds {
    static constexpr int LPT = HD / 8;           // lanes per token
    static constexpr int TPI = kWave / LPT;      // tokens per wave-wide load
    static constexpr int NSTREAM = kWaves * TPI; // independent softmax streams per workgroup
    float q[G][HD];
    float cs[HD / 2], sn[HD / 2];
    float knew[HD], vnew[HD];
    float acc[NSTREAM][G][HD];
    float ml[NSTREAM][G][2];
    // the launch reserves 64 bytes more than the struct: the first word behind it is the "last split to finish" flag
};

// cos/sin of pos * inv_freq with the product and the reduction to [-pi, pi] in double, the rest in float
__device__ __forceinline__ void rope_cos_sin(int pos, double inv_freq, float &cs, float &sn) {
    const double two_pi_hi = 6.283185307179586232, two_pi_lo = 2.4492935982947064e-16, inv_two_pi = 0.15915494309189535;
    double ang = (double)pos * inv_freq;
    double n = rint(ang * inv_two_pi);
    double r = fma(-n, two_pi_lo, fma(-n, two_pi_hi, ang));
    float rf = (float)r;
    cs = cosf(rf);
    sn = sinf(rf);
}

// Merge of the split partials of one (sequence, query head) by ONE wave: weights exp(max_s - max) / sum over splits
// are formed once (in the wave-private LDS strip w of max_splits floats), then every lane sums its share of the head
// dimension with sixteen loads in flight.  PCOH: the partials are read with device-coherent loads; OCOH: the result
// is written with a device-coherent store.
template <int HD, bool PCOH, bool OCOH, bool TAGGED = false>
__device__ __forceinline__ void merge_head(const DraftParams &p, int b, int hq, int nsplit, float *w, int step = 0) {
    const int lane = threadIdx.x & (kWave - 1);
    const int S = p.max_splits, PW = HD + 2;
    const float *src = p.attn_part + ((size_t)b * p.Hq + hq) * S * PW;
    auto store = [&](int dd, float r) {
        if (TAGGED) { // one sequence: the consumer polls the element itself
            st_tagged(p.attnt + (size_t)hq * HD + dd, r, step_tag(p, step, TS_ATTN));
            return;
        }
        st_f32<OCOH>(p.attn + (size_t)b * p.qd + (size_t)hq * HD + dd, r);
        if (p.attn_split) {
            uint16_t h, l;
            split_bf16(r, h, l);
            const size_t at = (size_t)b * p.a_stride + (size_t)hq * HD + dd;
            p.attn_split[at] = h;
            p.attn_split[p.a_lo + at] = l;
        }
    };
    // Up to 32 splits (the common case at one sequence): one round of loads.  Lane s reads the (max, sum) of split s,
    // and every lane reads its HD/64 elements of all splits before any of it is used.
    constexpr int ND = HD / kWave, NF = 32;
    if (nsplit <= NF) {
        float m = -INFINITY, l = 0.f, t[ND][NF];
        if (lane < nsplit) {
            m = ld_f32<PCOH>(src + (size_t)lane * PW + HD);
            l = ld_f32<PCOH>(src + (size_t)lane * PW + HD + 1);
        }
#pragma unroll
        for (int u = 0; u < NF; ++u)
#pragma unroll
            for (int k = 0; k < ND; ++k) t[k][u] = u < nsplit ? ld_f32<PCOH>(src + (size_t)u * PW + lane + k * kWave) : 0.f;
        float M = m;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, kWave));
        const float e = lane < nsplit ? expf(m - M) : 0.f;
        const float inv = 1.0f / wave_sum(l * e);
        float A[ND];
#pragma unroll
        for (int k = 0; k < ND; ++k) A[k] = 0.f;
#pragma unroll
        for (int u = 0; u < NF; ++u) {
            const float wu = __shfl(e, u, kWave);
#pragma unroll
            for (int k = 0; k < ND; ++k) A[k] += t[k][u] * wu;
        }
#pragma unroll
        for (int k = 0; k < ND; ++k) store(lane + k * kWave, A[k] * inv);
        return;
    }
    float M = -INFINITY;
    for (int s2 = lane; s2 < nsplit; s2 += kWave) {
        float m = ld_f32<PCOH>(src + (size_t)s2 * PW + HD);
        w[s2] = m;
        M = fmaxf(M, m);
    }
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, kWave));
    float Ls = 0.f;
    for (int s2 = lane; s2 < nsplit; s2 += kWave) {
        float e = expf(w[s2] - M);
        w[s2] = e;
        Ls += ld_f32<PCOH>(src + (size_t)s2 * PW + HD + 1) * e;
    }
    Ls = wave_sum(Ls);
    const float inv = 1.0f / Ls;
    // w[] was written by this wave's own lanes: LDS ops of one wave complete in order, no barrier needed
    for (int dd = lane; dd < HD; dd += kWave) {
        float A = 0.f;
        int s2 = 0;
        for (; s2 + 16 <= nsplit; s2 += 16) {
            float t[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) t[u] = ld_f32<PCOH>(src + (size_t)(s2 + u) * PW + dd);
#pragma unroll
            for (int u = 0; u < 16; ++u) A += t[u] * w[s2 + u];
        }
        for (; s2 < nsplit; ++s2) A += ld_f32<PCOH>(src + (size_t)s2 * PW + dd) * w[s2];
        store(dd, A * inv);
    }
}

// COH: q/k/v are read, and the appended cache entries, the result and the split partials written, with
// device-coherent accesses (the phases of a step run inside one kernel)
struct NoHook {
    __device__ __forceinline__ void operator()() const {}
};
// before_q: called once, by all threads, after the first cache loads have been requested and before q/k/v are read
// TAGGED (one sequence, implies COH): q/k/v are polled as tagged elements and the result is written as tagged elements
// GS: an item serves GT / GS of the GT query heads of a KV head (items: sequence, KV head, split, part of the heads);
// the parts read the same keys and values.  The phase's stages are bound by vector instructions per workgroup, which
// go with tokens x heads: halving the heads per item halves them where halving the tokens would double the partials.
template <int GT, int HD, bool COH = false, bool TICKET = false, class Hook = NoHook, bool TAGGED = false, int GS = 1>
__device__ __forceinline__ void phase_attn(const DraftParams &p, int step, int vb, int nvb, char *smem, Hook before_q = Hook()) {
    static_assert(GT % GS == 0, "whole heads per part");
    constexpr int G = GT / GS; // query heads per item
    using L = AttnLds<G, HD>;
    // U blocks of TPI tokens per wave and round: one round covers kWaves * U * TPI tokens (with half the heads per
    // item the registers allow a fifth block, and the single-launch kernel's splits of up to 160 tokens need one round)
    constexpr int LPT = L::LPT, TPI = L::TPI, NSTREAM = L::NSTREAM, U = GS > 1 ? 5 : 4;
    L &s = *reinterpret_cast<L *>(smem);
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int c = lane % LPT, tq = lane / LPT;
    const int T = p.split_tokens, S = p.max_splits;
    const int n_seq_items = p.B * p.Hkv * S, n_items = n_seq_items * GS;
    const float scale = 1.0f / sqrtf((float)HD);
    const int PW = HD + 2; // floats per (head, split) partial: acc[HD], max, sum

    bool first_item = true;
    for (int item = vb; item < n_items; item += nvb) {
        // the parts of one (KV head, split) are n_seq_items apart: workgroups of the same compute die when that is a
        // multiple of eight, so the second reads the keys and values from its L2
        const int part = item / n_seq_items, it1 = item % n_seq_items;
        const int b = it1 / (p.Hkv * S), rem = it1 % (p.Hkv * S), kvh = rem / S, sp = rem % S;
        const int h0 = kvh * GT + part * G; // the item's first query head
        const bool dead = seq_dead(p, b);
        if (p.kv_appended && dead) continue; // a row that is not part of the block (uniform for the workgroup)
        const int Lb = dead ? 0 : p.kv_len[b];
        const int len = Lb + step + 1, pnew = len - 1;
        const int nsplit = (len + T - 1) / T;
        if (sp >= nsplit) continue; // uniform for the workgroup
        const int t0 = sp * T, t1 = min(t0 + T, len);
        // `last`: this split appends the new position and scores it from the projection output; when every row's
        // entry is in the cache already (kv_appended) no split does, and the new position is one more cached token
        const bool last = (sp == nsplit - 1) && !p.kv_appended;
        const int ntok = last ? (t1 - 1 - t0) : (t1 - t0); // slots read from the cache
        const int cb = p.kv_appended ? b % p.ext_B : b;     // whose cache
        const uint16_t *kc = p.k_cache + ((size_t)cb * p.Hkv + kvh) * p.cap * HD;
        const uint16_t *vc = p.v_cache + ((size_t)cb * p.Hkv + kvh) * p.cap * HD;
        const float *qkv = p.qkv + (size_t)b * p.qkv_dim;
        const int nblk = (ntok + TPI - 1) / TPI;

        u32x4 kr[U], vr[U];
        bool ok[U];
        auto load_blocks = [&](int base) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int t = (base + u * kWaves) * TPI + tq;
                ok[u] = t < ntok;
                size_t off = (size_t)(t0 + (ok[u] ? t : 0)) * HD + c * 8; // slot t0 is always inside the cache
                kr[u] = ldg16(kc + off);
                vr[u] = ldg16(vc + off);
            }
        };
        load_blocks(wave); // in flight while q, the rotary table and the new key/value are prepared
        if (first_item) {
            before_q();
            first_item = false;
        }

        // Every global input of the prologue is requested before the first barrier, and the barriers order LDS
        // traffic only, so the cache blocks above stay in flight: thread t < G*HD/2 rotates the element pair
        // (t mod HD/2, + HD/2) of query head t / (HD/2); threads 256.. do the same for the new key, threads 384.. copy
        // the new value.  256 is a multiple of HD/2, so a thread that has both duties uses one pair of rotary factors.
        static_assert(G * HD / 2 <= kBlock && (kWave * 4) % (HD / 2) == 0 && kWave * 6 + HD <= kBlock, "thread roles");
        const bool has_q = tid < G * HD / 2;
        const bool has_k = last && tid >= kWave * 4 && tid < kWave * 4 + HD / 2;
        const bool has_v = last && tid >= kWave * 6 && tid < kWave * 6 + HD;
        const int jj = tid % (HD / 2), gq = tid / (HD / 2);
        float qa = 0.f, qb = 0.f, ka = 0.f, kb = 0.f, vraw = 0.f, cs = 1.f, sn = 0.f;
        const unsigned tag_in = TAGGED ? step_tag(p, step, TS_QKV) : 0u;
        // two elements of this sequence's q/k/v vector (tagged: polled together until both are there)
        auto ld_in2 = [&](const float *sa, const float *sb, float &va, float &vb) {
            if (TAGGED) {
                ld_tagged2(p, p.qkvt + (sa - qkv), p.qkvt + (sb - qkv), tag_in, va, vb);
            } else {
                va = ld_f32<COH>(sa);
                vb = ld_f32<COH>(sb);
            }
        };
        // what does not depend on the projection's output comes first (biases, the rotary factors): when q/k/v arrive,
        // nothing else is waited for
        float bqa = 0.f, bqb = 0.f, bka = 0.f, bkb = 0.f, bv = 0.f;
        if (has_q && p.b_q) {
            bqa = bf16_to_f32(p.b_q[(h0 + gq) * HD + jj]);
            bqb = bf16_to_f32(p.b_q[(h0 + gq) * HD + jj + HD / 2]);
        }
        if (has_k && p.b_k) {
            bka = bf16_to_f32(p.b_k[kvh * HD + jj]);
            bkb = bf16_to_f32(p.b_k[kvh * HD + jj + HD / 2]);
        }
        if (has_v && p.b_v) bv = bf16_to_f32(p.b_v[kvh * HD + (tid - kWave * 6)]);
        if (has_q || has_k) rope_cos_sin(pnew, p.rope_inv[jj], cs, sn);
        if (has_q) {
            const float *src = qkv + (size_t)(h0 + gq) * HD;
            ld_in2(src + jj, src + jj + HD / 2, qa, qb);
            qa += bqa;
            qb += bqb;
        }
        if (has_k) {
            const float *src = qkv + p.qd + (size_t)kvh * HD;
            ld_in2(src + jj, src + jj + HD / 2, ka, kb);
            ka += bka;
            kb += bkb;
        }
        if (has_v) {
            const float *src = qkv + p.qd + p.kvd + (size_t)kvh * HD + (tid - kWave * 6);
            float dummy;
            ld_in2(src, src, vraw, dummy);
            vraw += bv;
        }
        lds_barrier(); // LDS of the previous item is free
        if (has_q) {
            s.q[gq][jj] = (qa * cs - qb * sn) * scale;
            s.q[gq][jj + HD / 2] = (qb * cs + qa * sn) * scale;
        }
        if (has_k) {
            const uint16_t r0 = f32_to_bf16(ka * cs - kb * sn), r1 = f32_to_bf16(kb * cs + ka * sn);
            s.knew[jj] = bf16_to_f32(r0);
            s.knew[jj + HD / 2] = bf16_to_f32(r1);
            if (!dead && part == 0) { // every part needs the new key and value, one of them appends
                uint16_t *kdst = p.k_cache + (((size_t)b * p.Hkv + kvh) * p.cap + pnew) * HD;
                st_u16<COH>(kdst + jj, r0);
                st_u16<COH>(kdst + jj + HD / 2, r1);
            }
        }
        if (has_v) {
            const int e = tid - kWave * 6;
            const uint16_t r = f32_to_bf16(vraw);
            s.vnew[e] = bf16_to_f32(r);
            if (!dead && part == 0) st_u16<COH>(p.v_cache + (((size_t)b * p.Hkv + kvh) * p.cap + pnew) * HD + e, r);
        }
        lds_barrier();

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

        // nl: blocks of this round that exist for the wave (uniform): the others are skipped, not masked
        auto absorb = [&](const float(&sc)[U][G], const float(&vv)[U][8], const bool(&okk)[U], int nl) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float mb = mx[g];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (u < nl && okk[u]) mb = fmaxf(mb, sc[u][g]);
                if (mb == -INFINITY) continue;
                float alpha = expf(mx[g] - mb); // 0 when nothing was absorbed before
                float sm = sum[g] * alpha;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[g][e] *= alpha;
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (u < nl && okk[u]) {
                        float pr = expf(sc[u][g] - mb);
                        sm += pr;
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[g][e] += pr * vv[u][e];
                    }
                mx[g] = mb;
                sum[g] = sm;
            }
        };

        for (int base = wave; base < nblk; base += kWaves * U) {
            if (base != wave) load_blocks(base);
            const int nl = __builtin_amdgcn_readfirstlane(min(U, (nblk - base + kWaves - 1) / kWaves));
            float sc[U][G], vv[U][8];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (u >= nl) { // no such block: nothing of it is used
#pragma unroll
                    for (int g = 0; g < G; ++g) sc[u][g] = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) vv[u][e] = 0.f;
                    continue;
                }
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
            absorb(sc, vv, ok, nl);
        }
        if (last && wave == 0) { // the token being appended, from LDS; every lane group computes it, group 0 keeps it
            float sc[U][G], vv[U][8];
            bool okn[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                okn[u] = (u == 0) && (tq == 0);
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
            absorb(sc, vv, okn, 1);
        }
        // merge the lane groups of the workgroup
        // (a single split publishes its result as tagged elements that other workgroups act on at once: the appended
        // cache entry, written by waves of this workgroup above, is acknowledged first; the barriers below order it
        // before every wave's result stores)
        if (TAGGED && nsplit == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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
        lds_barrier();
        // wave g forms the weights of head g's streams once (lane = stream): exp(max_stream - max), zero for a stream
        // that saw no token; they replace the stream maxima in LDS, and the head's maximum and weighted sum go where
        // the rotary table used to be
        static_assert(NSTREAM <= kWave && G <= kWaves && G <= HD / 2, "one wave per head, one lane per stream");
        if (wave < G) {
            const float mm = lane < NSTREAM ? s.ml[lane][wave][0] : -INFINITY;
            const float ll = lane < NSTREAM ? s.ml[lane][wave][1] : 0.f;
            float M = mm;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, kWave));
            const float w = mm != -INFINITY ? expf(mm - M) : 0.f;
            const float Ls = wave_sum(ll * w);
            if (lane < NSTREAM) s.ml[lane][wave][0] = w;
            if (lane == 0) {
                s.cs[wave] = M;
                s.sn[wave] = Ls;
            }
        }
        lds_barrier();
        for (int o = tid; o < G * HD; o += kBlock) {
            int g = o / HD, dd = o % HD;
            const float M = s.cs[g], Ls = s.sn[g];
            float A = 0.f;
#pragma unroll 8
            for (int st = 0; st < NSTREAM; ++st) A += s.acc[st][g][dd] * s.ml[st][g][0];
            int hq = h0 + g;
            if (nsplit == 1) {
                const float r = A / Ls;
                if (TAGGED)
                    st_tagged(p.attnt + (size_t)hq * HD + dd, r, step_tag(p, step, TS_ATTN));
                else
                    st_f32<COH>(p.attn + (size_t)b * p.qd + (size_t)hq * HD + dd, r);
                if (!TAGGED && p.attn_split) {
                    uint16_t h, l;
                    split_bf16(r, h, l);
                    const size_t at = (size_t)b * p.a_stride + (size_t)hq * HD + dd;
                    p.attn_split[at] = h;
                    p.attn_split[p.a_lo + at] = l;
                }
            } else {
                float *dst = p.attn_part + (((size_t)b * p.Hq + hq) * S + sp) * PW;
                st_f32<COH || TICKET>(dst + dd, A);
                if (dd == 0) {
                    st_f32<COH || TICKET>(dst + HD, M);
                    st_f32<COH || TICKET>(dst + HD + 1, Ls);
                }
            }
        }
        if (TICKET && nsplit > 1) {
            // The workgroup whose split of this (sequence, KV head) is the last to finish merges the splits, one
            // query head per wave.  The partials above were written through to memory and have been acknowledged
            // (the wait below) before this workgroup draws its ticket, and the merging workgroup reads them past its
            // caches, so relaxed atomics suffice.  The last workgroup also puts the counter back to zero.
            int &last_to_arrive = *reinterpret_cast<int *>(smem + sizeof(L)); // behind the struct, clear of the strips
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (tid == 0) {
                int *ticket = p.attn_ticket + ((size_t)b * p.Hkv + kvh) * GS + part; // (GS > 1: one sequence)
                const int old = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (old == nsplit - 1) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                last_to_arrive = (old == nsplit - 1) ? 1 : 0;
            }
            __syncthreads();
            const bool merges = last_to_arrive != 0;
            if (merges && wave < G)
                merge_head<HD, true, COH, TAGGED>(p, b, h0 + wave, nsplit,
                                                  reinterpret_cast<float *>(smem) + (size_t)wave * S, step);
        }
    }
    if (first_item) before_q();
}

// ---------------------------------------------------------------------------------------------------
// phase 4: output projection (its residual add happens in the consumers)      (step 7)
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ void phase_oproj(const DraftParams &p, int, int vb, int nvb, char *smem) {
    const int d = p.d, K = p.qd;
    const int nbmax = p.nb_q;
    GemvLds l = gemv_lds(smem, K, nbmax, 1);
    for (int b0 = 0; b0 < p.B; b0 += nbmax) {
        int nb = min(nbmax, p.B - b0);
        auto stage = [&]() {
            __syncthreads();
            for (int i = 0; i < nb; ++i)
                stage_plain(p.attn + (size_t)(b0 + i) * K, K, l.kpad, l.hi + (size_t)i * l.kpad,
                            l.lo + (size_t)i * l.kpad);
            __syncthreads();
        };
        auto rowptr = [&](int, int row) { return p.w_o + (size_t)row * K; };
        auto epi = [&](int i, int row, float(&s)[1]) { p.o[(size_t)(b0 + i) * d + row] = s[0]; };
        gemv_auto<1, true>(rowptr, K, d, vb, nvb, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, stage, epi);
    }
}

// ---------------------------------------------------------------------------------------------------
// phase 5: MLP-input RMSNorm + gate and up projections (SiLU(gate) * up is formed by the consumer)   (step 8)
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ void phase_gateup(const DraftParams &p, int, int vb, int nvb, char *smem) {
    const int d = p.d, F = p.F;
    const int nbmax = p.nb_d;
    GemvLds l = gemv_lds(smem, d, nbmax, 1);
    for (int b0 = 0; b0 < p.B; b0 += nbmax) {
        int nb = min(nbmax, p.B - b0);
        auto stage = [&]() {
            stage_sequences(nb, [&](int i, bool whole) {
                const float *src = p.x + (size_t)(b0 + i) * d, *res = p.o + (size_t)(b0 + i) * d; // x1 = x + w_o attn
                uint16_t *hi = l.hi + (size_t)i * l.kpad, *lo = l.lo + (size_t)i * l.kpad;
                if (whole)
                    stage_rmsnorm<false>(src, p.g_mlp, d, p.eps, hi, lo, l.red, nullptr, nullptr, res);
                else
                    stage_rmsnorm_wave<false>(src, p.g_mlp, d, p.eps, hi, lo, nullptr, nullptr, res);
            });
        };
        // the 2F rows of [w_gate; w_up] are dealt out as one list: the two halves of a SwiGLU pair need not meet
        // here (the consumer multiplies them), which keeps every wave within one row of the average load
        auto rowptr = [&](int, int row) { return row < F ? p.w_gate + (size_t)row * d : p.w_up + (size_t)(row - F) * d; };
        auto epi = [&](int i, int row, float(&s)[1]) { p.gu[(size_t)(b0 + i) * 2 * F + row] = s[0]; };
        gemv_auto<1, true>(rowptr, d, 2 * F, vb, nvb, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, stage, epi);
    }
}

// ---------------------------------------------------------------------------------------------------
// phase 6: SiLU(gate) * up, down projection (its residual add happens in the consumer)   (steps 8-9)
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ void phase_down(const DraftParams &p, int, int vb, int nvb, char *smem) {
    const int d = p.d, K = p.F;
    const int nbmax = p.nb_down;
    GemvLds l = gemv_lds(smem, K, nbmax, 1);
    for (int b0 = 0; b0 < p.B; b0 += nbmax) {
        int nb = min(nbmax, p.B - b0);
        auto stage = [&]() {
            __syncthreads();
            for (int i = 0; i < nb; ++i)
                stage_swiglu(p.gu + (size_t)(b0 + i) * 2 * K, K, l.kpad, l.hi + (size_t)i * l.kpad,
                             l.lo + (size_t)i * l.kpad); // m = silu(w_gate y2) * (w_up y2)
            __syncthreads();
        };
        auto rowptr = [&](int, int row) { return p.w_down + (size_t)row * K; };
        auto epi = [&](int i, int row, float(&s)[1]) { p.dn[(size_t)(b0 + i) * d + row] = s[0]; };
        gemv_auto<1, true>(rowptr, K, d, vb, nvb, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, stage, epi);
    }
}

// ---------------------------------------------------------------------------------------------------
// phase 7: final RMSNorm + compressed output head + argmax                       (steps 9-10; Eq. (3))
// ---------------------------------------------------------------------------------------------------
// Row i of the compressed head is lm_head[ids[i]]; rows are dealt out in subset order, so every workgroup scans a
// contiguous, ascending range of subset indices (row mode: rows interleaved over the waves).  Each reporting thread
// keeps the best (logit, index) it has seen as a 64-bit key that orders by logit, then by lower index; the workgroup's
// best per sequence is stored as one candidate, and whoever needs the winner takes the maximum over the candidates.
__device__ __forceinline__ void phase_lmhead(const DraftParams &p, int step, int vb, int nvb, char *smem) {
    const int d = p.d, n = p.n;
    const int nbmax = p.nb_d;
    GemvLds l = gemv_lds(smem, d, nbmax, 1);
    for (int b0 = p.seq_lo; b0 < p.seq_hi; b0 += nbmax) { // the sequences that share this launch's id list
        int nb = min(nbmax, p.seq_hi - b0);
        auto stage = [&]() {
            stage_sequences(nb, [&](int i, bool whole) {
                const int b = b0 + i;
                // workgroup 0 also publishes the step's output hidden state: for the next step and for the caller
                float *hh = (vb == 0) ? p.hhat + (size_t)b * d : nullptr;
                float *ho = (vb == 0 && p.hidden_out) ? p.hidden_out + ((size_t)b * p.K + step) * d : nullptr;
                uint16_t *hi = l.hi + (size_t)i * l.kpad, *lo = l.lo + (size_t)i * l.kpad;
                // x2 = (x + w_o attn) + w_down m
                if (whole)
                    stage_rmsnorm<false>(p.x + (size_t)b * d, p.g_final, d, p.eps, hi, lo, l.red, hh, ho,
                                         p.o + (size_t)b * d, p.dn + (size_t)b * d);
                else
                    stage_rmsnorm_wave<false>(p.x + (size_t)b * d, p.g_final, d, p.eps, hi, lo, hh, ho,
                                              p.o + (size_t)b * d, p.dn + (size_t)b * d);
            });
        };
        // best (logit, index) seen by this thread: in row mode lane 0 of a wave reports every sequence, in tile
        // mode a thread reports one sequence only
        const bool rowmode = use_row_mode(nb, d);
        unsigned long long best[kRowModeMaxSeq];
#pragma unroll
        for (int i = 0; i < kRowModeMaxSeq; ++i) best[i] = 0ull;
        auto rowptr = [&](int, int row) {
            int r = p.ids ? p.ids[row] : row;
            return p.lm_head + (size_t)r * d;
        };
        auto epi = [&](int i, int row, float(&s)[1]) {
            if (p.logits_out) p.logits_out[((size_t)(b0 + i) * p.K + step) * p.logit_stride + row] = s[0];
            unsigned long long key = argmax_key(s[0], (uint32_t)row);
#pragma unroll
            for (int q = 0; q < kRowModeMaxSeq; ++q)
                if (q == (rowmode ? i : 0)) best[q] = key > best[q] ? key : best[q];
        };
        gemv_auto<1, false>(rowptr, d, n, vb, nvb, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, stage, epi);
        unsigned long long *red64 = reinterpret_cast<unsigned long long *>(l.partial); // free again after the barrier
        __syncthreads();
        if (rowmode) {
            if ((threadIdx.x & (kWave - 1)) == 0) {
#pragma unroll
                for (int i = 0; i < kRowModeMaxSeq; ++i) red64[(threadIdx.x / kWave) * kRowModeMaxSeq + i] = best[i];
            }
            __syncthreads();
            if ((int)threadIdx.x < nb) {
                unsigned long long m = 0ull;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    unsigned long long c = red64[w * kRowModeMaxSeq + threadIdx.x];
                    m = c > m ? c : m;
                }
                p.cand[((size_t)step * p.max_batch + b0 + threadIdx.x) * p.head_grid + vb] = m;
            }
        } else if ((int)threadIdx.x < 16 * nb) { // threads 16*i .. 16*i+15 hold candidates of sequence i
            unsigned long long m = best[0];
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) {
                unsigned long long o = __shfl_xor(m, off, kWave);
                m = o > m ? o : m;
            }
            if ((threadIdx.x & 15) == 0)
                p.cand[((size_t)step * p.max_batch + b0 + (threadIdx.x >> 4)) * p.head_grid + vb] = m;
        }
    }
}

// after the last step: publish the last draft id; one wave per sequence takes the maximum over the candidates
__device__ void phase_finalize(const DraftParams &p, int vb, int nvb) {
    const int lane = threadIdx.x & (kWave - 1);
    for (int b = vb * kWaves + threadIdx.x / kWave; b < p.B; b += nvb * kWaves) {
        const unsigned long long *cand = p.cand + ((size_t)(p.K - 1) * p.max_batch + b) * p.head_grid;
        unsigned long long best = 0ull;
        const int ncand = seq_head(p, b).cands;
        for (int w = lane; w < ncand; w += kWave) best = cand[w] > best ? cand[w] : best;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            unsigned long long o = __shfl_xor(best, off, kWave);
            best = o > best ? o : best;
        }
        if (lane == 0) p.draft_out[(size_t)b * p.K + p.K - 1] = seq_dead(p, b) ? -1 : key_token(p, b, best);
    }
}

// The attention phase as the single-launch kernel runs it.  Inlined: as a function of its own it saved and restored
// about a hundred registers per lane through scratch memory at every call (47 MB written and read back per draft step
// over the chip, for workgroups without an attention item too), which was most of the phase's 15 us.
template <int G, int HD, bool COH = false, bool TICKET = false, bool TAGGED = false, int GS = 1>
__device__ __forceinline__ void call_attn(const DraftParams &p, int step, int vb, int nvb, char *smem) {
    phase_attn<G, HD, COH, TICKET, NoHook, TAGGED, GS>(p, step, vb, nvb, smem);
}

} // namespace mtp
