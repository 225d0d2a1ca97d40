// C ABI of the FastMTP draft library for MI355X (gfx950): host-side validation, launch plan and kernel wrappers.
// See include/mtp_draft.h for the contract of every entry point.
#include "../../include/mtp_draft.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "phases.h"
#include "flow.h"
#include "batch_launch.h"

using namespace mtp;

namespace {

enum Phase : int { PH_PROJ = 0, PH_QKV, PH_ATTN, PH_OPROJ, PH_GATEUP, PH_DOWN, PH_LMHEAD, PH_COUNT };

// ---- kernels: one launch per phase ------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_proj(DraftParams p, int step) {
    extern __shared__ __align__(16) char smem[];
    phase_proj(p, step, blockIdx.x, gridDim.x, smem);
}
__global__ __launch_bounds__(kBlock) void k_qkv(DraftParams p, int step) {
    extern __shared__ __align__(16) char smem[];
    phase_qkv(p, step, blockIdx.x, gridDim.x, smem);
}
template <int G, int HD>
__global__ __launch_bounds__(kBlock) void k_attn(DraftParams p, int step) {
    extern __shared__ __align__(16) char smem[];
    phase_attn<G, HD, false, true>(p, step, blockIdx.x, gridDim.x, smem); // merges its own splits (tickets)
}
__global__ __launch_bounds__(kBlock) void k_oproj(DraftParams p, int step) {
    extern __shared__ __align__(16) char smem[];
    phase_oproj(p, step, blockIdx.x, gridDim.x, smem);
}
__global__ __launch_bounds__(kBlock) void k_gateup(DraftParams p, int step) {
    extern __shared__ __align__(16) char smem[];
    phase_gateup(p, step, blockIdx.x, gridDim.x, smem);
}
__global__ __launch_bounds__(kBlock) void k_down(DraftParams p, int step) {
    extern __shared__ __align__(16) char smem[];
    phase_down(p, step, blockIdx.x, gridDim.x, smem);
}
__global__ __launch_bounds__(kBlock) void k_lmhead(DraftParams p, int step) {
    extern __shared__ __align__(16) char smem[];
    phase_lmhead(p, step, blockIdx.x, gridDim.x, smem);
}
__global__ void k_finalize(DraftParams p) { phase_finalize(p, blockIdx.x, gridDim.x); }
template <int G, int HD>
__global__ __launch_bounds__(kBlock) void k_flow(DraftParams) {
    extern __shared__ __align__(16) char smem[];
    // the attention phase is called out of line and takes the parameters by reference: point it at the
    // kernel-argument segment (the struct is the only argument, at offset 0) instead of a per-lane stack copy
    const DraftParams *p = (const DraftParams *)__builtin_amdgcn_kernarg_segment_ptr();
    flow_steps<G, HD>(*p, smem);
}

// Sequential acceptance up to the first mismatch and the draft-cache length after it (Sec. 2.3 "Verification phase").
__global__ void k_accept(int B, int K, const int *draft, const int *target, int mode, int *kv_len, int *accept_len,
                         int *out_tokens, int *pending) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int *dr = draft + (size_t)b * K;
    const int *tg = target + (size_t)b * (K + 1);
    int a = 0;
    while (a < K && dr[a] == tg[a]) ++a;
    int *out = out_tokens + (size_t)b * (K + 1);
    for (int j = 0; j <= K; ++j) out[j] = j < a ? dr[j] : (j == a ? tg[a] : -1);
    accept_len[b] = a;
    if (mode == 0) {
        kv_len[b] += min(a + 1, K);
        pending[b] = (a == K) ? 1 : 0;
    } else {
        pending[b] = 0;
    }
}

// Several new positions per sequence: the cache length each (position, sequence) row starts from.  A sequence whose
// block does not fit (or whose length is invalid) gets -1 in every row, which the first phase reports; rows beyond
// a sequence's new positions are marked inactive.
__global__ void k_extend_prep(int B, int m_max, int cap, const int *kv_len, const int *ext_len, int *row_len) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= B * m_max) return;
    const int b = r % B, j = r / B;
    const int L = kv_len[b], m = ext_len[b];
    const bool bad = L < 0 || m < 0 || m > m_max || L + m > cap;
    row_len[r] = bad ? -1 : (j < m ? L + j : kRowInactive);
}
// A block of new positions: bias, rotary embedding and the bf16 cache append of EVERY row's key and value (the work the
// attention's last split does for the one new position of an ordinary step), so that one attention launch can serve
// all positions.  grid (rows, KV heads), HD/2 + HD threads: pairs of the key, then the elements of the value.
template <int HD>
__global__ void k_extend_append(DraftParams p) {
    const int r = blockIdx.x, kvh = blockIdx.y, tid = threadIdx.x;
    const int pos = p.kv_len[r]; // the row's own slot; negative: the row is not part of the block
    if (pos < 0 || pos >= p.cap) return;
    const int seq = r % p.ext_B;
    const float *qkv = p.qkv + (size_t)r * p.qkv_dim;
    const size_t slot = (((size_t)seq * p.Hkv + kvh) * p.cap + pos) * HD;
    if (tid < HD / 2) {
        const int e = tid;
        const float *src = qkv + p.qd + (size_t)kvh * HD;
        float a = src[e], bb = src[e + HD / 2], cs, sn;
        if (p.b_k) {
            a += bf16_to_f32(p.b_k[kvh * HD + e]);
            bb += bf16_to_f32(p.b_k[kvh * HD + e + HD / 2]);
        }
        rope_cos_sin(pos, p.rope_inv[e], cs, sn);
        p.k_cache[slot + e] = f32_to_bf16(a * cs - bb * sn);
        p.k_cache[slot + e + HD / 2] = f32_to_bf16(bb * cs + a * sn);
    } else if (tid < HD / 2 + HD) {
        const int e = tid - HD / 2;
        float v = qkv[p.qd + p.kvd + (size_t)kvh * HD + e];
        if (p.b_v) v += bf16_to_f32(p.b_v[kvh * HD + e]);
        p.v_cache[slot + e] = f32_to_bf16(v);
    }
}

__global__ void k_extend_finish(int B, int m_max, int cap, int *kv_len, const int *ext_len) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int L = kv_len[b], m = ext_len[b];
    if (L >= 0 && m >= 0 && m <= m_max && L + m <= cap) kv_len[b] = L + m;
}

// One id list per group of adjacent sequences: the tables the kernels look a sequence's list up in.
constexpr int kMaxListGroups = 16;
struct ListGroups {
    int count;
    int lo[kMaxListGroups], hi[kMaxListGroups]; // sequences [lo, hi)
    const int *ids[kMaxListGroups];             // null = the full vocabulary
    int n[kMaxListGroups], cands[kMaxListGroups];
};
__global__ void k_set_lists(ListGroups g, int *seq_list, const int **list_ids, int *list_n, int *list_cands) {
    for (int s = 0; s < g.count; ++s) {
        for (int b = g.lo[s] + threadIdx.x; b < g.hi[s]; b += blockDim.x) seq_list[b] = s;
        if (threadIdx.x == 0) {
            list_ids[s] = g.ids[s];
            list_n[s] = g.n[s];
            list_cands[s] = g.cands[s];
        }
    }
}

// ---- teacher-forced forward: cross-entropy of one step's logits (Eq. (1)) -------------------------------------------
__global__ void k_train_begin_step(int n_pos, int *kv_len, int *ext_len) { // a fresh cache and n_pos new positions
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        kv_len[0] = 0;
        ext_len[0] = n_pos;
    }
}
// one workgroup per position: logsumexp(z) - z[label] over the full vocabulary
__global__ __launch_bounds__(256) void k_train_row_ce(const float *__restrict__ logits, int V, const int *labels,
                                                      float *row_loss, int *err) {
    __shared__ float red_m[256 / kWave], red_s[256 / kWave];
    const float *z = logits + (size_t)blockIdx.x * V;
    // one pass: every thread keeps a running maximum and the sum of exp(z - maximum) of its elements (16-byte loads
    // where the row allows them), the pairs are combined at the end
    float m = -INFINITY, sum = 0.f;
    auto take = [&](float a, float b, float c, float d) {
        const float mm = fmaxf(fmaxf(a, b), fmaxf(c, d));
        if (mm > m) {
            sum *= expf(m - mm); // exp(-inf) = 0 the first time
            m = mm;
        }
        sum += (expf(a - m) + expf(b - m)) + (expf(c - m) + expf(d - m));
    };
    const int head = (int)((4 - (((size_t)blockIdx.x * V) & 3)) & 3); // elements before the first aligned one
    const int nvec = V > head ? (V - head) / 4 : 0;
    const f32x4 *z4 = reinterpret_cast<const f32x4 *>(z + head);
    int i = threadIdx.x;
    for (; i + 3 * 256 < nvec; i += 4 * 256) { // four loads in flight per thread
        const f32x4 v0 = z4[i], v1 = z4[i + 256], v2 = z4[i + 512], v3 = z4[i + 768];
        take(v0.x, v0.y, v0.z, v0.w);
        take(v1.x, v1.y, v1.z, v1.w);
        take(v2.x, v2.y, v2.z, v2.w);
        take(v3.x, v3.y, v3.z, v3.w);
    }
    for (; i < nvec; i += 256) {
        const f32x4 v = z4[i];
        take(v.x, v.y, v.z, v.w);
    }
    for (int e = threadIdx.x; e < V; e += 256) // the few elements outside the aligned middle
        if (e < head || e >= head + nvec * 4) take(z[e], -INFINITY, -INFINITY, -INFINITY);
    float wm = m;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) wm = fmaxf(wm, __shfl_xor(wm, off, kWave));
    sum = wave_sum(wm == -INFINITY ? 0.f : sum * expf(m - wm));
    if ((threadIdx.x & (kWave - 1)) == 0) {
        red_m[threadIdx.x / kWave] = wm;
        red_s[threadIdx.x / kWave] = sum;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int label = labels[blockIdx.x];
        if (label < 0 || label >= V) { // reported like an input token out of range; scored as id 0
            atomicOr(err, kErrTokenRange);
            label = 0;
        }
        const float M = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));
        float tot = 0.f;
#pragma unroll
        for (int w = 0; w < 256 / kWave; ++w) tot += red_m[w] == -INFINITY ? 0.f : red_s[w] * expf(red_m[w] - M);
        row_loss[blockIdx.x] = M + logf(tot) - z[label];
    }
}
// mean over the positions in a fixed order (one workgroup), and after the last step the weighted total of Eq. (1)
__global__ __launch_bounds__(256) void k_train_step_mean(const float *row_loss, int n_pos, float *loss_out, int k, int K,
                                                         float beta) {
    __shared__ float red[256 / kWave];
    float s = 0.f;
    for (int i = threadIdx.x; i < n_pos; i += 256) s += row_loss[i];
    s = wave_sum(s);
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = s;
    __syncthreads();
    if (threadIdx.x != 0) return;
    loss_out[k] = ((red[0] + red[1]) + (red[2] + red[3])) / (float)n_pos;
    if (k == K - 1) { // Eq. (2): alpha_j = beta^(j-1) / sum_i beta^(i-1)
        float wsum = 0.f, acc = 0.f, w = 1.f;
        for (int j = 0; j < K; ++j) {
            acc += w * loss_out[j];
            wsum += w;
            w *= beta;
        }
        loss_out[K] = acc / wsum;
    }
}

// Streaming-read probe: the access pattern of the weight stream (every wave requests 1 KiB per load, sixteen loads in
// flight, non-temporal) over a plain buffer, nothing else.  What it reaches is the ceiling the draft kernels are measured
// against.  Blocks of 16 KiB are dealt round robin to the waves of the grid; the XOR of everything read goes to out[0]
// so that the loads are kept.
__global__ __launch_bounds__(kBlock) void k_stream_probe(const u32x4 *__restrict__ src, long long blocks,
                                                         unsigned long long *out) {
    const int lane = threadIdx.x & (kWave - 1);
    const long long wave = (long long)blockIdx.x * kWaves + threadIdx.x / kWave, nwaves = (long long)gridDim.x * kWaves;
    uint32_t acc = 0;
    for (long long b = wave; b < blocks; b += nwaves) {
        u32x4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = __builtin_nontemporal_load(src + (b * 16 + u) * kWave + lane);
#pragma unroll
        for (int u = 0; u < 16; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) acc ^= __shfl_xor(acc, off, kWave);
    if (lane == 0 && acc == 0x9e3779b9u) out[0] = acc; // (practically never true: the store exists to keep the loads)
}

// a fill kernel instead of a memset node: calls that a caller may capture into a HIP graph record no hipMemsetAsync
__global__ void k_zero_words(unsigned long long *dst, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = 0ull;
}

typedef void (*phase_kernel_t)(DraftParams, int);

phase_kernel_t attn_kernel(int G, int HD) {
    if (HD == 128) {
        switch (G) {
        case 1: return k_attn<1, 128>;
        case 2: return k_attn<2, 128>;
        case 4: return k_attn<4, 128>;
        case 8: return k_attn<8, 128>;
        }
    } else if (HD == 64) {
        switch (G) {
        case 1: return k_attn<1, 64>;
        case 2: return k_attn<2, 64>;
        case 4: return k_attn<4, 64>;
        case 8: return k_attn<8, 64>;
        }
    }
    return nullptr;
}
typedef void (*fused_kernel_t)(DraftParams);
fused_kernel_t flow_kernel(int G, int HD) {
    if (HD == 128) {
        switch (G) {
        case 1: return k_flow<1, 128>;
        case 2: return k_flow<2, 128>;
        case 4: return k_flow<4, 128>;
        case 8: return k_flow<8, 128>;
        }
    } else if (HD == 64) {
        switch (G) {
        case 1: return k_flow<1, 64>;
        case 2: return k_flow<2, 64>;
        case 4: return k_flow<4, 64>;
        case 8: return k_flow<8, 64>;
        }
    }
    return nullptr;
}
// the matrix-core attention's item map: lengths and two orders of the sequences, full splits below each split index
size_t attn_map_bytes(int B, int max_splits) { return ((size_t)3 * B + max_splits + 2) * 4; }
size_t attn_lds_bytes(int G, int HD) {
    int tpi = kWave / (HD / 8), ns = kWaves * tpi;
    size_t fl = (size_t)G * HD + HD + 2 * HD + (size_t)ns * G * HD + (size_t)ns * G * 2;
    return fl * sizeof(float) + 64;
}

// ---- plan: how a call of B sequences is cut up ----------------------------------------------------------
constexpr int kTargetAttnItems = 256; // (sequence, KV head, split) items aimed for
constexpr int kMinSplitTokens = 128;
constexpr int kMaxSplitTokens = 4096;
constexpr int kMfmaAttnMinSplit = 256; // splits of at least this many tokens use the matrix-core attention
constexpr size_t kLdsSmallBatch = 72 * 1024;  // two workgroups per CU
constexpr size_t kLdsLargeBatch = 150 * 1024; // one workgroup per CU, more sequences per weight pass

int split_tokens_for(const mtp_config &c, int B) {
    long long t = ((long long)c.kv_capacity * B * c.n_kv_heads + kTargetAttnItems - 1) / kTargetAttnItems;
    t = std::max<long long>(t, kMinSplitTokens);
    t = (t + 63) / 64 * 64;
    // past this length a split costs more in waiting for the longest context than another item costs in set-up; the
    // launch then has more items than workgroups and hands them out one by one
    t = std::min<long long>(t, kMaxSplitTokens);
    return (int)t;
}
int max_splits_for(const mtp_config &c, int B) {
    int t = split_tokens_for(c, B);
    return (c.kv_capacity + t - 1) / t;
}
size_t attn_part_floats(const mtp_config &c) {
    size_t best = 0;
    for (int B = 1; B <= c.max_batch; ++B)
        best = std::max(best, (size_t)B * max_splits_for(c, B));
    return best * c.n_q_heads * (c.head_dim + 2);
}

bool config_ok(const mtp_config *c) {
    if (!c) return false;
    if (c->d_model < 256 || c->d_model > 8192 || c->d_model % 32) return false;
    if (c->head_dim != 64 && c->head_dim != 128) return false;
    if (c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads) return false;
    int G = c->n_q_heads / c->n_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8) return false;
    if (c->d_ffn < 256 || c->d_ffn % 8) return false;
    if (c->n_q_heads * c->head_dim < 256) return false; // every reduction length holds at least one 256-element chunk
    if (c->vocab_size < 1) return false;
    if (c->max_batch < 1 || c->max_batch > kBlock) return false;
    if (c->max_draft_steps < 1 || c->kv_capacity < c->max_draft_steps) return false;
    if (c->kv_capacity > 2048 * kMinSplitTokens) return false; // the merge keeps one weight per split per wave in LDS
    if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return false;
    if ((long long)c->n_q_heads * c->head_dim > 65536) return false;
    return true;
}

constexpr size_t kAlign = 256;
constexpr int kMaxFusedGrid = 1024; // workgroups of the single-launch kernel (one per CU)
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct WsLayout {
    size_t x, qkv, attn, o, gu, dn, hhat, err, cand, rope_inv, attn_part, total;
    size_t xt, qkvt, attnt, ot, gut, dnt, candt, tagged_end; // tagged hand-over vectors of the barrier-free kernel
    // batched path (max_batch above kBatchMinSeq - 1 only)
    size_t act0, act1, ssq, part, ticket, a_lo, attn_ticket, row_len, seq_list, list_ids, list_n, list_cands;
    int a_stride;
};

// the batched path serves calls with this many sequences or more; fewer take the row-streaming kernels
constexpr int kBatchMinSeq = 2;
constexpr int kMaxRowSeq = 4;          // sequences the row-streaming kernels serve at once
constexpr int kBatchPassSeq = 64;     // sequences per weight pass of the batched path
constexpr int kBatchGroupTiles = 8;   // weight tiles per wave and group
constexpr size_t kBatchTileBytes = 1024; // one 16 x 16 float tile of partial sums

// virtual 16-row tiles of the widest batched phase (gate/up pairs count twice)
size_t batch_max_tiles(const mtp_config &c) {
    size_t qkv = ((size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim + 15) / 16;
    return std::max({(size_t)(c.vocab_size + 15) / 16, 2 * (((size_t)c.d_ffn + 15) / 16), qkv,
                     ((size_t)c.d_model + 15) / 16});
}
WsLayout ws_layout(const mtp_config &c) {
    WsLayout l{};
    size_t mb = c.max_batch, d = c.d_model, qd = (size_t)c.n_q_heads * c.head_dim,
           kvd = (size_t)c.n_kv_heads * c.head_dim;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes);
        return o;
    };
    l.x = take(mb * d * 4);
    l.qkv = take(mb * (qd + 2 * kvd) * 4);
    l.attn = take(mb * qd * 4);
    l.o = take(mb * d * 4);
    l.gu = take(mb * (size_t)c.d_ffn * 2 * 4);
    l.dn = take(mb * d * 4);
    l.hhat = take(mb * d * 4);
    l.err = take(4);
    l.cand = take((size_t)c.max_draft_steps * mb * kMaxFusedGrid * 8);
    l.rope_inv = take((size_t)c.head_dim / 2 * 8);
    l.attn_part = take(attn_part_floats(c) * 4);
    // two per (sequence, KV head): the single-launch kernel deals a KV head's query heads to two items
    l.attn_ticket = take(mb * (size_t)c.n_kv_heads * 4 * 2 + 64); // + the attention launch's item counter
    l.row_len = take(mb * 4);
    l.seq_list = take(mb * 4);
    l.list_ids = take(kMaxListGroups * 8);
    l.list_n = take(kMaxListGroups * 4);
    l.list_cands = take(kMaxListGroups * 4);
    l.xt = take(d * 8);
    l.qkvt = take((qd + 2 * kvd) * 8);
    l.attnt = take(qd * 8);
    l.ot = take(d * 8);
    l.gut = take((size_t)c.d_ffn * 2 * 8);
    l.dnt = take(d * 8);
    l.candt = take((size_t)c.max_draft_steps * kMaxFusedGrid * 16);
    l.tagged_end = off;
    if (c.max_batch >= kBatchMinSeq) {
        size_t kmax = std::max({2 * d, qd, (size_t)c.d_ffn});
        l.a_stride = (int)((kmax + 31) / 32 * 32);
        l.a_lo = mb * (size_t)l.a_stride;
        l.act0 = take(2 * l.a_lo * 2);
        l.act1 = take(2 * l.a_lo * 2);
        l.ssq = take((size_t)3 * mb * (d / 16) * 4);
        // [reduction parts][tiles][sequence tiles]: split phases hold parts x tiles x sequence tiles <= 64 per
        // workgroup (of at most kMaxFusedGrid), unsplit ones every tile once
        size_t tiles = std::max(batch_max_tiles(c), (size_t)2 * kBatchGroupTiles * kMaxFusedGrid);
        l.part = take(tiles * (kBatchPassSeq / 16) * kBatchTileBytes);
        l.ticket = take((size_t)kMaxFusedGrid * 4);
    }
    l.total = off;
    return l;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

} // namespace

struct mtp_handle {
    mtp_config cfg;
    mtp_weights w;
    std::vector<const int *> subset_dev;
    std::vector<int> subset_n;
    char *ws;
    WsLayout lay;
    int num_cus;
    size_t lds_limit;
    phase_kernel_t attn_fn;
    fused_kernel_t flow_fn;        // one sequence: all phases of all steps in one launch
    unsigned long long flow_tags;  // hand-over tags given to earlier calls of that kernel
    size_t flow_lds_ok;            // largest LDS size for which a workgroup of that kernel was seen to fit a CU
    int mode;                    // 0: one launch per phase, 1: single launch for the whole call
    long long *trace;             // optional device buffer for phase time stamps
    int timing;         // 0 off, 1 whole call, 2 + phase: every launch of one phase
    hipEvent_t ev[2];   // whole call
    std::vector<hipEvent_t> pev; // per-step pairs for one phase
    int pev_used;
    bool ev_recorded;
};

extern "C" {

const char *mtp_status_string(int32_t s) {
    switch (s) {
    case MTP_OK: return "ok";
    case MTP_ERR_NULL: return "required pointer is NULL";
    case MTP_ERR_ALIGN: return "device pointer is not 16-byte aligned";
    case MTP_ERR_CONFIG: return "unsupported or inconsistent configuration";
    case MTP_ERR_BATCH: return "batch size outside [1, max_batch]";
    case MTP_ERR_STEPS: return "draft steps outside [1, max_draft_steps]";
    case MTP_ERR_SUBSET: return "invalid subset index or id list";
    case MTP_ERR_WORKSPACE: return "workspace too small";
    case MTP_ERR_HIP: return "HIP runtime call failed";
    case MTP_ERR_KV_OVERFLOW: return "kv_len + K exceeds kv_capacity for some sequence";
    case MTP_ERR_TOKEN_RANGE: return "token id outside the vocabulary";
    case MTP_ERR_MODE: return "unknown mode";
    case MTP_ERR_TIMEOUT: return "a workgroup waited too long at a grid barrier; results of that call are invalid";
    default: return "unknown status";
    }
}

size_t mtp_workspace_bytes(const mtp_config *cfg) {
    if (!config_ok(cfg)) return 0;
    return ws_layout(*cfg).total;
}

int32_t mtp_draft_init(mtp_handle **out, const mtp_config *cfg, const mtp_weights *w, int32_t n_subsets,
                       const int32_t *const *subset_ids, const int32_t *subset_sizes, void *workspace,
                       size_t workspace_bytes) {
    if (!out || !cfg || !w || !workspace) return MTP_ERR_NULL;
    *out = nullptr;
    if (!config_ok(cfg)) return MTP_ERR_CONFIG;
    const void *req[] = {w->embed, w->lm_head, w->g_hnorm, w->g_enorm, w->g_attn_norm, w->g_mlp_norm,
                         w->g_final_norm, w->w_proj, w->w_q, w->w_k, w->w_v, w->w_o, w->w_gate, w->w_up, w->w_down};
    for (const void *p : req)
        if (!p) return MTP_ERR_NULL;
    const void *all[] = {w->embed, w->lm_head, w->g_hnorm, w->g_enorm, w->g_attn_norm, w->g_mlp_norm,
                         w->g_final_norm, w->w_proj, w->w_q, w->w_k, w->w_v, w->b_q, w->b_k, w->b_v, w->w_o,
                         w->w_gate, w->w_up, w->w_down, workspace};
    for (const void *p : all)
        if (!aligned16(p)) return MTP_ERR_ALIGN;
    if (n_subsets < 0) return MTP_ERR_SUBSET;
    if (n_subsets > 0 && (!subset_ids || !subset_sizes)) return MTP_ERR_NULL;
    WsLayout lay = ws_layout(*cfg);
    if (workspace_bytes < lay.total) return MTP_ERR_WORKSPACE;

    // id lists: strictly ascending, inside the vocabulary
    std::vector<int32_t> host;
    for (int s = 0; s < n_subsets; ++s) {
        if (!subset_ids[s]) return MTP_ERR_NULL;
        if (!aligned16(subset_ids[s])) return MTP_ERR_ALIGN;
        int n = subset_sizes[s];
        if (n < 1 || n > cfg->vocab_size) return MTP_ERR_SUBSET;
        host.resize(n);
        hipError_t e = hipMemcpy(host.data(), subset_ids[s], (size_t)n * 4, hipMemcpyDeviceToHost);
        if (e != hipSuccess) {
            fprintf(stderr, "mtp_draft_init: reading subset %d failed: %s\n", s, hipGetErrorString(e));
            (void)hipGetLastError();
            return MTP_ERR_HIP;
        }
        if (host[0] < 0 || host[n - 1] >= cfg->vocab_size) return MTP_ERR_SUBSET;
        for (int i = 1; i < n; ++i)
            if (host[i] <= host[i - 1]) return MTP_ERR_SUBSET;
    }

    mtp_handle *h = new (std::nothrow) mtp_handle();
    if (!h) return MTP_ERR_HIP;
    h->cfg = *cfg;
    h->w = *w;
    for (int s = 0; s < n_subsets; ++s) {
        h->subset_dev.push_back(subset_ids[s]);
        h->subset_n.push_back(subset_sizes[s]);
    }
    h->ws = static_cast<char *>(workspace);
    h->lay = lay;
    h->timing = 0;
    h->ev_recorded = false;
    h->pev_used = 0;
    int dev = 0, cus = 0, lds = 0;
    bool ok = true;
    // the first HIP call that fails is named on stderr; the calls after it are skipped
    auto run = [&](hipError_t e, const char *what) {
        if (ok && e != hipSuccess) {
            fprintf(stderr, "mtp_draft_init: %s failed: %s\n", what, hipGetErrorString(e));
            ok = false;
        }
    };
    run(hipGetDevice(&dev), "hipGetDevice");
    if (ok) run(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev), "CU count query");
    if (ok) run(hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev), "LDS size query");
    if (ok) run(hipEventCreate(&h->ev[0]), "hipEventCreate");
    if (ok) run(hipEventCreate(&h->ev[1]), "hipEventCreate");
    if (ok) {
        h->pev.resize(2 * (size_t)cfg->max_draft_steps);
        for (auto &e : h->pev)
            if (ok) run(hipEventCreate(&e), "hipEventCreate");
    }
    h->num_cus = cus;
    h->lds_limit = (size_t)lds;
    h->attn_fn = attn_kernel(cfg->n_q_heads / cfg->n_kv_heads, cfg->head_dim);
    h->flow_fn = flow_kernel(cfg->n_q_heads / cfg->n_kv_heads, cfg->head_dim);
    h->flow_tags = 0;
    h->flow_lds_ok = 0;
    h->mode = 2;
    h->trace = nullptr;
    if (ok && (h->attn_fn == nullptr || h->flow_fn == nullptr)) {
        fprintf(stderr, "mtp_draft_init: no kernel for this head geometry\n");
        ok = false;
    }
    // allow the large-LDS launches
    const struct {
        const void *fn;
        const char *name;
    } fns[] = {{(const void *)k_proj, "k_proj"},         {(const void *)k_qkv, "k_qkv"},
               {(const void *)k_oproj, "k_oproj"},       {(const void *)k_gateup, "k_gateup"},
               {(const void *)k_down, "k_down"},         {(const void *)k_lmhead, "k_lmhead"},
               {(const void *)h->attn_fn, "k_attn"},
               {(const void *)h->flow_fn, "k_flow"}};
    for (const auto &f : fns)
        if (ok) run(hipFuncSetAttribute(f.fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)h->lds_limit), f.name);
    if (ok && !batch_allow_lds(h->lds_limit)) {
        fprintf(stderr, "mtp_draft_init: raising the LDS limit of the batched and matrix-core attention kernels failed\n");
        ok = false;
    }
    if (ok) run(hipMemset(workspace, 0, lay.total), "workspace clear");
    if (ok) {
        std::vector<double> inv((size_t)cfg->head_dim / 2);
        for (size_t j = 0; j < inv.size(); ++j)
            inv[j] = std::pow((double)cfg->rope_theta, -2.0 * (double)j / (double)cfg->head_dim);
        run(hipMemcpy(static_cast<char *>(workspace) + lay.rope_inv, inv.data(), inv.size() * 8, hipMemcpyHostToDevice),
            "rope table upload");
    }
    if (ok) run(hipDeviceSynchronize(), "hipDeviceSynchronize");
    if (!ok) {
        (void)hipGetLastError();
        delete h;
        return MTP_ERR_HIP;
    }
    *out = h;
    return MTP_OK;
}

} // extern "C"

namespace {
// The first draft step over a block of new positions (mtp_draft_extend) reuses the one-step pipeline with one row per
// (position, sequence); only the attention needs to know: it runs once per position over the real sequences.
struct ExtendCall {
    int B, m_max;           // real sequences, positions per sequence (rows = m_max * B)
    const int32_t *ext_len; // device [B]
    int32_t *kv_len;        // device [B], the real lengths (advanced at the end)
    bool logits_only = false; // the caller wants logits and no drafts (the training loss): many rows take the
                              // tiled matrix product for the output head
};

// B sequences (or rows), K steps; arguments checked by the callers
int32_t run_draft(mtp_handle *h, int32_t B, int32_t K, int32_t subset_index, const void *hidden_in,
                  const int32_t *token_in, void *k_cache, void *v_cache, const int32_t *kv_len,
                  const int32_t *forced_tokens, int32_t *draft_out, float *logits_out, float *hidden_out,
                  void *hip_stream, const ExtendCall *ext, const float *own_hidden = nullptr,
                  const int32_t *seq_subset = nullptr) {
    const mtp_config &c = h->cfg;
    // one id list per group of adjacent sequences (host array seq_subset [B]); subset_index is then ignored
    ListGroups groups{};
    int group_subset[kMaxListGroups];
    if (seq_subset) {
        for (int b = 0; b < B; ++b) {
            const int s = seq_subset[b];
            if (s < -1 || s >= (int)h->subset_dev.size()) return MTP_ERR_SUBSET;
            if (b > 0 && s == seq_subset[b - 1]) {
                groups.hi[groups.count - 1] = b + 1;
                continue;
            }
            for (int g = 0; g < groups.count; ++g) // a list may head one run of adjacent sequences only
                if (group_subset[g] == s) return MTP_ERR_SUBSET;
            if (groups.count == kMaxListGroups) return MTP_ERR_SUBSET;
            group_subset[groups.count] = s;
            const int g = groups.count++;
            groups.lo[g] = b;
            groups.hi[g] = b + 1;
            groups.ids[g] = s < 0 ? nullptr : h->subset_dev[s];
            groups.n[g] = s < 0 ? c.vocab_size : h->subset_n[s];
        }
        subset_index = seq_subset[0];
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    DraftParams p{};
    p.d = c.d_model;
    p.Hq = c.n_q_heads;
    p.Hkv = c.n_kv_heads;
    p.hd = c.head_dim;
    p.F = c.d_ffn;
    p.V = c.vocab_size;
    p.qd = c.n_q_heads * c.head_dim;
    p.kvd = c.n_kv_heads * c.head_dim;
    p.qkv_dim = p.qd + 2 * p.kvd;
    p.cap = c.kv_capacity;
    p.eps = c.rms_eps;
    p.theta = c.rope_theta;
    p.B = B;
    p.K = K;
    p.ids = subset_index < 0 ? nullptr : h->subset_dev[subset_index];
    p.n = subset_index < 0 ? c.vocab_size : h->subset_n[subset_index];
    const mtp_weights &w = h->w;
    auto u16 = [](const void *q) { return static_cast<const uint16_t *>(q); };
    p.embed = u16(w.embed);
    p.lm_head = u16(w.lm_head);
    p.g_h = u16(w.g_hnorm);
    p.g_e = u16(w.g_enorm);
    p.g_attn = u16(w.g_attn_norm);
    p.g_mlp = u16(w.g_mlp_norm);
    p.g_final = u16(w.g_final_norm);
    p.w_proj = u16(w.w_proj);
    p.w_q = u16(w.w_q);
    p.w_k = u16(w.w_k);
    p.w_v = u16(w.w_v);
    p.b_q = u16(w.b_q);
    p.b_k = u16(w.b_k);
    p.b_v = u16(w.b_v);
    p.w_o = u16(w.w_o);
    p.w_gate = u16(w.w_gate);
    p.w_up = u16(w.w_up);
    p.w_down = u16(w.w_down);
    p.hidden_in = u16(hidden_in);
    p.token_in = token_in;
    p.kv_len = kv_len;
    p.forced = forced_tokens;
    p.k_cache = static_cast<uint16_t *>(k_cache);
    p.v_cache = static_cast<uint16_t *>(v_cache);
    p.draft_out = draft_out;
    p.logits_out = logits_out;
    p.hidden_out = hidden_out;
    char *ws = h->ws;
    const WsLayout &l = h->lay;
    p.x = reinterpret_cast<float *>(ws + l.x);
    p.qkv = reinterpret_cast<float *>(ws + l.qkv);
    p.attn = reinterpret_cast<float *>(ws + l.attn);
    p.o = reinterpret_cast<float *>(ws + l.o);
    p.gu = reinterpret_cast<float *>(ws + l.gu);
    p.dn = reinterpret_cast<float *>(ws + l.dn);
    p.hhat = reinterpret_cast<float *>(ws + l.hhat);
    p.err = reinterpret_cast<int *>(ws + l.err);
    p.rope_inv = reinterpret_cast<const double *>(ws + l.rope_inv);
    p.attn_part = reinterpret_cast<float *>(ws + l.attn_part);
    p.attn_ticket = reinterpret_cast<int *>(ws + l.attn_ticket); // the vector attention merges its own splits
    p.attn_queue = p.attn_ticket + (size_t)2 * c.max_batch * c.n_kv_heads;
    p.cand = reinterpret_cast<unsigned long long *>(ws + l.cand);
    p.xt = reinterpret_cast<unsigned long long *>(ws + l.xt);
    p.qkvt = reinterpret_cast<unsigned long long *>(ws + l.qkvt);
    p.attnt = reinterpret_cast<unsigned long long *>(ws + l.attnt);
    p.ot = reinterpret_cast<unsigned long long *>(ws + l.ot);
    p.gut = reinterpret_cast<unsigned long long *>(ws + l.gut);
    p.dnt = reinterpret_cast<unsigned long long *>(ws + l.dnt);
    p.candt = reinterpret_cast<unsigned long long *>(ws + l.candt);
    p.bar_timeout = 200000000ll; // 2 s of the 100 MHz wall clock
    p.trace = h->trace;
    p.max_batch = c.max_batch;
    p.seq_lo = 0;
    p.seq_hi = B;
    p.logit_stride = p.n;
    for (int g = 0; g < groups.count; ++g) p.logit_stride = std::max(p.logit_stride, groups.n[g]);
    if (own_hidden) { // the first step starts from the head's own output of an earlier call
        if (hipMemcpyAsync(p.hhat, own_hidden, (size_t)B * p.d * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess)
            return MTP_ERR_HIP;
        p.own_hidden = 1;
    }
    const int att_B = B; // sequences (or rows of a block of positions) an attention launch covers
    p.split_tokens = split_tokens_for(c, att_B);
    p.max_splits = max_splits_for(c, att_B);
    if (ext) { // per-row cache lengths for the matrix phases
        int *row_len = reinterpret_cast<int *>(ws + l.row_len);
        hipLaunchKernelGGL(k_extend_prep, dim3((B + 255) / 256), dim3(256), 0, st, ext->B, ext->m_max, c.kv_capacity,
                           ext->kv_len, ext->ext_len, row_len);
        p.kv_len = row_len;
    }

    auto publish_lists = [&]() { // the groups' tables, once their candidate counts are known
        if (!groups.count) return;
        int *seq_list = reinterpret_cast<int *>(ws + l.seq_list);
        const int **list_ids = reinterpret_cast<const int **>(ws + l.list_ids);
        int *list_n = reinterpret_cast<int *>(ws + l.list_n), *list_cands = reinterpret_cast<int *>(ws + l.list_cands);
        hipLaunchKernelGGL(k_set_lists, dim3(1), dim3(256), 0, st, groups, seq_list, list_ids, list_n, list_cands);
        p.seq_list = seq_list;
        p.list_ids = list_ids;
        p.list_n = list_n;
        p.list_cands = list_cands;
    };
    // sequences per weight pass, bounded by LDS
    size_t budget = std::min(h->lds_limit, B <= 2 ? kLdsSmallBatch : kLdsLargeBatch);
    auto fit = [&](int Kdim, int nmat) {
        int nb = 1;
        while (nb < std::min(B, 16) && gemv_lds_bytes(Kdim, nb + 1, nmat) <= budget) ++nb;
        return nb;
    };
    p.nb_proj = fit(2 * p.d, 1);
    p.nb_d = fit(p.d, 2);
    p.nb_q = fit(p.qd, 1);
    p.nb_down = fit(p.F, 1);
    const size_t lds_proj = gemv_lds_bytes(2 * p.d, p.nb_proj, 1), lds_d1 = gemv_lds_bytes(p.d, p.nb_d, 1),
                 lds_d2 = gemv_lds_bytes(p.d, p.nb_d, 2), lds_q = gemv_lds_bytes(p.qd, p.nb_q, 1),
                 lds_down = gemv_lds_bytes(p.F, p.nb_down, 1),
                 lds_attn = std::max(attn_lds_bytes(p.Hq / p.Hkv, p.hd),
                                     // the matrix-core kernel's tiles or the merge's strips, flags, then the item map
                                     std::max(attn_mfma_lds_bytes(p.Hq / p.Hkv, p.hd), (size_t)kWaves * p.max_splits * 4) +
                                         64 + 16 + attn_map_bytes(att_B, p.max_splits));
    // the matrix-core attention over a block of positions (sixteen query columns)
    const size_t lds_attn_block = std::max(attn_mfma_block_lds_bytes(p.Hq / p.Hkv, p.hd) + 64,
                                           (size_t)kWaves * p.max_splits * 4 + 64);
    const size_t lds_max = std::max({lds_proj, lds_d2, lds_q, lds_down, lds_attn, ext ? lds_attn_block : 0});
    if (lds_max > h->lds_limit) return MTP_ERR_CONFIG;

    const int grid = std::min(h->num_cus, kMaxFusedGrid); // one 512-thread workgroup per CU: the register ring
                                                          // leaves no room for a second
    p.head_grid = grid;
    const int attn_items = att_B * p.Hkv * p.max_splits;
    // splits of at least kMfmaAttnMinSplit tokens: the matrix-core attention (below); one of its workgroups fills a
    // compute unit, and a workgroup that starts only when another has left would take its first item, a whole split
    // of the first sequences, at the very end
    const bool mfma_attn = p.split_tokens >= (ext && ext->m_max > 1 ? 2 * kMfmaAttnMinSplit : kMfmaAttnMinSplit);
    const int attn_grid = std::max(1, std::min(attn_items, h->num_cus * (mfma_attn ? 1 : 2)));
    // more items than workgroups: the matrix-core attention hands them out one by one (contexts differ in length)
    if (attn_items <= attn_grid) p.attn_queue = nullptr;

    const int tphase = h->timing >= 2 ? h->timing - 2 : -1;
    h->pev_used = 0;
    // One sequence and every reduction at least 512 long: all phases of all K steps in ONE launch whose workgroups hand
    // their results over as tagged elements (flow.h).  Its workgroups wait for one another, so all of them must be
    // resident at once: one per CU (the launch's LDS and registers leave no room for a second, and init has checked
    // that one fits).  A cooperative launch would have the runtime verify that, but it leaves a 20 us gap between
    // consecutive launches (measured: 464 us kernels every 485 us) where an ordinary launch leaves 5; on a device that
    // another kernel occupies at that moment the waits are bounded (MTP_ERR_TIMEOUT).  Mode 2 picks it where it
    // applies; more sequences, and shapes it does not serve, take one launch per phase in every mode.
    // Its tags count calls on the host, so a call that is being captured into a HIP graph - whose replays would all
    // carry the tags of the captured call - takes one launch per phase instead (those kernels keep no state across
    // calls on the host).
    const bool rows = B == 1 && p.d >= 512 && p.qd >= 512 && p.F >= 512;
    bool capturing = false;
    if (st != nullptr) { // (the legacy default stream cannot be captured, and asking about it disturbs other captures)
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(st, &cap) != hipSuccess) {
            (void)hipGetLastError();
            return MTP_ERR_HIP;
        }
        capturing = cap != hipStreamCaptureStatusNone;
    }
    if ((h->mode == 1 || h->mode == 2) && rows && tphase < 0 && !ext && !seq_subset && !capturing) {
        const int fgrid = std::min(h->num_cus, kMaxFusedGrid);
        size_t region = std::max(flow_gemv_region(p.d, p.qd, p.F), lds_attn);
        region = (region + 255) / 256 * 256;
        const size_t lds_flow = region + flow_tail_bytes(p.d, fgrid);
        bool fits = lds_flow <= h->lds_limit;
        if (fits && lds_flow > h->flow_lds_ok) { // once per LDS size: a workgroup of this kernel fits a compute unit
            int per_cu = 0;
            fits = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)h->flow_fn, kBlock, lds_flow) ==
                       hipSuccess &&
                   per_cu >= 1;
            if (fits)
                h->flow_lds_ok = lds_flow;
            else
                (void)hipGetLastError();
        }
        if (fits) {
            p.head_grid = fgrid;
            p.fused_gemv_bytes = (int)region;
            // The attention inside this kernel: its items are (KV head, split, half of the KV head's query heads), at
            // most as many as there are workgroups, in whole rounds of 32 tokens (8 waves x 4 tokens; up to five rounds
            // run as one, phase_attn's U): fewer, fuller splits beat more workgroups with a ragged last round (160
            // against 136 tokens at a capacity of 2112: 0.9 us per step).  Never shorter splits than the plan the
            // workspace was sized for.
            const int plan_tokens = p.split_tokens, plan_splits = p.max_splits;
            {
                const int parts = p.Hq / p.Hkv >= 2 ? 2 : 1; // kFlowAttnParts
                const long long want = ((long long)c.kv_capacity * p.Hkv * parts + fgrid - 1) / fgrid;
                const long long t = std::min<long long>(std::max<long long>(plan_tokens, (want + 31) / 32 * 32), kMaxSplitTokens);
                p.split_tokens = (int)t;
                p.max_splits = (int)((c.kv_capacity + t - 1) / t);
            }
            // tags of this call: tag_base + 1 .. tag_base + 8 K, never 0 and never reused: when the 32-bit counter would
            // wrap, the tagged vectors are cleared and the count starts over
            const unsigned long long need = 8ull * (unsigned long long)K + 8ull;
            if ((h->flow_tags & 0xffffffffull) + need > 0xffffffffull) {
                const size_t words = (l.tagged_end - l.xt) / 8;
                hipLaunchKernelGGL(k_zero_words, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st,
                                   reinterpret_cast<unsigned long long *>(ws + l.xt), (int)words);
                h->flow_tags = 0;
            }
            p.tag_base = (unsigned)h->flow_tags;
            void *args[] = {(void *)&p};
            if (h->timing == 1) (void)hipEventRecord(h->ev[0], st);
            const bool launched = hipLaunchKernel((const void *)h->flow_fn, dim3(fgrid), dim3(kBlock), args,
                                                  (unsigned)lds_flow, st) == hipSuccess;
            if (launched) {
                h->flow_tags += 8ull * (unsigned long long)K;
                if (h->timing == 1) {
                    (void)hipEventRecord(h->ev[1], st);
                    h->ev_recorded = true;
                }
                return MTP_OK;
            }
            (void)hipGetLastError();
            if (h->mode == 1) return MTP_ERR_HIP; // asked for explicitly
            // mode 2: the launch was refused: one launch per phase
            p.split_tokens = plan_tokens;
            p.max_splits = plan_splits;
        }
    }
    auto mark_begin = [&](int phase, int step) {
        if (phase == tphase) (void)hipEventRecord(h->pev[2 * (size_t)step], st);
    };
    auto mark_end = [&](int phase, int step) {
        if (phase == tphase) {
            (void)hipEventRecord(h->pev[2 * (size_t)step + 1], st);
            h->pev_used = step + 1;
        }
    };
    // long splits go to the matrix-core attention; short ones (small batch, short context) to the latency-lean
    // vector version
    // (a block of positions pays more set-up per item on the matrix cores, sixteen query columns: 320-token splits of a
    // four-position block take 40 us there and 26 us on the vector units)
    auto launch_attention_of = [&](const DraftParams &pa, int step) {
        if (mfma_attn)
            launch_attn_mfma(pa.Hq / pa.Hkv, pa.hd, pa, step, attn_grid, lds_attn, st);
        else
            hipLaunchKernelGGL(h->attn_fn, dim3(attn_grid), dim3(kBlock), lds_attn, st, pa, step);
    };
    // attention (both kernels merge their own splits)
    auto launch_attention = [&](int step) {
        if (!ext) {
            launch_attention_of(p, step);
            return;
        }
        // a block of new positions: every row's key and value go into the cache first, then one launch serves all
        // rows, each reading its sequence's cache up to and including its own slot (kv_len = the rows' lengths)
        DraftParams pa = p;
        pa.kv_appended = 1;
        pa.ext_B = ext->B;
        if (p.hd == 128)
            hipLaunchKernelGGL(k_extend_append<128>, dim3(B, p.Hkv), dim3(192), 0, st, pa);
        else
            hipLaunchKernelGGL(k_extend_append<64>, dim3(B, p.Hkv), dim3(96), 0, st, pa);
        if (mfma_attn && ext->m_max > 1) {
            // long splits: the positions of a sequence share its key/value reads (16 / G of them per item)
            const int G = pa.Hq / pa.Hkv, jp = 16 / G, jg = (ext->m_max + jp - 1) / jp;
            const int items = ext->B * pa.Hkv * pa.max_splits * jg;
            const int grid_b = std::max(1, std::min(items, h->num_cus * 2));
            pa.attn_queue = items > grid_b ? pa.attn_ticket + (size_t)2 * c.max_batch * c.n_kv_heads : nullptr;
            launch_attn_mfma_block(G, pa.hd, pa, 0, grid_b, lds_attn_block, st);
        } else {
            launch_attention_of(pa, 0);
        }
    };
    auto launch = [&](int phase, phase_kernel_t fn, int g, size_t lds, int step) {
        mark_begin(phase, step);
        hipLaunchKernelGGL(fn, dim3(g), dim3(kBlock), lds, st, p, step);
        mark_end(phase, step);
    };
    if (h->timing == 1) (void)hipEventRecord(h->ev[0], st);

    // Two or more sequences (or rows of a block of positions): the batched kernels, every weight read once per pass of
    // up to 64 sequences.  The row-streaming kernels serve up to four at once but at half their one-sequence rate from
    // the second on (a block of four positions at a 32768-row head: 404 us against 234 here); they remain for one
    // sequence, on request (mode 3), and for matrices of 2 GiB or more: the batched kernels' buffer loads address a
    // matrix with 32-bit offsets and mark missing rows with an offset of 2 GiB.
    const size_t widest = std::max({(size_t)p.V * p.d, (size_t)p.d * 2 * p.d, (size_t)p.F * p.d, (size_t)p.qd * p.d}) * 2;
    const bool rows_wanted = h->mode == 3 && B <= kMaxRowSeq; // the row-streaming kernels on request
    if (B >= kBatchMinSeq && !rows_wanted && widest < ((size_t)1 << 31)) {
        p.act[0] = reinterpret_cast<uint16_t *>(ws + l.act0);
        p.act[1] = reinterpret_cast<uint16_t *>(ws + l.act1);
        p.a_lo = l.a_lo;
        p.a_stride = l.a_stride;
        p.attn_split = p.act[0];
        p.ssq = reinterpret_cast<float *>(ws + l.ssq);
        p.part = reinterpret_cast<float *>(ws + l.part);
        p.ticket = reinterpret_cast<int *>(ws + l.ticket);
        size_t lds_bg[BG_COUNT];
        // units: 16-row tiles (gate/up: pairs of tiles); kdim: reduction length
        // One plan per call: passes of one call share it (a last, smaller pass runs a little off its optimum).
        // Up to 16 sequences a workgroup's waves split the reduction and a row group holds eight tiles; above, its
        // waves split the 64/NA tiles of a block.  A phase with fewer tiles than that per workgroup splits the
        // reduction over KP workgroups, each keeping at least four double steps.
        const int na = B <= 16 ? 1 : B <= 32 ? 2 : 4;
        // tiles a row group should hold: eight up to 16 sequences (one group of a wave), a full block of 64/NA above
        const int block_tiles = na == 1 ? kBatchGroupTiles : kWaves * (kBatchGroupTiles / na);
        auto plan = [&](int ph, int units, int nmat, int kdim) {
            const int nks = (kdim + 63) / 64; // double depth steps
            const long long ntv = (long long)units * nmat;
            int rg, kp = 1;
            if (na == 1 && ntv >= 4ll * grid) {
                rg = std::min(grid, units);
            } else {
                kp = (int)std::max(1ll, std::min<long long>((long long)grid * block_tiles / ntv,
                                                             na == 1 ? nks / kWaves : nks / 4));
                kp = std::max(1, std::min(kp, grid));
                rg = std::max(1, std::min(grid / kp, units));
            }
            p.bg_rg[ph] = rg;
            p.bg_kp[ph] = kp;
            // Split reductions: who adds the parts.  Up to 16 sequences the last workgroup of a row group to arrive
            // does (a relaxed ticket; the parts are written and read with device-coherent accesses, no cache is written
            // back or invalidated): config 3 runs 2.4 % faster than with a kernel of its own per phase.  Above 16
            // sequences a row group holds 64/NA tiles x NA sequence tiles of sums and the last workgroup becomes the
            // bottleneck (config 5: 8.6 % slower), so there a small epilogue kernel spread over the chip adds them -
            // except for the output head, whose epilogue kernel would leave four times as many argmax candidates
            // behind (measured: 122 vs 97 us at 64 sequences).
            p.bg_sep[ph] = (kp >= 2 && ph != BG_LMHEAD && na > 1) ? 1 : 0;
            lds_bg[ph] = bgemv_lds_bytes(((units + rg - 1) / rg) * 16);
        };
        plan(BG_PROJ, p.d / 16, 1, 2 * p.d);
        plan(BG_QKV, p.qkv_dim / 16, 1, p.d);
        plan(BG_OPROJ, p.d / 16, 1, p.qd);
        plan(BG_GATEUP, (p.F + 15) / 16, 2, p.d);
        plan(BG_DOWN, p.d / 16, 1, p.F);
        // the output head: one plan per id list (one list: one plan)
        struct HeadPlan {
            int rg, kp, sep;
            size_t lds;
        } head_plan[kMaxListGroups];
        const int n_heads = std::max(1, groups.count);
        int max_cands = 0;
        for (int g = 0; g < n_heads; ++g) {
            plan(BG_LMHEAD, ((groups.count ? groups.n[g] : p.n) + 15) / 16, 1, p.d);
            head_plan[g] = HeadPlan{p.bg_rg[BG_LMHEAD], p.bg_kp[BG_LMHEAD], p.bg_sep[BG_LMHEAD], lds_bg[BG_LMHEAD]};
            if (lds_bg[BG_LMHEAD] > h->lds_limit) return MTP_ERR_CONFIG;
            const int cands = p.bg_sep[BG_LMHEAD] ? batch_epilogue_grid(BG_LMHEAD, p, na) : p.bg_rg[BG_LMHEAD];
            if (groups.count) groups.cands[g] = cands;
            max_cands = std::max(max_cands, cands);
        }
        for (int ph = 0; ph < BG_COUNT; ++ph)
            if (lds_bg[ph] > h->lds_limit) return MTP_ERR_CONFIG;
        // candidates of the output head: one per row group, or one per workgroup of its separate epilogue, whose
        // grid is then this number for every pass of the call (workgroups without work leave "no candidate")
        p.head_grid = max_cands;
        publish_lists();
        // Many rows: matrix phases as tiled matrix products over all rows instead of one pass of the batched core per
        // 64.  The output head has hundreds of weight-row blocks at any row count, but its tiled form leaves no
        // candidates: for callers that want logits only (the training loss), from 65 rows on.  The body's phases have
        // as few as 32 blocks of weight rows and fill the chip only from four passes' worth of rows on (measured at
        // 128 rows: 1034 us per step against 757 with two passes, at 256 rows 1350 against 1458).
        const bool tiled = ext && ext->logits_only && B > kBatchPassSeq && !groups.count && logits_out;
        const bool tiled_body = B >= 4 * kBatchPassSeq;
        auto matrix_phase = [&](int timed_as, int ph, int step) {
            if ((ph == BG_LMHEAD ? tiled : tiled_body) && rows_gemm_serves(ph, p)) {
                launch_rows_gemm(ph, p, step, h->num_cus, st);
                mark_end(timed_as, step);
                return;
            }
            const int runs = ph == BG_LMHEAD ? n_heads : 1; // the output head: once per id list
            for (int g = 0; g < runs; ++g) {
                int lo = 0, hi = B;
                if (ph == BG_LMHEAD) {
                    p.bg_rg[ph] = head_plan[g].rg;
                    p.bg_kp[ph] = head_plan[g].kp;
                    p.bg_sep[ph] = head_plan[g].sep;
                    lds_bg[ph] = head_plan[g].lds;
                    if (groups.count) {
                        lo = groups.lo[g];
                        hi = groups.hi[g];
                        p.ids = groups.ids[g];
                        p.n = groups.n[g];
                    }
                }
                for (int b0 = lo; b0 < hi; b0 += kBatchPassSeq) {
                    p.b0 = b0;
                    p.nb = std::min(kBatchPassSeq, hi - b0);
                    launch_bgemv(ph, p, step, p.bg_rg[ph] * p.bg_kp[ph], lds_bg[ph], st);
                }
            }
            mark_end(timed_as, step);
        };
        for (int step = 0; step < K; ++step) {
            mark_begin(PH_PROJ, step);
            launch_bprep(p, step, st);
            matrix_phase(PH_PROJ, BG_PROJ, step);
            mark_begin(PH_QKV, step);
            matrix_phase(PH_QKV, BG_QKV, step);
            mark_begin(PH_ATTN, step);
            launch_attention(step);
            mark_end(PH_ATTN, step);
            mark_begin(PH_OPROJ, step);
            matrix_phase(PH_OPROJ, BG_OPROJ, step);
            mark_begin(PH_GATEUP, step);
            matrix_phase(PH_GATEUP, BG_GATEUP, step);
            mark_begin(PH_DOWN, step);
            matrix_phase(PH_DOWN, BG_DOWN, step);
            mark_begin(PH_LMHEAD, step);
            matrix_phase(PH_LMHEAD, BG_LMHEAD, step);
        }
        launch_bprep(p, K, st);
        if (ext)
            hipLaunchKernelGGL(k_extend_finish, dim3((ext->B + 63) / 64), dim3(64), 0, st, ext->B, ext->m_max,
                               c.kv_capacity, ext->kv_len, ext->ext_len);
        if (h->timing == 1) {
            (void)hipEventRecord(h->ev[1], st);
            h->ev_recorded = true;
        }
        if (hipGetLastError() != hipSuccess) return MTP_ERR_HIP;
        return MTP_OK;
    }
    for (int g = 0; g < groups.count; ++g) groups.cands[g] = grid; // every launch leaves one candidate per workgroup
    publish_lists();
    for (int step = 0; step < K; ++step) {
        launch(PH_PROJ, k_proj, grid, lds_proj, step);
        launch(PH_QKV, k_qkv, grid, lds_d1, step);
        mark_begin(PH_ATTN, step);
        launch_attention(step);
        mark_end(PH_ATTN, step);
        launch(PH_OPROJ, k_oproj, grid, lds_q, step);
        launch(PH_GATEUP, k_gateup, grid, lds_d2, step);
        launch(PH_DOWN, k_down, grid, lds_down, step);
        if (!groups.count) {
            launch(PH_LMHEAD, k_lmhead, grid, lds_d1, step);
        } else { // once per id list, over that list's sequences
            mark_begin(PH_LMHEAD, step);
            for (int g = 0; g < groups.count; ++g) {
                p.seq_lo = groups.lo[g];
                p.seq_hi = groups.hi[g];
                p.ids = groups.ids[g];
                p.n = groups.n[g];
                hipLaunchKernelGGL(k_lmhead, dim3(grid), dim3(kBlock), lds_d1, st, p, step);
            }
            mark_end(PH_LMHEAD, step);
        }
    }
    hipLaunchKernelGGL(k_finalize, dim3((B + kWaves - 1) / kWaves), dim3(kBlock), 0, st, p);
    if (ext)
        hipLaunchKernelGGL(k_extend_finish, dim3((ext->B + 63) / 64), dim3(64), 0, st, ext->B, ext->m_max,
                           c.kv_capacity, ext->kv_len, ext->ext_len);
    if (h->timing == 1) {
        (void)hipEventRecord(h->ev[1], st);
        h->ev_recorded = true;
    }
    if (hipGetLastError() != hipSuccess) return MTP_ERR_HIP;
    return MTP_OK;
}

} // namespace

extern "C" {

int32_t mtp_draft_steps(mtp_handle *h, int32_t B, int32_t K, int32_t subset_index, const void *hidden_in,
                        const int32_t *token_in, void *k_cache, void *v_cache, const int32_t *kv_len,
                        const int32_t *forced_tokens, int32_t *draft_out, float *logits_out, float *hidden_out,
                        void *hip_stream) {
    if (!h || !hidden_in || !token_in || !k_cache || !v_cache || !kv_len || !draft_out) return MTP_ERR_NULL;
    const void *ptrs[] = {hidden_in, token_in, k_cache, v_cache, kv_len, forced_tokens, draft_out, logits_out,
                          hidden_out};
    for (const void *p : ptrs)
        if (!aligned16(p)) return MTP_ERR_ALIGN;
    const mtp_config &c = h->cfg;
    if (B < 1 || B > c.max_batch) return MTP_ERR_BATCH;
    if (K < 1 || K > c.max_draft_steps) return MTP_ERR_STEPS;
    if (subset_index < -1 || subset_index >= (int)h->subset_dev.size()) return MTP_ERR_SUBSET;
    return run_draft(h, B, K, subset_index, hidden_in, token_in, k_cache, v_cache, kv_len, forced_tokens, draft_out,
                     logits_out, hidden_out, hip_stream, nullptr);
}

int32_t mtp_draft_steps_lists(mtp_handle *h, int32_t B, int32_t K, const int32_t *seq_subset, const void *hidden_in,
                              const int32_t *token_in, void *k_cache, void *v_cache, const int32_t *kv_len,
                              const int32_t *forced_tokens, int32_t *draft_out, float *logits_out, float *hidden_out,
                              void *hip_stream) {
    if (!h || !seq_subset || !hidden_in || !token_in || !k_cache || !v_cache || !kv_len || !draft_out)
        return MTP_ERR_NULL;
    const void *ptrs[] = {hidden_in, token_in, k_cache, v_cache, kv_len, forced_tokens, draft_out, logits_out,
                          hidden_out};
    for (const void *p : ptrs)
        if (!aligned16(p)) return MTP_ERR_ALIGN;
    const mtp_config &c = h->cfg;
    if (B < 1 || B > c.max_batch) return MTP_ERR_BATCH;
    if (K < 1 || K > c.max_draft_steps) return MTP_ERR_STEPS;
    return run_draft(h, B, K, 0, hidden_in, token_in, k_cache, v_cache, kv_len, forced_tokens, draft_out, logits_out,
                     hidden_out, hip_stream, nullptr, nullptr, seq_subset);
}

int32_t mtp_draft_continue(mtp_handle *h, int32_t B, int32_t K, int32_t subset_index, const float *own_hidden,
                           const int32_t *token_in, void *k_cache, void *v_cache, const int32_t *kv_len,
                           const int32_t *forced_tokens, int32_t *draft_out, float *logits_out, float *hidden_out,
                           void *hip_stream) {
    if (!h || !own_hidden || !token_in || !k_cache || !v_cache || !kv_len || !draft_out) return MTP_ERR_NULL;
    const void *ptrs[] = {own_hidden, token_in, k_cache, v_cache, kv_len, forced_tokens, draft_out, logits_out,
                          hidden_out};
    for (const void *p : ptrs)
        if (!aligned16(p)) return MTP_ERR_ALIGN;
    const mtp_config &c = h->cfg;
    if (B < 1 || B > c.max_batch) return MTP_ERR_BATCH;
    if (K < 1 || K > c.max_draft_steps) return MTP_ERR_STEPS;
    if (subset_index < -1 || subset_index >= (int)h->subset_dev.size()) return MTP_ERR_SUBSET;
    return run_draft(h, B, K, subset_index, own_hidden, token_in, k_cache, v_cache, kv_len, forced_tokens, draft_out,
                     logits_out, hidden_out, hip_stream, nullptr, own_hidden);
}

int32_t mtp_draft_extend(mtp_handle *h, int32_t B, int32_t m_max, int32_t subset_index, const void *hidden_in,
                         const int32_t *tokens, const int32_t *ext_len, void *k_cache, void *v_cache, int32_t *kv_len,
                         int32_t *draft_out, float *logits_out, float *hidden_out, void *hip_stream) {
    if (!h || !hidden_in || !tokens || !ext_len || !k_cache || !v_cache || !kv_len || !draft_out) return MTP_ERR_NULL;
    const void *ptrs[] = {hidden_in, tokens, ext_len, k_cache, v_cache, kv_len, draft_out, logits_out, hidden_out};
    for (const void *p : ptrs)
        if (!aligned16(p)) return MTP_ERR_ALIGN;
    const mtp_config &c = h->cfg;
    if (B < 1 || m_max < 1 || (long long)B * m_max > c.max_batch) return MTP_ERR_BATCH;
    if (subset_index < -1 || subset_index >= (int)h->subset_dev.size()) return MTP_ERR_SUBSET;
    const ExtendCall ext{B, m_max, ext_len, kv_len};
    return run_draft(h, B * m_max, 1, subset_index, hidden_in, tokens, k_cache, v_cache, kv_len, nullptr, draft_out,
                     logits_out, hidden_out, hip_stream, &ext);
}

size_t mtp_train_workspace_bytes(const mtp_config *cfg, int32_t n_pos) {
    if (!config_ok(cfg) || n_pos < 1) return 0;
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    return up((size_t)n_pos * cfg->vocab_size * 4) + up((size_t)n_pos * cfg->d_model * 4) + 2 * up((size_t)n_pos * 4) + 512;
}

int32_t mtp_train_loss(mtp_handle *h, int32_t n_pos, int32_t K, float beta, const void *hidden_in,
                       const int32_t *tokens, void *k_cache, void *v_cache, void *scratch, size_t scratch_bytes,
                       float *loss_out, void *hip_stream) {
    if (!h || !hidden_in || !tokens || !k_cache || !v_cache || !scratch || !loss_out) return MTP_ERR_NULL;
    const void *ptrs[] = {hidden_in, tokens, k_cache, v_cache, scratch, loss_out};
    for (const void *p : ptrs)
        if (!aligned16(p)) return MTP_ERR_ALIGN;
    const mtp_config &c = h->cfg;
    if (n_pos < 1 || n_pos > c.max_batch || n_pos > c.kv_capacity) return MTP_ERR_BATCH;
    if (K < 1 || K > 16 || !(beta > 0.f)) return MTP_ERR_STEPS;
    if (scratch_bytes < mtp_train_workspace_bytes(&c, n_pos)) return MTP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    char *s0 = static_cast<char *>(scratch);
    float *logits = reinterpret_cast<float *>(s0);
    float *hidden = reinterpret_cast<float *>(s0 + up((size_t)n_pos * c.vocab_size * 4));
    float *row_loss = reinterpret_cast<float *>(reinterpret_cast<char *>(hidden) + up((size_t)n_pos * c.d_model * 4));
    int32_t *draft = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(row_loss) + up((size_t)n_pos * 4));
    int32_t *kv_len = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(draft) + up((size_t)n_pos * 4));
    int32_t *ext_len = kv_len + 64;
    int *err = reinterpret_cast<int *>(h->ws + h->lay.err);
    const ExtendCall ext{1, n_pos, ext_len, kv_len, true};
    for (int k = 1; k <= K; ++k) {
        // Step k over all positions: the block-of-positions pipeline from an empty cache.  Position i consumes
        // (h^{k-1}_i, t_{i+k}): the main model's states at k = 1, the head's own output of step k-1 afterwards.
        hipLaunchKernelGGL(k_train_begin_step, dim3(1), dim3(64), 0, st, n_pos, kv_len, ext_len);
        const int32_t rc = run_draft(h, n_pos, 1, -1, hidden_in, tokens + k, k_cache, v_cache, kv_len, nullptr, draft,
                                     logits, hidden, hip_stream, &ext, k > 1 ? hidden : nullptr);
        if (rc != MTP_OK) return rc;
        hipLaunchKernelGGL(k_train_row_ce, dim3(n_pos), dim3(256), 0, st, logits, c.vocab_size, tokens + k + 1,
                           row_loss, err);
        hipLaunchKernelGGL(k_train_step_mean, dim3(1), dim3(256), 0, st, row_loss, n_pos, loss_out, k - 1, K, beta);
    }
    if (hipGetLastError() != hipSuccess) return MTP_ERR_HIP;
    return MTP_OK;
}

int32_t mtp_accept(mtp_handle *h, int32_t B, int32_t K, const int32_t *draft, const int32_t *target,
                   int32_t rollback_mode, int32_t *kv_len, int32_t *accept_len, int32_t *out_tokens,
                   int32_t *pending, void *hip_stream) {
    if (!h || !draft || !target || !kv_len || !accept_len || !out_tokens || !pending) return MTP_ERR_NULL;
    const void *ptrs[] = {draft, target, kv_len, accept_len, out_tokens, pending};
    for (const void *p : ptrs)
        if (!aligned16(p)) return MTP_ERR_ALIGN;
    if (B < 1 || B > h->cfg.max_batch) return MTP_ERR_BATCH;
    if (K < 1 || K > h->cfg.max_draft_steps) return MTP_ERR_STEPS;
    if (rollback_mode != 0 && rollback_mode != 1) return MTP_ERR_MODE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipLaunchKernelGGL(k_accept, dim3((B + 63) / 64), dim3(64), 0, st, B, K, draft, target, rollback_mode, kv_len,
                       accept_len, out_tokens, pending);
    if (hipGetLastError() != hipSuccess) return MTP_ERR_HIP;
    return MTP_OK;
}

int32_t mtp_poll_error(mtp_handle *h, void *hip_stream) {
    if (!h) return MTP_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    int word = 0;
    int *dev = reinterpret_cast<int *>(h->ws + h->lay.err);
    if (hipMemcpyAsync(&word, dev, 4, hipMemcpyDeviceToHost, st) != hipSuccess) return MTP_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return MTP_ERR_HIP;
    if (word != 0) {
        if (hipMemsetAsync(dev, 0, 4, st) != hipSuccess) return MTP_ERR_HIP;
        if (word & kErrBarrierTimeout) {
            // a kernel that gave up may have left arrival counters of the attention splits behind (the hand-over tags
            // need nothing: the next call's tags are larger than any the abandoned call wrote)
            if (hipMemsetAsync(h->ws + h->lay.attn_ticket, 0, (size_t)h->cfg.max_batch * h->cfg.n_kv_heads * 4 * 2 + 64, st) !=
                hipSuccess)
                return MTP_ERR_HIP;
        }
        if (hipStreamSynchronize(st) != hipSuccess) return MTP_ERR_HIP;
    }
    if (word & kErrBarrierTimeout) return MTP_ERR_TIMEOUT;
    if (word & kErrKvOverflow) return MTP_ERR_KV_OVERFLOW;
    if (word & kErrTokenRange) return MTP_ERR_TOKEN_RANGE;
    return MTP_OK;
}

int32_t mtp_stream_probe(const void *buffer, size_t bytes, void *out8, void *hip_stream) {
    if (!buffer || !out8) return MTP_ERR_NULL;
    if (!aligned16(buffer) || !aligned16(out8)) return MTP_ERR_ALIGN;
    const long long blocks = (long long)(bytes / (16 * 1024));
    if (blocks < 1) return MTP_ERR_CONFIG;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return MTP_ERR_HIP;
    hipLaunchKernelGGL(k_stream_probe, dim3(cus), dim3(kBlock), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const u32x4 *>(buffer), blocks, static_cast<unsigned long long *>(out8));
    if (hipGetLastError() != hipSuccess) return MTP_ERR_HIP;
    return MTP_OK;
}

int32_t mtp_set_timing(mtp_handle *h, int32_t mode) {
    if (!h) return MTP_ERR_NULL;
    if (mode < 0 || mode >= 2 + PH_COUNT) return MTP_ERR_MODE;
    h->timing = mode;
    h->ev_recorded = false;
    h->pev_used = 0;
    return MTP_OK;
}

int32_t mtp_set_launch_mode(mtp_handle *h, int32_t mode) {
    if (!h) return MTP_ERR_NULL;
    if (mode < 0 || mode > 3) return MTP_ERR_MODE;
    h->mode = mode;
    return MTP_OK;
}

size_t mtp_phase_trace_bytes(const mtp_config *cfg) {
    if (!config_ok(cfg)) return 0;
    return (size_t)cfg->max_draft_steps * kTraceSections * kTracePoints * kMaxFusedGrid * sizeof(long long);
}

int32_t mtp_set_phase_trace(mtp_handle *h, void *device_buffer) {
    if (!h) return MTP_ERR_NULL;
    if (!aligned16(device_buffer)) return MTP_ERR_ALIGN;
    h->trace = static_cast<long long *>(device_buffer);
    return MTP_OK;
}

float mtp_last_draft_ms(mtp_handle *h) {
    if (!h) return -1.f;
    float ms = 0.f;
    if (h->timing == 1 && h->ev_recorded) {
        if (hipEventSynchronize(h->ev[1]) != hipSuccess) return -1.f;
        if (hipEventElapsedTime(&ms, h->ev[0], h->ev[1]) != hipSuccess) return -1.f;
        return ms;
    }
    if (h->timing >= 2 && h->pev_used > 0) { // mean duration of the selected phase's launches
        float tot = 0.f;
        for (int s = 0; s < h->pev_used; ++s) {
            if (hipEventSynchronize(h->pev[2 * (size_t)s + 1]) != hipSuccess) return -1.f;
            if (hipEventElapsedTime(&ms, h->pev[2 * (size_t)s], h->pev[2 * (size_t)s + 1]) != hipSuccess) return -1.f;
            tot += ms;
        }
        return tot / (float)h->pev_used;
    }
    return -1.f;
}

void mtp_draft_destroy(mtp_handle *h) {
    if (!h) return;
    (void)hipEventDestroy(h->ev[0]);
    (void)hipEventDestroy(h->ev[1]);
    for (auto &e : h->pev) (void)hipEventDestroy(e);
    delete h;
}

} // extern "C"
