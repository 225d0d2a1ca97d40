// Single-launch path for ONE sequence without grid barriers (gfx950): all phases of all K draft steps in one
// kernel (one workgroup per compute unit, all resident) whose workgroups hand their results over element by element.
//
// A draft step at batch 1 is a chain of dependent matrix-vector products (Sec. 2.1) of 30-270 MB each; between two of
// them every workgroup needs the whole result vector of the phase before.  With a grid barrier that hand-over is a
// chain of its own (acknowledge the stores, arrive, count, release, poll, then load the vector: six to nine
// microseconds at 1-2 us per trip while HBM is busy) during which the weight stream runs dry.  Here
//  * every element of a vector that crosses between phases is a 64-bit word holding the float and a tag that names the
//    (call, step, phase) that produced it (device-coherent 8-byte accesses are single-copy atomic).  The consumer
//    polls the elements it needs until they carry the tag it expects: one store and one load separate the last
//    producer from the first consumer, and nobody counts arrivals;
//  * a wave's register ring of weight chunks is not drained at the end of a phase: the slots freed by the last chunks
//    of a phase are refilled with the first chunks of the NEXT phase (weights do not depend on activations), so the
//    memory system keeps streaming while results are handed over and staged;
//  * the projection is split into its hidden-state half and its embedding half (W_p c = W_p[:, :d] c_h + W_p[:, d:] c_e):
//    the hidden-state half needs no result of another workgroup (every workgroup normalises the step's output hidden
//    state itself), so it runs while the output head's argmax candidates travel;
//  * SiLU(gate) * up is formed by the wave that computed both rows, which halves what the down projection polls.
// Why a consumer can never see a tag NEWER than the one it waits for: a workgroup stores results of phase P+1 only
// after it has seen every result of phase P, i.e. after every workgroup has finished computing P and therefore
// finished reading the results of P-1; a vector is rewritten one whole step after it was read.
#pragma once
#include "phases.h"

namespace mtp {

// parts the query heads of a KV head are dealt to in the attention of the single-launch kernel (phase_attn, GS)
template <int G>
constexpr int kFlowAttnParts = G >= 2 ? 2 : 1;

// time stamps of every workgroup (mtp_set_phase_trace): [step][section][point][workgroup]
constexpr int kTraceSections = 8; // projection (embedding half), q/k/v, attention, output projection, gate/up, down,
                                  // output head, projection (hidden-state half)
constexpr int kTracePoints = 4;
enum : int { kTraceRequested = 0, kTraceReleased, kTraceStaged, kTraceDone };

// LDS region shared by the staged activations of every matrix phase (one sequence): bf16 hi then lo halves, each padded
// with zeros to whole 512-element blocks (a row's last block is multiplied in full: the weights beyond the row read as
// zeros, so what stands beside them only has to be finite)
__host__ __device__ inline int flow_kpad(int K) { return (K + 511) / 512 * 512; }
__host__ __device__ inline size_t flow_gemv_region(int d, int qd, int F) {
    int m = flow_kpad(d);
    m = flow_kpad(qd) > m ? flow_kpad(qd) : m;
    m = flow_kpad(F) > m ? flow_kpad(F) : m;
    return ((size_t)m * 4 + 255) / 256 * 256;
}

enum FlowPhase : int { FL_PROJH = 0, FL_PROJE, FL_QKV, FL_O, FL_GATEUP, FL_DOWN, FL_HEAD, FL_NONE };

// One matrix phase as a list of rows (run-time description): up to three matrices stacked row-wise.  PAIRED: the
// rows of [w_gate; w_up] dealt so that a wave gets row q of both, one after the other (its j-th row is gate or up row
// (j / 2) * nw + w for j < 2 * pair_rounds; the F % nw rows that are left over are dealt singly: gate rows to waves
// 0 .. rem-1, up rows to waves rem .. 2 rem - 1).  Virtual row v = w + j * nw, as in every other phase.
struct FlowJob {
    const uint16_t *base[3];
    int seg1, seg2; // first row of the second and of the third matrix
    int pitch;      // elements between consecutive rows of a matrix
    int K, rows;
    const int *ids; // optional row indirection (the compressed output head)
    int paired, pair_rounds, rem, nw;
    // The id list is read-only during the call and row indices are wave-uniform: a scalar load (a vector load would make
    // the wave wait for every weight chunk in flight before it can form the row's address).
    __device__ __forceinline__ int row_id(int v) const {
        typedef const int __attribute__((address_space(4))) *const_int_ptr;
        return ids ? *((const_int_ptr)(ids + min(v, rows - 1))) : 0;
    }
    // rid: the row's entry of the id list (ids jobs), fetched by the caller one chunk ahead
    __device__ __forceinline__ const uint16_t *rowptr(int v, int j, int rid) const {
        if (paired) {
            const int w = v - j * nw;
            int mat, r;
            if (j < 2 * pair_rounds) {
                mat = j & 1;
                r = (j >> 1) * nw + w;
            } else {
                mat = w < rem ? 0 : 1;
                r = pair_rounds * nw + (w < rem ? w : w - rem);
            }
            return (mat ? base[1] : base[0]) + (size_t)r * pitch; // (no run-time index: the struct stays in registers)
        }
        const int r = ids ? rid : v;
        const uint16_t *b = r < seg1 ? base[0] : r < seg2 ? base[1] : base[2];
        const int o = r < seg1 ? r : r < seg2 ? r - seg1 : r - seg2;
        return b + (size_t)o * pitch;
    }
};

__device__ __forceinline__ FlowJob flow_job(const DraftParams &p, int ph, int nw) {
    constexpr int kNone = 0x7fffffff;
    FlowJob j;
    j.base[1] = j.base[2] = nullptr;
    j.seg1 = j.seg2 = kNone;
    j.ids = nullptr;
    j.paired = 0;
    j.pair_rounds = j.rem = 0;
    j.nw = nw;
    switch (ph) {
    case FL_PROJH: j.base[0] = p.w_proj; j.pitch = 2 * p.d; j.K = p.d; j.rows = p.d; break;
    case FL_PROJE: j.base[0] = p.w_proj + p.d; j.pitch = 2 * p.d; j.K = p.d; j.rows = p.d; break;
    case FL_QKV:
        j.base[0] = p.w_q; j.base[1] = p.w_k; j.base[2] = p.w_v;
        j.seg1 = p.qd; j.seg2 = p.qd + p.kvd;
        j.pitch = p.d; j.K = p.d; j.rows = p.qkv_dim;
        break;
    case FL_O: j.base[0] = p.w_o; j.pitch = p.qd; j.K = p.qd; j.rows = p.d; break;
    case FL_GATEUP:
        j.base[0] = p.w_gate; j.base[1] = p.w_up;
        j.pitch = p.d; j.K = p.d; j.rows = 2 * p.F;
        j.paired = 1; j.pair_rounds = p.F / nw; j.rem = p.F % nw;
        break;
    case FL_DOWN: j.base[0] = p.w_down; j.pitch = p.F; j.K = p.F; j.rows = p.d; break;
    default: j.base[0] = p.lm_head; j.ids = p.ids; j.pitch = p.d; j.K = p.d; j.rows = p.n; break;
    }
    return j;
}

// a wave's share of a job: rows wr0, wr0 + nw, ...; chunks of eight 1 KiB loads, a chunk never straddles rows; the
// chunk count is padded to an odd number of at least three (a phase's first three chunks sit in register slot 0,
// register slot 1 and the LDS slot, the rest alternate between the register slots)
struct FlowGeom {
    int nblk, cpr, nrows, nreal, nchunks, wr_last;
};
__device__ __forceinline__ FlowGeom flow_geom(const FlowJob &j, int wr0, int nw) {
    FlowGeom g;
    g.nblk = (j.K + 511) / 512;
    g.cpr = (g.nblk + kChunkLoads - 1) / kChunkLoads;
    g.nrows = wr0 < j.rows ? (j.rows - wr0 + nw - 1) / nw : 0;
    g.nreal = g.nrows * g.cpr;
    g.nchunks = max(3, g.nreal | 1);
    g.wr_last = wr0 + max(g.nrows - 1, 0) * nw;
    return g;
}

// load cursor of a wave: which job it is requesting chunks of, and where in the wave's share it stands
struct FlowLoad {
    FlowJob j;
    FlowGeom g;
    int id;           // FlowPhase the cursor is in
    int row, jr, c, n; // next chunk: virtual row, its round, chunk within the row, chunks requested so far
    int rid;           // id-list entry of `row` (requested when the cursor moved there, used at the next request)
};
__device__ __forceinline__ void flow_load_begin(FlowLoad &L, const FlowJob &j, const FlowGeom &g, int id, int wr0) {
    L.j = j;
    L.g = g;
    L.id = id;
    L.row = wr0;
    L.jr = 0;
    L.c = 0;
    L.n = 0;
    L.rid = j.row_id(wr0);
}
// Request the cursor's next chunk into a ring slot.  Past the wave's last chunk (padding, or no next phase) the
// request goes to a zero-length buffer: it returns zeros and moves no data, so the ring is refilled without a branch
// around any load and the compiler can count the loads in flight.
__device__ __forceinline__ void flow_issue(FlowLoad &L, u32x4 (&buf)[kChunkLoads], int lane) {
    const bool live = L.n < L.g.nreal;
    const int v = live ? min(L.row, L.g.wr_last) : 0;
    const int jr = live ? L.jr : 0;
    const row_rsrc rs = make_row_rsrc(L.j.rowptr(v, jr, L.rid), live ? L.j.K * 2 : 0); // wave-uniform
    // The block's offset travels in the per-lane offset, which the buffer's range check covers: whatever lies beyond the
    // row (the tail of its last block, the empty slots of its last chunk) reads as zeros and moves no data.
    const int voff = lane * 16 + L.c * (kChunkLoads * 1024);
#pragma unroll
    for (int u = 0; u < kChunkLoads; ++u) buf[u] = row_load16<true>(rs, voff + u * 1024, 0);
    ++L.n;
    if (++L.c == L.g.cpr) {
        L.c = 0;
        L.row += L.j.nw;
        ++L.jr;
        L.rid = L.j.row_id(L.row);
    }
}

// The same request into the wave's LDS slot (8 KiB: eight loads of 1 KiB, each lane's 16 bytes where a register load
// would have put them).  The compiler counts these loads like the others but does not wait for them before LDS reads:
// the reader does (flow_wait_lds_slot).
constexpr int kLdsSlotBytes = kChunkLoads * 1024;
__device__ __forceinline__ void flow_issue_lds(FlowLoad &L, char *slot, int lane) {
    const bool live = L.n < L.g.nreal;
    const int v = live ? min(L.row, L.g.wr_last) : 0;
    const int jr = live ? L.jr : 0;
    const row_rsrc rs = make_row_rsrc(L.j.rowptr(v, jr, L.rid), live ? L.j.K * 2 : 0); // wave-uniform
    const int voff = lane * 16 + L.c * (kChunkLoads * 1024);
#pragma unroll
    for (int u = 0; u < kChunkLoads; ++u)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void *)(slot + u * 1024), 16,
                                                 voff + u * 1024, 0, 0, 2);
    ++L.n;
    if (++L.c == L.g.cpr) {
        L.c = 0;
        L.row += L.j.nw;
        ++L.jr;
        L.rid = L.j.row_id(L.row);
    }
}
// The LDS slot's chunk was requested before the two register chunks that follow it in the stream (sixteen loads) and
// loads complete in order: once at most sixteen requests are outstanding it has landed.
__device__ __forceinline__ void flow_wait_lds_slot() { asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); }

// ---- polling -----------------------------------------------------------------------------------------------
__device__ __forceinline__ row_rsrc make_vec_rsrc(const void *base, size_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
// 16 bytes past this compute die's caches (device scope); offsets beyond the buffer read zeros
__device__ __forceinline__ u32x4 ld_coherent16(row_rsrc rs, int byte_off) {
    return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, byte_off, 0, 16));
}
// two tagged elements per 16 bytes: (value, tag, value, tag)
__device__ __forceinline__ bool tags_ok(u32x4 w, unsigned tag) { return w.y == tag && w.w == tag; }

// This thread's elements e = (it * kBlock + tid) * 4 .. + 3 < n of a tagged vector (n a multiple of 4), polled until
// all of them carry `tag`.  NIT * kBlock * 4 >= n.
template <int NIT>
__device__ __forceinline__ void poll_vec(const DraftParams &p, const unsigned long long *src, int n, unsigned tag,
                                         float (&v)[NIT][4]) {
    const row_rsrc rs = make_vec_rsrc(src, (size_t)n * 8);
    PollClock clk;
    for (;;) {
        u32x4 w[NIT][2];
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int e = (it * kBlock + (int)threadIdx.x) * 4;
            w[it][0] = ld_coherent16(rs, e * 8); // beyond n: zeros, not checked
            w[it][1] = ld_coherent16(rs, e * 8 + 16);
        }
        bool ok = true;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int e = (it * kBlock + (int)threadIdx.x) * 4;
            if (e < n) ok = ok && tags_ok(w[it][0], tag) && tags_ok(w[it][1], tag);
            v[it][0] = __uint_as_float(w[it][0].x);
            v[it][1] = __uint_as_float(w[it][0].z);
            v[it][2] = __uint_as_float(w[it][1].x);
            v[it][3] = __uint_as_float(w[it][1].z);
        }
        if (ok || clk.expired(p)) break;
    }
}

// four consecutive tagged elements at each of two places, polled together
__device__ __forceinline__ void poll4x2(const DraftParams &p, row_rsrc rs, int a_byte, int b_byte, unsigned tag,
                                        float (&va)[4], float (&vb)[4]) {
    PollClock clk;
    for (;;) {
        const u32x4 a0 = ld_coherent16(rs, a_byte), a1 = ld_coherent16(rs, a_byte + 16), b0 = ld_coherent16(rs, b_byte),
                    b1 = ld_coherent16(rs, b_byte + 16);
        va[0] = __uint_as_float(a0.x);
        va[1] = __uint_as_float(a0.z);
        va[2] = __uint_as_float(a1.x);
        va[3] = __uint_as_float(a1.z);
        vb[0] = __uint_as_float(b0.x);
        vb[1] = __uint_as_float(b0.z);
        vb[2] = __uint_as_float(b1.x);
        vb[3] = __uint_as_float(b1.z);
        if ((tags_ok(a0, tag) && tags_ok(a1, tag) && tags_ok(b0, tag) && tags_ok(b1, tag)) || clk.expired(p)) break;
    }
}

// Workgroup barrier of this kernel: the wave's own LDS reads and writes have completed, nothing else is waited for.
// (A fence on LDS would also wait for the chunk that is on its way INTO the LDS slot, i.e. for every load in flight.)
__device__ __forceinline__ void flow_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// workgroup sum whose barriers order LDS traffic only (weight chunks stay in flight); red holds kWaves floats
__device__ __forceinline__ float block_sum_lds(float x, float *red) {
    x = wave_sum(x);
    flow_barrier();
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = x;
    flow_barrier();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) t += red[w];
    return t;
}
__device__ __forceinline__ unsigned long long block_max_u64_lds(unsigned long long v, unsigned long long *red64) {
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        unsigned long long o = __shfl_xor(v, off, kWave);
        v = o > v ? o : v;
    }
    flow_barrier();
    if ((threadIdx.x & (kWave - 1)) == 0) red64[threadIdx.x / kWave] = v;
    flow_barrier();
    unsigned long long r = 0ull;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) r = red64[w] > r ? red64[w] : r;
    return r;
}

// RMSNorm(u; gain) of the values this thread holds (v[it][q] = element (it * kBlock + tid) * 4 + q of a d-vector, gq[it]
// the four bf16 gains of the same elements) into hi/lo.  keep_raw (LDS, optional) receives u itself, keep_norm (LDS, optional) and out_global (optional) the result.
__device__ __forceinline__ void flow_norm(float (&v)[kMaxNormIter][4], const u32x2 (&gq)[kMaxNormIter], int d, int kpad, float eps,
                                          uint16_t *hi, uint16_t *lo, float *red, float *keep_raw, float *keep_norm,
                                          float *out_global) {
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < kMaxNormIter; ++it) {
        const int e = (it * kBlock + (int)threadIdx.x) * 4;
        if (e < d) {
#pragma unroll
            for (int q = 0; q < 4; ++q) ss += v[it][q] * v[it][q];
            if (keep_raw) *reinterpret_cast<f32x4 *>(keep_raw + e) = f32x4{v[it][0], v[it][1], v[it][2], v[it][3]};
        }
    }
    const float tot = block_sum_lds(ss, red);
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
    for (int it = 0; it < kMaxNormIter; ++it) {
        const int e = (it * kBlock + (int)threadIdx.x) * 4;
        if (e < d) {
            const u32x2 g = gq[it];
            float o[4];
            o[0] = lo_half(g.x) * (v[it][0] * inv);
            o[1] = hi_half(g.x) * (v[it][1] * inv);
            o[2] = lo_half(g.y) * (v[it][2] * inv);
            o[3] = hi_half(g.y) * (v[it][3] * inv);
            uint16_t h[4], l[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) split_bf16(o[q], h[q], l[q]);
            *reinterpret_cast<u32x2 *>(hi + e) =
                u32x2{(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
            *reinterpret_cast<u32x2 *>(lo + e) =
                u32x2{(uint32_t)l[0] | ((uint32_t)l[1] << 16), (uint32_t)l[2] | ((uint32_t)l[3] << 16)};
            const f32x4 w = {o[0], o[1], o[2], o[3]};
            if (keep_norm) *reinterpret_cast<f32x4 *>(keep_norm + e) = w;
            if (out_global) *reinterpret_cast<f32x4 *>(out_global + e) = w;
        } else if (e < kpad) { // the tail of the last 512-element block
            *reinterpret_cast<u32x2 *>(hi + e) = u32x2{0u, 0u};
            *reinterpret_cast<u32x2 *>(lo + e) = u32x2{0u, 0u};
        }
    }
}

// four floats of this thread -> hi/lo at element e
__device__ __forceinline__ void flow_split4(const float (&m)[4], uint16_t *hi, uint16_t *lo, int e) {
    uint16_t h[4], l[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) split_bf16(m[q], h[q], l[q]);
    *reinterpret_cast<u32x2 *>(hi + e) = u32x2{(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
    *reinterpret_cast<u32x2 *>(lo + e) = u32x2{(uint32_t)l[0] | ((uint32_t)l[1] << 16), (uint32_t)l[2] | ((uint32_t)l[3] << 16)};
}

__device__ __forceinline__ float silu_mul(float g, float u) { return (g / (1.0f + expf(-g))) * u; }

// LDS of the kernel: [activations hi/lo of the widest phase | attention scratch] then the residual stream (d floats),
// the wave-private strips of the projection's first half, and reduction scratch
__host__ __device__ inline size_t flow_part_floats(int d, int nvb) { return (size_t)kWaves * ((d + nvb * kWaves - 1) / (nvb * kWaves)) + 8; }
// bytes behind the shared region: the waves' LDS chunk slots, the residual stream, the projection's strips, scratch
__host__ __device__ inline size_t flow_tail_bytes(int d, int nvb) {
    return (size_t)kWaves * kLdsSlotBytes + ((size_t)d + flow_part_floats(d, nvb)) * 4 + 256;
}

// ---------------------------------------------------------------------------------------------------
// the kernel body
// ---------------------------------------------------------------------------------------------------
template <int G, int HD>
__device__ __forceinline__ void flow_steps(const DraftParams &p, char *smem) {
    const int vb = blockIdx.x, nvb = gridDim.x, d = p.d, F = p.F;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    const int nw = nvb * kWaves, wr0 = vb * kWaves + wave;
    char *slot = smem + p.fused_gemv_bytes + (size_t)wave * kLdsSlotBytes; // this wave's third chunk slot
    float *resid = reinterpret_cast<float *>(smem + p.fused_gemv_bytes + (size_t)kWaves * kLdsSlotBytes); // x, x1 = x + o,
                                                                           // then the step's output state
    const int part_rows = (d + nw - 1) / nw;                             // rows of the projection per wave
    float *ppart = resid + d + (size_t)wave * part_rows;                 // this wave's first-half sums
    unsigned long long *red64 = reinterpret_cast<unsigned long long *>(resid + d + flow_part_floats(d, nvb));
    float *red = reinterpret_cast<float *>(red64 + kWaves);

    auto stamp = [&](int step, int sec, int pt) {
        if (p.trace && threadIdx.x == 0)
            p.trace[(((size_t)step * kTraceSections + sec) * kTracePoints + pt) * nvb + vb] = wall_clock64();
    };
    if (vb == 0 && threadIdx.x == 0 && seq_dead(p, 0)) atomicOr(p.err, kErrKvOverflow);

    // winner of the output head of `step`: maximum over the workgroups' candidates, as a token id (all threads; barriers)
    auto winner = [&](int step) {
        const unsigned tag = step_tag(p, step, TS_CAND);
        const row_rsrc rs = make_vec_rsrc(p.candt + (size_t)step * p.head_grid * 2, (size_t)nvb * 16);
        unsigned long long best = 0ull;
        for (int w = threadIdx.x; w < nvb; w += kBlock) {
            u32x4 c;
            PollClock clk;
            do {
                c = ld_coherent16(rs, w * 16);
            } while (!tags_ok(c, tag) && !clk.expired(p));
            const unsigned long long key = ((unsigned long long)c.x << 32) | (unsigned long long)(0xffffffffu - c.z);
            best = key > best ? key : best;
        }
        best = block_max_u64_lds(best, red64);
        unsigned id = 0xffffffffu - (unsigned)best;
        if (id >= (unsigned)p.V) id = 0; // no workgroup had a candidate (cannot happen with n >= 1), or the wait gave up
        return (int)id;
    };

    u32x4 ring[2][kChunkLoads];
    FlowLoad L;
    L.id = FL_NONE;
    bool slot_late = false; // the LDS slot's chunk of the phase that begins has not been requested yet

    for (int step = 0; step < p.K; ++step) {
#pragma unroll 1
        for (int ph = FL_PROJH; ph <= FL_HEAD; ++ph) {
            const FlowJob job = flow_job(p, ph, nw);
            const FlowGeom g = flow_geom(job, wr0, nw);
            const int kpad = flow_kpad(job.K);
            uint16_t *act_hi = reinterpret_cast<uint16_t *>(smem), *act_lo = act_hi + kpad;
            const int sec = ph == FL_PROJH ? 7 : ph == FL_PROJE ? 0 : ph == FL_QKV ? 1 : ph + 0; // O..HEAD are 3..6
            if (L.id != ph) { // first phase of the call, or the phase after the attention: nothing was requested ahead
                flow_load_begin(L, job, g, ph, wr0);
                flow_issue(L, ring[0], lane);
                flow_issue(L, ring[1], lane);
                flow_issue_lds(L, slot, lane);
            }
            stamp(step, sec, kTraceRequested);
            flow_barrier(); // every wave has finished with the activations of the phase before

            // ---- stage this phase's input vector into LDS as bf16 hi + lo ------------------------------------------
            {
                float v[kMaxNormIter][4];
                // The gains of this phase's norm are requested before anything is polled: they do not depend on it, and a
                // load issued after the poll would add its own trip through the (busy) memory system to the hand-over.
                const uint16_t *gain = ph == FL_PROJH ? p.g_h : ph == FL_PROJE ? p.g_e : ph == FL_QKV ? p.g_attn
                                       : ph == FL_GATEUP ? p.g_mlp : p.g_final;
                u32x2 gq[kMaxNormIter];
#pragma unroll
                for (int it = 0; it < kMaxNormIter; ++it) {
                    const int e = (it * kBlock + (int)threadIdx.x) * 4;
                    gq[it] = (e < d && ph != FL_O && ph != FL_DOWN) ? *reinterpret_cast<const u32x2 *>(gain + e) : u32x2{0u, 0u};
                }
                switch (ph) {
                case FL_PROJH: {
                    if (step == 0) {
#pragma unroll
                        for (int it = 0; it < kMaxNormIter; ++it) {
                            const int e = (it * kBlock + (int)threadIdx.x) * 4;
                            if (e < d) {
                                if (!p.own_hidden) {
                                    const u32x2 raw = *reinterpret_cast<const u32x2 *>(p.hidden_in + e);
                                    v[it][0] = lo_half(raw.x);
                                    v[it][1] = hi_half(raw.x);
                                    v[it][2] = lo_half(raw.y);
                                    v[it][3] = hi_half(raw.y);
                                } else {
                                    const f32x4 raw = *reinterpret_cast<const f32x4 *>(p.hhat + e);
                                    v[it][0] = raw.x;
                                    v[it][1] = raw.y;
                                    v[it][2] = raw.z;
                                    v[it][3] = raw.w;
                                }
                            }
                        }
                    } else { // the head's own output of the step before: every workgroup kept it
#pragma unroll
                        for (int it = 0; it < kMaxNormIter; ++it) {
                            const int e = (it * kBlock + (int)threadIdx.x) * 4;
                            if (e < d) {
                                const f32x4 raw = *reinterpret_cast<const f32x4 *>(resid + e);
                                v[it][0] = raw.x;
                                v[it][1] = raw.y;
                                v[it][2] = raw.z;
                                v[it][3] = raw.w;
                            }
                        }
                    }
                    stamp(step, sec, kTraceReleased);
                    flow_norm(v, gq, d, kpad, p.eps, act_hi, act_lo, red, nullptr, nullptr, nullptr);
                    break;
                }
                case FL_PROJE: {
                    int tok;
                    if (step == 0) {
                        tok = p.token_in[0];
                    } else {
                        const int did = winner(step - 1);
                        tok = p.forced ? p.forced[step - 1] : did;
                        if (vb == 0 && threadIdx.x == 0) p.draft_out[step - 1] = seq_dead(p, 0) ? -1 : did;
                    }
                    if (tok < 0 || tok >= p.V) { // reported, and replaced by id 0 so that every access stays in bounds
                        if (threadIdx.x == 0) atomicOr(p.err, kErrTokenRange);
                        tok = 0;
                    }
                    stamp(step, sec, kTraceReleased);
                    const uint16_t *src = p.embed + (size_t)tok * d;
#pragma unroll
                    for (int it = 0; it < kMaxNormIter; ++it) {
                        const int e = (it * kBlock + (int)threadIdx.x) * 4;
                        if (e < d) {
                            const u32x2 raw = *reinterpret_cast<const u32x2 *>(src + e);
                            v[it][0] = lo_half(raw.x);
                            v[it][1] = hi_half(raw.x);
                            v[it][2] = lo_half(raw.y);
                            v[it][3] = hi_half(raw.y);
                        }
                    }
                    flow_norm(v, gq, d, kpad, p.eps, act_hi, act_lo, red, nullptr, nullptr, nullptr);
                    break;
                }
                case FL_QKV:
                    poll_vec<kMaxNormIter>(p, p.xt, d, step_tag(p, step, TS_X), v);
                    stamp(step, sec, kTraceReleased);
                    flow_norm(v, gq, d, kpad, p.eps, act_hi, act_lo, red, resid, nullptr, nullptr);
                    break;
                case FL_GATEUP: { // x1 = x + w_o a
                    poll_vec<kMaxNormIter>(p, p.ot, d, step_tag(p, step, TS_O), v);
                    stamp(step, sec, kTraceReleased);
#pragma unroll
                    for (int it = 0; it < kMaxNormIter; ++it) {
                        const int e = (it * kBlock + (int)threadIdx.x) * 4;
                        if (e < d) {
                            const f32x4 r = *reinterpret_cast<const f32x4 *>(resid + e);
                            v[it][0] = r.x + v[it][0];
                            v[it][1] = r.y + v[it][1];
                            v[it][2] = r.z + v[it][2];
                            v[it][3] = r.w + v[it][3];
                        }
                    }
                    flow_norm(v, gq, d, kpad, p.eps, act_hi, act_lo, red, resid, nullptr, nullptr);
                    break;
                }
                case FL_HEAD: { // x2 = x1 + w_down m; the step's output hidden state
                    poll_vec<kMaxNormIter>(p, p.dnt, d, step_tag(p, step, TS_DN), v);
                    stamp(step, sec, kTraceReleased);
#pragma unroll
                    for (int it = 0; it < kMaxNormIter; ++it) {
                        const int e = (it * kBlock + (int)threadIdx.x) * 4;
                        if (e < d) {
                            const f32x4 r = *reinterpret_cast<const f32x4 *>(resid + e);
                            v[it][0] = r.x + v[it][0];
                            v[it][1] = r.y + v[it][1];
                            v[it][2] = r.z + v[it][2];
                            v[it][3] = r.w + v[it][3];
                        }
                    }
                    float *ho = (vb == 0 && p.hidden_out) ? p.hidden_out + (size_t)step * d : nullptr;
                    flow_norm(v, gq, d, kpad, p.eps, act_hi, act_lo, red, nullptr, resid, ho);
                    break;
                }
                case FL_O: { // the attention's result, as it is
                    const int n = p.qd;
                    const unsigned tag = step_tag(p, step, TS_ATTN);
                    for (int e0 = 0; e0 < kpad; e0 += kMaxNormIter * kBlock * 4) {
                        poll_vec<kMaxNormIter>(p, p.attnt + e0, max(min(n - e0, kMaxNormIter * kBlock * 4), 0), tag, v);
#pragma unroll
                        for (int it = 0; it < kMaxNormIter; ++it) {
                            const int e = e0 + (it * kBlock + (int)threadIdx.x) * 4;
                            if (e < kpad) {
                                const float z[4] = {0.f, 0.f, 0.f, 0.f};
                                flow_split4(e < n ? v[it] : z, act_hi, act_lo, e);
                            }
                        }
                    }
                    stamp(step, sec, kTraceReleased);
                    break;
                }
                default: { // FL_DOWN: m = silu(gate) * up: formed by the producers except for the rows dealt singly
                    const int pn = (F / nw) * nw, rem = F - pn; // pairs, then rem gate values, then rem up values
                    const unsigned tag = step_tag(p, step, TS_GU);
                    const row_rsrc gu_rs = make_vec_rsrc(p.gut, (size_t)(F + rem) * 8);
                    for (int e0 = 0; e0 < kpad; e0 += kMaxNormIter * kBlock * 4) {
                        poll_vec<kMaxNormIter>(p, p.gut + e0, max(min(pn - e0, kMaxNormIter * kBlock * 4), 0), tag, v);
#pragma unroll
                        for (int it = 0; it < kMaxNormIter; ++it) {
                            const int e = e0 + (it * kBlock + (int)threadIdx.x) * 4;
                            if (e < kpad) {
                                float m[4] = {0.f, 0.f, 0.f, 0.f};
                                if (e < pn) {
#pragma unroll
                                    for (int q = 0; q < 4; ++q) m[q] = v[it][q];
                                } else if (e < F) { // a group of four never straddles: pn, rem and F are multiples of 8
                                    float gt[4], up[4];
                                    poll4x2(p, gu_rs, e * 8, (e + rem) * 8, tag, gt, up);
#pragma unroll
                                    for (int q = 0; q < 4; ++q) m[q] = silu_mul(gt[q], up[q]);
                                }
                                flow_split4(m, act_hi, act_lo, e);
                            }
                        }
                    }
                    stamp(step, sec, kTraceReleased);
                    break;
                }
                }
            }
            if (slot_late) { // the third chunk requested ahead for this phase (see the end of a phase)
                flow_issue_lds(L, slot, lane);
                slot_late = false;
            }
            flow_barrier();
            stamp(step, sec, kTraceStaged);

            // ---- stream this wave's rows --------------------------------------------------------------------------
            const int next = ph == FL_QKV ? FL_NONE : ph == FL_HEAD ? (step + 1 < p.K ? FL_PROJH : FL_NONE) : ph + 1;
            const unsigned out_tag = step_tag(p, step, ph == FL_PROJE ? TS_X : ph == FL_QKV ? TS_QKV : ph == FL_O ? TS_O
                                                       : ph == FL_GATEUP ? TS_GU : TS_DN);
            unsigned long long *out_t = ph == FL_PROJE ? p.xt : ph == FL_QKV ? p.qkvt : ph == FL_O ? p.ot
                                        : ph == FL_GATEUP ? p.gut : ph == FL_DOWN ? p.dnt : nullptr;
            float *logits = (ph == FL_HEAD && p.logits_out) ? p.logits_out + (size_t)step * p.n : nullptr;
            unsigned long long best = 0ull; // output head: best (logit, row) this wave has seen (lane 0)
            float gate_saved = 0.f;
            const int pair_rows = 2 * job.pair_rounds;
            const bool throttle = g.nchunks >= 8;

            f32x4 acc_h = {0.f, 0.f, 0.f, 0.f}, acc_l = {0.f, 0.f, 0.f, 0.f};
            const int dv = (lane & 15) - 4 * (lane >> 4); // which of this lane's four results lies on the diagonal
            int c_row = wr0, c_j = 0, c_c = 0;
            // one chunk: eight blocks of the row against the staged activations; w(u) = the chunk's u-th 1 KiB
            auto consume = [&](auto w) {
#pragma unroll
                for (int u = 0; u < kChunkLoads; ++u) {
                    // slots past the row's last block hold zero weights: they re-read the last block's activations
                    const int e0 = min(c_c * kChunkLoads + u, g.nblk - 1) * 512 + lane * 8;
                    const u32x4 ah = *reinterpret_cast<const u32x4 *>(act_hi + e0);
                    const u32x4 al = *reinterpret_cast<const u32x4 *>(act_lo + e0);
                    const u32x4 wv = w(u);
                    acc_h = mfma16(ah, wv, acc_h);
                    acc_l = mfma16(al, wv, acc_l);
                }
            };
            // the cursor moves on to the phase that follows once this phase's share is exhausted
            auto advance_cursor = [&]() {
                if (L.n >= L.g.nchunks && L.id == ph && next != FL_NONE) {
                    const FlowJob nj = flow_job(p, next, nw);
                    flow_load_begin(L, nj, flow_geom(nj, wr0, nw), next, wr0);
                }
            };
            auto row_end = [&](int n) {
                if (n < g.nreal && ++c_c == g.cpr) { // end of a row: sum the diagonal
                    c_c = 0;
                    const f32x4 t = acc_h + acc_l;
                    float val = dv == 0 ? t.x : dv == 1 ? t.y : dv == 2 ? t.z : dv == 3 ? t.w : 0.f;
                    val = wave_sum(val);
                    acc_h = f32x4{0.f, 0.f, 0.f, 0.f};
                    acc_l = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (lane == 0) {
                        const int li = c_j; // this wave's c_j-th row
                        switch (ph) {
                        case FL_PROJH: ppart[li] = val; break;
                        case FL_PROJE: st_tagged(out_t + c_row, ppart[li] + val, out_tag); break;
                        case FL_GATEUP: {
                            const int w = c_row - c_j * nw;
                            if (c_j < pair_rows) {
                                if ((c_j & 1) == 0)
                                    gate_saved = val;
                                else
                                    st_tagged(out_t + (c_j >> 1) * nw + w, silu_mul(gate_saved, val), out_tag);
                            } else { // dealt singly: gate values, then up values, behind the pairs
                                st_tagged(out_t + job.pair_rounds * nw + w, val, out_tag);
                            }
                            break;
                        }
                        case FL_HEAD: {
                            if (logits) logits[c_row] = val;
                            const unsigned long long key = argmax_key(val, (uint32_t)c_row);
                            best = key > best ? key : best;
                            break;
                        }
                        default: st_tagged(out_t + c_row, val, out_tag); break;
                        }
                    }
                    c_row += nw;
                    ++c_j;
                }
            };
            // Chunks n0 and n0 + 1 sit in the register slots; the phase's third chunk sits in the LDS slot and is taken
            // after the first two.  Every register slot is refilled as soon as it is free; the LDS slot is refilled once,
            // at the end of the phase, with the third chunk of the phase that follows.
            int pend = 0; // register slots whose refill waits for the end of the phase
            for (int n0 = 0; n0 < g.nchunks; n0 += (n0 == 0 ? 3 : 2)) {
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    consume([&](int u) { return ring[s][u]; });
                    advance_cursor();
                    // Long phases keep ONE chunk in flight per wave while they stream (the other slot's loads are waited
                    // for before the next request goes out): 16 MiB over the chip already covers the memory latency, more
                    // only deepens the queues, and the compute dies then share the bandwidth unevenly (output head: the
                    // odd-numbered dies finished 6 us after the even ones with two chunks in flight).  The other slots
                    // earn their keep at the ends of a phase, where the requests run ahead into the next one.
                    // The phase's last chunks (the cursor has moved on to the phase that follows): the row's result goes
                    // out first, and the slot's next request waits until the wave has published all its results.  A
                    // request can wait a microsecond for room in the memory queues, and other workgroups poll for
                    // these results.
                    if (L.id != ph) {
                        row_end(n0 + s);
                        pend |= 1 << s;
                    } else {
                        if (throttle) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                        flow_issue(L, ring[s], lane);
                        row_end(n0 + s);
                    }
                }
                if (n0 == 0) {
                    flow_wait_lds_slot();
                    consume([&](int u) { return *reinterpret_cast<const u32x4 *>(slot + u * 1024 + lane * 16); });
                    row_end(2);
                }
            }
            if (pend & 1) flow_issue(L, ring[0], lane);
            if (pend & 2) flow_issue(L, ring[1], lane);
            // The LDS slot's chunk of the next phase is requested by that phase, behind its polls (a wave's loads
            // complete in order, and a poll behind three chunks per wave returns 2 us later than behind two; with one
            // chunk or none in front of them the polls gain less than the memory system loses: 141.7 and 149.5 us per
            // step against 137.4).
            if (next != FL_NONE) { // (no next phase: nothing is written into LDS that the attention may be using)
                advance_cursor();
                slot_late = true;
            }
            if (ph == FL_HEAD) {
                // the workgroup's candidate: (logit, token id), each with the tag in its upper half
                const unsigned long long m = block_max_u64_lds(best, red64);
                if (threadIdx.x == 0) {
                    unsigned lg = 0u, id = 0xffffffffu; // no row in this workgroup: loses against every candidate
                    if (m != 0ull) {
                        const uint32_t row = key_index(m);
                        lg = (unsigned)(m >> 32);
                        id = p.ids ? (unsigned)p.ids[row] : row;
                    }
                    const unsigned tag = step_tag(p, step, TS_CAND);
                    unsigned long long *c = p.candt + ((size_t)step * p.head_grid + vb) * 2;
                    __hip_atomic_store(c, ((unsigned long long)tag << 32) | lg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(c + 1, ((unsigned long long)tag << 32) | id, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            stamp(step, sec, kTraceDone);
            if (ph == FL_QKV) { // attention: polls q, k, v itself and publishes its result as tagged elements
                stamp(step, 2, kTraceRequested);
                flow_barrier(); // the activations' LDS becomes the attention's
                stamp(step, 2, kTraceReleased);
                stamp(step, 2, kTraceStaged);
                call_attn<G, HD, true, true, true, kFlowAttnParts<G>>(p, step, vb, nvb, smem);
                stamp(step, 2, kTraceDone);
            }
        }
    }
    // publish the last draft id
    if (vb == 0) {
        flow_barrier();
        const int did = winner(p.K - 1);
        if (threadIdx.x == 0) p.draft_out[p.K - 1] = seq_dead(p, 0) ? -1 : did;
    }
}

} // namespace mtp
