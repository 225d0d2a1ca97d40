// Single-launch path: all phases of all K draft steps in one cooperative kernel (gfx950).
//
// Why it exists: at batch 1 a draft step is seven dependent matrix-vector products of 30-270 MB each.  A kernel
// boundary (or a grid barrier) costs several microseconds during which HBM idles, which is a large fraction of
// a phase that itself lasts 5-40 us.  Here every wave keeps a ring of weight chunks in registers; the first
// chunks of the NEXT phase are requested right after the wave has signalled the end of the current phase, so
// the memory system stays busy while the grid barrier completes and the new activations are staged.
//
// The barrier itself uses relaxed device-scope atomics only.  A release/acquire pair at device scope writes back
// and invalidates whole caches (each compute die has its own L2): measured 6 us per barrier idle and 15 us on top
// of a streaming phase, against 1.7 us and 5 us for the relaxed one.  What crosses a barrier - a few activation
// vectors, the argmax candidates, the appended cache entries, the attention partials - is instead written and read
// with device-coherent accesses (the <true> variants of the staging helpers and of ld_/st_ in device_utils.h),
// access by access; weights and the older part of the KV cache are read-only inside the kernel and go through the
// caches as usual.  An appended cache entry is written coherently by the one workgroup that owns it and read by
// ordinary loads afterwards: no cache can hold an older copy of a slot that this call has not read before.
#pragma once
#include "phases.h"

#ifndef FUSED_ATTN_CALL
#define FUSED_ATTN_CALL(p, step, vb, nvb, smem) call_attn<G, HD, true, true>(p, step, vb, nvb, smem)
#endif

namespace mtp {

constexpr int kBarriersPerStep = 7;

// ---------------------------------------------------------------------------------------------------
// split-phase grid barrier on a two-level tree of counters that only grow
// ---------------------------------------------------------------------------------------------------
// Workgroups are dealt to kBarGroups groups (blockIdx % kBarGroups, which follows the round-robin placement on
// the eight XCDs).  The last arrival of a group bumps the root; the last group publishes the barrier number in one
// flag per group, which the group's workgroups poll.  Same-address atomics are executed one after another at the
// memory side (~40 ns each), so the tree costs ~40 instead of ~256 serialized operations.
constexpr int kBarGroups = 8;
constexpr int kBarStride = 32; // 64-bit words between counters: one 256-byte line each
// layout of p.bar: [0] root, [kBarStride * (1 + g)] group counters, [kBarStride * (1 + kBarGroups + g)] flags
constexpr size_t kBarWords = (size_t)kBarStride * (1 + 2 * kBarGroups);

__device__ __forceinline__ void bar_arrive(const DraftParams &p, unsigned epoch) {
    // Each wave waits until its own device-coherent stores have been acknowledged, then the workgroup meets: the
    // workgroup barrier by itself orders accesses inside the CU only and need not wait for stores still in flight.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const int g = blockIdx.x % kBarGroups;
        const int gsize = ((int)gridDim.x - g + kBarGroups - 1) / kBarGroups;
        const unsigned long long e = p.bar_base + epoch; // barriers completed since the workspace was zeroed
        unsigned long long old =
            __hip_atomic_fetch_add(p.bar + kBarStride * (1 + g), 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old + 1 == e * (unsigned long long)gsize) {
            old = __hip_atomic_fetch_add(p.bar, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (old + 1 == e * (unsigned long long)kBarGroups) {
#pragma unroll
                for (int i = 0; i < kBarGroups; ++i)
                    __hip_atomic_store(p.bar + kBarStride * (1 + kBarGroups + i), e, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// Returns after barrier `epoch` has completed, or after the time limit (then the sticky error word is set and
// every later wait of every workgroup falls through, so the grid always drains).
__device__ __forceinline__ void bar_wait(const DraftParams &p, unsigned epoch) {
    if (threadIdx.x == 0) {
        const int g = blockIdx.x % kBarGroups;
        const unsigned long long e = p.bar_base + epoch;
        unsigned long long *flag = p.bar + kBarStride * (1 + kBarGroups + g);
        const long long t0 = wall_clock64();
        unsigned spins = 0;
        while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < e) {
            if ((++spins & 63u) == 0) {
                if (__hip_atomic_load(p.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kErrBarrierTimeout) break;
                if (wall_clock64() - t0 > p.bar_timeout) {
                    atomicOr(p.err, kErrBarrierTimeout);
                    break;
                }
            }
        }
    }
    lds_barrier(); // the other waves need not wait for their own prefetch here; also a compiler fence
}

template <int NMAT>
__device__ __forceinline__ GemvGeom gemv_geom(int K, int rows, int vb, int nvb) {
    int r0, r1;
    row_share(rows, vb, nvb, r0, r1);
    return gemv_geom_rows<NMAT>(K, r0, r1);
}

// LDS of the single-launch path: the matrix-vector region (reused by the attention phases), then the id strip of
// the compressed head, then small reduction scratch.
__host__ __device__ inline size_t fused_gemv_region(int d, int qd, int F, int nb) {
    size_t m = gemv_lds_bytes(2 * d, nb, 1);
    size_t a = gemv_lds_bytes(d, nb, 2), b = gemv_lds_bytes(qd, nb, 1), c = gemv_lds_bytes(F, nb, 1);
    m = a > m ? a : m;
    m = b > m ? b : m;
    m = c > m ? c : m;
    return (m + 255) / 256 * 256;
}

// ---- the six matrix-vector phases: row pointers, priming and running --------------------------------------
// Geometry is recomputed where it is needed (a few scalar instructions) instead of being kept live across phases.
struct RpProj {
    const DraftParams &p;
    __device__ __forceinline__ const uint16_t *operator()(int, int row) const { return p.w_proj + (size_t)row * 2 * p.d; }
};
struct RpQkv {
    const DraftParams &p;
    __device__ __forceinline__ const uint16_t *operator()(int, int row) const {
        if (row < p.qd) return p.w_q + (size_t)row * p.d;
        if (row < p.qd + p.kvd) return p.w_k + (size_t)(row - p.qd) * p.d;
        return p.w_v + (size_t)(row - p.qd - p.kvd) * p.d;
    }
};
struct RpO {
    const DraftParams &p;
    __device__ __forceinline__ const uint16_t *operator()(int, int row) const { return p.w_o + (size_t)row * p.qd; }
};
struct RpGateUp { // rows 0..F-1 are w_gate's, F..2F-1 w_up's
    const DraftParams &p;
    __device__ __forceinline__ const uint16_t *operator()(int, int row) const {
        return row < p.F ? p.w_gate + (size_t)row * p.d : p.w_up + (size_t)(row - p.F) * p.d;
    }
};
struct RpDown {
    const DraftParams &p;
    __device__ __forceinline__ const uint16_t *operator()(int, int row) const { return p.w_down + (size_t)row * p.F; }
};
struct RpHead { // compressed head: the workgroup's strip of the id list sits in LDS (copied once per call)
    const DraftParams &p;
    const int *ids_lds;
    int r0;
    __device__ __forceinline__ const uint16_t *operator()(int, int row) const {
        int r = p.ids ? ids_lds[row - r0] : row;
        return p.lm_head + (size_t)r * p.d;
    }
};

enum FusedPhase : int { FP_PROJ, FP_QKV, FP_O, FP_GATEUP, FP_DOWN, FP_HEAD };

template <int PH>
__device__ __forceinline__ void fused_prime(const DraftParams &p, Ring &ring, const int *ids_lds) {
    const int vb = blockIdx.x, nvb = gridDim.x;
    if (PH == FP_PROJ) {
        gemv_prime<1>(gemv_geom<1>(2 * p.d, p.d, vb, nvb), RpProj{p}, ring);
    } else if (PH == FP_QKV) {
        gemv_prime<1>(gemv_geom<1>(p.d, p.qkv_dim, vb, nvb), RpQkv{p}, ring);
    } else if (PH == FP_O) {
        gemv_prime<1>(gemv_geom<1>(p.qd, p.d, vb, nvb), RpO{p}, ring);
    } else if (PH == FP_GATEUP) {
        gemv_prime<1>(gemv_geom<1>(p.d, 2 * p.F, vb, nvb), RpGateUp{p}, ring);
    } else if (PH == FP_DOWN) {
        gemv_prime<1>(gemv_geom<1>(p.F, p.d, vb, nvb), RpDown{p}, ring);
    } else {
        GemvGeom q = gemv_geom<1>(p.d, p.n, vb, nvb);
        gemv_prime<1>(q, RpHead{p, ids_lds, q.r0}, ring);
    }
}

// One call = K steps.  Workgroup blockIdx.x of gridDim.x; all B sequences are staged together (one pass over the
// weights per phase).
template <int G, int HD>
__device__ __forceinline__ void fused_steps2(const DraftParams &p, char *smem) {
    const int vb = blockIdx.x, nvb = gridDim.x;
    const int d = p.d, nb = p.B, nbmax = p.B;
    char *gemv_smem = smem;
    int *ids_lds = reinterpret_cast<int *>(smem + p.fused_gemv_bytes);
    unsigned long long *red64 = reinterpret_cast<unsigned long long *>(smem + p.fused_gemv_bytes + p.fused_ids_bytes);
    unsigned epoch = 0;
    Ring ring;
    int stamp_i = 0;
    auto stamp = [&](int step) {
        if (p.trace && vb == 0 && threadIdx.x == 0 && stamp_i < 16) p.trace[step * 16 + stamp_i] = wall_clock64();
        ++stamp_i;
    };
    // this workgroup's slice of the id list never changes during the call
    if (p.ids) {
        int r0, r1;
        row_share(p.n, vb, nvb, r0, r1);
        for (int i = threadIdx.x; i < r1 - r0; i += kBlock) ids_lds[i] = p.ids[r0 + i];
    }
    __syncthreads();

    fused_prime<FP_PROJ>(p, ring, ids_lds); // cold start of the call
    for (int step = 0; step < p.K; ++step) {
        stamp_i = 0;
        stamp(step);
        // ---- projection ---------------------------------------------------------------------------------
        {
            GemvLds l = gemv_lds(gemv_smem, 2 * d, nbmax, 1);
            if (step > 0) bar_wait(p, epoch); // previous step's head candidates and hidden state are visible
            for (int i = 0; i < nb; ++i) {
                int tok;
                if (step == 0) {
                    tok = p.token_in[i];
                } else {
                    // winner of the previous step: maximum over the workgroups' candidates
                    unsigned long long best = 0ull;
                    const unsigned long long *cand = p.cand + ((size_t)(step - 1) * p.max_batch + i) * nvb;
                    for (int w = threadIdx.x; w < nvb; w += kBlock) {
                        const unsigned long long c = ld_u64<true>(cand + w);
                        best = c > best ? c : best;
                    }
                    best = block_max_u64(best, red64);
                    uint32_t bi = key_index(best);
                    if (bi >= (uint32_t)p.n) bi = 0;
                    int did = p.ids ? p.ids[bi] : (int)bi;
                    tok = p.forced ? p.forced[(size_t)i * (p.K - 1) + step - 1] : did;
                    if (vb == 0 && threadIdx.x == 0) p.draft_out[(size_t)i * p.K + step - 1] = seq_dead(p, i) ? -1 : did;
                }
                if (tok < 0 || tok >= p.V) {
                    if (threadIdx.x == 0) atomicOr(p.err, kErrTokenRange);
                    tok = 0;
                }
                if (step == 0 && vb == 0 && threadIdx.x == 0 && seq_dead(p, i)) atomicOr(p.err, kErrKvOverflow);
                uint16_t *hi = l.hi + (size_t)i * l.kpad, *lo = l.lo + (size_t)i * l.kpad;
                if (step == 0 && !p.own_hidden)
                    stage_rmsnorm<true>(p.hidden_in + (size_t)i * d, p.g_h, d, p.eps, hi, lo, l.red, nullptr);
                else
                    stage_rmsnorm<false, true>(p.hhat + (size_t)i * d, p.g_h, d, p.eps, hi, lo, l.red, nullptr);
                stage_rmsnorm<true>(p.embed + (size_t)tok * d, p.g_e, d, p.eps, hi + d, lo + d, l.red, nullptr);
            }
            __syncthreads();
            auto epi = [&](int i, int row, float(&s)[1]) { st_f32<true>(p.x + (size_t)i * d + row, s[0]); };
            gemv_run<1>(gemv_geom<1>(2 * d, d, vb, nvb), RpProj{p}, ring, nb, nbmax, l.hi, l.lo, l.kpad, l.partial,
                        epi);
        }
        stamp(step);
        bar_arrive(p, ++epoch);
        fused_prime<FP_QKV>(p, ring, ids_lds);
        bar_wait(p, epoch);
        stamp(step);
        // ---- q, k, v ------------------------------------------------------------------------------------
        {
            GemvLds l = gemv_lds(gemv_smem, d, nbmax, 1);
            for (int i = 0; i < nb; ++i)
                stage_rmsnorm<false, true>(p.x + (size_t)i * d, p.g_attn, d, p.eps, l.hi + (size_t)i * l.kpad,
                                     l.lo + (size_t)i * l.kpad, l.red, nullptr);
            __syncthreads();
            auto epi = [&](int i, int row, float(&s)[1]) { st_f32<true>(p.qkv + (size_t)i * p.qkv_dim + row, s[0]); };
            gemv_run<1>(gemv_geom<1>(d, p.qkv_dim, vb, nvb), RpQkv{p}, ring, nb, nbmax, l.hi, l.lo, l.kpad,
                        l.partial, epi);
        }
        stamp(step);
        bar_arrive(p, ++epoch);
        bar_wait(p, epoch);
        stamp(step);
        // ---- attention (the ring is empty here) ----------------------------------------------------------------
        FUSED_ATTN_CALL(p, step, vb, nvb, gemv_smem);
        stamp(step);
        bar_arrive(p, ++epoch); // the splits of a long context were merged by the workgroup that finished last
        fused_prime<FP_O>(p, ring, ids_lds);
        bar_wait(p, epoch);
        stamp(step);
        // ---- output projection -------------------------------------------------------------------------------
        {
            GemvLds l = gemv_lds(gemv_smem, p.qd, nbmax, 1);
            __syncthreads();
            for (int i = 0; i < nb; ++i)
                stage_plain<true>(p.attn + (size_t)i * p.qd, p.qd, l.kpad, l.hi + (size_t)i * l.kpad,
                            l.lo + (size_t)i * l.kpad);
            __syncthreads();
            auto epi = [&](int i, int row, float(&s)[1]) { st_f32<true>(p.o + (size_t)i * d + row, s[0]); };
            gemv_run<1>(gemv_geom<1>(p.qd, d, vb, nvb), RpO{p}, ring, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, epi);
        }
        stamp(step);
        bar_arrive(p, ++epoch);
        fused_prime<FP_GATEUP>(p, ring, ids_lds);
        bar_wait(p, epoch);
        stamp(step);
        // ---- gate / up ---------------------------------------------------------------------------------------
        {
            GemvLds l = gemv_lds(gemv_smem, d, nbmax, 1);
            for (int i = 0; i < nb; ++i)
                stage_rmsnorm<false, true>(p.x + (size_t)i * d, p.g_mlp, d, p.eps, l.hi + (size_t)i * l.kpad,
                                     l.lo + (size_t)i * l.kpad, l.red, nullptr, nullptr, p.o + (size_t)i * d);
            __syncthreads();
            auto epi = [&](int i, int row, float(&s)[1]) { st_f32<true>(p.gu + (size_t)i * 2 * p.F + row, s[0]); };
            gemv_run<1>(gemv_geom<1>(d, 2 * p.F, vb, nvb), RpGateUp{p}, ring, nb, nbmax, l.hi, l.lo, l.kpad,
                        l.partial, epi);
        }
        stamp(step);
        bar_arrive(p, ++epoch);
        fused_prime<FP_DOWN>(p, ring, ids_lds);
        bar_wait(p, epoch);
        stamp(step);
        // ---- down ------------------------------------------------------------------------------------------------
        {
            GemvLds l = gemv_lds(gemv_smem, p.F, nbmax, 1);
            __syncthreads();
            for (int i = 0; i < nb; ++i)
                stage_swiglu<true>(p.gu + (size_t)i * 2 * p.F, p.F, l.kpad, l.hi + (size_t)i * l.kpad,
                             l.lo + (size_t)i * l.kpad);
            __syncthreads();
            auto epi = [&](int i, int row, float(&s)[1]) { st_f32<true>(p.dn + (size_t)i * d + row, s[0]); };
            gemv_run<1>(gemv_geom<1>(p.F, d, vb, nvb), RpDown{p}, ring, nb, nbmax, l.hi, l.lo, l.kpad, l.partial,
                        epi);
        }
        stamp(step);
        bar_arrive(p, ++epoch);
        fused_prime<FP_HEAD>(p, ring, ids_lds);
        bar_wait(p, epoch);
        stamp(step);
        // ---- final norm + compressed head + argmax candidates --------------------------------------------------
        {
            GemvLds l = gemv_lds(gemv_smem, d, nbmax, 1);
            for (int i = 0; i < nb; ++i) {
                float *hh = (vb == 0) ? p.hhat + (size_t)i * d : nullptr;
                float *ho = (vb == 0 && p.hidden_out) ? p.hidden_out + ((size_t)i * p.K + step) * d : nullptr;
                stage_rmsnorm<false, true>(p.x + (size_t)i * d, p.g_final, d, p.eps, l.hi + (size_t)i * l.kpad,
                                     l.lo + (size_t)i * l.kpad, l.red, hh, ho, p.o + (size_t)i * d,
                                     p.dn + (size_t)i * d);
            }
            __syncthreads();
            unsigned long long best = 0ull;
            auto epi = [&](int i, int row, float(&s)[1]) {
                if (p.logits_out) p.logits_out[((size_t)i * p.K + step) * p.n + row] = s[0];
                unsigned long long key = argmax_key(s[0], (uint32_t)row);
                best = key > best ? key : best;
            };
            GemvGeom q = gemv_geom<1>(d, p.n, vb, nvb);
            gemv_run<1>(q, RpHead{p, ids_lds, q.r0}, ring, nb, nbmax, l.hi, l.lo, l.kpad, l.partial, epi);
            if ((int)threadIdx.x < 16 * nb) { // threads 16*i .. 16*i+15 hold candidates of sequence i
#pragma unroll
                for (int off = 1; off < 16; off <<= 1) {
                    unsigned long long o2 = __shfl_xor(best, off, kWave);
                    best = o2 > best ? o2 : best;
                }
                if ((threadIdx.x & 15) == 0)
                    st_u64<true>(p.cand + ((size_t)step * p.max_batch + (threadIdx.x >> 4)) * nvb + vb, best);
            }
        }
        stamp(step);
        bar_arrive(p, ++epoch);
        if (step + 1 < p.K) fused_prime<FP_PROJ>(p, ring, ids_lds); // same weights at every depth
        stamp(step);
    }
    // publish the last draft id
    bar_wait(p, epoch);
    if (vb == 0) {
        for (int i = 0; i < nb; ++i) {
            unsigned long long best = 0ull;
            const unsigned long long *cand = p.cand + ((size_t)(p.K - 1) * p.max_batch + i) * nvb;
            for (int w = threadIdx.x; w < nvb; w += kBlock) {
                const unsigned long long c = ld_u64<true>(cand + w);
                best = c > best ? c : best;
            }
            best = block_max_u64(best, red64);
            uint32_t bi = key_index(best);
            if (bi >= (uint32_t)p.n) bi = 0;
            if (threadIdx.x == 0)
                p.draft_out[(size_t)i * p.K + p.K - 1] = seq_dead(p, i) ? -1 : (p.ids ? p.ids[bi] : (int)bi);
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// the same call for ONE sequence on the row-streaming core (every reduction length at least 512)
// ---------------------------------------------------------------------------------------------------
// The six matrix phases of a step run through ONE copy of the row-streaming loop: a phase is a run-time description
// (where its rows are, how long they are, where the results go) and a case of the staging switch.  That keeps the
// kernel at 40 KiB of code instead of 68 (the instruction cache is 64 KiB per two CUs; its counters show a hit rate
// above 99.9 % either way) and costs nothing measurable.
//
// gemv_rowmode requests the wave's first rows itself and then calls the staging callback, so the wait for the previous
// phase's barrier sits at the start of that callback: the weights of a phase are on their way while the grid
// synchronises.  Rows are interleaved over all waves of the grid, so the id list is read from memory (it is small and
// stays in L2) instead of from a per-workgroup strip in LDS.
struct RowJob {
    const uint16_t *base[3]; // up to three matrices stacked row-wise (q, k, v; gate, up)
    int seg1, seg2;          // first row of the second and of the third matrix
    int K, rows;
    const int *ids;          // optional row indirection (the compressed output head)
    float *out;              // results (device-coherent stores), or null
    __device__ __forceinline__ const uint16_t *operator()(int, int row) const {
        const int r = ids ? ids[row] : row;
        const uint16_t *b = r < seg1 ? base[0] : r < seg2 ? base[1] : base[2];
        const int o = r < seg1 ? r : r < seg2 ? r - seg1 : r - seg2;
        return b + (size_t)o * K;
    }
};

__device__ __forceinline__ RowJob fused_row_job(const DraftParams &p, int ph, int step) {
    constexpr int kNone = 0x7fffffff;
    RowJob j;
    j.base[1] = j.base[2] = nullptr;
    j.seg1 = j.seg2 = kNone;
    j.ids = nullptr;
    switch (ph) {
    case FP_PROJ: j.base[0] = p.w_proj; j.K = 2 * p.d; j.rows = p.d; j.out = p.x; break;
    case FP_QKV:
        j.base[0] = p.w_q; j.base[1] = p.w_k; j.base[2] = p.w_v;
        j.seg1 = p.qd; j.seg2 = p.qd + p.kvd;
        j.K = p.d; j.rows = p.qkv_dim; j.out = p.qkv;
        break;
    case FP_O: j.base[0] = p.w_o; j.K = p.qd; j.rows = p.d; j.out = p.o; break;
    case FP_GATEUP:
        j.base[0] = p.w_gate; j.base[1] = p.w_up;
        j.seg1 = p.F;
        j.K = p.d; j.rows = 2 * p.F; j.out = p.gu;
        break;
    case FP_DOWN: j.base[0] = p.w_down; j.K = p.F; j.rows = p.d; j.out = p.dn; break;
    default:
        j.base[0] = p.lm_head; j.ids = p.ids; j.K = p.d; j.rows = p.n;
        j.out = p.logits_out ? p.logits_out + (size_t)step * p.n : nullptr;
        break;
    }
    return j;
}

template <int G, int HD>
__device__ __forceinline__ void fused_steps_rows(const DraftParams &p, char *smem) {
    const int vb = blockIdx.x, nvb = gridDim.x, d = p.d;
    unsigned long long *red64 = reinterpret_cast<unsigned long long *>(smem + p.fused_gemv_bytes);
    unsigned epoch = 0;
    int stamp_i = 0;
    auto stamp = [&](int step) {
        if (p.trace && vb == 0 && threadIdx.x == 0 && stamp_i < 16) p.trace[step * 16 + stamp_i] = wall_clock64();
        ++stamp_i;
    };
    if (vb == 0 && threadIdx.x == 0 && seq_dead(p, 0)) atomicOr(p.err, kErrKvOverflow);

    // winner of the output head of `step`: maximum over the workgroups' candidates (all threads; contains barriers)
    auto winner = [&](int step) {
        unsigned long long best = 0ull;
        const unsigned long long *cand = p.cand + (size_t)step * p.max_batch * nvb;
        for (int w = threadIdx.x; w < nvb; w += kBlock) {
            const unsigned long long c = ld_u64<true>(cand + w);
            best = c > best ? c : best;
        }
        best = block_max_u64(best, red64);
        uint32_t bi = key_index(best);
        if (bi >= (uint32_t)p.n) bi = 0;
        return p.ids ? p.ids[bi] : (int)bi;
    };

    for (int step = 0; step < p.K; ++step) {
        stamp_i = 0;
        stamp(step);
#pragma unroll 1
        for (int ph = FP_PROJ; ph <= FP_HEAD; ++ph) {
            const RowJob job = fused_row_job(p, ph, step);
            GemvLds l = gemv_lds(smem, job.K, 1, 1);
            auto stage = [&]() {
                if (step > 0 || ph != FP_PROJ) bar_wait(p, epoch); // the phase before (or the previous step's head)
                switch (ph) {
                case FP_PROJ: {
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
                    if (step == 0 && !p.own_hidden)
                        stage_rmsnorm<true>(p.hidden_in, p.g_h, d, p.eps, l.hi, l.lo, l.red, nullptr);
                    else
                        stage_rmsnorm<false, true>(p.hhat, p.g_h, d, p.eps, l.hi, l.lo, l.red, nullptr);
                    stage_rmsnorm<true>(p.embed + (size_t)tok * d, p.g_e, d, p.eps, l.hi + d, l.lo + d, l.red, nullptr);
                    break;
                }
                case FP_QKV: stage_rmsnorm<false, true>(p.x, p.g_attn, d, p.eps, l.hi, l.lo, l.red, nullptr); break;
                case FP_O: stage_plain<true>(p.attn, p.qd, l.kpad, l.hi, l.lo); break;
                case FP_GATEUP:
                    stage_rmsnorm<false, true>(p.x, p.g_mlp, d, p.eps, l.hi, l.lo, l.red, nullptr, nullptr, p.o);
                    break;
                case FP_DOWN: stage_swiglu<true>(p.gu, p.F, l.kpad, l.hi, l.lo); break;
                default: {
                    float *hh = (vb == 0) ? p.hhat : nullptr;
                    float *ho = (vb == 0 && p.hidden_out) ? p.hidden_out + (size_t)step * d : nullptr;
                    stage_rmsnorm<false, true>(p.x, p.g_final, d, p.eps, l.hi, l.lo, l.red, hh, ho, p.o, p.dn);
                    break;
                }
                }
                __syncthreads();
            };
            unsigned long long best = 0ull; // of the rows this lane reported (lane 0 of a wave reports)
            auto epi = [&](int, int row, float(&s)[1]) {
                if (job.out) st_f32<true>(job.out + row, s[0]);
                const unsigned long long key = argmax_key(s[0], (uint32_t)row);
                best = key > best ? key : best;
            };
            gemv_rowmode<1, 1, true>(job, job.K, job.rows, vb, nvb, 1, l.hi, l.lo, l.kpad, stage, epi);
            if (ph == FP_HEAD) {
                const unsigned long long m = block_max_u64(best, red64);
                if (threadIdx.x == 0) st_u64<true>(p.cand + (size_t)step * p.max_batch * nvb + vb, m);
            }
            stamp(step);
            bar_arrive(p, ++epoch);
            if (ph == FP_QKV) { // attention: no weights to request ahead
                bar_wait(p, epoch);
                call_attn<G, HD, true, true>(p, step, vb, nvb, smem);
                stamp(step);
                bar_arrive(p, ++epoch); // the splits of a long context were merged by the workgroup that finished last
            }
        }
    }
    // publish the last draft id
    bar_wait(p, epoch);
    if (vb == 0) {
        const int did = winner(p.K - 1);
        if (threadIdx.x == 0) p.draft_out[p.K - 1] = seq_dead(p, 0) ? -1 : did;
    }
}

} // namespace mtp
