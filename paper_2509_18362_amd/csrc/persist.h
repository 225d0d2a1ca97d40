// All K draft steps of ONE sequence in one cooperative kernel (gfx950): the phases of phases.h, row-streaming core,
// separated by grid barriers instead of kernel launches.
//
// What makes this faster than a launch per phase, where an earlier single-launch path (fused.h) was not:
//  * The barrier uses relaxed device-scope atomics only.  A release/acquire pair at device scope writes back and
//    invalidates whole caches (each compute die has its own L2); measured 6 us per barrier idle and 15 us on top of
//    a streaming phase, against 1.7 us and 5 us for the relaxed one.  The data that crosses a barrier - a few
//    activation vectors, the argmax candidates, the appended cache entries - is written and read with
//    device-coherent accesses instead (relaxed atomics, access by access); the weights and the rest of the KV cache
//    are read-only inside the kernel and go through the caches as usual.
//  * A phase requests its first weights (the register ring of the row-streaming core, 24 KiB per wave, 48 MiB per
//    chip) BEFORE it waits for the barrier of the phase before it: HBM keeps delivering while the workgroups
//    synchronise and stage their input, so the pipeline never drains between phases.
// Every wait is bounded by a wall-clock limit; on expiry the sticky error word is set and all later waits fall
// through, so the grid always drains.  The cooperative launch guarantees that all workgroups are resident.
#pragma once
#include "attn_mfma.h"
#include "fused.h"
#include "phases.h"

namespace mtp {

constexpr int kPersistBarriersPerStep = 8; // proj, qkv, attn, merge, oproj, gateup, down, head (merge: if split)

// arrive: every store of the phase has completed (the workgroup barrier waits for them), then one relaxed ticket
__device__ __forceinline__ void pbar_arrive(const DraftParams &p, unsigned epoch) {
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

__device__ __forceinline__ void pbar_wait(const DraftParams &p, unsigned epoch) {
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

struct GridSync {
    const DraftParams &p;
    unsigned arrived = 0, waited = 0;
    __device__ __forceinline__ void arrive() { pbar_arrive(p, ++arrived); }
    __device__ __forceinline__ void wait() {
        if (waited != arrived) {
            pbar_wait(p, arrived);
            waited = arrived;
        }
    }
};

// One call = K steps of sequence 0.  Workgroup blockIdx.x of gridDim.x (one per CU).
template <int G, int HD>
__device__ __forceinline__ void persist_steps(const DraftParams &p, char *smem) {
    const int vb = blockIdx.x, nvb = gridDim.x, d = p.d;
    GridSync sync{p};
    unsigned long long *red64 = reinterpret_cast<unsigned long long *>(smem + p.fused_gemv_bytes);
    if (vb == 0 && threadIdx.x == 0 && seq_dead(p, 0)) atomicOr(p.err, kErrKvOverflow);

    for (int step = 0; step < p.K; ++step) {
        // ---- embedding gather + dual RMSNorm + concat + 2d->d projection ------------------------------------
        {
            GemvLds l = gemv_lds(smem, 2 * d, 1, 1);
            auto stage = [&]() {
                sync.wait(); // the previous step's candidates and hidden state
                int tok;
                if (step == 0) {
                    tok = p.token_in[0];
                } else {
                    const int did = key_token(p, winner_key<true>(p, step - 1, 0, red64));
                    if (vb == 0 && threadIdx.x == 0) p.draft_out[step - 1] = seq_dead(p, 0) ? -1 : did;
                    tok = p.forced ? p.forced[step - 1] : did;
                }
                if (tok < 0 || tok >= p.V) { // reported, and replaced by id 0 so that every access stays in bounds
                    if (threadIdx.x == 0) atomicOr(p.err, kErrTokenRange);
                    tok = 0;
                }
                __syncthreads();
                if (step == 0)
                    stage_rmsnorm<true, false>(p.hidden_in, p.g_h, d, p.eps, l.hi, l.lo, l.red, nullptr);
                else
                    stage_rmsnorm<false, true>(p.hhat, p.g_h, d, p.eps, l.hi, l.lo, l.red, nullptr);
                stage_rmsnorm<true, false>(p.embed + (size_t)tok * d, p.g_e, d, p.eps, l.hi + d, l.lo + d, l.red, nullptr);
                __syncthreads();
            };
            auto rowptr = [&](int, int row) { return p.w_proj + (size_t)row * 2 * d; };
            auto epi = [&](int, int row, float(&s)[1]) { st_f32<true>(p.x + row, s[0]); };
            gemv_rowmode<1, 1, true>(rowptr, 2 * d, d, vb, nvb, 1, l.hi, l.lo, l.kpad, stage, epi);
            sync.arrive();
        }
        // ---- attention-input RMSNorm + q/k/v projection ----------------------------------------------------------
        {
            GemvLds l = gemv_lds(smem, d, 1, 1);
            auto stage = [&]() {
                sync.wait();
                __syncthreads();
                stage_rmsnorm<false, true>(p.x, p.g_attn, d, p.eps, l.hi, l.lo, l.red, nullptr);
                __syncthreads();
            };
            auto rowptr = [&](int, int row) {
                if (row < p.qd) return p.w_q + (size_t)row * d;
                if (row < p.qd + p.kvd) return p.w_k + (size_t)(row - p.qd) * d;
                return p.w_v + (size_t)(row - p.qd - p.kvd) * d;
            };
            auto epi = [&](int, int row, float(&s)[1]) { st_f32<true>(p.qkv + row, s[0]); };
            gemv_rowmode<1, 1, true>(rowptr, d, p.qkv_dim, vb, nvb, 1, l.hi, l.lo, l.kpad, stage, epi);
            sync.arrive();
        }
        // ---- attention (no weights to request ahead) ---------------------------------------------------------------
        {
            auto wait_qkv = [&]() { sync.wait(); }; // the cache loads of the first work item are requested before it
            if (p.mfma_attn)
                phase_attn_mfma<G, HD, true>(p, step, vb, nvb, smem, wait_qkv);
            else
                phase_attn<G, HD, true>(p, step, vb, nvb, smem, wait_qkv);
            sync.arrive();
        }
        if (p.max_splits > 1) {
            sync.wait();
            phase_attn_merge<HD, true>(p, step, vb, nvb, smem);
            sync.arrive();
        }
        // ---- output projection ---------------------------------------------------------------------------------------
        {
            GemvLds l = gemv_lds(smem, p.qd, 1, 1);
            auto stage = [&]() {
                sync.wait();
                __syncthreads();
                stage_plain<true>(p.attn, p.qd, l.kpad, l.hi, l.lo);
                __syncthreads();
            };
            auto rowptr = [&](int, int row) { return p.w_o + (size_t)row * p.qd; };
            auto epi = [&](int, int row, float(&s)[1]) { st_f32<true>(p.o + row, s[0]); };
            gemv_rowmode<1, 1, true>(rowptr, p.qd, d, vb, nvb, 1, l.hi, l.lo, l.kpad, stage, epi);
            sync.arrive();
        }
        // ---- MLP-input RMSNorm + gate and up projections (one list of 2F rows) ---------------------------------------
        {
            GemvLds l = gemv_lds(smem, d, 1, 1);
            auto stage = [&]() {
                sync.wait();
                __syncthreads();
                stage_rmsnorm<false, true>(p.x, p.g_mlp, d, p.eps, l.hi, l.lo, l.red, nullptr, nullptr, p.o); // x1 = x + w_o attn
                __syncthreads();
            };
            auto rowptr = [&](int, int row) {
                return row < p.F ? p.w_gate + (size_t)row * d : p.w_up + (size_t)(row - p.F) * d;
            };
            auto epi = [&](int, int row, float(&s)[1]) { st_f32<true>(p.gu + row, s[0]); };
            gemv_rowmode<1, 1, true>(rowptr, d, 2 * p.F, vb, nvb, 1, l.hi, l.lo, l.kpad, stage, epi);
            sync.arrive();
        }
        // ---- SiLU(gate) * up + down projection --------------------------------------------------------------------------
        {
            GemvLds l = gemv_lds(smem, p.F, 1, 1);
            auto stage = [&]() {
                sync.wait();
                __syncthreads();
                stage_swiglu<true>(p.gu, p.F, l.kpad, l.hi, l.lo);
                __syncthreads();
            };
            auto rowptr = [&](int, int row) { return p.w_down + (size_t)row * p.F; };
            auto epi = [&](int, int row, float(&s)[1]) { st_f32<true>(p.dn + row, s[0]); };
            gemv_rowmode<1, 1, true>(rowptr, p.F, d, vb, nvb, 1, l.hi, l.lo, l.kpad, stage, epi);
            sync.arrive();
        }
        // ---- final RMSNorm + output head over the listed rows + per-workgroup argmax candidate ---------------------------
        {
            GemvLds l = gemv_lds(smem, d, 1, 1);
            auto stage = [&]() {
                sync.wait();
                __syncthreads();
                // workgroup 0 also publishes the step's output hidden state: for the next step and for the caller
                float *hh = (vb == 0) ? p.hhat : nullptr;
                float *ho = (vb == 0 && p.hidden_out) ? p.hidden_out + (size_t)step * d : nullptr;
                stage_rmsnorm<false, true>(p.x, p.g_final, d, p.eps, l.hi, l.lo, l.red, hh, ho, p.o, p.dn); // x2 = x1 + w_down m
                __syncthreads();
            };
            unsigned long long best = 0ull; // of the rows this lane reported (lane 0 of a wave reports)
            auto rowptr = [&](int, int row) {
                int r = p.ids ? p.ids[row] : row;
                return p.lm_head + (size_t)r * d;
            };
            auto epi = [&](int, int row, float(&s)[1]) {
                if (p.logits_out) p.logits_out[(size_t)step * p.n + row] = s[0];
                const unsigned long long key = argmax_key(s[0], (uint32_t)row);
                best = key > best ? key : best;
            };
            gemv_rowmode<1, 1, false>(rowptr, d, p.n, vb, nvb, 1, l.hi, l.lo, l.kpad, stage, epi);
            const unsigned long long m = block_max_u64(best, red64);
            if (threadIdx.x == 0) st_u64<true>(p.cand + (size_t)step * p.max_batch * p.head_grid + vb, m);
            sync.arrive();
        }
    }
    // the last draft id
    sync.wait();
    if (vb == 0) {
        const int did = key_token(p, winner_key<true>(p, p.K - 1, 0, red64));
        if (threadIdx.x == 0) p.draft_out[p.K - 1] = seq_dead(p, 0) ? -1 : did;
    }
}

} // namespace mtp
