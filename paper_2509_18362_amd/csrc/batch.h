// Batched weight streaming for 5..64 sequences per pass (gfx950): every weight is read from HBM once per pass.
//
// The activations of a phase arrive already split into bf16 hi + lo, written to global memory by the phase before
// (they stay in L2), so the A operand of the 16x16x32 MFMA (16 sequences x 32 elements) is loaded straight into
// registers and reused for every weight tile the wave holds at that depth: no LDS staging, no barrier until a group
// of tiles is complete.  A wave keeps eight accumulators: 8/NA weight tiles (16 rows each) times NA sequence tiles.
//
// Work split of a phase over the grid: RG row groups times KP reduction parts.  Phases with many rows per workgroup
// (gate/up, the output head) use KP = 1; phases with one 16-row tile per workgroup would reload all activations for
// 16 rows, so they put eight tiles into a row group and split the reduction over KP workgroups instead.  Inside a
// workgroup the eight waves split the workgroup's reduction range; their sums meet in LDS, the workgroup's sums go
// to a partial buffer in global memory, and the LAST workgroup of a row group to arrive (a ticket counter) adds the
// KP partials in a fixed order and runs the phase's epilogue.  With KP = 1 the same code runs without the ticket.
//
// RMSNorm (Sec. 2.1) costs no pass over the activations here: the producer writes gain * u (split) and the sum of
// squares of its rows, and because W (s g*u) = s W (g*u), the consumer multiplies its results by
// s = 1/sqrt(mean(u^2) + eps) in the epilogue.
#pragma once
#include "phases.h"

namespace mtp {

constexpr int kBatchAcc = 8;      // accumulators per wave
constexpr int kBatchMaxSeq = 64;  // sequences per pass
// A lane offset at or beyond the end of every buffer (the host checks that each matrix is smaller than 2 GiB): such a
// load returns zeros and moves no data.  Adding the wave-uniform offset (a few MiB at most) cannot wrap it around.
constexpr uint32_t kOobOffset = 0x80000000u;


template <int NA>
struct BatchShape {
    static constexpr int TG = kBatchAcc / NA;   // weight tiles per group
    static constexpr int D = 2;                 // items (one double depth step of a group) in flight per wave
    static constexpr int NL = 2 * TG + 4 * NA;  // 16-byte loads per lane per item
};

// partial sums of the waves (or, for wide batches, the two activation buffers, which are smaller), the
// transposition strips, the norm scales, the ids of the row group
__host__ __device__ inline size_t batch_lds_bytes(int max_rows_per_wg) {
    return (size_t)kWaves * kBatchAcc * kWave * 16 + (size_t)kWaves * 2 * 2304 + kBatchMaxSeq * 4 +
           (size_t)max_rows_per_wg * 4 + 256;
}

// The bf16 hi/lo pair of one float, as the A operand wants it
__device__ __forceinline__ void store_split(uint16_t *hi, size_t lo_off, size_t idx, float v) {
    uint16_t h, l;
    split_bf16(v, h, l);
    hi[idx] = h;
    hi[lo_off + idx] = l;
}

// A 16-row x 128-byte tile travels from memory to the MFMA operand layout in two hops.  Loaded straight into the
// layout (lane (j, g): row j, bytes 32g..), every lane of a load instruction touches another row: sixteen 16-byte
// pieces per 64 B/clk address-unit pass, which caps a CU near 16 B/clk.  Instead a lane loads row (lane / 8) [+ 8],
// bytes 16 (lane % 8): eight lanes cover one 128-byte line, four times fewer address-unit cycles.  The wave then
// parks the two halves in a private LDS strip (row stride 144 bytes: the sixteen rows of a transposed read fall
// into different banks) and reads its operand pieces back.  LDS operations of one wave complete in order, so a strip
// can be rewritten right after it was read.
constexpr int kStripRow = 144, kStripBytes = 16 * kStripRow;
__device__ __forceinline__ void strip_park(char *strip, const u32x4 &rows_lo, const u32x4 &rows_hi) {
    const int lane = threadIdx.x & (kWave - 1);
    char *dst = strip + (lane >> 3) * kStripRow + (lane & 7) * 16;
    *reinterpret_cast<u32x4 *>(dst) = rows_lo;
    *reinterpret_cast<u32x4 *>(dst + 8 * kStripRow) = rows_hi;
}
// piece hf (0, 1) of lane (j, g): bytes 32 g + 16 hf of row j
__device__ __forceinline__ void strip_fetch(const char *strip, u32x4 &hf0, u32x4 &hf1) {
    const int lane = threadIdx.x & (kWave - 1);
    const char *src = strip + (lane & 15) * kStripRow + (lane >> 4) * 32;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    hf0 = *reinterpret_cast<const u32x4 *>(src);
    hf1 = *reinterpret_cast<const u32x4 *>(src + 16);
}

// s_b = 1/sqrt(mean(u_b^2) + eps) for the nb sequences of the pass, from the producers' per-tile sums of squares
__device__ __forceinline__ void batch_scales(const DraftParams &p, int kind, float *scale_lds) {
    const int bl = threadIdx.x >> 3, sub = threadIdx.x & 7;
    const int npart = p.d / 16;
    float s = 0.f;
    if (bl < p.nb) {
        const float *src = p.ssq + ((size_t)kind * p.max_batch + p.b0 + bl) * npart;
        // sixteen loads in flight at a time (one at a time, each behind the weight requests of its wave, this sum was
        // the longest chain of the kernel: 20 us in the two waves that hold sixteen sequences)
        for (int i0 = sub; i0 < npart; i0 += 8 * 16) {
            float t[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) t[u] = i0 + 8 * u < npart ? src[i0 + 8 * u] : 0.f;
#pragma unroll
            for (int u = 0; u < 16; ++u) s += t[u];
        }
    }
    s = oct_sum(s);
    if (sub == 0 && bl < kBatchMaxSeq) scale_lds[bl] = bl < p.nb ? 1.0f / sqrtf(s / (float)p.d + p.eps) : 0.f;
}

// Adds the KP parts of one epilogue slot (virtual tile vt, or the pair starting there, and sequence tile at) in the
// order of the parts and hands the sums to the phase's epilogue.  Called by whole waves.
// A workgroup's sums for the partial buffer: plain when a later kernel adds the parts, device-coherent when the last
// workgroup of this kernel does (uniform choice).
__device__ __forceinline__ void st_part(float *dst, f32x4 v, bool coherent) {
    if (coherent)
        st_f32x4<true>(dst, v);
    else
        *reinterpret_cast<f32x4 *>(dst) = v;
}

// COH: the parts are read past the caches (the caller is the last workgroup of a ticket, inside the kernel that
// wrote them).
template <int NA, bool COH = false, class Ph>
__device__ __forceinline__ void bg_slot_epilogue(const DraftParams &p, Ph &ph, int KP, int ntv, int vt, int at,
                                                 const float *scale_lds) {
    constexpr int NMAT = Ph::NMAT;
    const int lane = threadIdx.x & (kWave - 1), j = lane & 15, g = lane >> 4;
    f32x4 sums[NMAT];
#pragma unroll
    for (int m = 0; m < NMAT; ++m) {
        const float *src = p.part + (((size_t)(vt + m) * NA + at) * kWave + lane) * 4;
        const size_t kstride = (size_t)ntv * NA * kWave * 4;
        f32x4 sacc = {0.f, 0.f, 0.f, 0.f};
        for (int k2 = 0; k2 < KP; k2 += 8) { // eight loads in flight
            f32x4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                v[u] = ld_f32x4<COH>(src + (size_t)min(k2 + u, KP - 1) * kstride);
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (k2 + u < KP) sacc += v[u];
        }
        sums[m] = sacc;
    }
    ph.epi(at * 16 + g * 4, vt, j, sums, scale_lds);
}

// The end of a matrix phase: the workgroup's sums are in the partial buffer.  The last workgroup of the row group to
// arrive adds the KP parts in the order of the parts and runs the epilogue (KP = 1: no ticket).  slots(f) calls
// f(t, at) for every (first virtual tile relative to vt0, sequence tile) the calling WAVE is responsible for.
template <int NA, class Ph, class Slots>
__device__ __forceinline__ void bg_tail(const DraftParams &p, Ph &ph, int KP, int rg, int ntv, int vt0, char *smem,
                                        const float *scale_lds, Slots slots) {
    // Every wave waits for the acknowledgement of its own stores before the workgroup barrier: a workgroup-scope
    // barrier alone orders accesses inside the CU and need not wait for stores still on their way to memory.
    if (KP > 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (KP > 1) {
        // The sums were written through to memory (device-coherent stores) and acknowledged before the ticket is
        // drawn, and the last workgroup reads them past its caches: relaxed atomics suffice, and no cache is written
        // back or invalidated (a release/acquire pair here cost ~10 us per phase).
        int *flag = reinterpret_cast<int *>(smem); // the LDS of the main loop is dead now
        if (threadIdx.x == 0) {
            int old = __hip_atomic_fetch_add(p.ticket + rg, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *flag = (old == KP - 1);
            if (old == KP - 1) __hip_atomic_store(p.ticket + rg, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        const bool last = *flag != 0;
        __syncthreads();
        if (!last) return;
        slots([&](int t, int at) { bg_slot_epilogue<NA, true>(p, ph, KP, ntv, vt0 + t, at, scale_lds); });
    } else {
        slots([&](int t, int at) { bg_slot_epilogue<NA>(p, ph, KP, ntv, vt0 + t, at, scale_lds); }); // uniform per wave
    }
    ph.finish(rg, smem);
}

// ---------------------------------------------------------------------------------------------------
// the core.  Ph supplies:
//   NMAT (1, or 2 = adjacent tiles form (gate, up) pairs), STREAM (non-temporal weight loads), GATHER (rows through
//   the id list), SCALE (SSQ_* kind whose scale the epilogue needs, or -1),
//   K, rows (per matrix), in (hi array of the input activations),
//   tile(vt, base, mat_rows, row0, row_end): matrix (start, rows) and first row of virtual tile vt; rows at or past
//   row_end do not exist,
//   epi(bf, vt, j, sums[NMAT], scale_lds): results of sequences b0+bf .. +3 (components of the f32x4) for row j of
//   virtual tile vt (NMAT = 2: vt is the gate tile), run by all 64 lanes of a wave together,
//   finish(rg, smem): after the last epilogue of the row group (all threads).
// ---------------------------------------------------------------------------------------------------
template <int NA, class Ph>
__device__ __forceinline__ void bgemv(const DraftParams &p, Ph &ph, int RG, int KP, char *smem) {
    using S = BatchShape<NA>;
    constexpr int NMAT = Ph::NMAT, TG = S::TG, D = S::D, NL = S::NL;
    const int wg = blockIdx.x;
    if (wg >= RG * KP) return;
    const int kp = wg % KP, rg = wg / KP;
    const int lane = threadIdx.x & (kWave - 1), g = lane >> 4;
    // said explicitly to be wave-uniform: offsets and descriptors derived from it then stay in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    const int K = ph.K;
    const int units = (ph.rows + 15) / 16;
    const int u0 = (int)((long long)rg * units / RG), u1 = (int)((long long)(rg + 1) * units / RG);
    const int vt0 = u0 * NMAT, nvt = (u1 - u0) * NMAT, ntv = units * NMAT;
    const int ngroups = (nvt + TG - 1) / TG;
    // The reduction runs in double steps of 64 elements (128 bytes of a row): lane (j, g) holds bytes 32g .. 32g+32 of
    // the piece, of row j (weights) or sequence j (activations); its first 16 bytes feed one MFMA, the other 16 the
    // next - any assignment of elements to MFMA depth slots is fine as long as both operands use the same one.  Two
    // loads of a lane are neighbours, so a wave always consumes whole 128-byte lines.  Double steps are dealt to the
    // waves round robin: at any time the eight waves read eight neighbouring pieces of every row, 1 KiB in a row.
    const int nks = (K + 63) / 64;
    const int ksA = (int)((long long)kp * nks / KP), ksB = (int)((long long)(kp + 1) * nks / KP);
    const int per = max((ksB - ksA + kWaves - 1) / kWaves, 1); // items per group, the same for every wave

    f32x4 *partial = reinterpret_cast<f32x4 *>(smem);                           // [kWaves][kBatchAcc][kWave]
    char *strips = reinterpret_cast<char *>(partial + kWaves * kBatchAcc * kWave); // [kWaves][2] transposition strips
    float *scale_lds = reinterpret_cast<float *>(strips + kWaves * 2 * kStripBytes); // [kBatchMaxSeq]
    int *ids_lds = reinterpret_cast<int *>(scale_lds + kBatchMaxSeq);           // [rows of this row group]
    if (Ph::GATHER) {
        const int r0 = u0 * 16, nr = (u1 - u0) * 16;
        for (int i = threadIdx.x; i < nr; i += kBlock) {
            int pos = min(r0 + i, ph.rows - 1);
            ids_lds[i] = ph.ids ? ph.ids[pos] : pos;
        }
        __syncthreads();
    }

    // activations: one descriptor over the hi and lo arrays; lane (j, g) reads sequence at*16 + j
    const size_t lo_bytes = p.a_lo * 2;
    const row_rsrc ar = make_row_rsrc(ph.in, (int)(2 * lo_bytes));
    // a lane fetches sequence at*16 + lane/8 [+ 8], bytes 16 (lane % 8) of the 128-byte piece
    int voff_a[NA][2];
#pragma unroll
    for (int at = 0; at < NA; ++at)
#pragma unroll
        for (int h = 0; h < 2; ++h)
            voff_a[at][h] = (int)((size_t)min(p.b0 + at * 16 + (lane >> 3) + 8 * h, p.B - 1) * p.a_stride * 2 + (lane & 7) * 16);

    row_rsrc wr[TG];
    int voff_w[TG][2];
    auto setup_group = [&](int grp) {
#pragma unroll
        for (int ts = 0; ts < TG; ++ts) {
            const int t = grp * TG + ts;
            const uint16_t *base;
            int mat_rows, row0, row_end;
            ph.tile(vt0 + min(t, nvt - 1), base, mat_rows, row0, row_end);
            wr[ts] = make_row_rsrc(base, (int)((size_t)mat_rows * K * 2));
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int jr = (lane >> 3) + 8 * h, r = row0 + jr;
                const bool ok = t < nvt && r < row_end;
                const int phys = Ph::GATHER ? ids_lds[(min(t, nvt - 1) / NMAT) * 16 + jr] : r;
                voff_w[ts][h] = ok ? (int)((size_t)phys * K * 2 + (lane & 7) * 16) : (int)kOobOffset;
            }
        }
    };
    // The ring is refilled without any branch: a conditional load would leave the compiler unable to count the loads
    // in flight, and it would then wait for all of them before every use.  Items past the end of a group are
    // requested beyond the buffers' ends instead (zeros, no traffic) and contribute nothing.
    u32x4 ring[D][NL];
    auto issue = [&](u32x4(&slot)[NL], int idx) { // item idx of the current group
        const int ks = min(ksA + idx * kWaves + wave, nks - 1);
        const int soff = min(ks * 64, K - 64) * 2; // the last, ragged step is shifted left to stay inside the row
        const bool live = idx < per;
#pragma unroll
        for (int ts = 0; ts < TG; ++ts)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                slot[2 * ts + h] = row_load16<Ph::STREAM>(wr[ts], live ? voff_w[ts][h] : (int)kOobOffset, soff);
#pragma unroll
        for (int at = 0; at < NA; ++at)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int vo = live ? voff_a[at][h] : (int)kOobOffset;
                slot[2 * TG + 4 * at + h] = row_load16<false>(ar, vo, soff);
                slot[2 * TG + 4 * at + 2 + h] = row_load16<false>(ar, vo, soff + (int)lo_bytes);
            }
    };
    f32x4 acc[kBatchAcc];
#pragma unroll
    for (int a = 0; a < kBatchAcc; ++a) acc[a] = f32x4{0.f, 0.f, 0.f, 0.f};
    char *strip0 = strips + (size_t)wave * 2 * kStripBytes, *strip1 = strip0 + kStripBytes;
    float *part = p.part;
    // The norm scales for the epilogue (visible after the first group's barrier): BEFORE the weight requests.  Loads of a
    // wave return in order, so behind forty weight loads per wave these few values arrived a trip through the busy
    // memory system later each.
    if (Ph::SCALE >= 0 && !p.bg_sep[Ph::WHICH]) batch_scales(p, Ph::SCALE, scale_lds);
    for (int grp = 0; grp < ngroups; ++grp) {
        setup_group(grp);
        // One item ahead: the request for item i + 1 goes out when item i is about to be multiplied.  (Two items ahead -
        // both slots requested at the start, each refilled as it is used up - put 80 MiB of requests into the memory
        // system at once over the chip; the waves that came last then got their first data 20 us into the kernel and
        // every workgroup waited for them at its barrier.)
        issue(ring[0], 0);
        for (int n0 = 0; n0 < per; n0 += D) {
#pragma unroll
            for (int s = 0; s < D; ++s) {
                const int idx = n0 + s;
                issue(ring[(s + 1) % D], idx + 1);
                const int ksn = ksA + idx * kWaves + wave;
                const int ks = min(ksn, nks - 1);
                const int koff = min(ks * 64, K - 64);
                // 8-element pieces that were already counted by the step before (ragged end), or all pieces of a
                // step beyond the workgroup's range or the group's end, contribute zeros
                const int cut = (idx < per && ksn < ksB) ? (ks * 64 - koff) / 8 : 8;
                const uint32_t keep0 = g * 2 < cut ? 0u : 0xFFFFFFFFu, keep1 = g * 2 + 1 < cut ? 0u : 0xFFFFFFFFu;
                // the activations of the step, through the strips into operand layout
                u32x4 ah[NA][2], al[NA][2];
#pragma unroll
                for (int at = 0; at < NA; ++at) {
                    strip_park(strip0, ring[s][2 * TG + 4 * at], ring[s][2 * TG + 4 * at + 1]);
                    strip_park(strip1, ring[s][2 * TG + 4 * at + 2], ring[s][2 * TG + 4 * at + 3]);
                    strip_fetch(strip0, ah[at][0], ah[at][1]);
                    strip_fetch(strip1, al[at][0], al[at][1]);
                    ah[at][0] &= keep0;
                    al[at][0] &= keep0;
                    ah[at][1] &= keep1;
                    al[at][1] &= keep1;
                }
                // the weight tiles, one strip ahead of the MFMAs
                strip_park(strip0, ring[s][0], ring[s][1]);
#pragma unroll
                for (int ts = 0; ts < TG; ++ts) {
                    char *cur = (ts & 1) ? strip1 : strip0, *nxt = (ts & 1) ? strip0 : strip1;
                    u32x4 w0, w1;
                    strip_fetch(cur, w0, w1);
                    if (ts + 1 < TG) strip_park(nxt, ring[s][2 * ts + 2], ring[s][2 * ts + 3]);
#pragma unroll
                    for (int at = 0; at < NA; ++at) {
                        f32x4 a = acc[ts * NA + at];
                        a = mfma16(ah[at][0], w0, a);
                        a = mfma16(al[at][0], w0, a);
                        a = mfma16(ah[at][1], w1, a);
                        a = mfma16(al[at][1], w1, a);
                        acc[ts * NA + at] = a;
                    }
                }
            }
        }
        // group complete: meet the other waves in LDS, hand the sums to the partial buffer
        f32x4 *pb = partial;
        __syncthreads(); // the previous group's sums have been read; also drains the ring's trailing requests
#pragma unroll
        for (int a = 0; a < kBatchAcc; ++a) {
            pb[(wave * kBatchAcc + a) * kWave + lane] = acc[a];
            acc[a] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        __syncthreads();
        {
            const int a = wave; // this thread adds accumulator `wave`, element `lane`, of all waves
            f32x4 sum = pb[a * kWave + lane];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) sum += pb[(w * kBatchAcc + a) * kWave + lane];
            const int ts = a / NA, at = a % NA, t = grp * TG + ts;
            if (t < nvt)
                st_part(part + ((((size_t)kp * ntv + vt0 + t) * NA + at) * kWave + lane) * 4, sum,
                        KP > 1 && !p.bg_sep[Ph::WHICH]);
        }
    }

    if (p.bg_sep[Ph::WHICH]) return; // the epilogue runs as a kernel of its own (see bgemv_lds)
    bg_tail<NA>(p, ph, KP, rg, ntv, vt0, reinterpret_cast<char *>(partial), scale_lds, [&](auto f) {
        constexpr int NQ = kBatchAcc / NMAT; // (tile or pair, sequence tile) slots with an epilogue: one per wave
        if (wave < NQ)
            for (int grp = 0; grp < ngroups; ++grp) {
                const int t = grp * TG + (wave / NA) * NMAT;
                if (t < nvt) f(t, wave % NA);
            }
    });
}

// ---------------------------------------------------------------------------------------------------
// the core for 17..64 sequences (NA = 2 or 4 sequence tiles).  With the waves splitting the reduction, every wave
// would fetch 2*NA KiB of activations per KiB of weights from L2; here the waves split the TILES of a block instead
// (8/NA tiles per wave, 64/NA per block) and walk the reduction range together: the activations of a double step
// (NA*16 sequences x 64 elements, hi and lo) are fetched once per workgroup - each thread brings NA/2 pieces along
// with its weights - parked in one of two LDS buffers and read from there by all waves.  One barrier per step (it does
// not wait for loads in flight); no reduction across waves.  Everything else (row groups x reduction parts, partial
// buffer, ticket, epilogues) is as above.
// ---------------------------------------------------------------------------------------------------
template <int NA, class Ph>
__device__ __forceinline__ void bgemv_lds(const DraftParams &p, Ph &ph, int RG, int KP, char *smem) {
    static_assert(NA == 2 || NA == 4, "sequence tiles per pass");
    constexpr int NMAT = Ph::NMAT;
    constexpr int TW = kBatchAcc / NA; // weight tiles per wave
    constexpr int TB = kWaves * TW;    // weight tiles per block
    constexpr int NP = NA / 2;         // 16-byte pieces of the activation chunk per thread
    constexpr int D = 2;               // ring slots: the step being multiplied and the one requested ahead (sixteen
                                       // accumulators per wave at four sequence tiles, to halve the LDS reads per weight
                                       // byte, measured slower: 1236 against 1215 us per step at config 5)
    constexpr int NL = 2 * TW + NP;
    constexpr int AROW = 272;          // bytes per sequence in an LDS buffer: 128 hi, 128 lo, 16 to stagger the banks
    constexpr int ABYTES = NA * 16 * AROW;
    const int wg = blockIdx.x;
    if (wg >= RG * KP) return;
    const int kp = wg % KP, rg = wg / KP;
    const int lane = threadIdx.x & (kWave - 1), j = lane & 15, g = lane >> 4;
    // said explicitly to be wave-uniform: offsets and descriptors derived from it then stay in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    const int K = ph.K;
    const int units = (ph.rows + 15) / 16;
    const int u0 = (int)((long long)rg * units / RG), u1 = (int)((long long)(rg + 1) * units / RG);
    const int vt0 = u0 * NMAT, nvt = (u1 - u0) * NMAT, ntv = units * NMAT;
    const int nblocks = (nvt + TB - 1) / TB;
    const int nks = (K + 63) / 64;
    const int ksA = (int)((long long)kp * nks / KP), ksB = (int)((long long)(kp + 1) * nks / KP);
    const int steps = max(ksB - ksA, 1);

    char *abuf = smem;                                                    // [2][NA*16][AROW]
    char *strips = smem + 2 * ABYTES;                                     // [kWaves][2] transposition strips
    float *scale_lds = reinterpret_cast<float *>(strips + kWaves * 2 * kStripBytes); // [kBatchMaxSeq]
    int *ids_lds = reinterpret_cast<int *>(scale_lds + kBatchMaxSeq);     // [rows of this row group]
    if (Ph::GATHER) {
        const int r0 = u0 * 16, nr = (u1 - u0) * 16;
        for (int i = threadIdx.x; i < nr; i += kBlock) {
            int pos = min(r0 + i, ph.rows - 1);
            ids_lds[i] = ph.ids ? ph.ids[pos] : pos;
        }
        __syncthreads();
    }

    // this thread's pieces of the activation chunk: piece = (sequence, hi or lo, 16 bytes of the 128)
    const size_t lo_bytes = p.a_lo * 2;
    const row_rsrc ar = make_row_rsrc(ph.in, (int)(2 * lo_bytes));
    int voff_g[NP], off_l[NP];
#pragma unroll
    for (int r = 0; r < NP; ++r) {
        const int pid = threadIdx.x + r * kBlock, seq = pid >> 4, hl = (pid >> 3) & 1, c = pid & 7;
        voff_g[r] = (int)((size_t)min(p.b0 + seq, p.B - 1) * p.a_stride * 2 + c * 16 + (hl ? lo_bytes : 0));
        off_l[r] = seq * AROW + hl * 128 + c * 16;
    }

    // tiles (pairs of tiles) of a block are dealt to the waves round robin: a row group with few tiles still keeps
    // as many waves busy as it has tiles
    auto tile_of = [&](int tw) { return (tw / NMAT) * (kWaves * NMAT) + wave * NMAT + (tw % NMAT); };
    row_rsrc wr[TW];
    int voff_w[TW][2];
    auto setup_block = [&](int blk) {
#pragma unroll
        for (int tw = 0; tw < TW; ++tw) {
            const int t = blk * TB + tile_of(tw);
            const uint16_t *base;
            int mat_rows, row0, row_end;
            ph.tile(vt0 + min(t, nvt - 1), base, mat_rows, row0, row_end);
            wr[tw] = make_row_rsrc(base, (int)((size_t)mat_rows * K * 2));
#pragma unroll
            for (int h = 0; h < 2; ++h) { // a lane fetches row lane/8 [+ 8], bytes 16 (lane % 8): see strip_park
                const int jr = (lane >> 3) + 8 * h, r = row0 + jr;
                const bool ok = t < nvt && r < row_end;
                const int phys = Ph::GATHER ? ids_lds[(min(t, nvt - 1) / NMAT) * 16 + jr] : r;
                voff_w[tw][h] = ok ? (int)((size_t)phys * K * 2 + (lane & 7) * 16) : (int)kOobOffset;
            }
        }
    };
    // branch-free refill, as in the core above: steps past the end of the range are requested beyond the buffers' ends
    u32x4 ring[D][NL];
    auto issue = [&](u32x4(&slot)[NL], int idx) { // step idx of the current block
        const int ks = min(ksA + idx, nks - 1);
        const int soff = min(ks * 64, K - 64) * 2; // the last, ragged step is shifted left to stay inside the row
        const bool live = idx < steps;
#pragma unroll
        for (int tw = 0; tw < TW; ++tw)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                slot[2 * tw + h] = row_load16<Ph::STREAM>(wr[tw], live ? voff_w[tw][h] : (int)kOobOffset, soff);
#pragma unroll
        for (int r = 0; r < NP; ++r) slot[2 * TW + r] = row_load16<false>(ar, live ? voff_g[r] : (int)kOobOffset, soff);
    };
    f32x4 acc[kBatchAcc];
#pragma unroll
    for (int a = 0; a < kBatchAcc; ++a) acc[a] = f32x4{0.f, 0.f, 0.f, 0.f};
    char *strip0 = strips + (size_t)wave * 2 * kStripBytes, *strip1 = strip0 + kStripBytes;
    float *part = p.part;
    // (before the weight requests, see bgemv; visible after the first step's barrier)
    if (Ph::SCALE >= 0 && !p.bg_sep[Ph::WHICH]) batch_scales(p, Ph::SCALE, scale_lds);
    for (int blk = 0; blk < nblocks; ++blk) {
        setup_block(blk);
        issue(ring[0], 0); // one step ahead, as in bgemv
        for (int n0 = 0; n0 < steps; n0 += D) {
#pragma unroll
            for (int s = 0; s < D; ++s) {
                const int idx = n0 + s;
                issue(ring[(s + 1) % D], idx + 1);
                const int ksn = ksA + idx;
                const int ks = min(ksn, nks - 1);
                const int koff = min(ks * 64, K - 64);
                // pieces counted before (ragged end), or a step past the range: zeros
                const int cut = (idx < steps && ksn < ksB) ? (ks * 64 - koff) / 8 : 8;
                // Park the chunk.  The buffer was last read two steps ago, and every wave has passed the barrier of
                // the step in between since.
                char *ab = abuf + (idx & 1) * ABYTES;
#pragma unroll
                for (int r = 0; r < NP; ++r) *reinterpret_cast<u32x4 *>(ab + off_l[r]) = ring[s][2 * TW + r];
                lds_barrier();
                // all operands first, then the MFMAs ordered so that consecutive ones feed different accumulators
                u32x4 ah[NA][2], al[NA][2];
#pragma unroll
                for (int at = 0; at < NA; ++at) {
                    const char *row = ab + (at * 16 + j) * AROW + g * 32;
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf) {
                        const bool dead = g * 2 + hf < cut;
                        const uint32_t keep = dead ? 0u : 0xFFFFFFFFu; // a mask, not a branch around the LDS read
                        ah[at][hf] = *reinterpret_cast<const u32x4 *>(row + hf * 16) & keep;
                        al[at][hf] = *reinterpret_cast<const u32x4 *>(row + 128 + hf * 16) & keep;
                    }
                }
                // the weight tiles through the strips, one strip ahead of the MFMAs
                strip_park(strip0, ring[s][0], ring[s][1]);
#pragma unroll
                for (int tw = 0; tw < TW; ++tw) {
                    char *cur = (tw & 1) ? strip1 : strip0, *nxt = (tw & 1) ? strip0 : strip1;
                    u32x4 w[2];
                    strip_fetch(cur, w[0], w[1]);
                    if (tw + 1 < TW) strip_park(nxt, ring[s][2 * tw + 2], ring[s][2 * tw + 3]);
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf) {
#pragma unroll
                        for (int at = 0; at < NA; ++at) acc[tw * NA + at] = mfma16(ah[at][hf], w[hf], acc[tw * NA + at]);
#pragma unroll
                        for (int at = 0; at < NA; ++at) acc[tw * NA + at] = mfma16(al[at][hf], w[hf], acc[tw * NA + at]);
                    }
                }
            }
        }
        // block complete: this wave's sums go to the partial buffer
#pragma unroll
        for (int tw = 0; tw < TW; ++tw) {
            const int t = blk * TB + tile_of(tw);
#pragma unroll
            for (int at = 0; at < NA; ++at) {
                if (t < nvt)
                    st_part(part + ((((size_t)kp * ntv + vt0 + t) * NA + at) * kWave + lane) * 4, acc[tw * NA + at],
                            KP > 1 && !p.bg_sep[Ph::WHICH]);
                acc[tw * NA + at] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
        __syncthreads(); // the LDS buffers are free for the next block; drains the ring's trailing requests
    }
    // With many reduction parts the last workgroup of a row group would add parts x tiles x sequence tiles partial
    // tiles alone: the host then launches the epilogue as a kernel of its own, spread over the whole chip.
    if (p.bg_sep[Ph::WHICH]) return;
    bg_tail<NA>(p, ph, KP, rg, ntv, vt0, smem, scale_lds, [&](auto f) {
        for (int blk = 0; blk < nblocks; ++blk)
#pragma unroll
            for (int tw = 0; tw < TW; tw += NMAT) {
                const int t = blk * TB + tile_of(tw);
                if (t < nvt)
#pragma unroll
                    for (int at = 0; at < NA; ++at) f(t, at);
            }
    });
}

// ---------------------------------------------------------------------------------------------------
// the phases of a draft step (Sec. 2.1, Fig. 1) on the batched core
// ---------------------------------------------------------------------------------------------------
struct BgBase {
    static constexpr int NMAT = 1;
    static constexpr bool STREAM = true, GATHER = false;
    static constexpr int SCALE = -1;
    const DraftParams &p;
    int K, rows;
    const uint16_t *in;
    const int *ids = nullptr;
    __device__ BgBase(const DraftParams &p_, int K_, int rows_, const uint16_t *in_) : p(p_), K(K_), rows(rows_), in(in_) {}
    __device__ __forceinline__ void finish(int, char *) {}
    // sum over the sixteen rows of a tile of v*v, for the four sequences of this lane; lanes with j == 0 store it
    __device__ __forceinline__ void store_ssq(int kind, int bf, int vt, int j, const float (&v)[4]) const {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float s = row16_sum(v[c] * v[c]);
            const int bl = bf + c;
            if (j == 0 && bl < p.nb) p.ssq[((size_t)kind * p.max_batch + p.b0 + bl) * (p.d / 16) + vt] = s;
        }
    }
};

// 2d -> d projection of [RMSNorm(h); RMSNorm(E[token])] (already normalised by the preparation kernel).  Leaves x,
// and g_attn * x with its sums of squares for the q/k/v projection.
struct BgProj : BgBase {
    static constexpr int WHICH = BG_PROJ;
    __device__ BgProj(const DraftParams &p_) : BgBase(p_, 2 * p_.d, p_.d, p_.act[0]) {}
    __device__ __forceinline__ void tile(int vt, const uint16_t *&base, int &mat_rows, int &row0, int &row_end) const {
        base = p.w_proj;
        mat_rows = row_end = p.d;
        row0 = vt * 16;
    }
    __device__ __forceinline__ void epi(int bf, int vt, int j, const f32x4 (&s)[1], const float *) const {
        const int row = vt * 16 + j;
        const float v[4] = {s[0].x, s[0].y, s[0].z, s[0].w};
        const float gn = bf16_to_f32(p.g_attn[row]);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int bl = bf + c;
            if (bl < p.nb) {
                const size_t b = p.b0 + bl;
                p.x[b * p.d + row] = v[c];
                store_split(p.act[1], p.a_lo, b * p.a_stride + row, gn * v[c]);
            }
        }
        store_ssq(SSQ_X, bf, vt, j, v);
    }
};

// q/k/v projection of RMSNorm(x; g_attn); bias, rotary embedding and the cache append happen in the attention phase
struct BgQkv : BgBase {
    static constexpr int WHICH = BG_QKV;
    static constexpr int SCALE = SSQ_X;
    __device__ BgQkv(const DraftParams &p_) : BgBase(p_, p_.d, p_.qkv_dim, p_.act[1]) {}
    __device__ __forceinline__ void tile(int vt, const uint16_t *&base, int &mat_rows, int &row0, int &row_end) const {
        const int r = vt * 16;
        if (r < p.qd) {
            base = p.w_q;
            mat_rows = p.qd;
            row0 = r;
        } else if (r < p.qd + p.kvd) {
            base = p.w_k;
            mat_rows = p.kvd;
            row0 = r - p.qd;
        } else {
            base = p.w_v;
            mat_rows = p.kvd;
            row0 = r - p.qd - p.kvd;
        }
        row_end = mat_rows;
    }
    __device__ __forceinline__ void epi(int bf, int vt, int j, const f32x4 (&s)[1], const float *scale) const {
        const int row = vt * 16 + j;
        const float v[4] = {s[0].x, s[0].y, s[0].z, s[0].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int bl = bf + c;
            if (bl < p.nb) p.qkv[(size_t)(p.b0 + bl) * p.qkv_dim + row] = v[c] * scale[bl];
        }
    }
};

// output projection of the attention result; leaves x1 = x + W_o a, and g_mlp * x1 with its sums of squares
struct BgOproj : BgBase {
    static constexpr int WHICH = BG_OPROJ;
    __device__ BgOproj(const DraftParams &p_) : BgBase(p_, p_.qd, p_.d, p_.act[0]) {}
    __device__ __forceinline__ void tile(int vt, const uint16_t *&base, int &mat_rows, int &row0, int &row_end) const {
        base = p.w_o;
        mat_rows = row_end = p.d;
        row0 = vt * 16;
    }
    __device__ __forceinline__ void epi(int bf, int vt, int j, const f32x4 (&s)[1], const float *) const {
        const int row = vt * 16 + j;
        float v[4] = {s[0].x, s[0].y, s[0].z, s[0].w};
        const float gn = bf16_to_f32(p.g_mlp[row]);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int bl = bf + c;
            if (bl < p.nb) {
                const size_t b = p.b0 + bl;
                v[c] += p.x[b * p.d + row];
                p.o[b * p.d + row] = v[c];
                store_split(p.act[1], p.a_lo, b * p.a_stride + row, gn * v[c]);
            } else {
                v[c] = 0.f;
            }
        }
        store_ssq(SSQ_X1, bf, vt, j, v);
    }
};

// gate and up projections of RMSNorm(x1; g_mlp) as pairs of tiles; leaves m = silu(gate) * up, split
struct BgGateUp : BgBase {
    static constexpr int WHICH = BG_GATEUP;
    static constexpr int NMAT = 2;
    static constexpr int SCALE = SSQ_X1;
    __device__ BgGateUp(const DraftParams &p_) : BgBase(p_, p_.d, p_.F, p_.act[1]) {}
    __device__ __forceinline__ void tile(int vt, const uint16_t *&base, int &mat_rows, int &row0, int &row_end) const {
        base = (vt & 1) ? p.w_up : p.w_gate;
        mat_rows = row_end = p.F;
        row0 = (vt >> 1) * 16;
    }
    __device__ __forceinline__ void epi(int bf, int vt, int j, const f32x4 (&s)[2], const float *scale) const {
        const int row = (vt >> 1) * 16 + j;
        const float gv[4] = {s[0].x, s[0].y, s[0].z, s[0].w}, uv[4] = {s[1].x, s[1].y, s[1].z, s[1].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int bl = bf + c;
            if (bl < p.nb && row < p.F) {
                const float gs = gv[c] * scale[bl], us = uv[c] * scale[bl];
                store_split(p.act[0], p.a_lo, (size_t)(p.b0 + bl) * p.a_stride + row, (gs / (1.0f + expf(-gs))) * us);
            }
        }
    }
};

// down projection; leaves x2 = x1 + W_down m, and g_final * x2 with its sums of squares for the output head
struct BgDown : BgBase {
    static constexpr int WHICH = BG_DOWN;
    __device__ BgDown(const DraftParams &p_) : BgBase(p_, p_.F, p_.d, p_.act[0]) {}
    __device__ __forceinline__ void tile(int vt, const uint16_t *&base, int &mat_rows, int &row0, int &row_end) const {
        base = p.w_down;
        mat_rows = row_end = p.d;
        row0 = vt * 16;
    }
    __device__ __forceinline__ void epi(int bf, int vt, int j, const f32x4 (&s)[1], const float *) const {
        const int row = vt * 16 + j;
        float v[4] = {s[0].x, s[0].y, s[0].z, s[0].w};
        const float gn = bf16_to_f32(p.g_final[row]);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int bl = bf + c;
            if (bl < p.nb) {
                const size_t b = p.b0 + bl;
                v[c] += p.o[b * p.d + row];
                p.dn[b * p.d + row] = v[c];
                store_split(p.act[1], p.a_lo, b * p.a_stride + row, gn * v[c]);
            } else {
                v[c] = 0.f;
            }
        }
        store_ssq(SSQ_X2, bf, vt, j, v);
    }
};

// output head over the compressed vocabulary (Sec. 2.2, Eq. (3)): logits of RMSNorm(x2; g_final) against the listed
// rows, and per row group the best (logit, position) of every sequence
struct BgHead : BgBase {
    static constexpr int WHICH = BG_LMHEAD;
    static constexpr bool STREAM = false, GATHER = true;
    static constexpr int SCALE = SSQ_X2;
    int step;
    unsigned long long best[kBatchMaxSeq / 16][4] = {}; // by sequence tile; a lane sees four sequences of each
    __device__ BgHead(const DraftParams &p_, int step_) : BgBase(p_, p_.d, p_.n, p_.act[1]), step(step_) { ids = p_.ids; }
    __device__ __forceinline__ void tile(int vt, const uint16_t *&base, int &mat_rows, int &row0, int &row_end) const {
        base = p.lm_head;
        mat_rows = p.V;
        row_end = p.n;
        row0 = vt * 16;
    }
    __device__ __forceinline__ void epi(int bf, int vt, int j, const f32x4 (&s)[1], const float *scale) {
        const int pos = vt * 16 + j;
        const float v[4] = {s[0].x, s[0].y, s[0].z, s[0].w};
        const int at = bf >> 4;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int bl = bf + c;
            if (bl < p.nb && pos < p.n) {
                const float logit = v[c] * scale[bl];
                if (p.logits_out) p.logits_out[((size_t)(p.b0 + bl) * p.K + step) * p.logit_stride + pos] = logit;
                const unsigned long long key = argmax_key(logit, (uint32_t)pos);
#pragma unroll
                for (int a = 0; a < kBatchMaxSeq / 16; ++a) // static indices keep the array in registers
                    if (a == at) best[a][c] = key > best[a][c] ? key : best[a][c];
            }
        }
    }
    // candidates: maximum over the sixteen rows of a lane group, then over the waves that served the same sequences
    __device__ __forceinline__ void finish(int rg, char *smem) {
        unsigned long long *red = reinterpret_cast<unsigned long long *>(smem); // [kWaves][kBatchMaxSeq]
        __syncthreads();
        for (int i = threadIdx.x; i < kWaves * kBatchMaxSeq; i += kBlock) red[i] = 0ull;
        __syncthreads();
        const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
#pragma unroll
        for (int a = 0; a < kBatchMaxSeq / 16; ++a)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                unsigned long long m = best[a][c];
#pragma unroll
                for (int off = 1; off < 16; off <<= 1) {
                    unsigned long long o = __shfl_xor(m, off, kWave);
                    m = o > m ? o : m;
                }
                if ((lane & 15) == 0 && m != 0ull) red[wave * kBatchMaxSeq + a * 16 + (lane >> 4) * 4 + c] = m;
            }
        __syncthreads();
        if ((int)threadIdx.x < p.nb) {
            unsigned long long m = 0ull;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                unsigned long long c = red[w * kBatchMaxSeq + threadIdx.x];
                m = c > m ? c : m;
            }
            p.cand[((size_t)step * p.max_batch + p.b0 + threadIdx.x) * p.head_grid + rg] = m;
        }
    }
};

// The epilogue of a matrix phase as a kernel of its own: one wave per slot (tile or pair of tiles, sequence tile), any
// grid; phases that keep state per workgroup (the output head's candidates) finish per workgroup of THIS kernel.
template <int NA, class Ph>
__device__ __forceinline__ void phase_bepilogue(const DraftParams &p, Ph &ph, int KP, char *smem) {
    constexpr int NMAT = Ph::NMAT;
    float *scale_lds = reinterpret_cast<float *>(smem + kWaves * kBatchMaxSeq * 8); // behind finish()'s scratch
    if (Ph::SCALE >= 0) batch_scales(p, Ph::SCALE, scale_lds);
    __syncthreads();
    const int ntv = (ph.rows + 15) / 16 * NMAT, nslots = ntv / NMAT * NA;
    for (int id = blockIdx.x * kWaves + threadIdx.x / kWave; id < nslots; id += gridDim.x * kWaves)
        bg_slot_epilogue<NA>(p, ph, KP, ntv, (id / NA) * NMAT, id % NA, scale_lds);
    ph.finish(blockIdx.x, smem);
}

// ---------------------------------------------------------------------------------------------------
// preparation kernel, one workgroup per sequence, before every step and once after the last:
//   s > 0: the id drafted by step s-1 and its output hidden state  h_hat = RMSNorm(x2; g_final)
//   s < K: the input of step s, [RMSNorm(h; g_h); RMSNorm(E[token]; g_e)], split into bf16 hi + lo
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ void phase_bprep(const DraftParams &p, int step, char *smem) {
    const int b = blockIdx.x, d = p.d, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    float *ra = reinterpret_cast<float *>(smem), *rb = ra + kWaves, *rc = rb + kWaves; // [kWaves] each
    unsigned long long *rk = reinterpret_cast<unsigned long long *>(smem + 128);       // [kWaves]
    uint16_t *hi = p.act[0] + (size_t)b * p.a_stride;
    uint16_t *lo = hi + p.a_lo;
    if (step == 0 && tid == 0 && seq_overflows(p, b)) atomicOr(p.err, kErrKvOverflow);

    // Everything that can be asked for before the previous step's winner is known is asked for first, and the sums
    // of squares travel through ONE reduction together with the winner: the kernel is a chain of memory round trips
    // and barriers on sixteen to sixty-four CUs, not a bandwidth problem.
    auto split_store = [&](uint16_t *dh, uint16_t *dl, int e, const float (&o)[4]) {
        uint16_t h[4], l[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) split_bf16(o[q], h[q], l[q]);
        *reinterpret_cast<u32x2 *>(dh + e) = u32x2{(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
        *reinterpret_cast<u32x2 *>(dl + e) = u32x2{(uint32_t)l[0] | ((uint32_t)l[1] << 16), (uint32_t)l[2] | ((uint32_t)l[3] << 16)};
    };
    auto load_bf16x4 = [&](const uint16_t *src, int e, float (&v)[4]) {
        const u32x2 raw = *reinterpret_cast<const u32x2 *>(src + e);
        v[0] = lo_half(raw.x);
        v[1] = hi_half(raw.x);
        v[2] = lo_half(raw.y);
        v[3] = hi_half(raw.y);
    };
    auto checked = [&](int t) { // reported, and replaced by id 0 so that every access stays in bounds
        if (t < 0 || t >= p.V) {
            if (tid == 0) atomicOr(p.err, kErrTokenRange);
            t = 0;
        }
        return t;
    };

    // the previous step's candidates
    unsigned long long best = 0ull;
    if (step > 0) {
        const unsigned long long *cand = p.cand + ((size_t)(step - 1) * p.max_batch + b) * p.head_grid;
        const int ncand = seq_head(p, b).cands;
        for (int w = tid; w < ncand; w += kBlock) {
            const unsigned long long c = cand[w];
            best = c > best ? c : best;
        }
    }
    // the vector the hidden half is made of: step 0, the caller's hidden state (bf16) or the head's own output of an
    // earlier call (float); later, x2 of the previous step, which first becomes h_hat = RMSNorm(x2; g_final)
    const bool from_x2 = step > 0, src_float = from_x2 || p.own_hidden;
    const float *xf = from_x2 ? p.dn + (size_t)b * d : p.hhat + (size_t)b * d;
    float x[kMaxNormIter][4], ev[kMaxNormIter][4];
    float sx = 0.f, sg = 0.f, se = 0.f;
#pragma unroll
    for (int it = 0; it < kMaxNormIter; ++it) {
        const int e = (it * kBlock + tid) * 4;
        if (e < d) {
            if (src_float) {
                const f32x4 raw = *reinterpret_cast<const f32x4 *>(xf + e);
                x[it][0] = raw.x;
                x[it][1] = raw.y;
                x[it][2] = raw.z;
                x[it][3] = raw.w;
            } else {
                load_bf16x4(p.hidden_in + (size_t)b * d, e, x[it]);
            }
        }
    }
    // the token whose embedding forms the other half, where it does not depend on the winner
    const bool early_tok = step < p.K && (step == 0 || p.forced != nullptr);
    int tok = 0;
    if (early_tok) tok = checked(step == 0 ? p.token_in[b] : p.forced[(size_t)b * (p.K - 1) + step - 1]);
    auto load_embed = [&]() {
        float s = 0.f;
#pragma unroll
        for (int it = 0; it < kMaxNormIter; ++it) {
            const int e = (it * kBlock + tid) * 4;
            if (e < d) {
                load_bf16x4(p.embed + (size_t)tok * d, e, ev[it]);
#pragma unroll
                for (int q = 0; q < 4; ++q) s += ev[it][q] * ev[it][q];
            }
        }
        return s;
    };
    if (early_tok) se = load_embed();
#pragma unroll
    for (int it = 0; it < kMaxNormIter; ++it) {
        const int e = (it * kBlock + tid) * 4;
        if (e < d) {
            float gf[4] = {1.f, 1.f, 1.f, 1.f};
            if (from_x2) load_bf16x4(p.g_final, e, gf);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                sx += x[it][q] * x[it][q];
                sg += (gf[q] * x[it][q]) * (gf[q] * x[it][q]);
            }
        }
    }
    // one reduction: three sums and the winner
    sx = wave_sum(sx);
    sg = wave_sum(sg);
    se = wave_sum(se);
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const unsigned long long o = __shfl_xor(best, off, kWave);
        best = o > best ? o : best;
    }
    if (lane == 0) {
        ra[wave] = sx;
        rb[wave] = sg;
        rc[wave] = se;
        rk[wave] = best;
    }
    __syncthreads();
    sx = sg = se = 0.f;
    best = 0ull;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        sx += ra[w];
        sg += rb[w];
        se += rc[w];
        best = rk[w] > best ? rk[w] : best;
    }
    int did = 0;
    if (from_x2) {
        did = key_token(p, b, best);
        if (tid == 0) p.draft_out[(size_t)b * p.K + step - 1] = seq_dead(p, b) ? -1 : did;
    }
    // h_hat = g_final * (x2 * inv1); its own mean square is inv1^2 * mean((g_final x2)^2) up to rounding, which saves a
    // second reduction
    const float inv1 = 1.0f / sqrtf(sx / (float)d + p.eps);
    const float inv2 = from_x2 ? 1.0f / sqrtf(inv1 * inv1 * sg / (float)d + p.eps) : inv1;
    float *ho = (from_x2 && p.hidden_out) ? p.hidden_out + ((size_t)b * p.K + step - 1) * d : nullptr;
#pragma unroll
    for (int it = 0; it < kMaxNormIter; ++it) {
        const int e = (it * kBlock + tid) * 4;
        if (e < d) {
            float h[4];
            if (from_x2) {
                float gf[4];
                load_bf16x4(p.g_final, e, gf);
#pragma unroll
                for (int q = 0; q < 4; ++q) h[q] = gf[q] * (x[it][q] * inv1);
                const f32x4 w = {h[0], h[1], h[2], h[3]};
                *reinterpret_cast<f32x4 *>(p.hhat + (size_t)b * d + e) = w;
                if (ho) *reinterpret_cast<f32x4 *>(ho + e) = w;
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) h[q] = x[it][q];
            }
            if (step < p.K) {
                float gh[4], o[4];
                load_bf16x4(p.g_h, e, gh);
#pragma unroll
                for (int q = 0; q < 4; ++q) o[q] = gh[q] * (h[q] * inv2);
                split_store(hi, lo, e, o);
            }
        }
    }
    if (step >= p.K) return;
    if (!early_tok) { // the winner is the next input token
        tok = checked(did);
        se = load_embed();
        se = wave_sum(se);
        __syncthreads(); // rc has been read by everyone
        if (lane == 0) rc[wave] = se;
        __syncthreads();
        se = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) se += rc[w];
    }
    const float inve = 1.0f / sqrtf(se / (float)d + p.eps);
#pragma unroll
    for (int it = 0; it < kMaxNormIter; ++it) {
        const int e = (it * kBlock + tid) * 4;
        if (e < d) {
            float ge[4], o[4];
            load_bf16x4(p.g_e, e, ge);
#pragma unroll
            for (int q = 0; q < 4; ++q) o[q] = ge[q] * (ev[it][q] * inve);
            split_store(hi + d, lo + d, e, o);
        }
    }
}

} // namespace mtp
