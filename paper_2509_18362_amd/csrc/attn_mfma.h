// Split-KV GQA attention of one new token over the draft cache on the matrix cores (gfx950), for long contexts
// and batches: the vector-ALU version in phases.h spends about 130 instructions per four tokens and is
// instruction-bound well below the HBM rate; here a wave spends that on thirty-two.
//
// Same work items, same outputs and same split partials as phase_attn (steps 5 and 6 of the draft step; Sec. 2.1: the
// MTP head is one decoder layer, here with grouped-query attention over its own KV cache).  A wave takes 32 tokens
// per iteration:
//   S^T = K Q^T   16x16x32 MFMAs with the 16 tokens of a tile as rows and the query heads of the KV head as columns
//                 (G of 16 used); K rows are loaded whole (coalesced) and turned into the operand layout (a lane
//                 holds HD/4 consecutive elements of its token) through a wave-private LDS strip; the query sits in
//                 registers as bf16 hi + lo, pre-multiplied by log2(e)/sqrt(HD).
//   online softmax in the MFMA result layout: a lane holds 2 x 4 tokens of ONE head column, so the running maximum,
//                 the rescale factor and the running sum are per-lane scalars; the maximum of a step is combined
//                 over the four lane groups of a column with two shuffles.
//   O^T += V^T P  with the 16 dimensions of a block as rows and the heads as columns, contraction over the 32 tokens.
//                 The eight probabilities a lane just computed are exactly the eight contraction elements the P
//                 operand wants from it (tokens 4g..4g+3 of both tiles: the assignment of tokens to MFMA depth slots
//                 is free as long as both operands agree), split into bf16 hi + lo.  V has to be transposed.  At
//                 head dimension 128 a lane's eight 16-byte loads hold eight dimensions of eight tokens: the score
//                 tiles' rows are permuted (K passes through LDS anyway) so that these are the tokens of the lane's
//                 eight probabilities, and the operand of output block j is element j of the eight loads (a byte
//                 permute per pair), no LDS.  At head dimension 64 the wave parks its 32 V rows in a private LDS
//                 strip (row stride HD*2 + 16 bytes, which spreads the four lane groups over different banks) and
//                 gathers eight 16-bit values per lane and block.
// Loads of the next iteration (16 KiB per wave) are in flight while the current one is computed.
// Items (sequence, KV head, split) are numbered split-major; when there are more of them than workgroups they are
// handed out through a counter and (one position per sequence) numbered longest first.  For a block of new positions whose keys and values are already in the cache, 16 / G
// positions of a sequence sit beside the G query heads in the columns and share every key/value read.
#pragma once
#include "phases.h"

namespace mtp {

// JP: positions of one sequence served together (a block of new positions whose keys and values are in the cache
// already): their query heads sit side by side in the MFMA columns, NC = G * JP of 16, and share every key/value read.
template <int G, int HD, int JP = 1>
struct AttnMfmaLds {
    static constexpr int VS = HD * 2 + 16;  // bytes per parked V row
    static constexpr bool VREG = HD == 128;  // V goes from the load registers straight into the MFMA operand
    static constexpr int NSTREAM = kWaves + 1; // one softmax stream per wave, one for the token being appended
    static constexpr int NC = G * JP;          // query columns: (position, head of the group)
    static_assert(NC <= 16, "the columns of one MFMA tile");
    float q[NC][HD];
    float cs[JP][HD / 2], sn[JP][HD / 2];
    float knew[HD], vnew[HD];
    float acc[NSTREAM][NC][HD];
    float ml[NSTREAM][NC][2];
    alignas(16) unsigned char v[VREG ? 1 : kWaves][VREG ? 1 : 32][VS];
    alignas(16) unsigned char k[kWaves][16][VS]; // one K tile per wave on its way into the MFMA operand layout
    int len[JP], last[JP];                       // JP > 1: the positions' lengths, and whose splits this item completed
};

// TICKET: as in phase_attn, the workgroup whose split of a (sequence, KV head) finishes last merges the splits.
// QUEUE (and p.attn_queue set): the workgroups draw their items from one counter (p.attn_queue[0]) instead of taking
// every nvb-th: contexts of a batch differ in length, the host does not know them, and a fixed assignment leaves the
// launch waiting for the workgroup that happened to get the long ones.  The counter only grows, so every workgroup
// draws a number past the end and leaves; the last one to leave (p.attn_queue[1] counts them) puts both words back
// to zero for the next launch.
// JP > 1 (needs p.kv_appended and TICKET): an item is (sequence, KV head, split, group of JP positions); position j of
// sequence b is row j * p.ext_B + b of the call and sees the cache up to its own slot, so the columns of an item differ
// only in where their tokens end.
// MAP (needs QUEUE with a counter, JP == 1): the items are numbered longest first (below).
template <int G, int HD, bool COH = false, bool TICKET = false, class Hook = NoHook, bool QUEUE = false, int JP = 1,
          bool MAP = false>
__device__ void phase_attn_mfma(const DraftParams &p, int step, int vb, int nvb, char *smem, Hook before_q = Hook()) {
    using L = AttnMfmaLds<G, HD, JP>;
    constexpr int NC = L::NC;
    static_assert(JP == 1 || TICKET, "blocks of positions merge their splits by ticket");
    constexpr int NS = HD / 32;        // MFMA depth steps over the head dimension
    constexpr int NDB = HD / 16;       // 16-dimension blocks of the output
    constexpr int LPT = HD / 8;        // lanes per V row in a wave-wide load
    constexpr int TPI = kWave / LPT;   // V rows per wave-wide load
    constexpr int NV = 32 / TPI;       // loads per lane for the 32 V rows of an iteration
    constexpr int NSTREAM = L::NSTREAM;
    constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
    L &s = *reinterpret_cast<L *>(smem);
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int i16 = lane & 15, g4 = lane >> 4;
    const int T = p.split_tokens, S = p.max_splits;
    const int nseq = JP > 1 ? p.ext_B : p.B;             // sequences whose caches are read
    const int mpos = JP > 1 ? p.B / p.ext_B : 1;         // positions per sequence
    const int JG = (mpos + JP - 1) / JP;                 // groups of positions
    int n_items = nseq * p.Hkv * S * JG;
    const float scale = 1.0f / sqrtf((float)HD);
    const int PW = HD + 2; // floats per (head, split) partial: acc[HD], max, sum

    int &drawn = *reinterpret_cast<int *>(smem + sizeof(L) + 4); // the number thread 0 drew, for the workgroup
    const bool queue = QUEUE && p.attn_queue != nullptr; // uniform
    // One position per sequence, more items than workgroups: the items are numbered longest first - every full split (T tokens) of every sequence,
    // split by split, then the sequences' ragged final splits by decreasing length - and only splits that exist get a
    // number.  Handed out in that order the workgroups end within a short item of one another; numbered (sequence, KV
    // head, split) over the longest possible context, a long context's last full splits were drawn last and the
    // launch waited 100 us for them (and every number without a split cost a trip to the counter).
    // The map (behind the flags, attn_map_bytes): every workgroup derives it from the lengths, identically.  (With an
    // item per workgroup at most the launch takes the kernel without the map: nothing to balance, and the map would
    // delay the first loads.)
    // (behind the tiles and flags and behind the strips of the merge, which start at the front of the LDS)
    const size_t map_at = (max(sizeof(L), (size_t)kWaves * S * sizeof(float)) + 64 + 15) / 16 * 16;
    int *len_l = reinterpret_cast<int *>(smem + map_at); // [nseq] tokens seen
    int *ord = len_l + nseq;                                     // [nseq] sequences by decreasing length
    int *ord_r = ord + nseq;                                     // [nseq] sequences by decreasing ragged length
    int *pre = ord_r + nseq;                                     // [S + 1] full splits with index < sp, all sequences
    int n_full = 0;                                              // full splits of all sequences
    static_assert(!MAP || (JP == 1 && QUEUE), "the item map serves one position per sequence, handed out by the counter");
    constexpr bool mapped = MAP;
    if constexpr (mapped) {
        for (int t = tid; t < nseq; t += kBlock) len_l[t] = (seq_dead(p, t) ? 0 : p.kv_len[t]) + step + 1;
        __syncthreads();
        for (int t = tid; t < nseq; t += kBlock) {
            const int lt = len_l[t], rt = lt % T;
            int rank = 0, rank_r = 0;
            for (int u = 0; u < nseq; ++u) {
                const int lu = len_l[u], ru = lu % T;
                rank += (lu > lt || (lu == lt && u < t)) ? 1 : 0;
                rank_r += (ru > rt || (ru == rt && u < t)) ? 1 : 0;
            }
            ord[rank] = t;
            ord_r[rank_r] = t;
        }
        for (int sp = tid; sp <= S; sp += kBlock) {
            int n = 0;
            for (int u = 0; u < nseq; ++u) n += min(len_l[u] / T, sp);
            pre[sp] = n;
        }
        __syncthreads();
        n_full = pre[S];
        int n_ragged = 0;
        for (int u = 0; u < nseq; ++u) n_ragged += (len_l[u] % T) != 0 ? 1 : 0;
        n_items = (n_full + n_ragged) * p.Hkv;
    }
    // items 0 .. nvb-1 are the workgroups' first ones, the counter hands out those from nvb on
    auto draw = [&]() { return nvb + __hip_atomic_fetch_add(p.attn_queue, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
    int item = vb, next_item = 0, pending = 0; // pending: thread 0's next number, asked for at the start of an item
    auto hand_out = [&]() {                     // and handed to the workgroup at its end
        if (tid == 0) drawn = pending;
        __syncthreads();
        const int v = drawn;
        __syncthreads(); // read by all before thread 0 writes the next one
        return v;
    };
    bool first_item = true;
    for (;; item = next_item) {
        if (queue) {
            if (item >= n_items) break;
            if (tid == 0) pending = draw(); // on its way while this item is worked on
        } else {
            if (item >= n_items) break;
            next_item = item + nvb;
        }
        // split-major numbering: the splits of one (sequence, KV head) land on workgroups of different XCDs, and with
        // the counter the short final splits are drawn last
        int kvh = item % p.Hkv, b = item / p.Hkv % nseq, jg = item / (p.Hkv * nseq) % JG, sp = item / (p.Hkv * nseq * JG);
        if constexpr (mapped) {
            const int m = item / p.Hkv;
            if (m < n_full) { // the m-th full split: the sequences that have split sp lead the order by length
                sp = 0;
                while (pre[sp + 1] <= m) ++sp;
                b = ord[m - pre[sp]];
            } else {
                b = ord_r[m - n_full];
                sp = len_l[b] / T;
            }
            // (read from LDS: said explicitly to be the same in every lane, so that what is derived from them - the
            // cache pointers, the loop bounds - stays in scalar registers)
            b = __builtin_amdgcn_readfirstlane(b);
            sp = __builtin_amdgcn_readfirstlane(sp);
        }
        bool dead;
        int len = 0;      // tokens the longest position of the item sees
        int lenj[JP];     // per position (0: not part of the block)
        if constexpr (JP == 1) {
            dead = seq_dead(p, b);
            len = lenj[0] = (dead ? 0 : p.kv_len[b]) + step + 1;
        } else {
#pragma unroll
            for (int jp = 0; jp < JP; ++jp) {
                const int j = jg * JP + jp, r = min(j, mpos - 1) * nseq + b;
                lenj[jp] = (j < mpos && !seq_dead(p, r)) ? p.kv_len[r] + step + 1 : 0;
                len = max(len, lenj[jp]);
            }
            dead = len == 0;
        }
        const int pnew = len - 1;
        const int nsplit = (len + T - 1) / T;
        // a row that is not part of the block, or a split past the end of this context (uniform for the workgroup)
        if ((p.kv_appended && dead) || sp >= nsplit) {
            if (queue) next_item = hand_out();
            continue;
        }
        const int t0 = sp * T, t1 = min(t0 + T, len);
        const bool last = (sp == nsplit - 1) && !p.kv_appended; // as in phase_attn
        const int ntok = last ? (t1 - 1 - t0) : (t1 - t0);      // slots read from the cache
        const int cb = p.kv_appended ? b % p.ext_B : b;          // whose cache
        const uint16_t *kc = p.k_cache + (((size_t)cb * p.Hkv + kvh) * p.cap + t0) * HD;
        const uint16_t *vc = p.v_cache + (((size_t)cb * p.Hkv + kvh) * p.cap + t0) * HD;
        const float *qkv = p.qkv + (size_t)b * p.qkv_dim;
        const int niter = (ntok + 31) / 32;

        u32x4 kn[2][NS], vr[NV];
        // K like V: a lane group of HD/8 lanes covers one row, so a load instruction reads whole rows (loaded
        // straight into the operand layout every lane would touch another row, four times the address-unit work)
        auto load_k = [&](int it) {
#pragma unroll
            for (int tl = 0; tl < 2; ++tl)
#pragma unroll
                for (int u = 0; u < NS; ++u) {
                    // past the end: the last row again (an empty range: the first slot, which is inside the cache)
                    const int tok = max(min(it * 32 + tl * 16 + u * TPI + lane / LPT, ntok - 1), 0);
                    kn[tl][u] = ldg16(kc + (size_t)tok * HD + (lane % LPT) * 8);
                }
        };
        auto load_v = [&](int it) {
#pragma unroll
            for (int u = 0; u < NV; ++u) {
                const int tok = max(min(it * 32 + u * TPI + lane / LPT, ntok - 1), 0);
                vr[u] = ldg16(vc + (size_t)tok * HD + (lane % LPT) * 8);
            }
        };
        auto load_iter = [&](int it) {
            load_k(it);
            load_v(it);
        };
        // in flight while q, the rotary table and the new key/value are prepared.  None of the requests of this kernel
        // sits behind a branch: a request past the wave's last iteration reads the range's last row again (every lane
        // the same row: next to no traffic).  Behind a branch the compiler cannot count the loads in flight and waits
        // for ALL of them wherever it waits for any: the wait for V then also waited for the keys of the next
        // iteration, requested a moment before, and an iteration lasted a whole trip to memory.
        load_iter(wave);
        if (first_item) {
            before_q();
            first_item = false;
        }

        __syncthreads(); // LDS of the previous item is free
        for (int idx = tid; idx < JP * (HD / 2); idx += kBlock) {
            const int jp = idx / (HD / 2), e = idx % (HD / 2);
            int pos = pnew; // JP == 1
            if constexpr (JP > 1) {
                pos = 0;
#pragma unroll
                for (int u = 0; u < JP; ++u) pos = u == jp ? max(lenj[u] - 1, 0) : pos;
            }
            rope_cos_sin(pos, p.rope_inv[e], s.cs[jp][e], s.sn[jp][e]);
        }
        if constexpr (JP > 1) {
#pragma unroll
            for (int u = 0; u < JP; ++u)
                if (tid == u) s.len[u] = lenj[u];
        }
        __syncthreads();
        for (int idx = tid; idx < NC * HD / 2; idx += kBlock) {
            const int c = idx / (HD / 2), jj = idx % (HD / 2), jp = c / G, gq = c % G;
            // the row the column's query comes from (a position past the block: any row, the column is not used)
            const int row = JP > 1 ? min(jg * JP + jp, mpos - 1) * nseq + b : b;
            const float *src = p.qkv + (size_t)row * p.qkv_dim + (size_t)(kvh * G + gq) * HD;
            float a = ld_f32<COH>(src + jj), bb = ld_f32<COH>(src + jj + HD / 2), cs = s.cs[jp][jj], sn = s.sn[jp][jj];
            if (p.b_q) {
                a += bf16_to_f32(p.b_q[(kvh * G + gq) * HD + jj]);
                bb += bf16_to_f32(p.b_q[(kvh * G + gq) * HD + jj + HD / 2]);
            }
            s.q[c][jj] = (a * cs - bb * sn) * scale;
            s.q[c][jj + HD / 2] = (bb * cs + a * sn) * scale;
        }
        if (last) {
            uint16_t *kdst = p.k_cache + (((size_t)b * p.Hkv + kvh) * p.cap + pnew) * HD;
            uint16_t *vdst = p.v_cache + (((size_t)b * p.Hkv + kvh) * p.cap + pnew) * HD;
            if (tid >= kWave * 4 && tid < kWave * 4 + HD / 2) {
                int e = tid - kWave * 4;
                const float *src = qkv + p.qd + (size_t)kvh * HD;
                float a = ld_f32<COH>(src + e), bb = ld_f32<COH>(src + e + HD / 2), cs = s.cs[0][e], sn = s.sn[0][e];
                if (p.b_k) {
                    a += bf16_to_f32(p.b_k[kvh * HD + e]);
                    bb += bf16_to_f32(p.b_k[kvh * HD + e + HD / 2]);
                }
                uint16_t r0 = f32_to_bf16(a * cs - bb * sn), r1 = f32_to_bf16(bb * cs + a * sn);
                s.knew[e] = bf16_to_f32(r0);
                s.knew[e + HD / 2] = bf16_to_f32(r1);
                if (!dead) {
                    st_u16<COH>(kdst + e, r0);
                    st_u16<COH>(kdst + e + HD / 2, r1);
                }
            } else if (tid >= kWave * 6 && tid < kWave * 6 + HD) {
                int e = tid - kWave * 6;
                float vraw = ld_f32<COH>(qkv + p.qd + p.kvd + (size_t)kvh * HD + e);
                if (p.b_v) vraw += bf16_to_f32(p.b_v[kvh * HD + e]);
                uint16_t r = f32_to_bf16(vraw);
                s.vnew[e] = bf16_to_f32(r);
                if (!dead) st_u16<COH>(vdst + e, r);
            }
        }
        __syncthreads();

        // the query operand: column i16 = (position, query head), depth slot g4 holds elements g4*HD/4 + 8u .. +8 for step u
        u32x4 qh[NS], ql[NS];
#pragma unroll
        for (int u = 0; u < NS; ++u) {
            uint32_t h[4] = {0u, 0u, 0u, 0u}, l[4] = {0u, 0u, 0u, 0u};
            if (i16 < NC) {
                const float *src = &s.q[i16 < NC ? i16 : 0][g4 * (HD / 4) + u * 8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    uint16_t hh, ll;
                    split_bf16(src[e] * kLog2e, hh, ll);
                    h[e >> 1] |= (uint32_t)hh << ((e & 1) * 16);
                    l[e >> 1] |= (uint32_t)ll << ((e & 1) * 16);
                }
            }
            qh[u] = u32x4{h[0], h[1], h[2], h[3]};
            ql[u] = u32x4{l[0], l[1], l[2], l[3]};
        }

        // tokens of the split this lane's column sees: all of them, or up to its own position's end
        int lim = ntok;
        if constexpr (JP > 1) lim = min(max(s.len[min(i16 / G, JP - 1)] - t0, 0), ntok);
        float mx = -INFINITY, lsum = 0.f; // of head column i16, in units of log2
        f32x4 oacc[NDB];
#pragma unroll
        for (int db = 0; db < NDB; ++db) oacc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
        unsigned char *vrow = &s.v[L::VREG ? 0 : wave][0][0], *krow = &s.k[wave][0][0];
        // which parked K row becomes row i16 of a score tile: with V in registers, row 4 g + e is token 4 e + g of the
        // tile, so that a lane's eight scores belong to the eight tokens whose V rows it loaded
        const int krd = L::VREG ? (i16 & 3) * 4 + (i16 >> 2) : i16;

        for (int it = wave; it < niter; it += kWaves) {
            // park the V rows, then request the next iteration's rows into the same registers
            if constexpr (!L::VREG) {
#pragma unroll
                for (int u = 0; u < NV; ++u)
                    *reinterpret_cast<u32x4 *>(vrow + (size_t)(u * TPI + lane / LPT) * L::VS + (lane % LPT) * 16) = vr[u];
            }
            // K through the wave's strip into the operand layout: row i16, elements g4*HD/4 + 8u .. +8 for step u
            u32x4 kcur[2][NS];
#pragma unroll
            for (int tl = 0; tl < 2; ++tl) {
#pragma unroll
                for (int u = 0; u < NS; ++u)
                    *reinterpret_cast<u32x4 *>(krow + (size_t)(u * TPI + lane / LPT) * L::VS + (lane % LPT) * 16) = kn[tl][u];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int u = 0; u < NS; ++u)
                    kcur[tl][u] = *reinterpret_cast<const u32x4 *>(krow + (size_t)krd * L::VS + g4 * (HD / 2) + u * 16);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
            load_k(it + kWaves);
            if constexpr (!L::VREG) load_v(it + kWaves);

            // scores of 2 x 16 tokens against the G heads
            f32x4 sc[2];
#pragma unroll
            for (int tl = 0; tl < 2; ++tl) {
                f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int u = 0; u < NS; ++u) {
                    a = mfma16(kcur[tl][u], qh[u], a);
                    a = mfma16(kcur[tl][u], ql[u], a);
                }
                sc[tl] = a;
            }
            float sv[8] = {sc[0].x, sc[0].y, sc[0].z, sc[0].w, sc[1].x, sc[1].y, sc[1].z, sc[1].w};
            float tmax = -INFINITY;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int tok = it * 32 + (L::VREG ? e * 4 + g4 : (e >> 2) * 16 + g4 * 4 + (e & 3));
                sv[e] = tok < lim ? sv[e] : -INFINITY;
                tmax = fmaxf(tmax, sv[e]);
            }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 16, kWave));
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
            const float mnew = fmaxf(mx, tmax); // finite for a column that has seen a token (others: -inf, weights 0)
            const float alpha = (mx == mnew) ? 1.0f : __builtin_amdgcn_exp2f(mx - mnew);
            mx = mnew;
            float pv[8], psum = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                pv[e] = sv[e] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(sv[e] - mnew);
                psum += pv[e];
            }
            lsum = lsum * alpha + psum;
            uint32_t ph[4], pl[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint16_t h0, l0, h1, l1;
                split_bf16(pv[2 * e], h0, l0);
                split_bf16(pv[2 * e + 1], h1, l1);
                ph[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                pl[e] = (uint32_t)l0 | ((uint32_t)l1 << 16);
            }
            const u32x4 pH = {ph[0], ph[1], ph[2], ph[3]}, pL = {pl[0], pl[1], pl[2], pl[3]};

            if constexpr (L::VREG) {
                // the lane's load u holds dimensions 8 i16 .. +8 of token 4 u + g4, the token whose probability sits in
                // pv[u]: output block db takes dimension 8 i16 + db as its row i16, its eight depth elements are
                // element db of the eight loads (a byte permute per pair), no LDS in between
#pragma unroll
                for (int db = 0; db < NDB; ++db) {
                    const uint32_t sel = (db & 1) ? 0x07060302u : 0x05040100u;
                    uint32_t w[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t a = vr[2 * e][db >> 1], c = vr[2 * e + 1][db >> 1];
                        w[e] = __builtin_amdgcn_perm(c, a, sel);
                    }
                    const u32x4 va = {w[0], w[1], w[2], w[3]};
                    f32x4 o = oacc[db] * alpha;
                    o = mfma16(va, pH, o);
                    o = mfma16(va, pL, o);
                    oacc[db] = o;
                }
                load_v(it + kWaves); // the registers are free again
            } else {
            // the parked rows were written by this wave's own lanes; LDS operations of a wave complete in order
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                // rows = dimensions db*16 + i16; depth slot g4, element e = token 4 g4 + e (e < 4) or 16 + 4 g4 + e - 4
                const unsigned char *col = vrow + (db * 16 + i16) * 2;
                uint32_t w[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ta = (e < 2 ? 0 : 16) + g4 * 4 + (2 * e & 3), tb = ta + 1;
                    const uint32_t a = *reinterpret_cast<const uint16_t *>(col + (size_t)ta * L::VS);
                    const uint32_t c = *reinterpret_cast<const uint16_t *>(col + (size_t)tb * L::VS);
                    w[e] = a | (c << 16);
                }
                const u32x4 va = {w[0], w[1], w[2], w[3]};
                f32x4 o = oacc[db] * alpha;
                o = mfma16(va, pH, o);
                o = mfma16(va, pL, o);
                oacc[db] = o;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            }
        }

        // ---- merge the waves (and the token being appended) through LDS ----
        lsum += __shfl_xor(lsum, 16, kWave);
        lsum += __shfl_xor(lsum, 32, kWave);
        if (i16 < NC) {
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                const float o[4] = {oacc[db].x, oacc[db].y, oacc[db].z, oacc[db].w};
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    s.acc[wave][i16][L::VREG ? 8 * (4 * g4 + v) + db : db * 16 + g4 * 4 + v] = o[v];
            }
            if (g4 == 0) {
                s.ml[wave][i16][0] = mx * kLn2;
                s.ml[wave][i16][1] = lsum;
            }
        }
        if constexpr (JP == 1) {
            if (wave < G) { // stream kWaves: the new token, score q . k_new from LDS
                float a = 0.f;
                for (int e = lane; e < HD; e += kWave) a += s.q[wave][e] * s.knew[e];
                a = wave_sum(a);
                if (lane == 0) {
                    s.ml[kWaves][wave][0] = last ? a : -INFINITY;
                    s.ml[kWaves][wave][1] = 1.0f;
                }
                for (int e = lane; e < HD; e += kWave) s.acc[kWaves][wave][e] = last ? s.vnew[e] : 0.f;
            }
        } else if (tid < NC) { // every key and value is in the cache: no stream of its own for a new token
            s.ml[kWaves][tid][0] = -INFINITY;
            s.ml[kWaves][tid][1] = 1.0f;
        }
        __syncthreads();
        for (int o = tid; o < NC * HD; o += kBlock) {
            const int c = o / HD, dd = o % HD, jp = c / G, g = c % G;
            // the column's row of the call, and its own number of splits
            int row = b, nsplit_c = nsplit;
            if constexpr (JP > 1) {
                const int len_c = s.len[jp];
                nsplit_c = (len_c + T - 1) / T;
                if (len_c == 0 || sp >= nsplit_c) continue; // not part of the block, or this split is past its end
                row = (jg * JP + jp) * nseq + b;
            }
            float M = -INFINITY;
            for (int st = 0; st < NSTREAM; ++st) M = fmaxf(M, s.ml[st][c][0]);
            float Ls = 0.f, A = 0.f;
            for (int st = 0; st < NSTREAM; ++st) {
                float mm = s.ml[st][c][0];
                if (mm != -INFINITY) {
                    float w = expf(mm - M);
                    Ls += s.ml[st][c][1] * w;
                    A += s.acc[st][c][dd] * w;
                }
            }
            int hq = kvh * G + g;
            if (nsplit_c == 1) {
                const float r = A / Ls;
                st_f32<COH>(p.attn + (size_t)row * p.qd + (size_t)hq * HD + dd, r);
                if (p.attn_split) {
                    uint16_t h, l;
                    split_bf16(r, h, l);
                    const size_t at = (size_t)row * p.a_stride + (size_t)hq * HD + dd;
                    p.attn_split[at] = h;
                    p.attn_split[p.a_lo + at] = l;
                }
            } else {
                float *dst = p.attn_part + (((size_t)row * p.Hq + hq) * S + sp) * PW;
                st_f32<COH || TICKET>(dst + dd, A);
                if (dd == 0) {
                    st_f32<COH || TICKET>(dst + HD, M);
                    st_f32<COH || TICKET>(dst + HD + 1, Ls);
                }
            }
        }
        if (TICKET && nsplit > 1) { // see phase_attn: relaxed ticket, partials written and read past the caches
            int &last_to_arrive = *reinterpret_cast<int *>(smem + sizeof(L));
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if constexpr (JP == 1) {
                if (tid == 0) {
                    int *ticket = p.attn_ticket + (size_t)b * p.Hkv + kvh;
                    const int old = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (old == nsplit - 1) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    last_to_arrive = (old == nsplit - 1) ? 1 : 0;
                }
                __syncthreads();
                const bool merges = last_to_arrive != 0;
                if (merges && wave < G)
                    merge_head<HD, true, COH>(p, b, kvh * G + wave, nsplit, reinterpret_cast<float *>(smem) + (size_t)wave * S);
            } else {
                // one ticket per (row, KV head): a position counts the splits up to its own end
                if (tid < JP) {
                    const int len_c = s.len[tid], ns = (len_c + T - 1) / T;
                    int done = 0;
                    if (len_c > 0 && sp < ns && ns > 1) {
                        int *ticket = p.attn_ticket + (size_t)((jg * JP + tid) * nseq + b) * p.Hkv + kvh;
                        const int old = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if (old == ns - 1) {
                            __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            done = 1;
                        }
                    }
                    s.last[tid] = done;
                }
                __syncthreads();
                // s.len and s.last sit behind the tiles, the strips of the merge at the front of the LDS
                for (int jp = 0; jp < JP; ++jp)
                    if (s.last[jp] && wave < G)
                        merge_head<HD, true, COH>(p, (jg * JP + jp) * nseq + b, kvh * G + wave, (s.len[jp] + T - 1) / T,
                                                  reinterpret_cast<float *>(smem) + (size_t)wave * S);
            }
            __syncthreads(); // the strips and the flag are free again before the next item touches the LDS
        }
        if (queue) next_item = hand_out();
    }
    if (queue && tid == 0) {
        const int left = __hip_atomic_fetch_add(p.attn_queue + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (left == nvb - 1) { // every workgroup has drawn its last number
            __hip_atomic_store(p.attn_queue, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(p.attn_queue + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (first_item) before_q();
}

} // namespace mtp
