// The matrix phases over many rows at once (gfx950): one LDS-tiled matrix product on the matrix cores per phase, for
// calls with more rows than one pass of the batched core (batch.h) serves and no use for argmax candidates - the
// teacher-forced forward of Sec. 2.1, Eq. (1), whose output head runs over the whole vocabulary for every position.
// The batched core streams every weight once per 64 rows; here a weight tile is read once per block of BM rows and
// the blocks of one weight tile share an L2.
//
// A workgroup owns BM rows x BN weight rows of the result and walks the reduction in steps of 32 elements: both
// operands go through LDS (rows of 64 bytes padded to 80, which spreads the sixteen rows a quarter-wave reads over all
// banks), the next step's pieces are on their way from memory while the current one is multiplied, and each of the
// eight waves keeps a (BM/2) x (BN/4) piece in accumulators (MFMA tiles of 16 x 16), so one 16-byte LDS read feeds
// several MFMAs.  Activations are the bf16 hi + lo halves the producing phase left (the float value to 16 bits of
// mantissa): two MFMAs per weight fragment.  The phases and their epilogues are the batched core's (the Bg* structs:
// same operands, same result layout of a 16 x 16 tile), the output head is a variant that leaves logits only.
#pragma once
#include "batch.h"

namespace mtp {

constexpr int kRgBK = 32; // elements per reduction step
constexpr int kRgRound = 4; // the longest round of steps of any tiling (the host checks reduction lengths against it)
constexpr int kRgRow = kRgBK * 2 + 16; // bytes per LDS row

// 128 x 256 (the output head, gate/up at many rows): 80 KB, two workgroups per CU.  64 x 128: 40 KB; phases with
// 4096 weight rows still fill the chip at 512 rows.
template <int BM, int BN>
struct RowsGemmLds {
    alignas(16) unsigned char a_hi[2][BM][kRgRow];
    alignas(16) unsigned char a_lo[2][BM][kRgRow];
    alignas(16) unsigned char w[2][BN][kRgRow];
};

// workgroups of the launch for B rows and n weight rows: the M blocks of eight neighbouring N blocks form one group
template <int BM, int BN>
__host__ __device__ inline int rows_gemm_grid(int B, int n) {
    const int mb = (B + BM - 1) / BM, nb = (n + BN - 1) / BN;
    return (nb + 7) / 8 * 8 * mb;
}

// the output head for callers that want logits and no drafts: BgHead's operands, no candidates
struct BgHeadLogits : BgBase {
    static constexpr int WHICH = BG_LMHEAD;
    static constexpr bool STREAM = false, GATHER = true;
    static constexpr int SCALE = SSQ_X2;
    int step;
    __device__ BgHeadLogits(const DraftParams &p_, int step_) : BgBase(p_, p_.d, p_.n, p_.act[1]), step(step_) {
        ids = p_.ids;
    }
    __device__ __forceinline__ void tile(int vt, const uint16_t *&base, int &mat_rows, int &row0, int &row_end) const {
        base = p.lm_head;
        mat_rows = p.V;
        row_end = p.n;
        row0 = vt * 16;
    }
    __device__ __forceinline__ void epi(int bf, int vt, int j, const f32x4 (&s)[1], const float *scale) const {
        const int pos = vt * 16 + j;
        const float v[4] = {s[0].x, s[0].y, s[0].z, s[0].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int bl = bf + c;
            if (bl < p.nb && pos < p.n && p.logits_out)
                p.logits_out[((size_t)(p.b0 + bl) * p.K + step) * p.logit_stride + pos] = v[c] * scale[bl];
        }
    }
};

// pin: the DraftParams of the launch (all rows); the phase object is built on a copy whose (b0, nb) name the
// workgroup's rows, which is what the epilogues index with.
template <int BM, int BN, int PF, class Ph, class Make>
__device__ __forceinline__ void rows_gemm(const DraftParams &pin, Make make_phase, char *smem) {
    using L = RowsGemmLds<BM, BN>;
    constexpr int NMAT = Ph::NMAT;
    constexpr int TI = BM / 32, TJ = BN / 64;           // 16 x 16 tiles of a wave's piece
    static_assert(BN % 128 == 0, "weight rows per thread");
    static_assert(TJ % NMAT == 0, "pairs of tiles stay inside a wave's piece");
    L &s = *reinterpret_cast<L *>(smem);
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int i16 = lane & 15, g = lane >> 4;

    DraftParams p = pin;
    Ph ph = make_phase(p);
    const int K = ph.K, nk = K / kRgBK;
    const int ntv = ((ph.rows + 15) / 16) * NMAT; // virtual 16-row tiles
    const int MB = (pin.B + BM - 1) / BM, NB = (ntv * 16 + BN - 1) / BN;
    // Workgroups are dealt to the XCDs round robin.  The M blocks of one N block read the same weights: numbered
    // eight apart they run on the same XCD at about the same time, and its L2 serves all but the first.
    const int x = blockIdx.x, grp = x / (8 * MB), r = x % (8 * MB);
    const int mblk = r / 8, nblk = grp * 8 + (r & 7);
    if (nblk >= NB) return; // uniform
    p.b0 = mblk * BM;
    p.nb = min(BM, pin.B - p.b0);

    // global -> LDS: a thread moves 16-byte pieces of the 64-byte row slices, always chunk tid % 4 of its rows.
    // Activations, BM >= 128: rows tid / 4 (+ 128, ...), hi and lo of each; BM = 64: the lower half of the threads the
    // hi rows, the upper half the lo rows.  Weights: rows tid / 4 (+ 128, ...).
    constexpr int NAR = BM >= 128 ? BM / 128 : 1;  // activation rows per thread
    constexpr int NAP = BM >= 128 ? 2 * NAR : 1;   // activation pieces per thread (hi, lo of each row)
    constexpr int NWP = BN * 4 / kBlock;
    static_assert(BM == 64 || BM % 128 == 0, "activation rows per thread");
    const int lchunk = tid & 3;
    const bool upper = BM == 64 && tid >= kBlock / 2;
    const int arow = BM == 64 ? (tid & (kBlock / 2 - 1)) >> 2 : tid >> 2;
    const uint16_t *a_src[NAR];
#pragma unroll
    for (int i = 0; i < NAR; ++i)
        a_src[i] = ph.in + (size_t)min(p.b0 + arow + 128 * i, pin.B - 1) * p.a_stride + (upper ? p.a_lo : 0) + lchunk * 8;
    const int a_dst = (int)(upper ? offsetof(L, a_lo) : offsetof(L, a_hi)) + arow * kRgRow + lchunk * 16;
    const uint16_t *w_src[NWP];
#pragma unroll
    for (int h = 0; h < NWP; ++h) {
        const int n = nblk * BN + (tid >> 2) + 128 * h, vt = min(n >> 4, ntv - 1);
        const uint16_t *base;
        int mat_rows, row0, row_end;
        ph.tile(vt, base, mat_rows, row0, row_end);
        int wrow = min(row0 + (n & 15), row_end - 1);
        if (Ph::GATHER && ph.ids) wrow = ph.ids[wrow];
        w_src[h] = base + (size_t)wrow * K + lchunk * 8;
    }
    const int w_dst = (int)offsetof(L, w) + (tid >> 2) * kRgRow + lchunk * 16;
    constexpr int kStageA = BM * kRgRow, kStageW = BN * kRgRow; // a stage of each array
    // PF sets of registers: the pieces of step k + PF are requested while step k is multiplied and those of steps
    // k + 1 .. k + PF - 1 wait to be parked, so a request has PF steps' time to arrive (one step is shorter than a trip
    // to L2).  Requests past the last step repeat it (in bounds, parked into the buffer nobody reads any more): no
    // branch around a load, which would make the compiler wait for all loads in flight.  The host admits reduction
    // lengths of whole rounds of PF steps only.
    static_assert(PF % 2 == 0, "a round starts on LDS buffer 0");
    struct Pieces {
        u32x4 a[NAP], w[NWP];
    };
    auto fetch = [&](Pieces &q, int ks) {
        ks = min(ks, nk - 1);
#pragma unroll
        for (int i = 0; i < NAR; ++i) {
            q.a[i] = ldg16(a_src[i] + ks * kRgBK);
            if (NAP > 1) q.a[NAP - 1 - i] = ldg16(a_src[i] + p.a_lo + ks * kRgBK); // lo of row i in slot NAP-1-i
        }
#pragma unroll
        for (int h = 0; h < NWP; ++h) q.w[h] = ldg16(w_src[h] + ks * kRgBK);
    };
    auto park = [&](const Pieces &q, int st) {
        constexpr int kLo = (int)(offsetof(L, a_lo) - offsetof(L, a_hi));
#pragma unroll
        for (int i = 0; i < NAR; ++i) {
            *reinterpret_cast<u32x4 *>(smem + a_dst + i * 128 * kRgRow + st * kStageA) = q.a[i];
            if (NAP > 1) *reinterpret_cast<u32x4 *>(smem + a_dst + kLo + i * 128 * kRgRow + st * kStageA) = q.a[NAP - 1 - i];
        }
#pragma unroll
        for (int h = 0; h < NWP; ++h) *reinterpret_cast<u32x4 *>(smem + w_dst + h * 128 * kRgRow + st * kStageW) = q.w[h];
    };

    const int wm = wave >> 2, wn = wave & 3; // the wave's piece: rows (BM/2) wm .., weight rows (BN/4) wn ..
    f32x4 acc[TI][TJ];
#pragma unroll
    for (int ti = 0; ti < TI; ++ti)
#pragma unroll
        for (int tj = 0; tj < TJ; ++tj) acc[ti][tj] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto multiply = [&](int st) {
        u32x4 wf[TJ];
#pragma unroll
        for (int tj = 0; tj < TJ; ++tj)
            wf[tj] = *reinterpret_cast<const u32x4 *>(&s.w[st][(BN / 4) * wn + 16 * tj + i16][g * 16]);
#pragma unroll
        for (int ti = 0; ti < TI; ++ti) {
            const u32x4 ah = *reinterpret_cast<const u32x4 *>(&s.a_hi[st][(BM / 2) * wm + 16 * ti + i16][g * 16]);
            const u32x4 al = *reinterpret_cast<const u32x4 *>(&s.a_lo[st][(BM / 2) * wm + 16 * ti + i16][g * 16]);
#pragma unroll
            for (int tj = 0; tj < TJ; ++tj) {
                f32x4 a = acc[ti][tj];
                a = mfma16(ah, wf[tj], a);
                a = mfma16(al, wf[tj], a);
                acc[ti][tj] = a;
            }
        }
    };

    // s_b = 1/sqrt(mean(u_b^2) + eps) of the workgroup's rows from the producer's per-tile sums of squares: kBlock / BM
    // threads per row, asked for here (eight loads at a time) so that the epilogue finds it in a register
    constexpr int TPR = kBlock / BM;
    float my_scale = 0.f;
    if (Ph::SCALE >= 0) {
        const int npart = p.d / 16, sub = tid & (TPR - 1);
        const float *part = p.ssq + ((size_t)Ph::SCALE * p.max_batch + min(p.b0 + tid / TPR, pin.B - 1)) * npart;
        float sum = 0.f;
        for (int i0 = sub; i0 < npart; i0 += TPR * 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = i0 + u * TPR < npart ? part[i0 + u * TPR] : 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u) sum += v[u];
        }
#pragma unroll
        for (int off = 1; off < TPR; off <<= 1) sum += __shfl_xor(sum, off, kWave);
        my_scale = 1.0f / sqrtf(sum / (float)p.d + p.eps);
    }

    Pieces q[PF];
    fetch(q[0], 0);
    park(q[0], 0);
#pragma unroll
    for (int u = 1; u < PF; ++u) fetch(q[u], u);
    __syncthreads();
    for (int ks = 0; ks < nk; ks += PF) { // nk is a multiple of PF
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            fetch(q[u], ks + u + PF);             // q[u] held step ks + u, parked a step ago
            multiply(u & 1);
            park(q[(u + 1) % PF], (u + 1) & 1);   // step ks + u + 1; everyone left that buffer at the last barrier
            __syncthreads();
        }
    }

    // the tiles are dead: the rows' norm scales take their place (the barrier above ended the last reads)
    float *scale = reinterpret_cast<float *>(smem);
    if (Ph::SCALE >= 0) {
        if ((tid & (TPR - 1)) == 0) scale[tid / TPR] = my_scale;
        __syncthreads();
    }
    // D[i][j] of a 16 x 16 tile: lane (i16, g) holds rows 4 g + v (v = 0..3), weight row i16 - the batched core's layout
#pragma unroll
    for (int ti = 0; ti < TI; ++ti)
#pragma unroll
        for (int tj = 0; tj < TJ; tj += NMAT) {
            const int vt = (nblk * BN + (BN / 4) * wn + 16 * tj) >> 4;
            if (vt >= ntv) continue; // uniform per wave
            f32x4 sums[NMAT];
#pragma unroll
            for (int m = 0; m < NMAT; ++m) sums[m] = acc[ti][tj + m];
            ph.epi((BM / 2) * wm + 16 * ti + 4 * g, vt, i16, sums, scale);
        }
}

} // namespace mtp
