// Output head over many rows at once (gfx950): logits of RMSNorm(x2; g_final) against the listed rows of the LM head
// (Sec. 2.2, Eq. (3); with no list, against the whole vocabulary as the training objective of Sec. 2.1, Eq. (1)
// needs them) for every row of a block of positions, as ONE LDS-tiled matrix product on the matrix cores.
//
// The batched core (batch.h) serves 64 sequences per pass over the weights; a teacher-forced forward over hundreds of
// positions would stream the 1.2 GB of the full output head once per pass.  Here a workgroup owns a tile of 128
// positions x 256 head rows and walks the reduction in steps of 32 elements: both operands go through LDS (rows of
// 64 bytes padded to 80, which spreads the sixteen rows a quarter-wave reads over all banks), the next step's pieces
// are on their way from memory while the current one is multiplied, and every wave keeps a 64 x 64 piece of the tile
// in 16 accumulators (4 x 4 MFMA tiles of 16 x 16), so a 16-byte LDS read feeds four MFMAs.  Activations are the bf16
// hi + lo halves the down projection left (the float value to 16 bits of mantissa): two MFMAs per weight fragment.
// Only logits are produced (no argmax candidates): the caller is the training loss.
#pragma once
#include "phases.h"

namespace mtp {

constexpr int kHgBM = 128, kHgBN = 256, kHgBK = 32;
constexpr int kHgRow = kHgBK * 2 + 16; // bytes per LDS row

struct HeadGemmLds {
    alignas(16) unsigned char a_hi[2][kHgBM][kHgRow];
    alignas(16) unsigned char a_lo[2][kHgBM][kHgRow];
    alignas(16) unsigned char w[2][kHgBN][kHgRow];
    // 80 KB exactly: two workgroups share a CU's 160 KB.  The rows' norm scales sit in the padding of a_hi[0].
    __device__ float &scale(int row) { return *reinterpret_cast<float *>(&a_hi[0][row][kHgBK * 2]); }
};

// workgroups of the launch for B rows and n head rows: the M blocks of eight neighbouring N blocks form one group
__host__ __device__ inline int head_gemm_grid(int B, int n) {
    const int mb = (B + kHgBM - 1) / kHgBM, nb = (n + kHgBN - 1) / kHgBN;
    return (nb + 7) / 8 * 8 * mb;
}

__device__ __forceinline__ void phase_head_gemm(const DraftParams &p, int step, char *smem) {
    HeadGemmLds &s = *reinterpret_cast<HeadGemmLds *>(smem);
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int i16 = lane & 15, g = lane >> 4;
    const int MB = (p.B + kHgBM - 1) / kHgBM, NB = (p.n + kHgBN - 1) / kHgBN;
    // Workgroups are dealt to the XCDs round robin.  The M blocks of one N block read the same weights: numbered
    // eight apart they run on the same XCD at about the same time, and its L2 serves all but the first.
    const int x = blockIdx.x, grp = x / (8 * MB), r = x % (8 * MB);
    const int mblk = r / 8, nblk = grp * 8 + (r & 7);
    if (nblk >= NB) return; // uniform
    const int d = p.d, nk = d / kHgBK;

    // s_b = 1/sqrt(mean(x2_b^2) + eps) from the down projection's per-tile sums of squares, four threads per row
    {
        const int row = tid >> 2, sub = tid & 3, npart = d / 16;
        const int b = min(mblk * kHgBM + row, p.B - 1);
        const float *src = p.ssq + ((size_t)SSQ_X2 * p.max_batch + b) * npart;
        float sum = 0.f;
        for (int i = sub; i < npart; i += 4) sum += src[i];
        sum += __shfl_xor(sum, 1, kWave);
        sum += __shfl_xor(sum, 2, kWave);
        if (sub == 0) s.scale(row) = 1.0f / sqrtf(sum / (float)d + p.eps);
    }

    // global -> LDS: a thread moves 16 bytes of one activation row (hi and lo) and of two weight rows per step
    const int lrow = tid >> 2, lchunk = tid & 3;
    const int ab = min(mblk * kHgBM + lrow, p.B - 1);
    const uint16_t *a_src = p.act[1] + (size_t)ab * p.a_stride + lchunk * 8;
    const uint16_t *w_src[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int pos = min(nblk * kHgBN + lrow + 128 * h, p.n - 1);
        const int phys = p.ids ? p.ids[pos] : pos;
        w_src[h] = p.lm_head + (size_t)phys * d + lchunk * 8;
    }
    u32x4 ga_hi, ga_lo, gw[2];
    auto fetch = [&](int ks) {
        const int k0 = ks * kHgBK;
        ga_hi = ldg16(a_src + k0);
        ga_lo = ldg16(a_src + p.a_lo + k0);
        gw[0] = ldg16(w_src[0] + k0);
        gw[1] = ldg16(w_src[1] + k0);
    };
    auto park = [&](int st) {
        *reinterpret_cast<u32x4 *>(&s.a_hi[st][lrow][lchunk * 16]) = ga_hi;
        *reinterpret_cast<u32x4 *>(&s.a_lo[st][lrow][lchunk * 16]) = ga_lo;
        *reinterpret_cast<u32x4 *>(&s.w[st][lrow][lchunk * 16]) = gw[0];
        *reinterpret_cast<u32x4 *>(&s.w[st][lrow + 128][lchunk * 16]) = gw[1];
    };

    const int wm = wave >> 2, wn = wave & 3; // the wave's 64 x 64 piece: positions 64 wm .., head rows 64 wn ..
    f32x4 acc[4][4];
#pragma unroll
    for (int ti = 0; ti < 4; ++ti)
#pragma unroll
        for (int tj = 0; tj < 4; ++tj) acc[ti][tj] = f32x4{0.f, 0.f, 0.f, 0.f};

    fetch(0);
    park(0);
    __syncthreads();
    for (int ks = 0; ks < nk; ++ks) {
        const int st = ks & 1;
        if (ks + 1 < nk) fetch(ks + 1);
        u32x4 ah[4], al[4];
#pragma unroll
        for (int ti = 0; ti < 4; ++ti) {
            ah[ti] = *reinterpret_cast<const u32x4 *>(&s.a_hi[st][64 * wm + 16 * ti + i16][g * 16]);
            al[ti] = *reinterpret_cast<const u32x4 *>(&s.a_lo[st][64 * wm + 16 * ti + i16][g * 16]);
        }
#pragma unroll
        for (int tj = 0; tj < 4; ++tj) {
            const u32x4 wf = *reinterpret_cast<const u32x4 *>(&s.w[st][64 * wn + 16 * tj + i16][g * 16]);
#pragma unroll
            for (int ti = 0; ti < 4; ++ti) {
                f32x4 a = acc[ti][tj];
                a = mfma16(ah[ti], wf, a);
                a = mfma16(al[ti], wf, a);
                acc[ti][tj] = a;
            }
        }
        if (ks + 1 < nk) park(st ^ 1); // everyone left that buffer at the barrier of the step before
        __syncthreads();
    }

    // D[i][j]: lane (i16, g) holds position 4 g + v (v = 0..3) and head row i16 of every 16 x 16 tile
    if (!p.logits_out) return;
#pragma unroll
    for (int ti = 0; ti < 4; ++ti)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int ml = 64 * wm + 16 * ti + 4 * g + v, m = mblk * kHgBM + ml;
            if (m >= p.B) continue;
            const float sc = s.scale(ml);
            float *dst = p.logits_out + ((size_t)m * p.K + step) * p.logit_stride;
#pragma unroll
            for (int tj = 0; tj < 4; ++tj) {
                const int nn = nblk * kHgBN + 64 * wn + 16 * tj + i16;
                const float val = v == 0 ? acc[ti][tj].x : v == 1 ? acc[ti][tj].y : v == 2 ? acc[ti][tj].z : acc[ti][tj].w;
                if (nn < p.n) dst[nn] = val * sc;
            }
        }
}

} // namespace mtp
