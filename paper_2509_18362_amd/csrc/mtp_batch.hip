// Kernels of the batched draft path (two or more sequences per call) for gfx950.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "attn_mfma.h"
#include "batch.h"
#include "batch_launch.h"
#include "rows_gemm.h"

namespace mtp {
namespace {

// up to 16 sequences: the waves split the reduction; more: they split the tiles and share the activations in LDS
template <int NA, class Ph>
__device__ __forceinline__ void run_phase(const DraftParams &p, Ph &ph, int which, char *smem) {
    if constexpr (NA == 1)
        bgemv<1>(p, ph, p.bg_rg[which], p.bg_kp[which], smem);
    else
        bgemv_lds<NA>(p, ph, p.bg_rg[which], p.bg_kp[which], smem);
}

template <int PH, int NA>
__global__ __launch_bounds__(kBlock) void k_bgemv(DraftParams p, int step) {
    extern __shared__ __align__(16) char smem[];
    if constexpr (PH == BG_PROJ) {
        BgProj ph(p);
        run_phase<NA>(p, ph, PH, smem);
    } else if constexpr (PH == BG_QKV) {
        BgQkv ph(p);
        run_phase<NA>(p, ph, PH, smem);
    } else if constexpr (PH == BG_OPROJ) {
        BgOproj ph(p);
        run_phase<NA>(p, ph, PH, smem);
    } else if constexpr (PH == BG_GATEUP) {
        BgGateUp ph(p);
        run_phase<NA>(p, ph, PH, smem);
    } else if constexpr (PH == BG_DOWN) {
        BgDown ph(p);
        run_phase<NA>(p, ph, PH, smem);
    } else {
        BgHead ph(p, step);
        run_phase<NA>(p, ph, PH, smem);
    }
}

template <int PH, int NA>
__global__ __launch_bounds__(kBlock) void k_bepilogue(DraftParams p, int step) {
    __shared__ __align__(16) char smem[kWaves * kBatchMaxSeq * 8 + kBatchMaxSeq * 4];
    if constexpr (PH == BG_PROJ) {
        BgProj ph(p);
        phase_bepilogue<NA>(p, ph, p.bg_kp[PH], smem);
    } else if constexpr (PH == BG_QKV) {
        BgQkv ph(p);
        phase_bepilogue<NA>(p, ph, p.bg_kp[PH], smem);
    } else if constexpr (PH == BG_OPROJ) {
        BgOproj ph(p);
        phase_bepilogue<NA>(p, ph, p.bg_kp[PH], smem);
    } else if constexpr (PH == BG_GATEUP) {
        BgGateUp ph(p);
        phase_bepilogue<NA>(p, ph, p.bg_kp[PH], smem);
    } else if constexpr (PH == BG_DOWN) {
        BgDown ph(p);
        phase_bepilogue<NA>(p, ph, p.bg_kp[PH], smem);
    } else {
        BgHead ph(p, step);
        phase_bepilogue<NA>(p, ph, p.bg_kp[PH], smem);
    }
}

__global__ __launch_bounds__(kBlock) void k_bprep(DraftParams p, int step) {
    __shared__ __align__(16) char smem[256];
    phase_bprep(p, step, smem);
}

// a matrix phase over all p.B rows as one tiled matrix product (rows_gemm.h); at most 128 registers, so that two
// workgroups of the 80 KB tiling (four of the 40 KB one) share a CU
template <int PH>
__global__ __launch_bounds__(kBlock, 4) void k_rows_gemm(DraftParams p, int step) {
    extern __shared__ __align__(16) char smem[];
    if constexpr (PH == BG_PROJ)
        rows_gemm<64, 128, 4, BgProj>(p, [](const DraftParams &q) { return BgProj(q); }, smem);
    else if constexpr (PH == BG_QKV)
        rows_gemm<128, 128, 4, BgQkv>(p, [](const DraftParams &q) { return BgQkv(q); }, smem);
    else if constexpr (PH == BG_OPROJ)
        rows_gemm<64, 128, 4, BgOproj>(p, [](const DraftParams &q) { return BgOproj(q); }, smem);
    else if constexpr (PH == BG_GATEUP)
        rows_gemm<128, 128, 4, BgGateUp>(p, [](const DraftParams &q) { return BgGateUp(q); }, smem);
    else if constexpr (PH == BG_DOWN)
        rows_gemm<64, 128, 4, BgDown>(p, [](const DraftParams &q) { return BgDown(q); }, smem);
    else
        rows_gemm<128, 256, 2, BgHeadLogits>(p, [step](const DraftParams &q) { return BgHeadLogits(q, step); }, smem);
}

// q/k/v with the small tiles: for row counts whose small tiles still fit the chip one per CU
__global__ __launch_bounds__(kBlock, 4) void k_rows_gemm_qkv_small(DraftParams p, int step) {
    extern __shared__ __align__(16) char smem[];
    rows_gemm<64, 128, 4, BgQkv>(p, [](const DraftParams &q) { return BgQkv(q); }, smem);
}

template <int G, int HD>
__global__ __launch_bounds__(kBlock) void k_attn_mfma(DraftParams p, int step) {
    extern __shared__ __align__(16) char smem[];
    // merges its own splits (tickets), hands its items out one by one
    phase_attn_mfma<G, HD, false, true, NoHook, true>(p, step, blockIdx.x, gridDim.x, smem);
}

// the same with the items numbered longest first, for launches with more items than workgroups
template <int G, int HD>
__global__ __launch_bounds__(kBlock) void k_attn_mfma_lpt(DraftParams p, int step) {
    extern __shared__ __align__(16) char smem[];
    phase_attn_mfma<G, HD, false, true, NoHook, true, 1, true>(p, step, blockIdx.x, gridDim.x, smem);
}

// a block of new positions per sequence (keys and values already in the cache): the positions of a sequence share its
// key/value reads, 16 / G of them beside the G query heads in the MFMA columns
template <int G, int HD>
__global__ __launch_bounds__(kBlock) void k_attn_mfma_block(DraftParams p, int step) {
    extern __shared__ __align__(16) char smem[];
    phase_attn_mfma<G, HD, false, true, NoHook, true, 16 / G>(p, step, blockIdx.x, gridDim.x, smem);
}

typedef void (*bg_kernel_t)(DraftParams, int);
bg_kernel_t attn_mfma_block_kernel(int G, int HD) {
    if (HD == 128) {
        switch (G) {
        case 1: return k_attn_mfma_block<1, 128>;
        case 2: return k_attn_mfma_block<2, 128>;
        case 4: return k_attn_mfma_block<4, 128>;
        case 8: return k_attn_mfma_block<8, 128>;
        }
    } else if (HD == 64) {
        switch (G) {
        case 1: return k_attn_mfma_block<1, 64>;
        case 2: return k_attn_mfma_block<2, 64>;
        case 4: return k_attn_mfma_block<4, 64>;
        case 8: return k_attn_mfma_block<8, 64>;
        }
    }
    return nullptr;
}
// lpt: the launch hands its items out through the counter (more items than workgroups)
bg_kernel_t attn_mfma_kernel(int G, int HD, bool lpt) {
    if (HD == 128) {
        switch (G) {
        case 1: return lpt ? k_attn_mfma_lpt<1, 128> : k_attn_mfma<1, 128>;
        case 2: return lpt ? k_attn_mfma_lpt<2, 128> : k_attn_mfma<2, 128>;
        case 4: return lpt ? k_attn_mfma_lpt<4, 128> : k_attn_mfma<4, 128>;
        case 8: return lpt ? k_attn_mfma_lpt<8, 128> : k_attn_mfma<8, 128>;
        }
    } else if (HD == 64) {
        switch (G) {
        case 1: return lpt ? k_attn_mfma_lpt<1, 64> : k_attn_mfma<1, 64>;
        case 2: return lpt ? k_attn_mfma_lpt<2, 64> : k_attn_mfma<2, 64>;
        case 4: return lpt ? k_attn_mfma_lpt<4, 64> : k_attn_mfma<4, 64>;
        case 8: return lpt ? k_attn_mfma_lpt<8, 64> : k_attn_mfma<8, 64>;
        }
    }
    return nullptr;
}
template <int PH>
bg_kernel_t pick_na(int na) {
    return na == 1 ? k_bgemv<PH, 1> : na == 2 ? k_bgemv<PH, 2> : k_bgemv<PH, 4>;
}
bg_kernel_t pick(int phase, int na) {
    switch (phase) {
    case BG_PROJ: return pick_na<BG_PROJ>(na);
    case BG_QKV: return pick_na<BG_QKV>(na);
    case BG_OPROJ: return pick_na<BG_OPROJ>(na);
    case BG_GATEUP: return pick_na<BG_GATEUP>(na);
    case BG_DOWN: return pick_na<BG_DOWN>(na);
    default: return pick_na<BG_LMHEAD>(na);
    }
}
int tiles_for(int nb) { return nb <= 16 ? 1 : nb <= 32 ? 2 : 4; }
template <int PH>
bg_kernel_t pick_epilogue_na(int na) {
    return na == 1 ? k_bepilogue<PH, 1> : na == 2 ? k_bepilogue<PH, 2> : k_bepilogue<PH, 4>;
}
bg_kernel_t pick_epilogue(int phase, int na) {
    switch (phase) {
    case BG_PROJ: return pick_epilogue_na<BG_PROJ>(na);
    case BG_QKV: return pick_epilogue_na<BG_QKV>(na);
    case BG_OPROJ: return pick_epilogue_na<BG_OPROJ>(na);
    case BG_GATEUP: return pick_epilogue_na<BG_GATEUP>(na);
    case BG_DOWN: return pick_epilogue_na<BG_DOWN>(na);
    default: return pick_epilogue_na<BG_LMHEAD>(na);
    }
}

} // namespace

size_t bgemv_lds_bytes(int rows_per_group) { return batch_lds_bytes(rows_per_group); }

int batch_epilogue_grid(int phase, const DraftParams &p, int na) {
    const int rows = phase == BG_QKV ? p.qkv_dim : phase == BG_GATEUP ? p.F : phase == BG_LMHEAD ? p.n : p.d;
    const int slots = (rows + 15) / 16 * na;
    return std::min((slots + kWaves - 1) / kWaves, 1024);
}

size_t attn_mfma_lds_bytes(int G, int HD) {
    switch (HD * 16 + G) {
    case 128 * 16 + 1: return sizeof(AttnMfmaLds<1, 128>);
    case 128 * 16 + 2: return sizeof(AttnMfmaLds<2, 128>);
    case 128 * 16 + 4: return sizeof(AttnMfmaLds<4, 128>);
    case 128 * 16 + 8: return sizeof(AttnMfmaLds<8, 128>);
    case 64 * 16 + 1: return sizeof(AttnMfmaLds<1, 64>);
    case 64 * 16 + 2: return sizeof(AttnMfmaLds<2, 64>);
    case 64 * 16 + 4: return sizeof(AttnMfmaLds<4, 64>);
    case 64 * 16 + 8: return sizeof(AttnMfmaLds<8, 64>);
    }
    return 0;
}

size_t attn_mfma_block_lds_bytes(int G, int HD) {
    switch (HD * 16 + G) {
    case 128 * 16 + 1: return sizeof(AttnMfmaLds<1, 128, 16>);
    case 128 * 16 + 2: return sizeof(AttnMfmaLds<2, 128, 8>);
    case 128 * 16 + 4: return sizeof(AttnMfmaLds<4, 128, 4>);
    case 128 * 16 + 8: return sizeof(AttnMfmaLds<8, 128, 2>);
    case 64 * 16 + 1: return sizeof(AttnMfmaLds<1, 64, 16>);
    case 64 * 16 + 2: return sizeof(AttnMfmaLds<2, 64, 8>);
    case 64 * 16 + 4: return sizeof(AttnMfmaLds<4, 64, 4>);
    case 64 * 16 + 8: return sizeof(AttnMfmaLds<8, 64, 2>);
    }
    return 0;
}

void launch_attn_mfma(int G, int HD, const DraftParams &p, int step, int grid, size_t lds, hipStream_t st) {
    hipLaunchKernelGGL(attn_mfma_kernel(G, HD, p.attn_queue != nullptr), dim3(grid), dim3(kBlock), lds, st, p, step);
}
void launch_attn_mfma_block(int G, int HD, const DraftParams &p, int step, int grid, size_t lds, hipStream_t st) {
    hipLaunchKernelGGL(attn_mfma_block_kernel(G, HD), dim3(grid), dim3(kBlock), lds, st, p, step);
}

bool batch_allow_lds(size_t lds_limit) {
    bool ok = true;
    for (bg_kernel_t k : {k_rows_gemm<BG_GATEUP>, k_rows_gemm<BG_LMHEAD>})
        ok = ok && hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_limit) ==
                       hipSuccess;
    for (int hd = 64; hd <= 128; hd *= 2)
        for (int g = 1; g <= 8; g *= 2)
            ok = ok && hipFuncSetAttribute((const void *)attn_mfma_kernel(g, hd, false),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_limit) == hipSuccess &&
                 hipFuncSetAttribute((const void *)attn_mfma_kernel(g, hd, true),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_limit) == hipSuccess &&
                 hipFuncSetAttribute((const void *)attn_mfma_block_kernel(g, hd),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_limit) == hipSuccess;
    for (int ph = 0; ph < BG_COUNT; ++ph)
        for (int na = 1; na <= 4; na *= 2)
            ok = ok && hipFuncSetAttribute((const void *)pick(ph, na), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_limit) == hipSuccess;
    return ok;
}

void launch_bgemv(int phase, const DraftParams &p, int step, int grid, size_t lds, hipStream_t st) {
    const int na = tiles_for(p.nb);
    hipLaunchKernelGGL(pick(phase, na), dim3(grid), dim3(kBlock), lds, st, p, step);
    if (p.bg_sep[phase]) // one wave per (tile or pair of tiles, sequence tile)
        hipLaunchKernelGGL(pick_epilogue(phase, na),
                           dim3(phase == BG_LMHEAD ? p.head_grid : batch_epilogue_grid(phase, p, na)), dim3(kBlock), 0, st,
                           p, step);
}

bool rows_gemm_serves(int phase, const DraftParams &p) {
    const int K = phase == BG_PROJ ? 2 * p.d : phase == BG_OPROJ ? p.qd : phase == BG_DOWN ? p.F : p.d;
    return K % (kRgRound * kRgBK) == 0;
}
void launch_rows_gemm(int phase, const DraftParams &p, int step, int cus, hipStream_t st) {
    auto rows16 = [](int rows) { return (rows + 15) / 16 * 16; };
    auto small = [&](bg_kernel_t k, int n) {
        hipLaunchKernelGGL(k, dim3(rows_gemm_grid<64, 128>(p.B, n)), dim3(kBlock), sizeof(RowsGemmLds<64, 128>), st, p, step);
    };
    auto mid = [&](bg_kernel_t k, int n) {
        hipLaunchKernelGGL(k, dim3(rows_gemm_grid<128, 128>(p.B, n)), dim3(kBlock), sizeof(RowsGemmLds<128, 128>), st, p, step);
    };
    auto large = [&](bg_kernel_t k, int n) {
        hipLaunchKernelGGL(k, dim3(rows_gemm_grid<128, 256>(p.B, n)), dim3(kBlock), sizeof(RowsGemmLds<128, 256>), st, p, step);
    };
    switch (phase) {
    case BG_PROJ: small(k_rows_gemm<BG_PROJ>, p.d); break;
    case BG_QKV:
        // a tile count between one and two per CU costs two rounds: small tiles only while they fit one per CU
        if (rows_gemm_grid<64, 128>(p.B, rows16(p.qkv_dim)) <= cus)
            small(k_rows_gemm_qkv_small, rows16(p.qkv_dim));
        else
            mid(k_rows_gemm<BG_QKV>, rows16(p.qkv_dim));
        break;
    case BG_OPROJ: small(k_rows_gemm<BG_OPROJ>, p.d); break;
    case BG_GATEUP: mid(k_rows_gemm<BG_GATEUP>, 2 * rows16(p.F)); break;
    case BG_DOWN: small(k_rows_gemm<BG_DOWN>, p.d); break;
    default: large(k_rows_gemm<BG_LMHEAD>, rows16(p.n)); break;
    }
}

void launch_bprep(const DraftParams &p, int step, hipStream_t st) {
    hipLaunchKernelGGL(k_bprep, dim3(p.B), dim3(kBlock), 0, st, p, step);
}

} // namespace mtp
