// Host-side entry points of the batched path (kernels live in mtp_batch.hip, the caller in mtp_draft.hip).
#pragma once
#include <hip/hip_runtime.h>

#include "phases.h"

namespace mtp {

// dynamic LDS of a batched matrix phase whose row groups hold at most `rows_per_group` rows
size_t bgemv_lds_bytes(int rows_per_group);
// raises the dynamic-LDS limit of every batched kernel; false if a call failed
bool batch_allow_lds(size_t lds_limit);
// one batched matrix phase (BG_* index) for the sequences [p.b0, p.b0 + p.nb)
void launch_bgemv(int phase, const DraftParams &p, int step, int grid, size_t lds, hipStream_t st);
// workgroups of the separate epilogue kernel of a phase for `na` sequence tiles (at most 1024)
int batch_epilogue_grid(int phase, const DraftParams &p, int na);
// the preparation kernel before step `step` (step == K: after the last step), all sequences
void launch_bprep(const DraftParams &p, int step, hipStream_t st);

// a matrix phase (BG_* index) over all p.B rows as one tiled matrix product (rows_gemm.h); the output head leaves
// logits only, no candidates.  rows_gemm_serves: the phase's reduction length is a whole number of the tilings' rounds of steps
bool rows_gemm_serves(int phase, const DraftParams &p);
void launch_rows_gemm(int phase, const DraftParams &p, int step, int cus, hipStream_t st);

// matrix-core attention (attn_mfma.h): dynamic LDS, and the launch for query-group size G and head dimension HD
size_t attn_mfma_lds_bytes(int G, int HD);
void launch_attn_mfma(int G, int HD, const DraftParams &p, int step, int grid, size_t lds, hipStream_t st);
// the same for a block of new positions per sequence whose keys and values are in the cache (p.kv_appended, p.ext_B):
// positions_per_item = 16 / G positions of a sequence share its key/value reads
size_t attn_mfma_block_lds_bytes(int G, int HD);
void launch_attn_mfma_block(int G, int HD, const DraftParams &p, int step, int grid, size_t lds, hipStream_t st);

} // namespace mtp
