// High-frequency vocabulary list from a token stream (gfx950): occurrence counts per id, the n most frequent ids
// (equal counts: lower id first), written in ascending id order - the list the compressed output head is gathered
// with (Sec. 2.2, which takes the frequent tokens of a language from statistics over a corpus; Eq. (3)).
//
// Counting is the only part that touches much memory.  Global atomics on a long-tailed stream would pile up on the
// few hottest ids (same-address device atomics serialize at ~40 ns each), so every workgroup counts in LDS: the
// vocabulary is cut into chunks of kChunkBins ids (160 000 bytes of 32-bit counters, all the LDS of a CU), a
// workgroup scans its slice of the stream once per chunk and adds its non-zero bins to the global counts at the
// end.  A 151 680-id vocabulary is four chunks, i.e. the stream is read four times (the later passes of a stream that
// fits the 256 MB memory-side cache are served from there).
// Selection: a radix select over the 32-bit counts (four passes of eight bits) finds the count T of the n-th most
// frequent id and how many ids with exactly that count belong to the list; the compaction then walks the ids in
// ascending order and keeps those with count > T plus the first ties, placing them by prefix sums - the output is
// born sorted, nothing is sorted.  Both are spread over 64 workgroups with small one-workgroup steps in between (a
// single compute unit reads memory at ~20 GB/s: as one workgroup these steps took 0.5 ms, more than the counting).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <mutex>

#include "../../include/mtp_draft.h"

namespace {

constexpr int kHistBlock = 512;
constexpr int kChunkBins = 40000;   // 160 000 bytes of LDS
constexpr int kSelBlock = 1024;


__global__ void k_subset_clear(unsigned *counts, int V, unsigned *state, int state_words, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < V) counts[i] = 0u;
    if (i < state_words) state[i] = i == 2 ? (unsigned)n : 0u; // [2]: ids still to be found by the selection
}

// grid (slices, chunks): workgroup (s, c) counts the ids of chunk c in slice s of the stream
__global__ __launch_bounds__(kHistBlock) void k_subset_hist(const int *__restrict__ tokens, long long n_tokens, int V,
                                                            unsigned *counts, unsigned *state) {
    extern __shared__ unsigned bins[];
    const int c0 = blockIdx.y * kChunkBins;
    const int nb = min(kChunkBins, V - c0);
    for (int i = threadIdx.x; i < nb; i += kHistBlock) bins[i] = 0u;
    __syncthreads();
    // slices of whole 16-byte groups; the last slice also takes the tail
    const long long groups = n_tokens / 4;
    const long long per = (groups + gridDim.x - 1) / gridDim.x;
    const long long g0 = min(groups, per * blockIdx.x), g1 = min(groups, g0 + per);
    unsigned invalid = 0u;
    const bool count_invalid = blockIdx.y == 0;
    auto one = [&](int t) {
        const unsigned rel = (unsigned)(t - c0);
        if (rel < (unsigned)nb) atomicAdd(&bins[rel], 1u);
        if (count_invalid && (unsigned)t >= (unsigned)V) ++invalid;
    };
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    const i32x4 *t4 = reinterpret_cast<const i32x4 *>(tokens);
    for (long long g = g0 + threadIdx.x; g < g1; g += kHistBlock) {
        const i32x4 v = t4[g];
        one(v.x);
        one(v.y);
        one(v.z);
        one(v.w);
    }
    if (blockIdx.x == gridDim.x - 1)
        for (long long i = groups * 4 + threadIdx.x; i < n_tokens; i += kHistBlock) one(tokens[i]);
    if (count_invalid) {
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) invalid += __shfl_xor(invalid, off, 64);
        if ((threadIdx.x & 63) == 0 && invalid) atomicAdd(&state[0], invalid);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nb; i += kHistBlock) {
        const unsigned v = bins[i];
        if (v) atomicAdd(&counts[c0 + i], v);
    }
}

// ---- selection: T = the n-th largest count, r = how many ids with count == T belong to the n most frequent ----
// (1 <= r when n >= 1; #(count > T) = n - r).  A radix select, most significant byte first: a pass histograms byte
// `pass` of the counts that agree with the prefix found so far (kSelGroups workgroups, each in LDS first), a
// one-workgroup step then walks the 256 buckets from the top to the one that holds the n-th largest.  One compute unit
// reads only ~20 GB/s, so everything that touches all V counts is spread over many workgroups.
constexpr int kSelGroups = 64;
// state: [0] invalid ids, [1] prefix (finally T), [2] still needed (finally r), then 4 x 256 bucket counts, then
// per-workgroup (above, ties) totals of the compaction
constexpr int kStateHist = 8, kStateTotals = kStateHist + 4 * 256, kStateWordsFull = kStateTotals + 2 * kSelGroups;

__global__ __launch_bounds__(kSelBlock) void k_subset_sel_hist(const unsigned *__restrict__ counts, int V, int pass,
                                                               unsigned *state) {
    __shared__ unsigned hist[256];
    if (threadIdx.x < 256) hist[threadIdx.x] = 0u;
    __syncthreads();
    const int shift = 24 - 8 * pass;
    const unsigned mask = pass == 0 ? 0u : 0xffffffffu << (shift + 8), prefix = state[1];
    const int per = (V + gridDim.x - 1) / gridDim.x, v0 = blockIdx.x * per, v1 = min(V, v0 + per);
    for (int v = v0 + threadIdx.x; v < v1; v += kSelBlock) {
        const unsigned c = counts[v];
        if ((c & mask) == prefix) atomicAdd(&hist[(c >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (threadIdx.x < 256 && hist[threadIdx.x]) atomicAdd(&state[kStateHist + pass * 256 + threadIdx.x], hist[threadIdx.x]);
}

__global__ void k_subset_sel_walk(int pass, unsigned *state) { // one workgroup of 256 threads
    __shared__ unsigned hist[256];
    hist[threadIdx.x] = state[kStateHist + pass * 256 + threadIdx.x];
    __syncthreads();
    if (threadIdx.x != 0) return;
    unsigned need = state[2], acc = 0u;
    int b = 255;
    for (; b > 0; --b) { // from the largest byte value down to the bucket that holds the n-th largest
        if (acc + hist[b] >= need) break;
        acc += hist[b];
    }
    state[2] = need - acc;
    state[1] |= (unsigned)b << (24 - 8 * pass);
}

// inclusive scan of one value per thread over the workgroup; scratch holds one word per wave; returns the total too
__device__ __forceinline__ unsigned block_scan(unsigned v, unsigned *scratch, unsigned &total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const unsigned o = __shfl_up(v, off, 64);
        if (lane >= off) v += o;
    }
    __syncthreads(); // scratch of the previous scan has been read
    if (lane == 63) scratch[wave] = v;
    __syncthreads();
    unsigned base = 0u, tot = 0u;
    for (int w = 0; w < kSelBlock / 64; ++w) {
        const unsigned s = scratch[w];
        if (w < wave) base += s;
        tot += s;
    }
    total = tot;
    return v + base;
}

// ---- compaction: the ids in ascending order, those with count > T plus the first r ties ----
// Workgroup g owns a contiguous range of ids.  First every workgroup counts its (above, ties); then it adds up what the
// workgroups before it hold (at most kSelGroups pairs) and places its own ids by two workgroup scans.
__global__ __launch_bounds__(kSelBlock) void k_subset_cmp_count(const unsigned *__restrict__ counts, int V,
                                                                unsigned *state) {
    __shared__ unsigned scratch[kSelBlock / 64];
    const unsigned T = state[1];
    const int per = (V + gridDim.x - 1) / gridDim.x, v0 = blockIdx.x * per, v1 = min(V, v0 + per);
    unsigned above = 0u, ties = 0u;
    for (int v = v0 + threadIdx.x; v < v1; v += kSelBlock) {
        const unsigned c = counts[v];
        above += c > T ? 1u : 0u;
        ties += c == T ? 1u : 0u;
    }
    unsigned ta, tt;
    (void)block_scan(above, scratch, ta);
    (void)block_scan(ties, scratch, tt);
    if (threadIdx.x == 0) {
        state[kStateTotals + 2 * blockIdx.x] = ta;
        state[kStateTotals + 2 * blockIdx.x + 1] = tt;
    }
}

__global__ __launch_bounds__(kSelBlock) void k_subset_cmp_write(const unsigned *__restrict__ counts, int V, int n,
                                                                const unsigned *__restrict__ state, int *ids_out) {
    __shared__ unsigned scratch[kSelBlock / 64];
    const unsigned T = state[1], r = state[2];
    unsigned above_before = 0u, ties_before = 0u; // uniform
    for (int g = 0; g < (int)blockIdx.x; ++g) {
        above_before += state[kStateTotals + 2 * g];
        ties_before += state[kStateTotals + 2 * g + 1];
    }
    unsigned out_before = above_before + min(ties_before, r); // the first r ties in id order are kept
    const int per = (V + gridDim.x - 1) / gridDim.x, v0 = blockIdx.x * per, v1 = min(V, v0 + per);
    for (int vb = v0; vb < v1; vb += kSelBlock) {
        const int v = vb + threadIdx.x;
        const unsigned c = v < v1 ? counts[v] : 0u;
        const bool tie = v < v1 && c == T, above = v < v1 && c > T;
        unsigned tie_total, sel_total;
        const unsigned tie_incl = block_scan(tie ? 1u : 0u, scratch, tie_total);
        const bool take = above || (tie && ties_before + tie_incl <= r);
        const unsigned sel_incl = block_scan(take ? 1u : 0u, scratch, sel_total);
        if (take) {
            const unsigned pos = out_before + sel_incl - 1u;
            if (pos < (unsigned)n) ids_out[pos] = v;
        }
        ties_before += tie_total;
        out_before += sel_total;
    }
}

__global__ void k_subset_export(const unsigned *counts, int V, const unsigned *state, int *counts_out,
                                int *invalid_out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (counts_out && i < V) counts_out[i] = (int)counts[i];
    if (invalid_out && i == 0) invalid_out[0] = (int)state[0];
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- scratch of the entry point that allocates nothing ----------------------------------------------------------
// Counts and selection state of mtp_subset_build_static live in this array instead of a caller's workspace.  Each GPU
// the library runs on holds its own copy at its own address until the process ends; host code reaches it only through
// the per-device pointer below (the array's name is a host-side stand-in, not a device address).
constexpr int kStaticMaxVocab = 262144;
constexpr int kStateWordsFullStatic = 8 + 4 * 256 + 2 * 64; // = kStateWordsFull (spelled out: used in the array bound)
__device__ __align__(256) unsigned scratch[kStaticMaxVocab + kStateWordsFullStatic];
static_assert(kStateWordsFullStatic == kStateWordsFull, "scratch layout");
constexpr int kMaxDevices = 64;
unsigned *g_scratch_ptr[kMaxDevices]; // per device: address of that device's copy of `scratch`, null until looked up
bool g_lds_allowed[kMaxDevices];      // per device: the counting kernel may use all the LDS of a CU
std::mutex g_setup_mutex;

// once per device, with that device current: raise the LDS limit of the counting kernel and (for the static entry
// point) look up the device's copy of the scratch array
int32_t subset_setup(int dev, bool want_scratch, unsigned **scratch_out) {
    if (dev < 0 || dev >= kMaxDevices) return MTP_ERR_CONFIG;
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    if (!g_lds_allowed[dev]) {
        if (hipFuncSetAttribute((const void *)k_subset_hist, hipFuncAttributeMaxDynamicSharedMemorySize,
                                kChunkBins * 4) != hipSuccess) {
            (void)hipGetLastError();
            return MTP_ERR_HIP;
        }
        g_lds_allowed[dev] = true;
    }
    if (want_scratch) {
        if (!g_scratch_ptr[dev]) {
            unsigned *ptr = nullptr;
            if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
                (void)hipGetLastError();
                return MTP_ERR_HIP;
            }
            g_scratch_ptr[dev] = ptr;
        }
        *scratch_out = g_scratch_ptr[dev];
    }
    return MTP_OK;
}

// everything after the argument checks: `work` holds V counts followed by the selection state
int32_t subset_build_on(const int32_t *tokens, int64_t n_tokens, int32_t V, int32_t n, unsigned *work, int dev,
                        int32_t *ids_out, int32_t *counts_out, int32_t *invalid_out, hipStream_t st) {
    unsigned *counts = work;
    unsigned *state = counts + V;
    hipLaunchKernelGGL(k_subset_clear, dim3((V + kStateWordsFull + 255) / 256), dim3(256), 0, st, counts, V, state,
                       kStateWordsFull, n);
    int cus = 256;
    (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    const int chunks = (V + kChunkBins - 1) / kChunkBins;
    hipLaunchKernelGGL(k_subset_hist, dim3(cus, chunks), dim3(kHistBlock), kChunkBins * 4, st, tokens,
                       (long long)n_tokens, V, counts, state);
    if (n > 0) {
        for (int pass = 0; pass < 4; ++pass) {
            hipLaunchKernelGGL(k_subset_sel_hist, dim3(kSelGroups), dim3(kSelBlock), 0, st, counts, V, pass, state);
            hipLaunchKernelGGL(k_subset_sel_walk, dim3(1), dim3(256), 0, st, pass, state);
        }
        hipLaunchKernelGGL(k_subset_cmp_count, dim3(kSelGroups), dim3(kSelBlock), 0, st, counts, V, state);
        hipLaunchKernelGGL(k_subset_cmp_write, dim3(kSelGroups), dim3(kSelBlock), 0, st, counts, V, n, state, ids_out);
    }
    if (counts_out || invalid_out)
        hipLaunchKernelGGL(k_subset_export, dim3((V + 255) / 256), dim3(256), 0, st, counts, V, state, counts_out,
                           invalid_out);
    if (hipGetLastError() != hipSuccess) return MTP_ERR_HIP;
    return MTP_OK;
}

int32_t subset_check_args(const int32_t *tokens, int64_t n_tokens, int32_t vocab_size, int32_t n, const int32_t *ids_out,
                          const int32_t *counts_out, const int32_t *invalid_out) {
    if ((!tokens && n_tokens > 0) || (!ids_out && n > 0)) return MTP_ERR_NULL;
    if (!aligned16(tokens) || !aligned16(ids_out) || !aligned16(counts_out) || !aligned16(invalid_out))
        return MTP_ERR_ALIGN;
    if (vocab_size < 1 || n < 0 || n > vocab_size || n_tokens < 0 || n_tokens >= ((int64_t)1 << 31))
        return MTP_ERR_CONFIG;
    return MTP_OK;
}

} // namespace

extern "C" {

size_t mtp_subset_workspace_bytes(int32_t vocab_size) {
    if (vocab_size < 1) return 0;
    return ((size_t)vocab_size + kStateWordsFull) * 4;
}

int32_t mtp_subset_build(const int32_t *tokens, int64_t n_tokens, int32_t vocab_size, int32_t n, void *workspace,
                         size_t workspace_bytes, int32_t *ids_out, int32_t *counts_out, int32_t *invalid_out,
                         void *hip_stream) {
    if (!workspace) return MTP_ERR_NULL;
    if (!aligned16(workspace)) return MTP_ERR_ALIGN;
    const int32_t rc = subset_check_args(tokens, n_tokens, vocab_size, n, ids_out, counts_out, invalid_out);
    if (rc != MTP_OK) return rc;
    if (workspace_bytes < mtp_subset_workspace_bytes(vocab_size)) return MTP_ERR_WORKSPACE;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MTP_ERR_HIP;
    const int32_t rs = subset_setup(dev, false, nullptr);
    if (rs != MTP_OK) return rs;
    return subset_build_on(tokens, n_tokens, vocab_size, n, static_cast<unsigned *>(workspace), dev, ids_out, counts_out,
                           invalid_out, static_cast<hipStream_t>(hip_stream));
}

int32_t mtp_subset_static_max_vocab(void) { return kStaticMaxVocab; }

int32_t mtp_subset_build_static(const int32_t *tokens, int64_t n_tokens, int32_t vocab_size, int32_t n,
                                int32_t *ids_out, int32_t *counts_out, int32_t *invalid_out, void *hip_stream) {
    const int32_t rc = subset_check_args(tokens, n_tokens, vocab_size, n, ids_out, counts_out, invalid_out);
    if (rc != MTP_OK) return rc;
    if (vocab_size > kStaticMaxVocab) {
        fprintf(stderr, "mtp_subset_build_static: vocab_size %d exceeds the built-in scratch (%d ids); use "
                        "mtp_subset_build with a workspace\n", (int)vocab_size, kStaticMaxVocab);
        return MTP_ERR_WORKSPACE;
    }
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MTP_ERR_HIP;
    unsigned *work = nullptr;
    const int32_t rs = subset_setup(dev, true, &work); // first call on a device: symbol lookup; later: a table read
    if (rs != MTP_OK) return rs;
    return subset_build_on(tokens, n_tokens, vocab_size, n, work, dev, ids_out, counts_out, invalid_out,
                           static_cast<hipStream_t>(hip_stream));
}

} // extern "C"
