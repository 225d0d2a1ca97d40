// High-frequency vocabulary list from a token stream (gfx950): occurrence counts per id, the n most frequent ids
// (equal counts: lower id first), written in ascending id order - the list the compressed output head is gathered
// with (Sec. 2.2, which takes the frequent tokens of a language from statistics over a corpus; Eq. (3)).
//
// Counting is the only part that touches much memory.  Global atomics on a long-tailed stream would pile up on the
// few hottest ids (same-address device atomics serialize at ~40 ns each), so every workgroup counts in LDS.  The bins
// are 16 bits wide, two to a word (an LDS atomic adds 1 or 65536 to the word), so that all the LDS of a CU (160 000
// bytes) holds 80 000 ids and a 151 680-id vocabulary is two chunks: the stream is read twice (with 32-bit bins it was
// read four times).  A field cannot overflow: a workgroup scans its slice in blocks of 49 152 tokens, and between two
// blocks it sweeps its bins (16 bytes per read) and moves every field that has reached 16 384 to the global counts
// (few fields ever do).  At the end a workgroup stores its bins as they are and a second kernel adds the workgroups'
// copies up (every workgroup adding its non-zero fields to the global counts with atomics took longer than the counting;
// the entry point without a workspace still does that).  Every thread keeps the four 16-byte loads of the next round in
// flight while it counts.
// Selection: a radix select over the 32-bit counts (three passes of 11, 11 and 10 bits) finds the count T of the n-th
// most frequent id and how many ids with exactly that count belong to the list; the compaction then walks the ids in
// ascending order and keeps those with count > T plus the first ties, placing them by prefix sums - the output is
// born sorted, nothing is sorted.  Both are spread over 64 workgroups (a single compute unit reads memory at
// ~20 GB/s: as one workgroup these steps took 0.5 ms, more than the counting); the walk over a pass's buckets is done by
// every workgroup of the kernel that follows, as a scan (as a kernel of its own with a serial loop it took 13 us a pass).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <mutex>

#include "../../include/mtp_draft.h"

namespace {

constexpr int kHistBlock = 1024;
constexpr int kChunkIds = 80000;     // ids per chunk: 40 000 words of LDS, two 16-bit bins each
constexpr int kSweepBlock = 49152;   // tokens a workgroup counts between two sweeps
constexpr unsigned kSweepAt = 16384; // a sweep moves the fields that have reached this: 16 383 + 49 152 < 65 536
constexpr int kSelBlock = 1024;

__global__ void k_subset_clear(unsigned *counts, int V, unsigned *state, int state_words, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < V) counts[i] = 0u;
    if (i < state_words) state[i] = i == 2 ? (unsigned)n : 0u; // [2]: ids still to be found by the selection
}

// grid (slices, chunks): workgroup (s, c) counts the ids of chunk c in slice s of the stream.
// What bounds it (measured on streams of 2^26 tokens, uniform or long-tailed alike): the LDS retires about one lane's
// atomic per clock and CU, whatever the addresses - 109 us for 2^26 tokens over 256 CUs - and the vector instructions
// around an atomic (range check, address, increment) come on top; reading the stream twice takes 77 us and hides behind
// them.  Counting a stream's few hottest ids apart, per wave in scalar registers (they are what an LDS atomic is replayed
// for when lanes share an address), was built and measured: each compare per token costs more than the replays it saves.
__global__ __launch_bounds__(kHistBlock) void k_subset_hist(const int *__restrict__ tokens, long long n_tokens, int V,
                                                            unsigned *counts, unsigned *state, unsigned *partials) {
    extern __shared__ unsigned bins[]; // word w: ids c0 + 2 w (low half) and c0 + 2 w + 1 (high half)
    __shared__ unsigned invalid_wg;
    const int c0 = blockIdx.y * kChunkIds;
    const int nb = min(kChunkIds, V - c0), nw = (nb + 1) / 2, nw4 = (nw + 3) / 4 * 4; // (LDS holds kChunkIds / 2 words)
    for (int i4 = threadIdx.x * 4; i4 < nw4; i4 += kHistBlock * 4)
        *reinterpret_cast<uint4 *>(bins + i4) = uint4{0u, 0u, 0u, 0u};
    if (threadIdx.x == 0) invalid_wg = 0u;
    __syncthreads();
    // slices of whole 16-byte groups; the last slice also takes the tail
    const long long groups = n_tokens / 4;
    const long long per = (groups + gridDim.x - 1) / gridDim.x;
    const long long g0 = min(groups, per * blockIdx.x), g1 = min(groups, g0 + per);
    const bool count_invalid = blockIdx.y == 0;
    unsigned invalid = 0u; // uniform: ids outside the vocabulary this WAVE has seen
    auto popcount = [](unsigned long long m) { // kept where it is written (the compiler would collect the lane masks of
        unsigned c;                            // a whole round first, which do not fit the scalar registers)
        asm volatile("s_bcnt1_i32_b64 %0, %1" : "=s"(c) : "s"(m));
        return c;
    };
    // one token per lane; live: the lane holds a token (all lanes of the wave call this together)
    auto one = [&](int t, bool live) {
        const unsigned rel = (unsigned)(t - c0);
        if (live && rel < (unsigned)nb) atomicAdd(&bins[rel >> 1], 1u << ((rel & 1u) * 16u));
        if (count_invalid) invalid += popcount(__builtin_amdgcn_ballot_w64(live && (unsigned)t >= (unsigned)V));
    };
    // moves the fields of at least `at` to the global counts (at = 1: all that is left)
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    auto sweep = [&](unsigned at) {
        __syncthreads();
        if (at == 1u) { // everything that is left: consecutive lanes take consecutive words (the global atomics of a
            for (int i = threadIdx.x; i < nw; i += kHistBlock) { // wave then fall into few cache lines)
                const unsigned w = bins[i], lo = w & 0xffffu, hi = w >> 16;
                if (lo) atomicAdd(&counts[c0 + 2 * i], lo);
                if (hi) atomicAdd(&counts[c0 + 2 * i + 1], hi);
            }
            return;
        }
        const unsigned probe = 0xc000c000u; // kSweepAt = 2^14: a field at or above it has one of its two top bits set
        for (int i4 = threadIdx.x * 4; i4 < nw4; i4 += kHistBlock * 4) {
            u32x4 w4 = *reinterpret_cast<u32x4 *>(bins + i4);
            if (((w4.x | w4.y | w4.z | w4.w) & probe) == 0u) continue;
            unsigned w[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int i = i4 + q;
                const unsigned lo = w[q] & 0xffffu, hi = w[q] >> 16;
                if (lo >= at) {
                    atomicAdd(&counts[c0 + 2 * i], lo);
                    w[q] &= 0xffff0000u;
                }
                if (hi >= at) {
                    atomicAdd(&counts[c0 + 2 * i + 1], hi);
                    w[q] &= 0x0000ffffu;
                }
            }
            *reinterpret_cast<u32x4 *>(bins + i4) = u32x4{w[0], w[1], w[2], w[3]};
        }
        __syncthreads();
    };
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    const i32x4 *t4 = reinterpret_cast<const i32x4 *>(tokens);
    constexpr int kUnroll = 4;                                      // 16-byte loads per thread and round
    constexpr long long kIter = (long long)kHistBlock * kUnroll;    // groups per round of the workgroup
    static_assert(kSweepBlock % (kHistBlock * kUnroll * 4) == 0, "a block of tokens is a whole number of rounds");
    // the loads of round i + 1 are requested before round i is counted
    auto fetch = [&](long long gb, i32x4(&v)[kUnroll]) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const long long g = gb + (long long)u * kHistBlock + threadIdx.x;
            v[u] = g < g1 ? t4[g] : i32x4{0, 0, 0, 0};
        }
    };
    if (blockIdx.x == gridDim.x - 1) { // the stream's last one to three tokens, while the bins are still empty
        const long long i = groups * 4 + threadIdx.x;
        one(i < n_tokens ? tokens[i] : 0, i < n_tokens);
    }
    i32x4 v[kUnroll], vn[kUnroll];
    fetch(g0, vn);
    int since_sweep = 0; // tokens counted since the last sweep (uniform)
    for (long long gb = g0; gb < g1; gb += kIter) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = vn[u];
        fetch(gb + kIter, vn); // (past the slice's end: nothing is loaded)
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const bool live = gb + (long long)u * kHistBlock + threadIdx.x < g1;
            one(v[u].x, live);
            one(v[u].y, live);
            one(v[u].z, live);
            one(v[u].w, live);
        }
        since_sweep += (int)kIter * 4;
        if (since_sweep >= kSweepBlock && gb + kIter < g1) {
            sweep(kSweepAt);
            since_sweep = 0;
        }
    }
    // (the waves' counts of invalid ids meet in LDS first: same-address device atomics take ~40 ns each)
    if ((threadIdx.x & 63) == 0 && invalid) atomicAdd(&invalid_wg, invalid);
    // What is left in the bins: with room for it, the workgroup's bins go to memory as they are (k_subset_reduce adds
    // the workgroups' copies up); without, every non-zero field is added to the global counts (up to 80 000 atomics per
    // workgroup, 19 M over the grid when every id occurs: slower than the counting itself).
    if (partials) {
        __syncthreads();
        unsigned *dst = partials + ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * (kChunkIds / 2);
        for (int i4 = threadIdx.x * 4; i4 < nw4; i4 += kHistBlock * 4)
            *reinterpret_cast<u32x4 *>(dst + i4) = *reinterpret_cast<const u32x4 *>(bins + i4);
    } else {
        sweep(1u); // (begins with a barrier)
    }
    if (threadIdx.x == 0 && invalid_wg) atomicAdd(&state[0], invalid_wg);
}

// counts[id] += the sum over the slices' workgroups of the id's field; thread = one word (two ids) of one chunk.
// The final counts pass through here, so the first histogram pass of the selection (top digit) is taken along.
constexpr int kSelBuckets0 = 2048;
__global__ __launch_bounds__(256) void k_subset_reduce(const unsigned *__restrict__ partials, int slices, int V,
                                                       unsigned *counts, unsigned *hist0) {
    __shared__ unsigned hist[kSelBuckets0];
    for (int i = threadIdx.x; i < kSelBuckets0; i += 256) hist[i] = 0u;
    __syncthreads();
    const int c = blockIdx.y, c0 = c * kChunkIds, nb = min(kChunkIds, V - c0), nw = (nb + 1) / 2;
    const int w = blockIdx.x * blockDim.x + threadIdx.x;
    const bool has_lo = w < nw, has_hi = w < nw && 2 * w + 1 < nb;
    unsigned lo = 0u, hi = 0u;
    if (has_lo) {
        const unsigned *src = partials + (size_t)c * slices * (kChunkIds / 2) + w;
        int sl = 0;
        for (; sl + 32 <= slices; sl += 32) { // thirty-two loads in flight: the kernel is a chain of strided reads
            unsigned x[32];
#pragma unroll
            for (int u = 0; u < 32; ++u) x[u] = src[(size_t)(sl + u) * (kChunkIds / 2)];
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                lo += x[u] & 0xffffu;
                hi += x[u] >> 16;
            }
        }
        for (; sl < slices; ++sl) {
            const unsigned x = src[(size_t)sl * (kChunkIds / 2)];
            lo += x & 0xffffu;
            hi += x >> 16;
        }
        lo += counts[c0 + 2 * w]; // (the counting kernel, which may have added to these words, has finished)
        counts[c0 + 2 * w] = lo;
    }
    if (has_hi) {
        hi += counts[c0 + 2 * w + 1];
        counts[c0 + 2 * w + 1] = hi;
    }
    // top digit: almost every id has a zero there, so those are counted per wave (one LDS atomic instead of up to 128
    // on the same word)
    const unsigned dlo = lo >> 21, dhi = hi >> 21;
    const unsigned zeros = (unsigned)__popcll(__builtin_amdgcn_ballot_w64(has_lo && dlo == 0u)) +
                           (unsigned)__popcll(__builtin_amdgcn_ballot_w64(has_hi && dhi == 0u));
    if ((threadIdx.x & 63) == 0 && zeros) atomicAdd(&hist[0], zeros);
    if (has_lo && dlo) atomicAdd(&hist[dlo], 1u);
    if (has_hi && dhi) atomicAdd(&hist[dhi], 1u);
    __syncthreads();
    for (int i = threadIdx.x; i < kSelBuckets0; i += 256)
        if (hist[i]) atomicAdd(&hist0[i], hist[i]);
}

// ---- selection: T = the n-th largest count, r = how many ids with count == T belong to the n most frequent ----
// (1 <= r when n >= 1; #(count > T) = n - r).  A radix select, most significant digit first: pass p histograms digit
// p of the counts that agree with the prefix found so far (kSelGroups workgroups, each in LDS first); the kernel that
// follows walks the buckets from the top to the one that holds the n-th largest, every workgroup for itself.
constexpr int kSelGroups = 64;  // workgroups of a histogram pass of the selection
constexpr int kCmpGroups = 160; // workgroups of the compaction: one round of 1024 ids each at 151 680 ids
constexpr int kSelPasses = 3, kSelBuckets = 2048;
__host__ __device__ constexpr int sel_shift(int pass) { return pass == 0 ? 21 : pass == 1 ? 10 : 0; }
__host__ __device__ constexpr int sel_bits(int pass) { return pass == 2 ? 10 : 11; }
// state: [0] invalid ids, [1] T, [2] n, then r at [3]; [4 + 2 p], [5 + 2 p]: prefix and ids still needed after the walk
// of pass p; then kSelPasses x kSelBuckets bucket counts, then per-workgroup (above, ties) totals of the compaction
constexpr int kStateAfter = 4, kStateHist = 16, kStateTotals = kStateHist + kSelPasses * kSelBuckets,
              kStateWordsFull = kStateTotals + 2 * kCmpGroups;

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

// The walk over the buckets of pass `pass`, by the whole workgroup: from the largest digit down to the bucket that
// holds the need-th largest of the counts that agree with the prefix.  Returns the prefix extended by that digit and
// the ids still needed from inside the bucket.  Every workgroup of a kernel computes the same values; workgroup 0
// leaves them in the state for the kernels after this one (kStateAfter).
__device__ __forceinline__ void sel_walk(unsigned *state, int pass, unsigned *scratch, unsigned *found,
                                         unsigned &prefix, unsigned &need) {
    const unsigned prefix_in = pass == 0 ? 0u : state[kStateAfter + 2 * (pass - 1)];
    const unsigned need_in = pass == 0 ? state[2] : state[kStateAfter + 2 * (pass - 1) + 1];
    const unsigned *hist = state + kStateHist + pass * kSelBuckets;
    const int nbuckets = 1 << sel_bits(pass);
    // thread t holds buckets nbuckets - 1 - 2 t and nbuckets - 2 - 2 t: the scan runs from the top
    const int hi = nbuckets - 1 - 2 * (int)threadIdx.x, lo = hi - 1;
    const unsigned a = hi >= 0 ? hist[hi] : 0u, b = lo >= 0 ? hist[lo] : 0u;
    unsigned total;
    const unsigned incl = block_scan(a + b, scratch, total), excl = incl - (a + b);
    if (threadIdx.x == 0) { // fewer candidates than needed cannot happen (need <= their number); bucket 0 if it did
        found[0] = 0u;
        found[1] = need_in > total ? 0u : need_in;
    }
    __syncthreads();
    if (hi >= 0 && excl < need_in && need_in <= excl + a) {
        found[0] = (unsigned)hi;
        found[1] = need_in - excl;
    } else if (lo >= 0 && excl + a < need_in && need_in <= incl) {
        found[0] = (unsigned)lo;
        found[1] = need_in - excl - a;
    }
    __syncthreads();
    prefix = prefix_in | (found[0] << sel_shift(pass));
    need = found[1];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        state[kStateAfter + 2 * pass] = prefix;
        state[kStateAfter + 2 * pass + 1] = need;
    }
    __syncthreads(); // found and scratch may be reused
}

__global__ __launch_bounds__(kSelBlock) void k_subset_sel_hist(const unsigned *__restrict__ counts, int V, int pass,
                                                               unsigned *state) {
    __shared__ unsigned hist[kSelBuckets];
    __shared__ unsigned scratch[kSelBlock / 64], found[2];
    for (int i = threadIdx.x; i < kSelBuckets; i += kSelBlock) hist[i] = 0u;
    unsigned prefix = 0u, need = 0u;
    if (pass > 0) sel_walk(state, pass - 1, scratch, found, prefix, need);
    __syncthreads();
    const int shift = sel_shift(pass);
    const unsigned digit = (1u << sel_bits(pass)) - 1u;
    const unsigned mask = pass == 0 ? 0u : 0xffffffffu << sel_shift(pass - 1);
    const int per = (V + gridDim.x - 1) / gridDim.x, v0 = blockIdx.x * per, v1 = min(V, v0 + per);
    for (int v = v0 + threadIdx.x; v < v1; v += kSelBlock) {
        const unsigned c = counts[v];
        if ((c & mask) == prefix) atomicAdd(&hist[(c >> shift) & digit], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kSelBuckets; i += kSelBlock)
        if (hist[i]) atomicAdd(&state[kStateHist + pass * kSelBuckets + i], hist[i]);
}

// ---- compaction: the ids in ascending order, those with count > T plus the first r ties ----
// Workgroup g owns a contiguous range of ids.  First every workgroup counts its (above, ties); then it adds up what the
// workgroups before it hold (at most kSelGroups pairs) and places its own ids by two workgroup scans.
__global__ __launch_bounds__(kSelBlock) void k_subset_cmp_count(const unsigned *__restrict__ counts, int V,
                                                                unsigned *state) {
    __shared__ unsigned scratch[kSelBlock / 64], found[2];
    unsigned T, r; // the last walk: the prefix is now the whole count
    sel_walk(state, kSelPasses - 1, scratch, found, T, r);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        state[1] = T;
        state[3] = r;
    }
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
    const unsigned T = state[1], r = state[3];
    // what the workgroups before this one hold: summed by the whole workgroup
    unsigned above_before, ties_before;
    {
        const bool mine = threadIdx.x < blockIdx.x;
        (void)block_scan(mine ? state[kStateTotals + 2 * threadIdx.x] : 0u, scratch, above_before);
        (void)block_scan(mine ? state[kStateTotals + 2 * threadIdx.x + 1] : 0u, scratch, ties_before);
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
constexpr int kStateWordsFullStatic = 16 + 3 * 2048 + 2 * 160; // = kStateWordsFull (spelled out: used in the array bound)
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
                                kChunkIds * 2) != hipSuccess) {
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

// workgroups per chunk of the counting kernel: 256 workgroups in all (one per CU of the device this is written for),
// fixed so that the workspace size does not depend on the device
int subset_slices(int V) { return std::max(1, 256 / ((V + kChunkIds - 1) / kChunkIds)); }
size_t subset_partial_words(int V) { return (size_t)subset_slices(V) * ((V + kChunkIds - 1) / kChunkIds) * (kChunkIds / 2); }

// everything after the argument checks: `work` holds V counts followed by the selection state and, with_partials, by
// one copy of the bins per workgroup of the counting kernel
int32_t subset_build_on(const int32_t *tokens, int64_t n_tokens, int32_t V, int32_t n, unsigned *work, bool with_partials,
                        int32_t *ids_out, int32_t *counts_out, int32_t *invalid_out, hipStream_t st) {
    unsigned *counts = work;
    unsigned *state = counts + V;
    unsigned *partials = with_partials ? work + ((size_t)V + kStateWordsFull + 3) / 4 * 4 : nullptr; // 16-byte aligned
    hipLaunchKernelGGL(k_subset_clear, dim3((V + kStateWordsFull + 255) / 256), dim3(256), 0, st, counts, V, state,
                       kStateWordsFull, n);
    const int chunks = (V + kChunkIds - 1) / kChunkIds;
    const int slices = subset_slices(V);
    hipLaunchKernelGGL(k_subset_hist, dim3(slices, chunks), dim3(kHistBlock), kChunkIds * 2, st, tokens,
                       (long long)n_tokens, V, counts, state, partials);
    if (partials)
        hipLaunchKernelGGL(k_subset_reduce, dim3((kChunkIds / 2 + 255) / 256, chunks), dim3(256), 0, st, partials, slices,
                           V, counts, state + kStateHist);
    if (n > 0) {
        for (int pass = partials ? 1 : 0; pass < kSelPasses; ++pass) // (with partials, pass 0 was taken along above)
            hipLaunchKernelGGL(k_subset_sel_hist, dim3(kSelGroups), dim3(kSelBlock), 0, st, counts, V, pass, state);
        hipLaunchKernelGGL(k_subset_cmp_count, dim3(kCmpGroups), dim3(kSelBlock), 0, st, counts, V, state);
        hipLaunchKernelGGL(k_subset_cmp_write, dim3(kCmpGroups), dim3(kSelBlock), 0, st, counts, V, n, state, ids_out);
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
    return (((size_t)vocab_size + kStateWordsFull + 3) / 4 * 4 + subset_partial_words(vocab_size)) * 4;
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
    return subset_build_on(tokens, n_tokens, vocab_size, n, static_cast<unsigned *>(workspace), true, ids_out, counts_out,
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
    return subset_build_on(tokens, n_tokens, vocab_size, n, work, false, ids_out, counts_out, invalid_out,
                           static_cast<hipStream_t>(hip_stream));
}

} // extern "C"
