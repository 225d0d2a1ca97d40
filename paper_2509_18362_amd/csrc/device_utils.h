// Device-side helpers for the gfx950 draft kernels: bf16 packing, 64-lane reductions, MFMA wrappers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mtp {

constexpr int kWave = 64;
constexpr int kBlock = 512;            // threads per workgroup in every phase
constexpr int kWaves = kBlock / kWave; // 8

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round to nearest even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// x ~= hi + lo with hi, lo bf16: keeps 16 mantissa bits of a float activation through a bf16 MFMA
__device__ __forceinline__ void split_bf16(float x, uint16_t &hi, uint16_t &lo) {
    hi = f32_to_bf16(x);
    lo = f32_to_bf16(x - bf16_to_f32(hi));
}

__device__ __forceinline__ float lo_half(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float hi_half(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// ---- cross-lane sums -------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
// sum over the 16 lanes of a DPP row; every lane of the row gets the total
__device__ __forceinline__ float row16_sum(float x) {
    x += dpp_f32<0xB1>(x);  // quad_perm [1,0,3,2]
    x += dpp_f32<0x4E>(x);  // quad_perm [2,3,0,1]
    x += dpp_f32<0x141>(x); // row_half_mirror
    x += dpp_f32<0x140>(x); // row_mirror
    return x;
}
// sum over 8 consecutive lanes (aligned groups of 8)
__device__ __forceinline__ float oct_sum(float x) {
    x += dpp_f32<0xB1>(x);
    x += dpp_f32<0x4E>(x);
    x += dpp_f32<0x141>(x);
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
    x = row16_sum(x);
    x += __shfl_xor(x, 16, kWave);
    x += __shfl_xor(x, 32, kWave);
    return x;
}
// sum over the whole workgroup; red must hold kWaves floats; contains two barriers
__device__ __forceinline__ float block_sum(float x, float *red) {
    x = wave_sum(x);
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = x;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) t += red[w];
    return t;
}

// ---- argmax key: larger logit wins, then smaller index ------------------------------------------------
// (-0.0 and +0.0 compare equal as logits, so both map to the key of +0.0 and the index decides)
__device__ __forceinline__ uint32_t orderable(float f) {
    uint32_t u = __float_as_uint(f);
    u = (u == 0x80000000u) ? 0u : u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ unsigned long long argmax_key(float logit, uint32_t index) {
    return ((unsigned long long)orderable(logit) << 32) | (unsigned long long)(0xffffffffu - index);
}
__device__ __forceinline__ uint32_t key_index(unsigned long long key) { return 0xffffffffu - (uint32_t)key; }

// ---- 16x16x32 bf16 MFMA: D[i][j] += sum_k A[i][k] * B[k][j] -------------------------------------------
// lane l supplies A[l%16][(l/16)*8 .. +8] and B[(l/16)*8 .. +8][l%16]; it receives D[(l/16)*4 + v][l%16], v = 0..3
__device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
}

__device__ __forceinline__ u32x4 ldg16(const void *p) { return *reinterpret_cast<const u32x4 *>(p); }

// ---- device-coherent accesses ---------------------------------------------------------------------------
// Inside ONE kernel, data handed from a workgroup to workgroups on other compute dies (each die has its own L2)
// must bypass the non-coherent caches: relaxed atomics at device scope do exactly that, access by access, without
// the write-back and invalidation of whole caches that a release/acquire pair costs (about 4 us per barrier here).
// COH = false: plain accesses (data produced by an earlier kernel).
template <bool COH>
__device__ __forceinline__ float ld_f32(const float *p) {
    if (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *p;
}
template <bool COH>
__device__ __forceinline__ unsigned long long ld_u64(const unsigned long long *p) {
    if (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *p;
}
template <bool COH>
__device__ __forceinline__ f32x4 ld_f32x4(const float *p) { // 16-byte aligned
    if (COH) {
        const unsigned long long *q = reinterpret_cast<const unsigned long long *>(p);
        unsigned long long a = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned long long b = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return f32x4{__uint_as_float((uint32_t)a), __uint_as_float((uint32_t)(a >> 32)), __uint_as_float((uint32_t)b),
                     __uint_as_float((uint32_t)(b >> 32))};
    }
    return *reinterpret_cast<const f32x4 *>(p);
}
template <bool COH>
__device__ __forceinline__ void st_f32(float *p, float v) {
    if (COH)
        __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
        *p = v;
}
template <bool COH>
__device__ __forceinline__ void st_f32x4(float *p, f32x4 v) { // 16-byte aligned
    if (COH) {
        unsigned long long *q = reinterpret_cast<unsigned long long *>(p);
        __hip_atomic_store(q, (unsigned long long)__float_as_uint(v.x) | ((unsigned long long)__float_as_uint(v.y) << 32),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(q + 1, (unsigned long long)__float_as_uint(v.z) | ((unsigned long long)__float_as_uint(v.w) << 32),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        *reinterpret_cast<f32x4 *>(p) = v;
    }
}
template <bool COH>
__device__ __forceinline__ void st_u64(unsigned long long *p, unsigned long long v) {
    if (COH)
        __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
        *p = v;
}
template <bool COH>
__device__ __forceinline__ void st_u16(uint16_t *p, uint16_t v) {
    if (COH)
        __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
        *p = v;
}
// Row-streaming loads through a buffer descriptor: the wave-uniform row start and length sit in four scalar
// registers, the position inside the row in one more, and a single vector register (16 bytes per lane) serves every
// load.  No vector registers are spent - or recycled, which stalls on loads still in flight - on 64-bit address
// arithmetic, and an offset past the row's end would read zeros instead of faulting.
typedef __amdgpu_buffer_rsrc_t row_rsrc;
__device__ __forceinline__ row_rsrc make_row_rsrc(const uint16_t *uniform_row, int row_bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(uniform_row), 0, row_bytes, 0x00020000);
}
// STREAM: non-temporal load.  Data read this way does not displace what sits in the 256 MB memory-side cache, so
// a tensor read with plain loads (the output head) can stay there from one draft step to the next while the rest
// of the weights stream by.
template <bool STREAM>
__device__ __forceinline__ u32x4 row_load16(row_rsrc r, int lane_byte_off, int uniform_byte_off) {
    return __builtin_bit_cast(
        u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, lane_byte_off, uniform_byte_off, STREAM ? 2 : 0));
}

} // namespace mtp
