// Shared device helpers for the learned-cache kernels (gfx950, 64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gati {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
// 16 bytes of activation data.  A native vector type, so that a load is one
// global_load_dwordx4 and a masked select stays a whole-vector operation.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Streaming 16-byte load: the activation tensor is read exactly once, so it is fetched with
// the non-temporal hint and does not displace the (reused) weights and pooled features from
// the caches.  Measured on MI355X this is worth ~10 % of read bandwidth on its own.
__device__ __forceinline__ u32x4_t load_stream(const u32x4_t* p) { return __builtin_nontemporal_load(p); }

// v if keep, else all zero bits (0.0 in both element types).
__device__ __forceinline__ u32x4_t keep_or_zero(u32x4_t v, bool keep) {
    const u32x4_t z = {0u, 0u, 0u, 0u};
    return keep ? v : z;
}

// Number of active rows of a call: the device-side count when there is one, clamped
// to [0, n_max]; wave-uniform.
__device__ __forceinline__ int active_rows(const int32_t* __restrict__ n_dev, int n_max) {
    int n = n_dev ? *n_dev : n_max;
    n = n < 0 ? 0 : n;
    return n > n_max ? n_max : n;
}

// bf16 is the upper half of an fp32: widening is a shift.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Butterfly sum over the 64 lanes of a wave; every lane gets the same total, and the
// order of additions is fixed, so results are reproducible run to run.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// Element type tags for the activation tensor; a 16-byte vector holds kVec elements.
struct F32Tag { static constexpr int kVec = 4; static constexpr int kBytes = 4; };
struct BF16Tag { static constexpr int kVec = 8; static constexpr int kBytes = 2; };

// Sum of the elements of one 16-byte vector, fixed association.
template <typename Tag> __device__ __forceinline__ float vec_sum(const u32x4_t& v);
template <> __device__ __forceinline__ float vec_sum<F32Tag>(const u32x4_t& v) {
    return (__uint_as_float(v.x) + __uint_as_float(v.y)) + (__uint_as_float(v.z) + __uint_as_float(v.w));
}
// acc + lo + hi of a pair of bf16 values in one instruction (the products with 1.0 are exact; the
// sum is accumulated in fp32).
__device__ __forceinline__ float add_bf16_pair(uint32_t pair, float acc) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pair),
                                           __builtin_bit_cast(bf16x2_t, 0x3f803f80u), acc, false);
}
template <> __device__ __forceinline__ float vec_sum<BF16Tag>(const u32x4_t& v) {
    return add_bf16_pair(v.y, add_bf16_pair(v.x, 0.f)) + add_bf16_pair(v.w, add_bf16_pair(v.z, 0.f));
}

// Elements of one 16-byte vector as floats, in memory order.
template <typename Tag> __device__ __forceinline__ void vec_unpack(const u32x4_t& v, float* e);
template <> __device__ __forceinline__ void vec_unpack<F32Tag>(const u32x4_t& v, float* e) {
    e[0] = __uint_as_float(v.x); e[1] = __uint_as_float(v.y);
    e[2] = __uint_as_float(v.z); e[3] = __uint_as_float(v.w);
}
template <> __device__ __forceinline__ void vec_unpack<BF16Tag>(const u32x4_t& v, float* e) {
    e[0] = bf16_lo(v.x); e[1] = bf16_hi(v.x); e[2] = bf16_lo(v.y); e[3] = bf16_hi(v.y);
    e[4] = bf16_lo(v.z); e[5] = bf16_hi(v.z); e[6] = bf16_lo(v.w); e[7] = bf16_hi(v.w);
}

}  // namespace gati
