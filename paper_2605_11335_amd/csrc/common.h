// Shared device-side types for the block kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int uint32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int uint32x4 __attribute__((ext_vector_type(4)));

// A block's weight blob as the kernels see it: bytes [0, split) of the blob live in the
// block's resident buffer (`lo`), bytes [split, blob) in the staging slot the prefetch fills
// (`hi`); both pointers are biased so that `ptr + blob_offset` addresses the byte.  `split`
// is a multiple of 256, so an aligned 16-byte access never straddles the two.
struct WView {
    const char* lo;
    const char* hi;
    uint64_t split;
};

__device__ __forceinline__ const char* wv_ptr(const WView& w, uint64_t boff) {
    return (boff < w.split ? w.lo : w.hi) + boff;
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
    return __uint_as_float(((uint32_t)b) << 16);
}

__device__ __forceinline__ float wv_bf16(const WView& w, uint64_t boff_of_tensor, uint32_t idx) {
    return bf16_bits_to_float(*(const uint16_t*)wv_ptr(w, boff_of_tensor + 2ull * idx));
}

// Workgroup id -> logical tile id such that each XCD (workgroups are dealt round-robin to the
// 8 XCDs) walks one contiguous range of logical ids and so shares operands in its own L2.
__device__ __forceinline__ uint32_t xcd_contiguous_id(uint32_t bid, uint32_t nb) {
    const uint32_t q = nb >> 3, r = nb & 7u;
    const uint32_t xcd = bid & 7u, idx = bid >> 3;
    return xcd < r ? xcd * (q + 1) + idx : r * (q + 1) + (xcd - r) * q + idx;
}

// x * sigmoid(2u), u = sqrt(2/pi) (x + 0.044715 x^3): the tanh form of GELU.
__device__ __forceinline__ float gelu_tanh_f32(float x) {
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    const float en = __builtin_amdgcn_exp2f(u * -2.8853900817779268f);  // exp(-2u)
    return x * __builtin_amdgcn_rcpf(1.0f + en);
}

// x * Phi(x), the GELU the tanh form approximates.  erf by the rational-times-Gaussian formula of
// Abramowitz & Stegun 7.1.26 (absolute error below 1.5e-7, far under a bf16 ulp of the result):
// erf(z) = 1 - (a1 t + ... + a5 t^5) exp(-z^2), t = 1 / (1 + p z), z >= 0; odd in z.
__device__ __forceinline__ float gelu_erf_f32(float x) {
    const float z = fabsf(x) * 0.70710678118654752f;
    const float t = __frcp_rn(1.0f + 0.3275911f * z);
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    const float e = 1.0f - poly * exp2f(-1.4426950408889634f * z * z);       // erf(|x| / sqrt 2)
    return 0.5f * x + 0.5f * fabsf(x) * e;                                    // 0.5 x (1 + sign(x) e)
}

// splitmix64's output function: the per-word mixer of the streamed-bytes checksum.
__device__ __forceinline__ uint64_t cf_mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
constexpr uint64_t CF_GOLDEN64 = 0x9E3779B97F4A7C15ull;
