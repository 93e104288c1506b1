// Device-side helpers shared by the libtng kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tng {

constexpr int kNormNone = 0;
constexpr int kNormSub = 1;
constexpr int kNormQuot = 2;
constexpr int kNormComb = 3;
constexpr int kNormMean = 4;  // per-worker scalar reference mean(g_m)

constexpr int kBlock = 256;  // threads per workgroup: 4 wavefronts of 64
constexpr int kWave = 64;

struct U32x4 {
  uint32_t x, y, z, w;
};

// Streaming (non-temporal) 16-byte accesses: data that is touched once per kernel.
typedef float v4f_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float4 load_stream(const float4* p) {
  const v4f_t v = __builtin_nontemporal_load(reinterpret_cast<const v4f_t*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ void store_stream(float4* p, const float4& x) {
  v4f_t v;
  v.x = x.x;
  v.y = x.y;
  v.z = x.z;
  v.w = x.w;
  __builtin_nontemporal_store(v, reinterpret_cast<v4f_t*>(p));
}

// A pointer that was itself loaded from memory (a per-worker table of shard pointers) has no known
// address space, and loads through it become FLAT instructions: those count against the LDS counter
// as well, so the compiler drains every outstanding load before the next LDS access and the loads no
// longer overlap.  All such tables here hold device-memory pointers: say so.
template <typename T>
using GlobalPtr = const T __attribute__((address_space(1)))*;

template <typename T>
__device__ __forceinline__ GlobalPtr<T> as_global(const T* p) {
  return (GlobalPtr<T>)p;
}

// float4 number i of a 16-byte aligned global array of floats.
__device__ __forceinline__ float4 load4(GlobalPtr<float> p, uint64_t i) {
  const v4f_t v = reinterpret_cast<GlobalPtr<v4f_t>>(p)[i];
  return make_float4(v.x, v.y, v.z, v.w);
}

// 16 bytes at a 4-byte aligned address: rows of d floats start anywhere when d is not a multiple of
// 4.  Such loads and stores are legal for global memory on this target; the type only tells the
// compiler not to assume more alignment than there is (the instruction is the same).
typedef float v4f_u_t __attribute__((ext_vector_type(4), aligned(4)));

__device__ __forceinline__ float4 load4_stream_any(GlobalPtr<float> p, uint64_t i) {
  const v4f_u_t v = __builtin_nontemporal_load(reinterpret_cast<GlobalPtr<v4f_u_t>>(p) + i);
  return make_float4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ void store4_any(float* p, uint64_t i, const float4& x) {
  v4f_u_t v;
  v.x = x.x;
  v.y = x.y;
  v.z = x.z;
  v.w = x.w;
  reinterpret_cast<v4f_u_t*>(p)[i] = v;
}

// The same as a streaming (non-temporal) load: shard rows are touched once per pass.
__device__ __forceinline__ float4 load4_stream(GlobalPtr<float> p, uint64_t i) {
  const v4f_t v = __builtin_nontemporal_load(reinterpret_cast<GlobalPtr<v4f_t>>(p) + i);
  return make_float4(v.x, v.y, v.z, v.w);
}

// Store of a packed word that is not read again by the same kernel.  A small write stream next to a
// large read stream costs far more HBM time than its bytes; stores marked device-coherent (the sc1
// cache-policy bit, which is what a relaxed device-scope atomic store compiles to) measured a
// quarter cheaper for the packed codes than plain or non-temporal stores.  (The same bit on the
// decoded average made the following quantise pass slower, so that one keeps non-temporal stores.)
__device__ __forceinline__ void store_word_through(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// a ^ b ^ c in one instruction (three-input bitwise op of gfx950, truth table 0x96).
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).  One round sends the counter
// (c0,c1,c2,c3) to (hi(B*c2)^c1^k0, lo(B*c2), hi(A*c0)^c3^k1, lo(A*c0)); the key moves by two
// Weyl increments between rounds.  The key is wave-uniform, so the round keys live in SGPRs.
__device__ __forceinline__ U32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
  constexpr uint32_t A = 0xD2511F53u, B = 0xCD9E8D57u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t pa = (uint64_t)A * c0;
    const uint64_t pb = (uint64_t)B * c2;
    const uint32_t n0 = xor3((uint32_t)(pb >> 32), c1, k0);
    const uint32_t n2 = xor3((uint32_t)(pa >> 32), c3, k1);
    c1 = (uint32_t)pb;
    c3 = (uint32_t)pa;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return U32x4{c0, c1, c2, c3};
}

// Uniform on the 24-bit grid {0, 2^-24, ..., 1 - 2^-24}; both steps are exact in binary32.
__device__ __forceinline__ float uniform24(uint32_t word) {
  return (float)(word >> 8) * 0x1p-24f;
}

// Reference made safe to divide by (Eq. 2): |r| < eps -> copysign(eps, r).
__device__ __forceinline__ float clamp_ref(float r, float eps) {
  return fabsf(r) < eps ? copysignf(eps, r) : r;
}

// The vector handed to the coder.  r1 is g~ (SUB, COMB) or the clamped g~ (QUOT);
// r2 is the clamped g~' (COMB only).
template <int NORM>
__device__ __forceinline__ float normalize(float g, float r1, float r2) {
  if (NORM == kNormSub) return g - r1;
  if (NORM == kNormQuot) return g / r1;
  if (NORM == kNormComb) return (g - r1) / r2;
  return g;
}

// The quotient g / b of Eq. 2 for many g and one b: with inv_b = the correctly rounded binary64
// reciprocal of b, float(double(g) * inv_b) is the correctly rounded binary32 quotient whenever that
// quotient is zero or of normal size.  Why: the product is within 2^-52 (relative) of g / b, while a
// quotient of two binary32 numbers that is not itself a binary32 number stays at least 1 / (B N) >
// 2^-49 (relative) away from every midpoint N 2^k of two neighbouring binary32 numbers (B, N the
// integer significands of b and of the midpoint; N is odd and longer than 24 bits, so g = b N 2^k
// has no solution) -- the two roundings cannot land on different sides.  Below 2^-126 the midpoints
// are short enough to be hit exactly (g = 9 * 2^-149, b = 6), which is why callers test the result
// with is_subnormal and redo those few with the division itself.  Infinities, NaNs and zeros of g
// and an infinite b behave as in g / b (b is never zero: the reference is clamped away from it).
__device__ __forceinline__ float quotient_by_reciprocal(float g, double inv_b) {
  return (float)((double)g * inv_b);
}

__device__ __forceinline__ bool is_subnormal(float v) {
  return __builtin_amdgcn_classf(v, (1 << 4) | (1 << 7));  // -subnormal | +subnormal
}

// The same including the per-worker mean reference (mu = mean of the worker's gradient).
template <int NORM>
__device__ __forceinline__ float normalize_w(float g, float r1, float r2, float mu) {
  if (NORM == kNormMean) return g - mu;
  return normalize<NORM>(g, r1, r2);
}

// The same with the kind of normalisation and the raw (unclamped) references as run-time arguments.
__device__ __forceinline__ float normalize_dyn(int norm, float g, float ref, float ref2, float eps) {
  switch (norm) {
    case kNormSub: return g - ref;
    case kNormQuot: return g / clamp_ref(ref, eps);
    case kNormComb: return (g - ref) / clamp_ref(ref2, eps);
    default: return g;
  }
}

template <int NORM>
__device__ __forceinline__ float denormalize(float mean, float r1, float r2) {
  if (NORM == kNormSub) return r1 + mean;
  if (NORM == kNormQuot) return r1 * mean;
  if (NORM == kNormComb) {
    const float p = r2 * mean;
    return p + r1;
  }
  return mean;  // none; per-worker mean reference: every worker's mean was added back before averaging
}

// Stochastic rounding of |v|/R onto {0, 1/S, ..., 1} (section "Gradient Compression"; S = 1 is the
// ternary coder with P(z = 1) = |v|/R).  Returns level | sign << (BITS-1), sign cleared at level 0.
template <int BITS>
__device__ __forceinline__ uint32_t quantize_code(float v, float inv_r, uint32_t word) {
  constexpr int S = (1 << (BITS - 1)) - 1;
  if (BITS == 2) {
    // S = 1: x = min(|v|/R, 1) has floor 1 and fraction 0 when it reaches 1, else floor 0 and
    // fraction x, so level = [u < |v| * inv_r] without the clamp (u < 1 always): the same bits
    // as the general formula below, in fewer operations.
    const uint32_t level = uniform24(word) < fabsf(v) * inv_r ? 1u : 0u;
    return level | (((__float_as_uint(v) >> 31) & level) << 1);  // -0 has level 0, so its sign is dropped
  }
  const float a = fabsf(v);
  const float t = fminf(a * inv_r, 1.0f);
  const float x = t * (float)S;
  const int lo = (int)x;
  const float f = x - (float)lo;
  const uint32_t level = (uint32_t)lo + (uniform24(word) < f ? 1u : 0u);
  const uint32_t neg = (v < 0.0f && level != 0u) ? 1u : 0u;
  return level | (neg << (BITS - 1));
}

// Value of one code: +-(R/S) * level, level S giving R itself; the unused pattern
// "sign with level 0" decodes to +0.
template <int BITS>
__device__ __forceinline__ float decode_code(uint32_t code, float r, float step) {
  constexpr uint32_t S = (1u << (BITS - 1)) - 1u;
  const uint32_t level = code & S;
  const bool neg = ((code >> (BITS - 1)) & 1u) != 0u;
  float mag;
  if (BITS == 2) {
    mag = level ? r : 0.0f;
  } else {
    mag = (level == S) ? r : step * (float)level;
  }
  return (neg && level != 0u) ? -mag : mag;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}

// The largest of 64 non-negative floats, the same value in every lane (a wavefront-uniform register), by
// the data-parallel lane moves of the vector unit: within rows of 16 lanes by quad swaps and mirrors, then
// lane 15 of a row into the next row, lane 31 into the upper half; lane 63 holds the result.  Six
// instructions and a read of lane 63, no LDS round trips (wave_max above makes six of them).  The values
// are compared as integers, which for non-negative floats is the same order.
__device__ __forceinline__ float wave_max_nonneg(float x) {
  int v = (int)__float_as_uint(x);
  v = max(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false));   // quad_perm: [1, 0, 3, 2]
  v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false));   // quad_perm: [2, 3, 0, 1]
  v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xF, 0xF, false));  // row_half_mirror
  v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x140, 0xF, 0xF, false));  // row_mirror
  v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x142, 0xA, 0xF, false));  // row_bcast:15 into rows 1 and 3
  v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x143, 0xC, 0xF, false));  // row_bcast:31 into rows 2 and 3
  return __uint_as_float((uint32_t)__builtin_amdgcn_readlane(v, 63));
}

// max(|a|, |b|, c) in one instruction (the magnitudes are taken by the operand modifiers).
__device__ __forceinline__ float max3_abs(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, |%1|, |%2|, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

}  // namespace tng
