// Shared host/device helpers of the HIP library (gfx950 only).  Nothing in this file is
// used by, or derived from, the CPU oracle.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "medusa.h"

#define MEDUSA_HIP_TRY(expr)                     \
  do {                                           \
    hipError_t _e = (expr);                      \
    if (_e != hipSuccess) return MEDUSA_EHIP;    \
  } while (0)

// Launch-error check: catches bad configurations without synchronising.
#define MEDUSA_LAUNCH_CHECK()                          \
  do {                                                 \
    if (hipGetLastError() != hipSuccess) return MEDUSA_EHIP; \
  } while (0)

constexpr int kWave = 64;

// Device copy of the candidate-tree tables (Sec. 2.1.2).  Fixed-size POD so one
// allocation and one memcpy upload it.
struct TreeTables {
  int32_t T, K, S, n_leaves;
  int32_t topk_per_head[MEDUSA_MAX_HEADS];  // S_k
  int32_t head_base[MEDUSA_MAX_HEADS];      // index of head k's first entry in [root, top-S_1, top-S_2, ...]
  int32_t parent[MEDUSA_MAX_TREE_TOKENS];
  int32_t depth[MEDUSA_MAX_TREE_TOKENS];
  int32_t rank[MEDUSA_MAX_TREE_TOKENS];
  int32_t token_src[MEDUSA_MAX_TREE_TOKENS];
  uint64_t anc_mask[MEDUSA_MAX_TREE_TOKENS][2];
};

struct medusa_tree {
  TreeTables host;
  int32_t* paths;          // host [n_leaves][K+1]
  TreeTables* dev;         // device copy
  int device;              // device the copy lives on
};

typedef __bf16 bf16_t;
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((__vector_size__(8 * sizeof(__bf16))));   // MFMA operand
typedef float floatx4_t __attribute__((__vector_size__(4 * sizeof(float))));     // MFMA accumulator
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even (finite inputs; NaN stays NaN).
__device__ __forceinline__ uint32_t float_to_bf16_bits(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return float_to_bf16_bits(lo) | (float_to_bf16_bits(hi) << 16);
}

template <typename T> __device__ __forceinline__ float load_as_float(const T* p);
template <> __device__ __forceinline__ float load_as_float<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_as_float<uint16_t>(const uint16_t* p) { return bf16_bits_to_float(*p); }

template <typename T> __device__ __forceinline__ void store_from_float(T* p, float v);
template <> __device__ __forceinline__ void store_from_float<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_from_float<uint16_t>(uint16_t* p, float v) { *p = (uint16_t)float_to_bf16_bits(v); }

// Butterfly reductions over the 64 lanes of a wavefront; every lane ends with the result.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int o) {
  uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
  lo = __shfl_xor(lo, o, kWave);
  hi = __shfl_xor(hi, o, kWave);
  return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    uint64_t w = shfl_xor_u64(v, o);
    v = w > v ? w : v;
  }
  return v;
}

// Order-preserving key for (logit, token id): a larger key means a larger logit, or an equal
// logit and a lower id.  -0.0 is folded onto +0.0 so the two compare equal.
__device__ __forceinline__ uint64_t rank_key(float v, uint32_t id) {
  uint32_t u = __float_as_uint(v);
  if (u == 0x80000000u) u = 0;
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((uint64_t)u << 32) | (uint64_t)(0xffffffffu - id);
}
__device__ __forceinline__ uint32_t rank_key_id(uint64_t key) { return 0xffffffffu - (uint32_t)key; }

__host__ __device__ static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
