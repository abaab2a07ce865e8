// Argument block and epilogues shared by the GEMM/GEMV kernels of medusa_heads (Sec. 2.1.1).
#pragma once
#include "common.hpp"

enum { EPI_LOGITS = 0, EPI_RESID = 1 };


// acc[m][n] = sum_j W[k][n][j] * X[m*xs_m + k*xs_k + j]
struct GemmArgs {
  const void* W;       // [K][N][d]
  const void* X;       // activations, see strides
  const void* hidden;  // [M][d] residual source (EPI_RESID, N == d)
  void* out;           // EPI_LOGITS: float [M][K][N];  EPI_RESID: dtype [M][K][N]
  int M, N, d, K;
  long xs_m, xs_k;     // element strides of X between rows m and between heads k
  int rows_per_wg;     // GEMV kernels: weight rows per workgroup (multiple of 8)
};

typedef __bf16 dot2_t __attribute__((__vector_size__(2 * sizeof(__bf16))));

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dot2_t, a), __builtin_bit_cast(dot2_t, b), c, false);
}

__device__ __forceinline__ float silu_f32(float u) { return u / (1.0f + expf(-u)); }

template <int EPI, typename T>
__device__ __forceinline__ void epilogue_store(const GemmArgs& a, int m, int k, int n, float acc) {
  const size_t o = ((size_t)m * a.K + k) * a.N + n;
  if (EPI == EPI_LOGITS) {
    ((float*)a.out)[o] = acc;
  } else {
    const float h = load_as_float<T>((const T*)a.hidden + (size_t)m * a.d + n);
    store_from_float<T>((T*)a.out + o, silu_f32(acc) + h);
  }
}

// Large-M bf16 GEMM (own translation unit: it is compiled with its own code-generation options).
// Requires N * d and M * xs_m below 2^31 elements.  Returns a medusa status code.
int launch_gemm_big(const GemmArgs& a, int epi, hipStream_t stream);
