// medusa_heads (Sec. 2.1.1 of the Medusa paper): logits_k = W2_k . (SiLU(W1_k . h) + h).
//
// Both GEMMs are "skinny": M (batch rows, or batch x tree tokens) is tiny next to the
// d x d and V x d weight matrices, so the weights are streamed from HBM exactly once and
// the kernels are organised around that stream:
//   * M <= 4  (bf16): one wavefront per weight row, 16-byte non-temporal loads that cover
//                     1 KB of the row per instruction, packed bf16 dot products on the
//                     vector ALUs, activations resident in LDS.
//   * M  > 4  (bf16): 16x16x32 bf16 MFMA tiles; a workgroup owns 64 weight rows x up to 80
//                     activation rows, its four wavefronts interleave over the reduction
//                     dimension and are summed through LDS in a fixed order.
//   * fp32          : plain FMA version of the first scheme (small configurations only).
// The residual block's epilogue applies SiLU, adds h and rounds once to the storage type.
#include "common.hpp"

namespace {

enum { EPI_LOGITS = 0, EPI_RESID = 1 };

// acc[m][n] = sum_j W[k][n][j] * X[m*xs_m + k*xs_k + j]
struct GemmArgs {
  const void* W;       // [K][N][d]
  const void* X;       // activations, see strides
  const void* hidden;  // [M][d] residual source (EPI_RESID, N == d)
  void* out;           // EPI_LOGITS: float [M][K][N];  EPI_RESID: dtype [M][K][N]
  int M, N, d, K;
  long xs_m, xs_k;     // element strides of X between rows m and between heads k
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

// ---------------------------------------------------------------------------------------
// bf16, M <= 4 per block of rows: wave-per-row streaming GEMV.
// grid (row blocks, K, m blocks), 256 threads.  LDS: MB x d bf16.
// ---------------------------------------------------------------------------------------
constexpr int kGemvRowsPerWg = 64;

template <int MB, int EPI>
__global__ __launch_bounds__(256) void gemv_bf16_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4_t* xs = (u32x4_t*)smem;                 // [MB][d/8] 16-byte chunks
  const int chunks = a.d >> 3;
  const int k = blockIdx.y, m0 = blockIdx.z * MB;
  const uint16_t* X = (const uint16_t*)a.X;
  for (int i = threadIdx.x; i < MB * chunks; i += 256) {
    const int mm = i / chunks, c = i - mm * chunks;
    u32x4_t v = {0, 0, 0, 0};
    if (m0 + mm < a.M) v = *(const u32x4_t*)(X + (size_t)(m0 + mm) * a.xs_m + (size_t)k * a.xs_k + (size_t)c * 8);
    xs[i] = v;
  }
  __syncthreads();

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint16_t* W = (const uint16_t*)a.W + (size_t)k * a.N * a.d;
  const int n_begin = blockIdx.x * kGemvRowsPerWg;
  constexpr int R = 2, U = 4;
  for (int nb = n_begin + wave * R; nb < n_begin + kGemvRowsPerWg && nb < a.N; nb += 4 * R) {
    float acc[R][MB];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int mm = 0; mm < MB; ++mm) acc[r][mm] = 0.f;
    const u32x4_t* wrow[R];
#pragma unroll
    for (int r = 0; r < R; ++r) wrow[r] = (const u32x4_t*)(W + (size_t)min(nb + r, a.N - 1) * a.d);
    for (int c0 = 0; c0 < chunks; c0 += 64 * U) {
      u32x4_t w[R][U];
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int c = c0 + u * 64 + lane;
          w[r][u] = c < chunks ? __builtin_nontemporal_load(wrow[r] + c) : u32x4_t{0, 0, 0, 0};
        }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int c = min(c0 + u * 64 + lane, chunks - 1);
#pragma unroll
        for (int mm = 0; mm < MB; ++mm) {
          const u32x4_t x = xs[mm * chunks + c];
#pragma unroll
          for (int r = 0; r < R; ++r) {
            float s = acc[r][mm];
            s = dot2_bf16(w[r][u].x, x.x, s);
            s = dot2_bf16(w[r][u].y, x.y, s);
            s = dot2_bf16(w[r][u].z, x.z, s);
            s = dot2_bf16(w[r][u].w, x.w, s);
            acc[r][mm] = s;
          }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int mm = 0; mm < MB; ++mm) {
        const float s = wave_sum(acc[r][mm]);
        if (lane == 0 && nb + r < a.N && m0 + mm < a.M) epilogue_store<EPI, uint16_t>(a, m0 + mm, k, nb + r, s);
      }
  }
}

// ---------------------------------------------------------------------------------------
// fp32: same scheme with plain FMAs.  LDS: MB x d floats.
// ---------------------------------------------------------------------------------------
template <int MB, int EPI>
__global__ __launch_bounds__(256) void gemv_f32_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  floatx4_t* xs = (floatx4_t*)smem;             // [MB][d/4]
  const int chunks = a.d >> 2;
  const int k = blockIdx.y, m0 = blockIdx.z * MB;
  const float* X = (const float*)a.X;
  for (int i = threadIdx.x; i < MB * chunks; i += 256) {
    const int mm = i / chunks, c = i - mm * chunks;
    floatx4_t v = {0.f, 0.f, 0.f, 0.f};
    if (m0 + mm < a.M) v = *(const floatx4_t*)(X + (size_t)(m0 + mm) * a.xs_m + (size_t)k * a.xs_k + (size_t)c * 4);
    xs[i] = v;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* W = (const float*)a.W + (size_t)k * a.N * a.d;
  const int n_begin = blockIdx.x * kGemvRowsPerWg;
  for (int n = n_begin + wave; n < n_begin + kGemvRowsPerWg && n < a.N; n += 4) {
    float acc[MB];
#pragma unroll
    for (int mm = 0; mm < MB; ++mm) acc[mm] = 0.f;
    const floatx4_t* wrow = (const floatx4_t*)(W + (size_t)n * a.d);
    for (int c = lane; c < chunks; c += 64) {
      const floatx4_t w = wrow[c];
#pragma unroll
      for (int mm = 0; mm < MB; ++mm) {
        const floatx4_t x = xs[mm * chunks + c];
        acc[mm] = fmaf(w[0], x[0], fmaf(w[1], x[1], fmaf(w[2], x[2], fmaf(w[3], x[3], acc[mm]))));
      }
    }
#pragma unroll
    for (int mm = 0; mm < MB; ++mm) {
      const float s = wave_sum(acc[mm]);
      if (lane == 0 && m0 + mm < a.M) epilogue_store<EPI, float>(a, m0 + mm, k, n, s);
    }
  }
}

// ---------------------------------------------------------------------------------------
// bf16, M > 4: MFMA 16x16x32.  Workgroup tile = (16*MT activation rows) x (64 weight rows);
// the four wavefronts take reduction steps w, w+4, w+8, ... (32 elements each) and are summed
// through LDS in wave order.  Operand layout of v_mfma_f32_16x16x32_bf16: lane l supplies
// row/column (l % 16) and the eight reduction elements 8*(l/16) .. 8*(l/16)+7; it receives
// output column (l % 16), rows 4*(l/16) .. 4*(l/16)+3.  A = activations, B = weights.
// grid (ceil(N/64), K, ceil(M/(16*MT))), 256 threads, LDS 8*MT KB.
// ---------------------------------------------------------------------------------------
template <int MT, int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_bf16_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  floatx4_t* red = (floatx4_t*)smem;            // [4 waves][MT*2 tiles][64 lanes]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i16 = lane & 15, q = lane >> 4;
  const int k = blockIdx.y;
  const int n0 = blockIdx.x * 64, m0 = blockIdx.z * (16 * MT);
  const uint16_t* W = (const uint16_t*)a.W + (size_t)k * a.N * a.d;
  const uint16_t* X = (const uint16_t*)a.X + (size_t)k * a.xs_k;

  const uint16_t* wp[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) wp[j] = W + (size_t)min(n0 + 16 * j + i16, a.N - 1) * a.d + q * 8;
  const uint16_t* xp[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) xp[t] = X + (size_t)min(m0 + 16 * t + i16, a.M - 1) * a.xs_m + q * 8;

  floatx4_t acc[MT][4];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[t][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  const int steps = a.d >> 5;

  for (int s = wave; s < steps; s += 4) {
    bf16x8_t wf[4], xf[MT];
#pragma unroll
    for (int j = 0; j < 4; ++j) wf[j] = *(const bf16x8_t*)(wp[j] + (size_t)s * 32);
#pragma unroll
    for (int t = 0; t < MT; ++t) xf[t] = *(const bf16x8_t*)(xp[t] + (size_t)s * 32);
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[t], wf[j], acc[t][j], 0, 0, 0);
  }

  // Sum the four wavefronts' partial tiles through LDS, two of the four column tiles at a
  // time (keeps the buffer at 8*MT KB), always in wave order 0,1,2,3.
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    if (half) __syncthreads();
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) red[(wave * MT * 2 + t * 2 + jj) * 64 + lane] = acc[t][half * 2 + jj];
    __syncthreads();
    for (int tile = wave; tile < MT * 2; tile += 4) {
      floatx4_t s = red[tile * 64 + lane];
#pragma unroll
      for (int w = 1; w < 4; ++w) s += red[(w * MT * 2 + tile) * 64 + lane];
      const int t = tile >> 1, j = half * 2 + (tile & 1);
      const int n = n0 + 16 * j + i16;
      const int mb = m0 + 16 * t + 4 * q;
      if (n < a.N) {
        if (mb + 0 < a.M) epilogue_store<EPI, uint16_t>(a, mb + 0, k, n, s[0]);
        if (mb + 1 < a.M) epilogue_store<EPI, uint16_t>(a, mb + 1, k, n, s[1]);
        if (mb + 2 < a.M) epilogue_store<EPI, uint16_t>(a, mb + 2, k, n, s[2]);
        if (mb + 3 < a.M) epilogue_store<EPI, uint16_t>(a, mb + 3, k, n, s[3]);
      }
    }
  }
}

// Optional event pair recorded around the vocabulary-projection launch (benchmark hook).
hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;

template <int EPI>
int launch_gemm(const GemmArgs& a, medusa_dtype_t dtype, hipStream_t stream) {
  const dim3 block(256);
  if (dtype == MEDUSA_F32) {
    // activations of one m-block live in LDS: keep it within 64 KB
    const int MB = (size_t)4 * a.d * sizeof(float) <= 65536 ? 4 : 1;
    const dim3 grid(ceil_div(a.N, kGemvRowsPerWg), a.K, ceil_div(a.M, MB));
    const size_t lds = (size_t)MB * a.d * sizeof(float);
    if (MB == 4) hipLaunchKernelGGL((gemv_f32_kernel<4, EPI>), grid, block, lds, stream, a);
    else hipLaunchKernelGGL((gemv_f32_kernel<1, EPI>), grid, block, lds, stream, a);
  } else if (a.M <= 4) {
    int MB = a.M <= 1 ? 1 : (a.M <= 2 ? 2 : 4);
    while ((size_t)MB * a.d * sizeof(uint16_t) > 65536) MB >>= 1;   // activations of one m-block live in LDS
    const dim3 grid(ceil_div(a.N, kGemvRowsPerWg), a.K, ceil_div(a.M, MB));
    const size_t lds = (size_t)MB * a.d * sizeof(uint16_t);
    if (MB == 1) hipLaunchKernelGGL((gemv_bf16_kernel<1, EPI>), grid, block, lds, stream, a);
    else if (MB == 2) hipLaunchKernelGGL((gemv_bf16_kernel<2, EPI>), grid, block, lds, stream, a);
    else hipLaunchKernelGGL((gemv_bf16_kernel<4, EPI>), grid, block, lds, stream, a);
  } else {
    const int MT = a.M > 64 ? 5 : ceil_div(a.M, 16);
    const dim3 grid(ceil_div(a.N, 64), a.K, ceil_div(a.M, 16 * MT));
    const size_t lds = (size_t)4 * MT * 2 * 64 * sizeof(floatx4_t);
    switch (MT) {
      case 1: hipLaunchKernelGGL((gemm_mfma_bf16_kernel<1, EPI>), grid, block, lds, stream, a); break;
      case 2: hipLaunchKernelGGL((gemm_mfma_bf16_kernel<2, EPI>), grid, block, lds, stream, a); break;
      case 3: hipLaunchKernelGGL((gemm_mfma_bf16_kernel<3, EPI>), grid, block, lds, stream, a); break;
      case 4: hipLaunchKernelGGL((gemm_mfma_bf16_kernel<4, EPI>), grid, block, lds, stream, a); break;
      default: hipLaunchKernelGGL((gemm_mfma_bf16_kernel<5, EPI>), grid, block, lds, stream, a); break;
    }
  }
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}

}  // namespace

extern "C" int medusa_heads(const void* hidden, const void* w1, const void* w2, void* resid, float* logits, int M,
                            int d, int V, int K, medusa_dtype_t dtype, medusa_stream_t stream_) {
  if (!hidden || !w2 || !logits || (w1 && !resid)) return MEDUSA_EINVAL;
  if (M < 1 || d < 1 || V < 1 || K < 1) return MEDUSA_EINVAL;
  if (dtype != MEDUSA_F32 && dtype != MEDUSA_BF16) return MEDUSA_EINVAL;
  if (M > 4096 || K > MEDUSA_MAX_HEADS || d > 16384) return MEDUSA_EUNSUPPORTED;
  if (dtype == MEDUSA_BF16 ? (d % 64 != 0) : (d % 8 != 0)) return MEDUSA_EUNSUPPORTED;
  if ((size_t)M * K * V >= (size_t)1 << 40) return MEDUSA_EUNSUPPORTED;
  hipStream_t stream = (hipStream_t)stream_;
  GemmArgs a;
  a.d = d;
  a.M = M;
  a.K = K;
  a.hidden = hidden;
  if (w1) {
    a.W = w1;
    a.X = hidden;
    a.out = resid;
    a.N = d;
    a.xs_m = d;
    a.xs_k = 0;
    const int rc = launch_gemm<EPI_RESID>(a, dtype, stream);
    if (rc != MEDUSA_OK) return rc;
    a.X = resid;
    a.xs_m = (long)K * d;
    a.xs_k = d;
  } else {
    a.X = hidden;
    a.xs_m = d;
    a.xs_k = 0;
  }
  a.W = w2;
  a.out = logits;
  a.N = V;
  const bool prof = w1 && g_prof_start && g_prof_stop;
  if (prof) MEDUSA_HIP_TRY(hipEventRecord(g_prof_start, stream));
  const int rc = launch_gemm<EPI_LOGITS>(a, dtype, stream);
  if (prof && rc == MEDUSA_OK) MEDUSA_HIP_TRY(hipEventRecord(g_prof_stop, stream));
  return rc;
}

extern "C" int medusa_profile_set_events(void* start, void* stop) {
  if ((start == nullptr) != (stop == nullptr)) return MEDUSA_EINVAL;
  g_prof_start = (hipEvent_t)start;
  g_prof_stop = (hipEvent_t)stop;
  return MEDUSA_OK;
}
