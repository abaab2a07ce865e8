// medusa_heads (Sec. 2.1.1 of the Medusa paper): logits_k = W2_k . (SiLU(W1_k . h) + h).
//
// Both GEMMs are "skinny": M (batch rows, or batch x tree tokens) is tiny next to the
// d x d and V x d weight matrices, so the weights are streamed from HBM exactly once and
// the kernels are organised around that stream:
//   * M <= 4  (bf16): one wavefront per weight row, 16-byte non-temporal loads that cover
//                     1 KB of the row per instruction, packed bf16 dot products on the
//                     vector ALUs, activations resident in LDS.
//   * M  > 4  (bf16): 16x16x32 bf16 MFMA tiles fed from a double-buffered LDS tile that is
//                     filled with full-line loads several reduction steps ahead; up to 80
//                     activation rows x 128 weight rows per workgroup (128 x 128 for M > 80).
//   * fp32          : plain FMA version of the first scheme (small configurations only).
// The residual block's epilogue applies SiLU, adds h and rounds once to the storage type.
#include "gemm_args.hpp"

namespace {

// ---------------------------------------------------------------------------------------
// bf16, M <= 4 per block of rows: wave-per-row streaming GEMV.
// grid (row blocks, K, m blocks), 256 threads.  LDS: MB x d bf16.
// ---------------------------------------------------------------------------------------

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
  const int n_begin = blockIdx.x * a.rows_per_wg;
  constexpr int R = 2, U = 4;
  for (int nb = n_begin + wave * R; nb < n_begin + a.rows_per_wg && nb < a.N; nb += 4 * R) {
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
  const int n_begin = blockIdx.x * a.rows_per_wg;
  for (int n = n_begin + wave; n < n_begin + a.rows_per_wg && n < a.N; n += 4) {
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
// bf16, M > 4: LDS-staged MFMA GEMM (v_mfma_f32_16x16x32_bf16).
//
// Workgroup tile BM x BN = (WM*16*MT activation rows) x (WN*16*NT weight rows), four wavefronts
// arranged WM x WN, reduction in steps of BK elements (64 = one 128-byte line per row; 128 measured no faster:
// a stand-alone read kernel with this tile-wise pattern tops out at 5.3-5.7 TB/s on this chip
// whatever the bytes per row and step, against 6.2-7.0 TB/s for whole rows read in sequence).  Both
// operands are fetched with 16-byte loads in which 8 consecutive lanes cover one full 128-byte
// line of a row (at most half as many L2 requests per byte as loading MFMA operand layout directly, which
// measured request-bound at ~3.5 TB/s), held in registers PD reduction steps ahead of their use,
// then written to a double-buffered, padded LDS tile from which the wavefronts read their MFMA
// operands (lane l: row l%16, elements 8*(l/16)..+7 of a 32-element step).  One barrier per step.
// Output layout of the MFMA: lane l holds column l%16 (weight row), rows 4*(l/16)..+3
// (activation rows).  grid (ceil(N/BN), K, ceil(M/BM)), 256 threads.
// ---------------------------------------------------------------------------------------
template <int WM, int WN, int MT, int NT, int BK, int PD, int EPI>
__global__ __launch_bounds__(256) void gemm_lds_bf16_kernel(GemmArgs a) {
  constexpr int BM = WM * 16 * MT, BN = WN * 16 * NT;
  constexpr int CPR = BK / 8;                         // 16-byte chunks per row and reduction step
  static_assert(BK == 64, "the LDS swizzle below assumes 128-byte rows");
  constexpr int PITCH = BK * 2;                       // bytes per LDS row (unpadded, chunks swizzled)
  constexpr int CHUNKS = (BM + BN) * CPR;             // 16-byte chunks per reduction step
  constexpr int LPT = (CHUNKS + 255) / 256;           // chunks per thread per step
  constexpr int STAGE_BYTES = (BM + BN) * PITCH;
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * STAGE_BYTES];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, q4 = lane >> 4;
  const int wm = wave / WN, wn = wave - wm * WN;
  const int k = blockIdx.y;
  const int n0 = blockIdx.x * BN, m0 = blockIdx.z * BM;
  const uint16_t* W = (const uint16_t*)a.W + (size_t)k * a.N * a.d;
  const uint16_t* X = (const uint16_t*)a.X + (size_t)k * a.xs_k;

  // Per-thread source pointers and LDS offsets of its LPT chunks (rows clamped into range; the
  // surplus chunk ids of the last slot repeat the final chunk, which is harmless).
  const uint16_t* src[LPT];
  int dst[LPT];
#pragma unroll
  for (int it = 0; it < LPT; ++it) {
    const int id = min(it * 256 + tid, CHUNKS - 1);
    const int row = id / CPR, c = id - row * CPR;
    src[it] = row < BM ? X + (size_t)min(m0 + row, a.M - 1) * a.xs_m + c * 8
                       : W + (size_t)min(n0 + row - BM, a.N - 1) * a.d + c * 8;
    dst[it] = row * PITCH + ((c ^ ((row >> 1) & 7)) << 4);
  }

  floatx4_t acc[MT][NT];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[t][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  const int nk = a.d / BK;
  u32x4_t regs[PD][LPT];
  auto gload = [&](int step, u32x4_t (&r)[LPT]) {
    const int off = min(step, nk - 1) * BK;
#pragma unroll
    for (int it = 0; it < LPT; ++it) r[it] = *(const u32x4_t*)(src[it] + off);
  };
  auto lstore = [&](int buf, const u32x4_t (&r)[LPT]) {
#pragma unroll
    for (int it = 0; it < LPT; ++it) *(u32x4_t*)(lds + buf * STAGE_BYTES + dst[it]) = r[it];
  };
  // 16-byte chunk c of row r sits at chunk slot c ^ ((r >> 1) & 7): the fragment reads below (16 rows
  // x 4 chunks per instruction) and the row-major stores above then touch every LDS bank equally often
  // within each group of lanes the hardware serves together, which a padded pitch does not achieve.
  const int swz = (i16 >> 1) & 7;
  const int x_off = ((wm * MT) * 16 + i16) * PITCH;
  const int w_off = (BM + (wn * NT) * 16 + i16) * PITCH;
  auto compute = [&](int buf, uint32_t keep) {
    const unsigned char* base = lds + buf * STAGE_BYTES;
#pragma unroll
    for (int kk = 0; kk < BK / 32; ++kk) {
      bf16x8_t xf[MT], wf[NT];
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        u32x4_t bits = *(const u32x4_t*)(base + x_off + t * 16 * PITCH + (((kk * 4 + q4) ^ swz) << 4));
        bits &= keep;
        xf[t] = __builtin_bit_cast(bf16x8_t, bits);
      }
#pragma unroll
      for (int j = 0; j < NT; ++j)
        wf[j] = *(const bf16x8_t*)(base + w_off + j * 16 * PITCH + (((kk * 4 + q4) ^ swz) << 4));
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[t], wf[j], acc[t][j], 0, 0, 0);
    }
  };

  // Prologue: steps 0..PD-1 in flight, step 0 into LDS, then step PD replaces it in the registers.
#pragma unroll
  for (int s = 0; s < PD; ++s) gload(s, regs[s]);
  lstore(0, regs[0]);
  gload(PD, regs[0]);
  __syncthreads();
  // Main loop, unrolled by PD so that register-stage indices are compile-time.  It is branch-free:
  // steps past the end are clamped reloads whose activations are masked to zero.
  for (int i0 = 0; i0 < nk; i0 += PD) {
#pragma unroll
    for (int j = 0; j < PD; ++j) {
      const int i = i0 + j;
      compute(i & 1, (uint32_t) - (int)(i < nk));
      __builtin_amdgcn_sched_barrier(0);
      lstore((i + 1) & 1, regs[(j + 1) % PD]);           // step i+1 (loaded PD steps ago)
      __builtin_amdgcn_sched_barrier(0);
      gload(i + 1 + PD, regs[(j + 1) % PD]);
      __builtin_amdgcn_sched_barrier(0);
      __syncthreads();
    }
  }

#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int n = n0 + (wn * NT + j) * 16 + i16;
      const int mb = m0 + (wm * MT + t) * 16 + 4 * q4;
      if (n < a.N) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (mb + r < a.M) epilogue_store<EPI, uint16_t>(a, mb + r, k, n, acc[t][j][r]);
      }
    }
}

// Optional event pair recorded around the vocabulary-projection launch (benchmark hook).
hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;

// Weight rows per GEMV workgroup: 16 measured best on MI355X at 7B shapes (8, 32 and 64 were
// 1-10 % slower); fewer for small matrices so that the grid still covers the chip.
int gemv_rows_per_wg(int N, int K) {
  long rows = ((long)N * K / 1024) & ~7L;
  return rows < 8 ? 8 : (rows > 16 ? 16 : (int)rows);
}

template <int EPI>
int launch_gemm(const GemmArgs& a_in, medusa_dtype_t dtype, hipStream_t stream) {
  GemmArgs a = a_in;
  a.rows_per_wg = gemv_rows_per_wg(a.N, a.K);
  const int kGemvRowsPerWg = a.rows_per_wg;
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
  } else if (a.M <= 80) {
    // skinny: every wavefront sees all activation rows; 128 weight rows per workgroup when that
    // still yields a few hundred workgroups, else 64
    const int MT = ceil_div(a.M, 16);
    const bool wide = (long)ceil_div(a.N, 128) * a.K >= 200;   // measured at V = 32000: 52 us wide, 63 us narrow
    const dim3 grid(ceil_div(a.N, wide ? 128 : 64), a.K, 1);
#define MEDUSA_SKINNY(MT_)                                                                                         \
  case MT_:                                                                                                        \
    if (!wide) hipLaunchKernelGGL((gemm_lds_bf16_kernel<1, 4, MT_, 1, 64, 4, EPI>), grid, block, 0, stream, a);    \
    else hipLaunchKernelGGL((gemm_lds_bf16_kernel<1, 4, MT_, 2, 64, 4, EPI>), grid, block, 0, stream, a);          \
    break;
    switch (MT) {
      MEDUSA_SKINNY(1) MEDUSA_SKINNY(2) MEDUSA_SKINNY(3) MEDUSA_SKINNY(4) MEDUSA_SKINNY(5)
    }
#undef MEDUSA_SKINNY
  } else if ((size_t)a.N * a.d >= ((size_t)1 << 31) || (size_t)a.M * a.xs_m >= ((size_t)1 << 31)) {
    // byte offsets beyond 32 bits: 128 x 128 tile with 64-bit addressing, wavefronts 2 x 2, each 64 x 64
    const dim3 grid(ceil_div(a.N, 128), a.K, ceil_div(a.M, 128));
    hipLaunchKernelGGL((gemm_lds_bf16_kernel<2, 2, 4, 4, 64, 2, EPI>), grid, block, 0, stream, a);
  } else if ((size_t)a.N * a.d >= ((size_t)1 << 31) || (size_t)a.M * a.xs_m >= ((size_t)1 << 31)) {
    // element offsets beyond 31 bits: 128 x 128 tile with 64-bit addressing, wavefronts 2 x 2, each 64 x 64
    const dim3 grid(ceil_div(a.N, 128), a.K, ceil_div(a.M, 128));
    hipLaunchKernelGGL((gemm_lds_bf16_kernel<2, 2, 4, 4, 64, 2, EPI>), grid, block, 0, stream, a);
  } else {
    return launch_gemm_big(a, EPI, stream);
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
