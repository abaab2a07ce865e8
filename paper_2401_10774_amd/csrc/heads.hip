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

constexpr int kMaxSplitTiles = 1024;       // output tiles x heads a split reduction may cover

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
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint16_t* X = (const uint16_t*)a.X;
  const uint16_t* W = (const uint16_t*)a.W + (size_t)k * a.N * a.d;
  const int n_begin = blockIdx.x * a.rows_per_wg;
  const int n_end = min(n_begin + a.rows_per_wg, a.N);
  constexpr int R = 2, U = 4;

  // Work of a wavefront: row pairs nb = n_begin + 2 wave, + 8, ...; each row pair in batches of
  // U x 64 chunks.  The batches are software-pipelined: batch i+1 is requested before batch i is
  // multiplied, and the first batch before the activations are staged in LDS, so the weight stream
  // starts with the first instruction of the kernel.
  const int cpb = 64 * U;                       // chunks per batch and row
  const int bpr = (chunks + cpb - 1) / cpb;     // batches per row pair
  const int first_nb = n_begin + wave * R;
  const int n_pairs = first_nb < n_end ? (n_end - first_nb + 4 * R - 1) / (4 * R) : 0;
  const int n_batches = n_pairs * bpr;
  auto load_batch = [&](int bi, u32x4_t (&w)[R][U]) __attribute__((always_inline)) {
    const int pair = bi / bpr, c0 = (bi - pair * bpr) * cpb;
    const int nb = first_nb + pair * 4 * R;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const u32x4_t* wrow = (const u32x4_t*)(W + (size_t)min(nb + r, a.N - 1) * a.d);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int c = c0 + u * 64 + lane;
        w[r][u] = c < chunks ? __builtin_nontemporal_load(wrow + c) : u32x4_t{0, 0, 0, 0};
      }
    }
  };
  u32x4_t wa[R][U], wb[R][U];
  if (n_batches > 0) load_batch(0, wa);

  for (int i = threadIdx.x; i < MB * chunks; i += 256) {
    const int mm = i / chunks, c = i - mm * chunks;
    u32x4_t v = {0, 0, 0, 0};
    if (m0 + mm < a.M) v = *(const u32x4_t*)(X + x_row_offset<kHeadMajor<EPI>>(a, m0 + mm, k) + x_col_offset<kHeadMajor<EPI>>(a, c * 8));
    xs[i] = v;
  }
  __syncthreads();

  float acc[R][MB];
  auto multiply = [&](int bi, const u32x4_t (&w)[R][U]) __attribute__((always_inline)) {
    const int pair = bi / bpr, c0 = (bi - pair * bpr) * cpb;
    if (c0 == 0) {
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int mm = 0; mm < MB; ++mm) acc[r][mm] = 0.f;
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
    if (c0 + cpb >= chunks) {                   // last batch of the row pair: reduce and store
      const int nb = first_nb + pair * 4 * R;
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int mm = 0; mm < MB; ++mm) {
          const float s = wave_sum(acc[r][mm]);
          if (lane == 0 && nb + r < a.N && m0 + mm < a.M) epilogue_store<EPI, uint16_t>(a, m0 + mm, k, nb + r, s);
        }
    }
  };
  for (int bi = 0; bi < n_batches; bi += 2) {
    if (bi + 1 < n_batches) load_batch(bi + 1, wb);
    multiply(bi, wa);
    if (bi + 1 >= n_batches) break;
    if (bi + 2 < n_batches) load_batch(bi + 2, wa);
    multiply(bi + 1, wb);
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
    if (m0 + mm < a.M) v = *(const floatx4_t*)(X + x_row_offset<kHeadMajor<EPI>>(a, m0 + mm, k) + x_col_offset<kHeadMajor<EPI>>(a, c * 4));
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
//
// Split reduction: when the output has so few tiles that most of the chip would idle (the d x d
// and d x 4d/3 projections of a decoder block), ksplit workgroups share an output tile, each
// reducing a contiguous 1/ksplit of d (grid.z = m-tiles x ksplit).  They park their fp32 partial tiles in a workspace;
// the workgroup that arrives last adds them up in split order (so the result does not depend on
// which one that is) and runs the epilogue.
// ---------------------------------------------------------------------------------------
__device__ unsigned int g_gemm_ticket[kMaxSplitTiles];

template <int WM, int WN, int MT, int NT, int BK, int PD, int EPI, bool SPLIT = false>
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
  // (the split reduction is a template switch: its merge code would otherwise cost every
  // instantiation registers, and with them occupancy)
  const int n_split = SPLIT ? a.ksplit : 1, m_tile = blockIdx.z / n_split, split = blockIdx.z - m_tile * n_split;
  const int n0 = blockIdx.x * BN, m0 = m_tile * BM;
  const uint16_t* W = (const uint16_t*)a.W + (size_t)k * a.N * a.d;
  const uint16_t* X = (const uint16_t*)a.X;

  // Per-thread source pointers and LDS offsets of its LPT chunks (rows clamped into range; the
  // surplus chunk ids of the last slot repeat the final chunk, which is harmless).
  const uint16_t* src[LPT];
  int dst[LPT];
  bool is_x[LPT];
#pragma unroll
  for (int it = 0; it < LPT; ++it) {
    const int id = min(it * 256 + tid, CHUNKS - 1);
    const int row = id / CPR, c = id - row * CPR;
    is_x[it] = row < BM;
    src[it] = row < BM ? X + x_row_offset<kHeadMajor<EPI>>(a, min(m0 + row, a.M - 1), k) + c * 8
                       : W + (size_t)min(n0 + row - BM, a.N - 1) * a.d + c * 8;
    dst[it] = row * PITCH + ((c ^ ((row >> 1) & 7)) << 4);
  }

  floatx4_t acc[MT][NT];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[t][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  const int nk_all = a.d / BK;
  const int step0 = (int)((long)nk_all * split / n_split);
  const int nk = (int)((long)nk_all * (split + 1) / n_split) - step0;    // this workgroup's share of the reduction (>= 1)
  u32x4_t regs[PD][LPT];
  auto gload = [&](int step, u32x4_t (&r)[LPT]) {
    const int off_w = (step0 + min(step, nk - 1)) * BK;
    const int off_x = (int)x_col_offset<kHeadMajor<EPI>>(a, off_w);       // differs from off_w for head-major activations
#pragma unroll
    for (int it = 0; it < LPT; ++it) r[it] = *(const u32x4_t*)(src[it] + (is_x[it] ? off_x : off_w));
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

  if (SPLIT && n_split > 1) {
    // partial tile of this split: [fragment][register pair][thread], 8 bytes per thread and store
    const unsigned int tile = (k * gridDim.x + blockIdx.x) * (gridDim.z / n_split) + m_tile;
    constexpr int PART = MT * NT * 2 * 256;              // 8-byte words per partial tile
    uint64_t* part = (uint64_t*)a.ws + (size_t)tile * n_split * PART;
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int rp = 0; rp < 2; ++rp) {
          const uint64_t v = (uint64_t)__float_as_uint(acc[t][j][2 * rp]) | ((uint64_t)__float_as_uint(acc[t][j][2 * rp + 1]) << 32);
          store_agent(part + (size_t)split * PART + ((t * NT + j) * 2 + rp) * 256 + tid, v);
        }
    if (!last_workgroup_of(&g_gemm_ticket[tile], (unsigned int)n_split)) return;
    // Sum in split order.  The loads of a group of slots are all issued before the first sum (each is a
    // round trip to the memory side of the L2, where the other workgroups' stores are visible); splits
    // past the last one re-read the last one and are not added.
    constexpr int SLOTS = MT * NT * 2, GROUP = SLOTS >= 32 ? 8 : 4, MAXS = 8;
#pragma unroll
    for (int s0 = 0; s0 < SLOTS; s0 += GROUP) {
      uint64_t v[GROUP][MAXS];
#pragma unroll
      for (int g = 0; g < GROUP; ++g)
#pragma unroll
        for (int z = 0; z < MAXS; ++z) {
          const int slot = s0 + g < SLOTS ? s0 + g : SLOTS - 1;
          v[g][z] = load_agent(part + (size_t)min(z, n_split - 1) * PART + slot * 256 + tid);
        }
#pragma unroll
      for (int g = 0; g < GROUP; ++g) {
        if (s0 + g >= SLOTS) continue;
        float lo = 0.f, hi = 0.f;
#pragma unroll
        for (int z = 0; z < MAXS; ++z)
          if (z < n_split) {
            lo += __uint_as_float((uint32_t)v[g][z]);
            hi += __uint_as_float((uint32_t)(v[g][z] >> 32));
          }
        const int slot = s0 + g, frag = slot >> 1, rp = slot & 1;
        acc[frag / NT][frag % NT][2 * rp] = lo;
        acc[frag / NT][frag % NT][2 * rp + 1] = hi;
      }
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

// Which kernel a bf16 GEMM of M rows goes to, and in what shape.
//   M <= 4                         wave-per-row GEMV.
//   about one 192/128 x 256 tile per CU or more (M > 80)   the large-tile kernel (gemm_big.hip).
//   otherwise                      the LDS-staged kernel in its skinny arrangement: row blocks of
//     16*mt <= 128 activation rows (every wavefront sees all rows of its block), 128 weight rows
//     per workgroup when that alone gives a few hundred workgroups, else 64, and the reduction
//     split over up to 8 workgroups when even those are too few.  (Measured at M = 65,
//     N = d = 4096: 64-row tiles x 8 splits 21 us, 128-row tiles x 8 splits 27 us, unsplit 37 us:
//     the number of workgroups matters more than the activation re-reads.)
//   M > 80 and at least 200 tiles of 128 x 128: those tiles, wavefronts 2 x 2, unsplit (at M = 356
//     and 1040 the skinny arrangement was up to 1.5x faster below that tile count and up to 1.6x
//     slower above it; splitting the 128 x 128 kernel's reduction never paid for its 64 KB partials).
struct GemmPlan {
  enum { GEMV, SKINNY, SQUARE, BIG } kind;
  bool wide;
  int mt, m_blocks, ksplit;
};
GemmPlan plan_gemm(int M, int N, int d, int K, bool have_ws, bool wide_offsets) {
  GemmPlan p = {GemmPlan::GEMV, false, 1, 1, 1};
  if (M <= 4) return p;
  if (M > 80 && !wide_offsets) {                            // (the large-tile kernel addresses with 32-bit element offsets)
    const bool tall = ceil_div(M, 192) * 192 <= ceil_div(M, 128) * 128;
    if ((long)ceil_div(M, tall ? 192 : 128) * ceil_div(N, 256) * K >= 200) {
      p.kind = GemmPlan::BIG;
      return p;
    }
  }
  p.m_blocks = ceil_div(M, 128);
  if (M > 80 && (long)ceil_div(N, 128) * p.m_blocks * K >= 200) {
    // enough 128 x 128 tiles to fill the chip: wavefronts 2 x 2 (half the LDS reads per MFMA of the
    // skinny arrangement), never split
    p.kind = GemmPlan::SQUARE;
    p.wide = true;
    p.mt = 4;
    return p;
  }
  p.kind = GemmPlan::SKINNY;
  p.mt = ceil_div(ceil_div(M, p.m_blocks), 16);
  p.wide = (long)ceil_div(N, 128) * K * p.m_blocks >= 200;  // measured at V = 32000, M = 65: 52 us wide, 63 us narrow
  if (!have_ws) return p;
  const long tiles = (long)ceil_div(N, p.wide ? 128 : 64) * K * p.m_blocks;
  if (tiles >= 384 || tiles > kMaxSplitTiles) return p;
  long s = 512 / tiles;
  const long by_steps = (d / 64) / 8;                       // at least 8 reduction steps per split
  s = s < by_steps ? s : by_steps;
  p.ksplit = (int)(s < 1 ? 1 : (s > 8 ? 8 : s));
  return p;
}
// Workspace for the fp32 partial tiles of a split reduction (0 if this shape is not split).
size_t gemm_ws_bytes(int M, int N, int d, int K) {
  const GemmPlan p = plan_gemm(M, N, d, K, true, false);
  if (p.kind != GemmPlan::SKINNY || p.ksplit <= 1) return 0;
  const int frags = p.mt * (p.wide ? 2 : 1);                // accumulator fragments per thread
  return (size_t)ceil_div(N, p.wide ? 128 : 64) * K * p.m_blocks * p.ksplit * frags * 4 * 256 * sizeof(float);
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
  a.ksplit = 1;
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
  } else {
    const bool wide_offsets = (size_t)a.N * a.d >= ((size_t)1 << 31) || x_extent(a) >= ((size_t)1 << 31);
    const GemmPlan plan = plan_gemm(a.M, a.N, a.d, a.K, a.ws != nullptr, wide_offsets);
    if (plan.kind == GemmPlan::BIG) return launch_gemm_big(a, EPI, stream);
    const bool wide = plan.wide;
    a.ksplit = plan.ksplit;
    // split reductions exist for the epilogues tree_linear uses (medusa_heads passes no workspace)
    constexpr bool kCanSplit = EPI == EPI_PLAIN || EPI == EPI_GATED;
    const bool split = kCanSplit && a.ksplit > 1;
    if (!split) a.ksplit = 1;
    const dim3 grid(ceil_div(a.N, wide ? 128 : 64), a.K, plan.m_blocks * a.ksplit);
    if (plan.kind == GemmPlan::SQUARE) {
      hipLaunchKernelGGL((gemm_lds_bf16_kernel<2, 2, 4, 4, 64, 2, EPI, false>), grid, block, 0, stream, a);
      MEDUSA_LAUNCH_CHECK();
      return MEDUSA_OK;
    }
#define MEDUSA_SKINNY(MT_)                                                                                                     \
  case MT_:                                                                                                                    \
    if (split) {                                                                                                               \
      if (!wide) hipLaunchKernelGGL((gemm_lds_bf16_kernel<1, 4, MT_, 1, 64, 4, EPI, kCanSplit>), grid, block, 0, stream, a);   \
      else hipLaunchKernelGGL((gemm_lds_bf16_kernel<1, 4, MT_, 2, 64, 4, EPI, kCanSplit>), grid, block, 0, stream, a);         \
    } else {                                                                                                                   \
      if (!wide) hipLaunchKernelGGL((gemm_lds_bf16_kernel<1, 4, MT_, 1, 64, 4, EPI, false>), grid, block, 0, stream, a);       \
      else hipLaunchKernelGGL((gemm_lds_bf16_kernel<1, 4, MT_, 2, 64, 4, EPI, false>), grid, block, 0, stream, a);             \
    }                                                                                                                          \
    break;
    switch (plan.mt) {
      MEDUSA_SKINNY(1) MEDUSA_SKINNY(2) MEDUSA_SKINNY(3) MEDUSA_SKINNY(4) MEDUSA_SKINNY(5) MEDUSA_SKINNY(6)
      MEDUSA_SKINNY(7) MEDUSA_SKINNY(8)
    }
#undef MEDUSA_SKINNY
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
  GemmArgs a = {};
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

// Backbone linear layer on the tree tokens (App. G, operator table, parallel-decoding rows).
extern "C" size_t tree_linear_workspace_bytes(int B, int T, int d_in, int d_out, medusa_dtype_t dtype) {
  if (dtype != MEDUSA_BF16 || B < 1 || T < 1 || d_in < 64 || d_out < 1) return 0;
  return gemm_ws_bytes(B * T, d_out, d_in, 1);
}

extern "C" int tree_linear(const void* x, const void* w, const void* mul, void* y, int B, int T, int d_in, int d_out,
                           int x_heads, int y_heads, medusa_dtype_t dtype, void* workspace, size_t workspace_bytes,
                           medusa_stream_t stream_) {
  if (!x || !w || !y) return MEDUSA_EINVAL;
  if (B < 1 || T < 1 || d_in < 1 || d_out < 1 || x_heads < 0 || y_heads < 0) return MEDUSA_EINVAL;
  if (dtype != MEDUSA_F32 && dtype != MEDUSA_BF16) return MEDUSA_EINVAL;
  const long M = (long)B * T;
  if (M > 4096 || d_in > 65536) return MEDUSA_EUNSUPPORTED;
  const int gran = dtype == MEDUSA_BF16 ? 64 : 8;       // reduction elements the kernels fetch as one contiguous piece
  if (d_in % gran != 0) return MEDUSA_EUNSUPPORTED;
  if (x_heads > 0 && (d_in % x_heads != 0 || (d_in / x_heads) % gran != 0)) return MEDUSA_EUNSUPPORTED;
  if (y_heads > 0 && d_out % y_heads != 0) return MEDUSA_EINVAL;
  GemmArgs a = {};
  a.W = w;
  a.X = x;
  a.hidden = mul;
  a.out = y;
  a.M = (int)M;
  a.N = d_out;
  a.d = d_in;
  a.K = 1;
  a.xs_m = d_in;
  a.xs_k = 0;
  if (x_heads > 0) {
    a.x_T = T;
    a.x_heads = x_heads;
    a.x_dh = d_in / x_heads;
  }
  if (y_heads > 0) {
    a.y_T = T;
    a.y_heads = y_heads;
    a.y_dh = d_out / y_heads;
  }
  // the split reduction is an optimisation: without (enough) workspace the call runs unsplit
  if (workspace && dtype == MEDUSA_BF16 && workspace_bytes >= gemm_ws_bytes(a.M, a.N, a.d, 1) && gemm_ws_bytes(a.M, a.N, a.d, 1) > 0)
    a.ws = workspace;
  hipStream_t stream = (hipStream_t)stream_;
  return mul ? launch_gemm<EPI_GATED>(a, dtype, stream) : launch_gemm<EPI_PLAIN>(a, dtype, stream);
}

extern "C" int medusa_profile_set_events(void* start, void* stop) {
  if ((start == nullptr) != (stop == nullptr)) return MEDUSA_EINVAL;
  g_prof_start = (hipEvent_t)start;
  g_prof_stop = (hipEvent_t)stop;
  return MEDUSA_OK;
}
