// medusa_heads (Sec. 2.1.1 of the Medusa paper): logits_k = W2_k . (SiLU(W1_k . h) + h).
//
// Both GEMMs are "skinny": M (batch rows, or batch x tree tokens) is tiny next to the
// d x d and V x d weight matrices, so the weights are streamed from HBM exactly once and
// the kernels are organised around that stream:
//   * M <= 2  (bf16): one wavefront per weight row, 16-byte non-temporal loads that cover
//                     1 KB of the row per instruction, packed bf16 dot products on the
//                     vector ALUs, activations resident in LDS (also three or four rows on small matrices).
//   * more rows (bf16): 16x16x32 bf16 MFMA tiles.  Up to 96 activation rows per row block: 1 KB runs
//                     of 48-128 weight rows go from global memory straight into an LDS ring (the
//                     ring kernel); larger row blocks and short split reductions: a double-buffered
//                     LDS tile filled through registers several reduction steps ahead; from about
//                     a hundred rows on, 128 x 128 tiles or the large tiles of gemm_big.hip.
//   * fp32          : plain FMA version of the first scheme (small configurations only).
// The residual block's epilogue applies SiLU, adds h and rounds once to the storage type.
#include "gemm_args.hpp"

namespace {

constexpr int kMaxSplitTiles = 1024;       // output tiles x heads a split reduction may cover
constexpr int kMaxRows = 16384;            // activation rows per call (a batch of 128 trees of 128 tokens); grids and 32-bit offsets are sized for it

// ---------------------------------------------------------------------------------------
// bf16, M <= 4 per block of rows: wave-per-row streaming GEMV.
// grid (row blocks, K, m blocks), 256 threads.  LDS: MB x d bf16.
// ---------------------------------------------------------------------------------------

template <int MB, int EPI>
__global__ __launch_bounds__(MB >= 3 ? 512 : 256) void gemv_bf16_kernel(GemmArgs a) {
  constexpr int NWV = MB >= 3 ? 8 : 4;          // wavefronts per workgroup (more of them share the bigger LDS staging)
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
  const int n_pairs = first_nb < n_end ? (n_end - first_nb + NWV * R - 1) / (NWV * R) : 0;
  const int n_batches = n_pairs * bpr;
  auto load_batch = [&](int bi, u32x4_t (&w)[R][U]) __attribute__((always_inline)) {
    const int pair = bi / bpr, c0 = (bi - pair * bpr) * cpb;
    const int nb = first_nb + pair * NWV * R;
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

  for (int i = threadIdx.x; i < MB * chunks; i += 64 * NWV) {
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
      const int nb = first_nb + pair * NWV * R;
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

__device__ unsigned int g_gemm_ticket[kTicketSlots][kMaxSplitTiles];

// Tail shared by the MFMA kernels of this file.  On entry every thread holds, for each of its
// MT x NT accumulator fragments, rows m0 + (wm*MT + t)*16 + 4*(lane/16)..+3 of column
// n0 + (wn*NT + j)*16 + lane%16.  With a split reduction the partial tiles go to the workspace and
// only the workgroup that arrives last carries on, with the sum; then the epilogue stores.
template <int MT, int NT, int EPI, bool SPLIT>
__device__ __forceinline__ void finish_tile(const GemmArgs& a, floatx4_t (&acc)[MT][NT], int k, int m_tile, int split,
                                            int n_split, int n0, int m0, int wm, int wn) {
  const int tid = threadIdx.x, lane = tid & 63, i16 = lane & 15, q4 = lane >> 4;
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
    if (!last_workgroup_of(&g_gemm_ticket[a.ticket_slot][tile], (unsigned int)n_split)) return;
    // Sum in split order.  Every load is a round trip to the memory side of the L2 (where the other
    // workgroups' stores are visible), so as many as the registers hold are issued before the first
    // sum: the whole tile of ZB splits at a time, which is all of them for the usual split counts.
    constexpr int SLOTS = MT * NT * 2, ZB = SLOTS <= 10 ? 8 : (SLOTS <= 20 ? 4 : 2);
    float lo[SLOTS], hi[SLOTS];
#pragma unroll
    for (int sl = 0; sl < SLOTS; ++sl) lo[sl] = hi[sl] = 0.f;
    for (int z0 = 0; z0 < n_split; z0 += ZB) {
      uint64_t v[ZB][SLOTS];
#pragma unroll
      for (int zz = 0; zz < ZB; ++zz)
        if (z0 + zz < n_split) {
#pragma unroll
          for (int sl = 0; sl < SLOTS; ++sl) v[zz][sl] = load_agent(part + (size_t)(z0 + zz) * PART + sl * 256 + tid);
        }
#pragma unroll
      for (int zz = 0; zz < ZB; ++zz)
        if (z0 + zz < n_split) {
#pragma unroll
          for (int sl = 0; sl < SLOTS; ++sl) {
            lo[sl] += __uint_as_float((uint32_t)v[zz][sl]);
            hi[sl] += __uint_as_float((uint32_t)(v[zz][sl] >> 32));
          }
        }
    }
#pragma unroll
    for (int sl = 0; sl < SLOTS; ++sl) {
      const int frag = sl >> 1, rp = sl & 1;
      acc[frag / NT][frag % NT][2 * rp] = lo[sl];
      acc[frag / NT][frag % NT][2 * rp + 1] = hi[sl];
    }
  }

  if constexpr (EPI == EPI_SWIGLU) {
    // the wavefront's two fragments are the gate rows and the up rows of output columns 16b..16b+15
    static_assert(NT == 2, "gate and up fragments side by side");
    const int n = (n0 >> 1) + wn * 16 + i16, n_out = a.N >> 1;
    if (n >= n_out) return;
    const size_t col = out_col_offset<true>(a, n);
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const int mb = m0 + (wm * MT + t) * 16 + 4 * q4;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (mb + r >= a.M) continue;
        const float g = acc[t][0][r], u = acc[t][1][r];
        const float v = g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g)) * u;
        const size_t row = a.y_dh == 0 ? (size_t)(mb + r) * n_out : out_row_offset<true>(a, mb + r, k);
        store_from_float<uint16_t>((uint16_t*)a.out + row + col, v);
      }
    }
    return;
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

// ---------------------------------------------------------------------------------------
// bf16, more rows than the GEMV takes: LDS-staged MFMA GEMM (v_mfma_f32_16x16x32_bf16).
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

  finish_tile<MT, NT, EPI, SPLIT>(a, acc, k, m_tile, split, n_split, n0, m0, wm, wn);
}

// ---------------------------------------------------------------------------------------
// bf16, 4 < M <= ~128 per row block: skinny MFMA GEMM whose wavefronts split the reduction.
//
// Workgroup tile BM x BN = 16*MT activation rows x 16*NTW weight rows, reduction in stages of 128
// elements (256 bytes per row).  The four wavefronts each take one 32-element slice of a stage
// and the WHOLE tile: every 16-byte LDS chunk is then read by exactly one wavefront, where an
// arrangement that splits the weight rows over the wavefronts has each of them read all the
// activation rows (3.6x the LDS reads at MT = 5), and LDS time, not HBM, set the pace of that
// arrangement from M = 48 upwards.  After the loop the four partial tiles are added through LDS
// (in wavefront order), wavefront w ending up with the NTW/4 column fragments w*NTW/4.. of all
// rows: the accumulator layout finish_tile() expects for wavefronts arranged 1 x 4.
//
// Loads: thread t fetches, for each of the MT + NTW groups of 16 rows, the 16-byte chunk t%16 of
// row t/16 of the group: 16 consecutive lanes cover 256 contiguous bytes of a row.  They are
// held in registers PD stages ahead of their use and written to a double-buffered LDS tile with
// chunk c of row r at slot c ^ (r%16), which keeps both the row-major stores and the fragment
// reads (16 rows x 4 chunks per instruction) free of bank conflicts.  One barrier per stage.
// An odd number of 64-element steps leaves the second half of the last stage empty: wavefronts 2
// and 3 multiply zeros there.  grid (ceil(N/BN), K, ceil(M/BM)), 256 threads, dynamic LDS 2*(BM+BN)*256.
// (Reductions split over workgroups stay with the kernel above.)
// ---------------------------------------------------------------------------------------
template <int MT, int NTW, int PD, int EPI>
__global__ __launch_bounds__(256) void gemm_skinny_bf16_kernel(GemmArgs a) {
  constexpr int NT = NTW / 4;                         // column fragments a wavefront owns in the end
  constexpr int BM = 16 * MT, BN = 16 * NTW;
  constexpr int LPT = MT + NTW;                       // chunks per thread and stage
  constexpr int STAGE = (BM + BN) * 256;
  constexpr bool HM = kHeadMajor<EPI>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_dyn[];
  unsigned char* lds = lds_dyn;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, q4 = lane >> 4;
  const int k = blockIdx.y;
  const int m_tile = blockIdx.z;
  const int n0 = blockIdx.x * BN, m0 = m_tile * BM;
  // Byte offsets from the tile's first weight row (< 128 rows x d) and from X fit 32 bits.
  const unsigned char* Wt = (const unsigned char*)((const uint16_t*)a.W + ((size_t)k * a.N + n0) * a.d);
  const unsigned char* Xb = (const unsigned char*)a.X;
  const int r16 = tid >> 4, c16 = tid & 15, half = c16 >> 3;
  uint32_t goff[LPT];
#pragma unroll
  for (int it = 0; it < LPT; ++it)
    goff[it] = it < MT ? (uint32_t)(x_row_offset<HM>(a, min(m0 + it * 16 + r16, a.M - 1), k) * 2) + (c16 & 7) * 16
                       : (uint32_t)min((it - MT) * 16 + r16, a.N - 1 - n0) * (uint32_t)a.d * 2u + (c16 & 7) * 16;
  const int st_off = r16 * 256 + ((c16 ^ r16) << 4);  // (row%16 == r16 for every group of 16 rows)

  const int nk = a.d >> 6;                            // 64-element steps
  const int stages = (nk + 1) >> 1;
  // Every workgroup walks the reduction from a different stage, wrapping around (the sum's order
  // depends on the tile, not on the run).  All of a tile's rows are one row pitch apart, so the
  // pieces a workgroup requests together fall on few memory channels; workgroups that start in
  // lockstep at element 0 would all crowd the same ones (cold 262 MB matrix read this way, MI355X:
  // 4.5 TB/s in lockstep, 5.5-5.8 rotated).
  const int rot = (int)((blockIdx.x * 5u) % (unsigned)stages);
  auto rotated = [&](int stage) { const int st = min(stage, stages - 1) + rot; return st >= stages ? st - stages : st; };

  u32x4_t regs[PD][LPT];
  auto gload = [&](int stage_l, u32x4_t (&r)[LPT]) __attribute__((always_inline)) {
    // this thread's chunk lies in the first or second 64-element step of the stage; past the end
    // of the reduction the last step is fetched again (and never used)
    const int stage = rotated(stage_l);
    const int e0 = min(2 * stage, nk - 1) * 64, e1 = min(2 * stage + 1, nk - 1) * 64;
    const uint32_t so_w = (uint32_t)(half ? e1 : e0) * 2u;
    const uint32_t so_x = (uint32_t)(half ? x_col_offset<HM>(a, e1) : x_col_offset<HM>(a, e0)) * 2u;
#pragma unroll
    for (int it = 0; it < LPT; ++it)
      r[it] = it < MT ? *(const u32x4_t*)(Xb + (goff[it] + so_x)) : *(const u32x4_t*)(Wt + (goff[it] + so_w));
  };
  // (activation chunks of a half stage past the end of the reduction are stored as zeros)
  auto lstore = [&](int buf, int stage_l, const u32x4_t (&r)[LPT]) __attribute__((always_inline)) {
    unsigned char* b = lds + buf * STAGE + st_off;
    const uint32_t keep = (uint32_t) - (int)(2 * rotated(stage_l) + half < nk);
#pragma unroll
    for (int it = 0; it < LPT; ++it) *(u32x4_t*)(b + it * 4096) = it < MT ? (r[it] & keep) : r[it];
  };
  floatx4_t acc[MT][NTW];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int j = 0; j < NTW; ++j) acc[t][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  // fragment of this wavefront's slice: row i16 of a group of 16, chunk wave*4 + q4
  const int fr_off = i16 * 256 + (((wave * 4 + q4) ^ i16) << 4);
  bf16x8_t xf[MT], wf[NTW];
  auto lfrag = [&](int buf) __attribute__((always_inline)) {
    const unsigned char* b = lds + buf * STAGE + fr_off;
#pragma unroll
    for (int t = 0; t < MT; ++t) xf[t] = *(const bf16x8_t*)(b + t * 4096);
#pragma unroll
    for (int j = 0; j < NTW; ++j) wf[j] = *(const bf16x8_t*)(b + (MT + j) * 4096);
  };
  auto mfma = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < NTW; ++j)
#pragma unroll
      for (int t = 0; t < MT; ++t) acc[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[t], wf[j], acc[t][j], 0, 0, 0);
  };

  // Prologue: stages 0..PD-1 requested, stage 0 into LDS.
#pragma unroll
  for (int s = 0; s < PD; ++s) gload(s, regs[s]);
  lstore(0, 0, regs[0]);
  __syncthreads();
  // Main loop, unrolled by PD so that the register stage is a compile-time index.  On entry of
  // stage s its data is in LDS buffer s%2 and register stage s%PD is free.  Instruction order, given
  // to the scheduler as groups (masks: 0x008 MFMA, 0x020 global load, 0x100 LDS read, 0x200 LDS
  // store): the fragment reads, then the requests for stage s+PD under the first MFMAs, and the LDS
  // stores of stage s+1 -- which wait for that stage to arrive -- under the last ones.
  constexpr int NMF = MT * NTW;
  for (int s0 = 0; s0 < stages; s0 += PD) {
#pragma unroll
    for (int j = 0; j < PD; ++j) {
      const int s = s0 + j;
      if (s >= stages) break;
      const int cur = s & 1;
      lfrag(cur);
      gload(s + PD, regs[j]);
      mfma();
      lstore(cur ^ 1, s + 1, regs[(j + 1) % PD]);
      __builtin_amdgcn_sched_group_barrier(0x100, LPT, 0);
#pragma unroll
      for (int g = 0; g < LPT; ++g) {
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      }
      if (NMF > 2 * LPT) __builtin_amdgcn_sched_group_barrier(0x008, NMF - 2 * LPT, 0);
#pragma unroll
      for (int g = 0; g < LPT; ++g) {
        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      }
      __syncthreads();
    }
  }

  // Add the four wavefronts' partial tiles, RT groups of 16 rows at a time: each wavefront writes its
  // fragments (one 16-byte slot per lane), then collects the four partials of the fragments it owns.
  constexpr int RT = (2 * STAGE) / (4 * NTW * 1024) < MT ? (2 * STAGE) / (4 * NTW * 1024) : MT;
  static_assert(RT >= 1, "the reduction area must hold one group of rows");
  floatx4_t fin[MT][NT];
#pragma unroll
  for (int t0 = 0; t0 < MT; t0 += RT) {
    __syncthreads();                                     // the area (stage buffers, or the previous round) is free
#pragma unroll
    for (int t = t0; t < t0 + RT && t < MT; ++t)
#pragma unroll
      for (int j = 0; j < NTW; ++j)
        *(floatx4_t*)(lds + ((((t - t0) * 4 + wave) * NTW + j) * 64 + lane) * 16) = acc[t][j];
    __syncthreads();
#pragma unroll
    for (int t = t0; t < t0 + RT && t < MT; ++t)
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        floatx4_t sum = *(const floatx4_t*)(lds + ((((t - t0) * 4 + 0) * NTW + wave * NT + j) * 64 + lane) * 16);
#pragma unroll
        for (int w = 1; w < 4; ++w) sum += *(const floatx4_t*)(lds + ((((t - t0) * 4 + w) * NTW + wave * NT + j) * 64 + lane) * 16);
        fin[t][j] = sum;
      }
  }
  finish_tile<MT, NT, EPI, false>(a, fin, k, m_tile, 0, 1, n0, m0, 0, wave);
}

// ---------------------------------------------------------------------------------------
// bf16, up to 96 rows per row block (the ring kernel): the weights of a tile are fetched in 1 KB runs
// and nothing passes through registers on its way to LDS.
//
// Cold weights stream from HBM at 4.4 TB/s when a workgroup asks for 256 bytes of each of its 128
// rows at a time, at 5.3 TB/s for 1 KB of 32 rows (measured with a plain read kernel), so the
// reduction advances in super-stages of 512 elements, and within one the tile's NTW column fragments
// (16 weight rows x 1 KB each) take turns: sub-stage u = NTW S + j is fragment j of super-stage S.
// Weights and activation rows go from global memory straight into LDS (global_load_lds_dwordx4, one
// instruction = one row's 1 KB run): the weights into a ring of NR buffers of one sub-stage each, so
// that NR - 1 sub-stages are in flight whatever the register budget; the activation rows of a
// super-stage (16 MT x 1 KB) into a single slab.  Each wavefront copies the fragments of its
// 128-element slice of the slab into registers at j = 0 and keeps them for the super-stage, which
// frees the slab for the next one's rows, requested at j = 1.  As in the kernel above the
// wavefronts split the reduction, not the tile, and their partial tiles are added through LDS at the
// end.  The swizzle of the LDS rows (chunk c of row r in slot c ^ (r%16) of its 256-byte group: fragment
// reads free of bank conflicts) is applied on the global side: the lane that fills slot p fetches
// chunk p ^ (r%16).
// Per sub-stage and wavefront: wait until its own loads of sub-stage u have landed (the load counter:
// loads complete in order, so "at most n outstanding" with n = the loads issued after them), barrier,
// request sub-stage u + NR - 1 into the buffer sub-stage u - 1 has just left, read the four weight
// fragments of the wavefront's slice, 4 MT MFMAs.  The loads are invisible to the compiler (see
// load_to_lds_b128), and so is their completion.
// Elements past d in the last super-stage: the weights' chunk index is clamped (any finite value
// does), the activation fragments are zeroed in registers.
// Narrower tiles (NTW = 6, 4, 3, 2 fragments) exist so that an output of a few thousand columns
// still gives every CU a workgroup; the price is the activation rows, which every workgroup fetches.
// Cold 32000 x 4096 matrix on MI355X, against the register-staged kernel this one replaced: M = 5..16
// 48 -> 44 us (6.0 TB/s), M = 65 52.5 -> 49; 32000 x 5120: M = 16 59 -> 50, M = 65 76 -> 66.
// grid (ceil(N/(16 NTW)), K, ceil(M/BM)), 256 threads, dynamic LDS (16 MT + 16 NR) KB.
// ---------------------------------------------------------------------------------------
template <int MT, int NTW, int NR, int EPI, bool SPLIT = false>
__global__ __launch_bounds__(256) void gemm_ring_bf16_kernel(GemmArgs a) {
  constexpr int BM = 16 * MT, BN = 16 * NTW;
  constexpr int XL = MT * 4;                           // activation rows (load instructions) per wavefront and super-stage
  constexpr int WL = 4;                                // weight rows per wavefront and sub-stage
  constexpr int SLAB = BM * 1024, SUB = 16 * 1024;
  constexpr bool HM = kHeadMajor<EPI>;
  static_assert(NTW >= 2 && NTW <= 8, "the activation rows of the next super-stage are requested at j = 1");
  static_assert(NR >= 3 && NR <= 8, "the count of loads issued after a sub-stage's own assumes 3..8 buffers");
  static_assert(WL * (NR - 2) + XL <= 63, "load counter");
  constexpr int PASSES = 4 * MT * NTW <= 16 * (MT + NR) ? 1 : 2;   // the four partial tiles go through the loop's LDS whole, or in two halves of the row groups
  static_assert(MT % PASSES == 0 && 4 * (MT / PASSES) * NTW <= 16 * (MT + NR), "half of the four partial tiles must fit the LDS the loop used");
  static_assert(EPI != EPI_SWIGLU || NTW % 2 == 0, "gate and up fragments come in pairs");
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_dyn[];
  unsigned char* lds = lds_dyn;                        // [slab][ring of NR weight buffers]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, q4 = lane >> 4;
  const int k = blockIdx.y;
  // Split reduction (a template switch, as above): ksplit workgroups share a tile, each taking a
  // contiguous share of the super-stages (at least one: the host's business).
  const int n_split = SPLIT ? a.ksplit : 1, split = SPLIT ? (int)blockIdx.z : 0;
  // Row blocks of one column tile get workgroup ids 8 apart, which the hardware places on one die: the
  // first block's weights come from HBM, the others find them in that die's L2.  (With ids a whole
  // row of column tiles apart they land on different dies whenever the column tiles are no multiple
  // of 8, and every block streams the weights from HBM: N = 11008, 2 x 65 rows 44 against 34 us.)
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int col_tile = a.m_blocks > 1 ? (slot / a.m_blocks) * 8 + xcd : (int)blockIdx.x;
  const int m_tile = a.m_blocks > 1 ? slot % a.m_blocks : 0;
  const int n0 = col_tile * BN, m0 = m_tile * BM;
  if (n0 >= a.N) return;                               // (the whole workgroup, before any barrier)
  const unsigned char* Wt = (const unsigned char*)((const uint16_t*)a.W + ((size_t)k * a.N + n0) * a.d);
  const unsigned char* Xb = (const unsigned char*)a.X;
  const int n_super = (a.d + 511) >> 9;
  const int s_first = (int)((long)n_super * split / n_split);
  const int n_mine = (int)((long)n_super * (split + 1) / n_split) - s_first, total = n_mine * NTW;
  const int c_last = ((a.d - (n_super - 1) * 512) >> 3) - 1;   // last valid chunk of the last super-stage
  // every workgroup starts its share of the reduction at a different super-stage and wraps around (see the kernel above)
  const int rot = (int)(((unsigned)col_tile * 3u) % (unsigned)n_mine);
  auto rotated = [&](int S) { const int Sr = S + rot; return s_first + (Sr >= n_mine ? Sr - n_mine : Sr); };

  // Rows this wavefront fetches: weight rows 16 j + 4 i + wave of the tile, activation rows 4 q + wave
  // of the block; either way the row's index mod 16 is 4 i' + wave (i' = i, q%4), and the chunk
  // this lane fetches for slot `lane` of such a row is cidx[i'].
  const int w_last = a.N - 1 - n0;
  const uint32_t w_pitch = (uint32_t)a.d * 2u;
  int cidx[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) cidx[i] = (lane & ~15) | ((lane ^ (4 * i + wave)) & 15);
  uint32_t xoff[XL];
#pragma unroll
  for (int q = 0; q < XL; ++q) xoff[q] = (uint32_t)(x_row_offset<HM>(a, min(m0 + q * 4 + wave, a.M - 1), k) * 2);

  auto issue_w = [&](int S, int j, int buf) __attribute__((always_inline)) {
    const int Sw = rotated(S);
    unsigned char* dst = lds + SLAB + buf * SUB + wave * 1024;
#pragma unroll
    for (int i = 0; i < WL; ++i) {
      const int c = Sw == n_super - 1 ? min(cidx[i], c_last) : cidx[i];
      const uint32_t off = (uint32_t)min(j * 16 + i * 4 + wave, w_last) * w_pitch + (uint32_t)(Sw * 1024 + c * 16);
      load_to_lds_b128<true>(Wt + off, dst + i * 4096);
    }
  };
  auto issue_x = [&](int S) __attribute__((always_inline)) {
    const int Sx = rotated(S);
    uint32_t so[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = Sx == n_super - 1 ? min(cidx[i], c_last) : cidx[i];
      so[i] = (uint32_t)(x_col_offset<HM>(a, Sx * 512 + (c & ~7) * 8) * 2) + (c & 7) * 16;
    }
#pragma unroll
    for (int q = 0; q < XL; ++q) load_to_lds_b128<false>(Xb + (xoff[q] + so[q & 3]), lds + (q * 4 + wave) * 1024);
  };

  floatx4_t acc[MT][NTW];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int j = 0; j < NTW; ++j) acc[t][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  // fragment reads: row i16 of a group of 16, chunks wave*16 + ks*4 + q4 (this wavefront's 128 elements)
  int fr_off[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int c = wave * 16 + ks * 4 + q4;
    fr_off[ks] = i16 * 1024 + (((c & ~15) | ((c ^ i16) & 15)) << 4);
  }
  bf16x8_t xf[MT][4], wf[4];

  // Everything this wavefront has loaded so far the ordinary way must have arrived before the first
  // hand-counted load, or the counts below would include it.
  wait_loads_outstanding<0>();
  issue_x(0);
  // sub-stages 0 .. NR-2
  {
    int Sp = 0, jp = 0;
#pragma unroll
    for (int u = 0; u < NR - 1; ++u) {
      if (u < total) issue_w(Sp, jp, u);               // (a reduction shorter than the ring: every wait below is for everything)
      if (++jp == NTW) { jp = 0; ++Sp; }
    }
  }
  int buf = 0;                                         // buffer of sub-stage u
  int Sn = (NR - 1) / NTW, jn = (NR - 1) % NTW;        // super-stage and fragment of sub-stage u + NR - 1
  for (int S = 0; S < n_mine; ++S) {
    const bool last_super = rotated(S) == n_super - 1;
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
      const int u = S * NTW + j;
      // Loads issued after this sub-stage's own: the weights of sub-stages u+1 .. u+NR-2 and, for
      // j = 2 .. NR-1, the activation rows of the next super-stage (issued at j = 1, before that
      // step's weights).  At j = 0 the slab must be complete as well: its rows were requested NTW - 1
      // sub-stages ago.  Near the end fewer loads exist: wait for everything then.
      constexpr int kAfter0 = WL * (NR - 2 < NTW - 1 ? NR - 2 : NTW - 1);
      if (u + NR - 2 >= total) wait_loads_outstanding<0>();
      else if (j == 0) wait_loads_outstanding<kAfter0>();
      else if (j >= 2 && j <= NR - 1 && S + 1 < n_mine) wait_loads_outstanding<WL * (NR - 2) + XL>();
      else wait_loads_outstanding<WL * (NR - 2)>();
      lds_barrier();
      if (j == 1 && S + 1 < n_mine) issue_x(S + 1);
      if (u + NR - 1 < total) {
        issue_w(Sn, jn, buf == 0 ? NR - 1 : buf - 1);
        if (++jn == NTW) { jn = 0; ++Sn; }
      }
      if (j == 0) {
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {
            bf16x8_t f = *(const bf16x8_t*)(lds + t * 16384 + fr_off[ks]);
            if (last_super && wave * 16 + ks * 4 + q4 > c_last) f = bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
            xf[t][ks] = f;
          }
      }
      const unsigned char* wb = lds + SLAB + buf * SUB;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) wf[ks] = *(const bf16x8_t*)(wb + fr_off[ks]);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int t = 0; t < MT; ++t)
          acc[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[t][ks], wf[ks], acc[t][j], 0, 0, 0);
      buf = buf == NR - 1 ? 0 : buf + 1;
    }
  }

  // Add the four wavefronts' partial tiles: each writes its fragments (one 16-byte slot per lane), then
  // collects the four partials of the units it owns -- a unit is one fragment (one gate/up pair of
  // fragments for the SwiGLU epilogue), dealt out round-robin.  With a split reduction the sums go to
  // the workspace ([tile][split][unit slot][fragment of the unit][register pair][thread], 8 bytes per
  // thread and store, write-through); the workgroup that arrives last adds them in split order.
  // (Six row groups x eight fragments are 192 KB of partial tiles: they pass in two halves, row groups 0-2, then 3-5.)
  constexpr int PER = EPI == EPI_SWIGLU ? 2 : 1, UNITS = MT * NTW / PER, UPR = NTW / PER, NU = (UNITS + 3) / 4;
  constexpr int MTP = MT / PASSES, F = MTP * NTW;        // row groups and fragments per pass
  floatx4_t fin[NU][PER];
#pragma unroll
  for (int pass = 0; pass < PASSES; ++pass) {
    __syncthreads();
#pragma unroll
    for (int t = 0; t < MTP; ++t)
#pragma unroll
      for (int j = 0; j < NTW; ++j) *(floatx4_t*)(lds + (((wave * F + t * NTW + j) * 64 + lane) << 4)) = acc[pass * MTP + t][j];
    __syncthreads();
#pragma unroll
    for (int n = 0; n < NU; ++n) {
      const int unit = min(n * 4 + wave, UNITS - 1);     // (a surplus slot repeats the last unit and is never stored)
      const int t = unit / UPR, jj = unit - t * UPR;
      if (PASSES > 1 && t / MTP != pass) continue;
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        const int f = (t - pass * MTP) * NTW + jj * PER + e;
        floatx4_t sum = *(const floatx4_t*)(lds + (((0 * F + f) * 64 + lane) << 4));
#pragma unroll
        for (int w = 1; w < 4; ++w) sum += *(const floatx4_t*)(lds + (((w * F + f) * 64 + lane) << 4));
        fin[n][e] = sum;
      }
    }
  }
  if (SPLIT && n_split > 1) {
    const unsigned int tile = k * gridDim.x + blockIdx.x;
    constexpr int PART = NU * PER * 2 * 256;             // 8-byte words per partial tile
    uint64_t* part = (uint64_t*)a.ws + (size_t)tile * n_split * PART;
#pragma unroll
    for (int n = 0; n < NU; ++n)
#pragma unroll
      for (int e = 0; e < PER; ++e)
#pragma unroll
        for (int rp = 0; rp < 2; ++rp) {
          const uint64_t v = (uint64_t)__float_as_uint(fin[n][e][2 * rp]) | ((uint64_t)__float_as_uint(fin[n][e][2 * rp + 1]) << 32);
          store_agent(part + (size_t)split * PART + ((n * PER + e) * 2 + rp) * 256 + tid, v);
        }
    // (the ticket word lives in the dynamic LDS, which the sums above have left: this kernel has no static LDS to spare)
    if (!last_workgroup_of(&g_gemm_ticket[a.ticket_slot][tile], (unsigned int)n_split, (unsigned int*)lds)) return;
    // every load is a round trip to the memory side of the L2: all splits of a slot are requested together
    constexpr int SLOTS = NU * PER * 2;
#pragma unroll
    for (int sl = 0; sl < SLOTS; ++sl) {
      uint64_t v[8];
#pragma unroll
      for (int z = 0; z < 8; ++z)
        if (z < n_split) v[z] = load_agent(part + (size_t)z * PART + sl * 256 + tid);
      float lo = 0.f, hi = 0.f;
#pragma unroll
      for (int z = 0; z < 8; ++z)
        if (z < n_split) {
          lo += __uint_as_float((uint32_t)v[z]);
          hi += __uint_as_float((uint32_t)(v[z] >> 32));
        }
      fin[sl / (PER * 2)][(sl / 2) % PER][2 * (sl & 1)] = lo;
      fin[sl / (PER * 2)][(sl / 2) % PER][2 * (sl & 1) + 1] = hi;
    }
  }
#pragma unroll
  for (int n = 0; n < NU; ++n) {
    const int unit = n * 4 + wave;
    if (unit >= UNITS) break;
    const int t = unit / UPR, jj = unit - t * UPR;
    floatx4_t one[1][PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) one[0][e] = fin[n][e];
    finish_tile<1, PER, EPI, false>(a, one, k, m_tile, 0, 1, n0, m0, t, jj);
  }
}

// Which kernel a bf16 GEMM of M rows goes to, and in what shape.
//   M <= 2     wave-per-row GEMV (also three or four rows on a small matrix; not two rows of a long
//              reduction: see use_gemv).
//   M > 96     128 x 128 tiles (wavefronts 2 x 2, unsplit) or the large-tile kernel (gemm_big.hip)
//              with 128 or 192 x 256 tiles, whichever a small cost model prices lowest (below); if
//              none of them has enough tiles, as for fewer rows:
//   otherwise  a skinny arrangement: row blocks of 16*mt <= 128 activation rows.  Up to 96 rows per
//              block (mt <= 6): the ring kernel -- unsplit on tiles of 128, 96, 64 or 48 columns when
//              one of these widths gives 160 workgroups, else, with a workspace and a reduction long
//              enough, split over 2-8 workgroups per tile.  Everything else: the register-staged
//              kernels on 64-column tiles -- unsplit, the one whose wavefronts split the reduction;
//              with under 160 tiles and a workspace, the one whose wavefronts split the weight
//              rows, its reduction split over 2-8 workgroups (at M = 356 and 1040 the skinny
//              arrangement was up to 1.5x faster than 128 x 128 tiles below 200 of those and up to
//              1.6x slower above; splitting the 128 x 128 kernel's reduction never paid for its
//              64 KB partials).
// Workgroups along x of a ring kernel launch: the column tiles, or -- with several row blocks -- groups of
// 8 column tiles x row blocks (see the kernel), the last group padded.
// The wave-per-row GEMV stages its activation rows in LDS, M x d x 2 bytes per workgroup, and its
// wavefronts repeat every dot product for every row.  One or two rows: nothing streams the weights
// faster.  Three or four rows: the MFMA kernels win wherever the matrix is more than a few launch
// latencies long (us, four rows, GEMV against ring kernel: 32000 x 4096 50 / 44; 12288 x 4096 21.8 / 19.5;
// 4096 x 11008 30.7 / 20.7; 5120 x 13824 52 / 28; W1 and W2 of five heads at d = 5120, V = 32000:
// 293 / 279; but 1024 x 4096 9.9 / 10.9, 5120 x 5120 16.5 / 17.0).  Two rows of more than 8192
// elements (32 KB of staging): 5120 x 13824 33 / 28.
inline bool use_gemv(int M, int N, int d, int K) {
  if (M <= 1) return true;
  if (M == 2) return d <= 8192;
  return M <= 4 && (long)K * N * d <= ((long)8 << 20);
}
inline int ring_grid_x(int N, int ntw, int m_blocks) {
  const int cols = ceil_div(N, 16 * ntw);
  return m_blocks > 1 ? 8 * ceil_div(cols, 8) * m_blocks : cols;
}
struct GemmPlan {
  enum { GEMV, SKINNY, SQUARE, BIG } kind;
  bool wide;            // skinny: 128-column tiles; large tiles: 192 activation rows
  bool ring;            // skinny: the ring kernel (1 KB runs per weight row straight into an LDS ring)
  int ntw;              // skinny: column fragments (16 weight rows each) per workgroup
  int mt, m_blocks, ksplit;
};
GemmPlan plan_gemm(int M, int N, int d, int K, bool have_ws, bool wide_offsets) {
  GemmPlan p = {GemmPlan::GEMV, false, false, 8, 1, 1, 1};
  if (use_gemv(M, N, d, K)) return p;
  p.m_blocks = ceil_div(M, 128);
  if (M > 96) {
    // Three arrangements compete above 96 rows: 128 x 128 tiles (two workgroups share a CU) and
    // the large-tile kernel with 128 or 192 rows x 256 (one workgroup per CU).  What decides is
    // how evenly the tiles fill 256 CUs, so each candidate is priced with its measured time per
    // round of tiles (us at d = 4096, 7B shapes; the large tiles also wait for the weights'
    // first trip from HBM) and the cheapest one runs:
    //   128 x 128: 65 / 88 / 140 / 150 us for up to 1 / 2 / 3 / 4 tiles per CU, then 37.5 per tile,
    //              plus 0.3 x (weight bytes at 6 TB/s) per tile and CU;
    //   128 x 256: 68 per round of 256 tiles, 192 x 256: 88, plus 0.6 x (weight bytes at 6 TB/s).
    // 128 x 128 tiles need 200 of them, or a skinny launch that would exceed one workgroup per CU;
    // the large tiles need 120 (below that the skinny kernels win: M = 512, N = d = 4096 runs 42 us
    // skinny, 61 us large-tile).
    const double scale = d / 4096.0, w_us = (double)K * N * d * 2.0 / 6.0e6;
    const int mt_skinny = ceil_div(ceil_div(M, p.m_blocks), 16);
    const bool skinny_wide = mt_skinny <= 5 && (long)ceil_div(N, 128) * K * p.m_blocks >= 200;
    const long skinny_tiles = (long)ceil_div(N, skinny_wide ? 128 : 64) * K * p.m_blocks;
    const long sq_tiles = (long)ceil_div(N, 128) * p.m_blocks * K;
    double best = 1e30;
    int pick = GemmPlan::SKINNY;
    bool tall = false;
    int big_split = 1;
    if (sq_tiles >= 200 || skinny_tiles > 256) {
      const long n = (sq_tiles + 255) / 256;
      static const double t_sq[5] = {0., 65., 88., 140., 150.};
      best = (n <= 4 ? t_sq[n] : 37.5 * n) * scale + 0.3 * w_us * n;
      pick = GemmPlan::SQUARE;
    }
    if (!wide_offsets) {                                    // (the large-tile kernel addresses with 32-bit element offsets)
      for (int r = 128; r <= 192; r += 64) {
        const long tiles = (long)ceil_div(M, r) * ceil_div(N, 256) * K;
        if (tiles < 120) continue;
        // rounds: the busiest die decides (column tiles go round-robin over 8 dies of 32 CUs: 20 column
        // tiles x 12 row tiles are 240 tiles, yet 36 of them land on each of four dies)
        // (a last round of only a few workgroups runs a little faster than a full one: 0.8 + 0.2 x its fill; N = 5120,
        // M = 2048 on 192-row tiles puts 33 tiles on four of the dies and takes 1.9 rounds, M = 4160 with 66 takes 2.8)
        const long on_die = (long)ceil_div(ceil_div(N, 256), 8) * ceil_div(M, r) * K;
        const double die_rounds = on_die <= 32 ? 1.0 : (double)(on_die / 32) + (on_die % 32 ? 0.8 + 0.2 * (on_die % 32) / 32.0 : 0.0);
        const double rounds = die_rounds > (double)((tiles + 255) / 256) ? die_rounds : (double)((tiles + 255) / 256);
        // (rounds of 128-row tiles get dearer the more of them there are -- 70 us per round at two, 77 at three, 84 at
        // six, measured at N = 12288 -- while 192-row tiles hold 89-97: M = 4096, N = 12288 ran 507 us on 128-row tiles)
        const double per_round = r == 128 ? 68.0 + 3.0 * ((rounds < 7.0 ? rounds : 7.0) - 1.0) : 88.0;
        const double t = per_round * scale * rounds + 0.6 * w_us;
        // (from five rounds on the 128 x 128 price is the less certain one -- M = 2080, N = 11008 ran 301 us there
        // against 244 on 192-row tiles, priced 252 and 256 -- so it has to win by a twentieth)
        const double margin = pick == GemmPlan::SQUARE && sq_tiles > 4 * 256 ? 1.0 / 0.95 : 1.0;
        if (t < best * margin) { best = t; pick = GemmPlan::BIG; tall = r == 192; }
      }
      // A long reduction into few large tiles (the down projection of a batch of trees: M = 1040,
      // 11008 -> 4096 is 96 tiles of 192 x 256) can be split over 2 or 4 workgroups per tile when there
      // is a workspace.  Each split costs its partial tile (r KB) a write-through, a ticket and an
      // agent-scope read: about 5 us plus 0.3 us per MB of partial tiles (two splits) or 8 us plus 0.4 us per MB (four)
      // (M = 260..512, 11008 -> 4096 on 128-row tiles x 4 splits: 73-75 us measured, 73-76 priced; M = 161..260,
      // 13824 -> 5120: 83-86 measured, 88-92 priced; a 192-row tile split four ways runs as if its round took 110 us:
      // 105 us measured at M = 260, 11008 -> 4096).  A split plan has to beat the best unsplit one (the skinny
      // launch, where it fits one workgroup per CU, priced from a fit to its measured times; three or more
      // row blocks of it over a long reduction re-stream the weights and cost more: 11008 -> 4096 at M = 260..384 runs 81-97 us) by a
      // twentieth, and must fit one round on every
      // die: column tiles go round-robin over the 8 dies of 32 CUs each, rotated from split to split.  Measured on 8 weight shapes x
      // 10 row counts against the unsplit planning: 17 shapes 11-30 % faster (M = 1040, 11008 -> 4096:
      // 195 -> 145 us; M = 512: 100 -> 77; M = 420, 13824 -> 5120: 184 -> 134), none slower.
      if (have_ws && M > 128) {                             // (one row block: the skinny kernels are at their best)
        double unsplit = best;
        const double skinny_us = scale * (12.0 + 0.05 * M) * (N > 4096 ? N / 4096.0 : 1.0) * (p.m_blocks >= 3 && d > 6144 ? 1.15 : 1.0);   // (fit to M = 160..512 at 7B and 13B shapes)
        if (skinny_tiles <= 256 && skinny_us < unsplit) unsplit = skinny_us;
        double best_split = 0.95 * unsplit;
        for (int r = 128; r <= 192; r += 64)
          for (int sp = 2; sp <= 4; sp *= 2) {
            const long tiles = (long)ceil_div(M, r) * ceil_div(N, 256) * K;
            // workgroups on the busiest die: die x takes the column tiles c = x + 8/sp * s (mod 8) of split s
            const int n_col = ceil_div(N, 256);
            long per_die = 0;
            for (int x = 0; x < 8; ++x) {
              long cols = 0;
              for (int z = 0; z < sp; ++z) cols += n_col / 8 + (((x + 8 / sp * z) & 7) < n_col % 8 ? 1 : 0);
              per_die = cols > per_die ? cols : per_die;
            }
            per_die *= (long)ceil_div(M, r) * K;
            if (tiles < 32 || per_die > 32 || (d / 64) / sp < 16) continue;
            const double partial_mb = (double)tiles * sp * r * 1024.0 / 1.0e6;
            const double t = (r == 128 ? 68.0 : sp == 2 ? 88.0 : 110.0) * scale / sp + 0.6 * w_us + (sp == 2 ? 5.0 + 0.3 * partial_mb : 8.0 + 0.4 * partial_mb);
            if (t < best_split) { best_split = t; pick = GemmPlan::BIG; tall = r == 192; big_split = sp; }
          }
      }
    }
    if (pick == GemmPlan::BIG) {
      p.kind = GemmPlan::BIG;
      p.wide = tall;                                        // (for this kind: 192-row tiles)
      p.ksplit = big_split;
      return p;
    }
    if (pick == GemmPlan::SQUARE) {
      // wavefronts 2 x 2 (half the LDS reads per MFMA of the skinny arrangement), never split
      p.kind = GemmPlan::SQUARE;
      p.wide = true;
      p.mt = 4;
      return p;
    }
  }
  p.kind = GemmPlan::SKINNY;
  p.mt = ceil_div(ceil_div(M, p.m_blocks), 16);
  // More than 80 rows per block over a short reduction and a narrow output (the d x d projections):
  // rather than splitting the reduction of a few fat tiles, cut the rows into more blocks until
  // the unsplit launch has about one workgroup per CU; the blocks of a weight tile run side by side
  // and share its trip from HBM.  N = d = 4096 (us, one/two blocks against four): M = 128 23 -> 18,
  // M = 192 26 -> 21, M = 256 32 -> 24.5; N = d = 5120, M = 128: 38 -> 32.  Long reductions lose
  // (d = 11008, M = 128: 50 -> 54), fewer rows gain nothing (M = 64: 16 -> 15.4).
  if (p.mt >= 6 && d <= 6144) {
    const long per_block = (long)ceil_div(N, 64) * K;
    if (per_block * p.m_blocks < 160) {
      const int want = (int)((256 + per_block - 1) / per_block), most = ceil_div(M, 32);
      p.m_blocks = want < most ? want : most;
      p.mt = ceil_div(ceil_div(M, p.m_blocks), 16);
    }
  }
  p.wide = false;
  p.ntw = 4;                                                // (the register-staged kernels below: 64-column tiles)
  // The ring kernel takes up to 96 rows per block (six row groups leave the ring four buffers beside the 96 KB
  // slab, and the four partial tiles pass through LDS in two halves; still far ahead of everything else at
  // 81..96 rows -- the 89 tokens of the 13B tree: LM head 32000 x 5120 81 -> 64 us, 27648 x 5120 77 -> 59,
  // 15360 x 5120 45 -> 38 against 128 x 128 tiles or two blocks of 48 rows), or up to 192 rows as two blocks (the blocks of a
  // weight tile run side by side on one die and share its trip from HBM; with three or four blocks the
  // register-staged kernels below measured faster: N = 5120, d = 13824, M = 200 90 against 105 us).
  // Candidates, priced in units of one sub-stage (16 rows x 1 KB, roughly 0.6 us):
  //   unsplit, on tiles of 128, 96, 64 or 48 columns that give at least 160 workgroups: super-stages x
  //     rounds of 256 workgroups x (column fragments + the activation rows every workgroup fetches,
  //     which cost about a quarter of their bytes), + 2 for start and end;
  //   with a workspace, the reduction split over 2, 4 or 8 workgroups per tile of 128, 96 or 64 columns,
  //     at most one workgroup per CU in all: the longest share of super-stages x the same, + 5 for
  //     start, election and end, + the partial tiles the last workgroup fetches alone (splits x tile
  //     bytes, at what one CU can pull).  If the cheapest split leaves a workgroup under three
  //     super-stages the ring never fills (N = d = 4096: 21.5 us, 18.6 us below): no split candidate then.
  // Measured at M = 65 on MI355X: N = 12288, d = 4096 as 256 tiles of 48 columns 27.6 us (register-staged:
  // 35.7); N = 4096, d = 11008 as 64 columns x 4 splits 31 us, 128 x 8 40, 128 x 4 49 (register-staged
  // split: 34.5); at M = 97..160 the same matrix as 2 blocks x 64 columns x 2 splits 40-44 us (unsplit on
  // 48 columns 47-54, register-staged 41-55).  Against the register-staged kernels at M = 16..80 on 7B
  // and 13B projection shapes and the LM head: 7-30 % faster on weights from HBM, equal within 3 % on
  // weights the last-level cache holds.
  const int ring_blocks = p.mt <= 6 ? p.m_blocks : ceil_div(M, 80), ring_mt = ceil_div(ceil_div(M, ring_blocks), 16);
  if (ring_blocks <= 2 || p.mt <= 6) {
    const int n_super = (d + 511) / 512;
    const double per_stage = 0.25 * ring_mt;
    double best = 1e30;
    int ntw = 0, ks_best = 1;
    static const int widths[4] = {8, 6, 4, 3};
    for (int wi = 0; wi < 4; ++wi) {
      const long t = (long)ceil_div(N, 16 * widths[wi]) * K * ring_blocks;
      if (t < 160) continue;
      const double cost = (double)n_super * (double)((t + 255) / 256) * (widths[wi] + per_stage) + 2.0;
      if (cost < best) { best = cost; ntw = widths[wi]; ks_best = 1; }
    }
    if (have_ws) {
      double best_split = 1e30;
      int s_ntw = 0, s_ks = 0;
      for (int w = 8; w >= 4; w -= 2)
        for (int ks = 2; ks <= 8; ks *= 2) {
          const long t = (long)ceil_div(N, 16 * w) * K * ring_blocks;
          if (t * ks > 256 || ks > n_super) continue;
          const double cost = (double)ceil_div(n_super, ks) * (w + per_stage) + 5.0 + ks * ring_mt * w / 16.0;
          if (cost < best_split) { best_split = cost; s_ntw = w; s_ks = ks; }
        }
      if (s_ks > 1 && n_super / s_ks >= 3 && best_split < best) { best = best_split; ntw = s_ntw; ks_best = s_ks; }
    }
    if (ntw) {
      p.ring = true;
      p.ntw = ntw;
      p.wide = ntw == 8;
      p.ksplit = ks_best;
      p.m_blocks = ring_blocks;
      p.mt = ring_mt;
      return p;
    }
  }
  // Split the reduction only when the unsplit kernel would leave most of the chip idle (under 160
  // tiles): into the largest power of two of workgroups per tile that leaves each at least 16 steps
  // and the launch at most ~640 workgroups.  Measured at M = 65 (us, splits 1/2/4/8):
  // N = 4096, d = 4096: 25/24/18/19;  N = 4096, d = 11008: 67/54/36/35;  N = 5120, d = 13824: 83/65/57/54;
  // N = 11008, d = 4096: 32/37/36/45;  N = 13824, d = 5120: 41/48/53/63;  and with two or three row
  // blocks at N = d = 4096 (splits 1/2/4): M = 192 (128 tiles) 30/28/27, M = 260 (192 tiles) 31/38/42.
  const long tiles = (long)ceil_div(N, 64) * K * p.m_blocks;
  if (!have_ws || tiles >= 160) {
    // Unsplit.  With seven or eight row groups per workgroup the kernel runs out of registers for its
    // prefetch: one more row block then, if the launch stays within one workgroup per CU (M = 256,
    // N = d = 4096: 38 -> 31 us; N = 4096, d = 11008: 91 -> 75; but N = 11008, d = 4096: 78 -> 91).
    if (p.mt >= 7 && tiles / p.m_blocks * (p.m_blocks + 1) <= 256) {
      p.m_blocks += 1;
      p.mt = ceil_div(ceil_div(M, p.m_blocks), 16);
    }
    return p;
  }
  long cap = 640 / tiles;
  const long by_steps = (d / 64) / 16;
  cap = cap < by_steps ? cap : by_steps;
  while (p.ksplit * 2 <= cap && p.ksplit < 8) p.ksplit *= 2;
  return p;
}
// Workspace for the fp32 partial tiles of a split reduction (0 if this shape is not split).
size_t gemm_ws_bytes(int M, int N, int d, int K) {
  const GemmPlan p = plan_gemm(M, N, d, K, true, false);
  if (p.kind == GemmPlan::BIG && p.ksplit > 1) {            // partial tiles of the large-tile kernel: rows x 256 floats each
    const int rows = p.wide ? 192 : 128;
    return (size_t)8 * ceil_div(ceil_div(N, 256), 8) * ceil_div(M, rows) * K * p.ksplit * rows * 256 * sizeof(float);
  }
  if (p.kind != GemmPlan::SKINNY || p.ksplit <= 1) return 0;
  if (p.ring)                                               // per workgroup: ceil(mt*ntw/4) fragments per thread
    return (size_t)ring_grid_x(N, p.ntw, p.m_blocks) * K * p.ksplit * ceil_div(p.mt * p.ntw, 4) * 4 * 256 * sizeof(float);
  return (size_t)ceil_div(N, 64) * K * p.m_blocks * p.ksplit * p.mt * 4 * 256 * sizeof(float);   // mt accumulator fragments per thread
}

// Weight rows per GEMV workgroup: 16 measured best on MI355X at 7B shapes (8, 32 and 64 were
// 1-10 % slower); fewer for small matrices so that the grid still covers the chip.
int gemv_rows_per_wg(int N, int K, int M) {
  // (three or four activation rows cost a workgroup 30-40 KB of LDS staging: twice the weight rows
  // per workgroup then, if that still leaves the chip 500 workgroups: 62 -> 59 us at d = 5120, V = 32000)
  // (the kernel for three or four rows has eight wavefronts, each on two weight rows at a time)
  // (... and the grid is large: the residual blocks of four heads, 16-20 thousand weight rows, run 5-10 % faster with 16)
  if (M >= 3) return (long)N * K >= 65536 ? 32 : 16;
  long rows = ((long)N * K / 1024) & ~7L;
  return rows < 8 ? 8 : (rows > 16 ? 16 : (int)rows);
}

// Register stages of the skinny kernel: three while its MT + NTW chunks per thread and stage leave room.
constexpr int skinny_depth(int mt, int ntw) { return mt + ntw <= 13 ? 3 : 2; }
// Weight buffers of the ring kernel: what 160 KB of LDS hold beside the activation slab, at most 8.
constexpr int ring_depth(int mt) { return mt >= 6 ? 4 : mt == 5 ? 5 : (10 - mt > 8 ? 8 : 10 - mt); }

// The skinny kernels' LDS tiles exceed the 64 KB a kernel gets by default (the ring kernel takes all
// 160 KB of a CU): raise the limit once per kernel and device.
template <void (*Kernel)(GemmArgs)>
int launch_skinny(dim3 grid, size_t lds, hipStream_t stream, const GemmArgs& a) {
  static std::atomic<bool> raised[64];   // (set after the call succeeded; two threads racing here both make the same call)
  int dev = 0;
  MEDUSA_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return MEDUSA_EUNSUPPORTED;
  if (!raised[dev].load(std::memory_order_acquire)) {
    MEDUSA_HIP_TRY(hipFuncSetAttribute((const void*)Kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));   // the largest tile of these kernels
    raised[dev].store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL(Kernel, grid, dim3(256), lds, stream, a);
  return MEDUSA_OK;
}

template <int EPI>
int launch_gemm(const GemmArgs& a_in, int dtype, hipStream_t stream) {
  GemmArgs a = a_in;
  a.ksplit = 1;
  a.ticket_slot = ticket_slot(stream);
  a.rows_per_wg = gemv_rows_per_wg(a.N, a.K, dtype == MEDUSA_BF16 ? a.M : 1);
  const int kGemvRowsPerWg = a.rows_per_wg;
  const dim3 block(256);
  if (dtype == MEDUSA_F32) {
    // activations of one m-block live in LDS: keep it within 64 KB
    if ((size_t)a.d * sizeof(float) > 65536) return MEDUSA_EUNSUPPORTED;   // one activation row must fit the 64 KB staging
    const int MB = (size_t)4 * a.d * sizeof(float) <= 65536 ? 4 : 1;
    const dim3 grid(ceil_div(a.N, kGemvRowsPerWg), a.K, ceil_div(a.M, MB));
    const size_t lds = (size_t)MB * a.d * sizeof(float);
    if (MB == 4) hipLaunchKernelGGL((gemv_f32_kernel<4, EPI>), grid, block, lds, stream, a);
    else hipLaunchKernelGGL((gemv_f32_kernel<1, EPI>), grid, block, lds, stream, a);
  } else if (use_gemv(a.M, a.N, a.d, a.K)) {
    int MB = a.M <= 1 ? 1 : (a.M <= 2 ? 2 : 4);
    if ((size_t)a.d * sizeof(uint16_t) > 65536) return MEDUSA_EUNSUPPORTED;   // one activation row must fit the 64 KB staging
    while ((size_t)MB * a.d * sizeof(uint16_t) > 65536) MB >>= 1;   // activations of one m-block live in LDS
    const dim3 grid(ceil_div(a.N, kGemvRowsPerWg), a.K, ceil_div(a.M, MB));
    const size_t lds = (size_t)MB * a.d * sizeof(uint16_t);
    if (MB == 1) hipLaunchKernelGGL((gemv_bf16_kernel<1, EPI>), grid, block, lds, stream, a);
    else if (MB == 2) hipLaunchKernelGGL((gemv_bf16_kernel<2, EPI>), grid, block, lds, stream, a);
    else hipLaunchKernelGGL((gemv_bf16_kernel<4, EPI>), grid, dim3(512), lds, stream, a);
  } else {
    const bool wide_offsets = (size_t)a.N * a.d >= ((size_t)1 << 31) || x_extent(a) >= ((size_t)1 << 31);
    const GemmPlan plan = plan_gemm(a.M, a.N, a.d, a.K, a.ws != nullptr, wide_offsets);
    if (plan.kind == GemmPlan::BIG) {
      a.ksplit = plan.ksplit;
      return launch_gemm_big(a, EPI, plan.wide, stream);
    }
    a.ksplit = plan.ksplit;
    // split reductions exist for the epilogues tree_linear uses (medusa_heads passes no workspace)
    constexpr bool kCanSplit = EPI == EPI_PLAIN || EPI == EPI_GATED;
    const bool split = kCanSplit && a.ksplit > 1;
    if (!split) a.ksplit = 1;
    a.m_blocks = plan.m_blocks;
    const dim3 grid = plan.kind == GemmPlan::SKINNY && plan.ring
                          ? dim3(ring_grid_x(a.N, plan.ntw, plan.m_blocks), a.K, a.ksplit)
                          : dim3(ceil_div(a.N, plan.kind == GemmPlan::SKINNY ? 16 * plan.ntw : 128), a.K, plan.m_blocks * a.ksplit);
    // (every output tile of a split launch has a ticket counter: the planning stays far below their number)
    if (split && (long)grid.x * grid.y * (plan.ring ? 1 : plan.m_blocks) > kMaxSplitTiles) return MEDUSA_EUNSUPPORTED;
    if (plan.kind == GemmPlan::SQUARE) {
      hipLaunchKernelGGL((gemm_lds_bf16_kernel<2, 2, 4, 4, 64, 2, EPI, false>), grid, block, 0, stream, a);
      MEDUSA_LAUNCH_CHECK();
      return MEDUSA_OK;
    }
    // A split reduction leaves each workgroup only a few steps: there the kernel whose wavefronts split
    // the weight rows is faster (no sum over the wavefronts at the end; 21 against 24 us at M = 65,
    // N = d = 4096).  Unsplit, LDS time decides and the kernel whose wavefronts split the reduction wins.
#define MEDUSA_SKINNY(MT_)                                                                                                     \
  case MT_:                                                                                                                    \
    if (split && plan.ring) {                                                                                                  \
      constexpr int MR = MT_ <= 6 ? MT_ : 6, NR = ring_depth(MR);                                                        \
      const size_t ring_lds = (size_t)(NR + MR) * 16384;                                                                       \
      if (plan.ntw == 8) rc = launch_skinny<gemm_ring_bf16_kernel<MR, 8, NR, EPI, kCanSplit>>(grid, ring_lds, stream, a);      \
      else if (plan.ntw == 6) rc = launch_skinny<gemm_ring_bf16_kernel<MR, 6, NR, EPI, kCanSplit>>(grid, ring_lds, stream, a); \
      else rc = launch_skinny<gemm_ring_bf16_kernel<MR, 4, NR, EPI, kCanSplit>>(grid, ring_lds, stream, a);                    \
    } else if (split) {                                                                                                        \
      hipLaunchKernelGGL((gemm_lds_bf16_kernel<1, 4, MT_, 1, 64, 4, EPI, kCanSplit>), grid, block, 0, stream, a);              \
    } else if (plan.ring) {                                                                                                    \
      constexpr int MR = MT_ <= 6 ? MT_ : 6, NR = ring_depth(MR);                                                              \
      const size_t ring_lds = (size_t)(NR + MR) * 16384;                                                                       \
      if (plan.ntw == 8) rc = launch_skinny<gemm_ring_bf16_kernel<MR, 8, NR, EPI>>(grid, ring_lds, stream, a);                 \
      else if (plan.ntw == 6) rc = launch_skinny<gemm_ring_bf16_kernel<MR, 6, NR, EPI>>(grid, ring_lds, stream, a);            \
      else if (plan.ntw == 4) rc = launch_skinny<gemm_ring_bf16_kernel<MR, 4, NR, EPI>>(grid, ring_lds, stream, a);            \
      else rc = launch_skinny<gemm_ring_bf16_kernel<MR, 3, NR, EPI>>(grid, ring_lds, stream, a);                               \
    } else {                                                                                                                   \
      rc = launch_skinny<gemm_skinny_bf16_kernel<MT_, 4, skinny_depth(MT_, 4), EPI>>(grid, lds, stream, a);                    \
    }                                                                                                                          \
    break;
    const size_t lds = (size_t)2 * (plan.mt + 4) * 4096;
    int rc = MEDUSA_OK;
    switch (plan.mt) {
      MEDUSA_SKINNY(1) MEDUSA_SKINNY(2) MEDUSA_SKINNY(3) MEDUSA_SKINNY(4) MEDUSA_SKINNY(5) MEDUSA_SKINNY(6)
      MEDUSA_SKINNY(7) MEDUSA_SKINNY(8)
      default: return MEDUSA_EUNSUPPORTED;                  // (no plan asks for more than 128 rows per block)
    }
#undef MEDUSA_SKINNY
    if (rc != MEDUSA_OK) return rc;
  }
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}

}  // namespace

// medusa_heads; `ev` is null, or three events recorded before the residual-block kernel, between
// the two kernels and after the vocabulary projection.
static int heads_impl(const void* hidden, const void* w1, const void* w2, void* resid, float* logits, int M, int d, int V,
                      int K, int dtype, medusa_stream_t stream_, hipEvent_t* ev) {
  if (!hidden || !w2 || !logits || (w1 && !resid)) return MEDUSA_EINVAL;
  if (M < 1 || d < 1 || V < 1 || K < 1) return MEDUSA_EINVAL;
  if (dtype != MEDUSA_F32 && dtype != MEDUSA_BF16) return MEDUSA_EINVAL;
  if (M > kMaxRows || K > MEDUSA_MAX_HEADS || d > 16384) return MEDUSA_EUNSUPPORTED;
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
    if (ev) MEDUSA_HIP_TRY(hipEventRecord(ev[0], stream));
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
  if (ev) {
    if (!w1) MEDUSA_HIP_TRY(hipEventRecord(ev[0], stream));
    MEDUSA_HIP_TRY(hipEventRecord(ev[1], stream));
  }
  const int rc = launch_gemm<EPI_LOGITS>(a, dtype, stream);
  if (ev && rc == MEDUSA_OK) MEDUSA_HIP_TRY(hipEventRecord(ev[2], stream));
  return rc;
}

extern "C" int medusa_heads(const void* hidden, const void* w1, const void* w2, void* resid, float* logits, int M,
                            int d, int V, int K, int dtype, medusa_stream_t stream_) {
  return heads_impl(hidden, w1, w2, resid, logits, M, d, V, K, dtype, stream_, nullptr);
}

extern "C" int medusa_heads_timed(const void* hidden, const void* w1, const void* w2, void* resid, float* logits, int M,
                                  int d, int V, int K, int dtype, medusa_stream_t stream_, void* ev_begin,
                                  void* ev_between, void* ev_end) {
  if (!ev_begin || !ev_between || !ev_end) return MEDUSA_EINVAL;
  hipEvent_t ev[3] = {(hipEvent_t)ev_begin, (hipEvent_t)ev_between, (hipEvent_t)ev_end};
  return heads_impl(hidden, w1, w2, resid, logits, M, d, V, K, dtype, stream_, ev);
}

// The original model's logits at the tree tokens with the acceptance step's row reductions taken in the
// GEMM epilogue (Sec. 2.3.1 needs, per row, the arg-max and -- for typical acceptance -- the soft-max
// statistics; taken from the tile they cost no second pass over the B*T*V logits).
extern "C" size_t medusa_verify_stats_bytes(int M, int V) {
  if (M < 1 || V < 1) return 0;
  const size_t parts = 2 * (size_t)ceil_div(V, 256);
  return sizeof(FusedStatsHeader) + (size_t)M * kFusedMergedSlots * sizeof(RowPart) + (size_t)M * parts * sizeof(RowPart);
}

extern "C" int medusa_verify_fused_available(int M, int d, int V, int dtype) {
  if (M < 1 || d < 1 || V < 1 || dtype != MEDUSA_BF16 || d % 64 != 0 || M > 4096 || d > 16384) return 0;
  const bool wide_offsets = (size_t)V * d >= ((size_t)1 << 31) || (size_t)M * d + (size_t)2 * d >= ((size_t)1 << 31);
  return plan_gemm(M, V, d, 1, false, wide_offsets).kind == GemmPlan::BIG ? 1 : 0;
}

extern "C" int medusa_verify_logits(const void* hidden_tree, const void* w_lm, float* logits, void* stats, size_t stats_bytes,
                                    int M, int d, int V, int dtype, int mode, float temperature, medusa_stream_t stream_) {
  if (!hidden_tree || !w_lm || !logits || !stats) return MEDUSA_EINVAL;
  if (M < 1 || d < 1 || V < 1) return MEDUSA_EINVAL;
  if (dtype != MEDUSA_F32 && dtype != MEDUSA_BF16) return MEDUSA_EINVAL;
  if (mode != MEDUSA_GREEDY && mode != MEDUSA_TYPICAL) return MEDUSA_EINVAL;
  if (mode == MEDUSA_TYPICAL && !(temperature > 0.f)) return MEDUSA_EINVAL;
  if (!medusa_verify_fused_available(M, d, V, dtype)) return MEDUSA_EUNSUPPORTED;
  if (stats_bytes < medusa_verify_stats_bytes(M, V) || ((uintptr_t)stats & 255) != 0) return MEDUSA_EWORKSPACE;
  GemmArgs a = {};
  a.d = d;
  a.M = M;
  a.K = 1;
  a.hidden = hidden_tree;
  a.X = hidden_tree;
  a.xs_m = d;
  a.W = w_lm;
  a.out = logits;
  a.N = V;
  a.stats = (RowPart*)((unsigned char*)stats + sizeof(FusedStatsHeader) + (size_t)M * kFusedMergedSlots * sizeof(RowPart));
  a.stats_parts = 2 * ceil_div(V, 256);
  a.stats_k2 = mode == MEDUSA_TYPICAL ? 1.4426950408889634f / temperature : 0.f;
  return launch_gemm<EPI_LOGITS>(a, (medusa_dtype_t)dtype, (hipStream_t)stream_);
}

// Backbone linear layer on the tree tokens (App. G, operator table, parallel-decoding rows).
extern "C" size_t tree_linear_workspace_bytes(int B, int T, int d_in, int d_out, int dtype) {
  if (dtype != MEDUSA_BF16 || B < 1 || T < 1 || d_in < 64 || d_out < 1) return 0;
  return gemm_ws_bytes(B * T, d_out, d_in, 1);
}

extern "C" int tree_linear(const void* x, const void* w, const void* mul, void* y, int B, int T, int d_in, int d_out,
                           int x_heads, int y_heads, int dtype, void* workspace, size_t workspace_bytes,
                           medusa_stream_t stream_) {
  return tree_linear_segments(x, w, mul, y, B, T, d_in, d_out, x_heads, y_heads, 1, 0, dtype, workspace, workspace_bytes, stream_);
}

extern "C" int tree_linear_segments(const void* x, const void* w, const void* mul, void* y, int B, int T, int d_in, int d_out,
                                    int x_heads, int y_heads, int y_segments, size_t y_segment_stride, int dtype,
                                    void* workspace, size_t workspace_bytes, medusa_stream_t stream_) {
  if (!x || !w || !y) return MEDUSA_EINVAL;
  if (B < 1 || T < 1 || d_in < 1 || d_out < 1 || x_heads < 0 || y_heads < 0 || y_segments < 1) return MEDUSA_EINVAL;
  if (y_segments > 1) {
    // several head-major tensors: whole heads per segment, segments that do not overlap
    if (y_heads < 1 || d_out % y_segments != 0 || (d_out / y_segments) % y_heads != 0) return MEDUSA_EINVAL;
    if (y_segment_stride < (size_t)B * T * (d_out / y_segments) || y_segment_stride > ((size_t)1 << 40)) return MEDUSA_EINVAL;
    d_out /= y_segments;                                  // (per segment, for the layout arithmetic below)
  }
  if (dtype != MEDUSA_F32 && dtype != MEDUSA_BF16) return MEDUSA_EINVAL;
  const long M = (long)B * T;
  if (M > kMaxRows || d_in > 65536) return MEDUSA_EUNSUPPORTED;
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
  a.N = d_out * y_segments;
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
    if (y_segments > 1) {
      a.y_seg_heads = y_heads;
      a.y_seg_stride = (long)y_segment_stride;
    }
  }
  // the split reduction is an optimisation: without (enough) workspace the call runs unsplit
  if (workspace && dtype == MEDUSA_BF16 && workspace_bytes >= gemm_ws_bytes(a.M, a.N, a.d, 1) && gemm_ws_bytes(a.M, a.N, a.d, 1) > 0)
    a.ws = workspace;
  hipStream_t stream = (hipStream_t)stream_;
  return mul ? launch_gemm<EPI_GATED>(a, dtype, stream) : launch_gemm<EPI_PLAIN>(a, dtype, stream);
}

// Gate and up projections of the gated feed-forward in one pass over both weight matrices (App. G,
// operator table: X W_g and X W_u; the product SiLU(X W_g) * (X W_u) is what X W_d consumes).
extern "C" int tree_linear_swiglu(const void* x, const void* w_gu, void* y, int B, int T, int d_in, int d_out, int x_heads,
                                  int y_heads, int dtype, medusa_stream_t stream_) {
  if (!x || !w_gu || !y) return MEDUSA_EINVAL;
  if (B < 1 || T < 1 || d_in < 1 || d_out < 1 || x_heads < 0 || y_heads < 0) return MEDUSA_EINVAL;
  if (dtype != MEDUSA_F32 && dtype != MEDUSA_BF16) return MEDUSA_EINVAL;
  if (dtype != MEDUSA_BF16) return MEDUSA_EUNSUPPORTED;            // (fp32 callers use two tree_linear calls)
  const long M = (long)B * T;
  if (M > kMaxRows || d_in > 65536 || d_out > (1 << 24)) return MEDUSA_EUNSUPPORTED;
  if (d_in % 64 != 0 || d_out % 16 != 0) return MEDUSA_EUNSUPPORTED;
  if (x_heads > 0 && (d_in % x_heads != 0 || (d_in / x_heads) % 64 != 0)) return MEDUSA_EUNSUPPORTED;
  if (y_heads > 0 && d_out % y_heads != 0) return MEDUSA_EINVAL;
  GemmArgs a = {};
  a.W = w_gu;
  a.X = x;
  a.out = y;
  a.M = (int)M;
  a.N = 2 * d_out;
  a.d = d_in;
  a.K = 1;
  a.xs_m = d_in;
  a.ksplit = 1;
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
  hipStream_t stream = (hipStream_t)stream_;
  // Many rows (a batch of trees): the large-tile kernel, if the planning gives it this shape
  if (a.M > 96) {
    const bool wide_offsets = (size_t)a.N * a.d >= ((size_t)1 << 31) || x_extent(a) >= ((size_t)1 << 31);
    const GemmPlan plan = plan_gemm(a.M, a.N, a.d, 1, false, wide_offsets);
    if (plan.kind == GemmPlan::BIG) return launch_gemm_big(a, EPI_SWIGLU, plan.wide, stream);
  }
  // 128-column tiles (gate and up fragments of a column block side by side in a wavefront), row blocks
  // of at most 96 rows, never split: tuned for the tree-token range, correct for any M
  const int m_blocks = ceil_div(a.M, 96), mt = ceil_div(ceil_div(a.M, m_blocks), 16);
  // the ring kernel, with the tile width (whole gate/up pairs) priced as in plan_gemm
  int ntw = 8;
  {
    double best = 1e30;
    for (int w = 8; w >= 2; w -= 2) {
      const long t = (long)ceil_div(a.N, 16 * w) * m_blocks;
      const double cost = (double)((t + 255) / 256) * (w + 0.25 * mt + 1.0);
      if ((t >= 160 || w == 8) && cost < best) { best = cost; ntw = w; }
    }
  }
  a.m_blocks = m_blocks;
  const dim3 grid(ring_grid_x(a.N, ntw, m_blocks), 1, 1);
  int rc = MEDUSA_OK;
#define MEDUSA_SWIGLU(MT_)                                                                                                \
  case MT_: {                                                                                                             \
    constexpr int NR = ring_depth(MT_);                                                                                   \
    const size_t ring_lds = (size_t)(NR + MT_) * 16384;                                                                   \
    if (ntw == 8) rc = launch_skinny<gemm_ring_bf16_kernel<MT_, 8, NR, EPI_SWIGLU>>(grid, ring_lds, stream, a);           \
    else if (ntw == 6) rc = launch_skinny<gemm_ring_bf16_kernel<MT_, 6, NR, EPI_SWIGLU>>(grid, ring_lds, stream, a);      \
    else if (ntw == 4) rc = launch_skinny<gemm_ring_bf16_kernel<MT_, 4, NR, EPI_SWIGLU>>(grid, ring_lds, stream, a);      \
    else rc = launch_skinny<gemm_ring_bf16_kernel<MT_, 2, NR, EPI_SWIGLU>>(grid, ring_lds, stream, a);                    \
  } break;
  switch (mt) { MEDUSA_SWIGLU(1) MEDUSA_SWIGLU(2) MEDUSA_SWIGLU(3) MEDUSA_SWIGLU(4) MEDUSA_SWIGLU(5) MEDUSA_SWIGLU(6) default: return MEDUSA_EUNSUPPORTED; }
#undef MEDUSA_SWIGLU
  if (rc != MEDUSA_OK) return rc;
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}

extern "C" int medusa_gemm_plan(int M, int N, int d, int K, int have_workspace, int* plan6) {
  if (!plan6 || M < 1 || N < 1 || d < 1 || K < 1) return MEDUSA_EINVAL;
  const bool wide_offsets = (size_t)N * d >= ((size_t)1 << 31) || (size_t)M * d + (size_t)K * d + d >= ((size_t)1 << 31);
  const GemmPlan p = plan_gemm(M, N, d, K, have_workspace != 0, wide_offsets);
  plan6[0] = (int)p.kind; plan6[1] = p.kind == GemmPlan::SKINNY ? 16 * p.ntw : (p.kind == GemmPlan::BIG ? (p.wide ? 192 : 128) : 0); plan6[2] = p.ring; plan6[3] = p.mt; plan6[4] = p.m_blocks; plan6[5] = p.ksplit;
  return MEDUSA_OK;
}



