// Large-M bf16 GEMM of medusa_heads (Sec. 2.1.1): the vocabulary projection of every tree token
// of a batch (M = batch x tree tokens, several hundred to a few thousand rows).  At these sizes
// the contraction is MFMA-bound, so the kernel is built around keeping the matrix pipe issuing:
//
//   * Tile (32 MT) x 256 outputs per workgroup of 4 wavefronts (2 x 2), each wavefront
//     (16 MT) x 128 with all accumulators in registers; one workgroup per CU.  Against a 64 x 64
//     wavefront tile this halves the LDS bytes read per MFMA.
//   * Two LDS stages of 64 reduction elements.  Rows are 128 bytes, unpadded; the 16-byte chunk c of
//     row r is stored at chunk slot c ^ ((r >> 1) & 7), which makes both the row-major stores and the
//     fragment reads (16 rows x 4 chunks per instruction) bank-conflict free.
//   * One register stage of global loads in front of LDS: the data of stage i+2 is requested in the
//     second half of stage i and written to LDS in the first half of stage i+1.
//   * One barrier per stage, between the two 32-element halves of the stage:
//       first half : fragment reads of half 1 | MFMAs of half 0 | registers of stage i+1 -> LDS
//       barrier
//       second half: global loads of stage i+2 | fragment reads of half 0 of stage i+1 | MFMAs of half 1
//     LDS and global instructions are spread between the MFMAs and the last LDS store is followed
//     by a few MFMAs, so its latency is covered when the barrier comes.
//   * Workgroups are numbered so that the m-tiles of one weight tile run on the same XCD (dispatch
//     is round-robin over the 8 XCDs) next to each other in time: the weight tile comes from HBM once.
//
// This file is compiled with MFMA results kept in ordinary vector registers (see build.py); with the
// compiler's default choice the accumulators are copied between the two register files in every
// iteration (several hundred moves per 96 MFMAs).
#include "gemm_args.hpp"

namespace {

template <int MT, int NT, int EPI>
__global__ __launch_bounds__(256, 1) void gemm_big_bf16_kernel(GemmArgs a, int m_tiles, int n_tiles) {
  constexpr int BM = 32 * MT, BN = 32 * NT, ROWS = BM + BN;
  constexpr int LPT = ROWS / 32;                      // 16-byte chunks per thread and stage
  constexpr int STAGE = ROWS * 128;
  constexpr int NMF = MT * NT;                        // MFMAs per half stage
  constexpr int NRD = MT + NT;                        // fragment reads per half stage
  static_assert(LPT * 4096 <= 65536, "LDS store offsets must fit the instruction's immediate");
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * STAGE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, q4 = lane >> 4;
  const int wm = wave >> 1, wn = wave & 1;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int nt_local = slot / m_tiles;
  const int n_tile = nt_local * 8 + xcd;
  if (n_tile >= n_tiles) return;                      // whole workgroup leaves before any barrier
  const int m0 = (slot - nt_local * m_tiles) * BM, n0 = n_tile * BN;
  const int k = blockIdx.y;
  const unsigned char* Xb = (const unsigned char*)a.X + (size_t)k * a.xs_k * 2;
  const unsigned char* Wb = (const unsigned char*)a.W + (size_t)k * a.N * a.d * 2;

  // Chunk `it` of a thread: tile row it*32 + tid/8 (activation rows first, then weight rows), 16-byte
  // chunk tid%8.  Rows past the matrix edge are clamped (loaded twice, never stored).
  uint32_t goff[LPT];
#pragma unroll
  for (int it = 0; it < LPT; ++it) {
    const int row = it * 32 + (tid >> 3), c = tid & 7;
    goff[it] = it < MT ? (uint32_t)(((size_t)min(m0 + row, a.M - 1) * a.xs_m + c * 8) * 2)
                       : (uint32_t)(((size_t)min(n0 + row - BM, a.N - 1) * a.d + c * 8) * 2);
  }
  const int nk = a.d >> 6;
  u32x4_t G[LPT];
  auto gload = [&](int step, u32x4_t (&g)[LPT]) __attribute__((always_inline)) {
    const uint32_t so = (uint32_t)min(step, nk - 1) * 128u;      // past the end: harmless reload
#pragma unroll
    for (int it = 0; it < LPT; ++it) g[it] = *(const u32x4_t*)((it < MT ? Xb : Wb) + (goff[it] + so));
  };
  const int st_off = (tid >> 3) * 128 + (((tid & 7) ^ ((tid >> 4) & 7)) << 4);
  auto lstore = [&](int buf, const u32x4_t (&g)[LPT]) __attribute__((always_inline)) {
    unsigned char* b = lds + buf * STAGE + st_off;
#pragma unroll
    for (int it = 0; it < LPT; ++it) *(u32x4_t*)(b + it * 4096) = g[it];
  };
  const int swz = (i16 >> 1) & 7;
  const int x_row = (wm * MT * 16 + i16) * 128, w_row = (BM + wn * NT * 16 + i16) * 128;
  auto lfrag = [&](int buf, int half, bf16x8_t (&xf)[MT], bf16x8_t (&wf)[NT]) __attribute__((always_inline)) {
    const unsigned char* b = lds + buf * STAGE + (((half * 4 + q4) ^ swz) << 4);
#pragma unroll
    for (int t = 0; t < MT; ++t) xf[t] = *(const bf16x8_t*)(b + x_row + t * 2048);
#pragma unroll
    for (int j = 0; j < NT; ++j) wf[j] = *(const bf16x8_t*)(b + w_row + j * 2048);
  };
  floatx4_t acc[MT][NT];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[t][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  auto mfma = [&](const bf16x8_t (&xf)[MT], const bf16x8_t (&wf)[NT]) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[t], wf[j], acc[t][j], 0, 0, 0);
  };

  // Instruction order within a half stage, given to the scheduler as groups.  An LDS store of a
  // wavefront keeps the LDS busy for 8 clocks (a read for 4) and the four wavefronts store at the
  // same time, so stores are issued no closer than every second MFMA (32 clocks); closer, the LDS
  // queue fills and the wavefront -- and with it the matrix pipe -- stalls.  First half: fragment
  // reads (RPS per MFMA), then the stores, then MFMAs only, whose tail covers the latency of the
  // last store before the barrier.  Second half: global loads first (they have the longest way to
  // go), then the fragment reads.  Masks: 0x008 MFMA, 0x020 global load, 0x100 LDS read, 0x200 LDS store.
  constexpr int RPS = NMF >= NRD + 2 * LPT + 2 ? 1 : 2;
  static_assert(NMF >= NRD / RPS + 2 * LPT + 2 && NRD % RPS == 0, "not enough MFMAs to spread the memory instructions over");
  bf16x8_t xf0[MT], wf0[NT], xf1[MT], wf1[NT];
  gload(0, G);
  lstore(0, G);
  gload(1, G);
  __syncthreads();
  lfrag(0, 0, xf0, wf0);
  for (int i = 0; i < nk; ++i) {
    // On entry: LDS buffer i&1 holds stage i, (xf0, wf0) its first-half fragments and G the data of
    // stage i+1 (possibly still in flight).
    const int cur = i & 1;
    lfrag(cur, 1, xf1, wf1);
    mfma(xf0, wf0);
    lstore(cur ^ 1, G);
#pragma unroll
    for (int g = 0; g < NRD / RPS; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x100, RPS, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
#pragma unroll
    for (int g = 0; g < LPT; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, NMF, 0);
    __syncthreads();
    gload(i + 2, G);
    lfrag(cur ^ 1, 0, xf0, wf0);
    mfma(xf1, wf1);
#pragma unroll
    for (int g = 0; g < LPT; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
#pragma unroll
    for (int g = 0; g < NRD; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, NMF, 0);
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

template <int EPI>
int launch(const GemmArgs& a, hipStream_t stream) {
  // 192 x 256 or 128 x 256 tile, whichever pads M less (ties to the larger)
  const int n_tiles = ceil_div(a.N, 256);
  const bool tall = ceil_div(a.M, 192) * 192 <= ceil_div(a.M, 128) * 128;
  const int m_tiles = ceil_div(a.M, tall ? 192 : 128);
  const dim3 grid(8 * ceil_div(n_tiles, 8) * m_tiles, a.K), block(256);
  if (tall) hipLaunchKernelGGL((gemm_big_bf16_kernel<6, 8, EPI>), grid, block, 0, stream, a, m_tiles, n_tiles);
  else hipLaunchKernelGGL((gemm_big_bf16_kernel<4, 8, EPI>), grid, block, 0, stream, a, m_tiles, n_tiles);
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}

}  // namespace

int launch_gemm_big(const GemmArgs& a, int epi, hipStream_t stream) {
  if (a.d % 64 != 0 || a.d < 64) return MEDUSA_EUNSUPPORTED;
  if ((size_t)a.N * a.d >= ((size_t)1 << 31) || (size_t)a.M * a.xs_m >= ((size_t)1 << 31)) return MEDUSA_EUNSUPPORTED;
  return epi == EPI_LOGITS ? launch<EPI_LOGITS>(a, stream) : launch<EPI_RESID>(a, stream);
}
