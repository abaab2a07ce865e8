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

// SiLU from the hardware's exp2 and reciprocal instructions (about 1e-6 relative error; the result
// is rounded to bf16, 4e-3, right after).  The library expf is a function call here, and a call with
// the whole accumulator tile live spills it.
__device__ __forceinline__ float silu_fast(float u) {
  return u * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * u));
}

// Ticket counters of the split reduction (one per output tile and head), per stream slot; zero between launches.
constexpr int kMaxBigSplitTiles = 4096;
__device__ unsigned int g_big_ticket[kTicketSlots][kMaxBigSplitTiles];

// SPLIT: grid.z workgroups share an output tile, each reducing a contiguous 1/grid.z of d; they park
// their fp32 partial tiles in the workspace and the one that finishes last adds them up in split
// order (so the result does not depend on which one that is) and runs the epilogue.  For long
// reductions into few tiles (the down projection of a batch of trees): 96 tiles of 192 x 256 over
// d = 11008 keep 96 CUs busy for 240 us unsplit.
template <int MT, int NT, int EPI, bool SPLIT = false, bool STATS = false>
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
  // (with a split reduction the column tiles of split s are rotated by 8/splits * s dies: when the
  // number of column tiles is no multiple of 8, every die is then short of a tile in some splits
  // instead of the same dies in all of them)
  const int xcd = (blockIdx.x + (SPLIT ? (8 / (int)gridDim.z) * (int)blockIdx.z : 0)) & 7, slot = blockIdx.x >> 3;
  const int nt_local = slot / m_tiles;
  const int n_tile = nt_local * 8 + xcd;
  if (n_tile >= n_tiles) return;                      // whole workgroup leaves before any barrier
  const int m0 = (slot - nt_local * m_tiles) * BM, n0 = n_tile * BN;
  const int k = blockIdx.y;
  if (STATS && blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) {
    // what the acceptance kernel needs to know about the row reductions this launch leaves behind
    FusedStatsHeader* h = (FusedStatsHeader*)((unsigned char*)a.stats - (size_t)a.M * kFusedMergedSlots * sizeof(RowPart) - sizeof(FusedStatsHeader));
    h->n_parts = a.stats_parts;
    h->typical = a.stats_k2 > 0.f ? 1 : 0;
    h->k2 = a.stats_k2;
    h->rows = a.M;
  }
  const unsigned char* Xb = (const unsigned char*)a.X;
  const unsigned char* Wb = (const unsigned char*)a.W + (size_t)k * a.N * a.d * 2;

  // Chunk `it` of a thread: tile row it*32 + tid/8 (activation rows first, then weight rows), 16-byte
  // chunk tid%8.  Rows past the matrix edge are clamped (loaded twice, never stored).
  uint32_t goff[LPT];
#pragma unroll
  for (int it = 0; it < LPT; ++it) {
    const int row = it * 32 + (tid >> 3), c = tid & 7;
    goff[it] = it < MT ? (uint32_t)((x_row_offset<kHeadMajor<EPI>>(a, min(m0 + row, a.M - 1), k) + c * 8) * 2)
                       : (uint32_t)(((size_t)min(n0 + row - BM, a.N - 1) * a.d + c * 8) * 2);
  }
  const int nk_all = a.d >> 6;
  const int n_split = SPLIT ? (int)gridDim.z : 1, split = SPLIT ? (int)blockIdx.z : 0;
  const int step0 = (int)((long)nk_all * split / n_split);
  const int nk = (int)((long)nk_all * (split + 1) / n_split) - step0;   // this workgroup's share of the reduction (>= 1)
  u32x4_t G[LPT];
  auto gload = [&](int step, u32x4_t (&g)[LPT]) __attribute__((always_inline)) {
    const int j0 = (step0 + min(step, nk - 1)) * 64;             // past the end: harmless reload
    const uint32_t so_w = (uint32_t)j0 * 2u;
    const uint32_t so_x = (uint32_t)x_col_offset<kHeadMajor<EPI>>(a, j0) * 2u;    // differs from so_w for head-major activations
#pragma unroll
    for (int it = 0; it < LPT; ++it) g[it] = *(const u32x4_t*)((it < MT ? Xb : Wb) + (goff[it] + (it < MT ? so_x : so_w)));
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

  // Epilogue.  An MFMA result tile has four consecutive rows of one column per lane -- no two
  // neighbouring columns in one lane -- so storing from the registers would issue 2- and 4-byte
  // accesses.  Each wavefront therefore passes its tile, 16 rows at a time, through a private LDS
  // area (fp32, row pitch 132 words: conflict-free both ways) and reads it back with 8 consecutive
  // columns per lane: 16- and 32-byte accesses, four lanes covering a contiguous 32-column run.
  if (SPLIT && n_split > 1) {
    // partial tile of this split: [fragment][register pair][thread], 8 bytes per thread and store
    const unsigned int tile = blockIdx.y * gridDim.x + (slot << 3 | xcd);   // (the same for all splits of a tile: xcd is the rotated one)
    constexpr int PART = MT * NT * 2 * 256;            // 8-byte words per partial tile
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
    if (!last_workgroup_of(&g_big_ticket[a.ticket_slot][tile], (unsigned int)n_split)) return;
    // sum in split order; half a tile of one split is requested at a time (the other half of the
    // register file holds the sums)
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int j = 0; j < NT; ++j) acc[t][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    for (int z = 0; z < n_split; ++z) {
      const uint64_t* pz = part + (size_t)z * PART + tid;
#pragma unroll
      for (int t0 = 0; t0 < MT; t0 += MT / 2) {
        uint64_t v[MT / 2][NT][2];
#pragma unroll
        for (int t = 0; t < MT / 2; ++t)
#pragma unroll
          for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int rp = 0; rp < 2; ++rp) v[t][j][rp] = load_agent(pz + (((t0 + t) * NT + j) * 2 + rp) * 256);
#pragma unroll
        for (int t = 0; t < MT / 2; ++t)
#pragma unroll
          for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int rp = 0; rp < 2; ++rp) {
              acc[t0 + t][j][2 * rp] += __uint_as_float((uint32_t)v[t][j][rp]);
              acc[t0 + t][j][2 * rp + 1] += __uint_as_float((uint32_t)(v[t][j][rp] >> 32));
            }
      }
    }
  }
  __syncthreads();                                    // every wavefront is done with the stage buffers
  // EPI_SWIGLU: fragments 2j and 2j+1 of a wavefront are the gate rows and the up rows of the same 16
  // output columns (weights interleaved in blocks of 16 rows), so half as many fragments leave.
  constexpr bool SW = EPI == EPI_SWIGLU;
  constexpr int NTO = SW ? NT / 2 : NT;
  const int n_cols = SW ? a.N >> 1 : a.N, n_base = (SW ? n0 >> 1 : n0) + wn * 16 * NTO;
  constexpr int EP_PITCH = 16 * NTO + 4;              // words
  float* ep = (float*)lds + wave * 16 * EP_PITCH;
  static_assert(4 * 16 * EP_PITCH * 4 <= 2 * STAGE, "epilogue area must fit the stage buffers");
  const int er = lane >> 2, ec = (lane & 3) * 8;      // read-back: row, first column of the lane's 8
  const bool vec = a.vec_epilogue != 0;
#pragma unroll
  for (int t = 0; t < MT; ++t) {
#pragma unroll
    for (int j = 0; j < NTO; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        ep[(4 * q4 + r) * EP_PITCH + j * 16 + i16] = SW ? silu_fast(acc[t][2 * j][r]) * acc[t][2 * j + 1][r] : acc[t][j][r];
    const int m = m0 + (wm * MT + t) * 16 + er;
    const size_t row_off = m >= a.M ? 0 : (SW && a.y_dh == 0 ? (size_t)m * n_cols : out_row_offset<kHeadMajor<EPI>>(a, m, k));
    if (STATS) {
      // Row reductions for the acceptance step (Sec. 2.3.1), taken from the tile while it is in LDS so
      // that acceptance does not read the logits again: this lane's 32 values of row m (8 consecutive
      // columns in each of four 32-column runs), then the four lanes of the row.  A lane's columns
      // ascend and the key orders equal values by column, so the arg-max is the lowest column.
      uint64_t key = 0;
      float sm = -INFINITY, sS = 0.f, sU = 0.f;
      const float k2 = a.stats_k2;
      if (m < a.M) {
#pragma unroll
        for (int c = 0; c < NTO / 2; ++c) {
          const floatx4_t v0 = *(const floatx4_t*)(ep + er * EP_PITCH + c * 32 + ec);
          const floatx4_t v1 = *(const floatx4_t*)(ep + er * EP_PITCH + c * 32 + ec + 4);
          const float v[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
          const int n = n_base + c * 32 + ec;
          float bm = -INFINITY;
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (n + e < n_cols) {
              const uint64_t ke = rank_key(v[e], (uint32_t)(n + e));
              key = ke > key ? ke : key;
              bm = fmaxf(bm, v[e] * k2);
            }
          if (k2 > 0.f && bm > -INFINITY) {
            if (bm > sm) {                               // one rescale of the running sums per run of eight
              const float cf = sS > 0.f ? __builtin_amdgcn_exp2f(sm - bm) : 0.f;
              sU = sS > 0.f ? cf * (sU + (sm - bm) * sS) : 0.f;
              sS = cf * sS;
              sm = bm;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (n + e < n_cols) {
                const float dlt = v[e] * k2 - sm, p = __builtin_amdgcn_exp2f(dlt);
                sS += p;
                sU = fmaf(dlt, p, sU);
              }
          }
        }
      }
      // the four lanes of a row are a quad: two exchange steps
#pragma unroll
      for (int step = 0; step < 2; ++step) {
        const uint32_t klo = step == 0 ? dpp_u32<kDppQuadSwap1>((uint32_t)key) : dpp_u32<kDppQuadSwap2>((uint32_t)key);
        const uint32_t khi = step == 0 ? dpp_u32<kDppQuadSwap1>((uint32_t)(key >> 32)) : dpp_u32<kDppQuadSwap2>((uint32_t)(key >> 32));
        const uint64_t ko = ((uint64_t)khi << 32) | klo;
        key = ko > key ? ko : key;
        const float m2 = step == 0 ? dpp_f32<kDppQuadSwap1>(sm) : dpp_f32<kDppQuadSwap2>(sm);
        const float S2 = step == 0 ? dpp_f32<kDppQuadSwap1>(sS) : dpp_f32<kDppQuadSwap2>(sS);
        const float U2 = step == 0 ? dpp_f32<kDppQuadSwap1>(sU) : dpp_f32<kDppQuadSwap2>(sU);
        stats_merge(sm, sS, sU, m2, S2, U2);
      }
      if ((lane & 3) == 0 && m < a.M) {
        RowPart* p = a.stats + (size_t)m * a.stats_parts + (n_tile * 2 + wn);
        p->key = key;
        p->m = sm;
        p->S = sS;
        p->U = sU;
      }
    }
#pragma unroll
    for (int c = 0; c < NTO / 2; ++c) {
      const floatx4_t v0 = *(const floatx4_t*)(ep + er * EP_PITCH + c * 32 + ec);
      const floatx4_t v1 = *(const floatx4_t*)(ep + er * EP_PITCH + c * 32 + ec + 4);
      const float v[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
      const int n = n_base + c * 32 + ec;
      if (m >= a.M || n >= n_cols) continue;
      if (vec && n + 8 <= n_cols) {
        const size_t o = row_off + out_col_offset<kHeadMajor<EPI>>(a, n);
        if (EPI == EPI_LOGITS) {
          float* dst = (float*)a.out + o;
          *(floatx4_t*)dst = v0;
          *(floatx4_t*)(dst + 4) = v1;
        } else {
          float y[8];
          if (EPI == EPI_PLAIN || SW) {
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = v[e];
          } else {
            // EPI_RESID: hidden[m][n..] with row length d (= N);  EPI_GATED: mul[m][n..] with row length N
            const u32x4_t h = *(const u32x4_t*)((const uint16_t*)a.hidden + (size_t)m * a.N + n);
            const uint32_t hw[4] = {h.x, h.y, h.z, h.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const float u = bf16_bits_to_float((hw[e >> 1] >> (16 * (e & 1))) & 0xffffu);
              y[e] = EPI == EPI_RESID ? silu_fast(v[e]) + u : silu_fast(v[e]) * u;
            }
          }
          u32x4_t w;
          w.x = pack_bf16x2(y[0], y[1]);
          w.y = pack_bf16x2(y[2], y[3]);
          w.z = pack_bf16x2(y[4], y[5]);
          w.w = pack_bf16x2(y[6], y[7]);
          *(u32x4_t*)((uint16_t*)a.out + o) = w;
        }
      } else {
        // ragged or unaligned output: one element at a time
        for (int e = 0; e < 8; ++e) {
          if (n + e >= n_cols) break;
          const size_t o = row_off + out_col_offset<kHeadMajor<EPI>>(a, n + e);
          if (EPI == EPI_LOGITS) {
            ((float*)a.out)[o] = v[e];
          } else if (EPI == EPI_PLAIN || SW) {
            ((uint16_t*)a.out)[o] = (uint16_t)float_to_bf16_bits(v[e]);
          } else {
            const float u = bf16_bits_to_float(((const uint16_t*)a.hidden)[(size_t)m * a.N + n + e]);
            ((uint16_t*)a.out)[o] = (uint16_t)float_to_bf16_bits(EPI == EPI_RESID ? silu_fast(v[e]) + u : silu_fast(v[e]) * u);
          }
        }
      }
    }
  }
}

template <int EPI>
int launch(const GemmArgs& a_in, bool tall, hipStream_t stream) {
  GemmArgs a = a_in;
  // 16-byte epilogue accesses need 8-column runs that are contiguous and aligned in the output and
  // in the tensor the epilogue reads
  const size_t align = (size_t)a.out | (size_t)(EPI == EPI_RESID || EPI == EPI_GATED ? a.hidden : nullptr);
  a.vec_epilogue = (EPI == EPI_SWIGLU ? a.N % 16 == 0 : a.N % 8 == 0) && align % 16 == 0 && (a.y_dh == 0 || a.y_dh % 8 == 0) ? 1 : 0;
  // 192 x 256 or 128 x 256 tile, as the caller planned
  const int n_tiles = ceil_div(a.N, 256);
  const int m_tiles = ceil_div(a.M, tall ? 192 : 128);
  constexpr bool kCanSplit = EPI == EPI_PLAIN || EPI == EPI_GATED;     // (the epilogues tree_linear uses)
  const int gx = 8 * ceil_div(n_tiles, 8) * m_tiles;
  const int ksplit = kCanSplit && a.ws && a.ksplit > 1 && (long)gx * a.K <= kMaxBigSplitTiles ? a.ksplit : 1;
  const dim3 grid(gx, a.K, ksplit), block(256);
  if (EPI == EPI_LOGITS && a.stats != nullptr) {          // (its own instantiation: the plain kernel's code stays as it is)
    if (tall) hipLaunchKernelGGL((gemm_big_bf16_kernel<6, 8, EPI, false, EPI == EPI_LOGITS>), grid, block, 0, stream, a, m_tiles, n_tiles);
    else hipLaunchKernelGGL((gemm_big_bf16_kernel<4, 8, EPI, false, EPI == EPI_LOGITS>), grid, block, 0, stream, a, m_tiles, n_tiles);
  } else if (ksplit > 1) {
    if (tall) hipLaunchKernelGGL((gemm_big_bf16_kernel<6, 8, EPI, kCanSplit>), grid, block, 0, stream, a, m_tiles, n_tiles);
    else hipLaunchKernelGGL((gemm_big_bf16_kernel<4, 8, EPI, kCanSplit>), grid, block, 0, stream, a, m_tiles, n_tiles);
  } else {
    if (tall) hipLaunchKernelGGL((gemm_big_bf16_kernel<6, 8, EPI>), grid, block, 0, stream, a, m_tiles, n_tiles);
    else hipLaunchKernelGGL((gemm_big_bf16_kernel<4, 8, EPI>), grid, block, 0, stream, a, m_tiles, n_tiles);
  }
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}

}  // namespace

int launch_gemm_big(const GemmArgs& a, int epi, bool tall, hipStream_t stream) {
  if (a.d % 64 != 0 || a.d < 64) return MEDUSA_EUNSUPPORTED;
  if ((size_t)a.N * a.d >= ((size_t)1 << 31) || x_extent(a) >= ((size_t)1 << 31)) return MEDUSA_EUNSUPPORTED;
  switch (epi) {
    case EPI_LOGITS: return launch<EPI_LOGITS>(a, tall, stream);
    case EPI_RESID: return launch<EPI_RESID>(a, tall, stream);
    case EPI_PLAIN: return launch<EPI_PLAIN>(a, tall, stream);
    case EPI_GATED: return launch<EPI_GATED>(a, tall, stream);
    case EPI_SWIGLU: return launch<EPI_SWIGLU>(a, tall, stream);
  }
  return MEDUSA_EINVAL;
}
