// tree_attention (Sec. 2.1.2 of the Medusa paper): soft-max attention of the T tree tokens over
// the cached prefix plus the tree itself, where a tree token sees only its own continuation
// (ancestors and itself).  The tree mask is one 128-bit word per query row.
//
// bf16 path: split-K flash-decoding on 16x16x32 bf16 MFMA.
//   * One workgroup = one (sequence, KV head, block of up to 80 query rows, split of the key
//     range).  All G = Hq/Hkv query heads that share the KV head are handled together: their
//     G*T rows are contiguous in q and out.
//   * Keys are numbered prefix first, tree after (key L+u is tree node u), and processed in
//     64-key blocks; a split owns a contiguous run of blocks, computed from prefix_len[b] on
//     the device.  K and V tiles are fetched with full-line 16-byte loads one block ahead of
//     their use (registers), then parked in swizzled LDS tiles; K of block i+1 and V of block i
//     are written between the two barriers of block i, so single tiles suffice and two
//     workgroups fit on a CU to cover each other's latencies.
//   * Scores are formed transposed, S^T = K Q^T: wavefront w owns keys 16w..16w+15 of the block
//     for all query rows, so each lane owns one query column per tile and the row maximum needs
//     two cross-lane steps plus one exchange of 4 x rows floats through LDS.  The probabilities
//     go to LDS as bf16 [query][key]; in the second product O^T = V^T P^T wavefront w owns a
//     quarter of the head dimension for all query rows, so the output accumulators are never
//     merged across wavefronts.  Two barriers per 64 keys.
//   * The tree mask is the 128-bit ancestor word of the lane's query node shifted to the block's
//     key range; keys past the valid range are redirected to a valid row and masked, so stale or
//     poisoned cache rows are never used.
//   * A split writes its partial as fp16 output normalised by its own soft-max sum plus the
//     fp32 running maximum and sum; a second small kernel merges the splits in index order
//     (skipped when there is a single split), so results are run-to-run bit-identical.  Merging
//     inside the first kernel (last split elected by a ticket) was tried and measured slower:
//     one workgroup pulling all partials of a head is a serial tail of several round trips.
// fp32 path (and any D the MFMA path does not cover): one workgroup per query row, plain FMAs.
#include <math.h>

#include "common.hpp"

namespace {

constexpr int kBlkKeys = 64;

struct AttnArgs {
  const void *q, *k_tree, *v_tree, *k_cache, *v_cache;
  const int32_t* prefix_len;
  const TreeTables* tree;
  void* out;
  uint64_t* ws_o;    // [B*Hkv*n_splits][R][D/4] partial outputs, normalised by their own sum, 4 x fp16
  uint64_t* ws_ml;   // [B*Hkv*n_splits][R] (running max in log2 units, sum) as two floats
  int B, Hq, Hkv, T, Lcap, G, R, n_splits, row_blocks;
  float scale;
};

// ---------------------------------------------------------------------------------------
// Plain kernel: grid (T, Hq, B), 256 threads, one query row per workgroup.
// ---------------------------------------------------------------------------------------
template <typename E, int D>
__global__ __launch_bounds__(256) void tree_attn_plain_kernel(AttnArgs a) {
  constexpr int CH = 2048;                    // keys per pass
  constexpr int SL = 256 / D;                 // key slices accumulating in parallel
  __shared__ float s_q[D];
  __shared__ float s_p[CH];
  __shared__ float s_red[8];
  __shared__ float s_acc[256];
  const int t = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int kvh = g / a.G;
  const int L = min(max(a.prefix_len[b], 0), a.Lcap);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const E* qrow = (const E*)a.q + (((size_t)b * a.Hq + g) * a.T + t) * D;
  const E* kc = (const E*)a.k_cache + ((size_t)b * a.Hkv + kvh) * a.Lcap * D;
  const E* vc = (const E*)a.v_cache + ((size_t)b * a.Hkv + kvh) * a.Lcap * D;
  const E* kt = (const E*)a.k_tree + ((size_t)b * a.Hkv + kvh) * a.T * D;
  const E* vt = (const E*)a.v_tree + ((size_t)b * a.Hkv + kvh) * a.T * D;
  const uint64_t m0 = a.tree->anc_mask[t][0], m1 = a.tree->anc_mask[t][1];
  if (tid < D) s_q[tid] = load_as_float<E>(qrow + tid) * a.scale;
  __syncthreads();
  const int n_keys = L + a.T;
  const int dcol = tid % D, slice = tid / D;
  float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
  for (int c0 = 0; c0 < n_keys; c0 += CH) {
    const int cn = min(CH, n_keys - c0);
    float mx = -INFINITY;
    for (int j = tid; j < cn; j += 256) {
      const int key = c0 + j;
      float s = -INFINITY;
      const E* krow = nullptr;
      if (key < L) krow = kc + (size_t)key * D;
      else {
        const int u = key - L;
        if (((u < 64 ? m0 >> u : m1 >> (u - 64)) & 1ull) != 0) krow = kt + (size_t)u * D;
      }
      if (krow) {
        s = 0.f;
        for (int c = 0; c < D; ++c) s = fmaf(s_q[c], load_as_float<E>(krow + c), s);
      }
      s_p[j] = s;
      mx = fmaxf(mx, s);
    }
    mx = wave_max(mx);
    if (lane == 0) s_red[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
    const float m_new = fmaxf(m_run, mx);
    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
    float sum = 0.f;
    for (int j = tid; j < cn; j += 256) {
      const float p = expf(s_p[j] - m_safe);
      s_p[j] = p;
      sum += p;
    }
    sum = wave_sum(sum);
    if (lane == 0) s_red[4 + wave] = sum;
    __syncthreads();
    sum = s_red[4] + s_red[5] + s_red[6] + s_red[7];
    const float alpha = expf(m_run - m_safe);
    l_run = l_run * alpha + sum;
    acc *= alpha;
    for (int j = slice; j < cn; j += SL) {
      const float p = s_p[j];
      if (p != 0.f) {
        const int key = c0 + j;
        const E* vrow = key < L ? vc + (size_t)key * D : vt + (size_t)(key - L) * D;
        acc = fmaf(p, load_as_float<E>(vrow + dcol), acc);
      }
    }
    m_run = m_new;
    __syncthreads();
  }
  s_acc[tid] = acc;
  __syncthreads();
  if (tid < D) {
    float o = 0.f;
    for (int s = 0; s < SL; ++s) o += s_acc[s * D + tid];
    E* orow = (E*)a.out + (((size_t)b * a.Hq + g) * a.T + t) * D;
    store_from_float<E>(orow + tid, o / l_run);
  }
}

// ---------------------------------------------------------------------------------------
// MFMA split-K kernel, bf16.  grid (n_splits, Hkv*row_blocks, B), 256 threads.
// Operand layout of v_mfma_f32_16x16x32_bf16 (A: 16 x 32, B: 32 x 16, C: 16 x 16): lane l
// holds row (A) / column (B) l%16 and reduction elements 8*(l/16)..+7; it receives column
// l%16 and rows 4*(l/16)..+3 of C.
// ---------------------------------------------------------------------------------------
typedef short short4_t __attribute__((ext_vector_type(4)));

// Four bf16 of a transposed tile: within each group of 16 lanes, lane j of the group receives
// element (j % 4) of the 8-byte rows addressed by lanes j/4, j/4 + 4, j/4 + 8, j/4 + 12 of the
// group (ds_read_b64_tr_b16).  With lane r addressing V[key0 + r/4][d0 + 4*(r%4) .. +3], lane j
// receives V[key0 .. key0+3][d0 + j]: four consecutive keys of one head-dimension column.
__device__ __forceinline__ short4_t lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t*)p);
}

template <int D, int MT>
__global__ __launch_bounds__(256, 2) void tree_attn_mfma_kernel(AttnArgs a) {
  constexpr int KS = D / 32;                    // reduction steps of K Q^T
  constexpr int DPW = D / 64;                   // 16-wide output tiles of the head dimension per wavefront
  // LDS tiles are unpadded; the 16-byte chunk c of row r is stored at chunk slot c ^ swz(r), chosen
  // per tile so that its reads are bank-conflict free (a 64-lane 16-byte read is served in four
  // groups of 16 lanes that are not consecutive lanes, an 8-byte read in groups of 16 consecutive
  // lanes; padded pitches leave both kinds of read two-way conflicted):
  //   K, read as MFMA operands (16 rows x 4 chunks per instruction): swz = r & 15 (256-byte rows) or
  //     (r >> 1) & 7 (128-byte rows);
  //   V, read 8 bytes per lane transposed (4 rows x 32 bytes per 16 lanes): swz = 2 (r & 7), resp.
  //     2 ((r >> 1) & 3);
  //   P (128-byte rows, MFMA-operand reads, 8-byte writes): swz = (r >> 1) & 7.
  constexpr int PITCH = D * 2;                  // bytes per row of the K and V tiles
  constexpr int TENSOR_BYTES = kBlkKeys * PITCH;
  constexpr int PPITCH = kBlkKeys * 2;          // bytes per row of the probability tile
  constexpr int CPR = D / 8;                    // 16-byte chunks per K/V row
  constexpr int LPT = kBlkKeys * CPR / 256;     // chunks per thread per block and tensor
  __shared__ __attribute__((aligned(16))) unsigned char s_k[TENSOR_BYTES];
  __shared__ __attribute__((aligned(16))) unsigned char s_v[TENSOR_BYTES];
  __shared__ __attribute__((aligned(16))) unsigned char s_p[16 * MT * PPITCH];
  __shared__ __attribute__((aligned(16))) float s_max[16 * MT][4];   // block maximum per query row and wavefront
  __shared__ float s_sum[4][16 * MT];
  __shared__ uint64_t s_anc[16 * MT][2];        // ancestor mask of every query row of this workgroup

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, q4 = lane >> 4;
  const int split = blockIdx.x;
  const int kvh = blockIdx.y / a.row_blocks, rb = blockIdx.y - kvh * a.row_blocks;
  const int b = blockIdx.z;
  const int T = a.T, R = a.R;
  const int L = min(max(a.prefix_len[b], 0), a.Lcap);
  const int n_keys = L + T;
  const int nblk = ceil_div(n_keys, kBlkKeys);
  const int bps = ceil_div(nblk, a.n_splits);
  const int blk_lo = min(split * bps, nblk), blk_hi = min(nblk, blk_lo + bps);
  const int n_iter = blk_hi - blk_lo;
  const int row0 = rb * 16 * MT;

  const uint16_t* qg = (const uint16_t*)a.q + ((size_t)b * a.Hq + (size_t)kvh * a.G) * T * D;
  const uint16_t* kc = (const uint16_t*)a.k_cache + ((size_t)b * a.Hkv + kvh) * a.Lcap * D;
  const uint16_t* vc = (const uint16_t*)a.v_cache + ((size_t)b * a.Hkv + kvh) * a.Lcap * D;
  const uint16_t* kt = (const uint16_t*)a.k_tree + ((size_t)b * a.Hkv + kvh) * T * D;
  const uint16_t* vt = (const uint16_t*)a.v_tree + ((size_t)b * a.Hkv + kvh) * T * D;

  if (tid < 16 * MT) {
    const int tq = min(row0 + tid, R - 1) % T;
    s_anc[tid][0] = a.tree->anc_mask[tq][0];
    s_anc[tid][1] = a.tree->anc_mask[tq][1];
  }
  // Q^T fragments (B operand of K Q^T): column = query row, reduction = head dimension.
  bf16x8_t qf[MT][KS];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int r = min(row0 + 16 * mt + i16, R - 1);
#pragma unroll
    for (int c = 0; c < KS; ++c) qf[mt][c] = *(const bf16x8_t*)(qg + (size_t)r * D + 32 * c + 8 * q4);
  }

  // This thread's chunks of a K (or V) block: row in the block, element offset, LDS offset.
  auto swz_k = [](int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); };
  auto swz_v = [](int r) { return D == 128 ? 2 * (r & 7) : 2 * ((r >> 1) & 3); };
  int ch_row[LPT], ch_off[LPT], ch_dst_k[LPT], ch_dst_v[LPT];
#pragma unroll
  for (int it = 0; it < LPT; ++it) {
    const int id = it * 256 + tid;
    ch_row[it] = id / CPR;
    const int chunk = id - ch_row[it] * CPR;
    ch_off[it] = ch_row[it] * D + chunk * 8;
    ch_dst_k[it] = ch_row[it] * PITCH + ((chunk ^ swz_k(ch_row[it])) << 4);
    ch_dst_v[it] = ch_row[it] * PITCH + ((chunk ^ swz_v(ch_row[it])) << 4);
  }
  // One tensor's rows of block `iter` of this split (index clamped into the split's range;
  // the redundant reloads past the end are never used).
  auto gload = [&](int iter, const uint16_t* cache, const uint16_t* tree_rows, u32x4_t (&r)[LPT]) __attribute__((always_inline)) {
    const int key0 = (blk_lo + min(iter, n_iter - 1)) * kBlkKeys;
    if (key0 + kBlkKeys <= L) {                  // the common case: the whole block lies in the prefix
      const uint16_t* base = cache + (size_t)key0 * D;
#pragma unroll
      for (int it = 0; it < LPT; ++it) r[it] = *(const u32x4_t*)(base + ch_off[it]);
    } else {
#pragma unroll
      for (int it = 0; it < LPT; ++it) {
        const int key = min(key0 + ch_row[it], n_keys - 1);   // keys past the end repeat the last key (masked)
        const int col = ch_off[it] - ch_row[it] * D;
        const uint16_t* base = key < L ? cache + (size_t)key * D : tree_rows + (size_t)(key - L) * D;
        r[it] = *(const u32x4_t*)(base + col);
      }
    }
  };
  auto lstore = [&](unsigned char* tile, const int (&dst)[LPT], const u32x4_t (&r)[LPT]) __attribute__((always_inline)) {
#pragma unroll
    for (int it = 0; it < LPT; ++it) *(u32x4_t*)(tile + dst[it]) = r[it];
  };

  floatx4_t o[MT][DPW];
  float m_run[MT], l_run[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    m_run[mt] = -INFINITY;
    l_run[mt] = 0.f;
#pragma unroll
    for (int dd = 0; dd < DPW; ++dd) o[mt][dd] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  }
  const float sc = a.scale * 1.4426950408889634f;        // scores are kept in log2 units
  const int kswz = swz_k(i16);                           // (a wavefront's 16-key tile starts at a multiple of 16)
  const int kf_off = (16 * wave + i16) * PITCH;
  const int pswz = (i16 >> 1) & 7;
  const int p_wr_off = i16 * PPITCH + (((2 * wave + (q4 >> 1)) ^ pswz) << 4) + 8 * (q4 & 1);
  const int p_rd_off = i16 * PPITCH;
  // transposed V read: lane r of a 16-lane group addresses V[8*q4 + r/4 (+4)][16*dd' + 4*(r%4) .. +3]
  const int v_row = 8 * q4 + (i16 >> 2);
  const int v_chunk0 = 2 * (wave * DPW) + ((i16 & 3) >> 1), v_half = 8 * (i16 & 1);

  u32x4_t kreg[LPT], vreg[LPT];
  if (n_iter > 0) {
    gload(0, kc, kt, kreg);
    gload(0, vc, vt, vreg);
    lstore(s_k, ch_dst_k, kreg);
    gload(1, kc, kt, kreg);
  }
  __syncthreads();

  for (int i = 0; i < n_iter; ++i) {
    // here: K of block i is in LDS, K of block i+1 and V of block i are in registers (or in flight)
    const int key0 = (blk_lo + i) * kBlkKeys;
    // ---- S^T for this wavefront's 16 keys, all query tiles ----
    bf16x8_t kf[KS];
#pragma unroll
    for (int c = 0; c < KS; ++c) kf[c] = *(const bf16x8_t*)(s_k + kf_off + (((4 * c + q4) ^ kswz) << 4));
    floatx4_t sv[MT];
    const bool all_visible = key0 + kBlkKeys <= L;
    const int sh = L - key0;                              // position of tree node 0 inside the block
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      floatx4_t s = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < KS; ++c) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[c], qf[mt][c], s, 0, 0, 0);
      s *= sc;
      if (!all_visible) {
        // keys key0 .. key0+63: prefix keys are visible to all, tree key L+u iff ancestor bit u
        const uint64_t lo = s_anc[16 * mt + i16][0], hi = s_anc[16 * mt + i16][1];
        uint64_t tree_bits;
        if (sh >= 0) tree_bits = lo << sh;
        else if (sh > -64) tree_bits = (lo >> (-sh)) | (hi << (64 + sh));
        else tree_bits = hi >> (-sh - 64);
        const uint64_t vis = tree_bits | (sh > 0 ? (1ull << sh) - 1ull : 0ull);
        const uint32_t my = (uint32_t)(vis >> (16 * wave + 4 * q4));
#pragma unroll
        for (int r = 0; r < 4; ++r) s[r] = (my >> r) & 1u ? s[r] : -INFINITY;
      }
      sv[mt] = s;
      float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
      mx = rows_max(mx);
      if (q4 == 0) s_max[16 * mt + i16][wave] = mx;
    }
    __syncthreads();        // A: block maxima are visible; every wavefront has left block i-1 and the K tile
    // ---- online soft-max update, probabilities to LDS ----
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int c = 16 * mt + i16;
      const floatx4_t m4 = *(const floatx4_t*)s_max[c];
      const float mx = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3]));
      const float m_new = fmaxf(m_run[mt], mx);
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run[mt] - m_safe);
      const float p0 = __builtin_amdgcn_exp2f(sv[mt][0] - m_safe), p1 = __builtin_amdgcn_exp2f(sv[mt][1] - m_safe);
      const float p2 = __builtin_amdgcn_exp2f(sv[mt][2] - m_safe), p3 = __builtin_amdgcn_exp2f(sv[mt][3] - m_safe);
      l_run[mt] = l_run[mt] * alpha + ((p0 + p1) + (p2 + p3));
      m_run[mt] = m_new;
      // after the first blocks the running maximum rarely moves: skip the rescale when no row of
      // this tile needs it (alpha is exactly 1 then)
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int dd = 0; dd < DPW; ++dd) o[mt][dd] *= alpha;
      }
      u32x2_t w;
      w.x = pack_bf16x2(p0, p1);
      w.y = pack_bf16x2(p2, p3);
      *(u32x2_t*)(s_p + 16 * mt * PPITCH + p_wr_off) = w;
    }
    // tiles: K of the next block (the K tile is free since barrier A), V of this block (the V tile
    // was last read in block i-1, which every wavefront left before barrier A); then start the
    // loads that will be parked one block from now
    lstore(s_k, ch_dst_k, kreg);
    lstore(s_v, ch_dst_v, vreg);
    gload(i + 2, kc, kt, kreg);
    gload(i + 1, vc, vt, vreg);
    __syncthreads();        // B: probabilities, the V tile and the next K tile are visible
    // ---- O^T += V^T P^T for this wavefront's slice of the head dimension ----
#pragma unroll
    for (int ks = 0; ks < kBlkKeys / 32; ++ks) {
      bf16x8_t pf[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        pf[mt] = *(const bf16x8_t*)(s_p + 16 * mt * PPITCH + p_rd_off + (((4 * ks + q4) ^ pswz) << 4));
#pragma unroll
      for (int dd = 0; dd < DPW; ++dd) {
        const int r0 = 32 * ks + v_row, r1 = r0 + 4;
        const short4_t v0 = lds_read_tr16(s_v + r0 * PITCH + (((v_chunk0 + 2 * dd) ^ swz_v(r0)) << 4) + v_half);
        const short4_t v1 = lds_read_tr16(s_v + r1 * PITCH + (((v_chunk0 + 2 * dd) ^ swz_v(r1)) << 4) + v_half);
        typedef short short8_t __attribute__((ext_vector_type(8)));
        const short8_t v8 = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
        const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, v8);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) o[mt][dd] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[mt], o[mt][dd], 0, 0, 0);
      }
    }
  }

  // ---- totals of the soft-max denominators: over this lane's key slots, lanes, wavefronts ----
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    float l = l_run[mt];
    l = rows_sum(l);
    if (q4 == 0) s_sum[wave][16 * mt + i16] = l;
  }
  __syncthreads();
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int c = 16 * mt + i16;
    l_run[mt] = (s_sum[0][c] + s_sum[1][c]) + (s_sum[2][c] + s_sum[3][c]);
  }

  // ---- write: final output (single split) or the split's partial ----------------------------
  typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
  typedef float float4v_t __attribute__((ext_vector_type(4)));
  uint16_t* og = (uint16_t*)a.out + ((size_t)b * a.Hq + (size_t)kvh * a.G) * T * D;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int r = row0 + 16 * mt + i16;
    if (r >= R) continue;
    const float inv = l_run[mt] > 0.f ? 1.0f / l_run[mt] : 0.f;
    if (a.n_splits == 1) {
#pragma unroll
      for (int dd = 0; dd < DPW; ++dd) {
        u32x2_t w;
        w.x = pack_bf16x2(o[mt][dd][0] * inv, o[mt][dd][1] * inv);
        w.y = pack_bf16x2(o[mt][dd][2] * inv, o[mt][dd][3] * inv);
        *(u32x2_t*)(og + (size_t)r * D + 16 * (wave * DPW + dd) + 4 * q4) = w;
      }
    } else {
      const size_t unit = ((size_t)b * a.Hkv + kvh) * a.n_splits + split;
      uint64_t* prow = a.ws_o + (unit * R + r) * (D / 4);
#pragma unroll
      for (int dd = 0; dd < DPW; ++dd) {
        const float4v_t f = {o[mt][dd][0] * inv, o[mt][dd][1] * inv, o[mt][dd][2] * inv, o[mt][dd][3] * inv};
        prow[4 * (wave * DPW + dd) + q4] = __builtin_bit_cast(uint64_t, __builtin_convertvector(f, half4_t));
      }
      if (wave == 0 && q4 == 0) {
        const f32x2_t ml = {m_run[mt], l_run[mt]};
        a.ws_ml[unit * R + r] = __builtin_bit_cast(uint64_t, ml);
      }
    }
  }
}

// Merge the splits of a (sequence, KV head): grid (ceil(R*D/4 / 256), Hkv, B), 256 threads, one
// thread per (query row, four output columns), splits in index order.
template <int D>
__global__ __launch_bounds__(256) void tree_attn_combine_kernel(AttnArgs a) {
  typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
  const int u = blockIdx.x * 256 + threadIdx.x;
  const int kvh = blockIdx.y, b = blockIdx.z;
  const int R = a.R;
  if (u >= R * (D / 4)) return;
  const int r = u / (D / 4), c4 = u % (D / 4);
  const size_t unit0 = ((size_t)b * a.Hkv + kvh) * a.n_splits;
  float mm = -INFINITY;
  for (int sp = 0; sp < a.n_splits; ++sp) {
    const f32x2_t ml = __builtin_bit_cast(f32x2_t, a.ws_ml[(unit0 + sp) * R + r]);
    mm = fmaxf(mm, ml[0]);
  }
  float num[4] = {0.f, 0.f, 0.f, 0.f}, den = 0.f;
  for (int sp = 0; sp < a.n_splits; ++sp) {
    const f32x2_t ml = __builtin_bit_cast(f32x2_t, a.ws_ml[(unit0 + sp) * R + r]);
    const float w = ml[1] > 0.f ? __builtin_amdgcn_exp2f(ml[0] - mm) * ml[1] : 0.f;
    const half4_t h = __builtin_bit_cast(half4_t, a.ws_o[((unit0 + sp) * R + r) * (D / 4) + c4]);
    den += w;
#pragma unroll
    for (int e = 0; e < 4; ++e) num[e] += w * (float)h[e];
  }
  const float inv = 1.0f / den;
  uint16_t* og = (uint16_t*)a.out + ((size_t)b * a.Hq + (size_t)kvh * a.G) * a.T * D;
  u32x2_t w;
  w.x = pack_bf16x2(num[0] * inv, num[1] * inv);
  w.y = pack_bf16x2(num[2] * inv, num[3] * inv);
  *(u32x2_t*)(og + (size_t)r * D + 4 * c4) = w;
}

struct Plan {
  int mt, row_blocks, n_splits;
};

Plan make_plan(int B, int Hq, int Hkv, int T, int Lcap) {
  Plan p;
  const int R = (Hq / Hkv) * T;
  const int tiles = ceil_div(R, 16);
  p.mt = tiles >= 5 ? 5 : tiles;
  p.row_blocks = ceil_div(tiles, p.mt);
  const int blocks = ceil_div(Lcap + T, kBlkKeys);
  const int base = B * Hkv * p.row_blocks;
  // two workgroups fit on a CU: aim at ~2 x 256 of them, but keep at least four key blocks per
  // split: each split costs a partial write and read of about 80 keys' worth of bytes
  int want = 512 / base;
  const int cap = blocks / 4 > 1 ? blocks / 4 : 1;
  want = want < 1 ? 1 : (want > cap ? cap : want);
  p.n_splits = ceil_div(blocks, ceil_div(blocks, want));
  return p;
}

template <int D>
int launch_mfma(const AttnArgs& a, const Plan& p, hipStream_t stream) {
  const dim3 grid(a.n_splits, a.Hkv * a.row_blocks, a.B), block(256);
  switch (p.mt) {
    case 1: hipLaunchKernelGGL((tree_attn_mfma_kernel<D, 1>), grid, block, 0, stream, a); break;
    case 2: hipLaunchKernelGGL((tree_attn_mfma_kernel<D, 2>), grid, block, 0, stream, a); break;
    case 3: hipLaunchKernelGGL((tree_attn_mfma_kernel<D, 3>), grid, block, 0, stream, a); break;
    case 4: hipLaunchKernelGGL((tree_attn_mfma_kernel<D, 4>), grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL((tree_attn_mfma_kernel<D, 5>), grid, block, 0, stream, a); break;
  }
  MEDUSA_LAUNCH_CHECK();
  if (a.n_splits > 1) {
    hipLaunchKernelGGL((tree_attn_combine_kernel<D>), dim3(ceil_div(a.R * (D / 4), 256), a.Hkv, a.B), dim3(256), 0,
                       stream, a);
    MEDUSA_LAUNCH_CHECK();
  }
  return MEDUSA_OK;
}

}  // namespace

extern "C" size_t tree_attention_workspace_bytes(int B, int Hq, int Hkv, int T, int D, int Lcap) {
  if (B < 1 || Hq < 1 || Hkv < 1 || T < 1 || D < 1 || Lcap < 1 || Hq % Hkv != 0) return 0;
  const Plan p = make_plan(B, Hq, Hkv, T, Lcap);
  const size_t R = (size_t)(Hq / Hkv) * T;
  const size_t bytes = (size_t)B * Hkv * p.n_splits * R * (D * 2 + 8);   // fp16 rows + (max, sum)
  return (bytes + 255) & ~(size_t)255;
}

extern "C" int tree_attention(const void* q, const void* k_tree, const void* v_tree, const void* k_cache,
                              const void* v_cache, const int32_t* prefix_len, const medusa_tree_t* tree, void* out, int B,
                              int Hq, int Hkv, int D, int Lcap, float scale, medusa_dtype_t dtype, void* workspace,
                              size_t workspace_bytes, medusa_stream_t stream_) {
  if (!q || !k_tree || !v_tree || !k_cache || !v_cache || !prefix_len || !tree || !out) return MEDUSA_EINVAL;
  if (B < 1 || Hq < 1 || Hkv < 1 || Lcap < 1 || Hq % Hkv != 0) return MEDUSA_EINVAL;
  if (dtype != MEDUSA_F32 && dtype != MEDUSA_BF16) return MEDUSA_EINVAL;
  if (D != 64 && D != 128) return MEDUSA_EUNSUPPORTED;
  if (B > 65535 || Hq > 65535) return MEDUSA_EUNSUPPORTED;
  if (!tree->dev) return MEDUSA_EHIP;
  const int T = tree->host.T;
  const size_t need = tree_attention_workspace_bytes(B, Hq, Hkv, T, D, Lcap);
  if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255) != 0) return MEDUSA_EWORKSPACE;
  hipStream_t stream = (hipStream_t)stream_;
  const Plan p = make_plan(B, Hq, Hkv, T, Lcap);
  AttnArgs a;
  a.q = q; a.k_tree = k_tree; a.v_tree = v_tree; a.k_cache = k_cache; a.v_cache = v_cache;
  a.prefix_len = prefix_len;
  a.tree = tree->dev;
  a.out = out;
  a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.T = T; a.Lcap = Lcap;
  a.G = Hq / Hkv;
  a.R = a.G * T;
  a.n_splits = p.n_splits;
  a.row_blocks = p.row_blocks;
  a.scale = scale;
  a.ws_o = (uint64_t*)workspace;
  a.ws_ml = a.ws_o + (size_t)B * Hkv * p.n_splits * a.R * (D / 4);
  if (dtype == MEDUSA_F32) {
    const dim3 grid(T, Hq, B), block(256);
    if (D == 64) hipLaunchKernelGGL((tree_attn_plain_kernel<float, 64>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((tree_attn_plain_kernel<float, 128>), grid, block, 0, stream, a);
    MEDUSA_LAUNCH_CHECK();
    return MEDUSA_OK;
  }
  return D == 64 ? launch_mfma<64>(a, p, stream) : launch_mfma<128>(a, p, stream);
}
