// tree_attention (Sec. 2.1.2 of the Medusa paper): soft-max attention of the T tree tokens over
// the cached prefix plus the tree itself, where a tree token sees only its own continuation
// (ancestors and itself).  The tree mask is one 128-bit word per query row.
//
// bf16 path: split-K flash-decoding on 16x16x32 bf16 MFMA.
//   * One workgroup = one (sequence, KV head, block of up to 96 query rows, split of the key
//     range).  All G = Hq/Hkv query heads that share the KV head are handled together: their
//     G*T rows are contiguous in q and out.
//   * Keys are numbered prefix first, tree after (key L+u is tree node u), and processed in
//     64-key blocks; a split owns a contiguous run of blocks, computed from prefix_len[b] on
//     the device.  K and V tiles are fetched with full-line 16-byte loads one block ahead of
//     their use (registers), then parked in swizzled, double-buffered LDS tiles: one barrier
//     per block.
//   * A wavefront owns 16 query rows and, for them, all keys of a block and the whole head
//     dimension.  Scores are formed transposed, S^T = K Q^T, so each lane owns one query column:
//     the row maximum and sum take two cross-lane steps, and the probabilities go from the
//     accumulators straight into the second product O^T = V^T P^T as its B operand -- nothing
//     of the soft-max passes through LDS and no wavefront waits for another inside a block.
//     (An earlier version gave each wavefront 16 keys of the block for all rows in the first
//     product and a quarter of the head dimension in the second: fewer LDS reads, but the maxima
//     and the probabilities crossed LDS behind two more barriers; 20/48/78/140 us against
//     18/40/42/122 us now at the four bf16 benchmark shapes.)
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

#include <mutex>

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

typedef short short4_t __attribute__((ext_vector_type(4)));

// Four bf16 of a transposed tile: within each group of 16 lanes, lane j of the group receives
// element (j % 4) of the 8-byte rows addressed by lanes j/4, j/4 + 4, j/4 + 8, j/4 + 12 of the
// group (ds_read_b64_tr_b16).  With lane r addressing V[key0 + r/4][d0 + 4*(r%4) .. +3], lane j
// receives V[key0 .. key0+3][d0 + j]: four consecutive keys of one head-dimension column.
__device__ __forceinline__ short4_t lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t*)p);
}

// ---------------------------------------------------------------------------------------
// MFMA split-K kernel, bf16.  grid (n_splits, Hkv*row_blocks, B), 64*NW threads.
// Operand layout of v_mfma_f32_16x16x32_bf16 (A: 16 x 32, B: 32 x 16, C: 16 x 16): lane l
// holds row (A) / column (B) l%16 and reduction elements 8*(l/16)..+7; it receives column
// l%16 and rows 4*(l/16)..+3 of C.
// Wavefront w owns the MTW tiles of 16 query rows w*MTW.. of the workgroup's row block and, for
// them, ALL 64 keys of a block and the whole head dimension: the row maximum and
// sum need two cross-lane steps and no LDS, the probabilities go from the accumulators of
// S^T = K Q^T straight into the B operand of O^T = V^T P^T (lane l%16 = query row in both; the
// reduction slots of a 32-key step are keys 4*(l/16)..+3 of its two 16-key tiles, and the V
// fragment is read transposed in the same order), and the only barrier of a 64-key block is the
// one that publishes the next K and V tiles (double-buffered in LDS, fetched one block ahead into
// registers by all wavefronts together).
// ---------------------------------------------------------------------------------------
template <int D, int MTW, int NW>
__global__ __launch_bounds__(64 * NW, (NW + 3) / 4) void tree_attn_rows_kernel(AttnArgs a) {
  constexpr int KS = D / 32;                    // reduction steps of K Q^T
  constexpr int DT = D / 16;                    // 16-wide tiles of the head dimension
  constexpr int NTH = 64 * NW;
  constexpr int PITCH = D * 2;                  // bytes per row of the K and V tiles (unpadded, swizzled as above)
  constexpr int TENSOR_BYTES = kBlkKeys * PITCH;
  constexpr int CPR = D / 8;                    // 16-byte chunks per K/V row
  constexpr int CHUNKS = kBlkKeys * CPR;        // per block and tensor
  constexpr int LPT = (CHUNKS + NTH - 1) / NTH; // chunks per thread per block and tensor
  constexpr int ROWS = 16 * MTW * NW;           // query rows of a workgroup
  __shared__ __attribute__((aligned(16))) unsigned char s_kv[2][2][TENSOR_BYTES];   // [buffer][K, V]
  __shared__ uint64_t s_anc[ROWS][2];           // ancestor mask of every query row of this workgroup

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
  const int row0 = rb * ROWS + wave * 16 * MTW;          // first query row of this wavefront

  const uint16_t* qg = (const uint16_t*)a.q + ((size_t)b * a.Hq + (size_t)kvh * a.G) * T * D;
  const uint16_t* kc = (const uint16_t*)a.k_cache + ((size_t)b * a.Hkv + kvh) * a.Lcap * D;
  const uint16_t* vc = (const uint16_t*)a.v_cache + ((size_t)b * a.Hkv + kvh) * a.Lcap * D;
  const uint16_t* kt = (const uint16_t*)a.k_tree + ((size_t)b * a.Hkv + kvh) * T * D;
  const uint16_t* vt = (const uint16_t*)a.v_tree + ((size_t)b * a.Hkv + kvh) * T * D;

  for (int r = tid; r < ROWS; r += NTH) {
    const int tq = min(rb * ROWS + r, R - 1) % T;
    s_anc[r][0] = a.tree->anc_mask[tq][0];
    s_anc[r][1] = a.tree->anc_mask[tq][1];
  }
  // Q^T fragments (B operand of K Q^T): column = query row, reduction = head dimension.
  bf16x8_t qf[MTW][KS];
#pragma unroll
  for (int mt = 0; mt < MTW; ++mt) {
    const int r = min(row0 + 16 * mt + i16, R - 1);
#pragma unroll
    for (int c = 0; c < KS; ++c) qf[mt][c] = *(const bf16x8_t*)(qg + (size_t)r * D + 32 * c + 8 * q4);
  }

  // This thread's chunks of a K (or V) block (chunk ids past the block repeat the last chunk).
  auto swz_k = [](int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); };
  auto swz_v = [](int r) { return D == 128 ? 2 * (r & 7) : 2 * ((r >> 1) & 3); };
  int ch_row[LPT], ch_off[LPT], ch_dst_k[LPT], ch_dst_v[LPT];
#pragma unroll
  for (int it = 0; it < LPT; ++it) {
    const int id = min(it * NTH + tid, CHUNKS - 1);
    ch_row[it] = id / CPR;
    const int chunk = id - ch_row[it] * CPR;
    ch_off[it] = ch_row[it] * D + chunk * 8;
    ch_dst_k[it] = ch_row[it] * PITCH + ((chunk ^ swz_k(ch_row[it])) << 4);
    ch_dst_v[it] = ch_row[it] * PITCH + ((chunk ^ swz_v(ch_row[it])) << 4);
  }
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

  floatx4_t o[MTW][DT];
  float m_run[MTW], l_run[MTW];
#pragma unroll
  for (int mt = 0; mt < MTW; ++mt) {
    m_run[mt] = -INFINITY;
    l_run[mt] = 0.f;
#pragma unroll
    for (int dd = 0; dd < DT; ++dd) o[mt][dd] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  }
  const float sc = a.scale * 1.4426950408889634f;        // scores are kept in log2 units
  const int kswz = swz_k(i16);
  const int kf_off = i16 * PITCH;
  // transposed V read: lane r of a 16-lane group addresses V[4*q4 + r/4 (+16)][16*dd + 4*(r%4) .. +3]
  const int v_row = 4 * q4 + (i16 >> 2);
  const int v_chunk0 = (i16 & 3) >> 1, v_half = 8 * (i16 & 1);

  u32x4_t kreg[LPT], vreg[LPT];
  if (n_iter > 0) {
    gload(0, kc, kt, kreg);
    gload(0, vc, vt, vreg);
    lstore(s_kv[0][0], ch_dst_k, kreg);
    lstore(s_kv[0][1], ch_dst_v, vreg);
    gload(1, kc, kt, kreg);
    gload(1, vc, vt, vreg);
  }
  __syncthreads();

  for (int i = 0; i < n_iter; ++i) {
    // here: K and V of block i are in LDS buffer i%2, those of block i+1 in registers (or in flight)
    const unsigned char* s_k = s_kv[i & 1][0];
    const unsigned char* s_v = s_kv[i & 1][1];
    const int key0 = (blk_lo + i) * kBlkKeys;
    const bool all_visible = key0 + kBlkKeys <= L;
    const int sh = L - key0;                              // position of tree node 0 inside the block
    // ---- S^T = K Q^T: four tiles of 16 keys, this wavefront's query tiles ----
    floatx4_t sv[MTW][4];
#pragma unroll
    for (int kt4 = 0; kt4 < 4; ++kt4) {
      bf16x8_t kf[KS];
#pragma unroll
      for (int c = 0; c < KS; ++c) kf[c] = *(const bf16x8_t*)(s_k + 16 * kt4 * PITCH + kf_off + (((4 * c + q4) ^ kswz) << 4));
#pragma unroll
      for (int mt = 0; mt < MTW; ++mt) {
        floatx4_t acc = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < KS; ++c) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[c], qf[mt][c], acc, 0, 0, 0);
        sv[mt][kt4] = acc * sc;
      }
    }
    // the next block's tiles go to the other buffer (free since the barrier of block i-1); then
    // the requests for the block after it
    lstore(s_kv[(i & 1) ^ 1][0], ch_dst_k, kreg);
    lstore(s_kv[(i & 1) ^ 1][1], ch_dst_v, vreg);
    gload(i + 2, kc, kt, kreg);
    gload(i + 2, vc, vt, vreg);
    // ---- mask, online soft-max, probabilities as the B operand of the second product ----
    bf16x8_t pf[MTW][2];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
      if (!all_visible) {
        // keys key0 .. key0+63: prefix keys are visible to all, tree key L+u iff ancestor bit u
        const int row = wave * 16 * MTW + 16 * mt + i16;
        const uint64_t lo = s_anc[row][0], hi = s_anc[row][1];
        uint64_t tree_bits;
        if (sh >= 0) tree_bits = lo << sh;
        else if (sh > -64) tree_bits = (lo >> (-sh)) | (hi << (64 + sh));
        else tree_bits = hi >> (-sh - 64);
        const uint64_t vis = tree_bits | (sh > 0 ? (1ull << sh) - 1ull : 0ull);
#pragma unroll
        for (int kt4 = 0; kt4 < 4; ++kt4) {
          const uint32_t my = (uint32_t)(vis >> (16 * kt4 + 4 * q4));
#pragma unroll
          for (int r = 0; r < 4; ++r) sv[mt][kt4][r] = (my >> r) & 1u ? sv[mt][kt4][r] : -INFINITY;
        }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int kt4 = 0; kt4 < 4; ++kt4)
        mx = fmaxf(mx, fmaxf(fmaxf(sv[mt][kt4][0], sv[mt][kt4][1]), fmaxf(sv[mt][kt4][2], sv[mt][kt4][3])));
      mx = rows_max(mx);
      const float m_new = fmaxf(m_run[mt], mx);
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run[mt] - m_safe);
      float psum = 0.f;
      uint32_t pk[4][2];
#pragma unroll
      for (int kt4 = 0; kt4 < 4; ++kt4) {
        const float p0 = __builtin_amdgcn_exp2f(sv[mt][kt4][0] - m_safe), p1 = __builtin_amdgcn_exp2f(sv[mt][kt4][1] - m_safe);
        const float p2 = __builtin_amdgcn_exp2f(sv[mt][kt4][2] - m_safe), p3 = __builtin_amdgcn_exp2f(sv[mt][kt4][3] - m_safe);
        psum += (p0 + p1) + (p2 + p3);
        pk[kt4][0] = pack_bf16x2(p0, p1);
        pk[kt4][1] = pack_bf16x2(p2, p3);
      }
      l_run[mt] = l_run[mt] * alpha + psum;
      m_run[mt] = m_new;
      // after the first blocks the running maximum rarely moves: skip the rescale when no row of
      // this tile needs it (alpha is exactly 1 then)
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int dd = 0; dd < DT; ++dd) o[mt][dd] *= alpha;
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const u32x4_t w = {pk[2 * ks][0], pk[2 * ks][1], pk[2 * ks + 1][0], pk[2 * ks + 1][1]};
        pf[mt][ks] = __builtin_bit_cast(bf16x8_t, w);
      }
    }
    // ---- O^T += V^T P^T: reduction slots of step ks = keys 32*ks + 4*q4..+3 and 32*ks + 16 + 4*q4..+3 ----
#pragma unroll
    for (int dd = 0; dd < DT; ++dd) {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const int r0 = 32 * ks + v_row, r1 = r0 + 16;
        const short4_t v0 = lds_read_tr16(s_v + r0 * PITCH + (((v_chunk0 + 2 * dd) ^ swz_v(r0)) << 4) + v_half);
        const short4_t v1 = lds_read_tr16(s_v + r1 * PITCH + (((v_chunk0 + 2 * dd) ^ swz_v(r1)) << 4) + v_half);
        typedef short short8_t __attribute__((ext_vector_type(8)));
        const short8_t v8 = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
        const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, v8);
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) o[mt][dd] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[mt][ks], o[mt][dd], 0, 0, 0);
      }
    }
    __syncthreads();        // the next block's tiles are visible; every wavefront has left this block's
  }

  // ---- write: final output (single split) or the split's partial ----------------------------
  typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
  typedef float float4v_t __attribute__((ext_vector_type(4)));
  uint16_t* og = (uint16_t*)a.out + ((size_t)b * a.Hq + (size_t)kvh * a.G) * T * D;
#pragma unroll
  for (int mt = 0; mt < MTW; ++mt) {
    const float l = rows_sum(l_run[mt]);                  // over this lane's key slots and its three partner lanes
    const int r = row0 + 16 * mt + i16;
    if (r >= R) continue;
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    if (a.n_splits == 1) {
#pragma unroll
      for (int dd = 0; dd < DT; ++dd) {
        u32x2_t w;
        w.x = pack_bf16x2(o[mt][dd][0] * inv, o[mt][dd][1] * inv);
        w.y = pack_bf16x2(o[mt][dd][2] * inv, o[mt][dd][3] * inv);
        *(u32x2_t*)(og + (size_t)r * D + 16 * dd + 4 * q4) = w;
      }
    } else {
      const size_t unit = ((size_t)b * a.Hkv + kvh) * a.n_splits + split;
      uint64_t* prow = a.ws_o + (unit * R + r) * (D / 4);
#pragma unroll
      for (int dd = 0; dd < DT; ++dd) {
        const float4v_t f = {o[mt][dd][0] * inv, o[mt][dd][1] * inv, o[mt][dd][2] * inv, o[mt][dd][3] * inv};
        prow[4 * dd + q4] = __builtin_bit_cast(uint64_t, __builtin_convertvector(f, half4_t));
      }
      if (q4 == 0) {
        const f32x2_t ml = {m_run[mt], l};
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
  int nw, row_blocks, n_splits;
};

// One tile of 16 query rows per wavefront, up to six wavefronts per workgroup; more rows are cut
// into row blocks (which re-read K and V, from L2 when they run side by side).  Two tiles per
// wavefront halve the LDS reads per row but measured slower (the per-block chain of a wavefront
// doubles and one workgroup per CU has nothing to cover it with: 162 against 138 us at B = 16,
// G = 4).
Plan make_plan(int B, int Hq, int Hkv, int T, int Lcap) {
  Plan p;
  const int R = (Hq / Hkv) * T;
  const int tiles = ceil_div(R, 16);
  p.row_blocks = ceil_div(tiles, 6);
  p.nw = ceil_div(tiles, p.row_blocks);
  p.row_blocks = ceil_div(tiles, p.nw);
  const int blocks = ceil_div(Lcap + T, kBlkKeys);
  const int base = B * Hkv * p.row_blocks;
  // One workgroup runs per CU.  A single sequence has splits of equal length: one round of at most
  // 256 workgroups (8192 keys, 32 heads: 8 splits 39.5 us, 6 41.6, 10 53.6, 16 47.3).  A batch is
  // ragged (the host does not know the lengths): about twice as many workgroups even out the long
  // sequences (B = 4, 40 heads: 1/2/3/4 splits 50/47/43/47 us; B = 16, 8 KV heads x 3 row blocks:
  // 138/122/123).  At least four key blocks per split: each split costs a partial write and read
  // of about 80 keys' worth of bytes.
  int want = B == 1 ? 256 / base : ceil_div(448, base);
  const int cap = blocks / 4 > 1 ? blocks / 4 : 1;
  want = want < 1 ? 1 : (want > cap ? cap : want);
  p.n_splits = ceil_div(blocks, ceil_div(blocks, want));
  return p;
}

template <int D>
int launch_mfma(const AttnArgs& a, const Plan& p, hipStream_t stream) {
  const dim3 grid(a.n_splits, a.Hkv * a.row_blocks, a.B), block(64 * p.nw);
#define MEDUSA_ATTN(NW_) \
  case NW_: hipLaunchKernelGGL((tree_attn_rows_kernel<D, 1, NW_>), grid, block, 0, stream, a); break
  switch (p.nw) {
    MEDUSA_ATTN(1); MEDUSA_ATTN(2); MEDUSA_ATTN(3); MEDUSA_ATTN(4); MEDUSA_ATTN(5); MEDUSA_ATTN(6);
    default: return MEDUSA_EUNSUPPORTED;
  }
#undef MEDUSA_ATTN
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

// Scratch of tree_attention_static: the split partials live in this array instead of a caller
// workspace.  Every GPU the library runs on holds its own copy until the process ends; host code
// reaches it only through the per-device address looked up once below, never through the name.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
std::mutex g_scratch_mutex;
void* g_scratch_ptr[64] = {};

int static_scratch(void** out) {
  int dev = 0;
  MEDUSA_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return MEDUSA_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    MEDUSA_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || ((uintptr_t)p & 255) != 0) return MEDUSA_EHIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MEDUSA_OK;
}
}  // namespace

extern "C" size_t tree_attention_static_scratch_bytes(void) { return kStaticScratchBytes; }

extern "C" int tree_attention_static(const void* q, const void* k_tree, const void* v_tree, const void* k_cache,
                                     const void* v_cache, const int32_t* prefix_len, const medusa_tree_t* tree, void* out,
                                     int B, int Hq, int Hkv, int D, int Lcap, float scale, medusa_dtype_t dtype,
                                     medusa_stream_t stream_) {
  if (!tree) return MEDUSA_EINVAL;
  if (B < 1 || Hq < 1 || Hkv < 1 || Lcap < 1 || Hq % Hkv != 0) return MEDUSA_EINVAL;
  const size_t need = tree_attention_workspace_bytes(B, Hq, Hkv, tree->host.T, D, Lcap);
  if (need > kStaticScratchBytes) return MEDUSA_ESCRATCH;     // the shape's split partials exceed the built-in scratch
  void* ptr = nullptr;
  const int rc = static_scratch(&ptr);
  if (rc != MEDUSA_OK) return rc;
  return tree_attention(q, k_tree, v_tree, k_cache, v_cache, prefix_len, tree, out, B, Hq, Hkv, D, Lcap, scale, dtype, ptr,
                        kStaticScratchBytes, stream_);
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
