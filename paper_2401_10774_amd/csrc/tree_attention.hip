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
//     the device.  K and V tiles (and the Q tiles) go from global memory straight into swizzled LDS
//     tiles (global_load_lds_dwordx4: no registers, no LDS stores), one step of two blocks ahead of
//     their use, completion tracked by hand with the load counter: one barrier per step.
//   * A wavefront owns 16 query rows and, for them, all keys of a block and the whole head
//     dimension.  Scores are formed transposed, S^T = K Q^T, so each lane owns one query column:
//     the row maximum and sum take two cross-lane steps, and the probabilities go from the
//     accumulators straight into the second product O^T = V^T P^T as its B operand -- nothing
//     of the soft-max passes through LDS and no wavefront waits for another inside a block.
//     Two wavefronts share a row tile and take alternate blocks (independent soft-max streams,
//     merged once at the end): a block is one dependent chain LDS read -> MFMA -> soft-max -> LDS
//     read -> MFMA per wavefront, and what covers it is more wavefronts per SIMD (MI355X, four bf16
//     benchmark shapes: 17.6/39.7/45/132 us with one wavefront per tile, 17/37/42/105-110 with two).
//     (An earlier version gave each wavefront 16 keys of the block for all rows in the first
//     product and a quarter of the head dimension in the second: fewer LDS reads, but the maxima
//     and the probabilities crossed LDS behind two more barriers: 20/48/78/140 us.)
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
  int B, Hq, Hkv, T, Lcap, G, R, n_splits, row_blocks, ranked;
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

// Batches up to this size are served longest sequence first (see the kernel).
constexpr int kRankedBatch = 64;

// Four bf16 of a transposed tile: within each group of 16 lanes, lane j of the group receives
// element (j % 4) of the 8-byte rows addressed by lanes j/4, j/4 + 4, j/4 + 8, j/4 + 12 of the
// group (ds_read_b64_tr_b16).  With lane r addressing V[key0 + r/4][d0 + 4*(r%4) .. +3], lane j
// receives V[key0 .. key0+3][d0 + j]: four consecutive keys of one head-dimension column.
__device__ __forceinline__ short4_t lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t*)p);
}

// ---------------------------------------------------------------------------------------
// MFMA split-K kernel, bf16.  1-D grid of 8 * ceil(units / 8) * row_blocks workgroups, 64*NT*KH threads.
// Operand layout of v_mfma_f32_16x16x32_bf16 (A: 16 x 32, B: 32 x 16, C: 16 x 16): lane l
// holds row (A) / column (B) l%16 and reduction elements 8*(l/16)..+7; it receives column
// l%16 and rows 4*(l/16)..+3 of C.
// A workgroup walks its split of the key range in steps of KH blocks of 64 keys.  Wavefront
// w = h * NT + t owns the tile of 16 query rows t of the workgroup's row block and, in every step,
// block h of the step: for its rows it sees ALL 64 keys of that block and the whole head dimension,
// so the row maximum and sum need two cross-lane steps and no LDS, the probabilities go from the
// accumulators of S^T = K Q^T straight into the B operand of O^T = V^T P^T (lane l%16 = query row in
// both; the reduction slots of a 32-key step are keys 4*(l/16)..+3 of its two 16-key tiles, and the V
// fragment is read transposed in the same order), and the only barrier of a step is the one that
// publishes the next K and V tiles (double-buffered in LDS, fetched one step ahead into registers
// by all wavefronts together).  With KH = 2 the two wavefronts of a row tile run independent
// soft-max streams over alternating blocks -- twice the wavefronts per SIMD to hide each other's
// LDS and MFMA latencies, the same LDS reads per key -- and their (max, sum, O) are merged once,
// through LDS, in a fixed order after the loop.
// Workgroup order: the row blocks of one (sequence, KV head, split) get linear ids 8 apart, which
// the hardware places on the same die, so that the second and third row block find K and V in
// that die's L2.
// ---------------------------------------------------------------------------------------
template <int D, int NT, int KH, int WPT>
__global__ __launch_bounds__(64 * NT * WPT, (NT * WPT + 3) / 4) void tree_attn_rows_kernel(AttnArgs a) {
  constexpr int NW = NT * WPT;                  // WPT wavefronts per row tile share the KH blocks of a step
  constexpr int BPW = KH / WPT;                 // blocks of a step per wavefront
  constexpr int KS = D / 32;                    // reduction steps of K Q^T
  constexpr int DT = D / 16;                    // 16-wide tiles of the head dimension
  constexpr int NTH = 64 * NW;
  constexpr int PITCH = D * 2;                  // bytes per row of the K and V tiles (unpadded, swizzled as above)
  constexpr int TENSOR_BYTES = kBlkKeys * PITCH;
  constexpr int CPR = D / 8;                    // 16-byte chunks per K/V row
  constexpr int RPW = 64 / CPR;                 // K/V rows one wavefront-wide 16-byte-per-lane load covers (1 KB)
  constexpr int WLT = KH * kBlkKeys / RPW;      // wavefront loads per tensor and step
  constexpr int WL = 2 * WLT;                   // ... per step (K tiles, then V tiles)
  constexpr int LPW = (WL + NW - 1) / NW;       // loads a wavefront issues per step (the first WL % NW wavefronts; one less the others)
  constexpr int LMIN = WL / NW;                 // ... at least
  constexpr int STAGES = KH == 1 ? 4 : 2;       // steps resident in LDS: the ring the loads fill directly
  constexpr int ROWS = 16 * NT;                 // query rows of a workgroup
  constexpr int BUF_BYTES = 2 * KH * TENSOR_BYTES;          // one step: its K tiles, then its V tiles
  extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];
  unsigned char* s_kv = s_dyn;                                   // [STAGES][K, V][KH][TENSOR_BYTES]
  unsigned char* s_q = s_dyn + STAGES * BUF_BYTES;               // [NT][16 rows][PITCH]: the Q tiles
  uint64_t (*s_anc)[2] = (uint64_t (*)[2])(s_q + NT * 16 * PITCH);   // ancestor mask of every query row of this workgroup

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tile = wave % NT, half = wave / NT;
  const int i16 = lane & 15, q4 = lane >> 4;
  // linear id -> (die, slot on the die) -> (unit, row block); see the header comment
  const int units = a.B * a.Hkv * a.n_splits;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int unit = xcd + 8 * (slot / a.row_blocks), rb = slot % a.row_blocks;
  if (unit >= units) return;
  const int split = unit % a.n_splits;
  const int kvh = (unit / a.n_splits) % a.Hkv;
  // Longest sequences first: workgroups start in the order of their ids, so the sequence slot of this
  // id is given the sequence of that rank by prefix length (ties by index) -- a ragged batch then ends
  // on its short sequences instead of on a long one that started late.  The host does not know
  // the lengths; every workgroup ranks them itself (small batches only: B^2 comparisons; only when the
  // launch has more workgroups than CUs).  B = 16, prefixes 512..4096, 384 workgroups: 93 -> 85 us.
  int b = unit / (a.n_splits * a.Hkv);
  if (a.B > 1 && a.B <= kRankedBatch && a.ranked) {
    __shared__ int s_seq;
    if (tid < a.B) {
      const int mine = min(max(a.prefix_len[tid], 0), a.Lcap);
      int rank = 0;
      for (int u = 0; u < a.B; ++u) {
        const int other = min(max(a.prefix_len[u], 0), a.Lcap);
        rank += (other > mine || (other == mine && u < tid)) ? 1 : 0;
      }
      if (rank == b) s_seq = tid;
    }
    __syncthreads();
    b = s_seq;
  }
  const int T = a.T, R = a.R;
  const int L = min(max(a.prefix_len[b], 0), a.Lcap);
  const int n_keys = L + T;
  const int nblk = ceil_div(n_keys, kBlkKeys);
  const int bps = ceil_div(nblk, a.n_splits);
  const int blk_lo = min(split * bps, nblk), blk_hi = min(nblk, blk_lo + bps);
  const int n_iter = ceil_div(blk_hi - blk_lo, KH);
  const int row0 = rb * ROWS + tile * 16;                // first query row of this wavefront

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
  // K and V tiles go from global memory straight into LDS (global_load_lds_dwordx4: 16 bytes per lane,
  // the 64 lanes of an instruction fill 1 KB of LDS in lane order), no registers and no LDS stores in
  // between.  The tiles are stored with their 16-byte chunks XOR-swizzled per row (K for the
  // MFMA-operand reads, V for the 8-byte transposed reads), so the permutation is applied on the
  // global side: the lane that fills slot c' of row r fetches chunk c' ^ swz(r) of that row.
  // Load j of a step covers rows RPW*j .. of the step's K rows (j < WLT) or V rows; wavefront w issues
  // loads w, w + NW, ...
  auto swz_k = [](int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); };
  auto swz_v = [](int r) { return D == 128 ? 2 * (r & 7) : 2 * ((r >> 1) & 3); };
  // (addresses as integers: the choice between the four tensors stays a select on two registers)
  const uint64_t kc_u = (uint64_t)(uintptr_t)kc, vc_u = (uint64_t)(uintptr_t)vc;
  const uint64_t kt_u = (uint64_t)(uintptr_t)kt, vt_u = (uint64_t)(uintptr_t)vt;
  int ld_row[LPW], ld_colb[LPW];
  uint64_t ld_cache[LPW], ld_tree[LPW];
#pragma unroll
  for (int u = 0; u < LPW; ++u) {
    const int j = min(wave + u * NW, WL - 1);
    const bool is_v = j >= WLT;
    const int r = RPW * (j - (is_v ? WLT : 0)) + lane / CPR;          // row of the step: 0 .. 64*KH-1
    const int slot = lane % CPR;
    ld_row[u] = r;
    ld_colb[u] = ((slot ^ (is_v ? swz_v(r & 63) : swz_k(r & 63))) << 4);   // byte offset of the chunk inside the row
    ld_cache[u] = is_v ? vc_u : kc_u;
    ld_tree[u] = is_v ? vt_u : kt_u;
  }
  // keys of step `iter`: blocks blk_lo + KH*iter .. +KH-1; blocks at or past blk_hi belong to the next
  // split (or do not exist): their rows are fetched from the split's last key instead and masked
  auto issue_loads = [&](int iter) __attribute__((always_inline)) {
    const int blk0 = blk_lo + KH * iter;
    const int key0 = blk0 * kBlkKeys;
    unsigned char* stage = s_kv + (iter % STAGES) * BUF_BYTES;
    const bool fast = key0 + KH * kBlkKeys <= L && blk0 + KH <= blk_hi;   // the common case: the whole step lies in the prefix
    const int last_key = min(n_keys, blk_hi * kBlkKeys) - 1;
#pragma unroll
    for (int u = 0; u < LPW; ++u) {
      const int j = wave + u * NW;
      if (u == LPW - 1 && LPW != LMIN && j >= WL) break;      // (wave-uniform)
      uint64_t src;
      if (fast) src = ld_cache[u] + (uint64_t)(key0 + ld_row[u]) * PITCH + ld_colb[u];
      else {
        const int key = min(key0 + ld_row[u], last_key);      // keys past the end repeat the last key (masked)
        src = (key < L ? ld_cache[u] + (uint64_t)key * PITCH : ld_tree[u] + (uint64_t)(key - L) * PITCH) + ld_colb[u];
      }
      load_to_lds_b128((const void*)(uintptr_t)src, stage + j * 1024);
    }
  };
  // Wait until this wavefront's loads of all but the `ahead` most recently issued steps have landed
  // (loads complete in order; a wavefront has at least LMIN per step in flight, so this never waits
  // for less than needed).
  auto wait_loads = [&](int ahead) __attribute__((always_inline)) {
    constexpr int N1 = LMIN < 63 ? LMIN : 63, N2 = 2 * LMIN < 63 ? 2 * LMIN : 63;   // (the counter has six bits)
    if (ahead <= 0) __builtin_amdgcn_s_waitcnt(0x0F70);
    else if (ahead == 1) __builtin_amdgcn_s_waitcnt(0x0F70 | (N1 & 15) | ((N1 >> 4) << 14));
    else __builtin_amdgcn_s_waitcnt(0x0F70 | (N2 & 15) | ((N2 >> 4) << 14));
  };

  floatx4_t o[DT];
  float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
  for (int dd = 0; dd < DT; ++dd) o[dd] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  const float sc = a.scale * 1.4426950408889634f;        // scores are kept in log2 units
  const int kswz = swz_k(i16);
  const int kf_off = i16 * PITCH;
  // transposed V read: lane r of a 16-lane group addresses V[4*q4 + r/4 (+16)][16*dd + 4*(r%4) .. +3]
  const int v_row = 4 * q4 + (i16 >> 2);
  const int v_chunk0 = (i16 & 3) >> 1, v_half = 8 * (i16 & 1);

  // Everything this wavefront has loaded the ordinary way (prefix length, masks) is waited for here, so
  // that the compiler, which cannot see the loads into LDS, places no wait of its own inside the
  // loop: it would count only its own loads and thereby wait for the whole ring.
  __builtin_amdgcn_s_waitcnt(0x0F70);
  // The Q tiles take the same road as the K tiles (same swizzle), in front of the ring's first steps,
  // so that one memory latency covers both; the first wavefront of a row tile fetches it.
  if (half == 0) {
#pragma unroll
    for (int u = 0; u < 16 / RPW; ++u) {
      const int r = min(row0 + RPW * u + lane / CPR, R - 1);
      const int rl = RPW * u + lane / CPR;
      load_to_lds_b128(qg + (size_t)r * D + (((lane % CPR) ^ swz_k(rl)) << 3), s_q + tile * 16 * PITCH + u * 1024);
    }
  }
  // prologue: the first STAGES-1 steps are requested; every later step is requested STAGES-1 iterations ahead
#pragma unroll
  for (int st = 0; st < STAGES - 1; ++st)
    if (st < n_iter) issue_loads(st);
  // Q^T fragments (B operand of K Q^T): column = query row, reduction = head dimension; read behind
  // the first step's barrier
  bf16x8_t qf[KS];
#pragma unroll
  for (int c = 0; c < KS; ++c) qf[c] = bf16x8_t{};

  for (int i = 0; i < n_iter; ++i) {
    // steps i .. min(i + STAGES - 2, n_iter - 1) are in flight or in LDS; wait for this wavefront's part
    // of step i, then the barrier: everybody's part of step i is in LDS, and everybody has left step
    // i - 1, whose buffer the request for step i + STAGES - 1 may now overwrite
    wait_loads(min(STAGES - 2, n_iter - 1 - i));
    lds_barrier();
    if (i + STAGES - 1 < n_iter) issue_loads(i + STAGES - 1);
    if (i == 0) {
#pragma unroll
      for (int c = 0; c < KS; ++c) qf[c] = *(const bf16x8_t*)(s_q + tile * 16 * PITCH + kf_off + (((4 * c + q4) ^ kswz) << 4));
    }
    const unsigned char* s_stage = s_kv + (i % STAGES) * BUF_BYTES;
    // ---- S^T = K Q^T for this wavefront's blocks of the step: four tiles of 16 keys each.  All of
    // them are issued before the first soft-max, so that with two blocks per wavefront the matrix
    // pipe works on the second block's scores (and later on the first block's P V) while the vector
    // ALU runs a soft-max ----
    floatx4_t sv[BPW][4];
#pragma unroll
    for (int hb = 0; hb < BPW; ++hb) {
      const unsigned char* s_k = s_stage + (half * BPW + hb) * TENSOR_BYTES;
#pragma unroll
      for (int kt4 = 0; kt4 < 4; ++kt4) {
        bf16x8_t kf[KS];
#pragma unroll
        for (int c = 0; c < KS; ++c) kf[c] = *(const bf16x8_t*)(s_k + 16 * kt4 * PITCH + kf_off + (((4 * c + q4) ^ kswz) << 4));
        floatx4_t acc = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < KS; ++c) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[c], qf[c], acc, 0, 0, 0);
        sv[hb][kt4] = acc;
      }
    }
#pragma unroll
    for (int hb = 0; hb < BPW; ++hb) {
      const unsigned char* s_v = s_stage + (KH + half * BPW + hb) * TENSOR_BYTES;
      const int blk = blk_lo + KH * i + half * BPW + hb;     // this wavefront's block
      const int key0 = blk * kBlkKeys;
      const bool live = blk < blk_hi;
      const bool all_visible = live && key0 + kBlkKeys <= L;
      const int sh = L - key0;                              // position of tree node 0 inside the block
#pragma unroll
      for (int kt4 = 0; kt4 < 4; ++kt4) sv[hb][kt4] *= sc;
      // ---- mask, online soft-max, probabilities as the B operand of the second product ----
      bf16x8_t pf[2];
      if (!all_visible) {
        // keys key0 .. key0+63: prefix keys are visible to all, tree key L+u iff ancestor bit u
        const int row = tile * 16 + i16;
        const uint64_t lo = s_anc[row][0], hi = s_anc[row][1];
        uint64_t tree_bits;
        if (sh >= 64) tree_bits = 0;
        else if (sh >= 0) tree_bits = lo << sh;
        else if (sh > -64) tree_bits = (lo >> (-sh)) | (hi << (64 + sh));
        else if (sh > -128) tree_bits = hi >> (-sh - 64);
        else tree_bits = 0;
        uint64_t vis = tree_bits | (sh >= 64 ? ~0ull : (sh > 0 ? (1ull << sh) - 1ull : 0ull));
        if (!live) vis = 0;
#pragma unroll
        for (int kt4 = 0; kt4 < 4; ++kt4) {
          const uint32_t my = (uint32_t)(vis >> (16 * kt4 + 4 * q4));
#pragma unroll
          for (int r = 0; r < 4; ++r) sv[hb][kt4][r] = (my >> r) & 1u ? sv[hb][kt4][r] : -INFINITY;
        }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int kt4 = 0; kt4 < 4; ++kt4)
        mx = fmaxf(mx, fmaxf(fmaxf(sv[hb][kt4][0], sv[hb][kt4][1]), fmaxf(sv[hb][kt4][2], sv[hb][kt4][3])));
      mx = rows_max(mx);
      const float m_new = fmaxf(m_run, mx);
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
      float psum = 0.f;
      uint32_t pk[4][2];
#pragma unroll
      for (int kt4 = 0; kt4 < 4; ++kt4) {
        const float p0 = __builtin_amdgcn_exp2f(sv[hb][kt4][0] - m_safe), p1 = __builtin_amdgcn_exp2f(sv[hb][kt4][1] - m_safe);
        const float p2 = __builtin_amdgcn_exp2f(sv[hb][kt4][2] - m_safe), p3 = __builtin_amdgcn_exp2f(sv[hb][kt4][3] - m_safe);
        psum += (p0 + p1) + (p2 + p3);
        pk[kt4][0] = pack_bf16x2(p0, p1);
        pk[kt4][1] = pack_bf16x2(p2, p3);
      }
      l_run = l_run * alpha + psum;
      m_run = m_new;
      // after the first blocks the running maximum rarely moves: skip the rescale when no row of
      // this tile needs it (alpha is exactly 1 then)
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int dd = 0; dd < DT; ++dd) o[dd] *= alpha;
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const u32x4_t w = {pk[2 * ks][0], pk[2 * ks][1], pk[2 * ks + 1][0], pk[2 * ks + 1][1]};
        pf[ks] = __builtin_bit_cast(bf16x8_t, w);
      }
      // ---- O^T += V^T P^T: reduction slots of step ks = keys 32*ks + 4*q4..+3 and 32*ks + 16 + 4*q4..+3 ----
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
        for (int dd = 0; dd < DT; ++dd) {
          const int r0 = 32 * ks + v_row, r1 = r0 + 16;
          const short4_t v0 = lds_read_tr16(s_v + r0 * PITCH + (((v_chunk0 + 2 * dd) ^ swz_v(r0)) << 4) + v_half);
          const short4_t v1 = lds_read_tr16(s_v + r1 * PITCH + (((v_chunk0 + 2 * dd) ^ swz_v(r1)) << 4) + v_half);
          typedef short short8_t __attribute__((ext_vector_type(8)));
          const short8_t v8 = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
          const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, v8);
          o[dd] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[ks], o[dd], 0, 0, 0);
        }
      }
    }
  }
  __syncthreads();          // every wavefront has left the last step's tiles

  // ---- the KH soft-max streams of a row tile are merged in LDS (K/V tiles are dead after the last barrier) ----
  if (WPT > 1) {
    float* s_m = (float*)s_kv;                            // [NT][DT*4 + 2][64]
    constexpr int SLOTS = DT * 4 + 2;
    if (half == 1) {
      float* dst = s_m + (size_t)tile * SLOTS * 64 + lane;
#pragma unroll
      for (int dd = 0; dd < DT; ++dd)
#pragma unroll
        for (int e = 0; e < 4; ++e) dst[(4 * dd + e) * 64] = o[dd][e];
      dst[(DT * 4) * 64] = m_run;
      dst[(DT * 4 + 1) * 64] = l_run;
    }
    __syncthreads();
    if (half == 1) return;
    const float* src = s_m + (size_t)tile * SLOTS * 64 + lane;
    const float m1 = src[(DT * 4) * 64], l1 = src[(DT * 4 + 1) * 64];
    const float m_new = fmaxf(m_run, m1);
    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
    const float a0 = __builtin_amdgcn_exp2f(m_run - m_safe), a1 = __builtin_amdgcn_exp2f(m1 - m_safe);
#pragma unroll
    for (int dd = 0; dd < DT; ++dd)
#pragma unroll
      for (int e = 0; e < 4; ++e) o[dd][e] = o[dd][e] * a0 + src[(4 * dd + e) * 64] * a1;
    l_run = l_run * a0 + l1 * a1;
    m_run = m_new;
  }

  // ---- write: final output (single split) or the split's partial ----------------------------
  typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
  typedef float float4v_t __attribute__((ext_vector_type(4)));
  uint16_t* og = (uint16_t*)a.out + ((size_t)b * a.Hq + (size_t)kvh * a.G) * T * D;
  const float l = rows_sum(l_run);                      // over this lane's key slots and its three partner lanes
  const int r = row0 + i16;
  if (r >= R) return;
  const float inv = l > 0.f ? 1.0f / l : 0.f;
  if (a.n_splits == 1) {
#pragma unroll
    for (int dd = 0; dd < DT; ++dd) {
      u32x2_t w;
      w.x = pack_bf16x2(o[dd][0] * inv, o[dd][1] * inv);
      w.y = pack_bf16x2(o[dd][2] * inv, o[dd][3] * inv);
      *(u32x2_t*)(og + (size_t)r * D + 16 * dd + 4 * q4) = w;
    }
  } else {
    const size_t punit = ((size_t)b * a.Hkv + kvh) * a.n_splits + split;
    uint64_t* prow = a.ws_o + (punit * R + r) * (D / 4);
#pragma unroll
    for (int dd = 0; dd < DT; ++dd) {
      const float4v_t f = {o[dd][0] * inv, o[dd][1] * inv, o[dd][2] * inv, o[dd][3] * inv};
      prow[4 * dd + q4] = __builtin_bit_cast(uint64_t, __builtin_convertvector(f, half4_t));
    }
    if (q4 == 0) {
      const f32x2_t ml = {m_run, l};
      a.ws_ml[punit * R + r] = __builtin_bit_cast(uint64_t, ml);
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
  uint16_t* og = (uint16_t*)a.out + ((size_t)b * a.Hq + (size_t)kvh * a.G) * a.T * D;
  float num[4] = {0.f, 0.f, 0.f, 0.f}, den = 0.f, mm = -INFINITY;
  // splits in groups of eight: all (max, sum) pairs and partial rows of a group are requested before
  // the first is used (one memory round trip for up to eight splits), then folded in index order
  for (int s0 = 0; s0 < a.n_splits; s0 += 8) {
    uint64_t ml_raw[8], o_raw[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int sp = min(s0 + j, a.n_splits - 1);
      ml_raw[j] = a.ws_ml[(unit0 + sp) * R + r];
      o_raw[j] = a.ws_o[((unit0 + sp) * R + r) * (D / 4) + c4];
    }
    float gm = mm;
#pragma unroll
    for (int j = 0; j < 8; ++j) gm = fmaxf(gm, __builtin_bit_cast(f32x2_t, ml_raw[j])[0]);
    if (gm != mm) {                                       // rescale what the earlier groups have summed
      const float f = mm == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mm - gm);
      den *= f;
#pragma unroll
      for (int e = 0; e < 4; ++e) num[e] *= f;
      mm = gm;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (s0 + j >= a.n_splits) break;
      const f32x2_t ml = __builtin_bit_cast(f32x2_t, ml_raw[j]);
      const float w = ml[1] > 0.f ? __builtin_amdgcn_exp2f(ml[0] - mm) * ml[1] : 0.f;
      const half4_t h = __builtin_bit_cast(half4_t, o_raw[j]);
      den += w;
#pragma unroll
      for (int e = 0; e < 4; ++e) num[e] += w * (float)h[e];
    }
  }
  const float inv = 1.0f / den;
  u32x2_t w;
  w.x = pack_bf16x2(num[0] * inv, num[1] * inv);
  w.y = pack_bf16x2(num[2] * inv, num[3] * inv);
  *(u32x2_t*)(og + (size_t)r * D + 4 * c4) = w;
}

struct Plan {
  int nt, kh, row_blocks, n_splits;
};

// One tile of 16 query rows per wavefront, up to six tiles per workgroup; more rows are cut
// into row blocks (which re-read K and V, from L2: they run side by side on one die).  Two tiles per
// wavefront halve the LDS reads per row but measured slower (the per-block chain of a wavefront
// doubles and one workgroup per CU has nothing to cover it with: 162 against 138 us at B = 16,
// G = 4).
Plan make_plan(int B, int Hq, int Hkv, int T, int Lcap) {
  Plan p;
  const int R = (Hq / Hkv) * T;
  const int tiles = ceil_div(R, 16);
  p.row_blocks = ceil_div(tiles, 6);
  p.nt = ceil_div(tiles, p.row_blocks);
  p.row_blocks = ceil_div(tiles, p.nt);
  p.kh = 2;
  const int blocks = ceil_div(Lcap + T, kBlkKeys);
  const int base = B * Hkv * p.row_blocks;
  // One workgroup runs per CU.  A single sequence has splits of equal length: one round of at most
  // 256 workgroups (8192 keys, 32 heads: 8 splits 39.5 us, 6 41.6, 10 53.6, 16 47.3; 4096 keys: 8
  // splits 37.7 us, 6 39.7, 5 43.5, 10 52.3).  A batch that gives 160 workgroups by itself is not
  // split at all -- every split costs its start-up, a partial write and the merge launch, and the
  // ragged lengths even out over the CUs' queues (B = 4, 40 heads: 1/2/3/4 splits 39/42/42/47 us;
  // B = 16, 8 KV heads x 3 row blocks: 93/97/105/106) -- smaller batches up to one round.  At least four
  // key blocks per split: each split costs a partial write and read of about 80 keys' worth of bytes.
  int want = B == 1 ? 256 / base : (base >= 160 ? 1 : ceil_div(256, base));
  const int cap = blocks / 4 > 1 ? blocks / 4 : 1;
  want = want < 1 ? 1 : (want > cap ? cap : want);
  p.n_splits = ceil_div(blocks, ceil_div(blocks, want));
  return p;
}

// The kernel's LDS tiles exceed the 64 KB a kernel gets by default: raise the limit once per kernel and device.
template <int D, int NT, int KH, int WPT>
int launch_rows(const AttnArgs& a, hipStream_t stream) {
  static std::atomic<bool> raised[64];   // (set after the call succeeded; two threads racing here both make the same call)
  int dev = 0;
  MEDUSA_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return MEDUSA_EUNSUPPORTED;
  const size_t lds = (size_t)(KH == 1 ? 4 : 2) * 2 * KH * kBlkKeys * D * 2 + (size_t)NT * 16 * D * 2 + (size_t)16 * NT * 16;   // the ring of steps + the Q tiles + the rows' ancestor masks
  if (!raised[dev].load(std::memory_order_acquire)) {
    MEDUSA_HIP_TRY(hipFuncSetAttribute((const void*)tree_attn_rows_kernel<D, NT, KH, WPT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    raised[dev].store(true, std::memory_order_release);
  }
  const int units = a.B * a.Hkv * a.n_splits;
  const dim3 grid(8 * ceil_div(units, 8) * a.row_blocks), block(64 * NT * WPT);
  hipLaunchKernelGGL((tree_attn_rows_kernel<D, NT, KH, WPT>), grid, block, lds, stream, a);
  return MEDUSA_OK;
}

template <int D>
int launch_mfma(const AttnArgs& a, const Plan& p, hipStream_t stream) {
  int rc = MEDUSA_EUNSUPPORTED;
#define MEDUSA_ATTN(NT_) \
  case NT_: rc = p.kh == 2 ? launch_rows<D, NT_, 2, 2>(a, stream) : launch_rows<D, NT_, 1, 1>(a, stream); break
  switch (p.nt) {
    MEDUSA_ATTN(1); MEDUSA_ATTN(2); MEDUSA_ATTN(3); MEDUSA_ATTN(4); MEDUSA_ATTN(5); MEDUSA_ATTN(6);
    default: return MEDUSA_EUNSUPPORTED;
  }
#undef MEDUSA_ATTN
  if (rc != MEDUSA_OK) return rc;
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
                                     int B, int Hq, int Hkv, int D, int Lcap, float scale, int dtype,
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
                              int Hq, int Hkv, int D, int Lcap, float scale, int dtype, void* workspace,
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
  a.ranked = (long)B * Hkv * p.n_splits * p.row_blocks > 256 ? 1 : 0;   // (one round of workgroups starts all at once: nothing to order)
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
