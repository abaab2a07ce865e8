// tree_attention (Sec. 2.1.2 of the Medusa paper): soft-max attention of the T tree tokens over
// the cached prefix plus the tree itself, where a tree token sees only its own continuation
// (ancestors and itself).  The tree mask is one 128-bit word per query row.
//
// bf16 path: split-K flash-decoding on 16x16x32 bf16 MFMA.
//   * One workgroup = one (sequence, KV head, block of up to 80 query rows, split of the key
//     range).  All G = Hq/Hkv query heads that share the KV head are handled together: their
//     G*T rows are contiguous in q and out.
//   * The key range of a sequence is the list of 32-key blocks [prefix blocks ..., tree blocks
//     ...]; a split owns a contiguous run of blocks and its four wavefronts take blocks
//     round-robin.  Each wavefront is an independent online-soft-max worker: K is read from
//     HBM straight into MFMA operand layout, scores are formed transposed (S^T = K Q^T) so the
//     probabilities are already in the operand layout of the second product O^T = V^T P^T,
//     and only V passes through a private LDS tile to be read transposed.
//   * The wavefronts' partial (max, sum, O) are merged through LDS in a fixed order; splits
//     are merged by a second small kernel (skipped when there is a single split).
// fp32 path (and any D the MFMA path does not cover): one workgroup per query row, plain FMAs.
#include <math.h>

#include "common.hpp"

namespace {

constexpr int kBlkKeys = 32;

struct AttnArgs {
  const void *q, *k_tree, *v_tree, *k_cache, *v_cache;
  const int32_t* prefix_len;
  const TreeTables* tree;
  void* out;
  float* ws_o;       // [B*Hkv*n_splits][R][D] un-normalised partial outputs
  float* ws_ml;      // [B*Hkv*n_splits][R][2] (running max in log2 units, sum)
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
// l%16 and rows 4*(l/16)..+3 of C.  The reduction index may be permuted freely as long as A
// and B agree, which is what lets P^T be consumed where S^T was produced.
// ---------------------------------------------------------------------------------------
template <int D, int MT>
__global__ __launch_bounds__(256) void tree_attn_mfma_kernel(AttnArgs a) {
  constexpr int KS = D / 32;                  // reduction steps of K Q^T
  constexpr int DT = D / 16;                  // 16-wide tiles of the head dimension
  constexpr int VSTR = D + 8;                 // padded LDS row stride of the V tile (elements)
  constexpr int V_BYTES = 4 * kBlkKeys * VSTR * 2;
  constexpr int MERGE_BYTES = 2 * MT * DT * 64 * 16;
  constexpr int POOL = V_BYTES > MERGE_BYTES ? V_BYTES : MERGE_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char pool[POOL];
  __shared__ float s_m[4][16 * MT];
  __shared__ float s_l[2][16 * MT];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i16 = lane & 15, q4 = lane >> 4;
  const int split = blockIdx.x;
  const int kvh = blockIdx.y / a.row_blocks, rb = blockIdx.y - kvh * a.row_blocks;
  const int b = blockIdx.z;
  const int T = a.T, R = a.R;
  const int L = min(max(a.prefix_len[b], 0), a.Lcap);
  const int nblk_p = ceil_div(L, kBlkKeys), nblk = nblk_p + ceil_div(T, kBlkKeys);
  const int bps = ceil_div(nblk, a.n_splits);
  const int blk_lo = split * bps, blk_hi = min(nblk, blk_lo + bps);
  const int row0 = rb * 16 * MT;

  const uint16_t* qg = (const uint16_t*)a.q + ((size_t)b * a.Hq + (size_t)kvh * a.G) * T * D;
  const uint16_t* kc = (const uint16_t*)a.k_cache + ((size_t)b * a.Hkv + kvh) * a.Lcap * D;
  const uint16_t* vc = (const uint16_t*)a.v_cache + ((size_t)b * a.Hkv + kvh) * a.Lcap * D;
  const uint16_t* kt = (const uint16_t*)a.k_tree + ((size_t)b * a.Hkv + kvh) * T * D;
  const uint16_t* vt = (const uint16_t*)a.v_tree + ((size_t)b * a.Hkv + kvh) * T * D;

  // Q^T fragments (B operand): column = query row, reduction = head dimension.
  bf16x8_t qf[MT][KS];
  int tq[MT];                                  // tree node of this lane's query column
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int r = min(row0 + 16 * mt + i16, R - 1);
    tq[mt] = r % T;
#pragma unroll
    for (int c = 0; c < KS; ++c) qf[mt][c] = *(const bf16x8_t*)(qg + (size_t)r * D + 32 * c + 8 * q4);
  }

  floatx4_t o[MT][DT];
  float m_run[MT], l_run[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    m_run[mt] = -INFINITY;
    l_run[mt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[mt][dt] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  }
  const float sc = a.scale * 1.4426950408889634f;      // scores are kept in log2 units
  uint16_t* vt_lds = (uint16_t*)pool + wave * kBlkKeys * VSTR;

  for (int blk = blk_lo + wave; blk < blk_hi; blk += 4) {
    const bool is_tree = blk >= nblk_p;
    const int key0 = (is_tree ? blk - nblk_p : blk) * kBlkKeys;
    const int nvalid = is_tree ? T : L;
    const uint16_t* kbase = is_tree ? kt : kc;
    const uint16_t* vbase = is_tree ? vt : vc;

    // K fragments (A operand): row = key, reduction = head dimension.  Rows past the valid
    // range are redirected to the last valid row and masked below.
    bf16x8_t kf[2][KS];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int key = min(key0 + 16 * j + i16, nvalid - 1);
#pragma unroll
      for (int c = 0; c < KS; ++c) kf[j][c] = *(const bf16x8_t*)(kbase + (size_t)key * D + 32 * c + 8 * q4);
    }
    // V tile -> this wavefront's LDS region, row-major with padded stride.
    {
      constexpr int CPR = D / 8;               // 16-byte chunks per row
#pragma unroll
      for (int it = 0; it < kBlkKeys * CPR / 64; ++it) {
        const int id = it * 64 + lane;
        const int row = id / CPR, col = id - row * CPR;
        const int key = min(key0 + row, nvalid - 1);
        const u32x4_t v = *(const u32x4_t*)(vbase + (size_t)key * D + col * 8);
        *(u32x4_t*)(vt_lds + row * VSTR + col * 8) = v;
      }
    }

    // S^T tiles and the online soft-max, one 16-row query tile at a time.
    bf16x8_t pf[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      floatx4_t s[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        s[j] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < KS; ++c) s[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[j][c], qf[mt][c], s[j], 0, 0, 0);
      }
      // visibility of key (key0 + 16j + 4*q4 + r) for this lane's query column
      uint32_t vis;
      {
        const int left = nvalid - key0;        // >= 1
        vis = left >= 32 ? 0xffffffffu : ((1u << left) - 1u);
        if (is_tree) vis &= (uint32_t)(a.tree->anc_mask[tq[mt]][key0 >> 6] >> (key0 & 63));
      }
      float mx = -INFINITY;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const bool ok = (vis >> (16 * j + 4 * q4 + r)) & 1u;
          const float v = ok ? s[j][r] * sc : -INFINITY;
          s[j][r] = v;
          mx = fmaxf(mx, v);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
      mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
      const float m_new = fmaxf(m_run[mt], mx);
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = exp2f(m_run[mt] - m_safe);
      float psum = 0.f;
      float p[8];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          p[4 * j + r] = exp2f(s[j][r] - m_safe);
          psum += p[4 * j + r];
        }
      l_run[mt] = l_run[mt] * alpha + psum;
      m_run[mt] = m_new;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[mt][dt] *= alpha;
      // P^T fragment (B operand): reduction slot e <-> key 4*q4 + e (tile 0), 16 + 4*q4 + e - 4 (tile 1)
      u32x4_t packed;
      packed.x = pack_bf16x2(p[0], p[1]);
      packed.y = pack_bf16x2(p[2], p[3]);
      packed.z = pack_bf16x2(p[4], p[5]);
      packed.w = pack_bf16x2(p[6], p[7]);
      pf[mt] = __builtin_bit_cast(bf16x8_t, packed);
    }

    // O^T += V^T P^T.  A operand: row = head-dimension index, reduction slots as above.
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      uint16_t e[8];
#pragma unroll
      for (int x = 0; x < 8; ++x) {
        const int row = x < 4 ? 4 * q4 + x : 16 + 4 * q4 + (x - 4);
        e[x] = vt_lds[row * VSTR + 16 * dt + i16];
      }
      u32x4_t packed;
      packed.x = (uint32_t)e[0] | ((uint32_t)e[1] << 16);
      packed.y = (uint32_t)e[2] | ((uint32_t)e[3] << 16);
      packed.z = (uint32_t)e[4] | ((uint32_t)e[5] << 16);
      packed.w = (uint32_t)e[6] | ((uint32_t)e[7] << 16);
      const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, packed);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) o[mt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[mt], o[mt][dt], 0, 0, 0);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

  // ---- merge the four wavefronts (fixed order) -------------------------------------------
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    l_run[mt] += __shfl_xor(l_run[mt], 16, kWave);
    l_run[mt] += __shfl_xor(l_run[mt], 32, kWave);
    if (q4 == 0) s_m[wave][16 * mt + i16] = m_run[mt];
  }
  __syncthreads();                               // also: every wavefront is done with its V tile
  float m_all[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int c = 16 * mt + i16;
    const float mm = fmaxf(fmaxf(s_m[0][c], s_m[1][c]), fmaxf(s_m[2][c], s_m[3][c]));
    m_all[mt] = mm;
    const float w = exp2f(m_run[mt] - (mm == -INFINITY ? 0.f : mm));
    l_run[mt] *= w;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[mt][dt] *= w;
  }
  floatx4_t* mbuf = (floatx4_t*)pool;           // [2][MT*DT][64]
  // round 1: waves 2,3 -> LDS; waves 0,1 add.  round 2: wave 1 -> LDS; wave 0 adds.
  if (wave >= 2) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) mbuf[((wave - 2) * MT * DT + mt * DT + dt) * 64 + lane] = o[mt][dt];
      if (q4 == 0) s_l[wave - 2][16 * mt + i16] = l_run[mt];
    }
  }
  __syncthreads();
  if (wave < 2) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[mt][dt] += mbuf[(wave * MT * DT + mt * DT + dt) * 64 + lane];
      l_run[mt] += s_l[wave][16 * mt + i16];
    }
  }
  __syncthreads();
  if (wave == 1) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) mbuf[(mt * DT + dt) * 64 + lane] = o[mt][dt];
      if (q4 == 0) s_l[0][16 * mt + i16] = l_run[mt];
    }
  }
  __syncthreads();
  if (wave != 0) return;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[mt][dt] += mbuf[(mt * DT + dt) * 64 + lane];
    l_run[mt] += s_l[0][16 * mt + i16];
  }

  // ---- write: final output (single split) or the split's partial ----------------------------
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int r = row0 + 16 * mt + i16;
    if (r >= R) continue;
    if (a.n_splits == 1) {
      const float inv = 1.0f / l_run[mt];
      uint16_t* orow = (uint16_t*)a.out + ((size_t)b * a.Hq + (size_t)kvh * a.G) * T * D + (size_t)r * D;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        u32x2_t w;
        w.x = pack_bf16x2(o[mt][dt][0] * inv, o[mt][dt][1] * inv);
        w.y = pack_bf16x2(o[mt][dt][2] * inv, o[mt][dt][3] * inv);
        *(u32x2_t*)(orow + 16 * dt + 4 * q4) = w;
      }
    } else {
      const size_t unit = ((size_t)b * a.Hkv + kvh) * a.n_splits + split;
      float* prow = a.ws_o + (unit * R + r) * D;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) *(floatx4_t*)(prow + 16 * dt + 4 * q4) = o[mt][dt];
      if (q4 == 0) {
        a.ws_ml[(unit * R + r) * 2 + 0] = m_all[mt];
        a.ws_ml[(unit * R + r) * 2 + 1] = l_run[mt];
      }
    }
  }
}

// Merge the splits of one query row.  grid (R, Hkv, B), D threads.
template <int D>
__global__ __launch_bounds__(D) void tree_attn_combine_kernel(AttnArgs a) {
  const int r = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z, dcol = threadIdx.x;
  const size_t unit0 = ((size_t)b * a.Hkv + kvh) * a.n_splits;
  float mm = -INFINITY;
  for (int s = 0; s < a.n_splits; ++s) mm = fmaxf(mm, a.ws_ml[((unit0 + s) * a.R + r) * 2]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < a.n_splits; ++s) {
    const size_t row = (unit0 + s) * a.R + r;
    const float w = exp2f(a.ws_ml[row * 2] - mm);
    den += w * a.ws_ml[row * 2 + 1];
    num += w * a.ws_o[row * D + dcol];
  }
  uint16_t* orow = (uint16_t*)a.out + ((size_t)b * a.Hq + (size_t)kvh * a.G) * a.T * D + (size_t)r * D;
  orow[dcol] = (uint16_t)float_to_bf16_bits(num / den);
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
  const int blocks = ceil_div(Lcap, kBlkKeys) + ceil_div(T, kBlkKeys);
  const int base = B * Hkv * p.row_blocks;
  int want = ceil_div(384, base);
  const int cap = blocks / 8 > 1 ? blocks / 8 : 1;   // at least ~256 keys per split
  p.n_splits = want < 1 ? 1 : (want > cap ? cap : want);
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
    hipLaunchKernelGGL((tree_attn_combine_kernel<D>), dim3(a.R, a.Hkv, a.B), dim3(D), 0, stream, a);
    MEDUSA_LAUNCH_CHECK();
  }
  return MEDUSA_OK;
}

}  // namespace

extern "C" size_t tree_attention_workspace_bytes(int B, int Hq, int Hkv, int T, int D, int Lcap) {
  if (B < 1 || Hq < 1 || Hkv < 1 || T < 1 || D < 1 || Lcap < 1 || Hq % Hkv != 0) return 0;
  const Plan p = make_plan(B, Hq, Hkv, T, Lcap);
  const size_t R = (size_t)(Hq / Hkv) * T;
  const size_t bytes = (size_t)B * Hkv * p.n_splits * R * (D + 2) * sizeof(float);
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
  a.ws_o = (float*)workspace;
  a.ws_ml = a.ws_o + (size_t)B * Hkv * p.n_splits * a.R * D;
  if (dtype == MEDUSA_F32) {
    const dim3 grid(T, Hq, B), block(256);
    if (D == 64) hipLaunchKernelGGL((tree_attn_plain_kernel<float, 64>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((tree_attn_plain_kernel<float, 128>), grid, block, 0, stream, a);
    MEDUSA_LAUNCH_CHECK();
    return MEDUSA_OK;
  }
  return D == 64 ? launch_mfma<64>(a, p, stream) : launch_mfma<128>(a, p, stream);
}
