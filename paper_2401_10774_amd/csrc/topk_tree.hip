// medusa_topk_tree (Sec. 2.1.2 of the Medusa paper): per-head top-S_k token ids, the greedy
// root token, and the gather of both into the fixed candidate tree.
//
// Two launches.  Stage 1 scans the logits once: every (row, chunk) workgroup keeps per-lane
// sorted candidate lists in registers and merges them with wavefront max-reductions on a
// 64-bit (value, inverted id) key, so ties resolve to the lower token id everywhere.
// Stage 2 (one wavefront per sequence) merges the chunk winners, writes topk_ids and gathers
// tree_tokens / position_ids from the node tables.
#include "common.hpp"

namespace {

constexpr int kChunks = 8;          // workgroups per logits row in stage 1
constexpr int kMaxS = MEDUSA_MAX_TOPK;

// Insert key into a descending list of compile-time length S (registers only).
template <int S>
__device__ __forceinline__ void list_insert(uint64_t (&list)[S], uint64_t key) {
  if (key <= list[S - 1]) return;
#pragma unroll
  for (int i = 0; i < S; ++i) {
    const bool gt = key > list[i];
    const uint64_t hi = gt ? key : list[i];
    key = gt ? list[i] : key;
    list[i] = hi;
  }
}

// The wavefront's S largest keys, in descending order; entry r is left in `out[r]` on every
// lane.  Each lane contributes a descending list; the winner of a round pops its head.
template <int S>
__device__ __forceinline__ void wave_top(uint64_t (&list)[S], uint64_t (&out)[S]) {
#pragma unroll
  for (int r = 0; r < S; ++r) {
    const uint64_t best = wave_max_u64(list[0]);
    out[r] = best;
    if (list[0] == best && best != 0) {   // keys are unique (ids differ); 0 = empty slot
#pragma unroll
      for (int i = 0; i + 1 < S; ++i) list[i] = list[i + 1];
      list[S - 1] = 0;
    }
  }
}

// rows: [B*(K+1)] logits rows of length V; row index b*(K+1)+0 is the LM head, +k head k.
// part: [rows][kChunks][kMaxS] keys (0 = empty).
template <int S>
__global__ __launch_bounds__(256) void topk_stage1(const float* __restrict__ medusa_logits, const float* __restrict__ lm_logits,
                                                   int V, int K_heads, int K, uint64_t* __restrict__ part) {
  __shared__ uint64_t cand[4][S];
  const int row = blockIdx.y;                       // b*(K+1) + h
  const int b = row / (K + 1), h = row - b * (K + 1);
  const float* src = h == 0 ? lm_logits + (size_t)b * V : medusa_logits + ((size_t)b * K_heads + (h - 1)) * V;
  const int per = ceil_div(V, kChunks);
  const int lo = blockIdx.x * per, hi = min(V, lo + per);
  uint64_t list[S];
#pragma unroll
  for (int i = 0; i < S; ++i) list[i] = 0;
  for (int i = lo + threadIdx.x; i < hi; i += 256) list_insert<S>(list, rank_key(src[i], (uint32_t)i));
  uint64_t top[S];
  wave_top<S>(list, top);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < S; ++i) cand[wave][i] = top[i];
  }
  __syncthreads();
  if (wave == 0) {
    // 4*S <= 64 candidates, one per lane; S rounds of wavefront max
    uint64_t mine[1] = {lane < 4 * S ? cand[lane / S][lane % S] : 0};
    uint64_t* dst = part + ((size_t)row * kChunks + blockIdx.x) * kMaxS;
#pragma unroll
    for (int r = 0; r < S; ++r) {
      const uint64_t best = wave_max_u64(mine[0]);
      if (mine[0] == best) mine[0] = 0;
      if (lane == 0) dst[r] = best;
    }
    if (lane == 0)
      for (int r = S; r < kMaxS; ++r) dst[r] = 0;
  }
}

// One wavefront per sequence.
__global__ __launch_bounds__(64) void topk_stage2(const uint64_t* __restrict__ part, const TreeTables* __restrict__ tree,
                                                  const int32_t* __restrict__ prefix_len, int32_t* __restrict__ topk_ids,
                                                  int32_t* __restrict__ tree_tokens, int32_t* __restrict__ position_ids) {
  __shared__ int32_t flat[1 + MEDUSA_MAX_HEADS * kMaxS];
  const int b = blockIdx.x, lane = threadIdx.x;
  const int K = tree->K, S = tree->S, T = tree->T;
  for (int h = 0; h <= K; ++h) {
    const int want = h == 0 ? 1 : tree->topk_per_head[h - 1];
    const uint64_t* src = part + ((size_t)b * (K + 1) + h) * kChunks * kMaxS;
    // kChunks*kMaxS = 128 candidates: two per lane
    uint64_t c0 = src[lane], c1 = src[lane + 64];
    for (int r = 0; r < want; ++r) {
      const uint64_t mx = c0 > c1 ? c0 : c1;
      const uint64_t best = wave_max_u64(mx);
      if (c0 == best) c0 = 0;
      else if (c1 == best) c1 = 0;
      if (lane == 0) {
        const int32_t id = (int32_t)rank_key_id(best);
        if (h == 0) flat[0] = id;
        else {
          flat[tree->head_base[h - 1] + r] = id;
          topk_ids[((size_t)b * K + (h - 1)) * S + r] = id;
        }
      }
    }
    if (h > 0 && lane == 0)
      for (int r = want; r < S; ++r) topk_ids[((size_t)b * K + (h - 1)) * S + r] = -1;
  }
  __syncthreads();
  const int L = prefix_len[b];
  for (int t = lane; t < T; t += 64) {
    tree_tokens[(size_t)b * T + t] = flat[tree->token_src[t]];
    position_ids[(size_t)b * T + t] = L + tree->depth[t];
  }
}

}  // namespace

extern "C" size_t medusa_topk_tree_workspace_bytes(int B, int K) {
  if (B < 1 || K < 0) return 0;
  return (size_t)B * (K + 1) * kChunks * kMaxS * sizeof(uint64_t);
}

extern "C" int medusa_topk_tree(const float* medusa_logits, const float* lm_logits, const medusa_tree_t* tree,
                                const int32_t* prefix_len, int B, int V, int K_heads, int32_t* topk_ids,
                                int32_t* tree_tokens, int32_t* position_ids, void* workspace, size_t workspace_bytes,
                                medusa_stream_t stream_) {
  if (!tree || !lm_logits || !prefix_len || !tree_tokens || !position_ids) return MEDUSA_EINVAL;
  const int K = tree->host.K, S = tree->host.S;
  if (K > 0 && (!medusa_logits || !topk_ids)) return MEDUSA_EINVAL;
  if (B < 1 || V < 1 || K_heads < K) return MEDUSA_EINVAL;
  if (S > V) return MEDUSA_EINVAL;
  if (!tree->dev) return MEDUSA_EHIP;
  if (!workspace || workspace_bytes < medusa_topk_tree_workspace_bytes(B, K)) return MEDUSA_EWORKSPACE;
  hipStream_t stream = (hipStream_t)stream_;
  uint64_t* part = (uint64_t*)workspace;
  const dim3 grid(kChunks, B * (K + 1));
  const int Sc = S <= 1 ? 1 : (S <= 2 ? 2 : (S <= 4 ? 4 : (S <= 8 ? 8 : 16)));
  switch (Sc) {
    case 1: hipLaunchKernelGGL(topk_stage1<1>, grid, dim3(256), 0, stream, medusa_logits, lm_logits, V, K_heads, K, part); break;
    case 2: hipLaunchKernelGGL(topk_stage1<2>, grid, dim3(256), 0, stream, medusa_logits, lm_logits, V, K_heads, K, part); break;
    case 4: hipLaunchKernelGGL(topk_stage1<4>, grid, dim3(256), 0, stream, medusa_logits, lm_logits, V, K_heads, K, part); break;
    case 8: hipLaunchKernelGGL(topk_stage1<8>, grid, dim3(256), 0, stream, medusa_logits, lm_logits, V, K_heads, K, part); break;
    default: hipLaunchKernelGGL(topk_stage1<16>, grid, dim3(256), 0, stream, medusa_logits, lm_logits, V, K_heads, K, part); break;
  }
  MEDUSA_LAUNCH_CHECK();
  hipLaunchKernelGGL(topk_stage2, dim3(B), dim3(64), 0, stream, part, tree->dev, prefix_len, topk_ids, tree_tokens,
                     position_ids);
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}
