// medusa_topk_tree (Sec. 2.1.2 of the Medusa paper): per-head top-S_k token ids, the greedy
// root token, and the gather of both into the fixed candidate tree.
//
// One launch.  Every (row, chunk) workgroup scans its slice of one logits row once: each lane
// keeps a sorted candidate list in registers, lists are merged with wavefront max-reductions on
// a 64-bit (value, inverted id) key, so ties resolve to the lower token id everywhere.  The last
// workgroup of a sequence to finish (ticket counter) merges the chunk winners of that
// sequence's K+1 rows, writes topk_ids and gathers tree_tokens / position_ids from the node
// tables.
#include "common.hpp"

namespace {

constexpr int kMaxChunks = 16;      // upper bound of workgroups per logits row (sizes the partial buffer)
constexpr int kMaxS = MEDUSA_MAX_TOPK;
constexpr int kMaxBatch = 4096;

// Ticket counters of the "last workgroup of a sequence" election, per stream slot; zero between launches.
__device__ unsigned int g_topk_ticket[kTicketSlots][kMaxBatch];

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

// rows: [B*(K+1)] logits rows of length V; row index b*(K+1)+0 is the LM head, +h head h.
// part: [rows][kMaxChunks][S] keys (0 = empty).  grid (chunks, B*(K+1)), 256 threads.
template <int S>
__global__ __launch_bounds__(256) void topk_tree_kernel(const float* __restrict__ medusa_logits,
                                                        const float* __restrict__ lm_logits, int V, int K_heads,
                                                        uint64_t* __restrict__ part, const TreeTables* __restrict__ tree,
                                                        const int32_t* __restrict__ prefix_len,
                                                        int32_t* __restrict__ topk_ids, int32_t* __restrict__ tree_tokens,
                                                        int32_t* __restrict__ position_ids, int K, int slot) {
  __shared__ uint64_t cand[4][S];
  __shared__ int32_t flat[1 + MEDUSA_MAX_HEADS * kMaxS];
  const int chunks = gridDim.x;                     // (K = tree->K comes as an argument: the row decode below needs it at once)
  const int row = blockIdx.y;                       // b*(K+1) + h
  const int b = row / (K + 1), h = row - b * (K + 1);
  const float* src = h == 0 ? lm_logits + (size_t)b * V : medusa_logits + ((size_t)b * K_heads + (h - 1)) * V;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint64_t list[S];
#pragma unroll
  for (int i = 0; i < S; ++i) list[i] = 0;
  if ((V & 3) == 0) {                               // rows are 16-byte aligned: four logits per load
    const int per = ceil_div(V >> 2, chunks);
    const int lo = blockIdx.x * per, hi = min(V >> 2, lo + per);
    const floatx4_t* src4 = (const floatx4_t*)src;
    // independent 16-byte loads first, the (branchy) insertions after
    for (int i0 = lo + threadIdx.x; i0 < hi; i0 += 2 * 256) {
      floatx4_t v[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) v[u] = src4[min(i0 + u * 256, hi - 1)];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int i = i0 + u * 256;
        if (i < hi) {
#pragma unroll
          for (int e = 0; e < 4; ++e) list_insert<S>(list, rank_key(v[u][e], (uint32_t)(4 * i + e)));
        }
      }
    }
  } else {
    const int per = ceil_div(V, chunks);
    const int lo = blockIdx.x * per, hi = min(V, lo + per);
    for (int i = lo + threadIdx.x; i < hi; i += 256) list_insert<S>(list, rank_key(src[i], (uint32_t)i));
  }
  uint64_t top[S];
  wave_top<S>(list, top);
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < S; ++i) cand[wave][i] = top[i];
  }
  __syncthreads();
  if (wave == 0) {
    // 4*S <= 64 candidates, one per lane; S rounds of wavefront max
    uint64_t mine = lane < 4 * S ? cand[lane / S][lane % S] : 0;
    uint64_t* dst = part + ((size_t)row * kMaxChunks + blockIdx.x) * S;
#pragma unroll
    for (int r = 0; r < S; ++r) {
      const uint64_t best = wave_max_u64(mine);
      if (mine == best) mine = 0;
      if (lane == 0) store_agent(dst + r, best);
    }
  }

  // ---- the sequence's last workgroup merges the chunk winners and fills the tree ------------
  if (!last_workgroup_of(&g_topk_ticket[slot][b], (unsigned)(chunks * (K + 1)))) return;
  // Everything needed from memory is requested before the first use: the tree-table entries of this
  // thread's node, the prefix length, and the chunk winners of the rows this wavefront merges
  // (row hh goes to wavefront hh % 4), so that the merge costs one round trip, not one per row.
  const int Smax = tree->S, T = tree->T;
  const int L = prefix_len[b];
  constexpr int TPT = (MEDUSA_MAX_TREE_TOKENS + 255) / 256;          // tree nodes per thread
  int my_src[TPT], my_depth[TPT];
#pragma unroll
  for (int u = 0; u < TPT; ++u) {
    const int t = threadIdx.x + u * 256;
    my_src[u] = t < T ? tree->token_src[t] : 0;
    my_depth[u] = t < T ? tree->depth[t] : 0;
  }
  constexpr int PER_LANE = (kMaxChunks * S + 63) / 64;
  constexpr int RPW = (MEDUSA_MAX_HEADS + 1 + 3) / 4;                // rows per wavefront
  uint64_t c[RPW][PER_LANE];
  int want[RPW], base[RPW];
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    const int hh = wave + 4 * q;
    want[q] = hh > K ? 0 : (hh == 0 ? 1 : tree->topk_per_head[hh - 1]);
    base[q] = hh > K || hh == 0 ? 0 : tree->head_base[hh - 1];
    const uint64_t* p = part + ((size_t)b * (K + 1) + min(hh, K)) * kMaxChunks * S;
#pragma unroll
    for (int j = 0; j < PER_LANE; ++j) c[q][j] = hh <= K && j * 64 + lane < chunks * S ? load_agent(p + j * 64 + lane) : 0;
  }
#pragma unroll
  for (int q = 0; q < RPW; ++q) {
    const int hh = wave + 4 * q;
    if (hh > K) break;
    for (int r = 0; r < want[q]; ++r) {
      uint64_t mx = c[q][0];
#pragma unroll
      for (int j = 1; j < PER_LANE; ++j) mx = c[q][j] > mx ? c[q][j] : mx;
      const uint64_t best = wave_max_u64(mx);
      bool done = false;                              // keys are unique: exactly one slot matches
#pragma unroll
      for (int j = 0; j < PER_LANE; ++j) {
        if (!done && c[q][j] == best) { c[q][j] = 0; done = true; }
      }
      if (lane == 0) {
        const int32_t id = (int32_t)rank_key_id(best);
        if (hh == 0) flat[0] = id;
        else {
          flat[base[q] + r] = id;
          topk_ids[((size_t)b * K + (hh - 1)) * Smax + r] = id;
        }
      }
    }
    if (hh > 0 && lane == 0)
      for (int r = want[q]; r < Smax; ++r) topk_ids[((size_t)b * K + (hh - 1)) * Smax + r] = -1;
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < TPT; ++u) {
    const int t = threadIdx.x + u * 256;
    if (t < T) {
      tree_tokens[(size_t)b * T + t] = flat[my_src[u]];
      position_ids[(size_t)b * T + t] = L + my_depth[u];
    }
  }
}

}  // namespace

extern "C" size_t medusa_topk_tree_workspace_bytes(int B, int K) {
  if (B < 1 || K < 0) return 0;
  return (size_t)B * (K + 1) * kMaxChunks * kMaxS * sizeof(uint64_t);
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
  if (B > kMaxBatch) return MEDUSA_EUNSUPPORTED;
  if (!tree->dev) return MEDUSA_EHIP;
  if (!workspace || workspace_bytes < medusa_topk_tree_workspace_bytes(B, K) || ((uintptr_t)workspace & 7) != 0)
    return MEDUSA_EWORKSPACE;
  hipStream_t stream = (hipStream_t)stream_;
  uint64_t* part = (uint64_t*)workspace;
  // every workgroup ends with a ticket round trip: aim at about two workgroups per CU (80 rows of
  // 32000 logits: 17.8 / 14.1 / 12.6 / 11.8 / 12.4 us with 2 / 3 / 4 / 6 / 8 workgroups per row)
  int chunks = 512 / (B * (K + 1));
  chunks = chunks < 1 ? 1 : (chunks > kMaxChunks ? kMaxChunks : chunks);
  const dim3 grid(chunks, B * (K + 1)), block(256);
  const int Sc = S <= 1 ? 1 : (S <= 2 ? 2 : (S <= 4 ? 4 : (S <= 8 ? 8 : 16)));
#define MEDUSA_TOPK(S_)                                                                                         \
  hipLaunchKernelGGL(topk_tree_kernel<S_>, grid, block, 0, stream, medusa_logits, lm_logits, V, K_heads, part, \
                     tree->dev, prefix_len, topk_ids, tree_tokens, position_ids, K, ticket_slot(stream))
  switch (Sc) {
    case 1: MEDUSA_TOPK(1); break;
    case 2: MEDUSA_TOPK(2); break;
    case 4: MEDUSA_TOPK(4); break;
    case 8: MEDUSA_TOPK(8); break;
    default: MEDUSA_TOPK(16); break;
  }
#undef MEDUSA_TOPK
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}
