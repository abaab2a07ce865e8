// kv_commit (Fig. 1 of the Medusa paper: the accepted prefix is the next step's context):
// append the accepted path's tree K/V rows to every layer of the cache, then grow prefix_len.
// Pure index arithmetic and 16-byte copies: bit-exact by construction.  One launch, one workgroup
// per (layer, sequence, path slot), so that a long accepted path costs no more time than a short
// one.  Every workgroup reads the old prefix_len.  In place, each takes a ticket afterwards and
// the workgroup that draws the last one writes the new lengths, once all others are done with the
// old ones; with a second array for the new lengths nobody has to wait: workgroup (0, 0) writes them.
#include "common.hpp"

namespace {

// Ticket counter of the "last workgroup" election, per stream slot; zero between launches.
__device__ unsigned int g_commit_ticket[kTicketSlots];

// grid (NL*B, path_stride), 256 threads.  One workgroup moves one accepted row (path slot) of all KV
// heads of one (layer, sequence), K and V; workgroups of slots beyond accept_len have nothing to move.
__global__ __launch_bounds__(256) void kv_commit_kernel(u32x4_t* __restrict__ k_cache, u32x4_t* __restrict__ v_cache,
                                                        const u32x4_t* __restrict__ k_tree, const u32x4_t* __restrict__ v_tree,
                                                        const int32_t* __restrict__ path_nodes, int path_stride,
                                                        const int32_t* __restrict__ accept_len,
                                                        const int32_t* prefix_len, int32_t* prefix_len_out, int B,
                                                        int Hkv, int T, int Lcap, int vec_per_row, int in_place, int slot) {
  const int lb = blockIdx.x;                  // l*B + b
  const int j = blockIdx.y;                   // path slot
  const int b = lb % B;
  // the three small loads do not depend on each other: they go out together
  const int a = min(max(accept_len[b], 0), path_stride);
  const int L = prefix_len[b];
  const int node = path_nodes[(size_t)b * path_stride + j];
  const int dst = L + j;
  if (j < a && node >= 0 && node < T && dst >= 0 && dst < Lcap) {
    // Work item i: tensor (K, V), head, 16-byte chunk.  Four items per thread and round, so that
    // their row loads are in flight together.
    const int per_head = vec_per_row, total = 2 * Hkv * per_head;
    for (int base = 0; base < total; base += 4 * 256) {
      size_t src_i[4], dst_i[4];
      bool ok[4], which[4];
      u32x4_t val[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = base + u * 256 + threadIdx.x;
        int rem = min(i, total - 1);
        which[u] = rem >= Hkv * per_head;
        rem -= which[u] * Hkv * per_head;
        const int h = rem / per_head, c = rem - h * per_head;
        ok[u] = i < total;
        const size_t lbh = (size_t)lb * Hkv + h;
        src_i[u] = (lbh * T + node) * vec_per_row + c;
        dst_i[u] = (lbh * Lcap + dst) * vec_per_row + c;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (ok[u]) val[u] = which[u] ? v_tree[src_i[u]] : k_tree[src_i[u]];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (ok[u]) (which[u] ? v_cache : k_cache)[dst_i[u]] = val[u];
    }
  }
  if (in_place ? !last_workgroup_of(&g_commit_ticket[slot], gridDim.x * gridDim.y) : (blockIdx.x | blockIdx.y) != 0) return;
  for (int bb = threadIdx.x; bb < B; bb += 256) {
    const int aa = min(max(accept_len[bb], 0), path_stride);
    prefix_len_out[bb] = min(max(prefix_len[bb], 0) + aa, Lcap);
  }
}

// grid (chunks, B), 256 threads: copies 4-byte words of the row selected by best_node[b] (clamped to
// the tree) from `src` [B, T, words] to `dst` [B, words]; blockIdx.z picks the (src, dst) pair.
__global__ __launch_bounds__(256) void carry_over_kernel(const uint32_t* __restrict__ src0, uint32_t* __restrict__ dst0,
                                                         int words0, const uint32_t* __restrict__ src1,
                                                         uint32_t* __restrict__ dst1, int words1,
                                                         const int32_t* __restrict__ best_node, int T) {
  const int b = blockIdx.y;
  const uint32_t* src = blockIdx.z ? src1 : src0;
  uint32_t* dst = blockIdx.z ? dst1 : dst0;
  const int words = blockIdx.z ? words1 : words0;
  if (!src || !dst) return;
  const int node = min(max(best_node[b], 0), T - 1);
  const uint32_t* row = src + ((size_t)b * T + node) * words;
  for (int i = blockIdx.x * 256 + threadIdx.x; i < words; i += gridDim.x * 256) dst[(size_t)b * words + i] = row[i];
}

}  // namespace

extern "C" int medusa_carry_over(const void* hidden_tree, const float* verify_logits, const int32_t* best_node,
                                 void* h_next, float* lm_next, int B, int T, int d, int V, int dtype,
                                 medusa_stream_t stream_) {
  if (!best_node || (!hidden_tree != !h_next) || (!verify_logits != !lm_next) || (!h_next && !lm_next)) return MEDUSA_EINVAL;
  if (B < 1 || T < 1 || (h_next && d < 1) || (lm_next && V < 1)) return MEDUSA_EINVAL;
  if (dtype != MEDUSA_F32 && dtype != MEDUSA_BF16) return MEDUSA_EINVAL;
  if (h_next && dtype == MEDUSA_BF16 && d % 2 != 0) return MEDUSA_EUNSUPPORTED;
  if (B > 65535) return MEDUSA_EUNSUPPORTED;
  const int words_h = h_next ? (dtype == MEDUSA_BF16 ? d / 2 : d) : 0, words_l = lm_next ? V : 0;
  const int longest = words_h > words_l ? words_h : words_l;
  int chunks = ceil_div(longest, 1024);
  chunks = chunks > 64 ? 64 : chunks;
  hipLaunchKernelGGL(carry_over_kernel, dim3(chunks, B, 2), dim3(256), 0, (hipStream_t)stream_, (const uint32_t*)hidden_tree,
                     (uint32_t*)h_next, words_h, (const uint32_t*)verify_logits, (uint32_t*)lm_next, words_l, best_node, T);
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}

extern "C" int kv_commit(void* k_cache, void* v_cache, const void* k_tree, const void* v_tree, const int32_t* path_nodes,
                         int path_stride, const int32_t* accept_len, int32_t* prefix_len, int32_t* prefix_len_out, int NL,
                         int B, int Hkv, int T, int D, int Lcap, int dtype, medusa_stream_t stream_) {
  if (!k_cache || !v_cache || !k_tree || !v_tree || !path_nodes || !accept_len || !prefix_len) return MEDUSA_EINVAL;
  if (NL < 1 || B < 1 || Hkv < 1 || T < 1 || D < 1 || Lcap < 1 || path_stride < 1) return MEDUSA_EINVAL;
  if (dtype != MEDUSA_F32 && dtype != MEDUSA_BF16) return MEDUSA_EINVAL;
  const size_t row_bytes = (size_t)D * (dtype == MEDUSA_F32 ? 4 : 2);
  if (row_bytes % 16 != 0) return MEDUSA_EUNSUPPORTED;
  if ((size_t)NL * B > 0x7fffffffu || path_stride > 65535) return MEDUSA_EUNSUPPORTED;
  hipStream_t stream = (hipStream_t)stream_;
  hipLaunchKernelGGL(kv_commit_kernel, dim3(NL * B, path_stride), dim3(256), 0, stream, (u32x4_t*)k_cache, (u32x4_t*)v_cache,
                     (const u32x4_t*)k_tree, (const u32x4_t*)v_tree, path_nodes, path_stride, accept_len, prefix_len,
                     prefix_len_out ? prefix_len_out : prefix_len, B, Hkv, T, Lcap, (int)(row_bytes / 16),
                     (int)(!prefix_len_out || prefix_len_out == prefix_len), ticket_slot(stream));
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}
