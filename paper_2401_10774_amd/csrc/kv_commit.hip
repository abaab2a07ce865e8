// kv_commit (Fig. 1 of the Medusa paper: the accepted prefix is the next step's context):
// append the accepted path's tree K/V rows to every layer of the cache, then grow prefix_len.
// Pure index arithmetic and 16-byte copies: bit-exact by construction.
#include "common.hpp"

namespace {

// grid (NL*B*Hkv), 256 threads.  One workgroup moves the <= K+1 accepted rows of one
// (layer, sequence, KV head) for both K and V.
__global__ __launch_bounds__(256) void kv_commit_kernel(u32x4_t* __restrict__ k_cache, u32x4_t* __restrict__ v_cache,
                                                        const u32x4_t* __restrict__ k_tree, const u32x4_t* __restrict__ v_tree,
                                                        const int32_t* __restrict__ path_nodes, int path_stride,
                                                        const int32_t* __restrict__ accept_len,
                                                        const int32_t* __restrict__ prefix_len, int B, int Hkv, int T,
                                                        int Lcap, int vec_per_row) {
  const int lbh = blockIdx.x;                 // (l*B + b)*Hkv + h
  const int b = (lbh / Hkv) % B;
  const int a = min(max(accept_len[b], 0), path_stride);
  const int L = prefix_len[b];
  const size_t cache_base = (size_t)lbh * Lcap * vec_per_row;
  const size_t tree_base = (size_t)lbh * T * vec_per_row;
  const int per_tensor = a * vec_per_row;
  for (int i = threadIdx.x; i < 2 * per_tensor; i += 256) {
    const int which = i >= per_tensor;
    const int rem = i - which * per_tensor;
    const int j = rem / vec_per_row, c = rem - j * vec_per_row;
    const int node = path_nodes[(size_t)b * path_stride + j];
    const int dst = L + j;
    if (node < 0 || node >= T || dst < 0 || dst >= Lcap) continue;
    const size_t src_i = tree_base + (size_t)node * vec_per_row + c;
    const size_t dst_i = cache_base + (size_t)dst * vec_per_row + c;
    if (which) v_cache[dst_i] = v_tree[src_i];
    else k_cache[dst_i] = k_tree[src_i];
  }
}

__global__ void prefix_advance_kernel(int32_t* __restrict__ prefix_len, const int32_t* __restrict__ accept_len, int B,
                                      int path_stride, int Lcap) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) {
    const int a = min(max(accept_len[b], 0), path_stride);
    prefix_len[b] = min(max(prefix_len[b], 0) + a, Lcap);
  }
}

}  // namespace

extern "C" int kv_commit(void* k_cache, void* v_cache, const void* k_tree, const void* v_tree, const int32_t* path_nodes,
                         int path_stride, const int32_t* accept_len, int32_t* prefix_len, int NL, int B, int Hkv, int T,
                         int D, int Lcap, medusa_dtype_t dtype, medusa_stream_t stream_) {
  if (!k_cache || !v_cache || !k_tree || !v_tree || !path_nodes || !accept_len || !prefix_len) return MEDUSA_EINVAL;
  if (NL < 1 || B < 1 || Hkv < 1 || T < 1 || D < 1 || Lcap < 1 || path_stride < 1) return MEDUSA_EINVAL;
  if (dtype != MEDUSA_F32 && dtype != MEDUSA_BF16) return MEDUSA_EINVAL;
  const size_t row_bytes = (size_t)D * (dtype == MEDUSA_F32 ? 4 : 2);
  if (row_bytes % 16 != 0) return MEDUSA_EUNSUPPORTED;
  if ((size_t)NL * B * Hkv > 0x7fffffffu) return MEDUSA_EUNSUPPORTED;
  hipStream_t stream = (hipStream_t)stream_;
  hipLaunchKernelGGL(kv_commit_kernel, dim3(NL * B * Hkv), dim3(256), 0, stream, (u32x4_t*)k_cache, (u32x4_t*)v_cache,
                     (const u32x4_t*)k_tree, (const u32x4_t*)v_tree, path_nodes, path_stride, accept_len, prefix_len, B,
                     Hkv, T, Lcap, (int)(row_bytes / 16));
  MEDUSA_LAUNCH_CHECK();
  hipLaunchKernelGGL(prefix_advance_kernel, dim3(ceil_div(B, 256)), dim3(256), 0, stream, prefix_len, accept_len, B,
                     path_stride, Lcap);
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}
