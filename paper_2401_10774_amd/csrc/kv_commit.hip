// kv_commit (Fig. 1 of the Medusa paper: the accepted prefix is the next step's context):
// append the accepted path's tree K/V rows to every layer of the cache, then grow prefix_len.
// Pure index arithmetic and 16-byte copies: bit-exact by construction.  One launch: every
// workgroup reads the old prefix_len before it takes a ticket, and the workgroup that draws the
// last ticket writes the new lengths (in place, or to a second array) once all others are done.
#include "common.hpp"

namespace {

// Ticket counter of the "last workgroup" election; zero between launches.  Shared by all calls
// on a GPU: calls that overlap on different streams would race.
__device__ unsigned int g_commit_ticket;

// grid (NL*B), 256 threads.  One workgroup moves the <= K+1 accepted rows of all KV heads of one
// (layer, sequence), K and V.  Few, fat workgroups keep the number of tickets small.
__global__ __launch_bounds__(256) void kv_commit_kernel(u32x4_t* __restrict__ k_cache, u32x4_t* __restrict__ v_cache,
                                                        const u32x4_t* __restrict__ k_tree, const u32x4_t* __restrict__ v_tree,
                                                        const int32_t* __restrict__ path_nodes, int path_stride,
                                                        const int32_t* __restrict__ accept_len,
                                                        const int32_t* prefix_len, int32_t* prefix_len_out, int B,
                                                        int Hkv, int T, int Lcap, int vec_per_row) {
  const int lb = blockIdx.x;                  // l*B + b
  const int b = lb % B;
  const int a = min(max(accept_len[b], 0), path_stride);
  const int L = prefix_len[b];
  const int per_head = a * vec_per_row;       // 16-byte chunks per head and tensor
  const int total = 2 * Hkv * per_head;
  for (int i = threadIdx.x; i < total; i += 256) {
    const int which = i >= Hkv * per_head;
    int rem = i - which * Hkv * per_head;
    const int h = rem / per_head;
    rem -= h * per_head;
    const int j = rem / vec_per_row, c = rem - j * vec_per_row;
    const int node = path_nodes[(size_t)b * path_stride + j];
    const int dst = L + j;
    if (node < 0 || node >= T || dst < 0 || dst >= Lcap) continue;
    const size_t lbh = (size_t)lb * Hkv + h;
    const size_t src_i = (lbh * T + node) * vec_per_row + c;
    const size_t dst_i = (lbh * Lcap + dst) * vec_per_row + c;
    if (which) v_cache[dst_i] = v_tree[src_i];
    else k_cache[dst_i] = k_tree[src_i];
  }
  if (!last_workgroup_of(&g_commit_ticket, gridDim.x)) return;
  for (int bb = threadIdx.x; bb < B; bb += 256) {
    const int aa = min(max(accept_len[bb], 0), path_stride);
    prefix_len_out[bb] = min(max(prefix_len[bb], 0) + aa, Lcap);
  }
}

}  // namespace

extern "C" int kv_commit(void* k_cache, void* v_cache, const void* k_tree, const void* v_tree, const int32_t* path_nodes,
                         int path_stride, const int32_t* accept_len, int32_t* prefix_len, int32_t* prefix_len_out, int NL,
                         int B, int Hkv, int T, int D, int Lcap, medusa_dtype_t dtype, medusa_stream_t stream_) {
  if (!k_cache || !v_cache || !k_tree || !v_tree || !path_nodes || !accept_len || !prefix_len) return MEDUSA_EINVAL;
  if (NL < 1 || B < 1 || Hkv < 1 || T < 1 || D < 1 || Lcap < 1 || path_stride < 1) return MEDUSA_EINVAL;
  if (dtype != MEDUSA_F32 && dtype != MEDUSA_BF16) return MEDUSA_EINVAL;
  const size_t row_bytes = (size_t)D * (dtype == MEDUSA_F32 ? 4 : 2);
  if (row_bytes % 16 != 0) return MEDUSA_EUNSUPPORTED;
  if ((size_t)NL * B > 0x7fffffffu) return MEDUSA_EUNSUPPORTED;
  hipStream_t stream = (hipStream_t)stream_;
  hipLaunchKernelGGL(kv_commit_kernel, dim3(NL * B), dim3(256), 0, stream, (u32x4_t*)k_cache, (u32x4_t*)v_cache,
                     (const u32x4_t*)k_tree, (const u32x4_t*)v_tree, path_nodes, path_stride, accept_len, prefix_len,
                     prefix_len_out ? prefix_len_out : prefix_len, B, Hkv, T, Lcap, (int)(row_bytes / 16));
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}
