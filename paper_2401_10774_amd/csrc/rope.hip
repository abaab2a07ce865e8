// tree_rope: rotary position embedding of the tree tokens' queries and keys at the tree's
// positional indices (Sec. 2.1.2: position = prefix length + depth of the node; the indices are
// the position_ids table medusa_topk_tree emits).  Half-split pairing of the Llama family: element
// j < D/2 and element j + D/2 form a pair, rotated by position * theta^(-2j/D).
//
// The tensors are tiny (B x heads x T x D elements), so this is a latency-bound kernel: one
// wavefront per (sequence, head, token) row, in place.  Angles are formed and reduced in double
// precision: at positions in the thousands a float angle would cost 3-4 decimal digits of the
// rotation.
#include "common.hpp"

namespace {

struct RopeArgs {
  void* q;                    // [B][Hq][T][D]
  void* k;                    // [B][Hkv][T][D]
  const int32_t* position_ids;  // [B][T]
  int B, Hq, Hkv, T, D;
  double neg_log2_theta_2_over_d;   // -(2/D) * log2(theta)
};

template <typename E>
__global__ __launch_bounds__(256) void tree_rope_kernel(RopeArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long rows_q = (long)a.B * a.Hq * a.T, rows = rows_q + (long)a.B * a.Hkv * a.T;
  const long row = (long)blockIdx.x * 4 + wave;
  if (row >= rows) return;
  const bool is_q = row < rows_q;
  const long r = is_q ? row : row - rows_q;
  const int H = is_q ? a.Hq : a.Hkv;
  const int t = (int)(r % a.T);
  const int b = (int)(r / ((long)H * a.T));
  E* x = (E*)(is_q ? a.q : a.k) + r * a.D;
  const double pos = (double)a.position_ids[(long)b * a.T + t];
  const int half = a.D >> 1;
  for (int j = lane; j < half; j += 64) {
    const double ang = pos * exp2((double)j * a.neg_log2_theta_2_over_d);
    double s, c;
    sincos(ang, &s, &c);
    const double lo = (double)load_as_float<E>(x + j), hi = (double)load_as_float<E>(x + j + half);
    store_from_float<E>(x + j, (float)(lo * c - hi * s));
    store_from_float<E>(x + j + half, (float)(hi * c + lo * s));
  }
}

}  // namespace

extern "C" int tree_rope(void* q, void* k, const int32_t* position_ids, int B, int Hq, int Hkv, int T, int D, float theta,
                         medusa_dtype_t dtype, medusa_stream_t stream_) {
  if (!q || !k || !position_ids) return MEDUSA_EINVAL;
  if (B < 1 || Hq < 1 || Hkv < 1 || T < 1 || D < 2 || (D & 1) || !(theta > 0.f)) return MEDUSA_EINVAL;
  if (dtype != MEDUSA_F32 && dtype != MEDUSA_BF16) return MEDUSA_EINVAL;
  RopeArgs a;
  a.q = q;
  a.k = k;
  a.position_ids = position_ids;
  a.B = B;
  a.Hq = Hq;
  a.Hkv = Hkv;
  a.T = T;
  a.D = D;
  a.neg_log2_theta_2_over_d = -(2.0 / D) * log2((double)theta);
  const long rows = (long)B * (Hq + Hkv) * T;
  if (rows > ((long)1 << 30)) return MEDUSA_EUNSUPPORTED;
  const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
  hipStream_t stream = (hipStream_t)stream_;
  if (dtype == MEDUSA_BF16) hipLaunchKernelGGL(tree_rope_kernel<uint16_t>, grid, block, 0, stream, a);
  else hipLaunchKernelGGL(tree_rope_kernel<float>, grid, block, 0, stream, a);
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}
