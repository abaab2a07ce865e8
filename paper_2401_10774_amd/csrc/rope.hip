// tree_rope: rotary position embedding of the tree tokens' queries and keys at the tree's
// positional indices (Sec. 2.1.2: position = prefix length + depth of the node; the indices are
// the position_ids table medusa_topk_tree emits).  Half-split pairing of the Llama family: element
// j < D/2 and element j + D/2 form a pair, rotated by position * theta^(-2j/D).
//
// The tensors are small (B x heads x T x D elements), in place.  Angles are formed and reduced in
// double precision: at positions in the thousands a float angle would cost 3-4 decimal digits of
// the rotation.  One workgroup per token, so that the trigonometry is done once per token and
// wavefront rather than once per head (16 x 65 tokens, 40 head rows: 16.6 -> about 6 us).
#include "common.hpp"

namespace {

struct RopeArgs {
  void* q;                    // [B][Hq][T][D]
  void* k;                    // [B][Hkv][T][D]
  const int32_t* position_ids;  // [B][T]
  int B, Hq, Hkv, T, D;
  double neg_log2_theta_2_over_d;   // -(2/D) * log2(theta)
};

// grid (B*T), 256 threads: one workgroup per tree token.  The angles depend on the token's position
// and on the element pair only, not on the head, so each wavefront evaluates sine and cosine once per
// pair (in double: positions reach several thousand and fp32 outputs are checked to 1e-5) and then
// walks over its share of the Hq + Hkv head rows of that token.
template <typename E>
__global__ __launch_bounds__(1024) void tree_rope_kernel(RopeArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
  const int b = blockIdx.x / a.T, t = blockIdx.x - b * a.T;
  const double pos = (double)a.position_ids[(long)b * a.T + t];
  const int half = a.D >> 1, rows = a.Hq + a.Hkv;
  auto row_ptr = [&](int hr) {
    hr = hr < rows ? hr : rows - 1;                       // (surplus slots of a batch repeat the last row and are not stored)
    const bool is_q = hr < a.Hq;
    const int h = is_q ? hr : hr - a.Hq, H = is_q ? a.Hq : a.Hkv;
    return (E*)(is_q ? a.q : a.k) + (((long)b * H + h) * a.T + t) * a.D;
  };
  for (int j = lane; j < half; j += 64) {
    const double ang = pos * exp2((double)j * a.neg_log2_theta_2_over_d);
    double s, c;
    sincos(ang, &s, &c);
    // four head rows at a time, their loads requested together
    for (int hr0 = wave; hr0 < rows; hr0 += 4 * n_waves) {
      E* x[4];
      float lo[4], hi[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        x[u] = row_ptr(hr0 + u * n_waves);
        lo[u] = load_as_float<E>(x[u] + j);
        hi[u] = load_as_float<E>(x[u] + j + half);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (hr0 + u * n_waves >= rows) break;
        store_from_float<E>(x[u] + j, (float)((double)lo[u] * c - (double)hi[u] * s));
        store_from_float<E>(x[u] + j + half, (float)((double)hi[u] * c + (double)lo[u] * s));
      }
    }
  }
}

// tree_interleave_gate_up: the weight layout tree_linear_swiglu reads -- rows 32b..32b+15 of the
// output are rows 16b..16b+15 of w_gate, rows 32b+16..32b+31 the same rows of w_up.  A one-time
// copy per weight pair: grid (2*d_out), 256 threads, one output row per workgroup in 16-byte pieces.
__global__ __launch_bounds__(256) void interleave_gate_up_kernel(const u32x4_t* __restrict__ w_gate, const u32x4_t* __restrict__ w_up,
                                                                 u32x4_t* __restrict__ w_gu, int row_chunks) {
  const int row = blockIdx.x, blk = row >> 5, r = row & 31;
  const u32x4_t* src = (r < 16 ? w_gate : w_up) + ((size_t)blk * 16 + (r & 15)) * row_chunks;
  u32x4_t* dst = w_gu + (size_t)row * row_chunks;
  for (int c = threadIdx.x; c < row_chunks; c += 256) dst[c] = src[c];
}

}  // namespace

extern "C" int tree_interleave_gate_up(const void* w_gate, const void* w_up, void* w_gu, int d_out, int d_in, int dtype,
                                       medusa_stream_t stream_) {
  if (!w_gate || !w_up || !w_gu) return MEDUSA_EINVAL;
  if (d_out < 1 || d_in < 1) return MEDUSA_EINVAL;
  if (dtype != MEDUSA_F32 && dtype != MEDUSA_BF16) return MEDUSA_EINVAL;
  const size_t row_bytes = (size_t)d_in * (dtype == MEDUSA_BF16 ? 2 : 4);
  if (d_out % 16 != 0 || row_bytes % 16 != 0 || d_out > (1 << 24)) return MEDUSA_EUNSUPPORTED;
  if ((((uintptr_t)w_gate | (uintptr_t)w_up | (uintptr_t)w_gu) & 15) != 0) return MEDUSA_EUNSUPPORTED;
  hipLaunchKernelGGL(interleave_gate_up_kernel, dim3(2 * d_out), dim3(256), 0, (hipStream_t)stream_, (const u32x4_t*)w_gate,
                     (const u32x4_t*)w_up, (u32x4_t*)w_gu, (int)(row_bytes / 16));
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}

extern "C" int tree_rope(void* q, void* k, const int32_t* position_ids, int B, int Hq, int Hkv, int T, int D, float theta,
                         int dtype, medusa_stream_t stream_) {
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
  if ((long)B * T > ((long)1 << 30)) return MEDUSA_EUNSUPPORTED;
  // wavefronts per token: enough for one batch of four head rows each, at most 16
  int n_waves = (Hq + Hkv + 3) / 4;
  n_waves = n_waves < 1 ? 1 : (n_waves > 16 ? 16 : n_waves);
  const dim3 grid((unsigned)((long)B * T)), block(64 * n_waves);
  hipStream_t stream = (hipStream_t)stream_;
  if (dtype == MEDUSA_BF16) hipLaunchKernelGGL(tree_rope_kernel<uint16_t>, grid, block, 0, stream, a);
  else hipLaunchKernelGGL(tree_rope_kernel<float>, grid, block, 0, stream, a);
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}
