// Argument block and epilogues shared by the GEMM/GEMV kernels: medusa_heads (Sec. 2.1.1) and the
// backbone linear layers on the tree tokens (App. G, operator table).
#pragma once
#include "common.hpp"

// Epilogues: EPI_LOGITS  float  out[m][k][n] = acc                      (vocabulary projections)
//            EPI_RESID   dtype  out[m][k][n] = SiLU(acc) + hidden[m][n]   (residual block of a head)
//            EPI_PLAIN   dtype  out(m, n)    = acc                        (backbone linear layers)
//            EPI_GATED   dtype  out(m, n)    = SiLU(acc) * mul[m][n]      (gate projection times up projection)
//            EPI_SWIGLU  dtype  out(m, c)    = SiLU(acc(m, gate row of c)) * acc(m, up row of c): W holds gate and up
//                               rows interleaved in blocks of 16 (rows 32b..32b+15 gate, 32b+16..32b+31 up, of
//                               output columns 16b..16b+15); out has N/2 columns.  128-column skinny tiles only.
enum { EPI_LOGITS = 0, EPI_RESID = 1, EPI_PLAIN = 2, EPI_GATED = 3, EPI_SWIGLU = 4 };

// acc[m][n] = sum_j W[k][n][j] * X(m, k, j)
// X is either row-major with strides (x_dh == 0): X[m*xs_m + k*xs_k + j], or head-major
// [B][x_heads][x_T][x_dh] with m = b*x_T + t and j = head*x_dh + e (the layout tree attention
// writes).  The EPI_PLAIN / EPI_GATED output is row-major [M][N] (y_dh == 0) or head-major
// [B][y_heads][y_T][y_dh] with n = head*y_dh + e (the layout tree attention reads), or several such
// tensors a fixed stride apart, each taking y_heads consecutive heads of the N columns.
struct GemmArgs {
  const void* W;       // [K][N][d]
  const void* X;       // activations
  const void* hidden;  // [M][d] residual source (EPI_RESID, N == d);  [M][N] multiplier (EPI_GATED)
  void* out;
  int M, N, d, K;
  long xs_m, xs_k;     // element strides of X between rows m and between heads k (row-major X)
  int x_T, x_heads, x_dh;
  int y_T, y_heads, y_dh;
  int y_seg_heads;     // > 0: the head-major output is several tensors [B][y_heads][y_T][y_dh], y_seg_stride elements apart,
  long y_seg_stride;   //      each taking y_seg_heads (= y_heads) consecutive heads of the N columns (Q, K, V of one projection call)
  int rows_per_wg;     // GEMV kernels: weight rows per workgroup (multiple of 8)
  int m_blocks;        // ring kernel: row blocks (its grid.x interleaves them with the column tiles, see there)
  int ksplit;          // skinny MFMA kernel: workgroups that share one output tile, each reducing 1/ksplit of d
  void* ws;            // their fp32 partial tiles (ksplit > 1)
  int ticket_slot;     // which set of ticket counters a split reduction uses (one per stream, see common.hpp)
  int vec_epilogue;    // large-M kernel: 8-column runs of the output (and of `hidden`) are contiguous and 16-byte aligned
  // EPI_LOGITS, large-M kernel only: when `stats` is set every wavefront also reduces its 16-row x 128-column
  // pieces of the logits to RowParts (arg-max key; soft-max statistics when stats_k2 > 0) for medusa_accept_fused
  RowPart* stats;      // [M][stats_parts]
  int stats_parts;     // = 2 * column tiles
  float stats_k2;      // log2(e) / temperature, or 0: keys only
};

// Element offset of X(m, k, 0) and of column j relative to it.  Chunks of up to x_dh consecutive
// j (aligned) are contiguous in either layout.
// The head-major forms exist only for the epilogues tree_linear uses (HM): the kernels of
// medusa_heads are compiled without them.
template <int EPI>
constexpr bool kHeadMajor = EPI == 2 || EPI == 3 || EPI == 4;      // EPI_PLAIN, EPI_GATED, EPI_SWIGLU

template <bool HM>
__device__ __forceinline__ size_t x_row_offset(const GemmArgs& a, int m, int k) {
  if (!HM || a.x_dh == 0) return (size_t)m * a.xs_m + (size_t)k * a.xs_k;
  const int b = m / a.x_T, t = m - b * a.x_T;
  return ((size_t)b * a.x_heads * a.x_T + t) * a.x_dh;
}
template <bool HM>
__device__ __forceinline__ size_t x_col_offset(const GemmArgs& a, int j) {
  if (!HM || a.x_dh == 0) return (size_t)j;
  const int head = j / a.x_dh;
  return (size_t)head * a.x_T * a.x_dh + (j - head * a.x_dh);
}
// Element offset of the output at (m, k, n) = out_row_offset + out_col_offset.
template <bool HM>
__device__ __forceinline__ size_t out_row_offset(const GemmArgs& a, int m, int k) {
  if (!HM || a.y_dh == 0) return ((size_t)m * a.K + k) * a.N;
  const int b = m / a.y_T, t = m - b * a.y_T;
  return ((size_t)b * a.y_heads * a.y_T + t) * a.y_dh;
}
template <bool HM>
__device__ __forceinline__ size_t out_col_offset(const GemmArgs& a, int n) {
  if (!HM || a.y_dh == 0) return (size_t)n;
  int head = n / a.y_dh;
  const int e = n - head * a.y_dh;
  size_t seg_off = 0;
  if (a.y_seg_heads > 0) {
    const int seg = head / a.y_seg_heads;
    head -= seg * a.y_seg_heads;
    seg_off = (size_t)seg * a.y_seg_stride;
  }
  return seg_off + (size_t)head * a.y_T * a.y_dh + e;
}

typedef __bf16 dot2_t __attribute__((__vector_size__(2 * sizeof(__bf16))));

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dot2_t, a), __builtin_bit_cast(dot2_t, b), c, false);
}

__device__ __forceinline__ float silu_f32(float u) { return u / (1.0f + expf(-u)); }

template <int EPI, typename T>
__device__ __forceinline__ void epilogue_store(const GemmArgs& a, int m, int k, int n, float acc) {
  const size_t o = out_row_offset<kHeadMajor<EPI>>(a, m, k) + out_col_offset<kHeadMajor<EPI>>(a, n);
  if (EPI == EPI_LOGITS) {
    ((float*)a.out)[o] = acc;
  } else if (EPI == EPI_RESID) {
    const float h = load_as_float<T>((const T*)a.hidden + (size_t)m * a.d + n);
    store_from_float<T>((T*)a.out + o, silu_f32(acc) + h);
  } else if (EPI == EPI_PLAIN) {
    store_from_float<T>((T*)a.out + o, acc);
  } else {
    const float u = load_as_float<T>((const T*)a.hidden + (size_t)m * a.N + n);
    store_from_float<T>((T*)a.out + o, silu_f32(acc) * u);
  }
}

// Upper bound of the element offsets the kernels form into X (host side, for 32-bit offset checks).
inline size_t x_extent(const GemmArgs& a) {
  return a.x_dh == 0 ? (size_t)a.M * a.xs_m + (size_t)a.K * a.xs_k + a.d : (size_t)a.M * a.d + a.d;
}

// Large-M bf16 GEMM (own translation unit: it is compiled with its own code-generation options).
// Requires every element offset into W and X below 2^31.  Tiles of 192 (tall) or 128 activation rows
// x 256 weight rows.  Returns a medusa status code.
int launch_gemm_big(const GemmArgs& a, int epi, bool tall, hipStream_t stream);
