// Shared host/device helpers of the HIP library (gfx950 only).  Nothing in this file is
// used by, or derived from, the CPU oracle.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include "medusa.h"

#define MEDUSA_HIP_TRY(expr)                     \
  do {                                           \
    hipError_t _e = (expr);                      \
    if (_e != hipSuccess) return MEDUSA_EHIP;    \
  } while (0)

// Launch-error check: catches bad configurations without synchronising.
#define MEDUSA_LAUNCH_CHECK()                          \
  do {                                                 \
    if (hipGetLastError() != hipSuccess) return MEDUSA_EHIP; \
  } while (0)

constexpr int kWave = 64;

// Device copy of the candidate-tree tables (Sec. 2.1.2).  Fixed-size POD so one
// allocation and one memcpy upload it.
struct TreeTables {
  int32_t T, K, S, n_leaves;
  int32_t topk_per_head[MEDUSA_MAX_HEADS];  // S_k
  int32_t head_base[MEDUSA_MAX_HEADS];      // index of head k's first entry in [root, top-S_1, top-S_2, ...]
  int32_t parent[MEDUSA_MAX_TREE_TOKENS];
  int32_t depth[MEDUSA_MAX_TREE_TOKENS];
  int32_t rank[MEDUSA_MAX_TREE_TOKENS];
  int32_t token_src[MEDUSA_MAX_TREE_TOKENS];
  uint64_t anc_mask[MEDUSA_MAX_TREE_TOKENS][2];
};

struct medusa_tree {
  TreeTables host;
  int32_t* paths;          // host [n_leaves][K+1]
  TreeTables* dev;         // device copy
  int device;              // device the copy lives on
};

typedef __bf16 bf16_t;
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((__vector_size__(8 * sizeof(__bf16))));   // MFMA operand
typedef float floatx4_t __attribute__((__vector_size__(4 * sizeof(float))));     // MFMA accumulator
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// fp32 -> bf16, round to nearest even, with the hardware converter (v_cvt_pk_bf16_f32).
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2v_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2v_t));
}
__device__ __forceinline__ uint32_t float_to_bf16_bits(float x) { return pack_bf16x2(x, 0.f) & 0xffffu; }

template <typename T> __device__ __forceinline__ float load_as_float(const T* p);
template <> __device__ __forceinline__ float load_as_float<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_as_float<uint16_t>(const uint16_t* p) { return bf16_bits_to_float(*p); }

template <typename T> __device__ __forceinline__ void store_from_float(T* p, float v);
template <> __device__ __forceinline__ void store_from_float<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_from_float<uint16_t>(uint16_t* p, float v) { *p = (uint16_t)float_to_bf16_bits(v); }

// Wavefront reductions; every lane ends with the result.  Inside a 16-lane row the exchange uses
// DPP (quad permutes, then half-row and row mirrors: no LDS crossbar); the four row results are
// combined through scalar registers.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) { return __uint_as_float(dpp_u32<CTRL>(__float_as_uint(v))); }
constexpr int kDppQuadSwap1 = 0xB1;   // quad_perm [1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;   // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // row_half_mirror
constexpr int kDppMirror = 0x140;     // row_mirror

__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_f32<kDppQuadSwap1>(v);
  v += dpp_f32<kDppQuadSwap2>(v);
  v += dpp_f32<kDppHalfMirror>(v);
  v += dpp_f32<kDppMirror>(v);
  return v;
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_f32<kDppQuadSwap1>(v));
  v = fmaxf(v, dpp_f32<kDppQuadSwap2>(v));
  v = fmaxf(v, dpp_f32<kDppHalfMirror>(v));
  v = fmaxf(v, dpp_f32<kDppMirror>(v));
  return v;
}
__device__ __forceinline__ float readlane_f32(float v, int lane) {
  return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(v), lane));
}
__device__ __forceinline__ float wave_sum(float v) {
  v = row16_sum(v);
  return (readlane_f32(v, 0) + readlane_f32(v, 16)) + (readlane_f32(v, 32) + readlane_f32(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
  v = row16_max(v);
  return fmaxf(fmaxf(readlane_f32(v, 0), readlane_f32(v, 16)), fmaxf(readlane_f32(v, 32), readlane_f32(v, 48)));
}
template <int CTRL>
__device__ __forceinline__ uint64_t dpp_max_u64(uint64_t v) {
  const uint32_t lo = dpp_u32<CTRL>((uint32_t)v), hi = dpp_u32<CTRL>((uint32_t)(v >> 32));
  const uint64_t w = ((uint64_t)hi << 32) | lo;
  return w > v ? w : v;
}
__device__ __forceinline__ uint64_t readlane_u64(uint64_t v, int lane) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, lane);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), lane);
  return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
  v = dpp_max_u64<kDppQuadSwap1>(v);
  v = dpp_max_u64<kDppQuadSwap2>(v);
  v = dpp_max_u64<kDppHalfMirror>(v);
  v = dpp_max_u64<kDppMirror>(v);
  const uint64_t a = readlane_u64(v, 0), b = readlane_u64(v, 16), c = readlane_u64(v, 32), d = readlane_u64(v, 48);
  const uint64_t ab = a > b ? a : b, cd = c > d ? c : d;
  return ab > cd ? ab : cd;
}

// Ticket counters of the elections below live in device arrays of the library, one set per STREAM
// SLOT: the host maps every stream it sees to a slot (ticket_slot(), first come first served), so calls
// on different streams use different counters and may overlap; calls on one stream are ordered
// anyway.  There are kTicketSlots slots per process; streams beyond that share the last one (and must
// then not overlap among themselves).
constexpr int kTicketSlots = 16;
int ticket_slot(hipStream_t stream);

// "Last workgroup of a group" election for single-launch two-phase kernels.  Every workgroup
// calls it once after it has written its partial results with store_agent(); exactly one call per
// group of `total` workgroups returns true, and that workgroup may then read all partials of
// the group with load_agent().  On this multi-die GPU a device-wide fence costs a write-back of
// the die's L2, so no fence is used: partials are written through to the device-coherent level
// (agent-scope stores), each wavefront waits until its own stores are acknowledged, and only
// then is the ticket taken; readers bypass the non-coherent caches the same way.  The counter
// returns to zero, so it needs no initialisation between launches.
template <typename T>
__device__ __forceinline__ T load_agent(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void store_agent(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// All-reduce over the four 16-lane rows of a wavefront (lanes l%16 + {0, 16, 32, 48}) with the
// row-swap instructions of gfx950: v_permlane16_swap exchanges the odd rows of its first operand with
// the even rows of its second, v_permlane32_swap the upper half of the first with the lower half of
// the second, so op(first, second) after a swap of (x, x) combines x with its partner row / half in
// every lane.  Two vector-ALU instructions per step instead of an LDS round trip (ds_bpermute).
typedef unsigned int u32pair_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float rows_max(float x) {
  const unsigned int u = __float_as_uint(x);
  const u32pair_t a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const unsigned int v = __float_as_uint(fmaxf(__uint_as_float(a.x), __uint_as_float(a.y)));
  const u32pair_t b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return fmaxf(__uint_as_float(b.x), __uint_as_float(b.y));
}
__device__ __forceinline__ float rows_sum(float x) {
  const unsigned int u = __float_as_uint(x);
  const u32pair_t a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const unsigned int v = __float_as_uint(__uint_as_float(a.x) + __uint_as_float(a.y));
  const u32pair_t b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return __uint_as_float(b.x) + __uint_as_float(b.y);
}

// Workgroup barrier that waits for this wavefront's LDS accesses only.  __syncthreads() also carries
// a fence that waits for every global load in flight, which would empty the ring of K/V steps below
// once per step.  The "memory" clobber keeps the compiler from moving memory operations across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// 16 bytes per lane from global memory straight into LDS (global_load_lds_dwordx4): lane l's bytes land
// at lds_base + 16 l; lds_base is wavefront-uniform and travels in M0.  An assembly statement on
// purpose: where the compiler sees such a load it also decides where to wait for it, and it waits for
// every load in flight before the first LDS read it cannot tell apart from the destination -- once
// per step, which again empties the ring.  Completion is tracked by hand with the load counter.
// STREAM marks data read once (weights of a skinny GEMM): the load carries the non-temporal hint.
template <bool STREAM = false>
__device__ __forceinline__ void load_to_lds_b128(const void* gptr, unsigned char* lds_base) {
  const uint32_t m0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds_base);
  if (STREAM) asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off nt" : : "s"(m0), "v"(gptr) : "memory", "m0");
  else asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(m0), "v"(gptr) : "memory", "m0");
}
// Wait until at most N of this wavefront's vector-memory loads are outstanding (they complete in order).
template <int N>
__device__ __forceinline__ void wait_loads_outstanding() {
  static_assert(N >= 0 && N <= 63, "the counter has six bits");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Election of the workgroup that arrives last among `total` that share `counter` (zero before the first
// arrives, zero again after the last): every caller's earlier stores are complete before it takes
// its ticket.  Called by all threads of the workgroup; true in every thread of the last one.
// `s_ticket` is a word of LDS no thread of the workgroup uses for anything else during the call.
__device__ __forceinline__ bool last_workgroup_of(unsigned int* counter, unsigned int total, unsigned int* s_ticket) {
  __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): this wavefront's loads and stores are complete
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned int t = atomicAdd(counter, 1u);
    if (t == total - 1) atomicExch(counter, 0u);
    *s_ticket = t;
  }
  __syncthreads();
  return *s_ticket == total - 1;
}
__device__ __forceinline__ bool last_workgroup_of(unsigned int* counter, unsigned int total) {
  __shared__ unsigned int s_ticket;
  return last_workgroup_of(counter, total, &s_ticket);
}

// Order-preserving key for (logit, token id): a larger key means a larger logit, or an equal
// logit and a lower id.  -0.0 is folded onto +0.0 so the two compare equal.
__device__ __forceinline__ uint64_t rank_key(float v, uint32_t id) {
  uint32_t u = __float_as_uint(v);
  if (u == 0x80000000u) u = 0;
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((uint64_t)u << 32) | (uint64_t)(0xffffffffu - id);
}
__device__ __forceinline__ uint32_t rank_key_id(uint64_t key) { return 0xffffffffu - (uint32_t)key; }

__host__ __device__ static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Reduction of a slice of one logits row (medusa_accept, Sec. 2.3.1): the arg-max as a rank_key and,
// for the soft-max of typical / sampled acceptance, in log2 units (t = logit * log2(e) / temperature):
// m = max t, S = sum 2^(t - m), U = sum (t - m) 2^(t - m).  Slices merge with stats_merge().
struct RowPart {
  uint64_t key;
  float m, S, U;
  float pad;
};
__device__ __forceinline__ void stats_merge(float& m, float& S, float& U, float m2, float S2, float U2) {
  const float mn = fmaxf(m, m2);
  const float c1 = S > 0.f ? __builtin_amdgcn_exp2f(m - mn) : 0.f, d1 = S > 0.f ? m - mn : 0.f;
  const float c2 = S2 > 0.f ? __builtin_amdgcn_exp2f(m2 - mn) : 0.f, d2 = S2 > 0.f ? m2 - mn : 0.f;
  U = c1 * (U + d1 * S) + c2 * (U2 + d2 * S2);
  S = c1 * S + c2 * S2;
  m = mn;
}
// Row reductions a vocabulary-projection kernel leaves behind for medusa_accept_fused: a header, one
// merged RowPart slot group per row (filled by the acceptance kernel), then n_parts RowParts per row.
struct FusedStatsHeader {
  int32_t n_parts;      // partials per row the producer wrote
  int32_t typical;      // 1: m, S, U are valid (the producer ran with a temperature); 0: keys only
  float k2;             // log2(e) / temperature the producer used
  int32_t rows;
  int32_t pad[60];
};
static_assert(sizeof(FusedStatsHeader) == 256, "header is one 256-byte block");
constexpr int kFusedMergedSlots = 8;                       // slots per row in the merged area (= the scan kernel's chunk bound)
