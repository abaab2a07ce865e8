// medusa_accept (Sec. 2.3.1 of the Medusa paper): greedy or typical acceptance of the tree's
// candidates and selection of the longest accepted prefix.
//
// One launch.  The only pass over the B*T*V logits: each (row, chunk) workgroup reduces its slice
// to an arg-max key and, in typical mode, the soft-max statistics
//   m = max z,  S = sum exp(z - m),  U = sum (z - m) exp(z - m),   z = logit / temperature,
// from which  ln p(x) = z_x - m - ln S  and the entropy  H = ln S - U / S  (kept in log2 units
// inside the scan so that the exponential is the hardware's 2^x).
// The last workgroup of a sequence to finish (ticket counter) then merges the chunks with one
// thread per node, evaluates every node's test on its parent's row, turns the pass bits into
// two 64-bit ballots and decides acceptance of node t as  (anc_mask[t] & ~pass) == 0  -- no
// pointer chasing.  The winner is the accepted node of greatest depth and, at equal depth,
// lowest index.
#include <math.h>

#include "common.hpp"

namespace {

constexpr int kAccMaxChunks = 8;   // upper bound of workgroups per logits row (sizes the partial buffer)
constexpr int kMaxBatch = 4096;

// Ticket counters of the "last workgroup of a sequence" election, per stream slot; zero between launches.
__device__ unsigned int g_accept_ticket[kTicketSlots][kMaxBatch];

template <bool TYPICAL>
__device__ __forceinline__ void row_stats(const float* __restrict__ logits, int V, float inv_temp,
                                          RowPart* __restrict__ part, int chunks) {
  __shared__ uint64_t s_key[4];
  __shared__ float s_m[4], s_S[4], s_U[4];
  const size_t row = blockIdx.y;
  const float* src = logits + row * V;
  // arg-max: a thread visits its elements in increasing index order, so a strict ">" keeps the
  // lowest index among equal values (and treats -0.0 as equal to +0.0)
  float best = -INFINITY;
  int best_i = -1;
  // soft-max statistics in log2 units: t = z * log2(e), m = max t, S = sum 2^(t-m), U = sum (t-m) 2^(t-m)
  float m = -INFINITY, S = 0.f, U = 0.f;
  const float k2 = inv_temp * 1.4426950408889634f;
  auto visit_max = [&](float x, int i) {
    if (x > best || best_i < 0) {
      best = x;
      best_i = i;
    }
  };
  auto visit = [&](float x, int i) {
    visit_max(x, i);
    if (TYPICAL) {
      const float t = x * k2;
      if (t > m) {                       // new running maximum: rescale what has been summed
        const float c = S > 0.f ? __builtin_amdgcn_exp2f(m - t) : 0.f;
        U = S > 0.f ? c * (U + (m - t) * S) : 0.f;
        S = c * S + 1.f;                 // the new element contributes 2^0 = 1 and (t - t) * 1 = 0
        m = t;
      } else {
        const float e = __builtin_amdgcn_exp2f(t - m);
        S += e;
        U += (t - m) * e;
      }
    }
  };
  if ((V & 3) == 0) {                    // rows are 16-byte aligned: four logits per load
    const int per = ceil_div(V >> 2, chunks);
    const int lo = blockIdx.x * per, hi = min(V >> 2, lo + per);
    const floatx4_t* src4 = (const floatx4_t*)src;
    // eight independent 16-byte loads in flight per thread before the visits consume them
    constexpr int NB = 8;
    for (int i0 = lo + threadIdx.x; i0 < hi; i0 += NB * 256) {
      floatx4_t v[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) v[u] = src4[min(i0 + u * 256, hi - 1)];
      float bm = -INFINITY;
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int i = i0 + u * 256;
        if (i < hi) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            visit_max(v[u][e], 4 * i + e);
            if (TYPICAL) {
              v[u][e] *= k2;
              bm = fmaxf(bm, v[u][e]);
            }
          }
        }
      }
      if (TYPICAL) {
        // the batch's maximum first, one rescale of the running sums for all 32 values, then
        // branch-free accumulation: one exp2 per value instead of a divergent branch with one on each side
        if (bm > m) {
          const float c = S > 0.f ? __builtin_amdgcn_exp2f(m - bm) : 0.f;
          U = S > 0.f ? c * (U + (m - bm) * S) : 0.f;
          S = c * S;
          m = bm;
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          if (i0 + u * 256 < hi) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float d = v[u][e] - m, p = __builtin_amdgcn_exp2f(d);
              S += p;
              U = fmaf(d, p, U);
            }
          }
        }
      }
    }
  } else {
    const int per = ceil_div(V, chunks);
    const int lo = blockIdx.x * per, hi = min(V, lo + per);
    for (int i = lo + threadIdx.x; i < hi; i += 256) visit(src[i], i);
  }
  uint64_t key = best_i >= 0 ? rank_key(best, (uint32_t)best_i) : 0;
  key = wave_max_u64(key);
  if (TYPICAL) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float m2 = __shfl_xor(m, o, kWave), S2 = __shfl_xor(S, o, kWave), U2 = __shfl_xor(U, o, kWave);   // 6 steps, once per workgroup
      stats_merge(m, S, U, m2, S2, U2);
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) {
    s_key[wave] = key;
    s_m[wave] = m;
    s_S[wave] = S;
    s_U[wave] = U;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) {
      key = s_key[w] > key ? s_key[w] : key;
      if (TYPICAL) stats_merge(m, S, U, s_m[w], s_S[w], s_U[w]);
    }
    RowPart* p = part + row * kAccMaxChunks + blockIdx.x;
    store_agent(&p->key, key);
    store_agent(&p->m, m);
    store_agent(&p->S, S);
    store_agent(&p->U, U);
  }
}

// Runs in the 256 threads of one workgroup; threads >= 128 only take part in the barriers.
template <bool TYPICAL>
__device__ __forceinline__ void accept_finalize(int b, const float* __restrict__ logits,
                                                const int32_t* __restrict__ tree_tokens,
                                                const TreeTables* __restrict__ tree, const RowPart* __restrict__ part,
                                                int V, int chunks, float inv_temp, float eps, float delta,
                                                int32_t* __restrict__ accept_len, int32_t* __restrict__ best_node,
                                                int32_t* __restrict__ path_nodes, int32_t* __restrict__ accepted_tokens,
                                                int32_t* __restrict__ next_root) {
  __shared__ int32_t s_arg[MEDUSA_MAX_TREE_TOKENS];
  __shared__ float s_m[MEDUSA_MAX_TREE_TOKENS], s_lnS[MEDUSA_MAX_TREE_TOKENS], s_H[MEDUSA_MAX_TREE_TOKENS];
  __shared__ uint64_t s_pass[2];
  __shared__ uint32_t s_best[2];
  __shared__ uint64_t s_anc[MEDUSA_MAX_TREE_TOKENS][2];
  __shared__ int32_t s_tok[MEDUSA_MAX_TREE_TOKENS];
  const int t = threadIdx.x;
  const int T = tree->T, K = tree->K;
  const int lane = t & 63, wave = t >> 6;
  // Everything this thread will need from memory is requested up front, so that the workgroup pays
  // one round trip, not one per phase: its node's tree-table entries, its token, and all partials.
  int par = 0, tok = -1, dep = 0;
  uint64_t anc0 = 0, anc1 = 0;
  if (t < T) {
    par = tree->parent[t];
    dep = tree->depth[t];
    anc0 = tree->anc_mask[t][0];
    anc1 = tree->anc_mask[t][1];
    tok = tree_tokens[(size_t)b * T + t];
    const RowPart* p = part + ((size_t)b * T + t) * kAccMaxChunks;
    uint64_t keys[kAccMaxChunks];
    float pm[kAccMaxChunks], pS[kAccMaxChunks], pU[kAccMaxChunks];
#pragma unroll
    for (int c = 0; c < kAccMaxChunks; ++c)
      if (c < chunks) {
        keys[c] = load_agent(&p[c].key);
        if (TYPICAL) {
          pm[c] = load_agent(&p[c].m);
          pS[c] = load_agent(&p[c].S);
          pU[c] = load_agent(&p[c].U);
        }
      }
    uint64_t key = keys[0];
    float m = 0.f, S = 0.f, U = 0.f;
    if (TYPICAL) {
      m = pm[0];
      S = pS[0];
      U = pU[0];
    }
#pragma unroll
    for (int c = 1; c < kAccMaxChunks; ++c)
      if (c < chunks) {
        key = keys[c] > key ? keys[c] : key;
        if (TYPICAL) stats_merge(m, S, U, pm[c], pS[c], pU[c]);
      }
    s_anc[t][0] = anc0;
    s_anc[t][1] = anc1;
    s_tok[t] = tok;
    s_arg[t] = (int32_t)rank_key_id(key);
    if (TYPICAL) {
      // statistics are in log2 units: ln S stays ln S, the entropy is ln S - ln 2 * U / S
      const float lnS = logf(S);
      s_m[t] = m;
      s_lnS[t] = lnS;
      s_H[t] = lnS - 0.6931471805599453f * U / S;
    }
  }
  __syncthreads();
  bool pass = false;
  if (t == 0) pass = true;                                   // the root is accepted unconditionally
  else if (t < T) {
    if (!TYPICAL) {
      pass = tok == s_arg[par];
    } else if (tok >= 0 && tok < V) {
      const float t2 = logits[((size_t)b * T + par) * V + tok] * (inv_temp * 1.4426950408889634f);
      const float p_tok = expf((t2 - s_m[par]) * 0.6931471805599453f - s_lnS[par]);
      const float thr = fminf(eps, delta * expf(-s_H[par]));
      pass = p_tok > thr;
    }
  }
  const uint64_t bal = __ballot(pass);
  if (lane == 0 && wave < 2) s_pass[wave] = bal;
  __syncthreads();
  const uint64_t fail0 = ~s_pass[0], fail1 = ~s_pass[1];
  uint32_t score = 0;
  if (t < T && (anc0 & fail0) == 0 && (anc1 & fail1) == 0)
    score = ((uint32_t)(dep + 1) << 8) | (uint32_t)(255 - t);   // deeper first, then lower index
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) score = max(score, (uint32_t)__shfl_xor((int)score, o, kWave));
  if (lane == 0 && wave < 2) s_best[wave] = score;
  __syncthreads();
  score = max(s_best[0], s_best[1]);
  const int best = 255 - (int)(score & 255u);
  const int alen = (int)(score >> 8);
  if (t == 0) {
    accept_len[b] = alen;
    best_node[b] = best;
    next_root[b] = s_arg[best];
  }
  if (t <= K) {
    // ancestors have smaller indices than descendants, so the j-th set bit of the winner's
    // ancestor mask is its ancestor at depth j
    int node = -1;
    if (t < alen) {
      int seen = 0;
      for (int u = 0; u < T; ++u) {
        if ((s_anc[best][u >> 6] >> (u & 63)) & 1ull) {
          if (seen == t) { node = u; break; }
          ++seen;
        }
      }
    }
    path_nodes[(size_t)b * (K + 1) + t] = node;
    accepted_tokens[(size_t)b * (K + 1) + t] = node >= 0 ? s_tok[node] : -1;
  }
}

// grid (chunks, B*T), 256 threads.
template <bool TYPICAL>
__global__ __launch_bounds__(256) void accept_kernel(const float* __restrict__ logits, const int32_t* __restrict__ tree_tokens,
                                                     const TreeTables* __restrict__ tree, RowPart* __restrict__ part, int V, int slot,
                                                     float inv_temp, float eps, float delta, int32_t* __restrict__ accept_len,
                                                     int32_t* __restrict__ best_node, int32_t* __restrict__ path_nodes,
                                                     int32_t* __restrict__ accepted_tokens, int32_t* __restrict__ next_root) {
  const int chunks = gridDim.x;
  row_stats<TYPICAL>(logits, V, inv_temp, part, chunks);
  const int T = tree->T;
  const int b = blockIdx.y / T;
  if (!last_workgroup_of(&g_accept_ticket[slot][b], (unsigned)(chunks * T))) return;
  accept_finalize<TYPICAL>(b, logits, tree_tokens, tree, part, V, chunks, inv_temp, eps, delta, accept_len, best_node, path_nodes,
                           accepted_tokens, next_root);
}

// Rejection-sampling acceptance (the scheme Sec. 2 and Sec. 2.3.1 name; the rule is stated at
// medusa_accept_sampled in the header).  Runs in the 256 threads of the sequence's last workgroup.
// Per node: w = 2^(t_tok - m_parent), the candidate's unnormalised probability under its parent's
// row (S_parent = the row's sum of such terms); child i is tested with u_i * (S - sum of the earlier
// siblings' w) < w_i and passes if no earlier sibling did.  The walk from the root follows the passing
// children; since at most one child of a node passes, the accepted nodes form one chain and the
// ancestor-mask test of the greedy/typical path applies unchanged.  The next token is drawn from the
// last accepted node's row without its children's tokens, by inversion in token order: every thread
// sums a contiguous slice of the row, a scan over the 256 slice sums finds the slice that holds
// u_0 * total, and that slice's thread walks it.
__device__ __forceinline__ void accept_finalize_sampled(int b, const float* __restrict__ logits,
                                                        const int32_t* __restrict__ tree_tokens,
                                                        const TreeTables* __restrict__ tree, const RowPart* __restrict__ part,
                                                        const float* __restrict__ uniforms, int V, int chunks, float inv_temp,
                                                        int32_t* __restrict__ accept_len, int32_t* __restrict__ best_node,
                                                        int32_t* __restrict__ path_nodes, int32_t* __restrict__ accepted_tokens,
                                                        int32_t* __restrict__ next_token) {
  __shared__ float s_m[MEDUSA_MAX_TREE_TOKENS], s_S[MEDUSA_MAX_TREE_TOKENS], s_w[MEDUSA_MAX_TREE_TOKENS];
  __shared__ uint64_t s_bits[2], s_pass[2];
  __shared__ uint32_t s_best[2];
  __shared__ uint64_t s_anc[MEDUSA_MAX_TREE_TOKENS][2];
  __shared__ int32_t s_tok[MEDUSA_MAX_TREE_TOKENS], s_par[MEDUSA_MAX_TREE_TOKENS];
  __shared__ float s_sum[256];
  __shared__ int s_kid_tok[MEDUSA_MAX_TOPK + 1];
  __shared__ int s_nkids, s_slice;
  __shared__ float s_target, s_before;
  const int t = threadIdx.x;
  const int T = tree->T, K = tree->K;
  const int lane = t & 63, wave = t >> 6;
  const float k2 = inv_temp * 1.4426950408889634f;
  int par = -1, tok = -1, dep = 0;
  uint64_t anc0 = 0, anc1 = 0;
  float u = 0.f;
  if (t < T) {
    par = tree->parent[t];
    dep = tree->depth[t];
    anc0 = tree->anc_mask[t][0];
    anc1 = tree->anc_mask[t][1];
    tok = tree_tokens[(size_t)b * T + t];
    u = uniforms[(size_t)b * T + t];
    const RowPart* p = part + ((size_t)b * T + t) * kAccMaxChunks;
    float m = load_agent(&p[0].m), S = load_agent(&p[0].S), U = 0.f;
    for (int c = 1; c < chunks; ++c) stats_merge(m, S, U, load_agent(&p[c].m), load_agent(&p[c].S), 0.f);
    s_m[t] = m;
    s_S[t] = S;
    s_anc[t][0] = anc0;
    s_anc[t][1] = anc1;
    s_tok[t] = tok;
    s_par[t] = par;
  }
  __syncthreads();
  float w = 0.f;
  if (t >= 1 && t < T && tok >= 0 && tok < V) w = __builtin_amdgcn_exp2f(logits[((size_t)b * T + par) * V + tok] * k2 - s_m[par]);
  if (t < T) s_w[t] = w;
  __syncthreads();
  // the node's own test, with the mass of its earlier siblings (consecutive lower indices) taken out of the row's sum
  bool test = false;
  int first_sib = t;
  if (t >= 1 && t < T) {
    while (first_sib - 1 >= 1 && s_par[first_sib - 1] == par) --first_sib;
    float removed = 0.f;
    for (int c = first_sib; c < t; ++c) removed += s_w[c];
    test = u * (s_S[par] - removed) < w;
  }
  const uint64_t tb = __ballot(test);
  if (lane == 0 && wave < 2) s_bits[wave] = tb;
  __syncthreads();
  bool pass = t == 0;                                        // the root is accepted unconditionally
  if (t >= 1 && t < T && test) {
    pass = true;
    for (int c = first_sib; c < t; ++c) pass = pass && !((s_bits[c >> 6] >> (c & 63)) & 1ull);   // an earlier sibling was taken
  }
  const uint64_t pb = __ballot(pass);
  if (lane == 0 && wave < 2) s_pass[wave] = pb;
  __syncthreads();
  const uint64_t fail0 = ~s_pass[0], fail1 = ~s_pass[1];
  uint32_t score = 0;
  if (t < T && (anc0 & fail0) == 0 && (anc1 & fail1) == 0) score = ((uint32_t)(dep + 1) << 8) | (uint32_t)(255 - t);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) score = max(score, (uint32_t)__shfl_xor((int)score, o, kWave));
  if (lane == 0 && wave < 2) s_best[wave] = score;
  __syncthreads();
  score = max(s_best[0], s_best[1]);
  const int best = 255 - (int)(score & 255u);
  const int alen = (int)(score >> 8);
  if (t == 0) {
    accept_len[b] = alen;
    best_node[b] = best;
    int n = 0;
    for (int c = best + 1; c < T; ++c)
      if (s_par[c] == best && n < MEDUSA_MAX_TOPK) s_kid_tok[n++] = s_tok[c];
    s_nkids = n;
  }
  if (t <= K) {
    int node = -1;
    if (t < alen) {
      int seen = 0;
      for (int c = 0; c < T; ++c) {
        if ((s_anc[best][c >> 6] >> (c & 63)) & 1ull) {
          if (seen == t) { node = c; break; }
          ++seen;
        }
      }
    }
    path_nodes[(size_t)b * (K + 1) + t] = node;
    accepted_tokens[(size_t)b * (K + 1) + t] = node >= 0 ? s_tok[node] : -1;
  }
  __syncthreads();
  // ---- draw the next token from the row of `best` without its children's tokens ----
  const float* row = logits + ((size_t)b * T + best) * V;
  const float m_best = s_m[best];
  const int nk = s_nkids;
  const int per = ceil_div(V, 256), lo = min(t * per, V), hi = min(V, lo + per);
  bool has_kid = false;
  for (int c = 0; c < nk; ++c) has_kid = has_kid || (s_kid_tok[c] >= lo && s_kid_tok[c] < hi);
  auto weight = [&](int y) {
    float wy = __builtin_amdgcn_exp2f(row[y] * k2 - m_best);
    if (has_kid)
      for (int c = 0; c < nk; ++c) wy = s_kid_tok[c] == y ? 0.f : wy;
    return wy;
  };
  float sum = 0.f;
  for (int y = lo; y < hi; ++y) sum += weight(y);
  s_sum[t] = sum;
  __syncthreads();
  if (t == 0) {
    float total = 0.f;
    for (int j = 0; j < 256; ++j) total += s_sum[j];
    const float target = uniforms[(size_t)b * T] * total;
    float before = 0.f;
    int slice = 0;
    for (int j = 0; j < 256; ++j) {                        // the first slice whose cumulative sum exceeds the target
      if (before + s_sum[j] > target) { slice = j; break; }
      before += s_sum[j];
      slice = j;
    }
    if (!(before + s_sum[slice] > target)) {               // rounding at the upper end: the last slice with any mass
      before = 0.f;
      int last = 0;
      for (int j = 0; j < 256; ++j) if (s_sum[j] > 0.f) last = j;
      for (int j = 0; j < last; ++j) before += s_sum[j];
      slice = last;
    }
    s_slice = slice;
    s_target = target;
    s_before = before;
  }
  __syncthreads();
  if (t == s_slice) {
    float cum = s_before;
    int pick = -1, last_pos = -1;
    for (int y = lo; y < hi; ++y) {
      const float wy = weight(y);
      if (wy > 0.f) last_pos = y;
      cum += wy;
      if (pick < 0 && cum > s_target) pick = y;
    }
    next_token[b] = pick >= 0 ? pick : (last_pos >= 0 ? last_pos : max(lo, 0));
  }
}

// grid (chunks, B*T), 256 threads.
__global__ __launch_bounds__(256) void accept_sampled_kernel(const float* __restrict__ logits, const int32_t* __restrict__ tree_tokens,
                                                             const TreeTables* __restrict__ tree, RowPart* __restrict__ part,
                                                             const float* __restrict__ uniforms, int V, int slot, float inv_temp,
                                                             int32_t* __restrict__ accept_len, int32_t* __restrict__ best_node,
                                                             int32_t* __restrict__ path_nodes, int32_t* __restrict__ accepted_tokens,
                                                             int32_t* __restrict__ next_token) {
  const int chunks = gridDim.x;
  row_stats<true>(logits, V, inv_temp, part, chunks);
  const int T = tree->T;
  const int b = blockIdx.y / T;
  if (!last_workgroup_of(&g_accept_ticket[slot][b], (unsigned)(chunks * T))) return;
  accept_finalize_sampled(b, logits, tree_tokens, tree, part, uniforms, V, chunks, inv_temp, accept_len, best_node, path_nodes,
                          accepted_tokens, next_token);
}

}  // namespace

extern "C" int medusa_accept_sampled(const float* logits, const int32_t* tree_tokens, const medusa_tree_t* tree,
                                     const float* uniforms, int B, int V, float temperature, int32_t* accept_len,
                                     int32_t* best_node, int32_t* path_nodes, int32_t* accepted_tokens, int32_t* next_token,
                                     void* workspace, size_t workspace_bytes, medusa_stream_t stream_) {
  if (!logits || !tree_tokens || !tree || !uniforms || !accept_len || !best_node || !path_nodes || !accepted_tokens || !next_token)
    return MEDUSA_EINVAL;
  if (B < 1 || V < 1 || !(temperature > 0.f)) return MEDUSA_EINVAL;
  if (B > kMaxBatch) return MEDUSA_EUNSUPPORTED;
  const int T = tree->host.T;
  if ((long)B * T > 65535) return MEDUSA_EUNSUPPORTED;
  if (!tree->dev) return MEDUSA_EHIP;
  if (!workspace || workspace_bytes < medusa_accept_workspace_bytes(B, T, V) || ((uintptr_t)workspace & 7) != 0)
    return MEDUSA_EWORKSPACE;
  int chunks = 260 / (B * T);
  chunks = chunks < 1 ? 1 : (chunks > kAccMaxChunks ? kAccMaxChunks : chunks);
  hipLaunchKernelGGL(accept_sampled_kernel, dim3(chunks, B * T), dim3(256), 0, (hipStream_t)stream_, logits, tree_tokens,
                     tree->dev, (RowPart*)workspace, uniforms, V, ticket_slot((hipStream_t)stream_), 1.0f / temperature, accept_len, best_node, path_nodes,
                     accepted_tokens, next_token);
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}

namespace {
// Acceptance from the row reductions a vocabulary-projection kernel left behind (medusa_verify_logits):
// grid (B*T), 256 threads.  A workgroup merges the n_parts partials of its row -- a few KB instead of the
// row's V logits --, publishes the result and takes a ticket; the last workgroup of a sequence runs
// the same final step as the scanning kernel.  A header mismatch (statistics produced for another
// mode or temperature) is reported as accept_len = -1.
template <bool TYPICAL>
__global__ __launch_bounds__(256) void accept_fused_kernel(const float* __restrict__ logits, const int32_t* __restrict__ tree_tokens,
                                                           const TreeTables* __restrict__ tree, const FusedStatsHeader* __restrict__ hdr,
                                                           int V, int slot, float k2_want, float eps, float delta,
                                                           int32_t* __restrict__ accept_len, int32_t* __restrict__ best_node,
                                                           int32_t* __restrict__ path_nodes, int32_t* __restrict__ accepted_tokens,
                                                           int32_t* __restrict__ next_root) {
  __shared__ uint64_t s_key[4];
  __shared__ float s_m[4], s_S[4], s_U[4];
  const int T = tree->T;
  const int row = blockIdx.x, b = row / T;
  const int n_parts = hdr->n_parts;
  const bool ok = hdr->rows == (int)gridDim.x && n_parts >= 1 && n_parts <= 2 * ceil_div(V, 256) && (!TYPICAL || (hdr->typical == 1 && hdr->k2 == k2_want));
  RowPart* merged = (RowPart*)(hdr + 1);
  const RowPart* part = merged + (size_t)gridDim.x * kFusedMergedSlots + (size_t)row * (ok ? n_parts : 0);
  uint64_t key = 0;
  float m = -INFINITY, S = 0.f, U = 0.f;
  if (ok) {
    for (int i = threadIdx.x; i < n_parts; i += 256) {
      const RowPart p = part[i];
      key = p.key > key ? p.key : key;
      if (TYPICAL) stats_merge(m, S, U, p.m, p.S, p.U);
    }
  }
  key = wave_max_u64(key);
  if (TYPICAL) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float m2 = __shfl_xor(m, o, kWave), S2 = __shfl_xor(S, o, kWave), U2 = __shfl_xor(U, o, kWave);
      stats_merge(m, S, U, m2, S2, U2);
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) {
    s_key[wave] = key;
    s_m[wave] = m;
    s_S[wave] = S;
    s_U[wave] = U;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) {
      key = s_key[w] > key ? s_key[w] : key;
      if (TYPICAL) stats_merge(m, S, U, s_m[w], s_S[w], s_U[w]);
    }
    RowPart* p = merged + (size_t)row * kFusedMergedSlots;
    store_agent(&p->key, key);
    store_agent(&p->m, m);
    store_agent(&p->S, S);
    store_agent(&p->U, U);
  }
  if (!last_workgroup_of(&g_accept_ticket[slot][b], (unsigned)T)) return;
  if (!ok) {
    if (threadIdx.x == 0) accept_len[b] = -1;
    return;
  }
  accept_finalize<TYPICAL>(b, logits, tree_tokens, tree, merged, V, 1, k2_want * 0.6931471805599453f, eps, delta, accept_len, best_node,
                           path_nodes, accepted_tokens, next_root);
}
}  // namespace

extern "C" int medusa_accept_fused(const float* logits, const void* stats, const int32_t* tree_tokens, const medusa_tree_t* tree,
                                   int B, int V, int mode, float temperature, float eps, float delta, int32_t* accept_len,
                                   int32_t* best_node, int32_t* path_nodes, int32_t* accepted_tokens, int32_t* next_root,
                                   medusa_stream_t stream_) {
  if (!logits || !stats || !tree_tokens || !tree || !accept_len || !best_node || !path_nodes || !accepted_tokens || !next_root)
    return MEDUSA_EINVAL;
  if (B < 1 || V < 1) return MEDUSA_EINVAL;
  if (mode != MEDUSA_GREEDY && mode != MEDUSA_TYPICAL) return MEDUSA_EINVAL;
  if (mode == MEDUSA_TYPICAL && !(temperature > 0.f)) return MEDUSA_EINVAL;
  if (B > kMaxBatch || ((uintptr_t)stats & 255) != 0) return MEDUSA_EUNSUPPORTED;
  const int T = tree->host.T;
  if (!tree->dev) return MEDUSA_EHIP;
  static_assert(kFusedMergedSlots == kAccMaxChunks, "the final step reads the merged rows with the scan kernel's stride");
  hipStream_t stream = (hipStream_t)stream_;
  const FusedStatsHeader* hdr = (const FusedStatsHeader*)stats;
  const float k2 = mode == MEDUSA_TYPICAL ? 1.4426950408889634f / temperature : 0.f;
  if (mode == MEDUSA_TYPICAL)
    hipLaunchKernelGGL(accept_fused_kernel<true>, dim3(B * T), dim3(256), 0, stream, logits, tree_tokens, tree->dev, hdr, V, ticket_slot(stream), k2, eps,
                       delta, accept_len, best_node, path_nodes, accepted_tokens, next_root);
  else
    hipLaunchKernelGGL(accept_fused_kernel<false>, dim3(B * T), dim3(256), 0, stream, logits, tree_tokens, tree->dev, hdr, V, ticket_slot(stream), k2, eps,
                       delta, accept_len, best_node, path_nodes, accepted_tokens, next_root);
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}

extern "C" size_t medusa_accept_workspace_bytes(int B, int T, int V) {
  (void)V;
  if (B < 1 || T < 1) return 0;
  return (size_t)B * T * kAccMaxChunks * sizeof(RowPart);
}

extern "C" int medusa_accept(const float* logits, const int32_t* tree_tokens, const medusa_tree_t* tree, int B, int V,
                             int mode, float temperature, float eps, float delta, int32_t* accept_len,
                             int32_t* best_node, int32_t* path_nodes, int32_t* accepted_tokens, int32_t* next_root,
                             void* workspace, size_t workspace_bytes, medusa_stream_t stream_) {
  if (!logits || !tree_tokens || !tree || !accept_len || !best_node || !path_nodes || !accepted_tokens || !next_root)
    return MEDUSA_EINVAL;
  if (B < 1 || V < 1) return MEDUSA_EINVAL;
  if (mode != MEDUSA_GREEDY && mode != MEDUSA_TYPICAL) return MEDUSA_EINVAL;
  if (mode == MEDUSA_TYPICAL && !(temperature > 0.f)) return MEDUSA_EINVAL;
  if (B > kMaxBatch) return MEDUSA_EUNSUPPORTED;
  const int T = tree->host.T;
  if ((long)B * T > 65535) return MEDUSA_EUNSUPPORTED;     // logits rows ride on the grid's second dimension
  if (!tree->dev) return MEDUSA_EHIP;
  if (!workspace || workspace_bytes < medusa_accept_workspace_bytes(B, T, V) || ((uintptr_t)workspace & 7) != 0)
    return MEDUSA_EWORKSPACE;
  hipStream_t stream = (hipStream_t)stream_;
  RowPart* part = (RowPart*)workspace;
  // every workgroup ends with a ticket round trip, so few, fat workgroups win: about one per CU
  // (measured at 65 rows: 8.3 us with 3-4 chunks, 12 us with 8; at 1040 rows: 35 us with 1, 65 us with 4)
  int chunks = 260 / (B * T);
  chunks = chunks < 1 ? 1 : (chunks > kAccMaxChunks ? kAccMaxChunks : chunks);
  const dim3 grid(chunks, B * T);
  const float inv_temp = mode == MEDUSA_TYPICAL ? 1.0f / temperature : 1.0f;
  if (mode == MEDUSA_TYPICAL)
    hipLaunchKernelGGL(accept_kernel<true>, grid, dim3(256), 0, stream, logits, tree_tokens, tree->dev, part, V, ticket_slot(stream), inv_temp,
                       eps, delta, accept_len, best_node, path_nodes, accepted_tokens, next_root);
  else
    hipLaunchKernelGGL(accept_kernel<false>, grid, dim3(256), 0, stream, logits, tree_tokens, tree->dev, part, V, ticket_slot(stream), inv_temp,
                       eps, delta, accept_len, best_node, path_nodes, accepted_tokens, next_root);
  MEDUSA_LAUNCH_CHECK();
  return MEDUSA_OK;
}
