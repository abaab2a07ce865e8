// Candidate-tree tables (Sec. 2.1.2 of the Medusa paper; sparse node sets as in Sec. 2.3.3).
// Host-side construction, one device upload.  Node numbering: root = 0, then depth-major and
// lexicographic by rank tuple within a depth, so the children of a node are consecutive and
// every ancestor has a smaller index than its descendants.
#include <algorithm>
#include <array>
#include <cstring>
#include <new>
#include <vector>

#include <mutex>

#include "common.hpp"

namespace {

typedef std::array<int32_t, MEDUSA_MAX_HEADS> RankTuple;  // padded with -1

struct Node {
  RankTuple r;
  int len;
};

bool node_less(const Node& a, const Node& b) {
  if (a.len != b.len) return a.len < b.len;
  return std::lexicographical_compare(a.r.begin(), a.r.begin() + a.len, b.r.begin(), b.r.begin() + b.len);
}
bool node_equal(const Node& a, const Node& b) {
  return a.len == b.len && std::equal(a.r.begin(), a.r.begin() + a.len, b.r.begin());
}

int find_node(const std::vector<Node>& nodes, const Node& key) {
  auto it = std::lower_bound(nodes.begin(), nodes.end(), key, node_less);
  if (it == nodes.end() || !node_equal(*it, key)) return -1;
  return (int)(it - nodes.begin());
}

// `cand` holds the candidate nodes (root excluded), any order.
int build(std::vector<Node>& cand, int K, medusa_tree_t** out) {
  if ((int)cand.size() + 1 > MEDUSA_MAX_TREE_TOKENS) return MEDUSA_EUNSUPPORTED;
  Node root;
  root.r.fill(-1);
  root.len = 0;
  std::vector<Node> nodes;
  nodes.push_back(root);
  nodes.insert(nodes.end(), cand.begin(), cand.end());
  std::sort(nodes.begin(), nodes.end(), node_less);
  for (size_t i = 1; i < nodes.size(); ++i)
    if (node_equal(nodes[i - 1], nodes[i])) return MEDUSA_EINVAL;  // duplicate (or a second root)

  medusa_tree* t = new (std::nothrow) medusa_tree;
  if (!t) return MEDUSA_EINVAL;
  std::memset(&t->host, 0, sizeof(TreeTables));
  t->paths = nullptr;
  t->dev = nullptr;
  TreeTables& h = t->host;
  const int T = (int)nodes.size();
  h.T = T;
  h.K = K;
  int max_len = 0;
  for (int i = 0; i < T; ++i) {
    const Node& n = nodes[i];
    max_len = std::max(max_len, n.len);
    h.depth[i] = n.len;
    if (n.len == 0) {
      h.parent[i] = -1;
      h.rank[i] = -1;
      continue;
    }
    Node p = n;
    p.len = n.len - 1;
    p.r[p.len] = -1;
    const int pi = find_node(nodes, p);
    if (pi < 0) {  // not prefix-closed
      delete t;
      return MEDUSA_EINVAL;
    }
    h.parent[i] = pi;
    h.rank[i] = n.r[n.len - 1];
    h.topk_per_head[n.len - 1] = std::max(h.topk_per_head[n.len - 1], n.r[n.len - 1] + 1);
  }
  if (max_len != K) {
    delete t;
    return MEDUSA_EINVAL;
  }
  h.S = 0;
  int base = 1;
  for (int k = 0; k < K; ++k) {
    h.head_base[k] = base;
    base += h.topk_per_head[k];
    h.S = std::max(h.S, h.topk_per_head[k]);
  }
  std::vector<char> has_child(T, 0);
  for (int i = 0; i < T; ++i) {
    h.token_src[i] = i == 0 ? 0 : h.head_base[h.depth[i] - 1] + h.rank[i];
    uint64_t m[2] = {0, 0};
    if (i > 0) {
      m[0] = h.anc_mask[h.parent[i]][0];  // parents precede children in this numbering
      m[1] = h.anc_mask[h.parent[i]][1];
      has_child[h.parent[i]] = 1;
    }
    m[i >> 6] |= 1ull << (i & 63);
    h.anc_mask[i][0] = m[0];
    h.anc_mask[i][1] = m[1];
  }
  // candidates: root-to-leaf paths, leaves in lexicographic order of their rank tuples
  std::vector<int> leaves;
  for (int i = 0; i < T; ++i)
    if (!has_child[i]) leaves.push_back(i);
  std::sort(leaves.begin(), leaves.end(), [&](int a, int b) {
    const Node &x = nodes[a], &y = nodes[b];
    return std::lexicographical_compare(x.r.begin(), x.r.begin() + x.len, y.r.begin(), y.r.begin() + y.len);
  });
  h.n_leaves = (int)leaves.size();
  t->paths = new (std::nothrow) int32_t[(size_t)h.n_leaves * (K + 1)];
  if (!t->paths) {
    delete t;
    return MEDUSA_EINVAL;
  }
  for (int p = 0; p < h.n_leaves; ++p) {
    int32_t* row = t->paths + (size_t)p * (K + 1);
    for (int j = 0; j <= K; ++j) row[j] = -1;
    for (int u = leaves[p]; u >= 0; u = h.parent[u]) row[h.depth[u]] = u;
  }
  // Device copy.  Without a usable GPU the handle still serves the host-side queries
  // (medusa_tree_query / medusa_tree_tables); every kernel call then fails with MEDUSA_EHIP.
  t->device = -1;
  if (hipGetDevice(&t->device) == hipSuccess && hipMalloc((void**)&t->dev, sizeof(TreeTables)) == hipSuccess) {
    if (hipMemcpy(t->dev, &t->host, sizeof(TreeTables), hipMemcpyHostToDevice) != hipSuccess) {
      (void)hipFree(t->dev);
      delete[] t->paths;
      delete t;
      return MEDUSA_EHIP;
    }
  } else {
    (void)hipGetLastError();
    t->dev = nullptr;
    t->device = -1;
  }
  *out = t;
  return MEDUSA_OK;
}

}  // namespace

// Stream -> ticket slot (see common.hpp).  A handle that is reused after its stream was destroyed keeps
// its slot, which is harmless.
int ticket_slot(hipStream_t stream) {
  static std::mutex mu;
  static hipStream_t seen[kTicketSlots];
  static int n_seen = 0;
  std::lock_guard<std::mutex> lock(mu);
  for (int i = 0; i < n_seen; ++i)
    if (seen[i] == stream) return i;
  if (n_seen < kTicketSlots) {
    seen[n_seen] = stream;
    return n_seen++;
  }
  return kTicketSlots - 1;
}

extern "C" const char* medusa_status_string(int status) {
  switch (status) {
    case MEDUSA_OK: return "ok";
    case MEDUSA_EINVAL: return "invalid argument";
    case MEDUSA_EUNSUPPORTED: return "size outside the supported range";
    case MEDUSA_EWORKSPACE: return "workspace missing or too small";
    case MEDUSA_EHIP: return "HIP runtime error";
    case MEDUSA_ESCRATCH: return "shape needs more scratch than the library's built-in array holds";
    default: return "unknown status";
  }
}

extern "C" int medusa_tree_create_cartesian(const int32_t* branching, int K, medusa_tree_t** out) {
  if (!branching || !out || K < 0) return MEDUSA_EINVAL;
  if (K > MEDUSA_MAX_HEADS) return MEDUSA_EUNSUPPORTED;
  long total = 0, level = 1;
  for (int k = 0; k < K; ++k) {
    if (branching[k] < 1) return MEDUSA_EINVAL;
    if (branching[k] > MEDUSA_MAX_TOPK) return MEDUSA_EUNSUPPORTED;
    level *= branching[k];
    total += level;
    if (total + 1 > MEDUSA_MAX_TREE_TOKENS) return MEDUSA_EUNSUPPORTED;
  }
  std::vector<Node> cand, frontier, next;
  Node root;
  root.r.fill(-1);
  root.len = 0;
  frontier.push_back(root);
  for (int k = 0; k < K; ++k) {
    next.clear();
    for (const Node& p : frontier)
      for (int r = 0; r < branching[k]; ++r) {
        Node c = p;
        c.r[c.len++] = r;
        next.push_back(c);
      }
    cand.insert(cand.end(), next.begin(), next.end());
    frontier.swap(next);
  }
  return build(cand, K, out);
}

extern "C" int medusa_tree_create_nodes(const int32_t* ranks, int n_nodes, int K, medusa_tree_t** out) {
  if (!out || n_nodes < 0 || K < 0 || (n_nodes > 0 && !ranks)) return MEDUSA_EINVAL;
  if (K > MEDUSA_MAX_HEADS || n_nodes + 1 > MEDUSA_MAX_TREE_TOKENS) return MEDUSA_EUNSUPPORTED;
  if (n_nodes > 0 && K == 0) return MEDUSA_EINVAL;
  std::vector<Node> cand;
  for (int i = 0; i < n_nodes; ++i) {
    Node n;
    n.r.fill(-1);
    n.len = 0;
    bool ended = false;
    for (int k = 0; k < K; ++k) {
      const int32_t r = ranks[(size_t)i * K + k];
      if (r < 0) {
        ended = true;
        continue;
      }
      if (ended) return MEDUSA_EINVAL;  // a rank after the -1 padding began
      if (r >= MEDUSA_MAX_TOPK) return MEDUSA_EUNSUPPORTED;
      n.r[n.len++] = r;
    }
    if (n.len == 0) return MEDUSA_EINVAL;  // the root is implicit
    cand.push_back(n);
  }
  return build(cand, K, out);
}

// Sec. 2.3.3: with a_k^(i) the accuracy of the i-th best prediction of head k, a node
// (i_1..i_k) is estimated to be correct with probability prod_j a_j^(i_j) and adds exactly that
// much to the expected acceptance length, so the best tree of a given size is grown greedily:
// repeatedly add the not-yet-included child of an included node with the highest estimate.
// Ties: shallower node first, then the lexicographically smaller rank tuple.
extern "C" int medusa_tree_create_optimized(const double* accuracy, int K, int S, int n_nodes, medusa_tree_t** out,
                                            double* expected_accept_len) {
  if (!accuracy || !out || K < 1 || S < 1 || n_nodes < 0) return MEDUSA_EINVAL;
  if (K > MEDUSA_MAX_HEADS || S > MEDUSA_MAX_TOPK || n_nodes + 1 > MEDUSA_MAX_TREE_TOKENS) return MEDUSA_EUNSUPPORTED;
  for (int i = 0; i < K * S; ++i)
    if (!(accuracy[i] >= 0.0 && accuracy[i] <= 1.0)) return MEDUSA_EINVAL;
  struct Cand {
    Node n;
    double p;
  };
  auto better = [](const Cand& a, const Cand& b) {   // strict "a is chosen before b"
    if (a.p != b.p) return a.p > b.p;
    return node_less(a.n, b.n);
  };
  std::vector<Cand> frontier, chosen;
  Node root;
  root.r.fill(-1);
  root.len = 0;
  auto push_children = [&](const Node& parent, double p) {
    if (parent.len >= K) return;
    for (int r = 0; r < S; ++r) {
      Cand c;
      c.n = parent;
      c.n.r[c.n.len++] = r;
      c.p = p * accuracy[(size_t)parent.len * S + r];
      frontier.push_back(c);
    }
  };
  push_children(root, 1.0);
  double expect = 1.0;                                // the root is always accepted
  while ((int)chosen.size() < n_nodes && !frontier.empty()) {
    size_t best = 0;
    for (size_t i = 1; i < frontier.size(); ++i)
      if (better(frontier[i], frontier[best])) best = i;
    const Cand c = frontier[best];
    frontier.erase(frontier.begin() + best);
    chosen.push_back(c);
    expect += c.p;
    push_children(c.n, c.p);
  }
  if ((int)chosen.size() < n_nodes) return MEDUSA_EINVAL;   // fewer than n_nodes nodes exist for this K, S
  std::vector<Node> cand;
  int depth = 0;
  for (const Cand& c : chosen) {
    cand.push_back(c.n);
    depth = std::max(depth, c.n.len);
  }
  if (expected_accept_len) *expected_accept_len = expect;
  return build(cand, depth, out);
}

extern "C" int medusa_tree_destroy(medusa_tree_t* tree) {
  if (!tree) return MEDUSA_EINVAL;
  int rc = MEDUSA_OK;
  if (tree->dev && hipFree(tree->dev) != hipSuccess) rc = MEDUSA_EHIP;
  delete[] tree->paths;
  delete tree;
  return rc;
}

extern "C" int medusa_tree_query(const medusa_tree_t* tree, int32_t* T, int32_t* K, int32_t* n_leaves, int32_t* S,
                                 int32_t* topk_per_head) {
  if (!tree) return MEDUSA_EINVAL;
  if (T) *T = tree->host.T;
  if (K) *K = tree->host.K;
  if (n_leaves) *n_leaves = tree->host.n_leaves;
  if (S) *S = tree->host.S;
  if (topk_per_head)
    for (int k = 0; k < tree->host.K; ++k) topk_per_head[k] = tree->host.topk_per_head[k];
  return MEDUSA_OK;
}

extern "C" int medusa_tree_tables(const medusa_tree_t* tree, int32_t* parent, int32_t* depth, int32_t* rank,
                                  int32_t* token_src, uint64_t* anc_mask, int32_t* paths) {
  if (!tree) return MEDUSA_EINVAL;
  const TreeTables& h = tree->host;
  const size_t n = (size_t)h.T * sizeof(int32_t);
  if (parent) std::memcpy(parent, h.parent, n);
  if (depth) std::memcpy(depth, h.depth, n);
  if (rank) std::memcpy(rank, h.rank, n);
  if (token_src) std::memcpy(token_src, h.token_src, n);
  if (anc_mask) std::memcpy(anc_mask, h.anc_mask, (size_t)h.T * 2 * sizeof(uint64_t));
  if (paths) std::memcpy(paths, tree->paths, (size_t)h.n_leaves * (h.K + 1) * sizeof(int32_t));
  return MEDUSA_OK;
}
