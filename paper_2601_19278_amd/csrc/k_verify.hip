// Glue between the drafted tree and the target model's verification pass (paper Sec. 2.1,
// Fig. 3 "Tree Attention"): position ids of the tree nodes, and the temperature-0 acceptance
// walk over the tree given the target model's own next token at every node.
//
// One wavefront per sequence.  A tree has at most DART_MAX_BUDGET = 128 nodes, two per lane.
// Parents precede children in the node order the pruning kernel emits, and a node is at most
// DART_MAX_K edges below the root, so every walk here is bounded.
#include "common.h"
#include "dart_internal.h"

namespace dart {

__global__ __launch_bounds__(64) void tree_verify_kernel(
    const int32_t *__restrict__ tokens, const int32_t *__restrict__ parents,
    const int32_t *__restrict__ n_nodes, const int32_t *__restrict__ target_next,
    const int32_t *__restrict__ ctx_len, int budget, int path_cap,
    int32_t *__restrict__ position_ids, int32_t *__restrict__ accept_path,
    int32_t *__restrict__ n_accepted, int32_t *__restrict__ next_token) {
  const int seq = blockIdx.x, lane = threadIdx.x;
  tokens += (size_t)seq * budget;
  parents += (size_t)seq * budget;
  const int n = min(max(n_nodes[seq], 0), budget);

  // position ids: prefix length + depth below the root
  if (position_ids) {
    const int base = ctx_len ? ctx_len[seq] : 0;
    for (int i = lane; i < budget; i += 64) {
      int depth = -1;
      if (i < n) {
        depth = 0;
        int j = i;
        for (int hops = 0; hops <= DART_MAX_K; ++hops) {   // bounded walk
          const int p = parents[j];
          if (p < 0 || p >= n) break;
          j = p;
          ++depth;
        }
      }
      position_ids[(size_t)seq * budget + i] = depth < 0 ? -1 : base + depth;
    }
  }
  if (!target_next) return;
  target_next += (size_t)seq * budget;
  accept_path += (size_t)seq * path_cap;

  // acceptance walk: among the children of the current node, the one carrying the target's
  // token (sibling tokens are distinct; the lowest node index wins otherwise)
  int tok[2], par[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int i = lane + 64 * q;
    tok[q] = i < n ? tokens[i] : -1;
    par[q] = i < n ? parents[i] : -2;
  }
  int cur = 0, len = 1;
  if (lane == 0) accept_path[0] = 0;
  int want = target_next[0];
  while (len < path_cap) {
    const uint64_t m0 = __ballot(par[0] == cur && tok[0] == want);
    const uint64_t m1 = __ballot(par[1] == cur && tok[1] == want);
    int nxt = -1;
    if (m0) nxt = __ffsll((unsigned long long)m0) - 1;
    else if (m1) nxt = 64 + __ffsll((unsigned long long)m1) - 1;
    if (nxt < 0) break;
    if (lane == 0) accept_path[len] = nxt;
    cur = nxt;
    want = target_next[cur];
    ++len;
  }
  for (int i = len + lane; i < path_cap; i += 64) accept_path[i] = -1;
  if (lane == 0) {
    n_accepted[seq] = len - 1;
    next_token[seq] = want;
  }
}

hipError_t launch_tree_verify(int batch, const int32_t *tokens, const int32_t *parents,
                              const int32_t *n_nodes, const int32_t *target_next,
                              const int32_t *ctx_len, int budget, int path_cap,
                              int32_t *position_ids, int32_t *accept_path, int32_t *n_accepted,
                              int32_t *next_token, hipStream_t st) {
  hipLaunchKernelGGL(tree_verify_kernel, dim3(batch), dim3(64), 0, st, tokens, parents, n_nodes,
                     target_next, ctx_len, budget, path_cap, position_ids, accept_path, n_accepted,
                     next_token);
  return hipGetLastError();
}

}  // namespace dart
