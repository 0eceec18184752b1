// Planning steps of the execute-while-load scheme as pure integer functions (host code):
// which order a sub-group receives the model's blocks in (Section 4.2, Algorithm 1), how N
// nodes are dealt into k sub-groups, which nodes form which execution pipeline (Section 4.3,
// Algorithm 2), how many steps a binomial-pipeline multicast takes (Section 4.2) and one
// schedule that takes exactly that many.  The loader accepts blocks in any order; these
// functions say which order a cluster would send.
#include "../../include/ls_stage.h"
#include "kernels.hpp"

#include <cstdint>
#include <vector>

namespace {

ls_status bad(const char* what) {
  ls::set_last_error("%s", what);
  return LS_ERR_INVALID_ARG;
}

// chunk c of b blocks cut into k pieces of ceil(b/k) (trailing pieces may be short or empty)
inline void span_of(int b, int k, int c, int* lo, int* hi) {
  const int piece = (b + k - 1) / k;
  const long first = (long)piece * c, last = first + piece;
  *lo = (int)(first < b ? first : b);
  *hi = (int)(last < b ? last : b);
}

}  // namespace

extern "C" {

ls_status ls_plan_chunk_span(int n_blocks, int k, int chunk, int* lo, int* hi) {
  if (n_blocks < 1 || k < 1 || chunk < 0 || chunk >= k || !lo || !hi) return bad("ls_plan_chunk_span: bad arguments");
  span_of(n_blocks, k, chunk, lo, hi);
  return LS_OK;
}

ls_status ls_plan_kway_order(int n_blocks, int k, int group, int32_t* order) {
  if (n_blocks < 1 || k < 1 || group < 0 || group >= k || !order) return bad("ls_plan_kway_order: bad arguments");
  int w = 0;
  // walk the ring of chunks once, starting at the group's own chunk
  for (int c = group, seen = 0; seen < k; ++seen, c = (c + 1 == k ? 0 : c + 1)) {
    int lo, hi;
    span_of(n_blocks, k, c, &lo, &hi);
    while (lo < hi) order[w++] = lo++;
  }
  return LS_OK;
}

ls_status ls_plan_subgroup_sizes(int n_nodes, int k, int32_t* sizes) {
  if (n_nodes < 1 || k < 1 || k > n_nodes || !sizes) return bad("ls_plan_subgroup_sizes: bad arguments");
  const int q = n_nodes / k, r = n_nodes % k;
  for (int i = 0; i < k; ++i) sizes[i] = q + (i < r);
  return LS_OK;
}

ls_status ls_plan_pipelines(const int32_t* sizes, int k, int32_t* group_out, int32_t* index_out, int32_t* pipe_start,
                            int capacity, int* n_pipes) {
  if (!sizes || k < 1 || !group_out || !index_out || !pipe_start || !n_pipes || capacity < 0)
    return bad("ls_plan_pipelines: bad arguments");
  long total = 0;
  for (int i = 0; i < k; ++i) {
    if (sizes[i] < 0) return bad("ls_plan_pipelines: negative sub-group size");
    total += sizes[i];
  }
  if (total > capacity) {
    ls::set_last_error("ls_plan_pipelines: %ld nodes, room for %d", total, capacity);
    return LS_ERR_OOM;
  }
  // A pipeline takes the t-th node of every sub-group that has one (sub-group order); the
  // deepest sub-group's surplus nodes, which would stand alone, form one last pipeline.
  int deepest = 0, second = 0, who = -1;  // largest and second-largest size
  for (int i = 0; i < k; ++i) {
    if (sizes[i] > deepest) { second = deepest; deepest = sizes[i]; who = i; }
    else if (sizes[i] > second) second = sizes[i];
  }
  int w = 0, np = 0;
  for (int t = 0; t < second; ++t) {
    pipe_start[np++] = w;
    for (int i = 0; i < k; ++i)
      if (sizes[i] > t) { group_out[w] = i; index_out[w] = t; ++w; }
  }
  if (deepest > second) {
    pipe_start[np++] = w;
    for (int t = second; t < deepest; ++t) { group_out[w] = who; index_out[w] = t; ++w; }
  }
  pipe_start[np] = w;
  *n_pipes = np;
  return LS_OK;
}

int ls_plan_multicast_steps(int n_blocks, int n_nodes) {
  if (n_blocks < 1 || n_nodes < 1) return (int)bad("ls_plan_multicast_steps: bad arguments");
  int doublings = 0;
  for (long reach = 1; reach < n_nodes; reach <<= 1) ++doublings;
  return n_blocks + doublings - 1;
}

ls_status ls_plan_multicast_schedule(int n_blocks, int n_nodes, int32_t* dest, int32_t* block, int capacity_steps,
                                     int* n_steps) {
  if (n_blocks < 1 || n_nodes < 2 || (n_nodes & (n_nodes - 1)) || !dest || !block || !n_steps || capacity_steps < 0)
    return bad("ls_plan_multicast_schedule: bad arguments (n_nodes must be a power of two >= 2)");
  int dims = 0;
  while ((1 << dims) < n_nodes) ++dims;
  const int steps = n_blocks + dims - 1;
  if (steps > capacity_steps) {
    ls::set_last_error("ls_plan_multicast_schedule: %d steps, room for %d", steps, capacity_steps);
    return LS_ERR_OOM;
  }
  // held[u] = bitmap of the blocks node u holds, 64 per word; node 0 starts with all of them
  const int words = (n_blocks + 63) / 64;
  std::vector<uint64_t> held((size_t)n_nodes * words, 0), next;
  for (int k = 0; k < n_blocks; ++k) held[k >> 6] |= 1ull << (k & 63);
  for (int s = 0; s < steps; ++s) {
    const int bit = 1 << (s % dims);
    next = held;  // transfers of a step take effect together
    for (int u = 0; u < n_nodes; ++u) {
      const int v = u ^ bit;
      const uint64_t* hu = &held[(size_t)u * words];
      const uint64_t* hv = &held[(size_t)v * words];
      int pick = -1;
      const int fresh = s < n_blocks ? s : n_blocks - 1;  // what the source injects at this step
      if (u == 0 && !((hv[fresh >> 6] >> (fresh & 63)) & 1)) pick = fresh;
      for (int w = words - 1; w >= 0 && pick < 0; --w) {
        const uint64_t useful = hu[w] & ~hv[w];
        if (useful) pick = w * 64 + 63 - __builtin_clzll(useful);
      }
      dest[(size_t)s * n_nodes + u] = pick < 0 ? -1 : v;
      block[(size_t)s * n_nodes + u] = pick;
      if (pick >= 0) next[(size_t)v * words + (pick >> 6)] |= 1ull << (pick & 63);
    }
    held.swap(next);
  }
  // the construction meets the step count of Section 4.2: every node now holds every block
  for (int u = 0; u < n_nodes; ++u)
    for (int k = 0; k < n_blocks; ++k)
      if (!((held[(size_t)u * words + (k >> 6)] >> (k & 63)) & 1)) {
        ls::set_last_error("ls_plan_multicast_schedule: node %d lacks block %d after %d steps", u, k, steps);
        return LS_ERR_INVALID_ARG;
      }
  *n_steps = steps;
  return LS_OK;
}

}  // extern "C"
