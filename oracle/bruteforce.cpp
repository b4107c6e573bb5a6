// Exhaustive search over every assignment of a tiny instance (N <= 8 actions), used to report
// the optimality gap of the greedy eviction heuristic (Alg. 1 of ARL-Tangram, arXiv 2603.13019).
//
// TEST INFRASTRUCTURE ONLY, written separately from tangram_oracle.cpp: durations come in as a
// table, the completion "heap" is a sorted vector, and there is no dynamic program at all.
//
// Every action gets a home node and either a unit count (it starts now) or "wait" (it is
// estimated by sequential insertion at its minimum units, Alg. 2).  The value of an assignment is
//   sum over started actions of (backlog[node] + dur)  +  sum over nodes of estimate(waiting there)
// which is Eq. 2 with the paper's approximation for the actions left in the queue.
#include <algorithm>
#include <cstdint>
#include <vector>

namespace {
constexpr int64_t INF = INT64_MAX;
struct Inst { int N, M, K, depth; const int32_t* k_list; const int64_t* dur; const int32_t* free_units; const int64_t* backlog; };

int64_t wait_cost(const Inst& in, int node, std::vector<int64_t> rel, const std::vector<int>& waiting) {
  const int H = (int)rel.size();
  std::vector<int> w;
  for (int i : waiting) {
    bool any = false;
    for (int q = 0; q < in.K; ++q) any |= in.dur[i * in.K + q] != INF && in.k_list[q] <= H;
    if (any) w.push_back(i);
  }
  if (w.empty()) return 0;
  int64_t best = INF;
  for (int d = 1; d <= in.depth; ++d) {
    std::vector<int64_t> r = rel;
    int64_t obj = 0; bool valid = true;
    for (size_t x = 0; x < w.size() && valid; ++x) {
      const int i = w[x];
      int want = x == 0 ? d : 1, q = -1;
      for (int c = 0; c < in.K; ++c)
        if (in.dur[i * in.K + c] != INF && in.k_list[c] <= H && --want == 0) { q = c; break; }
      if (q < 0) { valid = false; break; }
      const int u = in.k_list[q];
      std::sort(r.begin(), r.end());
      const int64_t fin = r[u - 1] + in.dur[i * in.K + q];
      for (int c = 0; c < u; ++c) r[c] = fin;
      obj += fin;
    }
    if (valid) best = std::min(best, obj);
  }
  return best;
}

int64_t value(const Inst& in, const int* node, const int* opt /* -1 = wait */) {
  int64_t total = 0;
  for (int j = 0; j < in.M; ++j) {
    std::vector<int64_t> rel; std::vector<int> waiting; int used = 0;
    for (int i = 0; i < in.N; ++i) {
      if (node[i] != j) continue;
      if (opt[i] < 0) { waiting.push_back(i); continue; }
      const int k = in.k_list[opt[i]];
      const int64_t fin = in.backlog[j] + in.dur[i * in.K + opt[i]];
      total += fin; used += k;
      for (int c = 0; c < k; ++c) rel.push_back(fin);
    }
    if (used > in.free_units[j]) return INF;
    for (int c = used; c < in.free_units[j]; ++c) rel.push_back(in.backlog[j]);
    total += wait_cost(in, j, rel, waiting);
  }
  return total;
}

void search(const Inst& in, int i, std::vector<int>& node, std::vector<int>& opt, std::vector<int>& used,
            int64_t& best, std::vector<int>& bnode, std::vector<int>& bopt, bool all_start) {
  if (i == in.N) {
    const int64_t v = value(in, node.data(), opt.data());
    if (v < best) { best = v; bnode = node; bopt = opt; }
    return;
  }
  for (int j = 0; j < in.M; ++j) {
    node[i] = j;
    if (!all_start) { opt[i] = -1; search(in, i + 1, node, opt, used, best, bnode, bopt, all_start); }
    for (int q = 0; q < in.K; ++q) {
      if (in.dur[i * in.K + q] == INF || used[j] + in.k_list[q] > in.free_units[j]) continue;
      opt[i] = q; used[j] += in.k_list[q];
      search(in, i + 1, node, opt, used, best, bnode, bopt, all_start);
      used[j] -= in.k_list[q];
    }
  }
}
}  // namespace

extern "C" {
int64_t bf_value(int N, int M, int K, int depth, const int32_t* k_list, const int64_t* dur, const int32_t* free_units,
                 const int64_t* backlog, const int32_t* node, const int32_t* opt) {
  Inst in{N, M, K, depth, k_list, dur, free_units, backlog};
  return value(in, node, opt);
}
int64_t bf_best(int N, int M, int K, int depth, const int32_t* k_list, const int64_t* dur, const int32_t* free_units,
                const int64_t* backlog, int all_start, int32_t* node_out, int32_t* opt_out) {
  Inst in{N, M, K, depth, k_list, dur, free_units, backlog};
  std::vector<int> node(N, 0), opt(N, -1), used(M, 0), bn(N, -1), bo(N, -1);
  int64_t best = INF;
  search(in, 0, node, opt, used, best, bn, bo, all_start != 0);
  for (int i = 0; i < N; ++i) { node_out[i] = bn[i]; opt_out[i] = bo[i]; }
  return best;
}
}
