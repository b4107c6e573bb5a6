// CPU oracle of the action-level elastic scheduling step (ARL-Tangram, arXiv 2603.13019).
//
// TEST INFRASTRUCTURE ONLY.  A plain, single-threaded, deliberately unoptimised
// restatement of what the scheduling step computes, written from the paper:
//   * Eq. 1 (Sec. 4.1)      duration of an action on m units, in integer microseconds
//   * Eq. 2 (Sec. 4.2)      action completion time = queueing + execution
//   * Alg. 1 (Sec. 4.2)     FCFS candidate prefix at minimum units, greedy tail eviction
//   * Alg. 2 (App. A)       approximated objective: exact part + completion-heap estimate
//   * Alg. 3 (App. B)       DPArrange over used units (basic operator)
//   * Alg. 4 (App. B)       DPArrange over free-chunk states (GPU operator, sizes 1/2/4/8)
//   * Sec. 5.1-5.3          capacity models: quota, per-node cores + trajectory pin, buddy chunks
//   * Sec. 5.2              which cores an action gets: one NUMA domain if any can hold it
//   * Sec. 5.3 + Alg. 4      optionally the whole GPU cluster as one pool of chunks
// It shares no code, header, table or helper with the HIP library; only tests, the
// smoke check and the benchmark's CPU-baseline leg may call it.
//
// Every function below is pinned by tests against closed forms, brute force or an
// independent second algorithm (tests/test_oracle_*.py); none is "parity unpinned".
//
// Integer conventions: times are int64 microseconds relative to the snapshot instant,
// durations are rounded up and never below 1, INF = INT64_MAX marks "not a candidate".

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <functional>
#include <queue>
#include <vector>

namespace {

constexpr int64_t INF = INT64_MAX;
enum { T_CPU = 0, T_GPU = 1, T_API = 2, N_TYPES = 3 };
enum { R_NONE = 0, R_PREFIX = 1, R_EVICTED = 2, R_INFEASIBLE = 3 };

struct Tables {
  int K;
  const int32_t* k_list;       // ascending unit counts
  const int32_t* type_k;       // how many leading entries of k_list each type may use
  const uint32_t* speedup_q16; // [class][q] = round(65536 * E(k_q) * k_q)
  int depth;
  const int64_t* restore_us = nullptr;   // [service] time to bring a service back from host memory
};

struct Act {
  int type, model;
  int64_t T, age;
  uint32_t kmask, param;
  int pin, task;
  int aux = 0;                 // second component of the cost vector (Sec. 4.1), e.g. memory with CPU cores
  int service = -1;            // long-lived service the action calls (Sec. 5.3), -1: none
  uint64_t extra = 0;          // further quotas the action draws one token from each (Sec. 4.1), by rank among the API nodes
};

struct Node {
  int type, cap, free;
  int aux_free = INT32_MAX;    // what the node has left of the second resource
  uint64_t resident = 0;       // bit s set: service s is cached in the node's device memory (Sec. 5.3)
  int64_t backlog;
  int chunks[4];               // free chunks of size 1,2,4,8 (GPU nodes)
  std::vector<int64_t> busy;   // release time of every unit held by a running action
  std::vector<char> core_free; // [cap] 1: the core is free (CPU nodes of a problem that gives the core topology)
};

// ---- Eq. 1: getDur(m) = T_ori / (E(m) * m), rounded up to whole microseconds -------------
int64_t duration(const Tables& tb, const Act& a, int q) {
  const int64_t k = tb.k_list[q];
  if (a.model == 0) return a.T;                       // elasticity unknown: constant
  unsigned __int128 num, den;
  if (a.model == 1) {                                 // Amdahl: E(k) = 1 / ((1-p) k + p)
    const int64_t p = a.param;                        // parallel fraction in ppm
    num = (unsigned __int128)a.T * (unsigned __int128)((1000000 - p) * k + p);
    den = (unsigned __int128)1000000 * k;
  } else {                                            // table: E(k) k = speedup / 65536
    num = (unsigned __int128)a.T * 65536u;
    den = tb.speedup_q16[(size_t)a.param * tb.K + q];
  }
  int64_t d = (int64_t)((num + den - 1) / den);
  return d < 1 ? 1 : d;
}

// Sec. 5.3 (evict on execution): an action whose service is resident on the node runs at once;
// otherwise the service is restored from host memory first, which delays the action by the
// service's restore time on that node.
int64_t restore_delay(const Tables& tb, const Act& a, const Node& nd) {
  if (a.service < 0 || !tb.restore_us || (nd.resident >> a.service & 1ull)) return 0;
  return tb.restore_us[a.service];
}

// allowed option indices of an action (Sec. 4.1: the discrete set of unit counts)
std::vector<int> options(const Tables& tb, const Act& a) {
  std::vector<int> o;
  for (int q = 0; q < tb.type_k[a.type]; ++q)
    if (a.kmask >> q & 1u) {
      o.push_back(q);
      if (a.model == 0) break;                        // non-elastic: minimum units only
    }
  return o;
}

std::vector<int> options_on(const Tables& tb, const Act& a, const Node& nd) {
  std::vector<int> o;
  for (int q : options(tb, a))
    if (tb.k_list[q] <= nd.cap) o.push_back(q);
  return o;
}

// ---- Sec. 5.3: chunk allocation on counts of free chunks --------------------------------
int chunk_level(int k) { int a = 0; while ((1 << a) < k) ++a; return a; }

bool chunk_fits(const int c[4], int k) {
  for (int b = chunk_level(k); b < 4; ++b) if (c[b] > 0) return true;
  return false;
}

bool chunk_take(int c[4], int k) {                    // smallest chunk of level >= a, split down
  const int a = chunk_level(k);
  if (a > 3) return false;
  for (int b = a; b < 4; ++b)
    if (c[b] > 0) {
      --c[b];
      for (int x = a; x < b; ++x) ++c[x];
      return true;
    }
  return false;
}

// ---- Sec. 5.2: the set of cores of an action ----------------------------------------------
// Cores [d*numa, (d+1)*numa) form NUMA domain d.  The manager names the cores an action runs
// on and prefers cores of one domain.  Reading used here: if some domain has k free cores, take
// the domain with the fewest free cores among those (the least leftover; lowest domain on ties);
// otherwise take whole domains, the one with the most free cores first (lowest on ties), which
// spans as few domains as k cores can; inside a domain the lowest-numbered free cores go first.
// Returns the chosen cores in increasing order and clears them in `free_`.
std::vector<int> take_cores(std::vector<char>& free_, int numa, int k) {
  const int cap = (int)free_.size(), D = (cap + numa - 1) / numa;
  auto count = [&](int d) { int c = 0; for (int x = d * numa; x < std::min(cap, (d + 1) * numa); ++x) c += free_[x]; return c; };
  std::vector<int> got;
  auto take_from = [&](int d, int want) {
    for (int x = d * numa; x < std::min(cap, (d + 1) * numa) && want > 0; ++x)
      if (free_[x]) { free_[x] = 0; got.push_back(x); --want; }
  };
  int best = -1;
  for (int d = 0; d < D; ++d) {
    const int c = count(d);
    if (c >= k && (best < 0 || c < count(best))) best = d;
  }
  if (best >= 0) take_from(best, k);
  else {
    int left = k;
    while (left > 0) {
      int big = -1;
      for (int d = 0; d < D; ++d) if (count(d) > 0 && (big < 0 || count(d) > count(big))) big = d;
      if (big < 0) break;                              // fewer than k free cores: the caller never asks for that
      const int c = std::min(count(big), left);
      take_from(big, c);
      left -= c;
    }
  }
  std::sort(got.begin(), got.end());
  return got;
}

// ---- Alg. 3: DPArrange with the basic operator (state = units used) ----------------------
// dur[i*K+q] = duration of task i with k_list[q] units, INF if the option is not allowed.
int64_t dp_units(int m, const int64_t* dur, const int32_t* k_list, int K, int U, int32_t* k_out) {
  int64_t sum_max = 0;
  for (int i = 0; i < m; ++i) {
    int mx = 0;
    for (int q = 0; q < K; ++q) if (dur[(size_t)i * K + q] != INF) mx = k_list[q];
    sum_max += mx;
  }
  const int n = (int)std::min<int64_t>(U, sum_max);
  std::vector<std::vector<int64_t>> dp(m + 1, std::vector<int64_t>(n + 1, INF));
  std::vector<std::vector<int>> choice(m + 1, std::vector<int>(n + 1, -1));
  dp[0][0] = 0;
  for (int i = 1; i <= m; ++i)
    for (int j = 0; j <= n; ++j)
      for (int q = 0; q < K; ++q) {
        const int64_t t = dur[(size_t)(i - 1) * K + q];
        const int jp = j - k_list[q];
        if (t == INF || jp < 0 || dp[i - 1][jp] == INF) continue;
        if (dp[i - 1][jp] + t < dp[i][j]) { dp[i][j] = dp[i - 1][jp] + t; choice[i][j] = q; }
      }
  int js = -1;
  for (int j = 0; j <= n; ++j) if (dp[m][j] != INF && (js < 0 || dp[m][j] < dp[m][js])) js = j;
  if (js < 0) return INF;
  const int64_t best = dp[m][js];
  for (int i = m, j = js; i >= 1; --i) {
    const int q = choice[i][j];
    if (k_out) k_out[i - 1] = k_list[q];
    j -= k_list[q];
  }
  return best;
}

// ---- Alg. 3 with Alg. 4's operator (state = encoded counts of free chunks) ---------------
struct Radix { int n[4]; int size() const { return (n[0]+1)*(n[1]+1)*(n[2]+1)*(n[3]+1); } };
int encode(const Radix& r, const int c[4]) {
  return c[0] + (r.n[0]+1) * (c[1] + (r.n[1]+1) * (c[2] + (r.n[2]+1) * c[3]));
}
void decode(const Radix& r, int j, int c[4]) {
  c[0] = j % (r.n[0]+1); j /= (r.n[0]+1);
  c[1] = j % (r.n[1]+1); j /= (r.n[1]+1);
  c[2] = j % (r.n[2]+1); j /= (r.n[2]+1);
  c[3] = j;
}

int64_t dp_chunks(int m, const int64_t* dur, const int32_t* k_list, int K, const int start[4], int32_t* k_out) {
  Radix r;                                            // a split never leaves two equal new chunks
  for (int x = 0; x < 4; ++x) r.n[x] = std::max(start[x], 1);
  const int S = r.size();
  std::vector<std::vector<int64_t>> dp(m + 1, std::vector<int64_t>(S, INF));
  std::vector<std::vector<int>> from(m + 1, std::vector<int>(S, -1)), opt(m + 1, std::vector<int>(S, -1));
  dp[0][encode(r, start)] = 0;
  for (int i = 1; i <= m; ++i)
    for (int s = 0; s < S; ++s) {
      if (dp[i - 1][s] == INF) continue;
      for (int q = 0; q < K; ++q) {
        const int64_t t = dur[(size_t)(i - 1) * K + q];
        if (t == INF) continue;
        int c[4]; decode(r, s, c);
        if (!chunk_take(c, k_list[q])) continue;
        const int s2 = encode(r, c);
        if (dp[i - 1][s] + t < dp[i][s2]) { dp[i][s2] = dp[i - 1][s] + t; from[i][s2] = s; opt[i][s2] = q; }
      }
    }
  int ss = -1;
  for (int s = 0; s < S; ++s) if (dp[m][s] != INF && (ss < 0 || dp[m][s] < dp[m][ss])) ss = s;
  if (ss < 0) return INF;
  const int64_t best = dp[m][ss];
  for (int i = m, s = ss; i >= 1; --i) {
    if (k_out) k_out[i - 1] = k_list[opt[i][s]];
    s = from[i][s];
  }
  return best;
}

// ---- Alg. 2, estimate(): sequential insertion into the completion heap -------------------
// heap: release time of every unit; ac_dur[a*K+q]: durations of the waiting actions (INF = not
// allowed); all but the first use their minimum units, the first tries its d-th smallest option.
int64_t estimate(const std::vector<int64_t>& heap0, int n_ac, const int64_t* ac_dur,
                 const int32_t* k_list, int K, int depth) {
  const int H = (int)heap0.size();
  std::vector<std::vector<int>> opts;                 // usable options per waiting action
  std::vector<int> keep;
  for (int a = 0; a < n_ac; ++a) {
    std::vector<int> o;
    for (int q = 0; q < K; ++q) if (ac_dur[(size_t)a * K + q] != INF && k_list[q] <= H) o.push_back(q);
    if (!o.empty()) { keep.push_back(a); opts.push_back(o); }   // cannot ever fit: left out
  }
  if (keep.empty()) return 0;
  int64_t best = INF;
  for (int d = 1; d <= depth; ++d) {
    if ((int)opts[0].size() < d) break;
    std::priority_queue<int64_t, std::vector<int64_t>, std::greater<int64_t>> h(heap0.begin(), heap0.end());
    int64_t obj = 0;
    for (size_t x = 0; x < keep.size(); ++x) {
      const int q = (x == 0) ? opts[0][d - 1] : opts[x][0];
      const int u = k_list[q];
      int64_t ts = 0;
      for (int c = 0; c < u; ++c) { ts = h.top(); h.pop(); }    // start when the u-th unit frees
      const int64_t fin = ts + ac_dur[(size_t)keep[x] * K + q];
      for (int c = 0; c < u; ++c) h.push(fin);
      obj += fin;
    }
    best = std::min(best, obj);
  }
  return best;
}

struct StepOut {
  std::vector<int32_t> node, units;
  std::vector<int64_t> act;
  std::vector<uint8_t> reason;
  std::vector<int64_t> node_obj;                      // final approximated objective per node, -1 if none
  std::vector<int32_t> home;                          // node an action was admitted to (kept when evicted)
  std::vector<std::vector<int>> cores;                // cores of every selected CPU action (numa_cores > 0)
  std::vector<int32_t> extra_used;                    // tokens taken from a quota by actions of other quotas
  std::vector<int> visit;                             // the order in which the queue was visited (a permutation of 0..N-1)
};

// Order in which a pool's waiting queue is visited (Sec. 4.2: FCFS in the paper, which notes
// that the algorithm also runs on top of other orderings).  ORDER_COST is one such other order:
// ascending least estimated ACT (Eq. 2) over the action's candidates at the snapshot, i.e. the
// smallest entry of its row of the score tensor; equal keys keep their FCFS rank.
enum { ORDER_FCFS = 0, ORDER_COST = 1 };

// ---- one scheduling step on one snapshot (Alg. 1 applied per resource pool) -------------
StepOut step(const Tables& tb, const std::vector<Act>& acts, std::vector<Node> nodes, int order_policy = ORDER_FCFS,
             int numa_cores = 0, bool gpu_pooled = false, bool queue_prefix = false) {
  const int N = (int)acts.size(), M = (int)nodes.size(), K = tb.K;
  // Sec. 5.3 / Alg. 4: the GPU manager runs the algorithm for the GPU cluster as a whole, and the
  // state of Alg. 4 counts the chunks of every size it has, whichever node they are on.  In that
  // mode the first GPU node stands for the pool: it gets the chunks, units and running actions of
  // all GPU nodes (which share one backlog), the others have nothing left to give.  The nodes
  // themselves come back at the end, when every selected action is given a real chunk.
  std::vector<std::vector<int>> real_chunks(M, std::vector<int>(4, 0));
  int pool = -1;
  if (gpu_pooled)
    for (int j = 0; j < M; ++j) {
      if (nodes[j].type != T_GPU) continue;
      for (int x = 0; x < 4; ++x) real_chunks[j][x] = nodes[j].chunks[x];
      if (pool < 0) { pool = j; continue; }
      Node& P = nodes[pool];
      P.cap += nodes[j].cap; P.free += nodes[j].free;
      for (int x = 0; x < 4; ++x) { P.chunks[x] += nodes[j].chunks[x]; nodes[j].chunks[x] = 0; }
      P.busy.insert(P.busy.end(), nodes[j].busy.begin(), nodes[j].busy.end());
      nodes[j].free = 0; nodes[j].busy.clear();
    }
  StepOut o;
  o.node.assign(N, -1); o.units.assign(N, 0); o.act.assign(N, -1); o.reason.assign(N, R_NONE);
  o.node_obj.assign(M, -1); o.home.assign(N, -1); o.cores.assign(N, {}); o.extra_used.assign(M, 0);

  // static infeasibility: no option, bad pin, or minimum units above every candidate node
  std::vector<int> kmin(N, 0);
  for (int i = 0; i < N; ++i) {
    const Act& a = acts[i];
    std::vector<int> op = options(tb, a);
    bool ok = !op.empty();
    if (ok) {
      kmin[i] = tb.k_list[op[0]];
      if (a.pin >= 0) ok = a.pin < M && nodes[a.pin].type == a.type && kmin[i] <= nodes[a.pin].cap;
      else {
        ok = false;
        for (int j = 0; j < M; ++j) if (nodes[j].type == a.type && kmin[i] <= nodes[j].cap) ok = true;
      }
    }
    if (!ok) o.reason[i] = R_INFEASIBLE;
  }

  std::vector<int> visit(N);
  for (int i = 0; i < N; ++i) visit[i] = i;
  if (order_policy == ORDER_COST) {
    std::vector<int64_t> key(N, INF);
    for (int i = 0; i < N; ++i) {
      if (o.reason[i] == R_INFEASIBLE) continue;
      const Act& a = acts[i];
      for (int j = 0; j < M; ++j) {
        if (nodes[j].type != a.type || (a.pin >= 0 && a.pin != j)) continue;
        for (int q : options_on(tb, a, nodes[j]))
          key[i] = std::min(key[i], nodes[j].backlog + restore_delay(tb, a, nodes[j]) + duration(tb, a, q));
      }
    }
    std::stable_sort(visit.begin(), visit.end(), [&](int x, int y) { return key[x] < key[y]; });
  }
  o.visit = visit;

  // Alg. 1, admission: prefix of the visiting order admitted with minimum units; node choice by least estimated ACT
  // Second, co-constrained resource (Sec. 4.1: the cost of an action is a vector; Sec. 5.2: a node
  // must have the cores for the action and the memory for the whole trajectory when the
  // trajectory's first action is placed).  An action that is free to choose its node needs
  // `aux` of it on top of its units; an action pinned to a node belongs to a trajectory whose
  // share was taken when it was placed there, so it is not charged again.
  std::vector<int> aux_rem(M);
  for (int j = 0; j < M; ++j) aux_rem[j] = nodes[j].aux_free;
  std::vector<int> rem(M);
  std::vector<std::vector<int>> placed(M), waiting_pinned(M);
  std::vector<char> closed(M, 0);
  std::vector<int> ch(M * 4);
  for (int j = 0; j < M; ++j) { rem[j] = nodes[j].free; for (int x = 0; x < 4; ++x) ch[j*4+x] = nodes[j].chunks[x]; }
  char type_closed[N_TYPES] = {0, 0, 0};
  auto fits = [&](int j, int k) {
    return nodes[j].type == T_GPU ? chunk_fits(&ch[j*4], k) : rem[j] >= k;
  };
  // Several quotas per action (Sec. 4.1: one action may query several websites, each with its own
  // quota, and each is a component of its cost vector): besides the quota it is pinned to, the
  // action draws one token from every quota named in `extra` and is admitted only if all have one.
  std::vector<int> api_nodes;
  for (int j = 0; j < M; ++j) if (nodes[j].type == T_API) api_nodes.push_back(j);
  auto extras_fit = [&](const Act& a) {
    for (size_t r = 0; r < api_nodes.size() && r < 64; ++r)
      if ((a.extra >> r & 1ull) && rem[api_nodes[r]] < 1) return false;
    return true;
  };
  // queue_prefix: Alg. 1 as printed takes the longest prefix of the whole waiting queue that the
  // resources accommodate, so the first action that does not fit ends the admission for every
  // action behind it, of whatever kind.  Otherwise a misfit only closes its own pool (its node,
  // if it is pinned), as the managers of Sec. 5.2 schedule their resources independently.
  bool queue_closed = false;
  for (int i : visit) {
    if (o.reason[i] == R_INFEASIBLE) continue;
    const Act& a = acts[i];
    if (queue_closed || type_closed[a.type] || (a.pin >= 0 && closed[a.pin])) {
      o.reason[i] = R_PREFIX;
      if (a.pin >= 0) waiting_pinned[a.pin].push_back(i);
      continue;
    }
    int bj = -1; int64_t be = INF;
    for (int j = 0; j < M; ++j) {
      if (nodes[j].type != a.type || closed[j]) continue;
      if (a.pin >= 0 && a.pin != j) continue;
      if (!fits(j, kmin[i])) continue;
      if (a.pin < 0 && a.aux > aux_rem[j]) continue;
      if (a.extra && !extras_fit(a)) continue;
      int qs = -1;
      for (int q : options_on(tb, a, nodes[j])) if (fits(j, tb.k_list[q])) qs = q;
      const int64_t e = nodes[j].backlog + restore_delay(tb, a, nodes[j]) + duration(tb, a, qs);   // Eq. 2 on this node
      if (e < be) { be = e; bj = j; }
    }
    if (bj < 0) {
      if (a.pin >= 0) { closed[a.pin] = 1; waiting_pinned[a.pin].push_back(i); }
      else type_closed[a.type] = 1;
      if (queue_prefix) queue_closed = true;
      o.reason[i] = R_PREFIX;
      continue;
    }
    o.node[i] = bj; o.home[i] = bj;
    if (a.pin < 0) aux_rem[bj] -= a.aux;
    for (size_t r = 0; r < api_nodes.size() && r < 64; ++r)
      if (a.extra >> r & 1ull) { rem[api_nodes[r]] -= 1; o.extra_used[api_nodes[r]] += 1; }
    if (nodes[bj].type == T_GPU) chunk_take(&ch[bj*4], kmin[i]); else rem[bj] -= kmin[i];
    placed[bj].push_back(i);
  }

  // Alg. 1, per node: DPArrange + greedy tail eviction on the approximated objective
  for (int j = 0; j < M; ++j) {
    const std::vector<int>& C = placed[j];
    const int m = (int)C.size();
    if (m == 0) continue;
    const Node& nd = nodes[j];
    bool any_elastic = false;
    for (int i : C) if (acts[i].model != 0) any_elastic = true;
    std::vector<int32_t> ks(m);
    int L = m;
    if (!any_elastic) {
      for (int x = 0; x < m; ++x) ks[x] = kmin[C[x]];
    } else {
      auto dur_row = [&](int i, int64_t* row) {
        for (int q = 0; q < K; ++q) row[q] = INF;
        for (int q : options_on(tb, acts[i], nd)) row[q] = restore_delay(tb, acts[i], nd) + duration(tb, acts[i], q);
      };
      std::vector<int64_t> cdur((size_t)m * K);
      for (int x = 0; x < m; ++x) dur_row(C[x], &cdur[(size_t)x * K]);
      // Alg. 2: exact part by DPArrange, rest of this pool's queue estimated on the heap
      auto objective = [&](int Lc, std::vector<int32_t>& kk) -> int64_t {
        kk.assign(Lc, 0);
        const int64_t exact = nd.type == T_GPU
            ? dp_chunks(Lc, cdur.data(), tb.k_list, K, nd.chunks, kk.data())
            : dp_units(Lc, cdur.data(), tb.k_list, K, nd.free, kk.data());
        std::vector<int64_t> heap(nd.busy);
        int used = 0;
        for (int x = 0; x < Lc; ++x) {
          int q = 0; while (tb.k_list[q] != kk[x]) ++q;
          for (int c = 0; c < kk[x]; ++c) heap.push_back(nd.backlog + cdur[(size_t)x * K + q]);
          used += kk[x];
        }
        for (int c = used; c < nd.free; ++c) heap.push_back(nd.backlog);
        std::vector<int> ac(C.begin() + Lc, C.end());
        ac.insert(ac.end(), waiting_pinned[j].begin(), waiting_pinned[j].end());
        std::vector<int64_t> adur((size_t)ac.size() * K);
        for (size_t x = 0; x < ac.size(); ++x) dur_row(ac[x], &adur[x * K]);
        const int64_t approx = estimate(heap, (int)ac.size(), adur.data(), tb.k_list, K, tb.depth);
        return exact + (int64_t)Lc * nd.backlog + approx;
      };
      std::vector<int32_t> kk;
      int64_t obj = objective(L, ks);
      while (L > 1) {
        const int64_t nobj = objective(L - 1, kk);
        if (nobj >= obj) break;                        // a tie stops the eviction
        obj = nobj; ks = kk; --L;
      }
      o.node_obj[j] = obj;
    }
    std::vector<char> core_free = nd.core_free;
    for (int x = 0; x < m; ++x) {
      const int i = C[x];
      if (x >= L) { o.node[i] = -1; o.reason[i] = R_EVICTED; continue; }
      int q = 0; while (tb.k_list[q] != ks[x]) ++q;
      o.units[i] = ks[x];
      o.act[i] = acts[i].age + nd.backlog + restore_delay(tb, acts[i], nd) + duration(tb, acts[i], q);
      // Sec. 5.2: the selected actions of a node name their cores one after the other, in visiting order
      if (numa_cores > 0 && nd.type == T_CPU) o.cores[i] = take_cores(core_free, numa_cores, ks[x]);
      // pooled GPUs: the action's chunk is the smallest free chunk of the cluster that is large
      // enough (Sec. 5.3's rule over all nodes), on the lowest-numbered node that has one
      if (j == pool) {
        int best = -1, best_level = 4;
        for (int r = 0; r < M; ++r) {
          if (nodes[r].type != T_GPU) continue;
          for (int b = chunk_level(ks[x]); b < best_level; ++b)
            if (real_chunks[r][b] > 0) { best = r; best_level = b; break; }
        }
        int c[4] = {real_chunks[best][0], real_chunks[best][1], real_chunks[best][2], real_chunks[best][3]};
        chunk_take(c, ks[x]);
        for (int b = 0; b < 4; ++b) real_chunks[best][b] = c[b];
        o.node[i] = best;
      }
    }
  }
  return o;
}

}  // namespace

// =========================================================================================
// flat C entry points (loaded by the tests through ctypes)
// =========================================================================================
extern "C" {

struct orc_problem {
  int32_t B, N, M, K, n_classes, n_tasks, depth, order_policy;
  const int32_t* k_list; const int32_t* type_k; const uint32_t* speedup_q16;
  const uint8_t* node_type; const int32_t* node_cap; const int32_t* node_free;
  const int64_t* node_backlog_us; const uint8_t* node_chunks;
  const int32_t* node_busy_off; const int64_t* node_busy_rel_us;
  const uint8_t* act_type; const uint8_t* act_model; const int64_t* act_t_ori_us; const int64_t* act_age_us;
  const uint32_t* act_kmask; const uint32_t* act_param; const int32_t* act_pin_node; const int32_t* act_task;
  const int32_t* node_aux_free; const int32_t* act_aux;     // both or neither; NULL: no second resource
  const int32_t* act_service; const uint64_t* node_resident; const int64_t* restore_us;   // all or none
  const uint64_t* act_quota_mask;                           // [B*N] further quotas of an API action, or NULL
  const uint64_t* node_core_free; int32_t numa_cores;       // [B*M*4] free-core bitmaps of CPU nodes, or NULL (then numa_cores = 0)
  int32_t gpu_pooled;                                       // 1: the GPU nodes of a snapshot form one pool of chunks (Alg. 4's state)
  int32_t queue_prefix;                                     // 1: one admitted prefix of the whole queue (Alg. 1 as printed) instead of one per pool
};

struct orc_summary {
  int64_t sum_act_us;
  int32_t n_assigned, n_prefix, n_evicted, n_infeasible;
  int64_t units_used[3], units_free[3];
  double mean_act_us, util[3];
};

struct orc_trace {
  int32_t S, A, M, K, n_classes, depth, max_ticks, cache_slots;   // cache_slots: services a node keeps resident
  int64_t tick_us;
  const int32_t* k_list; const int32_t* type_k; const uint32_t* speedup_q16;
  const uint8_t* node_type; const int32_t* node_cap; const int32_t* quota_rate; const int64_t* quota_tok0_micro;
  const int64_t* arrival_us; const uint8_t* act_type; const uint8_t* act_model; const int64_t* act_t_ori_us;
  const uint32_t* act_kmask; const uint32_t* act_param; const int32_t* act_pin_node;
  const int32_t* act_service; const int64_t* restore_us;           // both or neither (Sec. 5.3)
  const uint64_t* act_quota_mask;                                  // [S*A] further quotas of an API action (Sec. 4.1), or NULL
  int32_t queue_prefix;                                            // 1: every step admits one prefix of the whole waiting queue
  const int32_t* node_aux; const int32_t* act_aux;                 // [S*M], [S*A] second resource (Sec. 4.1, 5.2); both or neither
  int32_t numa_cores;                                              // > 0: CPU actions are given named cores (Sec. 5.2), all free at time 0
  int32_t order_policy;                                            // ORDER_FCFS, or ORDER_COST: every step visits the queue by least estimated ACT
  int32_t gpu_pooled;                                              // 1: every step sees the GPU nodes as one pool of chunks (Sec. 5.3, Alg. 4)
  int32_t cache_per_gpu;                                           // 1: every GPU of a GPU node keeps its own cache of services (Sec. 5.3)
};

}  // extern "C"

namespace {

Tables tables_of(const orc_problem* p) {
  return Tables{p->K, p->k_list, p->type_k, p->speedup_q16, p->depth, p->act_service ? p->restore_us : nullptr};
}

std::vector<Act> acts_of(const orc_problem* p, int b) {
  std::vector<Act> v(p->N);
  for (int i = 0; i < p->N; ++i) {
    const size_t g = (size_t)b * p->N + i;
    v[i] = Act{p->act_type[g], p->act_model[g], p->act_t_ori_us[g], p->act_age_us ? p->act_age_us[g] : 0,
               p->act_kmask[g], p->act_param[g], p->act_pin_node[g], p->act_task ? p->act_task[g] : 0,
               p->act_aux ? p->act_aux[g] : 0, p->act_service ? p->act_service[g] : -1,
               p->act_quota_mask ? p->act_quota_mask[g] : 0};
  }
  return v;
}

std::vector<Node> nodes_of(const orc_problem* p, int b) {
  std::vector<Node> v(p->M);
  for (int j = 0; j < p->M; ++j) {
    const size_t g = (size_t)b * p->M + j;
    Node& nd = v[j];
    nd.type = p->node_type[g]; nd.cap = p->node_cap[g]; nd.free = p->node_free[g];
    nd.backlog = p->node_backlog_us[g];
    nd.aux_free = p->node_aux_free ? p->node_aux_free[g] : INT32_MAX;
    nd.resident = p->node_resident ? p->node_resident[g] : 0;
    for (int x = 0; x < 4; ++x) nd.chunks[x] = 0;
    if (nd.type == T_GPU) {
      if (p->node_chunks) for (int x = 0; x < 4; ++x) nd.chunks[x] = p->node_chunks[g * 4 + x];
      else { nd.chunks[3] = nd.free / 8; for (int x = 0; x < 3; ++x) nd.chunks[x] = (nd.free % 8) >> x & 1; }
    }
    if (p->node_busy_off)
      nd.busy.assign(p->node_busy_rel_us + p->node_busy_off[g], p->node_busy_rel_us + p->node_busy_off[g + 1]);
    if (p->node_core_free && nd.type == T_CPU) {
      nd.core_free.resize(nd.cap);
      for (int c = 0; c < nd.cap; ++c) nd.core_free[c] = (char)(p->node_core_free[g * 4 + c / 64] >> (c % 64) & 1ull);
    }
  }
  return v;
}

}  // namespace

extern "C" {

int64_t orc_duration(int model, int64_t T, uint32_t param, int k, uint32_t speedup) {
  int32_t kl[1] = {k}; int32_t tk[3] = {1, 1, 1}; uint32_t sp[1] = {speedup};
  Tables tb{1, kl, tk, sp, 1};
  Act a{0, model, T, 0, 1u, model == 2 ? 0u : param, -1, 0};
  return duration(tb, a, 0);
}

// Score tensor (Eq. 1 + Eq. 2 for every type-compatible candidate): for snapshot b, then type t,
// a block [actions of type t in FCFS order][nodes of type t in index order][type_k[t]].
int64_t orc_num_candidates(const orc_problem* p) {
  int64_t total = 0;
  for (int b = 0; b < p->B; ++b)
    for (int t = 0; t < N_TYPES; ++t) {
      int64_t na = 0, nn = 0;
      for (int i = 0; i < p->N; ++i) na += p->act_type[(size_t)b * p->N + i] == t;
      for (int j = 0; j < p->M; ++j) nn += p->node_type[(size_t)b * p->M + j] == t;
      total += na * nn * p->type_k[t];
    }
  return total;
}

void orc_score(const orc_problem* p, int64_t* cost) {
  const Tables tb = tables_of(p);
  size_t w = 0;
  for (int b = 0; b < p->B; ++b) {
    const std::vector<Act> acts = acts_of(p, b);
    const std::vector<Node> nodes = nodes_of(p, b);
    for (int t = 0; t < N_TYPES; ++t)
      for (int i = 0; i < p->N; ++i) {
        if (acts[i].type != t) continue;
        const std::vector<int> op = options(tb, acts[i]);
        for (int j = 0; j < p->M; ++j) {
          if (nodes[j].type != t) continue;
          for (int q = 0; q < tb.type_k[t]; ++q) {
            const bool ok = std::find(op.begin(), op.end(), q) != op.end() && tb.k_list[q] <= nodes[j].cap &&
                            (acts[i].pin < 0 || acts[i].pin == j);
            cost[w++] = ok ? nodes[j].backlog + restore_delay(tb, acts[i], nodes[j]) + duration(tb, acts[i], q) : INF;
          }
        }
      }
  }
}

void orc_assign(const orc_problem* p, int32_t* node, int32_t* units, int64_t* act_us, uint8_t* reason,
                orc_summary* summary, int32_t* node_used, int64_t* task_sum, int64_t* node_obj, int32_t* home,
                uint64_t* core_set) {
  const Tables tb = tables_of(p);
  for (int b = 0; b < p->B; ++b) {
    const std::vector<Act> acts = acts_of(p, b);
    const std::vector<Node> nodes = nodes_of(p, b);
    const StepOut o = step(tb, acts, nodes, p->order_policy, p->node_core_free ? p->numa_cores : 0, p->gpu_pooled != 0,
                           p->queue_prefix != 0);
    const size_t a0 = (size_t)b * p->N, n0 = (size_t)b * p->M;
    orc_summary s;
    std::memset(&s, 0, sizeof s);
    if (node_used) for (int j = 0; j < p->M; ++j) node_used[n0 + j] = 0;
    if (task_sum) for (int t = 0; t < p->n_tasks; ++t) task_sum[(size_t)b * p->n_tasks + t] = 0;
    for (int j = 0; j < p->M; ++j) s.units_free[nodes[j].type] += nodes[j].free;
    for (int i = 0; i < p->N; ++i) {
      node[a0 + i] = o.node[i]; units[a0 + i] = o.units[i]; act_us[a0 + i] = o.act[i]; reason[a0 + i] = o.reason[i];
      switch (o.reason[i]) {
        case R_PREFIX: ++s.n_prefix; break;
        case R_EVICTED: ++s.n_evicted; break;
        case R_INFEASIBLE: ++s.n_infeasible; break;
        default:
          ++s.n_assigned; s.sum_act_us += o.act[i]; s.units_used[acts[i].type] += o.units[i];
          if (node_used) node_used[n0 + o.node[i]] += o.units[i];
          if (task_sum) task_sum[(size_t)b * p->n_tasks + acts[i].task] += o.act[i];
      }
    }
    for (int j = 0; j < p->M; ++j) {                   // tokens drawn from further quotas count as used units
      s.units_used[T_API] += o.extra_used[j];
      if (node_used) node_used[n0 + j] += o.extra_used[j];
    }
    s.mean_act_us = s.n_assigned ? (double)s.sum_act_us / (double)s.n_assigned : 0.0;
    for (int t = 0; t < N_TYPES; ++t)
      s.util[t] = s.units_free[t] ? (double)s.units_used[t] / (double)s.units_free[t] : 0.0;
    if (summary) summary[b] = s;
    if (node_obj) for (int j = 0; j < p->M; ++j) node_obj[n0 + j] = o.node_obj[j];
    if (home) for (int i = 0; i < p->N; ++i) home[a0 + i] = o.home[i];
    if (core_set)
      for (int i = 0; i < p->N; ++i) {
        for (int w = 0; w < 4; ++w) core_set[(a0 + i) * 4 + w] = 0;
        for (int c : o.cores[i]) core_set[(a0 + i) * 4 + c / 64] |= 1ull << (c % 64);
      }
  }
}

// One allocation of Sec. 5.2 on a map of free cores (free_[c] = 0/1, updated); cores_out gets the k core ids.
int orc_take_cores(uint8_t* free_, int cap, int numa_cores, int k, int32_t* cores_out) {
  std::vector<char> f(free_, free_ + cap);
  const std::vector<int> got = take_cores(f, numa_cores, k);
  for (int c = 0; c < cap; ++c) free_[c] = (uint8_t)f[c];
  for (size_t x = 0; x < got.size(); ++x) cores_out[x] = got[x];
  return (int)got.size();
}

int64_t orc_dp_units(int m, const int64_t* dur, const int32_t* k_list, int K, int U, int32_t* k_out) {
  return dp_units(m, dur, k_list, K, U, k_out);
}

int64_t orc_dp_chunks(int m, const int64_t* dur, const int32_t* k_list, int K, const uint8_t* chunks, int32_t* k_out) {
  const int st[4] = {chunks[0], chunks[1], chunks[2], chunks[3]};
  return dp_chunks(m, dur, k_list, K, st, k_out);
}

int64_t orc_estimate(const int64_t* heap, int H, int n_ac, const int64_t* ac_dur, const int32_t* k_list, int K, int depth) {
  return estimate(std::vector<int64_t>(heap, heap + H), n_ac, ac_dur, k_list, K, depth);
}

int orc_chunk_take(uint8_t* chunks, int k) {
  int c[4] = {chunks[0], chunks[1], chunks[2], chunks[3]};
  const bool ok = chunk_take(c, k);
  for (int x = 0; x < 4; ++x) chunks[x] = (uint8_t)c[x];
  return ok;
}

int orc_chunk_encode_roundtrip(const uint8_t* bound, int j, uint8_t* out) {
  Radix r; for (int x = 0; x < 4; ++x) r.n[x] = bound[x];
  int c[4]; decode(r, j, c);
  for (int x = 0; x < 4; ++x) out[x] = (uint8_t)c[x];
  return encode(r, c);
}

// ---- trace replay: the step above run every tick on the live cluster state ---------------
// free GPUs of an 8-GPU node are a bit mask; a free chunk is a maximal aligned free block.
static void mask_chunks(int mask, int c[4]) {
  c[0] = c[1] = c[2] = c[3] = 0;
  for (int lvl = 3; lvl >= 0; --lvl) {
    const int sz = 1 << lvl;
    for (int s = 0; s < 8; s += sz) {
      const int blk = ((1 << sz) - 1) << s;
      if ((mask & blk) != blk) continue;
      bool parent_free = false;
      if (lvl < 3) { const int ps = s & ~(2 * sz - 1); const int pb = ((1 << (2 * sz)) - 1) << ps; parent_free = (mask & pb) == pb; }
      if (!parent_free) ++c[lvl];
    }
  }
}

static int mask_alloc(int& mask, int k) {               // best fit, lowest address; returns start
  const int a = chunk_level(k);
  for (int lvl = a; lvl < 4; ++lvl) {
    const int sz = 1 << lvl;
    for (int s = 0; s < 8; s += sz) {
      const int blk = ((1 << sz) - 1) << s;
      if ((mask & blk) != blk) continue;
      if (lvl < 3) { const int ps = s & ~(2 * sz - 1); const int pb = ((1 << (2 * sz)) - 1) << ps; if ((mask & pb) == pb) continue; }
      mask &= ~(((1 << (1 << a)) - 1) << s);
      return s;
    }
  }
  return -1;
}

// Sec. 5.3, with a cache on every GPU: the allocation takes from the lowest level that has a free chunk, as above;
// among that level's free chunks one that already caches the requested service comes first.  A block of GPUs caches
// a service when every GPU of it does.  Taken here: the first free chunk of the level that holds an aligned block of
// the action's size caching the service, and the first such block of it; without one, the first chunk's first block.
static int mask_alloc_cached(int& mask, int k, int sv, const uint64_t* gpu_res, bool* hit) {
  const int a = chunk_level(k), need = 1 << a;
  *hit = false;
  for (int lvl = a; lvl < 4; ++lvl) {
    const int sz = 1 << lvl;
    std::vector<int> chunks;                               // starts of the free chunks of this level, ascending
    for (int s = 0; s < 8; s += sz) {
      const int blk = ((1 << sz) - 1) << s;
      if ((mask & blk) != blk) continue;
      if (lvl < 3) { const int ps = s & ~(2 * sz - 1); const int pb = ((1 << (2 * sz)) - 1) << ps; if ((mask & pb) == pb) continue; }
      chunks.push_back(s);
    }
    if (chunks.empty()) continue;
    int take = chunks[0];
    for (size_t c = 0; c < chunks.size() && !*hit; ++c)
      for (int b = chunks[c]; b < chunks[c] + sz && !*hit; b += need) {
        bool all = true;
        for (int g = b; g < b + need; ++g) all = all && (gpu_res[g] >> sv & 1ull);
        if (all) { take = b; *hit = true; }
      }
    mask &= ~(((1 << need) - 1) << take);
    return take;
  }
  return -1;
}

int orc_mask_chunks(int mask, uint8_t* out) { int c[4]; mask_chunks(mask, c); for (int x = 0; x < 4; ++x) out[x] = (uint8_t)c[x]; return 0; }
int orc_mask_alloc(int* mask, int k) { return mask_alloc(*mask, k); }

// `ext` (NULL, or [S * ORC_N_EXTENTS]) only observes: per scenario, the largest value over all steps of the
// sizes a step works on (list lengths, candidates per node, heap entries ...).  No decision reads it.
enum { ORC_EXT_WAIT_CPU = 0, ORC_EXT_WAIT_GPU, ORC_EXT_WAIT_API, ORC_EXT_RUNNING, ORC_EXT_CAND_CPU_ELASTIC,
       ORC_EXT_CAND_GPU_ELASTIC, ORC_EXT_CAND_NODE, ORC_EXT_CAND_STEP, ORC_EXT_PINNED_WAIT_STEP, ORC_EXT_BUSY_UNITS,
       ORC_EXT_HEAP_ENTRIES, ORC_EXT_CHUNK_STATES, ORC_EXT_DP_CELLS, ORC_EXT_NODES_CPU, ORC_EXT_NODES_GPU,
       ORC_EXT_NODES_API, ORC_N_EXTENTS };

static void replay_run(const orc_trace* t, int s_lo, int s_hi, int64_t* start_us, int64_t* finish_us, int32_t* units,
                       int32_t* node, double* mean_act, int64_t* p99_act, int32_t* n_started, int32_t* n_ticks,
                       uint64_t* core_set, int64_t* ext) {
  const Tables tb{t->K, t->k_list, t->type_k, t->speedup_q16, t->depth, t->act_service ? t->restore_us : nullptr};
  const int A = t->A, M = t->M;
  for (int s = s_lo; s < s_hi; ++s) {
    const size_t a0 = (size_t)s * A, n0 = (size_t)s * M;
    struct Run { int64_t fin; int node, k, gstart, aux; std::vector<int> cores; };
    std::vector<Run> running;
    std::vector<int> rem(M, 0), gmask(M, 0);
    std::vector<int64_t> tok(M, 0);
    // Sec. 5.3: every node caches up to cache_slots services; a restored service stays resident
    // until it is the least recently used one when room is needed.  Nothing is resident at first.
    std::vector<uint64_t> resident(M, 0);
    std::vector<int64_t> used_at((size_t)M * 64, 0);        // per node and service: sequence number of its last use
    std::vector<int64_t> seq(M, 0);
    // cache_per_gpu: on GPU nodes the cache belongs to the GPU - each keeps up to cache_slots services of its own,
    // least recently used out first.  An action finds its service resident when every GPU of the block it is given
    // caches it; afterwards every GPU of the block does, as its most recently used one.  The step keeps its
    // per-node view: it counts a service as resident on a node when any GPU of the node caches it, so what an
    // action really waits for a restore is known only once it has its GPUs (never less than the step assumed).
    const bool per_gpu = t->cache_per_gpu != 0 && tb.restore_us;
    std::vector<uint64_t> gpu_res(per_gpu ? (size_t)M * 8 : 0, 0);
    std::vector<int64_t> gpu_used(per_gpu ? (size_t)M * 8 * 64 : 0, 0);
    // Second resource of a node (Sec. 4.1, 5.2: e.g. memory next to cores): an action that is free to choose
    // its node holds its demand from start to finish; pinned actions hold none (the share of their
    // trajectory is not part of a trace).
    std::vector<int> aux_rem(M, INT32_MAX);
    // Sec. 5.2: the CPU manager names the cores of every action.  All cores are free at time 0; an action keeps
    // the cores the step gave it (tg_assign's rule, node by node in visiting order) until it finishes.
    const int numa = core_set ? t->numa_cores : 0;
    std::vector<std::vector<char>> core_free(M);
    if (numa > 0)
      for (int i = 0; i < A; ++i) for (int w = 0; w < 4; ++w) core_set[(a0 + i) * 4 + w] = 0;
    for (int j = 0; j < M; ++j) {
      if (numa > 0 && t->node_type[n0 + j] == T_CPU) core_free[j].assign(t->node_cap[n0 + j], 1);
      if (t->node_aux) aux_rem[j] = t->node_aux[n0 + j];
      rem[j] = t->node_cap[n0 + j];
      if (t->node_type[n0 + j] == T_GPU) gmask[j] = (1 << t->node_cap[n0 + j]) - 1;
      if (t->node_type[n0 + j] == T_API) tok[j] = t->quota_tok0_micro[n0 + j];
    }
    for (int i = 0; i < A; ++i) { start_us[a0 + i] = -1; finish_us[a0 + i] = -1; units[a0 + i] = 0; node[a0 + i] = -1; }
    std::vector<int> waiting;
    int next = 0, started = 0, tick = 0;
    for (; tick < t->max_ticks && started < A; ++tick) {
      const int64_t now = (int64_t)tick * t->tick_us;
      // (1) finished actions give their units back
      for (size_t r = 0; r < running.size();) {
        if (running[r].fin <= now) {
          const Run& u = running[r];
          if (t->node_type[n0 + u.node] == T_GPU) gmask[u.node] |= ((1 << (1 << chunk_level(u.k))) - 1) << u.gstart;
          rem[u.node] += u.k;
          if (t->node_aux) aux_rem[u.node] += u.aux;
          for (int c : u.cores) core_free[u.node][c] = 1;
          running[r] = running.back(); running.pop_back();
        } else ++r;
      }
      // (2) quotas refill (Sec. 5.1, quota-based pattern), in millionths of a token
      if (tick > 0)
        for (int j = 0; j < M; ++j)
          if (t->node_type[n0 + j] == T_API)
            tok[j] = std::min<int64_t>((int64_t)t->node_cap[n0 + j] * 1000000, tok[j] + (int64_t)t->quota_rate[n0 + j] * t->tick_us);
      // (3) waiting queue in arrival order
      while (next < A && t->arrival_us[a0 + next] <= now) waiting.push_back(next++);
      if (waiting.empty()) continue;
      std::vector<Act> acts;
      for (int i : waiting)
        acts.push_back(Act{t->act_type[a0 + i], t->act_model[a0 + i], t->act_t_ori_us[a0 + i], now - t->arrival_us[a0 + i],
                           t->act_kmask[a0 + i], t->act_param[a0 + i], t->act_pin_node[a0 + i], 0,
                           t->act_aux ? t->act_aux[a0 + i] : 0,
                           t->act_service ? t->act_service[a0 + i] : -1,
                           t->act_quota_mask ? t->act_quota_mask[a0 + i] : 0});
      std::vector<Node> nodes(M);
      for (int j = 0; j < M; ++j) {
        Node& nd = nodes[j];
        nd.type = t->node_type[n0 + j]; nd.cap = t->node_cap[n0 + j]; nd.backlog = 0;
        nd.resident = resident[j];
        if (per_gpu && nd.type == T_GPU) for (int g = 0; g < 8; ++g) nd.resident |= gpu_res[(size_t)j * 8 + g];
        nd.aux_free = aux_rem[j];
        if (numa > 0 && nd.type == T_CPU) nd.core_free = core_free[j];
        for (int x = 0; x < 4; ++x) nd.chunks[x] = 0;
        if (nd.type == T_API) nd.free = (int)(tok[j] / 1000000);
        else if (nd.type == T_GPU) { mask_chunks(gmask[j], nd.chunks); nd.free = __builtin_popcount(gmask[j]); }
        else nd.free = rem[j];
      }
      for (const Run& u : running)                       // executing queue seeds the completion heap
        if (nodes[u.node].type != T_API)
          for (int c = 0; c < u.k; ++c) nodes[u.node].busy.push_back(u.fin - now);
      // (4) the scheduling step; (5) selected actions start now
      // Sec. 4.2: the step also runs on top of another ordering of the queue; the waiting queue itself stays in
      // arrival order, every step orders it anew (the estimates change with what is resident where)
      // gpu_pooled: the step schedules the GPU cluster as one resource and names, for every action it selects, the
      // node whose chunk it takes; the action then holds GPUs of that node until it finishes
      const StepOut o = step(tb, acts, nodes, t->order_policy, numa, t->gpu_pooled != 0, t->queue_prefix != 0);
      if (ext) {
        int64_t* e = ext + (size_t)s * ORC_N_EXTENTS;
        auto up = [&](int x, int64_t v) { if (v > e[x]) e[x] = v; };
        int64_t wk[3] = {0, 0, 0};
        for (const Act& a : acts) ++wk[a.type];
        up(ORC_EXT_WAIT_CPU, wk[T_CPU]); up(ORC_EXT_WAIT_GPU, wk[T_GPU]); up(ORC_EXT_WAIT_API, wk[T_API]);
        up(ORC_EXT_RUNNING, (int64_t)running.size());
        std::vector<int> cand(M, 0), elastic(M, 0);
        int64_t cand_step = 0, pinned_wait = 0;
        for (size_t w = 0; w < acts.size(); ++w) {
          if (o.home[w] >= 0) { ++cand[o.home[w]]; ++cand_step; if (acts[w].model != 0) elastic[o.home[w]] = 1; }
          else if (o.reason[w] == R_PREFIX && acts[w].pin >= 0) ++pinned_wait;
        }
        up(ORC_EXT_CAND_STEP, cand_step); up(ORC_EXT_PINNED_WAIT_STEP, pinned_wait);
        Node pooled;                                              // what the step made of the GPU nodes under gpu_pooled
        int pool = -1;
        if (t->gpu_pooled)
          for (int j = 0; j < M; ++j) {
            if (nodes[j].type != T_GPU) continue;
            if (pool < 0) { pool = j; pooled = nodes[j]; continue; }
            pooled.free += nodes[j].free;
            for (int x = 0; x < 4; ++x) pooled.chunks[x] += nodes[j].chunks[x];
            pooled.busy.insert(pooled.busy.end(), nodes[j].busy.begin(), nodes[j].busy.end());
          }
        for (int j = 0; j < M; ++j) {
          if (cand[j] == 0) continue;
          const Node& nd = j == pool ? pooled : nodes[j];
          up(ORC_EXT_CAND_NODE, cand[j]);
          if (nd.type == T_API) continue;
          up(ORC_EXT_BUSY_UNITS, (int64_t)nd.busy.size());
          up(ORC_EXT_HEAP_ENTRIES, (int64_t)nd.busy.size() + nd.free);
          if (nd.type == T_GPU) {
            int64_t st = 1;
            for (int x = 0; x < 4; ++x) st *= std::max(nd.chunks[x], 1) + 1;
            up(ORC_EXT_CHUNK_STATES, st);
            if (elastic[j]) up(ORC_EXT_CAND_GPU_ELASTIC, cand[j]);
          } else {
            if (elastic[j]) { up(ORC_EXT_CAND_CPU_ELASTIC, cand[j]); up(ORC_EXT_DP_CELLS, (int64_t)nd.free + 1); }
          }
        }
      }
      // selected actions start in the order the step visited them (chunks and cache slots are handed out in the
      // order its allocation assumed; under FCFS that is the arrival order); the others keep waiting, in arrival order
      std::vector<int> still;
      for (size_t w = 0; w < waiting.size(); ++w) if (o.node[w] < 0) still.push_back(waiting[w]);
      for (int w : o.visit) {
        const int i = waiting[w];
        if (o.node[w] < 0) continue;
        const int j = o.node[w], k = o.units[w];
        int q = 0; while (tb.k_list[q] != k) ++q;
        // realised = modelled duration: the delay is the one the step saw (residency at the tick's start) -
        // except with a cache per GPU, below
        int64_t dur = restore_delay(tb, acts[w], nodes[j]) + duration(tb, acts[w], q);
        const int sv = acts[w].service;
        int gstart = -1;
        if (per_gpu && nodes[j].type == T_GPU && sv >= 0) {
          // the delay is the one of the GPUs the action gets: none if all of them cache the service
          bool hit;
          gstart = mask_alloc_cached(gmask[j], k, sv, &gpu_res[(size_t)j * 8], &hit);
          dur = (hit ? 0 : tb.restore_us[sv]) + duration(tb, acts[w], q);
          ++seq[j];
          for (int g = gstart; g < gstart + (1 << chunk_level(k)); ++g) {
            uint64_t& res = gpu_res[(size_t)j * 8 + g];
            int64_t* used = &gpu_used[((size_t)j * 8 + g) * 64];
            if (!(res >> sv & 1ull) && __builtin_popcountll(res) >= t->cache_slots) {
              int victim = -1;
              for (int x = 0; x < 64; ++x)
                if ((res >> x & 1ull) && (victim < 0 || used[x] < used[victim])) victim = x;
              res &= ~(1ull << victim);
            }
            res |= 1ull << sv;
            used[sv] = seq[j];
          }
        }
        else if (sv >= 0 && tb.restore_us) {                 // the service is (now) resident and most recently used
          if (!(resident[j] >> sv & 1ull) && __builtin_popcountll(resident[j]) >= t->cache_slots) {
            int victim = -1;
            for (int x = 0; x < 64; ++x)
              if ((resident[j] >> x & 1ull) && (victim < 0 || used_at[(size_t)j * 64 + x] < used_at[(size_t)j * 64 + victim])) victim = x;
            resident[j] &= ~(1ull << victim);
          }
          resident[j] |= 1ull << sv;
          used_at[(size_t)j * 64 + sv] = ++seq[j];
        }
        Run u{now + dur, j, k, 0, t->act_aux && acts[w].pin < 0 ? acts[w].aux : 0};
        if (nodes[j].type == T_API) {
          tok[j] -= (int64_t)k * 1000000;
          int r = 0;                                         // one token of every further quota it names (Sec. 4.1)
          for (int x = 0; x < M; ++x)
            if (t->node_type[n0 + x] == T_API) { if (r < 64 && (acts[w].extra >> r & 1ull)) tok[x] -= 1000000; ++r; }
        }
        else {
          if (nodes[j].type == T_GPU) u.gstart = gstart >= 0 ? gstart : mask_alloc(gmask[j], k);
          rem[j] -= k;
          if (t->node_aux) aux_rem[j] -= u.aux;
          if (numa > 0 && nodes[j].type == T_CPU) {
            u.cores = o.cores[w];
            for (int c : u.cores) { core_free[j][c] = 0; core_set[(a0 + i) * 4 + c / 64] |= 1ull << (c % 64); }
          }
          running.push_back(u);
        }
        start_us[a0 + i] = now; finish_us[a0 + i] = now + dur; units[a0 + i] = k; node[a0 + i] = j;
        ++started;
      }
      waiting.swap(still);
    }
    std::vector<int64_t> acts_done;
    int64_t sum = 0;
    for (int i = 0; i < A; ++i)
      if (start_us[a0 + i] >= 0) { acts_done.push_back(finish_us[a0 + i] - t->arrival_us[a0 + i]); sum += acts_done.back(); }
    std::sort(acts_done.begin(), acts_done.end());
    const int n = (int)acts_done.size();
    n_started[s] = n; n_ticks[s] = tick;
    mean_act[s] = n ? (double)sum / (double)n : 0.0;
    p99_act[s] = n ? acts_done[(size_t)((99 * (int64_t)n + 99) / 100) - 1] : -1;   // nearest rank
  }
}

void orc_replay(const orc_trace* t, int s_lo, int s_hi, int64_t* start_us, int64_t* finish_us, int32_t* units,
                int32_t* node, double* mean_act, int64_t* p99_act, int32_t* n_started, int32_t* n_ticks,
                uint64_t* core_set /* [S*A*4] or NULL; written when numa_cores > 0 */) {
  replay_run(t, s_lo, s_hi, start_us, finish_us, units, node, mean_act, p99_act, n_started, n_ticks, core_set, nullptr);
}

// The same replay, reporting only what it observed: ext[s * 16 + x] = the largest value of extent x over the
// steps of scenario s (rows of scenarios outside [s_lo, s_hi) are left alone).  Used to check, on the CPU, the
// capacities a batched implementation sizes its buffers with.
void orc_replay_extents(const orc_trace* t, int s_lo, int s_hi, int64_t* ext) {
  const size_t nA = (size_t)t->S * t->A;
  std::vector<int64_t> st(nA), fi(nA), p99(t->S);
  std::vector<int32_t> un(nA), no(nA), ns(t->S), nt(t->S);
  std::vector<double> mean(t->S);
  std::vector<uint64_t> cs(t->numa_cores > 0 ? nA * 4 : 0);
  for (int s = s_lo; s < s_hi; ++s) {
    int64_t* e = ext + (size_t)s * ORC_N_EXTENTS;
    for (int x = 0; x < ORC_N_EXTENTS; ++x) e[x] = 0;
    for (int j = 0; j < t->M; ++j) {
      const int ty = t->node_type[(size_t)s * t->M + j];
      ++e[ty == T_CPU ? ORC_EXT_NODES_CPU : ty == T_GPU ? ORC_EXT_NODES_GPU : ORC_EXT_NODES_API];
    }
  }
  replay_run(t, s_lo, s_hi, st.data(), fi.data(), un.data(), no.data(), mean.data(), p99.data(), ns.data(), nt.data(),
             cs.empty() ? nullptr : cs.data(), ext);
}

}  // extern "C"
