// tg_assign: one scheduling step (Alg. 1 of the paper) for every snapshot of a problem.
//
//   tg_dur_kernel      Eq. 1 once per (action, option)              fully parallel
//   tg_order_kernel    only for the second visiting order: keys + sort of every pool's queue
//   tg_place_kernel    Alg. 1's prefix admission at minimum units, node choice by least
//                      estimated completion time (Eq. 2)            one wavefront per (snapshot, kind)
//   tg_stop_kernel     only for the whole-queue prefix: where the admission of a snapshot ends, between two
//                      passes of tg_place_kernel
//   tg_lists_kernel    groups admitted / waiting-pinned actions by node, FCFS inside a node
//   tg_node_kernel     the rest of Alg. 1 per node: DPArrange (Alg. 3 / Alg. 4) + greedy tail
//                      eviction on the approximated objective (Alg. 2)   one wavefront per node
//   tg_pool_map_kernel (pooled GPUs) the real chunk of every selected GPU action, Sec. 5.3
//   tg_cores_kernel    (problems with a core topology) the cores of every selected CPU action, Sec. 5.2
//   tg_summary_kernel  per-snapshot sums, counts, utilisation
//
// The admission loop is sequential by definition (every action sees the capacity left by the
// ones before it), so tg_place_kernel keeps the node table of its pool in registers (LDS for
// very wide pools) and spends its 64 lanes on the argmin over nodes; parallelism comes from the
// batch of snapshots.  The per-node stage runs as up to three concurrent launches, one per class
// of candidate count, whose persistent wavefronts pull nodes from class lists.
#include <algorithm>
#include <atomic>

#include "tg_step.h"

namespace {

struct AssignWs {
  int64_t* dur;      // [B*N*K] getDur per option, TG_INF where the option is not allowed
  int32_t* slot;     // [B*N]   position of an action inside its node's list
  int32_t* order;    // [B*N]   admitted actions grouped by node
  int32_t* dorder;   // [B*N]   waiting actions pinned to a node (deferred by the prefix rule)
  int32_t *nl_off, *nl_cnt, *dl_off, *dl_cnt;   // [B*M] list extents per node
  int32_t* class_list;   // [kClasses][B*M] nodes with candidates, binned by how many
  int32_t* class_ctl;    // [2*kClasses + 2] per class: number of nodes, next node to hand out; then, for the light
                         // class, how many of its nodes were filed at the front and at the back of its list
  int32_t* visit;        // [B*N] TG_ORDER_COST: action ids grouped by kind in visiting order (else unused)
  uint64_t* gkey;        // [B*N] whole-queue prefix under TG_ORDER_COST: (key, action id) of every action (else unused)
  uint64_t* stop;        // [B]   whole-queue prefix: place in the visiting order at which the admission ends (else unused)
  uint64_t *okey_a, *okey_b;   // [B*N] each, TG_ORDER_COST with a pool too large for one workgroup's sort: sorted runs of
                               // keys, merged from one buffer into the other (else unused)
};

// Nodes are processed in classes of candidate count so that the LDS a wavefront needs (the
// choice table grows with m) does not cap the occupancy of the many small nodes.  The
// launches run side by side; a node holds at most as many candidates as it has free units, so
// the number of nodes with more than 16 / 64 free units (known when the problem is built)
// bounds the heavier classes; how the LDS of a CU is split between the launches is decided in
// tg_assign below.
constexpr int kClasses = 3;
constexpr int kSelRows = 24;     // prefix lengths backtracked per batch (a heavy wavefront of a 128-core cluster then fits 20 KB of LDS)
constexpr int kLightBatch = 8;   // nodes of the light class a wavefront takes per fetch
constexpr int kClassCap0 = 16, kClassCap1 = 64;
__host__ __device__ constexpr int class_cap(int c) { return c == 0 ? kClassCap0 : c == 1 ? kClassCap1 : 1 << 30; }

constexpr int kOrderTile = 8192;      // TG_ORDER_COST: keys one workgroup sorts in LDS; larger pools are sorted tile by tile and merged

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

size_t carve(const tg_problem* p, char* base, AssignWs* w) {
  const size_t nA = (size_t)p->dev.B * p->dev.N, nN = (size_t)p->dev.B * p->dev.M;
  size_t off = 0;
  auto take = [&](size_t bytes) { char* r = base + off; off += align256(bytes); return r; };
  char* a = take(nA * p->dev.K * 8); char* b = take(nA * 4); char* c = take(nA * 4); char* d = take(nA * 4);
  char* e = take(nN * 4); char* f = take(nN * 4); char* g = take(nN * 4); char* h = take(nN * 4);
  char* cl = take(nN * 4 * kClasses); char* cc = take((2 * kClasses + 2) * 4);
  char* vi = take(p->order_policy == TG_ORDER_COST ? nA * 4 : 0);
  char* gk = take(p->queue_prefix && p->order_policy == TG_ORDER_COST ? nA * 8 : 0);
  char* st = take(p->queue_prefix ? (size_t)p->dev.B * 8 : 0);
  const bool big_sort = p->order_policy == TG_ORDER_COST && p->max_actions_of_kind > kOrderTile;
  char* ka = take(big_sort ? nA * 8 : 0); char* kb = take(big_sort ? nA * 8 : 0);
  if (w) {
    w->okey_a = (uint64_t*)ka; w->okey_b = (uint64_t*)kb;
    w->class_list = (int32_t*)cl; w->class_ctl = (int32_t*)cc; w->visit = (int32_t*)vi;
    w->gkey = (uint64_t*)gk; w->stop = (uint64_t*)st;
    w->dur = (int64_t*)a; w->slot = (int32_t*)b; w->order = (int32_t*)c; w->dorder = (int32_t*)d;
    w->nl_off = (int32_t*)e; w->nl_cnt = (int32_t*)f; w->dl_off = (int32_t*)g; w->dl_cnt = (int32_t*)h;
  }
  return off;
}

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void tg_dur_kernel(TgDev P, int64_t* __restrict__ dur, int32_t* __restrict__ class_ctl) {
  const size_t x = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (x < 2 * kClasses + 2) class_ctl[x] = 0;
  const size_t total = (size_t)P.B * P.N * P.K;
  if (x >= total) return;
  const size_t g = x / P.K;
  const int q = (int)(x - g * P.K);
  int64_t d = TG_INF;
  if (P.act_kmask[g] >> q & 1u) {
    const int model = P.act_model[g];
    const uint32_t param = P.act_param[g];
    const uint32_t sp = model == TG_MODEL_TABLE ? P.speedup[param * P.K + q] : 0u;
    d = tg_duration(model, P.act_T[g], param, P.k_list[q], sp);
  }
  dur[x] = d;
}

// ------------------------------------------------------------------------------------------
// TG_ORDER_COST: the visiting order of one pool = its actions sorted by (least estimated ACT
// over the action's candidates, FCFS rank).  Durations do not grow with the units (Eq. 1 with
// E(k) k nondecreasing), so on a node the best option is the largest allowed one its capacity
// admits, and nodes that admit the same number of options differ only in their backlog: the key
// of an unpinned action is a minimum over at most K+1 groups of nodes, each represented by its
// smallest backlog.  Keys and ranks are packed into one 64-bit word (key < 2^46, rank < 2^17)
// and sorted by a bitonic network in LDS; one workgroup per (snapshot, kind).
constexpr int kOrderThreads = 256;
constexpr uint64_t kOrderKeyInf = (1ull << 46) - 1;
constexpr int kMergeTile = 2048;      // merged keys one workgroup of the merge kernel produces

struct OrderLds {
  unsigned long long minback[TG_MAX_K + 1];                       // by number of options the capacity admits
  unsigned long long minres[TG_MAX_SERVICES][TG_MAX_K + 1];       // the same over the nodes a service is resident on
};

// Smallest backlog of every group of nodes of the pool (all threads of the workgroup take part).
__device__ static inline void order_minima(const TgDev& P, const TgBlock& blk, int Mt, OrderLds& L) {
  const int tid = threadIdx.x;
  const uint64_t* words = P.node_word + blk.n_off;                            // backlog | options admitted << 48, rank order
  const bool svc = P.act_service != nullptr;
  if (tid <= TG_MAX_K) L.minback[tid] = ~0ull;
  if (svc) for (int x = tid; x < TG_MAX_SERVICES * (TG_MAX_K + 1); x += kOrderThreads) (&L.minres[0][0])[x] = ~0ull;
  __syncthreads();
  for (int r = tid; r < Mt; r += kOrderThreads) {
    const uint64_t nw = words[r];
    atomicMin(&L.minback[nw >> 48], (unsigned long long)(nw & 0xffffffffffffull));
    if (svc)
      for (uint64_t left = P.node_res_k[blk.n_off + r]; left; left &= left - 1)
        atomicMin(&L.minres[__builtin_ctzll(left)][nw >> 48], (unsigned long long)(nw & 0xffffffffffffull));
  }
  __syncthreads();
}

// Key of one action: its least estimated ACT (Eq. 2) over its candidates, kOrderKeyInf if it has none.
__device__ static inline uint64_t order_key(const TgDev& P, const TgBlock& blk, const int64_t* __restrict__ dur, const OrderLds& L,
                                            size_t abase, size_t nbase, int id, int Kt) {
  const size_t g = abase + id;
  uint64_t best = kOrderKeyInf;
  if (P.act_static[g]) return best;
  const uint64_t* words = P.node_word + blk.n_off;
  const bool svc = P.act_service != nullptr;
  const uint32_t mask = P.act_kmask[g];
  const int64_t* drow = dur + g * P.K;
  const int pin = P.act_pin[g];
  const int sv = svc ? P.act_service[g] : -1;
  const uint64_t rest = sv >= 0 ? (uint64_t)P.restore[sv] : 0;               // paid where the service is not resident
  if (pin >= 0) {
    const int pr = P.node_rank[nbase + pin];
    const uint64_t nw = words[pr];
    const uint32_t ok = mask & ((1u << (nw >> 48)) - 1u);
    const uint64_t delay = sv >= 0 && !(P.node_res_k[blk.n_off + pr] >> sv & 1ull) ? rest : 0;
    if (ok) best = (nw & 0xffffffffffffull) + delay + (uint64_t)drow[31 - __builtin_clz(ok)];
  } else {
    for (int c = 1; c <= Kt; ++c) {                                         // nodes whose capacity admits options 0..c-1
      uint64_t mb = L.minback[c];
      const uint32_t ok = mask & ((1u << c) - 1u);
      if (mb == ~0ull || ok == 0) continue;
      mb += rest;                                                           // any node, restoring; or one that has the service
      if (sv >= 0 && L.minres[sv][c] < mb) mb = L.minres[sv][c];
      const uint64_t e = mb + (uint64_t)drow[31 - __builtin_clz(ok)];
      best = e < best ? e : best;
    }
  }
  return best;
}

// Bitonic sort of s_key[0 .. n_pad) in LDS, ascending (all threads of the workgroup).
__device__ static inline void order_sort_lds(uint64_t* s_key, int n_pad) {
  const int tid = threadIdx.x;
  for (int k = 2; k <= n_pad; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int x = tid; x < n_pad; x += kOrderThreads) {
        const int y = x ^ j;
        if (y > x) {
          const uint64_t a = s_key[x], c = s_key[y];
          const bool up = (x & k) == 0;
          if ((a > c) == up) { s_key[x] = c; s_key[y] = a; }
        }
      }
      __syncthreads();
    }
}

// Pools of at most kOrderTile actions: one workgroup per (snapshot, kind) computes the keys, sorts them and
// writes the visiting order.
__global__ __launch_bounds__(kOrderThreads) void tg_order_kernel(TgDev P, const int64_t* __restrict__ dur, const TgBlock* __restrict__ blocks,
                                                                 int32_t* __restrict__ visit, int n_pad_max,
                                                                 uint64_t* __restrict__ gkey) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint64_t* s_key = reinterpret_cast<uint64_t*>(smem);                       // [n_pad]
  __shared__ OrderLds L;
  const int b = blockIdx.x / 3, t = blockIdx.x - 3 * b, tid = threadIdx.x;
  const int a0 = P.tact_off[b * 4 + t], Nt = P.tact_off[b * 4 + t + 1] - a0;
  const int n0 = P.tnode_off[b * 4 + t], Mt = P.tnode_off[b * 4 + t + 1] - n0;
  if (Nt == 0) return;
  const size_t abase = (size_t)b * P.N, nbase = (size_t)b * P.M;
  const int32_t* acts = P.tact_idx + abase + a0;
  const TgBlock blk = blocks[b * 3 + t];
  order_minima(P, blk, Mt, L);
  int n_pad = 1;
  while (n_pad < Nt) n_pad <<= 1;
  const int Kt = P.type_k[t];
  for (int x = tid; x < n_pad; x += kOrderThreads) {
    uint64_t key = ~0ull;                                                     // padding sorts behind everything
    if (x < Nt) {
      const int id = acts[x];
      const uint64_t best = order_key(P, blk, dur, L, abase, nbase, id, Kt);
      key = best << 17 | (uint32_t)x;
      if (gkey) gkey[abase + id] = best << 17 | (uint32_t)id;                 // place in the order of the whole queue
    }
    s_key[x] = key;
  }
  __syncthreads();
  order_sort_lds(s_key, n_pad);
  for (int x = tid; x < Nt; x += kOrderThreads) visit[abase + a0 + x] = acts[(int)(s_key[x] & 0x1ffff)];
}

// Larger pools, first step: workgroup (pool, tile) computes the keys of kOrderTile consecutive actions of the
// pool, sorts them in LDS and writes the sorted run to `runs` (laid out like the pool's slice of the visiting order).
__global__ __launch_bounds__(kOrderThreads) void tg_order_runs_kernel(TgDev P, const int64_t* __restrict__ dur, const TgBlock* __restrict__ blocks,
                                                                      uint64_t* __restrict__ runs, uint64_t* __restrict__ gkey) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint64_t* s_key = reinterpret_cast<uint64_t*>(smem);                       // [kOrderTile]
  __shared__ OrderLds L;
  const int pool = blockIdx.x, b = pool / 3, t = pool - 3 * b, tid = threadIdx.x;   // pools along x: there can be more than 65 535
  const int a0 = P.tact_off[b * 4 + t], Nt = P.tact_off[b * 4 + t + 1] - a0;
  const int n0 = P.tnode_off[b * 4 + t], Mt = P.tnode_off[b * 4 + t + 1] - n0;
  const int x0 = (int)blockIdx.y * kOrderTile;
  if (x0 >= Nt) return;
  const size_t abase = (size_t)b * P.N, nbase = (size_t)b * P.M;
  const int32_t* acts = P.tact_idx + abase + a0;
  const TgBlock blk = blocks[b * 3 + t];
  order_minima(P, blk, Mt, L);
  const int cnt = min(kOrderTile, Nt - x0);
  int n_pad = 1;
  while (n_pad < cnt) n_pad <<= 1;
  const int Kt = P.type_k[t];
  for (int y = tid; y < n_pad; y += kOrderThreads) {
    uint64_t key = ~0ull;
    if (y < cnt) {
      const int x = x0 + y, id = acts[x];
      const uint64_t best = order_key(P, blk, dur, L, abase, nbase, id, Kt);
      key = best << 17 | (uint32_t)x;
      if (gkey) gkey[abase + id] = best << 17 | (uint32_t)id;
    }
    s_key[y] = key;
  }
  __syncthreads();
  order_sort_lds(s_key, n_pad);
  for (int y = tid; y < cnt; y += kOrderThreads) runs[abase + a0 + x0 + y] = s_key[y];
}

// Number of elements of a[0 .. na) that precede the `diag`-th element of the merge of a and b (keys are distinct).
template <class Ptr>
__device__ static inline int merge_split(Ptr a, int na, Ptr b, int nb, int diag) {
  int lo = max(0, diag - nb), hi = min(diag, na);
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;                                          // take mid+1 from a?  a[mid] must precede b[diag-mid-1]
    if (a[mid] < b[diag - mid - 1]) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// Larger pools, merge step: sorted runs of `run` keys are merged pairwise into runs of 2 * run (src -> dst).
// Workgroup (pool, tile) produces kMergeTile consecutive keys of the result: it finds by bisection which
// stretch of either run they come from, loads both stretches into LDS and every thread merges 8 keys from its
// own split point.  The last pass writes the visiting order itself instead of keys.
__global__ __launch_bounds__(kOrderThreads) void tg_order_merge_kernel(TgDev P, const uint64_t* __restrict__ src, uint64_t* __restrict__ dst,
                                                                       int32_t* __restrict__ visit, int run) {
  __shared__ uint64_t s_in[kMergeTile];
  __shared__ int s_split[2];
  const int pool = blockIdx.x, b = pool / 3, t = pool - 3 * b, tid = threadIdx.x;
  const int a0 = P.tact_off[b * 4 + t], Nt = P.tact_off[b * 4 + t + 1] - a0;
  const int o0 = (int)blockIdx.y * kMergeTile;                               // first key of the result this workgroup writes
  if (o0 >= Nt) return;
  const size_t abase = (size_t)b * P.N;
  const int32_t* acts = P.tact_idx + abase + a0;
  const uint64_t* in = src + abase + a0;
  const int pair0 = o0 / (2 * run) * (2 * run);                              // kMergeTile divides 2 * run: a tile lies in one pair
  const int na = min(run, Nt - pair0), nb = min(run, max(0, Nt - pair0 - run));
  const uint64_t* A = in + pair0;
  const uint64_t* Bq = A + na;
  const int d0 = o0 - pair0, d1 = min(d0 + kMergeTile, na + nb);
  if (tid < 2) s_split[tid] = merge_split(A, na, Bq, nb, tid == 0 ? d0 : d1);
  __syncthreads();
  const int sa0 = s_split[0], sa1 = s_split[1], sb0 = d0 - sa0, sb1 = d1 - sa1;
  const int ca = sa1 - sa0, cb = sb1 - sb0;                                  // ca + cb = d1 - d0 <= kMergeTile
  for (int x = tid; x < ca; x += kOrderThreads) s_in[x] = A[sa0 + x];
  for (int x = tid; x < cb; x += kOrderThreads) s_in[ca + x] = Bq[sb0 + x];
  __syncthreads();
  constexpr int kPer = kMergeTile / kOrderThreads;
  const int total = ca + cb, my0 = min(tid * kPer, total), my1 = min(my0 + kPer, total);
  int ia = merge_split(s_in, ca, s_in + ca, cb, my0), ib = my0 - ia;
  for (int o = my0; o < my1; ++o) {
    const bool from_a = ib >= cb || (ia < ca && s_in[ia] < s_in[ca + ib]);
    const uint64_t k = from_a ? s_in[ia] : s_in[ca + ib];
    ia += from_a; ib += !from_a;
    if (visit) visit[abase + a0 + o0 + o] = acts[(int)(k & 0x1ffff)];
    else dst[abase + a0 + o0 + o] = k;
  }
}

// ------------------------------------------------------------------------------------------
// Whole-queue prefix: the admission of a snapshot ends at the first action, in the visiting
// order of the whole queue, that a pass with one prefix per pool makes wait (before it nothing is
// closed, so both rules agree up to there).  stop[b] = that action's place in the order.
__global__ __launch_bounds__(256) void tg_stop_kernel(TgDev P, tg_assign_out O, const uint64_t* __restrict__ gkey,
                                                      uint64_t* __restrict__ stop) {
  __shared__ unsigned long long s_min;
  const int b = blockIdx.x;
  if (threadIdx.x == 0) s_min = ~0ull;
  __syncthreads();
  uint64_t m = ~0ull;
  for (int i = threadIdx.x; i < P.N; i += 256) {
    const size_t g = (size_t)b * P.N + i;
    if (O.defer_reason[g] != TG_DEFER_PREFIX) continue;
    const uint64_t k = gkey ? gkey[g] : (uint64_t)i;
    m = k < m ? k : m;
  }
  m = tg_wave_min_u64(m);
  if ((threadIdx.x & (TG_WAVE - 1)) == 0) atomicMin(&s_min, (unsigned long long)m);
  __syncthreads();
  if (threadIdx.x == 0) stop[b] = s_min;
}

// ------------------------------------------------------------------------------------------
// MAXR / MAXR_EXT / LDS_TABLE: the variants of tg_place_pool compiled into this instantiation;
// the host picks the narrowest one that takes every pool of the problem.
// WHOLE_QUEUE: with `stop` the pool's actions behind stop[b] in the order of the whole queue
// (gkey: their places under TG_ORDER_COST, else the action id is the place) are not admitted.
template <int MAXR, int MAXR_EXT, bool LDS_TABLE, bool WHOLE_QUEUE>
__global__ __launch_bounds__(TG_WAVE) void tg_place_kernel(TgDev P, const int64_t* __restrict__ dur,
                                                           const int64_t* __restrict__ cost,
                                                           const TgBlock* __restrict__ blocks, AssignWs W,
                                                           tg_assign_out O, int lds_nodes, const int32_t* __restrict__ visit,
                                                           const uint64_t* __restrict__ gkey, const uint64_t* __restrict__ stop) {
  extern __shared__ __align__(16) unsigned char smem[];
  TgPoolLds S;
  tg_pool_lds_carve(smem, lds_nodes, &S);
  const int b = blockIdx.x / 3, t = blockIdx.x - 3 * b, lane = threadIdx.x;
  const int a0 = P.tact_off[b * 4 + t], Nt = P.tact_off[b * 4 + t + 1] - a0;
  const int n0 = P.tnode_off[b * 4 + t], Mt = P.tnode_off[b * 4 + t + 1] - n0;
  const size_t abase = (size_t)b * P.N, nbase = (size_t)b * P.M;
  const int32_t* acts = (visit ? visit : P.tact_idx) + abase + a0;   // visiting order of the pool
  const int32_t* nodes = P.tnode_idx + nbase + n0;
  if (lane < TG_MAX_K) S.k[lane] = P.k_list[lane];
  for (int r = lane; r < Mt; r += TG_WAVE) {
    const size_t g = nbase + nodes[r];
    S.back[r] = P.node_backlog[g];
    S.lim[r] = t == TG_TYPE_GPU ? (int32_t)P.node_chunks[g] : P.node_free[g];
    S.cnt[r] = 0; S.dcnt[r] = 0; S.closed[r] = 0;
    if (P.node_aux) S.aux[r] = P.node_aux[g];
    if (P.node_resident) S.res[r] = P.node_resident[g];
  }
  __syncthreads();

  TgPlaceIo io;
  io.act_kmask = P.act_kmask + abase; io.act_static = P.act_static + abase; io.act_pin = P.act_pin + abase;
  io.act_aux = P.act_aux ? P.act_aux + abase : nullptr;
  io.act_service = P.act_service ? P.act_service + abase : nullptr; io.restore = P.restore;
  io.act_quota = P.act_quota && t == TG_TYPE_API ? P.act_quota + abase : nullptr;
  io.act_pin_rank = P.act_pin_rank + abase;
  io.node_rank = P.node_rank + nbase; io.nodes = nodes; io.dur = dur + abase * P.K; io.K = P.K; io.Kt = P.type_k[t];
  io.cost = nullptr; io.cost_row_len = 0;
  if (cost) { const TgBlock blk = blocks[b * 3 + t]; io.cost = cost + blk.cost_off; io.cost_row_len = blk.M_t * blk.K_t; }
  io.out_node = O.node + abase; io.out_units = O.units + abase; io.out_act = O.act_us + abase;
  io.out_reason = O.defer_reason + abase; io.slot = W.slot + abase;
  int n_adm = Nt;
  if constexpr (WHOLE_QUEUE) {
    if (stop) n_adm = tg_prefix_len(acts, Nt, gkey ? gkey + abase : nullptr, stop[b]);
  }
  tg_place_pool<MAXR, MAXR_EXT, LDS_TABLE>(S, io, acts, n_adm, Mt, t == TG_TYPE_GPU, lane);
  if constexpr (WHOLE_QUEUE) tg_place_tail(S, io, acts, n_adm, Nt, lane);   // everybody behind the end of the prefix waits

  tg_pool_extents(S, nodes, Mt, a0, W.nl_off + nbase, W.nl_cnt + nbase, W.dl_off + nbase, W.dl_cnt + nbase, lane);
}

// The same admission decided in rounds of up to 64 actions (tg_place_pool_rounds): plain problems (no second
// resource, services or further quotas), estimates recomputed, pools of up to 64 R nodes whose backlogs lie
// within 2^31 us of each other.
// R2: the table width of the GPU and API pools where they are narrower than the CPU pools' R (a wavefront pays for
// every slot of its table in every round).
template <int R, int R2>
__global__ __launch_bounds__(TG_WAVE) void tg_place_rounds_kernel(TgDev P, const int64_t* __restrict__ dur, AssignWs W,
                                                                  tg_assign_out O, int lds_nodes, const int32_t* __restrict__ visit) {
  extern __shared__ __align__(16) unsigned char smem[];
  TgPoolLds S;
  tg_pool_lds_carve(smem, lds_nodes, &S);
  const int b = blockIdx.x / 3, t = blockIdx.x - 3 * b, lane = threadIdx.x;
  const int a0 = P.tact_off[b * 4 + t], Nt = P.tact_off[b * 4 + t + 1] - a0;
  const int n0 = P.tnode_off[b * 4 + t], Mt = P.tnode_off[b * 4 + t + 1] - n0;
  const size_t abase = (size_t)b * P.N, nbase = (size_t)b * P.M;
  const int32_t* acts = (visit ? visit : P.tact_idx) + abase + a0;   // visiting order of the pool
  const int32_t* nodes = P.tnode_idx + nbase + n0;
  if (lane < TG_MAX_K) S.k[lane] = P.k_list[lane];
  for (int r = lane; r < Mt; r += TG_WAVE) {
    const size_t g = nbase + nodes[r];
    S.back[r] = P.node_backlog[g];
    S.lim[r] = t == TG_TYPE_GPU ? (int32_t)P.node_chunks[g] : P.node_free[g];
    S.cnt[r] = 0; S.dcnt[r] = 0; S.closed[r] = 0;
  }
  __syncthreads();
  TgPlaceIo io;
  io.act_kmask = P.act_kmask + abase; io.act_static = P.act_static + abase; io.act_pin = P.act_pin + abase;
  io.act_aux = nullptr; io.act_service = nullptr; io.restore = nullptr; io.act_quota = nullptr;
  io.act_pin_rank = P.act_pin_rank + abase;
  io.node_rank = P.node_rank + nbase; io.nodes = nodes; io.dur = dur + abase * P.K; io.K = P.K; io.Kt = P.type_k[t];
  io.cost = nullptr; io.cost_row_len = 0;
  io.out_node = O.node + abase; io.out_units = O.units + abase; io.out_act = O.act_us + abase;
  io.out_reason = O.defer_reason + abase; io.slot = W.slot + abase;
  if (t == TG_TYPE_GPU) tg_place_pool_rounds<R2, true>(S, io, acts, Nt, Mt, lane);
  else if (t == TG_TYPE_API && R2 != R) tg_place_pool_rounds<R2, false>(S, io, acts, Nt, Mt, lane);
  else tg_place_pool_rounds<R, false>(S, io, acts, Nt, Mt, lane);
  tg_pool_extents(S, nodes, Mt, a0, W.nl_off + nbase, W.nl_cnt + nbase, W.dl_off + nbase, W.dl_cnt + nbase, lane);
}

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void tg_lists_kernel(TgDev P, AssignWs W, tg_assign_out O) {
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t nA = (size_t)P.B * P.N, nN = (size_t)P.B * P.M;
  if (g < nA) {
    const int b = (int)(g / P.N), i = (int)(g - (size_t)b * P.N);
    const int r = O.defer_reason[g];
    if (r == TG_SELECTED) {
      const size_t n = (size_t)b * P.M + O.node[g];
      W.order[(size_t)b * P.N + W.nl_off[n] + W.slot[g]] = i;
    } else if (r == TG_DEFER_PREFIX && P.act_pin[g] >= 0) {
      const size_t n = (size_t)b * P.M + P.act_pin[g];
      W.dorder[(size_t)b * P.N + W.dl_off[n] + W.slot[g]] = i;
    }
  }
  // one thread per node: class bins (one atomic per wavefront and class), defaults of idle nodes
  const bool is_node = g >= nA && g < nA + nN;
  const size_t gn = g - nA;
  int cls = -1;
  if (is_node) {
    const int m = W.nl_cnt[gn];
    if (O.node_obj) O.node_obj[gn] = -1;
    if (m == 0) { if (O.node_used) O.node_used[gn] = 0; }
    else cls = m <= kClassCap0 ? 0 : m <= kClassCap1 ? 1 : 2;
  }
  // Places in the class lists: the four wavefronts of the workgroup add up their counts in LDS and one thread takes
  // the workgroup's stretch of every list with one atomic each (thousands of wavefronts on one counter would queue).
  // Order inside a class does not matter.  The light class holds most nodes and is handed out in batches: its dearer
  // nodes (GPU nodes: chunk states instead of unit counts) are filed from the front of the list, the others from the
  // back, so that the batches taken last are the cheap ones.
  __shared__ int s_cnt[4][4], s_base[4];                          // [wavefront][list], list = heavier classes 1, 2, light front, light back
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool dear = cls == 0 && P.node_type[is_node ? gn : 0] == TG_TYPE_GPU;
  const int which = cls == 1 ? 0 : cls == 2 ? 1 : dear ? 2 : cls == 0 ? 3 : -1;
  uint64_t bal[4];
#pragma unroll
  for (int l = 0; l < 4; ++l) { bal[l] = __ballot(which == l); if (lane == 0) s_cnt[wave][l] = __popcll(bal[l]); }
  __syncthreads();
  if (threadIdx.x < 4) {
    const int l = threadIdx.x, total = s_cnt[0][l] + s_cnt[1][l] + s_cnt[2][l] + s_cnt[3][l];
    int32_t* ctr = &W.class_ctl[l == 0 ? 2 : l == 1 ? 4 : l == 2 ? 2 * kClasses : 2 * kClasses + 1];
    s_base[l] = total ? atomicAdd(ctr, total) : 0;
  }
  __syncthreads();
  if (which >= 0) {
    int before = 0;
    for (int w = 0; w < wave; ++w) before += s_cnt[w][which];
    const size_t at = (size_t)s_base[which] + before + __popcll(bal[which] & ((1ull << lane) - 1ull));
    if (which == 0) W.class_list[nN + at] = (int32_t)gn;
    else if (which == 1) W.class_list[2 * nN + at] = (int32_t)gn;
    else if (which == 2) W.class_list[at] = (int32_t)gn;
    else W.class_list[nN - 1 - at] = (int32_t)gn;
  }
}

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(TG_WAVE) void tg_node_kernel(TgDev P, const int64_t* __restrict__ dur, AssignWs W,
                                                          tg_assign_out O, TgNodeLdsPlan plan, int cls, int grid0, int grid1,
                                                          int grid2) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x;
  const size_t nN = (size_t)P.B * P.M;
  // own class first, then the lighter ones (their nodes fit into this launch's LDS block too)
  int cur = cls;
  const int n_front = W.class_ctl[2 * kClasses];                  // light class: entries filed from the front of its list,
  const int n_light = n_front + W.class_ctl[2 * kClasses + 1];    // and all of them
  int n_nodes = cur == 0 ? n_light : W.class_ctl[2 * cur];
  const int32_t* list = W.class_list + (size_t)cur * nN;
  bool first = true;
  for (;;) {
    // A batch of nodes per fetch (the lighter the class, the more): lane j reads the table
    // entries of the batch's j-th node, so the counter and the node tables cost one memory
    // round trip per batch instead of several per node.  The head of every list belongs to the
    // wavefronts of the class's own launch, one batch each by their index (thousands of
    // wavefronts start together: no queue at the counter); everything behind it is handed out
    // by the counter.
    const int batch = cur == 0 ? kLightBatch : cur == 1 ? 2 : 1;
    const int head = (cur == 0 ? grid0 : cur == 1 ? grid1 : grid2) * batch;
    int idx0 = 0;
    if (first) idx0 = (int)blockIdx.x * batch;
    else {
      if (lane == 0) idx0 = head + atomicAdd(&W.class_ctl[2 * cur + 1], batch);   // next unprocessed nodes of the class
      idx0 = __builtin_amdgcn_readfirstlane(idx0);
    }
    first = false;
    if (idx0 >= n_nodes) {
      if (cur == 0) break;
      --cur;
      n_nodes = cur == 0 ? n_light : W.class_ctl[2 * cur];
      list = W.class_list + (size_t)cur * nN;
      continue;
    }
    const int nb = min(batch, n_nodes - idx0);
    int my_gn = 0, my_type = 0, my_cap = 0, my_free = 0, my_m = 0, my_off = 0, my_nd = 0, my_doff = 0, my_boff = 0, my_nbusy = 0;
    uint32_t my_chunks = 0;
    int64_t my_backlog = 0, my_resident = 0;
    if (lane < nb) {
      const int at = idx0 + lane;                                 // the light list continues from its far end
      my_gn = cur == 0 && at >= n_front ? list[nN - 1 - (size_t)(at - n_front)] : list[at];
      my_type = P.node_type[my_gn]; my_cap = P.node_cap[my_gn]; my_free = P.node_free[my_gn];
      my_backlog = P.node_backlog[my_gn]; my_chunks = P.node_chunks[my_gn];
      my_m = W.nl_cnt[my_gn]; my_off = W.nl_off[my_gn]; my_nd = W.dl_cnt[my_gn]; my_doff = W.dl_off[my_gn];
      if (P.has_busy) { my_boff = P.node_busy_off[my_gn]; my_nbusy = P.node_busy_off[my_gn + 1] - my_boff; }
      if (P.node_resident) my_resident = (int64_t)P.node_resident[my_gn];
    }
    // Light nodes in closed form, eight at a time (lane = 8 * node + candidate).  On a CPU node or quota with
    // nobody waiting, nothing running and at most 8 candidates whose individually fastest options fit the free
    // units together, DPArrange is not constrained: its table decomposes and every candidate takes its fastest
    // allowed option (fewest units among equals: the only allocation with the least total and, among those, the
    // fewest units).  The eviction loop then stops at once: without its last candidate the objective trades that
    // candidate's fastest duration for an estimate that starts it no earlier than the backlog on one of its first
    // `depth` options, which is never less.  Alg. 1's result is therefore everybody selected on those units, the
    // objective the sum of the durations plus the backlog once per candidate.
    uint64_t fast_done = 0;                                         // bit 8j: node j of the batch is finished
    if (cur == 0 && !P.act_service) {
      const int sj = lane >> 3, slot = lane & 7;
      const int s_gn = __shfl(my_gn, sj), s_type = __shfl(my_type, sj), s_cap = __shfl(my_cap, sj), s_free = __shfl(my_free, sj);
      const int s_m = __shfl(my_m, sj), s_off = __shfl(my_off, sj), s_nd = __shfl(my_nd, sj), s_nbusy = __shfl(my_nbusy, sj);
      const int64_t s_backlog = __shfl(my_backlog, sj);
      const bool elig = sj < nb && s_type != TG_TYPE_GPU && s_nd == 0 && s_nbusy == 0 && s_m >= 1 && s_m <= 8;
      const bool cand = elig && slot < s_m;
      const size_t abase = (size_t)(s_gn / P.M) * P.N;
      size_t ga = 0;
      if (cand) ga = abase + W.order[abase + s_off + slot];
      uint32_t mask = 0;
      int model = 0;
      int64_t age = 0, d[TG_MAX_K];
#pragma unroll
      for (int q = 0; q < TG_MAX_K; ++q) d[q] = TG_INF;
      if (cand) {
        mask = P.act_kmask[ga]; model = P.act_model[ga]; age = P.act_age[ga];
#pragma unroll
        for (int q = 0; q < TG_MAX_K; ++q) if (q < P.K) d[q] = dur[ga * P.K + q];
      }
      int64_t bd = TG_INF;
      int bk = 0;
#pragma unroll
      for (int q = 0; q < TG_MAX_K; ++q) {                          // ascending units, strict <: fewer units win ties
        const int kq = P.k_list[q < P.K ? q : 0];
        if (q < P.K && (mask >> q & 1u) && kq <= s_cap && d[q] < bd) { bd = d[q]; bk = kq; }
      }
      int tot_k = cand ? bk : 0, any_el = cand && model != TG_MODEL_NONE ? 1 : 0;
      int64_t tot_d = cand && bd != TG_INF ? bd : 0;
      int bad = cand && bd == TG_INF ? 1 : 0;                       // cannot happen after admission; then the general path decides
#pragma unroll
      for (int o = 1; o < 8; o <<= 1) {
        tot_k += __shfl_xor(tot_k, o); any_el |= __shfl_xor(any_el, o); bad |= __shfl_xor(bad, o); tot_d += __shfl_xor(tot_d, o);
      }
      const bool node_ok = elig && !bad && tot_k <= s_free;
      if (cand && node_ok) {
        O.units[ga] = bk;
        O.act_us[ga] = age + s_backlog + bd;
      }
      if (node_ok && slot == 0) {
        if (O.node_obj) O.node_obj[s_gn] = any_el ? tot_d + (int64_t)s_m * s_backlog : -1;
        if (O.node_used) O.node_used[s_gn] = tot_k;
      }
      fast_done = __ballot(node_ok && slot == 0);
    }
    for (int j = 0; j < nb; ++j) {
      if (fast_done >> (8 * j) & 1ull) continue;
      const int gn = __builtin_amdgcn_readlane(my_gn, j);
      const int b = gn / P.M;
      const size_t abase = (size_t)b * P.N;
      TgNodeIn in;
      in.type = __builtin_amdgcn_readlane(my_type, j); in.cap = __builtin_amdgcn_readlane(my_cap, j);
      in.free_units = __builtin_amdgcn_readlane(my_free, j);
      in.backlog = tg_readlane_i64(my_backlog, j); in.chunks = (uint32_t)__builtin_amdgcn_readlane((int)my_chunks, j);
      in.m = __builtin_amdgcn_readlane(my_m, j); in.clist = W.order + abase + __builtin_amdgcn_readlane(my_off, j);
      in.nd = __builtin_amdgcn_readlane(my_nd, j); in.dlist = W.dorder + abase + __builtin_amdgcn_readlane(my_doff, j);
      in.n_busy = __builtin_amdgcn_readlane(my_nbusy, j);
      in.busy = P.node_busy_rel + __builtin_amdgcn_readlane(my_boff, j);
      const bool single = in.m == 1 && in.nd == 0;                // one candidate, nobody waiting: no table, no heap
      // the release times are read by every objective evaluation: keep them behind the plan's block
      tg_wave_sync();                                             // the previous node's readers are done
      if (!single)
        for (int c = lane; c < in.n_busy; c += TG_WAVE) reinterpret_cast<int64_t*>(smem + plan.total)[c] = in.busy[c];
      in.busy_lds_off = plan.total;
      in.act_model = P.act_model + abase; in.act_kmask = P.act_kmask + abase; in.dur = dur + abase * P.K;
      in.K = P.K; in.depth = P.depth;
      in.kword = tg_pack_k(P.k_list);
      in.act_service = P.act_service ? P.act_service + abase : nullptr; in.restore = P.restore;
      in.resident = (uint64_t)tg_readlane_i64(my_resident, j);
      TgNodeOut out;
      out.node = O.node + abase; out.units = O.units + abase; out.act = O.act_us + abase; out.reason = O.defer_reason + abase;
      out.age = P.act_age + abase;
      int used = 0;
      const int64_t obj = single ? tg_node_single(in, out, lane, &used) : tg_node_schedule(smem, plan, in, out, lane, &used);
      if (lane == 0) {
        if (O.node_obj) O.node_obj[gn] = obj;
        if (O.node_used) O.node_used[gn] = used;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
constexpr int kTaskLds = 2048;

__global__ __launch_bounds__(256) void tg_summary_kernel(TgDev P, tg_assign_out O) {
  __shared__ long long s_sum;
  __shared__ int s_cnt[4];
  __shared__ long long s_used[3], s_free[3];
  __shared__ long long s_task[kTaskLds];
  const int b = blockIdx.x, tid = threadIdx.x;
  const size_t abase = (size_t)b * P.N, nbase = (size_t)b * P.M;
  const bool task_lds = O.task_sum_us && P.n_tasks <= kTaskLds;
  if (tid == 0) s_sum = 0;
  if (tid < 4) s_cnt[tid] = 0;
  if (tid < 3) { s_used[tid] = 0; s_free[tid] = 0; }
  if (task_lds) for (int k = tid; k < P.n_tasks; k += 256) s_task[k] = 0;
  else if (O.task_sum_us) for (int k = tid; k < P.n_tasks; k += 256) O.task_sum_us[(size_t)b * P.n_tasks + k] = 0;
  __syncthreads();
  long long sum = 0, used[3] = {0, 0, 0}, fr[3] = {0, 0, 0};
  int cnt[4] = {0, 0, 0, 0};
  for (int i = tid; i < P.N; i += 256) {
    const size_t g = abase + i;
    const int r = O.defer_reason[g];
    ++cnt[r];
    if (r == TG_SELECTED) {
      const long long a = O.act_us[g];
      sum += a;
      used[P.act_type[g]] += O.units[g];
      if (P.act_quota && P.act_quota[g]) {                      // tokens of the action's further quotas (Sec. 4.1)
        uint64_t more = P.act_quota[g];
        used[TG_TYPE_API] += __popcll(more);
        const int32_t* api = P.tnode_idx + nbase + P.tnode_off[b * 4 + TG_TYPE_API];
        if (O.node_used)
          for (; more; more &= more - 1) atomicAdd(&O.node_used[nbase + api[__ffsll((unsigned long long)more) - 1]], 1);
      }
      if (task_lds) atomicAdd((unsigned long long*)&s_task[P.act_task[g]], (unsigned long long)a);
      else if (O.task_sum_us) atomicAdd((unsigned long long*)&O.task_sum_us[(size_t)b * P.n_tasks + P.act_task[g]], (unsigned long long)a);
    }
  }
  for (int j = tid; j < P.M; j += 256) fr[P.node_type[nbase + j]] += P.node_free[nbase + j];
  // wavefront-level integer sums first, one LDS atomic per wavefront and quantity
  for (int o = 32; o > 0; o >>= 1) {
    sum += __shfl_xor(sum, o);
    for (int k = 0; k < 4; ++k) cnt[k] += __shfl_xor(cnt[k], o);
    for (int k = 0; k < 3; ++k) { used[k] += __shfl_xor(used[k], o); fr[k] += __shfl_xor(fr[k], o); }
  }
  if ((tid & 63) == 0) {
    atomicAdd((unsigned long long*)&s_sum, (unsigned long long)sum);
    for (int k = 0; k < 4; ++k) atomicAdd(&s_cnt[k], cnt[k]);
    for (int k = 0; k < 3; ++k) {
      atomicAdd((unsigned long long*)&s_used[k], (unsigned long long)used[k]);
      atomicAdd((unsigned long long*)&s_free[k], (unsigned long long)fr[k]);
    }
  }
  __syncthreads();
  if (task_lds) for (int k = tid; k < P.n_tasks; k += 256) O.task_sum_us[(size_t)b * P.n_tasks + k] = s_task[k];
  if (tid == 0) {
    tg_summary s;
    s.sum_act_us = s_sum;
    s.n_selected = s_cnt[0]; s.n_prefix = s_cnt[1]; s.n_evicted = s_cnt[2]; s.n_infeasible = s_cnt[3];
    for (int k = 0; k < 3; ++k) {
      s.units_used[k] = s_used[k]; s.units_free[k] = s_free[k];
      s.util[k] = s_free[k] ? (double)s_used[k] / (double)s_free[k] : 0.0;
    }
    s.mean_act_us = s_cnt[0] ? (double)s_sum / (double)s_cnt[0] : 0.0;
    O.summary[b] = s;
  }
}

// ------------------------------------------------------------------------------------------
// Sec. 5.2: which cores every selected CPU action runs on.  One wavefront per node, lane d holds
// the free cores of NUMA domain d (a domain has 4..64 cores, so it lies inside one 64-bit word
// of the node's map and a node of up to 256 cores has at most 64 domains).  The node's selected
// actions take their cores one after the other in the order of its candidate list.

__global__ __launch_bounds__(256) void tg_cores_clear_kernel(unsigned long long* core_set, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) core_set[i] = 0;
}

constexpr int kCoresWaves = 4;

__global__ __launch_bounds__(kCoresWaves * TG_WAVE) void tg_cores_kernel(TgDev P, AssignWs W, tg_assign_out O) {
  const int wave = threadIdx.x / TG_WAVE, lane = threadIdx.x % TG_WAVE;
  const size_t gn = (size_t)blockIdx.x * kCoresWaves + wave;
  if (gn >= (size_t)P.B * P.M || P.node_type[gn] != TG_TYPE_CPU) return;       // the wavefronts of a workgroup never meet
  const int m = W.nl_cnt[gn];
  if (m == 0) return;
  const size_t abase = (gn / P.M) * (size_t)P.N;
  const int32_t* list = W.order + abase + W.nl_off[gn];
  const int nc = P.numa_cores, cap = P.node_cap[gn];
  const int n_dom = (cap + nc - 1) / nc;
  const int word = (lane * nc) >> 6, shift = (lane * nc) & 63;
  uint64_t dm = 0;                                                // free cores of this lane's domain
  if (lane < n_dom) {
    dm = P.node_cores[gn * 4 + word] >> shift;
    if (nc < 64) dm &= (1ull << nc) - 1;
  }
  for (int base = 0; base < m; base += TG_WAVE) {
    const int n = m - base < TG_WAVE ? m - base : TG_WAVE;
    const int my_a = lane < n ? list[base + lane] : 0;
    const int my_k = lane < n ? O.units[abase + my_a] : 0;
    for (int l = 0; l < n; ++l) {
      const int a = __builtin_amdgcn_readlane(my_a, l), k = __builtin_amdgcn_readlane(my_k, l);
      if (k == 0) continue;                                       // evicted: no cores
      bool one_domain;
      const uint64_t take = tg_take_cores(dm, k, lane, &one_domain);
      // the map of every action was cleared before this kernel: only the words that get cores are touched
      if (take) {
        unsigned long long* dst = (unsigned long long*)O.core_set + (abase + a) * 4 + word;
        if (one_domain) *dst = take << shift;
        else atomicOr(dst, (unsigned long long)(take << shift));  // several domains may share a word; OR commutes
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Pooled GPUs (Sec. 5.3, Alg. 4): the node stage has scheduled the pool as one resource at the
// snapshot's first GPU node.  One wavefront per snapshot, lane r = the r-th GPU node with its
// own free chunks: the pool's selected actions, in list order, each take the smallest free
// chunk of the cluster that holds them, on the lowest-numbered node that has one - the same
// sequence of takes the pool's chunk counts went through, so every take succeeds.
__global__ __launch_bounds__(TG_WAVE) void tg_pool_map_kernel(TgDev P, AssignWs W, tg_assign_out O) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const size_t abase = (size_t)b * P.N, nbase = (size_t)b * P.M;
  const int n0 = P.tnode_off[b * 4 + TG_TYPE_GPU], n_gpu = P.tnode_off[b * 4 + TG_TYPE_GPU + 1] - n0;
  if (n_gpu == 0) return;
  const int32_t* gpu_nodes = P.tnode_idx + nbase + n0;            // index order; at most 8 of them
  const int my_node = lane < n_gpu ? gpu_nodes[lane] : -1;
  uint32_t chunks = lane < n_gpu ? P.node_chunks_real[nbase + my_node] : 0u;
  int used = 0;
  const size_t pool = nbase + gpu_nodes[0];
  const int m = W.nl_cnt[pool];
  const int32_t* list = W.order + abase + W.nl_off[pool];
  for (int base = 0; base < m; base += TG_WAVE) {
    const int n = m - base < TG_WAVE ? m - base : TG_WAVE;
    const int my_a = lane < n ? list[base + lane] : 0;
    const int my_k = lane < n ? O.units[abase + my_a] : 0;
    int my_dst = -1;
    for (int l = 0; l < n; ++l) {
      const int k = __builtin_amdgcn_readlane(my_k, l);
      if (k == 0) continue;                                       // evicted
      int level = 4;                                              // smallest free chunk of this node that holds k
      for (int x = 3; x >= tg_chunk_level(k); --x) if ((chunks >> (8 * x)) & 0xffu) level = x;
      const uint32_t best = tg_wave_min_u32(level < 4 ? (uint32_t)level << 8 | (uint32_t)lane : 0xffffffffu);
      if (best == 0xffffffffu) continue;                          // cannot happen: the pool's counts had such a chunk
      const int r = (int)(best & 0xffu);
      const int dst = __builtin_amdgcn_readlane(my_node, r);
      if (lane == r) { chunks = tg_chunk_take(chunks, k); used += k; }
      if (lane == l) my_dst = dst;
    }
    if (lane < n && my_dst >= 0) O.node[abase + my_a] = my_dst;
  }
  if (O.node_used && lane < n_gpu) O.node_used[nbase + my_node] = used;
}

}  // namespace

extern "C" int tg_assign_workspace_bytes(const tg_problem* p, size_t* bytes) {
  if (!p || !bytes) return TG_E_INVALID_ARG;
  *bytes = carve(p, nullptr, nullptr);
  return TG_OK;
}

namespace {
int check_assign_args(const tg_problem* p, const tg_assign_out* out, const void* d_ws, size_t ws_bytes) {
  if (!p || !out || !out->node || !out->units || !out->act_us || !out->defer_reason || !out->summary)
    return TG_E_INVALID_ARG;
  if (out->core_set && !p->dev.node_cores) return TG_E_INVALID_ARG;
  if (!d_ws || ((uintptr_t)d_ws & 255) || ws_bytes < carve(p, nullptr, nullptr)) return TG_E_WORKSPACE;
  return TG_OK;
}
}  // namespace

namespace {
int assign_launch(const tg_problem* p, const int64_t* d_cost, const tg_assign_out* out, void* d_ws, hipStream_t s,
                  hipEvent_t before_nodes, bool prepare_only);
}  // namespace

extern "C" int tg_step_on(const tg_problem* p, int64_t* d_cost, const tg_assign_out* out, void* d_ws, size_t ws_bytes,
                          void* hip_stream, void* score_stream) {
  const int rc = check_assign_args(p, out, d_ws, ws_bytes);
  if (rc) return rc;
  if ((!d_cost && p->n_candidates) || ((uintptr_t)d_cost & 15) || score_stream == hip_stream) return TG_E_INVALID_ARG;
  hipStream_t s = (hipStream_t)hip_stream, ss = (hipStream_t)score_stream;
  // everything that can fail for a reason other than a launch comes first: on such an error nothing has been launched
  const int rp = assign_launch(p, nullptr, out, d_ws, s, nullptr, true);
  if (rp) return rp;
  // The assignment does not read the tensor, so the two could run side by side - but the score kernels and the
  // per-node stage both live on the vector ALUs' issue slots (measured: next to each other each takes as long as
  // both in a row), and the score kernels' short workgroups need all of the chip's wavefront slots to keep HBM busy.
  // So: a large tensor (4 GB and more) is written first, with the chip to itself, and the assignment follows; a
  // small one is written next to the first, light kernels of the assignment (durations, admission, lists: a few
  // wavefronts per compute unit, too short to matter) and only the per-node stage waits for it.  Forked from and
  // joined back into the caller's stream.
  const bool big = p->n_candidates >= (1ll << 29);
  TG_HIP_CHECK(hipEventRecord(p->ev_score_fork, s));
  TG_HIP_CHECK(hipStreamWaitEvent(ss, p->ev_score_fork, 0));
  const int rs = tg_launch_score(p, d_cost, ss);
  TG_HIP_CHECK(hipEventRecord(p->ev_score_done, ss));
  if (big) TG_HIP_CHECK(hipStreamWaitEvent(s, p->ev_score_done, 0));
  const int ra = assign_launch(p, nullptr, out, d_ws, s, big ? nullptr : p->ev_score_done, false);
  if (!big) TG_HIP_CHECK(hipStreamWaitEvent(s, p->ev_score_done, 0));
  return rs ? rs : ra;
}

extern "C" int tg_step(const tg_problem* p, int64_t* d_cost, const tg_assign_out* out, void* d_ws, size_t ws_bytes,
                       void* hip_stream) {
  if (!p) return TG_E_INVALID_ARG;
  return tg_step_on(p, d_cost, out, d_ws, ws_bytes, hip_stream, p->score_stream);
}

// Workspace of tg_assign_static: one array per GPU in the library's own device data, so that the entry
// point never allocates.  Host code reaches it only through the address hipGetSymbolAddress returns for
// the current device (the array's name is no device address on the host), looked up once per device.
static __device__ __align__(256) unsigned char scratch[TG_STATIC_WS_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

int static_workspace(void** ptr) {
  int dev = -1;
  TG_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return TG_E_HIP;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {                                                       // first call on this device (racing threads find the same address)
    TG_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || ((uintptr_t)p & 255)) return TG_E_HIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return TG_OK;
}

}  // namespace

extern "C" int tg_assign(const tg_problem* p, const int64_t* d_cost, const tg_assign_out* out, void* d_ws,
                         size_t ws_bytes, void* hip_stream) {
  const int rc_args = check_assign_args(p, out, d_ws, ws_bytes);
  if (rc_args) return rc_args;
  return assign_launch(p, d_cost, out, d_ws, (hipStream_t)hip_stream, nullptr, false);
}

extern "C" int tg_assign_static(const tg_problem* p, const int64_t* d_cost, const tg_assign_out* out, void* hip_stream) {
  if (!p) return TG_E_INVALID_ARG;
  if (carve(p, nullptr, nullptr) > (size_t)TG_STATIC_WS_BYTES) return TG_E_STATIC_WS;
  void* ws = nullptr;
  const int rc_ws = static_workspace(&ws);
  if (rc_ws) return rc_ws;
  const int rc_args = check_assign_args(p, out, ws, TG_STATIC_WS_BYTES);
  if (rc_args) return rc_args;
  return assign_launch(p, d_cost, out, ws, (hipStream_t)hip_stream, nullptr, false);
}

namespace {
// before_nodes: an event the per-node stage waits for (tg_step: the score kernels), or nullptr.
// prepare_only: do what can fail before anything is launched (the kernels' LDS limits) and return.
int assign_launch(const tg_problem* p, const int64_t* d_cost, const tg_assign_out* out, void* d_ws, hipStream_t s,
                  hipEvent_t before_nodes, bool prepare_only) {
  const TgDev& P = p->dev;
  AssignWs W;
  carve(p, (char*)d_ws, &W);
  const size_t nA = (size_t)P.B * P.N;

  const size_t place_lds = tg_pool_lds_bytes(p->max_nodes_of_kind);
  TgNodeLdsPlan plans[kClasses];
  int max_lds = 0;
  for (int c = 0; c < kClasses; ++c) {
    plans[c] = tg_node_lds_plan(p->max_free_cpu, p->max_free_gpu, p->max_chunk_states, p->max_heap, P.K, class_cap(c), kSelRows);
    max_lds = plans[c].total > max_lds ? plans[c].total : max_lds;
  }
  const int busy_lds = ((p->max_heap + 1) & ~1) * 8;              // a node's busy list has at most max_heap entries
  max_lds += busy_lds;
  if (max_lds > 64 * 1024)
    TG_HIP_CHECK(hipFuncSetAttribute((const void*)tg_node_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, max_lds));

  const size_t nN = (size_t)P.B * P.M;
  if (!prepare_only) hipLaunchKernelGGL(tg_dur_kernel, dim3((unsigned)((nA * P.K + 255) / 256)), dim3(256), 0, s, P, W.dur, W.class_ctl);
  const int32_t* visit = nullptr;
  if (p->order_policy == TG_ORDER_COST) {
    uint64_t* gkey = p->queue_prefix ? W.gkey : nullptr;
    if (p->max_actions_of_kind <= kOrderTile) {
      int n_pad = 1;
      while (n_pad < p->max_actions_of_kind) n_pad <<= 1;
      const size_t order_lds = (size_t)n_pad * 8;
      if (order_lds > 48 * 1024)
        TG_HIP_CHECK(hipFuncSetAttribute((const void*)tg_order_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)order_lds));
      if (!prepare_only) hipLaunchKernelGGL(tg_order_kernel, dim3(P.B * 3), dim3(kOrderThreads), order_lds, s, P, W.dur, p->d_blocks, W.visit, n_pad, gkey);
    } else {
      // a pool too large for one workgroup: sorted runs of kOrderTile keys, then pairwise merges of the runs
      const size_t runs_lds = (size_t)kOrderTile * 8;
      TG_HIP_CHECK(hipFuncSetAttribute((const void*)tg_order_runs_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)runs_lds));
      const unsigned pools = (unsigned)P.B * 3;
      if (!prepare_only) {
        hipLaunchKernelGGL(tg_order_runs_kernel, dim3(pools, (p->max_actions_of_kind + kOrderTile - 1) / kOrderTile), dim3(kOrderThreads),
                           runs_lds, s, P, W.dur, p->d_blocks, W.okey_a, gkey);
        const uint64_t* src = W.okey_a;
        uint64_t* dst = W.okey_b;
        const unsigned tiles = (unsigned)((p->max_actions_of_kind + kMergeTile - 1) / kMergeTile);
        for (int run = kOrderTile; run < p->max_actions_of_kind; run *= 2) {
          const bool last = 2 * (int64_t)run >= p->max_actions_of_kind;
          hipLaunchKernelGGL(tg_order_merge_kernel, dim3(pools, tiles), dim3(kOrderThreads), 0, s, P, src, dst, last ? W.visit : nullptr, run);
          const uint64_t* was = src; src = dst; dst = const_cast<uint64_t*>(was);
        }
      }
    }
    visit = W.visit;
  }
  // the rows of the score tensor are in FCFS order: another visiting order recomputes Eq. 2 instead
  {
    // the node table of a pool lives in registers (1, 4 or 16 nodes per lane) unless the estimates
    // come from the score tensor or a pool has more than 1024 nodes (then: a table in LDS)
    const int64_t* place_cost = visit ? nullptr : d_cost;
    const bool ext = P.act_aux || P.act_service || P.act_quota;
    const int mk = p->max_nodes_of_kind;
    const int width = place_cost || mk > 16 * TG_WAVE ? 0 : mk <= TG_WAVE ? 1 : mk <= 4 * TG_WAVE ? 4 : 16;
    using PlaceKernel = void (*)(TgDev, const int64_t*, const int64_t*, const TgBlock*, AssignWs, tg_assign_out, int, const int32_t*,
                                 const uint64_t*, const uint64_t*);
    PlaceKernel k = width == 0 ? tg_place_kernel<0, 0, true, false>
                  : width == 1 ? (ext ? tg_place_kernel<1, 1, false, false> : tg_place_kernel<1, 0, false, false>)
                  : width == 4 ? (ext ? tg_place_kernel<4, 4, false, false> : tg_place_kernel<4, 0, false, false>)
                               : (ext ? tg_place_kernel<16, 16, false, false> : tg_place_kernel<16, 0, false, false>);
    if (!ext && width != 0 && p->backlog_spread < (1ll << 31)) {
      // plain problem: the admission in rounds of up to 64 actions
      using RoundsKernel = void (*)(TgDev, const int64_t*, AssignWs, tg_assign_out, int, const int32_t*);
      const int mo = p->max_nodes_not_cpu;
      const int width2 = mo <= TG_WAVE ? 1 : mo <= 4 * TG_WAVE ? 4 : 16;
      RoundsKernel kr = width == 1 ? tg_place_rounds_kernel<1, 1>
                      : width == 4 ? (width2 == 1 ? tg_place_rounds_kernel<4, 1> : tg_place_rounds_kernel<4, 4>)
                      : width2 == 1 ? tg_place_rounds_kernel<16, 1> : width2 == 4 ? tg_place_rounds_kernel<16, 4> : tg_place_rounds_kernel<16, 16>;
      if (place_lds > 64 * 1024)
        TG_HIP_CHECK(hipFuncSetAttribute((const void*)kr, hipFuncAttributeMaxDynamicSharedMemorySize, (int)place_lds));
      if (!prepare_only) hipLaunchKernelGGL(kr, dim3(P.B * 3), dim3(TG_WAVE), place_lds, s, P, W.dur, W, *out, p->max_nodes_of_kind, visit);
    } else {
      if (place_lds > 64 * 1024)
        TG_HIP_CHECK(hipFuncSetAttribute((const void*)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)place_lds));
      if (!prepare_only) hipLaunchKernelGGL(k, dim3(P.B * 3), dim3(TG_WAVE), place_lds, s, P, W.dur, place_cost, p->d_blocks, W, *out,
                         p->max_nodes_of_kind, visit, nullptr, nullptr);
    }
    if (p->queue_prefix) {
      // one prefix of the whole queue: the pass above (one prefix per pool) finds where it ends, a
      // second pass admits the actions before that place and leaves the others waiting
      const uint64_t* gkey = visit ? W.gkey : nullptr;
      PlaceKernel k2 = tg_place_kernel<0, 0, true, true>;
      if (place_lds > 64 * 1024)
        TG_HIP_CHECK(hipFuncSetAttribute((const void*)k2, hipFuncAttributeMaxDynamicSharedMemorySize, (int)place_lds));
      if (!prepare_only) hipLaunchKernelGGL(tg_stop_kernel, dim3(P.B), dim3(256), 0, s, P, *out, gkey, W.stop);
      if (!prepare_only) hipLaunchKernelGGL(k2, dim3(P.B * 3), dim3(TG_WAVE), place_lds, s, P, W.dur, place_cost, p->d_blocks, W, *out,
                         p->max_nodes_of_kind, visit, gkey, W.stop);
    }
  }
  if (!prepare_only) hipLaunchKernelGGL(tg_lists_kernel, dim3((unsigned)((nA + nN + 255) / 256)), dim3(256), 0, s, P, W, *out);
  // Persistent wavefronts pull nodes of their class and, when it is exhausted, of the lighter
  // classes.  The classes are independent and each is bound by the latency of its own
  // wavefronts, so the two light classes run on side streams next to the heavy one.
  if (prepare_only) return TG_OK;
  if (before_nodes) TG_HIP_CHECK(hipStreamWaitEvent(s, before_nodes, 0));
  TG_HIP_CHECK(hipEventRecord(p->ev_fork, s));
  // LDS decides how many wavefronts a CU holds.  The heaviest class that can have nodes gets one
  // wavefront per possible node as far as 80 % of a CU's LDS go - 90 % where there can be many more
  // heavy nodes than such wavefronts (a heavy wavefront is bound by its own latency, and the light
  // ones cannot take its nodes); its wavefronts that find no node of their own (and those that
  // finish early) serve the class below, so the middle class is only launched from what the light
  // class - the bulk of the nodes - leaves over.
  const size_t bound[kClasses] = {nN, p->nodes_free_gt16, p->nodes_free_gt64};
  const int kCus = 256, kLdsPerCu = 160 * 1024, kLdsGranule = 1024;   // allocations are rounded up (granule assumed, not documented)
  const int heavy = bound[2] > 0 ? 2 : bound[1] > 0 ? 1 : 0;      // classes above it are empty
  int per_cu[kClasses] = {0, 0, 0}, bytes[kClasses], want[kClasses];
  for (int c = 0; c < kClasses; ++c) {
    bytes[c] = (plans[c].total + busy_lds + kLdsGranule - 1) / kLdsGranule * kLdsGranule;
    want[c] = (int)std::min<size_t>((bound[c] + kCus - 1) / kCus, 32);
  }
  int lds_left = kLdsPerCu;
  if (heavy > 0) {
    per_cu[heavy] = std::max(1, std::min(want[heavy], kLdsPerCu * 8 / 10 / bytes[heavy]));
    if (bound[heavy] >= (size_t)8 * kCus * per_cu[heavy])
      per_cu[heavy] = std::max(per_cu[heavy], std::min(want[heavy], kLdsPerCu * 9 / 10 / bytes[heavy]));
    lds_left -= per_cu[heavy] * bytes[heavy];
  }
  // a thin heavy launch cannot absorb a long middle list: then the middle class keeps wavefronts of its own
  const int own1 = heavy == 2 && per_cu[2] < 3 && bound[1] > (size_t)kCus * per_cu[2] ? std::min(want[1], 4) : 0;
  per_cu[0] = std::max(1, std::min(want[0], (lds_left - own1 * bytes[1]) / bytes[0]));
  lds_left = std::max(0, lds_left - per_cu[0] * bytes[0]);
  if (heavy == 2) per_cu[1] = std::min(std::max(own1, std::min(want[1], 1)), lds_left / bytes[1]);
  bool forked[2] = {false, false};
  int grids[kClasses];
  for (int c = 0; c < kClasses; ++c)
    grids[c] = per_cu[c] == 0 ? 0 : (int)std::max<size_t>(1, std::min<size_t>(bound[c], (size_t)kCus * per_cu[c]));
  for (int c = kClasses - 1; c >= 0; --c) {                     // heaviest class first
    if (per_cu[c] == 0) continue;
    const unsigned grid = (unsigned)grids[c];
    hipStream_t cs = c < 2 ? p->side_stream[c] : s;
    if (c < 2) { TG_HIP_CHECK(hipStreamWaitEvent(cs, p->ev_fork, 0)); forked[c] = true; }
    hipLaunchKernelGGL(tg_node_kernel, dim3(grid), dim3(TG_WAVE), plans[c].total + busy_lds, cs, P, W.dur, W, *out, plans[c], c,
                       grids[0], grids[1], grids[2]);
    if (c < 2) TG_HIP_CHECK(hipEventRecord(p->ev_join[c], cs));
  }
  for (int c = 0; c < 2; ++c) if (forked[c]) TG_HIP_CHECK(hipStreamWaitEvent(s, p->ev_join[c], 0));
  if (P.node_chunks_real) hipLaunchKernelGGL(tg_pool_map_kernel, dim3(P.B), dim3(TG_WAVE), 0, s, P, W, *out);
  if (out->core_set) {
    hipLaunchKernelGGL(tg_cores_clear_kernel, dim3((unsigned)((nA * 4 + 255) / 256)), dim3(256), 0, s,
                       (unsigned long long*)out->core_set, nA * 4);
    hipLaunchKernelGGL(tg_cores_kernel, dim3((unsigned)((nN + kCoresWaves - 1) / kCoresWaves)), dim3(kCoresWaves * TG_WAVE), 0, s,
                       P, W, *out);
  }
  hipLaunchKernelGGL(tg_summary_kernel, dim3(P.B), dim3(256), 0, s, P, *out);
  return hipGetLastError() == hipSuccess ? TG_OK : TG_E_HIP;
}
}  // namespace
