// tg_replay_trace: S independent arrival traces, one persistent workgroup per scenario.
//
// Every tick the workgroup runs the same scheduling step as tg_assign (the wavefront-level
// functions of tg_step.h) on the scenario's live state: the three resource pools are placed,
// the nodes that received candidates run DPArrange + eviction in a per-node LDS block, and
// selected actions start at the tick (GPU nodes also update their cache of resident services
// then).  The tick loop is bounded by max_ticks, so every wavefront leaves the kernel.
//
// A workgroup is ONE wavefront (kWaves): a tick is a chain of dependent memory accesses that
// keeps a wavefront waiting most of the time, and registers allow eight wavefronts per CU
// whatever their grouping - eight scenarios in flight per CU finish a batch of thousands twice
// as fast as two scenarios with four wavefronts each, whose extra wavefronts mostly idle at
// barriers.  The code below is written for kWaves wavefronts (kinds and nodes are dealt out
// by wavefront index); the LDS of the placement and of the node stage overlap, since the
// placement tables are dead when the node stage begins, so that eight workgroups fit a CU.
//
// Live state per scenario (global workspace, L2 resident): free cores per CPU node, free-GPU
// bit mask per GPU node (a free chunk is a maximal aligned free block, so releasing coalesces
// by itself), micro-tokens per quota, the running set (finish, node, units, first GPU), one
// FCFS waiting list per resource kind and, with services, the resident set of every node with
// the last use of each service.
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "tg_step.h"

struct TgTraceDev {
  int S, A, M, K, n_classes, depth, max_ticks, cache_slots;
  int queue_prefix;               // 1: every step admits one prefix of the whole waiting queue (Alg. 1 as printed)
  int64_t tick_us;
  int k_list[TG_MAX_K];
  int type_k[4];
  const uint8_t* node_type; const int32_t* node_cap; const int32_t* quota_rate; const int64_t* quota_tok0;
  const int32_t* node_rank; const int32_t* tnode_idx; const int32_t* tnode_off;   // [S*M], [S*M], [S*4]
  const int64_t* arrival; const uint8_t* act_type; const uint8_t* act_model; const uint8_t* act_static;
  const int64_t* act_T; const uint32_t* act_kmask; const uint32_t* act_param; const int32_t* act_pin;
  const uint32_t* speedup;
  const int32_t* act_service;     // [S*A] service of a GPU action or -1; nullptr: the trace has no services (Sec. 5.3)
  const int64_t* restore;         // [TG_MAX_SERVICES]
  const uint64_t* act_quota;      // [S*A] further quotas of an API action (ranks among the scenario's API nodes), or nullptr (Sec. 4.1)
  const int32_t* node_aux;        // [S*M] second resource of every node, or nullptr: none (Sec. 4.1, 5.2)
  const int32_t* act_aux;         // [S*A] what an action that is free to choose its node holds of it while it runs
  int numa_cores;                 // > 0: CPU actions get named cores, NUMA domains of this many (Sec. 5.2)
  int gpu_pooled;                 // 1: every step sees the GPU nodes of the scenario as one pool of chunks (Sec. 5.3, Alg. 4)
  int cache_per_gpu;              // 1 (only with services): every GPU of a GPU node keeps its own cache (Sec. 5.3)
  int order_cost;                 // 1: every step visits the waiting queue by least estimated ACT (Sec. 4.2), ties by arrival
  const int32_t* kind_cap;        // [S*3] largest node of every kind in the scenario (-1: none); only with order_cost
};

// What the sizes of a trace's tables follow from: nodes of every kind in one scenario, capacities.
struct TraceMaxima {
  int nodes_kind[3];        // most nodes of a kind in one scenario
  int max_cap_cpu;          // largest CPU node
  int max_free_gpu;         // GPUs of the largest GPU resource a step schedules: a node's 8, or those of a pool
  int max_heap;             // largest CPU or GPU resource: entries of Alg. 2's heap
  int max_chunk_states;     // states of Alg. 4's table on one GPU resource
};

// Most states (product of max(count, 1) + 1 over the four chunk sizes) the summed free-chunk counts of n 8-GPU nodes
// can have, n = 0..5: the largest product over all sums of n count vectors, each the counts of one of the 256 free
// masks of a node.  Six nodes could reach 810, above TG_MAX_CHUNK_STATES.
constexpr int kPoolNodesMax = 5;
constexpr int kPoolStates[kPoolNodesMax + 1] = {1, 40, 100, 196, 324, 512};

struct tg_trace {
  TgTraceDev dev;
  void* d_arena;
  size_t arena_bytes;
  TraceMaxima mx;
};

namespace {

constexpr int kWaves = 1;
constexpr int kThreads = kWaves * TG_WAVE;

struct ReplayWs {
  int64_t* dur;        // [S*A*K]
  int32_t* slot;       // [S*A]
  int32_t* order;      // [S*A]
  int32_t* dorder;     // [S*A]
  int32_t* wlist;      // [S*3*A] waiting list per kind
  int64_t* run_fin;    // [S*A]
  int32_t* run_info;   // [S*A] node | units << 16 | first GPU << 24
  uint8_t* reason;     // [S*A]
  int32_t *nl_off, *nl_cnt, *dl_off, *dl_cnt;   // [S*M]
  int32_t* live_free;  // [S*M] free cores / free-GPU mask
  int64_t* live_tok;   // [S*M]
  // service cache (only with services)
  uint64_t* live_res;  // [S*M] services resident on the node
  int32_t* used_at;    // [S*M*64] per node and service: sequence number of its last use
  int32_t* use_seq;    // [S*M] uses counted so far
  // second resource (only with node_aux / act_aux)
  int32_t* live_aux;   // [S*M] what the node has left
  int32_t* run_aux;    // [S*A] what the running action holds, alongside run_fin / run_info
  // named cores (only with numa_cores > 0)
  uint64_t* live_cores;  // [S*M*4] free cores of every CPU node
  int32_t* run_id;       // [S*A] the running action's id (its cores are in the output map), alongside run_fin / run_info
  // second visiting order (only with order_cost)
  uint64_t* gpu_res;     // [S*M*8] services resident on every GPU of a node (only with cache_per_gpu; used_at then has 8 x 64 per node)
  int32_t* resume;       // [S*16] what a scenario needs besides the arrays above to go on where a call stopped
  uint64_t* okey;        // [S*A] (least estimated ACT of the action << 17) | action id: its place in the visiting order
  uint64_t* okey0;       // [S*A] the same without any restore delay, and
  uint64_t* skey;        // [S*A] the keys of a waiting list in list order (both only with order_cost and services)
  int32_t* wlist2;       // [S*3*A] the other half of the waiting lists' ping-pong (new arrivals are merged into the sorted list)
};

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

size_t carve(const TgTraceDev& T, char* base, ReplayWs* w) {
  const size_t nA = (size_t)T.S * T.A, nN = (size_t)T.S * T.M;
  size_t off = 0;
  auto take = [&](size_t bytes) { char* r = base + off; off += align256(bytes); return r; };
  char* p[14];
  p[0] = take(nA * T.K * 8); p[1] = take(nA * 4); p[2] = take(nA * 4); p[3] = take(nA * 4); p[4] = take(nA * 3 * 4);
  p[5] = take(nA * 8); p[6] = take(nA * 4); p[7] = take(nA);
  for (int x = 8; x < 13; ++x) p[x] = take(nN * 4);
  p[13] = take(nN * 8);
  const bool svc = T.act_service != nullptr;
  const size_t caches = T.cache_per_gpu ? 8 : 1;                  // per node
  char* q0 = take(svc ? nN * 8 : 0); char* q1 = take(svc ? nN * caches * 64 * 4 : 0); char* q2 = take(svc ? nN * 4 : 0);
  char* q3 = take(T.cache_per_gpu ? nN * 8 * 8 : 0);
  char* x0 = take(T.node_aux ? nN * 4 : 0); char* x1 = take(T.node_aux ? nA * 4 : 0);
  char* c0 = take(T.numa_cores ? nN * 32 : 0); char* c1 = take(T.numa_cores ? nA * 4 : 0);
  char* k0 = take(T.order_cost ? nA * 8 : 0); char* k1 = take(T.order_cost ? nA * 3 * 4 : 0);
  char* k2 = take(T.order_cost && svc ? nA * 8 : 0); char* k3 = take(T.order_cost && svc ? nA * 8 : 0);
  char* rs = take((size_t)T.S * 16 * 4);
  if (w) {
    w->resume = (int32_t*)rs; w->gpu_res = (uint64_t*)q3;
    w->okey = (uint64_t*)k0; w->wlist2 = (int32_t*)k1; w->okey0 = (uint64_t*)k2; w->skey = (uint64_t*)k3;
    w->live_cores = (uint64_t*)c0; w->run_id = (int32_t*)c1;
    w->live_aux = (int32_t*)x0; w->run_aux = (int32_t*)x1;
    w->live_res = (uint64_t*)q0; w->used_at = (int32_t*)q1; w->use_seq = (int32_t*)q2;
    w->dur = (int64_t*)p[0]; w->slot = (int32_t*)p[1]; w->order = (int32_t*)p[2]; w->dorder = (int32_t*)p[3];
    w->wlist = (int32_t*)p[4]; w->run_fin = (int64_t*)p[5]; w->run_info = (int32_t*)p[6]; w->reason = (uint8_t*)p[7];
    w->nl_off = (int32_t*)p[8]; w->nl_cnt = (int32_t*)p[9]; w->dl_off = (int32_t*)p[10]; w->dl_cnt = (int32_t*)p[11];
    w->live_free = (int32_t*)p[12]; w->live_tok = (int64_t*)p[13];
  }
  return off;
}

__global__ __launch_bounds__(256) void tg_trace_dur_kernel(TgTraceDev T, int64_t* __restrict__ dur) {
  const size_t x = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t total = (size_t)T.S * T.A * T.K;
  if (x >= total) return;
  const size_t g = x / T.K;
  const int q = (int)(x - g * T.K);
  int64_t d = TG_INF;
  if (T.act_kmask[g] >> q & 1u) {
    const int model = T.act_model[g];
    const uint32_t param = T.act_param[g];
    const uint32_t sp = model == TG_MODEL_TABLE ? T.speedup[param * T.K + q] : 0u;
    d = tg_duration(model, T.act_T[g], param, T.k_list[q], sp);
  }
  dur[x] = d;
}

// Second visiting order: the key of an action is its least estimated ACT over its candidates (Eq. 2).  In a replay
// every backlog is 0 and, without services, nothing is restored, so the key is the action's duration on the largest
// allowed option that the largest node it may use admits (durations do not grow with the units) - a constant of the
// action.  Packed with the action id (ids ascend with the arrivals) into its place in the visiting order.
constexpr uint64_t kKeyInf = (1ull << 46) - 1;

__global__ __launch_bounds__(256) void tg_trace_key_kernel(TgTraceDev T, const int64_t* __restrict__ dur, uint64_t* __restrict__ okey,
                                                           uint64_t* __restrict__ okey0) {
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= (size_t)T.S * T.A) return;
  const int s = (int)(g / T.A), i = (int)(g - (size_t)s * T.A);
  uint64_t key = kKeyInf;
  if (!T.act_static[g]) {
    const int ty = T.act_type[g], pin = T.act_pin[g];
    const int cap = pin >= 0 ? T.node_cap[(size_t)s * T.M + pin] : T.kind_cap[s * 3 + ty];
    int c = 0;
    while (c < T.type_k[ty] && T.k_list[c] <= cap) ++c;
    const uint32_t ok = T.act_kmask[g] & ((1u << c) - 1u);
    if (ok) key = (uint64_t)dur[g * T.K + (31 - __builtin_clz(ok))];
  }
  okey[g] = key << 17 | (uint32_t)i;
  if (T.act_service) okey0[g] = key << 17 | (uint32_t)i;          // the replay adds this tick's restore delay to it
}

// free chunks (sizes 1,2,4,8) of an 8-GPU node as packed 8-bit counts: a chunk is an aligned
// free block whose enclosing block of twice the size is not entirely free
__device__ inline uint32_t mask_chunks(uint32_t m) {
  if (m == 0xffu) return 1u << 24;
  uint32_t c = 0;
#pragma unroll
  for (int half = 0; half < 8; half += 4) {
    const uint32_t h = (m >> half) & 0xfu;
    if (h == 0xfu) { c += 1u << 16; continue; }
#pragma unroll
    for (int pair = 0; pair < 4; pair += 2) {
      const uint32_t p = (h >> pair) & 0x3u;
      if (p == 0x3u) c += 1u << 8; else c += __popc(p);
    }
  }
  return c;
}

// best fit, lowest address (Sec. 5.3): returns the first GPU of the allocation and clears its bits
__device__ inline int mask_alloc(uint32_t& m, int k) {
  const int a = tg_chunk_level(k);
  for (int lvl = a; lvl < 4; ++lvl) {
    const int sz = 1 << lvl;
    for (int s = 0; s < 8; s += sz) {
      const uint32_t blk = ((1u << sz) - 1u) << s;
      if ((m & blk) != blk) continue;
      if (lvl < 3) {
        const int ps = s & ~(2 * sz - 1);
        const uint32_t pb = ((1u << (2 * sz)) - 1u) << ps;
        if ((m & pb) == pb) continue;
      }
      m &= ~(((1u << (1 << a)) - 1u) << s);
      return s;
    }
  }
  return -1;
}

// Stable in-place compaction of list[0..n) keeping the entries with keep(id); returns the new
// length.  All threads of the workgroup take part.
template <class Keep>
__device__ inline int compact_stable(int32_t* list, int n, Keep keep, int* s_wave_cnt) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int out = 0;
  for (int base = 0; base < n; base += kThreads) {
    const int x = base + tid;
    int id = 0, k = 0;
    if (x < n) { id = list[x]; k = keep(id) ? 1 : 0; }
    const uint64_t bal = __ballot(k);
    if (lane == 0) s_wave_cnt[wave] = __popcll(bal);
    __syncthreads();                       // also: every read of this chunk precedes its writes
    int before = 0, total = 0;
    for (int w = 0; w < kWaves; ++w) { const int c = s_wave_cnt[w]; if (w < wave) before += c; total += c; }
    if (k) list[out + before + __popcll(bal & ((1ull << lane) - 1ull))] = id;
    out += total;
    __syncthreads();
  }
  return out;
}

struct ReplayLds {
  int pool_nodes[3];   // node-table capacity of each kind's placement block
  int pool_off[3];     // byte offsets of those blocks
  int node_off;        // first per-node block
  int node_waves;      // wavefronts that own a per-node block (DPArrange + eviction): 4, 2 or 1
  int busy_slots;
};

// Node counts and capacities of every scenario (host arrays of the description).
int trace_maxima(const tg_trace_desc* d, TraceMaxima* mx) {
  *mx = TraceMaxima{{0, 0, 0}, 0, 8, 0, 60};   // an 8-GPU node never has more than 4,2,1,1 free chunks of size 1,2,4,8
  const bool pooled = (d->flags & TG_TRACE_GPU_POOLED) != 0;
  for (int s = 0; s < d->S; ++s) {
    int cnt[3] = {0, 0, 0};
    for (int j = 0; j < d->M; ++j) {
      const size_t g = (size_t)s * d->M + j;
      const int ty = d->node_type[g], cap = d->node_cap[g];
      if (ty >= TG_N_TYPES || cap < 0) return TG_E_INVALID_ARG;
      if (ty == TG_TYPE_GPU && cap != 8) return TG_E_INVALID_ARG;
      if (ty == TG_TYPE_CPU && cap > TG_MAX_CPU_UNITS) return TG_E_RANGE;
      ++cnt[ty];
      if (ty != TG_TYPE_API) mx->max_heap = std::max(mx->max_heap, cap);
      if (ty == TG_TYPE_CPU) mx->max_cap_cpu = std::max(mx->max_cap_cpu, cap);
    }
    for (int k = 0; k < 3; ++k) {
      mx->nodes_kind[k] = std::max(mx->nodes_kind[k], cnt[k]);
      if (cnt[k] > TG_MAX_NODES_OF_KIND) return TG_E_RANGE;
    }
    if (pooled && cnt[TG_TYPE_GPU] > kPoolNodesMax) return TG_E_RANGE;
  }
  if (pooled && mx->nodes_kind[TG_TYPE_GPU] > 0) {                // the pool is one resource of all the scenario's GPUs
    const int n = mx->nodes_kind[TG_TYPE_GPU];
    mx->max_free_gpu = 8 * n;
    mx->max_heap = std::max(mx->max_heap, 8 * n);
    mx->max_chunk_states = std::max(mx->max_chunk_states, kPoolStates[n]);
  }
  return TG_OK;
}

// LDS of a workgroup: one placement block per kind (one for all kinds when a single wavefront places them one
// after the other) and, in the same bytes, one per-node block for each wavefront that runs DPArrange - the
// placement tables are exported to the workspace before the node stage begins.  8 / kWaves workgroups fit a CU
// when the total stays under that share of its LDS; beyond it fewer wavefronts get a per-node block.
int replay_layout(const TraceMaxima& mx, int K, ReplayLds* LD, TgNodeLdsPlan* plan, size_t* lds_bytes) {
  *plan = tg_node_lds_plan(mx.max_cap_cpu, mx.max_free_gpu, mx.max_chunk_states, mx.max_heap, K, 1 << 30, 8, TG_WAVE);
  LD->busy_slots = (mx.max_heap + 1 + 1) & ~1;
  size_t pools = 0;
  for (int k = 0; k < 3; ++k) {
    LD->pool_nodes[k] = std::max(mx.nodes_kind[k], 1);
    const size_t bytes = (tg_pool_lds_bytes(LD->pool_nodes[k]) + 15) & ~size_t(15);
    LD->pool_off[k] = kWaves == 1 ? 0 : (int)pools;               // one wavefront places the kinds one after the other
    pools = kWaves == 1 ? std::max(pools, bytes) : pools + bytes;
  }
  LD->node_off = 0;                                               // the placement blocks are dead when the node stage begins
  const size_t node_bytes = (size_t)plan->total + (size_t)LD->busy_slots * 8;
  const size_t share = 160 * 1024 / (8 / kWaves) - 512;           // of a CU's LDS, next to the kernel's static ~0.3 KB
  LD->node_waves = kWaves;
  while (LD->node_waves > 1 && LD->node_waves * node_bytes > share) LD->node_waves >>= 1;
  *lds_bytes = std::max<size_t>({pools, LD->node_waves * node_bytes, 1024});   // 1 KB: the histogram of the statistics
  return *lds_bytes > 160 * 1024 - 2048 ? TG_E_RANGE : TG_OK;
}

// WHOLE_QUEUE: every step admits one prefix of the whole waiting queue (two admission passes per tick).
// COST: every step visits the queue by least estimated ACT; the waiting lists are kept sorted by (key, id).
template <bool WHOLE_QUEUE, bool COST>
__global__ __launch_bounds__(kThreads) void tg_replay_kernel(TgTraceDev T, ReplayWs W, tg_replay_out O, ReplayLds LD,
                                                             TgNodeLdsPlan plan, int restart, int n_ticks) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_wcnt[3], s_next, s_started, s_nrun, s_wave_cnt[kWaves], s_sel[2], s_newcnt[3], s_pos[TG_WAVE];
  __shared__ unsigned long long s_stop;
  __shared__ long long s_sum;
  const int s = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int A = T.A, M = T.M, K = T.K;
  const size_t abase = (size_t)s * A, nbase = (size_t)s * M;

  unsigned char* node_mem = smem + LD.node_off + (size_t)(wave < LD.node_waves ? wave : 0) * (size_t)(plan.total + LD.busy_slots * 8);
  int64_t* s_busy = reinterpret_cast<int64_t*>(node_mem + plan.total);

  const int64_t* arrival = T.arrival + abase;
  const uint8_t* act_type = T.act_type + abase;
  const int64_t* dur = W.dur + abase * K;
  int32_t* wl[3] = {W.wlist + abase * 3, W.wlist + abase * 3 + A, W.wlist + abase * 3 + 2 * (size_t)A};
  int32_t* wl_other[3] = {nullptr, nullptr, nullptr};            // COST: where the next merge of a kind's list writes
  uint64_t* okey = COST ? W.okey + abase : nullptr;
  if constexpr (COST)
    for (int ty = 0; ty < 3; ++ty) wl_other[ty] = W.wlist2 + abase * 3 + (size_t)ty * A;
  int64_t* run_fin = W.run_fin + abase;
  int32_t* run_info = W.run_info + abase;
  int32_t* live_free = W.live_free + nbase;
  int64_t* live_tok = W.live_tok + nbase;
  int32_t *nl_off = W.nl_off + nbase, *nl_cnt = W.nl_cnt + nbase, *dl_off = W.dl_off + nbase, *dl_cnt = W.dl_cnt + nbase;
  int32_t* order = W.order + abase;
  int32_t* dorder = W.dorder + abase;
  int32_t* slot = W.slot + abase;
  uint8_t* reason = W.reason + abase;
  int32_t* o_node = O.node + abase;
  int32_t* o_units = O.units + abase;
  int64_t* o_start = O.start_us + abase;
  int64_t* o_fin = O.finish_us + abase;

  // restart: every scenario at time 0.  Otherwise the call goes on where the last one on this workspace and these
  // outputs stopped: everything but a few counters lives in them.
  int32_t* resume = W.resume + (size_t)s * 16;
  const int resume_mark = 0x54470000 ^ (A * 31 + M);              // left behind by every call; a workspace without it has nothing to go on from
  if (!restart && resume[9] != resume_mark) {
    if (tid == 0) O.n_ticks[s] = -1;
    return;
  }
  int tick = 0, last_tick = 0;
  if (restart) {
  for (int i = tid; i < A; i += kThreads) { o_node[i] = -1; o_units[i] = 0; o_start[i] = -1; o_fin[i] = -1; }
  if (T.numa_cores) {
    for (size_t i = tid; i < (size_t)A * 4; i += kThreads) O.core_set[abase * 4 + i] = 0;
    for (int x = tid; x < M * 4; x += kThreads) {                 // every core of a CPU node is free at time 0
      const int j = x >> 2, w = x & 3, cap = T.node_cap[nbase + j];
      const int bits = T.node_type[nbase + j] == TG_TYPE_CPU ? min(max(cap - 64 * w, 0), 64) : 0;
      W.live_cores[(nbase + j) * 4 + w] = bits == 64 ? ~0ull : (1ull << bits) - 1ull;
    }
  }
  for (int j = tid; j < M; j += kThreads) {
    const int ty = T.node_type[nbase + j], cap = T.node_cap[nbase + j];
    live_free[j] = ty == TG_TYPE_GPU ? (int)((1u << cap) - 1u) : cap;
    live_tok[j] = ty == TG_TYPE_API ? T.quota_tok0[nbase + j] : 0;
    nl_cnt[j] = 0; dl_cnt[j] = 0;
    if (T.act_service) { W.live_res[nbase + j] = 0; W.use_seq[nbase + j] = 0; }   // nothing resident at time 0
    if (T.cache_per_gpu) for (int g = 0; g < 8; ++g) W.gpu_res[(nbase + j) * 8 + g] = 0;
    if (T.node_aux) W.live_aux[nbase + j] = T.node_aux[nbase + j];
  }
  if (tid == 0) { s_wcnt[0] = s_wcnt[1] = s_wcnt[2] = 0; s_next = 0; s_started = 0; s_nrun = 0; }
  } else {
    if (tid == 0) { s_wcnt[0] = resume[0]; s_wcnt[1] = resume[1]; s_wcnt[2] = resume[2]; s_next = resume[3]; s_started = resume[4]; s_nrun = resume[5]; }
    tick = resume[6]; last_tick = resume[7];
    if constexpr (COST) {                                         // which buffer holds the waiting list of a kind
      const int parity = resume[8];
      for (int ty = 0; ty < 3; ++ty)
        if (parity >> ty & 1) { int32_t* o = wl[ty]; wl[ty] = wl_other[ty]; wl_other[ty] = o; }
    }
  }
  __syncthreads();

  const int tick_end = (int)min((int64_t)T.max_ticks, (int64_t)tick + n_ticks);   // this call's share of simulated time
  while (tick < tick_end) {
    if (s_started >= A) break;
    // nothing waiting: jump to the tick of the next arrival (releases and refills commute with idle ticks)
    if (s_wcnt[0] + s_wcnt[1] + s_wcnt[2] == 0) {
      const int64_t na = arrival[s_next];                       // s_next < A because not everything has started
      const int64_t tk = (na + T.tick_us - 1) / T.tick_us;
      if (tk >= tick_end) { tick = tick_end; break; }
      if ((int)tk > tick) tick = (int)tk;
    }
    const int64_t now = (int64_t)tick * T.tick_us;
    const int dticks = tick - last_tick;
    last_tick = tick;
    __syncthreads();                       // everyone has read the shared counters of the previous tick

    // (1) finished actions give their units back; the running set is compacted (order is free)
    {
      const int n = s_nrun;
      int out = 0;
      for (int base = 0; base < n; base += kThreads) {
        const int x = base + tid;
        int keep = 0, info = 0, held = 0, rid = 0;
        int64_t fin = 0;
        if (x < n) {
          fin = run_fin[x]; info = run_info[x];
          if (T.node_aux) held = W.run_aux[abase + x];
          if (T.numa_cores) rid = W.run_id[abase + x];
          keep = fin > now;
          if (!keep) {
            const int node = info & 0xffff, k = (info >> 16) & 0xff, g0 = (info >> 24) & 0xff;
            if (held) atomicAdd(&W.live_aux[nbase + node], held);   // the second resource comes back with the units
            if (T.numa_cores && T.node_type[nbase + node] == TG_TYPE_CPU) {   // and so do the cores
              for (int w = 0; w < 4; ++w) {
                const int id = rid;
                const unsigned long long cs = O.core_set[(abase + id) * 4 + w];
                if (cs) atomicOr((unsigned long long*)&W.live_cores[(nbase + node) * 4 + w], cs);
              }
            }
            if (T.node_type[nbase + node] == TG_TYPE_GPU) atomicOr(&live_free[node], (int)(((1u << (1 << tg_chunk_level(k))) - 1u) << g0));
            else atomicAdd(&live_free[node], k);
          }
        }
        const uint64_t bal = __ballot(keep);
        if (lane == 0) s_wave_cnt[wave] = __popcll(bal);
        __syncthreads();
        int before = 0, total = 0;
        for (int w = 0; w < kWaves; ++w) { const int c = s_wave_cnt[w]; if (w < wave) before += c; total += c; }
        if (keep) {
          const int d = out + before + __popcll(bal & ((1ull << lane) - 1ull));
          run_fin[d] = fin; run_info[d] = info;
          if (T.node_aux) W.run_aux[abase + d] = held;
          if (T.numa_cores) W.run_id[abase + d] = rid;
        }
        out += total;
        __syncthreads();
      }
      if (tid == 0) s_nrun = out;
    }
    // (2) quota refill for the ticks since the last step (saturating, so idle ticks compose)
    if (dticks > 0) {
      const int q0 = T.tnode_off[s * 4 + TG_TYPE_API], nq = T.tnode_off[s * 4 + TG_TYPE_API + 1] - q0;
      for (int r = tid; r < nq; r += kThreads) {
        const int j = T.tnode_idx[nbase + q0 + r];
        const int64_t capu = (int64_t)T.node_cap[nbase + j] * 1000000, inc = (int64_t)T.quota_rate[nbase + j] * T.tick_us;
        int64_t tok = live_tok[j];
        if (inc > 0) {
          const int64_t need = capu - tok;
          tok = (need <= 0 || (int64_t)dticks >= (need + inc - 1) / inc) ? (tok > capu ? tok : capu) : tok + dticks * inc;
        }
        live_tok[j] = tok;
      }
    }
    // (3) arrivals join their kind's waiting list in arrival order
    if (wave == 0) {                                              // 64 trace entries per pass; arrivals ascend
      int nx = s_next;
      int wc[3] = {s_wcnt[0], s_wcnt[1], s_wcnt[2]};
      for (;;) {
        const int x = nx + lane;
        const bool due = x < A && arrival[x] <= now;
        const int ty = due ? act_type[x] : -1;
        const uint64_t bal = __ballot(due);
#pragma unroll
        for (int t = 0; t < 3; ++t) {
          const uint64_t tb = __ballot(ty == t);
          if (ty == t) wl[t][wc[t] + __popcll(tb & ((1ull << lane) - 1ull))] = x;
          wc[t] += __popcll(tb);
        }
        nx += __popcll(bal);
        if (bal != ~0ull) break;
      }
      if (lane == 0) {
        if constexpr (COST) { s_newcnt[0] = wc[0] - s_wcnt[0]; s_newcnt[1] = wc[1] - s_wcnt[1]; s_newcnt[2] = wc[2] - s_wcnt[2]; }
        s_next = nx; s_wcnt[0] = wc[0]; s_wcnt[1] = wc[1]; s_wcnt[2] = wc[2];
      }
    }
    if constexpr (COST) {
      // The arrivals of this tick sit behind the sorted part of their kind's list.  They are merged into it 64 at a
      // time: wavefront 0 ranks the 64 among themselves and finds by bisection how many old entries precede each
      // (keys are distinct: the id is part of them); every old entry then moves up by the number of new ones that
      // precede it, into the list's other buffer.
      __threadfence_block();
      __syncthreads();
      for (int ty = 0; ty < 3; ++ty) {
        if (ty == TG_TYPE_GPU && T.act_service) {
          // With services the keys follow the caches (Sec. 5.3): an action whose service is cached on no node it may
          // run on is dearer by the restore time.  So this tick's keys of all waiting GPU actions are written anew
          // and the list is ordered from scratch, by counting for every entry the keys below its own (keys are
          // distinct: the id is part of them) - 64 keys at a time across the lanes.
          const int n = s_wcnt[ty];
          if (n == 0) continue;
          const int g0 = T.tnode_off[s * 4 + TG_TYPE_GPU], n_gpu = T.tnode_off[s * 4 + TG_TYPE_GPU + 1] - g0;
          uint64_t any = 0;                                         // cached on some GPU node
          for (int r = lane; r < n_gpu; r += TG_WAVE) any |= W.live_res[nbase + T.tnode_idx[nbase + g0 + r]];
          any = (uint64_t)tg_wave_or_u32((uint32_t)any) | (uint64_t)tg_wave_or_u32((uint32_t)(any >> 32)) << 32;
          const int32_t* src = wl[ty];
          int32_t* dst = wl_other[ty];
          uint64_t* skey = W.skey + abase;
          for (int x = tid; x < n; x += kThreads) {
            const int id = src[x];
            uint64_t key = W.okey0[abase + id] >> 17;
            const int sv = T.act_service[abase + id];
            if (sv >= 0 && key != kKeyInf) {
              const int pin = T.act_pin[abase + id];
              const uint64_t res = pin >= 0 ? W.live_res[nbase + pin] : any;
              if (!(res >> sv & 1ull)) key += (uint64_t)T.restore[sv];
            }
            const uint64_t packed = key << 17 | (uint32_t)id;
            okey[id] = packed; skey[x] = packed;
          }
          __threadfence_block();
          __syncthreads();
          for (int xb = 0; xb < n; xb += kThreads) {
            const int x = xb + tid;
            const uint64_t mine = x < n ? skey[x] : ~0ull;
            int rank = 0;
            for (int base = 0; base < n; base += TG_WAVE) {
              const uint64_t kb = base + lane < n ? skey[base + lane] : ~0ull;
              const int c = min(TG_WAVE, n - base);
              for (int m = 0; m < c; ++m) rank += (uint64_t)tg_readlane_i64((int64_t)kb, m) < mine ? 1 : 0;
            }
            if (x < n) dst[rank] = (int)(mine & 0x1ffffu);
          }
          __threadfence_block();
          __syncthreads();
          wl_other[ty] = wl[ty]; wl[ty] = dst;
          continue;
        }
        int n_new = s_newcnt[ty], n_old = s_wcnt[ty] - n_new;
        while (n_new > 0) {
          const int32_t* src = wl[ty];
          int32_t* dst = wl_other[ty];
          const int c = min(TG_WAVE, n_new);
          if (wave == 0) {
            const int id = lane < c ? src[n_old + lane] : 0;
            const uint64_t key = lane < c ? okey[id] : ~0ull;
            int rank = 0;
            for (int m = 0; m < c; ++m) rank += (uint64_t)tg_readlane_i64((int64_t)key, m) < key ? 1 : 0;
            int lo = 0, hi = n_old;                                // old entries that precede this one
            while (__any(lo < hi)) {
              const int mid = (lo + hi) >> 1;
              const bool go = lo < hi;
              const uint64_t k = go ? okey[src[mid]] : 0;
              if (go) { if (k < key) lo = mid + 1; else hi = mid; }
            }
            if (lane < c) { s_pos[rank] = lo; dst[lo + rank] = id; }
          }
          __syncthreads();
          for (int x = tid; x < n_old; x += kThreads) {           // s_pos ascends: new entries with s_pos <= x precede old entry x
            int lo = 0, hi = c;
            while (lo < hi) { const int mid = (lo + hi) >> 1; if (s_pos[mid] <= x) lo = mid + 1; else hi = mid; }
            dst[x + lo] = src[x];
          }
          for (int x = n_old + c + tid; x < n_old + n_new; x += kThreads) dst[x] = src[x];   // arrivals still to be merged
          __threadfence_block();
          __syncthreads();
          wl_other[ty] = wl[ty]; wl[ty] = dst;
          n_old += c; n_new -= c;
        }
      }
    }
    __threadfence_block();
    __syncthreads();
    const int wc0 = s_wcnt[0], wc1 = s_wcnt[1], wc2 = s_wcnt[2];
    const int wcs[3] = {wc0, wc1, wc2};
    const int woff[3] = {0, wc0, wc0 + wc1};

    // (4a) admission + node choice, one wavefront per resource kind.  With the whole-queue prefix a first pass
    // (one prefix per kind) shows where the admission ends - at the first waiting action, in arrival order, that it
    // defers - and a second pass admits only the actions before that one.
    constexpr int n_pass = WHOLE_QUEUE ? 2 : 1;
    for (int pass = 0; pass < n_pass; ++pass) {
    for (int ty = wave; ty < 3; ty += kWaves) {
      if (wcs[ty] == 0) continue;                                 // nobody waits for this kind: its list lengths are still zero
      const int n0 = T.tnode_off[s * 4 + ty], Mt_all = T.tnode_off[s * 4 + ty + 1] - n0;
      const int32_t* nodes = T.tnode_idx + nbase + n0;
      // pooled GPUs: the first GPU node stands for the pool, with the free chunks of all of them (at most 5 nodes)
      const bool pooled = T.gpu_pooled && ty == TG_TYPE_GPU;
      const int Mt = pooled ? min(Mt_all, 1) : Mt_all;
      int32_t pool_chunks = 0;
      if (pooled) pool_chunks = tg_wave_sum_i32(lane < Mt_all ? (int32_t)mask_chunks((uint32_t)live_free[nodes[lane]]) : 0);
      TgPoolLds S;
      tg_pool_lds_carve(smem + LD.pool_off[ty], LD.pool_nodes[ty], &S);
      if (lane < TG_MAX_K) S.k[lane] = T.k_list[lane];
      for (int r = lane; r < Mt; r += TG_WAVE) {
        const int j = nodes[r];
        S.back[r] = 0;
        S.lim[r] = pooled ? pool_chunks
                 : ty == TG_TYPE_GPU ? (int32_t)mask_chunks((uint32_t)live_free[j])
                 : ty == TG_TYPE_API ? (int32_t)(live_tok[j] / 1000000) : live_free[j];
        S.cnt[r] = 0; S.dcnt[r] = 0; S.closed[r] = 0;
        if (T.act_service) S.res[r] = W.live_res[nbase + j];
        if (T.node_aux) S.aux[r] = W.live_aux[nbase + j];
      }
      tg_wave_sync();
      TgPlaceIo io;
      io.act_kmask = T.act_kmask + abase; io.act_static = T.act_static + abase; io.act_pin = T.act_pin + abase;
      io.act_aux = T.act_aux ? T.act_aux + abase : nullptr;
      io.act_quota = T.act_quota && ty == TG_TYPE_API ? T.act_quota + abase : nullptr;
      io.act_service = T.act_service ? T.act_service + abase : nullptr; io.restore = T.restore;
      io.act_pin_rank = nullptr;
      io.node_rank = T.node_rank + nbase; io.nodes = nodes; io.dur = dur; io.cost = nullptr; io.cost_row_len = 0;
      io.K = K; io.Kt = T.type_k[ty];
      io.out_node = o_node; io.out_units = o_units; io.out_act = nullptr; io.out_reason = reason; io.slot = slot;
      const int n_adm = pass == 0 ? wcs[ty] : tg_prefix_len(wl[ty], wcs[ty], okey, (uint64_t)s_stop);   // the lists ascend in place (FCFS: the id)
      tg_place_pool<4, 1>(S, io, wl[ty], n_adm, Mt, ty == TG_TYPE_GPU, lane);
      if constexpr (WHOLE_QUEUE) { if (pass == 1) tg_place_tail(S, io, wl[ty], n_adm, wcs[ty], lane); }
      tg_pool_extents(S, nodes, Mt, woff[ty], nl_off, nl_cnt, dl_off, dl_cnt, lane);
    }
    __threadfence_block();
    __syncthreads();
    if (pass + 1 < n_pass) {
      if (tid == 0) s_stop = ~0ull;
      __syncthreads();
      unsigned long long first = ~0ull;                           // place, in the order of the whole queue, of the first action that waits
      for (int ty = 0; ty < 3; ++ty)
        for (int x = tid; x < wcs[ty]; x += kThreads) {
          const int id = wl[ty][x];
          const unsigned long long place = COST ? okey[id] : (unsigned long long)id;
          if (reason[id] == TG_DEFER_PREFIX && place < first) first = place;
        }
      if (first != ~0ull) atomicMin(&s_stop, first);
      __syncthreads();
      if (s_stop == ~0ull) break;                                 // nobody waits: both rules agree
    }
    }
    // (4b) group candidates and waiting pinned actions by node (the three lists as one range: their loads travel together)
    const int wtot = wc0 + wc1 + wc2;
    for (int x = tid; x < wtot; x += kThreads) {
      const int ty = x < woff[1] ? 0 : x < woff[2] ? 1 : 2;
      const int32_t* list = ty == 0 ? wl[0] : ty == 1 ? wl[1] : wl[2];
      const int id = list[x - (ty == 0 ? 0 : ty == 1 ? woff[1] : woff[2])];
      const int r = reason[id];
      if (r == TG_SELECTED) order[nl_off[o_node[id]] + slot[id]] = id;
      else if (r == TG_DEFER_PREFIX && T.act_pin[abase + id] >= 0) dorder[dl_off[T.act_pin[abase + id]] + slot[id]] = id;
    }
    __threadfence_block();
    __syncthreads();
    // (4c) per node: DPArrange + greedy eviction; the running actions of the node seed the heap
    int n_seen = 0;                                               // nodes with candidates met so far
    for (int jb = 0; jb < M; jb += TG_WAVE) {
     // every wavefront looks at the same 64 list lengths and takes every kWaves-th node that has candidates
     const int jn = jb + lane;
     const int my_m = jn < M ? nl_cnt[jn] : 0;
     // A node with one candidate and nobody waiting for it needs no table and no heap (as tg_node_single): its
     // action takes the fastest allowed option that fits.  All such nodes of the 64 at once, lane = node - their
     // loads travel together instead of node after node.
     bool lone = false;
     if (my_m == 1) {
       const int ty = T.node_type[nbase + jn];
       lone = dl_cnt[jn] == 0 && !(T.gpu_pooled && ty == TG_TYPE_GPU);
       if (lone && wave == 0) {
         const int id = order[nl_off[jn]];
         const uint32_t mask = T.act_kmask[abase + id];
         const bool elastic = T.act_model[abase + id] != TG_MODEL_NONE;
         const int cap = T.node_cap[nbase + jn];
         const uint32_t lf = (uint32_t)live_free[jn];
         const int free_units = ty == TG_TYPE_API ? (int)(live_tok[jn] / 1000000) : (int)lf;
         const uint32_t chunks = ty == TG_TYPE_GPU ? mask_chunks(lf) : 0;
         int64_t delay = 0;
         if (T.act_service) {
           const int sv = T.act_service[abase + id];
           if (sv >= 0 && !(W.live_res[nbase + jn] >> sv & 1ull)) delay = T.restore[sv];
         }
         const int q_min = __builtin_ctz(mask);
         uint64_t best = ~0ull;
         int k_best = T.k_list[0];
         for (int q = 0; q < K; ++q) {
           if (!(mask >> q & 1u) || !(elastic || q == q_min)) continue;
           const int64_t d = dur[(size_t)id * K + q];
           const int kq = T.k_list[q];
           uint64_t key = ~0ull;
           if (!elastic) key = (uint64_t)(d + delay) << 12;        // runs on its minimum units (Alg. 1)
           else if (d != TG_INF && kq <= cap) {
             if (ty == TG_TYPE_GPU) {
               if (kq <= tg_chunk_largest(chunks)) {               // ties: the option that leaves the smaller chunk state
                 const int r0 = max((int)(chunks & 0xff), 1) + 1, r1 = max((int)(chunks >> 8 & 0xff), 1) + 1,
                           r2 = max((int)(chunks >> 16 & 0xff), 1) + 1;
                 const uint32_t c = tg_chunk_take(chunks, kq);
                 const int code = (int)(c & 0xff) + r0 * ((int)(c >> 8 & 0xff) + r1 * ((int)(c >> 16 & 0xff) + r2 * (int)(c >> 24)));
                 key = (uint64_t)(d + delay) << 12 | (uint32_t)code;
               }
             } else if (kq <= free_units) key = (uint64_t)(d + delay) << 12 | (uint32_t)kq;   // ties: fewer units
           }
           if (key < best) { best = key; k_best = kq; }
         }
         o_units[id] = k_best;
       }
     }
     uint64_t todo = __ballot(my_m > 0 && !lone);
     while (todo) {
      const int jl = __ffsll((unsigned long long)todo) - 1;
      todo &= todo - 1;
      if ((n_seen++ & (LD.node_waves - 1)) != wave) continue;     // wavefronts without a block take none
      const int j = jb + jl;
      const int m = __builtin_amdgcn_readlane(my_m, jl);
      const int ty = T.node_type[nbase + j];
      const bool pooled = T.gpu_pooled && ty == TG_TYPE_GPU;      // j is the first GPU node: it stands for all of them
      const bool single = m == 1 && dl_cnt[j] == 0;               // one candidate, nobody waiting: no table, no heap
      int nb = 0;
      if (ty != TG_TYPE_API && !single) {
        const int n = s_nrun;
        for (int base = 0; base < n; base += TG_WAVE) {
          const int x = base + lane;
          int k = 0;
          int64_t fin = 0;
          if (x < n) {
            const int info = run_info[x], on = info & 0xffff;
            if (pooled ? T.node_type[nbase + on] == TG_TYPE_GPU : on == j) { k = (info >> 16) & 0xff; fin = run_fin[x] - now; }
          }
          const int inc = tg_wave_scan_i32(k);
          for (int c = 0; c < k; ++c) s_busy[nb + inc - k + c] = fin;
          nb += __builtin_amdgcn_readlane(inc, TG_WAVE - 1);
        }
      }
      TgNodeIn in;
      in.type = ty; in.cap = T.node_cap[nbase + j];
      const uint32_t lf = (uint32_t)live_free[j];
      in.free_units = ty == TG_TYPE_GPU ? __popc(lf) : ty == TG_TYPE_API ? (int)(live_tok[j] / 1000000) : (int)lf;
      in.chunks = ty == TG_TYPE_GPU ? mask_chunks(lf) : 0;
      if (pooled) {                                               // units, free GPUs and free chunks of the whole pool
        const int g0 = T.tnode_off[s * 4 + TG_TYPE_GPU], n_gpu = T.tnode_off[s * 4 + TG_TYPE_GPU + 1] - g0;
        const uint32_t mf = lane < n_gpu ? (uint32_t)live_free[T.tnode_idx[nbase + g0 + lane]] : 0u;
        in.cap = 8 * n_gpu;
        in.free_units = tg_wave_sum_i32(__popc(mf));
        in.chunks = (uint32_t)tg_wave_sum_i32(lane < n_gpu ? (int32_t)mask_chunks(mf) : 0);
      }
      in.backlog = 0;
      in.m = m; in.clist = order + nl_off[j]; in.nd = dl_cnt[j]; in.dlist = dorder + dl_off[j];
      in.n_busy = nb; in.busy = nullptr; in.busy_lds_off = plan.total;
      in.act_model = T.act_model + abase; in.act_kmask = T.act_kmask + abase; in.dur = dur; in.K = K; in.depth = T.depth;
      in.kword = tg_pack_k(T.k_list);
      in.act_service = T.act_service ? T.act_service + abase : nullptr; in.restore = T.restore;
      in.resident = T.act_service ? W.live_res[nbase + j] : 0;
      TgNodeOut out;
      out.node = o_node; out.units = o_units; out.act = nullptr; out.reason = reason; out.age = nullptr;
      int used_units;
      if (single) tg_node_single(in, out, lane, &used_units);
      else tg_node_schedule(node_mem, plan, in, out, lane, &used_units);
     }
    }
    __threadfence_block();
    __syncthreads();
    // (5) selected actions start now.  CPU / API: any order; GPU nodes: FCFS order on the mask
    for (int x = tid; x < wtot; x += kThreads) {
      {
        const int ty = x < woff[1] ? 0 : x < woff[2] ? 1 : 2;
        const int32_t* list = ty == 0 ? wl[0] : ty == 1 ? wl[1] : wl[2];
        const int id = list[x - (ty == 0 ? 0 : ty == 1 ? woff[1] : woff[2])];
        const int j = o_node[id];
        if (j < 0) continue;
        const int k = o_units[id];
        int q = 0;
        while (q < K - 1 && T.k_list[q] != k) ++q;
        // realised = modelled duration: the restore delay is the one the step saw (residency at the tick's start)
        int64_t delay = 0;
        if (T.act_service && ty == TG_TYPE_GPU) {
          const int sv = T.act_service[abase + id];
          if (sv >= 0 && !(W.live_res[nbase + j] >> sv & 1ull)) delay = T.restore[sv];
        }
        const int64_t fin = now + delay + dur[(size_t)id * K + q];
        o_start[id] = now; o_fin[id] = fin;
        atomicAdd(&s_started, 1);
        if (ty == TG_TYPE_API) {
          atomicAdd((unsigned long long*)&live_tok[j], (unsigned long long)(-(int64_t)k * 1000000));
          if (T.act_quota) {                                      // one token of every further quota the action names
            const int32_t* api = T.tnode_idx + nbase + T.tnode_off[s * 4 + TG_TYPE_API];
            for (uint64_t more = T.act_quota[abase + id]; more; more &= more - 1)
              atomicAdd((unsigned long long*)&live_tok[api[__builtin_ctzll(more)]], (unsigned long long)(-1000000ll));
          }
        }
        else if (ty == TG_TYPE_CPU) {
          atomicSub(&live_free[j], k);
          const int d = atomicAdd(&s_nrun, 1);
          run_fin[d] = fin; run_info[d] = j | k << 16;
          if (T.numa_cores) W.run_id[abase + d] = id;
          if (T.node_aux) {                                       // held from start to finish by an action that chose its node
            const int held = T.act_pin[abase + id] < 0 ? T.act_aux[abase + id] : 0;
            W.run_aux[abase + d] = held;
            if (held) atomicSub(&W.live_aux[nbase + j], held);
          }
        }
      }
    }
    if (T.act_service) __syncthreads();                           // the residency of the tick's start has been read
    if (T.gpu_pooled) {
      // The pool's selected actions, in list order, take their real chunks (Sec. 5.3's rule over the cluster): the
      // smallest free chunk that holds the action, on the lowest-numbered node that has one - the same sequence of
      // takes the pool's chunk counts went through in the step, so every take succeeds.  One thread: the order matters.
      const int g0 = T.tnode_off[s * 4 + TG_TYPE_GPU], n_gpu = T.tnode_off[s * 4 + TG_TYPE_GPU + 1] - g0;
      if (tid == 0 && n_gpu > 0) {
        const int32_t* gpu_nodes = T.tnode_idx + nbase + g0;
        const int pool = gpu_nodes[0], m = nl_cnt[pool];
        for (int x = 0; x < m; ++x) {
          const int id = order[nl_off[pool] + x];
          if (o_node[id] < 0) break;                              // evicted tail
          const int k = o_units[id], lvl = tg_chunk_level(k);
          int best = -1, best_level = 4;
          for (int r = 0; r < n_gpu; ++r) {
            const uint32_t c = mask_chunks((uint32_t)live_free[gpu_nodes[r]]);
            for (int b = lvl; b < best_level; ++b)
              if ((c >> (8 * b)) & 0xffu) { best = r; best_level = b; break; }
          }
          if (best < 0) { o_node[id] = -1; continue; }           // cannot happen: the pool's counts had such a chunk
          const int j = gpu_nodes[best];
          uint32_t mk = (uint32_t)live_free[j];
          const int first = mask_alloc(mk, k) & 7;
          live_free[j] = (int)mk;
          int q = 0;
          while (q < K - 1 && T.k_list[q] != k) ++q;
          const int d = atomicAdd(&s_nrun, 1);
          run_fin[d] = now + dur[(size_t)id * K + q]; run_info[d] = j | k << 16 | first << 24;
          if (T.numa_cores) W.run_id[abase + d] = id;
          o_node[id] = j;
        }
      }
    }
    for (int r = tid; r < (T.gpu_pooled ? 0 : T.tnode_off[s * 4 + 2] - T.tnode_off[s * 4 + 1]); r += kThreads) {
      const int j = T.tnode_idx[nbase + T.tnode_off[s * 4 + 1] + r];
      const int m = nl_cnt[j];
      if (m == 0) continue;
      uint32_t mk = (uint32_t)live_free[j];
      int aux_left = T.node_aux ? W.live_aux[nbase + j] : 0;
      const uint64_t res0 = T.act_service ? W.live_res[nbase + j] : 0;
      uint64_t res = res0;
      int32_t* used = W.used_at + (nbase + j) * 64;
      int seq = T.act_service ? W.use_seq[nbase + j] : 0;
      for (int x = 0; x < m; ++x) {
        const int id = order[nl_off[j] + x];
        if (o_node[id] < 0) break;                                // evicted tail
        const int k = o_units[id];
        int q = 0;
        while (q < K - 1 && T.k_list[q] != k) ++q;
        const int sv = T.act_service ? T.act_service[abase + id] : -1;
        int g0;
        int64_t delay = 0;
        if (T.cache_per_gpu && sv >= 0) {
          // A cache on every GPU (Sec. 5.3): the allocation takes from the lowest level that has a free chunk; of
          // that level's chunks the first that holds a block of the action's size whose GPUs all cache the service
          // gives that block.  Masks of 8 GPUs; a block or chunk is marked at its first GPU.
          uint64_t* gr = W.gpu_res + (nbase + j) * 8;
          const int a = tg_chunk_level(k);
          uint32_t f[4], hb = 0;
          for (int g = 0; g < 8; ++g) hb |= (uint32_t)(gr[g] >> sv & 1ull) << g;
          f[0] = mk;
          f[1] = f[0] & (f[0] >> 1) & 0x55u; f[2] = f[1] & (f[1] >> 2) & 0x11u; f[3] = f[2] & (f[2] >> 4) & 0x01u;
          if (a >= 1) hb = hb & (hb >> 1) & 0x55u;
          if (a >= 2) hb = hb & (hb >> 2) & 0x11u;
          if (a >= 3) hb = hb & (hb >> 4) & 0x01u;
          g0 = 0;
          bool hit = false;
          for (int lvl = a; lvl < 4; ++lvl) {
            uint32_t top = f[lvl];                                // free blocks of the level that are no part of a larger free block
            if (lvl < 3) top &= ~(f[lvl + 1] | f[lvl + 1] << (1 << lvl));
            if (!top) continue;
            const uint32_t pick = hb & top * ((1u << (1 << lvl)) - 1u);   // blocks caching it inside these chunks
            hit = pick != 0;
            g0 = __builtin_ctz(hit ? pick : top);
            break;
          }
          mk &= ~(((1u << (1 << a)) - 1u) << g0);
          if (!hit) delay = T.restore[sv];
          ++seq;
          for (int g = g0; g < g0 + (1 << a); ++g) {              // resident and most recently used on every GPU of the block
            uint64_t rg = gr[g];
            int32_t* ug = W.used_at + ((nbase + j) * 8 + g) * 64;
            if (!(rg >> sv & 1ull) && (int)__popcll(rg) >= T.cache_slots) {
              int victim = -1;
              for (uint64_t left = rg; left; left &= left - 1) {
                const int y = __builtin_ctzll(left);
                if (victim < 0 || ug[y] < ug[victim]) victim = y;
              }
              rg &= ~(1ull << victim);
            }
            gr[g] = rg | 1ull << sv;
            ug[sv] = seq;
          }
          o_fin[id] = now + delay + dur[(size_t)id * K + q];     // known only now: the step saw the node's caches together
        }
        else g0 = mask_alloc(mk, k) & 7;
        const int d = atomicAdd(&s_nrun, 1);
        if (sv >= 0 && !T.cache_per_gpu) {
          if (!(res0 >> sv & 1ull)) delay = T.restore[sv];
          // the service is resident from now on and the most recently used one (Sec. 5.3, LRU)
          if (!(res >> sv & 1ull) && (int)__popcll(res) >= T.cache_slots) {
            int victim = -1;
            for (uint64_t left = res; left; left &= left - 1) {   // ascending id: the smaller one wins ties
              const int y = __builtin_ctzll(left);
              if (victim < 0 || used[y] < used[victim]) victim = y;
            }
            res &= ~(1ull << victim);
          }
          res |= 1ull << sv;
          used[sv] = ++seq;
        }
        run_fin[d] = now + delay + dur[(size_t)id * K + q]; run_info[d] = j | k << 16 | g0 << 24;
        if (T.numa_cores) W.run_id[abase + d] = id;
        if (T.node_aux) {
          const int held = T.act_pin[abase + id] < 0 ? T.act_aux[abase + id] : 0;
          W.run_aux[abase + d] = held;
          aux_left -= held;
        }
      }
      live_free[j] = (int)mk;
      if (T.node_aux) W.live_aux[nbase + j] = aux_left;
      if (T.cache_per_gpu) {                                      // what the next step sees of this node: cached on any of its GPUs
        res = 0;
        for (int g = 0; g < 8; ++g) res |= W.gpu_res[(nbase + j) * 8 + g];
      }
      if (T.act_service) { W.live_res[nbase + j] = res; W.use_seq[nbase + j] = seq; }
    }
    // (5b) named cores (Sec. 5.2): the selected actions of a CPU node take theirs one after the other in list order,
    // lane = NUMA domain; every wavefront looks at the same 64 list lengths and takes every kWaves-th node with a list
    if (T.numa_cores) {
      const int nc = T.numa_cores;
      const int word = (lane * nc) >> 6, shift = (lane * nc) & 63;
      int seen = 0;
      for (int jb = 0; jb < M; jb += TG_WAVE) {
        const int jn = jb + lane;
        uint64_t todo = __ballot(jn < M && nl_cnt[jn < M ? jn : 0] > 0 && T.node_type[nbase + (jn < M ? jn : 0)] == TG_TYPE_CPU);
        while (todo) {
          const int j = jb + __builtin_ctzll(todo);
          todo &= todo - 1;
          if ((seen++ & (kWaves - 1)) != wave) continue;
          const int m = nl_cnt[j], n_dom = (T.node_cap[nbase + j] + nc - 1) / nc;
          uint64_t dm = 0, gone = 0;                              // free cores of this lane's domain; what it gives in this tick
          if (lane < n_dom) {
            dm = W.live_cores[(nbase + j) * 4 + word] >> shift;
            if (nc < 64) dm &= (1ull << nc) - 1;
          }
          for (int x = 0; x < m; ++x) {
            const int a = order[nl_off[j] + x];
            if (o_node[a] < 0) break;                             // evicted tail
            bool one_domain;
            const uint64_t take = tg_take_cores(dm, o_units[a], lane, &one_domain);
            gone |= take;
            if (take) atomicOr((unsigned long long*)&O.core_set[(abase + a) * 4 + word], (unsigned long long)(take << shift));
          }
          if (gone) atomicAnd((unsigned long long*)&W.live_cores[(nbase + j) * 4 + word], ~(unsigned long long)(gone << shift));
        }
      }
    }
    __threadfence_block();
    __syncthreads();                                              // the GPU nodes' lists have been read
    for (int j = tid; j < M; j += kThreads) { nl_cnt[j] = 0; dl_cnt[j] = 0; }
    // waiting lists keep the actions that did not start, in order
    for (int ty = 0; ty < 3; ++ty) {
      const int n = compact_stable(wl[ty], wcs[ty], [&](int id) { return o_node[id] < 0; }, s_wave_cnt);
      if (tid == 0) s_wcnt[ty] = n;
    }
    __syncthreads();
    ++tick;
  }

  // ---- per-scenario statistics: mean and nearest-rank p99 of ACT = finish - arrival ----------
  __syncthreads();
  if (tid == 0) {
    resume[0] = s_wcnt[0]; resume[1] = s_wcnt[1]; resume[2] = s_wcnt[2]; resume[3] = s_next; resume[4] = s_started; resume[5] = s_nrun;
    resume[6] = tick; resume[7] = last_tick;
    int parity = 0;
    if constexpr (COST)
      for (int ty = 0; ty < 3; ++ty) parity |= (wl[ty] != W.wlist + abase * 3 + (size_t)ty * A ? 1 : 0) << ty;
    resume[8] = parity; resume[9] = resume_mark;
  }
  if (tid == 0) { s_sum = 0; s_stop = 0; }
  __syncthreads();
  const int n_started = s_started;
  long long sum = 0;
  unsigned long long act_bits = 0;                                // OR of all ACTs: which bytes of them are in use at all
  for (int i = tid; i < A; i += kThreads)
    if (o_start[i] >= 0) { const long long act = o_fin[i] - arrival[i]; sum += act; act_bits |= (unsigned long long)act; }
  atomicAdd((unsigned long long*)&s_sum, (unsigned long long)sum);
  atomicOr(&s_stop, act_bits);                                    // (the admission's stop mark is not needed any more)
  __syncthreads();
  // radix select of the rank-th smallest ACT, one byte per pass from the top
  int* s_hist = reinterpret_cast<int*>(smem);                     // the tables of the ticks are dead
  int64_t p99 = -1;
  if (n_started > 0) {
    int rank = (int)((99ll * n_started + 99) / 100);             // 1-based
    uint64_t prefix = 0;
    const int top = s_stop ? (63 - __builtin_clzll(s_stop)) & ~7 : 0;   // bytes above it are zero in every ACT: their passes would pick bin 0
    for (int shift = top; shift >= 0; shift -= 8) {
      for (int b = tid; b < 256; b += kThreads) s_hist[b] = 0;
      __syncthreads();
      for (int i = tid; i < A; i += kThreads)
        if (o_start[i] >= 0) {
          const uint64_t key = (uint64_t)(o_fin[i] - arrival[i]);
          if (shift == top || (key >> (shift + 8)) == prefix) atomicAdd(&s_hist[(key >> shift) & 255], 1);
        }
      __syncthreads();
      if (tid == 0) {
        int cum = 0, bin = 0;
        for (; bin < 256; ++bin) { if (cum + s_hist[bin] >= rank) break; cum += s_hist[bin]; }
        s_sel[0] = bin; s_sel[1] = rank - cum;
      }
      __syncthreads();
      prefix = prefix << 8 | (uint64_t)s_sel[0];
      rank = s_sel[1];
      __syncthreads();
    }
    p99 = (int64_t)prefix;
  }
  if (tid == 0) {
    O.n_started[s] = n_started;
    O.n_ticks[s] = tick;
    O.mean_act_us[s] = n_started ? (double)s_sum / (double)n_started : 0.0;
    O.p99_act_us[s] = p99;
  }
}

}  // namespace

extern "C" int tg_build_trace(const tg_trace_desc* d, void* hip_stream, tg_trace** out) {
  if (!d || !out) return TG_E_INVALID_ARG;
  *out = nullptr;
  const int S = d->S, A = d->A, M = d->M, K = d->K;
  if (S < 1 || A < 1 || M < 1 || (d->flags & ~(uint32_t)(TG_TRACE_QUEUE_PREFIX | TG_TRACE_GPU_POOLED | TG_TRACE_CACHE_PER_GPU)) != 0 || d->max_ticks < 1 || d->tick_us < 1) return TG_E_INVALID_ARG;
  if (d->depth < 1 || d->depth > TG_MAX_DEPTH) return TG_E_INVALID_ARG;
  const bool svc = d->act_service != nullptr;
  if (svc != (d->restore_us != nullptr)) return TG_E_INVALID_ARG;
  if ((d->node_aux != nullptr) != (d->act_aux != nullptr)) return TG_E_INVALID_ARG;
  if (d->numa_cores != 0 && d->numa_cores != 4 && d->numa_cores != 8 && d->numa_cores != 16 && d->numa_cores != 32 &&
      d->numa_cores != 64) return TG_E_INVALID_ARG;
  if (d->order_policy != TG_ORDER_FCFS && d->order_policy != TG_ORDER_COST) return TG_E_INVALID_ARG;
  const bool pooled = (d->flags & TG_TRACE_GPU_POOLED) != 0;
  if (pooled && (d->act_service || d->node_aux)) return TG_E_INVALID_ARG;            // a pool has no per-node cache or second resource
  if (svc) {
    if (d->n_services < 1 || d->n_services > TG_MAX_SERVICES || d->cache_slots < 1 || d->cache_slots > TG_MAX_SERVICES) return TG_E_INVALID_ARG;
    for (int x = 0; x < d->n_services; ++x) if (d->restore_us[x] < 0 || d->restore_us[x] >= TG_T_ORI_LIMIT) return TG_E_RANGE;
  }
  if (A > TG_MAX_ACTIONS || M > 65535 || (int64_t)S * A >= (1ll << 31) || (int64_t)S * M >= (1ll << 31)) return TG_E_RANGE;
  if (d->tick_us >= TG_TIME_LIMIT || (int64_t)d->max_ticks * d->tick_us >= (1ll << 44)) return TG_E_RANGE;
  if (K < 1 || K > TG_MAX_K || !d->k_list || !d->type_k) return TG_E_INVALID_ARG;
  for (int q = 0; q < K; ++q) {
    if (d->k_list[q] < 1 || d->k_list[q] > TG_MAX_UNIT || (q && d->k_list[q] <= d->k_list[q - 1])) return TG_E_INVALID_ARG;
  }
  for (int t = 0; t < 3; ++t) if (d->type_k[t] < 0 || d->type_k[t] > K) return TG_E_INVALID_ARG;
  if (d->type_k[TG_TYPE_API] > 1) return TG_E_INVALID_ARG;
  for (int q = 0; q < d->type_k[TG_TYPE_GPU]; ++q) {
    const int k = d->k_list[q];
    if (!(k == 1 || k == 2 || k == 4 || k == 8)) return TG_E_INVALID_ARG;
  }
  if (d->n_classes < 0 || (d->n_classes > 0 && !d->speedup_q16)) return TG_E_INVALID_ARG;
  for (int c = 0; c < d->n_classes; ++c)
    for (int q = 0; q < K; ++q) {
      const uint32_t sp = d->speedup_q16[c * K + q];
      if (sp < 65536u || sp > 65536u * (uint32_t)d->k_list[q] || (q && sp < d->speedup_q16[c * K + q - 1])) return TG_E_ELASTICITY;
    }
  if (!d->node_type || !d->node_cap || !d->quota_rate || !d->quota_tok0_micro || !d->arrival_us || !d->act_type ||
      !d->act_model || !d->act_t_ori_us || !d->act_kmask || !d->act_param || !d->act_pin_node)
    return TG_E_INVALID_ARG;

  TraceMaxima mx;
  const int mx_err = trace_maxima(d, &mx);
  if (mx_err != TG_OK) return mx_err;
  const size_t nN = (size_t)S * M, nA = (size_t)S * A;
  std::vector<char> host;
  auto add = [&](size_t bytes) { size_t off = (host.size() + 255) & ~size_t(255); host.resize(off + bytes, 0); return off; };
  tg_trace* t = new (std::nothrow) tg_trace();
  if (!t) return TG_E_NOMEM;
  std::memset(t, 0, sizeof *t);
  t->mx = mx;
  try {
    const size_t o_ntype = add(nN), o_ncap = add(nN * 4), o_rate = add(nN * 4), o_tok = add(nN * 8), o_rank = add(nN * 4),
                 o_tnidx = add(nN * 4), o_tnoff = add((size_t)S * 16);
    const size_t o_arr = add(nA * 8), o_atype = add(nA), o_amodel = add(nA), o_astat = add(nA), o_aT = add(nA * 8),
                 o_amask = add(nA * 4), o_aparam = add(nA * 4), o_apin = add(nA * 4);
    const size_t o_asvc = add(svc ? nA * 4 : 0), o_rest = add(svc ? TG_MAX_SERVICES * 8 : 0);
    const size_t o_aquota = add(d->act_quota_mask ? nA * 8 : 0);
    const bool aux = d->node_aux != nullptr;
    const size_t o_naux = add(aux ? nN * 4 : 0), o_aaux = add(aux ? nA * 4 : 0);
    if (aux) {
      for (size_t g = 0; g < nN; ++g) if (d->node_aux[g] < 0) { delete t; return TG_E_INVALID_ARG; }
      for (size_t g = 0; g < nA; ++g) if (d->act_aux[g] < 0) { delete t; return TG_E_INVALID_ARG; }
      std::memcpy(host.data() + o_naux, d->node_aux, nN * 4);
      std::memcpy(host.data() + o_aaux, d->act_aux, nA * 4);
    }
    const size_t o_kcap = add(d->order_policy == TG_ORDER_COST ? (size_t)S * 3 * 4 : 0);
    const size_t o_speed = add(std::max<size_t>((size_t)d->n_classes * K, 1) * 4);
    auto at = [&](size_t off) { return host.data() + off; };
    std::vector<int> max_cap((size_t)S * 3, -1);
    for (int s = 0; s < S; ++s) {
      int cnt[3] = {0, 0, 0};
      for (int j = 0; j < M; ++j) {
        const size_t g = (size_t)s * M + j;
        const int ty = d->node_type[g], cap = d->node_cap[g];
        if (ty >= TG_N_TYPES || cap < 0) { delete t; return TG_E_INVALID_ARG; }
        if (ty == TG_TYPE_GPU && cap != 8) { delete t; return TG_E_INVALID_ARG; }
        if (ty == TG_TYPE_CPU && cap > TG_MAX_CPU_UNITS) { delete t; return TG_E_RANGE; }
        if (ty == TG_TYPE_API) {
          const int64_t tok = d->quota_tok0_micro[g];
          if (d->quota_rate[g] < 0 || tok < 0 || tok > (int64_t)cap * 1000000) { delete t; return TG_E_INVALID_ARG; }
          if ((int64_t)d->quota_rate[g] * d->tick_us >= (1ll << 50)) { delete t; return TG_E_RANGE; }
        }
        ((uint8_t*)at(o_ntype))[g] = (uint8_t)ty;
        ((int32_t*)at(o_ncap))[g] = cap;
        ((int32_t*)at(o_rate))[g] = d->quota_rate[g];
        ((int64_t*)at(o_tok))[g] = d->quota_tok0_micro[g];
        ((int32_t*)at(o_rank))[g] = cnt[ty]++;
        max_cap[(size_t)s * 3 + ty] = std::max(max_cap[(size_t)s * 3 + ty], cap);
      }
      int32_t* off = (int32_t*)at(o_tnoff) + (size_t)s * 4;
      off[0] = 0; off[1] = cnt[0]; off[2] = cnt[0] + cnt[1]; off[3] = M;
      int fill[3] = {off[0], off[1], off[2]};
      for (int j = 0; j < M; ++j) ((int32_t*)at(o_tnidx))[(size_t)s * M + fill[d->node_type[(size_t)s * M + j]]++] = j;
      int64_t sumT = 0, prev = 0;
      for (int i = 0; i < A; ++i) {
        const size_t g = (size_t)s * A + i;
        const int ty = d->act_type[g], model = d->act_model[g];
        if (ty >= TG_N_TYPES || model > TG_MODEL_TABLE || (ty == TG_TYPE_API && model != TG_MODEL_NONE)) { delete t; return TG_E_INVALID_ARG; }
        const int64_t T = d->act_t_ori_us[g], arr = d->arrival_us[g];
        if (T < 1 || T >= TG_T_ORI_LIMIT || arr < 0 || arr >= TG_TIME_LIMIT) { delete t; return TG_E_RANGE; }
        if (arr < prev) { delete t; return TG_E_INVALID_ARG; }
        prev = arr;
        sumT += T;
        const uint32_t param = d->act_param[g];
        if (model == TG_MODEL_AMDAHL && param > 1000000u) { delete t; return TG_E_ELASTICITY; }
        if (model == TG_MODEL_TABLE && param >= (uint32_t)d->n_classes) { delete t; return TG_E_ELASTICITY; }
        uint32_t mask = d->act_kmask[g] & ((1u << d->type_k[ty]) - 1u);
        if (model == TG_MODEL_NONE) mask &= (~mask + 1u);
        int pin = d->act_pin_node[g];
        if (pin < 0) pin = -1;
        if (pooled && ty == TG_TYPE_GPU && pin >= 0) { delete t; return TG_E_INVALID_ARG; }   // a pool has no pins
        bool infeasible = mask == 0;
        if (!infeasible) {
          const int kmin = d->k_list[__builtin_ctz(mask)];
          if (pin >= 0) infeasible = pin >= M || d->node_type[(size_t)s * M + pin] != ty || kmin > d->node_cap[(size_t)s * M + pin];
          else infeasible = kmin > max_cap[(size_t)s * 3 + ty];
        }
        if (d->act_quota_mask) {                             // further quotas: a pinned API action names other API nodes
          const uint64_t more = d->act_quota_mask[g];
          if (more) {
            const bool pinned_api = ty == TG_TYPE_API && pin >= 0 && pin < M && d->node_type[(size_t)s * M + pin] == TG_TYPE_API;
            if (!pinned_api || (cnt[TG_TYPE_API] < 64 && (more >> cnt[TG_TYPE_API])) ||
                (more >> ((int32_t*)at(o_rank))[(size_t)s * M + pin] & 1ull)) { delete t; return TG_E_INVALID_ARG; }
          }
          ((uint64_t*)at(o_aquota))[g] = more;
        }
        if (pin >= M) pin = M;
        if (svc) {
          const int sv = d->act_service[g] < 0 ? -1 : d->act_service[g];
          if (sv >= d->n_services || (sv >= 0 && ty != TG_TYPE_GPU)) { delete t; return TG_E_INVALID_ARG; }
          ((int32_t*)at(o_asvc))[g] = sv;
        }
        ((int64_t*)at(o_arr))[g] = arr;
        ((uint8_t*)at(o_atype))[g] = (uint8_t)ty;
        ((uint8_t*)at(o_amodel))[g] = (uint8_t)model;
        ((uint8_t*)at(o_astat))[g] = infeasible;
        ((int64_t*)at(o_aT))[g] = T;
        ((uint32_t*)at(o_amask))[g] = mask;
        ((uint32_t*)at(o_aparam))[g] = param;
        ((int32_t*)at(o_apin))[g] = pin;
      }
      if (sumT >= TG_SUM_T_LIMIT) { delete t; return TG_E_RANGE; }
    }
    if (d->order_policy == TG_ORDER_COST) std::memcpy(at(o_kcap), max_cap.data(), (size_t)S * 3 * 4);
    if (d->n_classes) std::memcpy(at(o_speed), d->speedup_q16, (size_t)d->n_classes * K * 4);
    if (svc) std::memcpy(at(o_rest), d->restore_us, (size_t)d->n_services * 8);

    t->arena_bytes = host.size();
    if (hipMalloc(&t->d_arena, t->arena_bytes) != hipSuccess) { delete t; return TG_E_NOMEM; }
    hipStream_t st = (hipStream_t)hip_stream;
    if (hipMemcpyAsync(t->d_arena, host.data(), t->arena_bytes, hipMemcpyHostToDevice, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) {
      (void)hipFree(t->d_arena); delete t; return TG_E_HIP;
    }
    char* base = (char*)t->d_arena;
    TgTraceDev& v = t->dev;
    v.S = S; v.A = A; v.M = M; v.K = K; v.n_classes = d->n_classes; v.depth = d->depth; v.max_ticks = d->max_ticks;
    v.tick_us = d->tick_us;
    for (int q = 0; q < TG_MAX_K; ++q) v.k_list[q] = q < K ? d->k_list[q] : 0;
    for (int k = 0; k < 3; ++k) v.type_k[k] = d->type_k[k];
    v.type_k[3] = 0;
    v.node_type = (const uint8_t*)(base + o_ntype); v.node_cap = (const int32_t*)(base + o_ncap);
    v.quota_rate = (const int32_t*)(base + o_rate); v.quota_tok0 = (const int64_t*)(base + o_tok);
    v.node_rank = (const int32_t*)(base + o_rank); v.tnode_idx = (const int32_t*)(base + o_tnidx);
    v.tnode_off = (const int32_t*)(base + o_tnoff);
    v.arrival = (const int64_t*)(base + o_arr); v.act_type = (const uint8_t*)(base + o_atype);
    v.act_model = (const uint8_t*)(base + o_amodel); v.act_static = (const uint8_t*)(base + o_astat);
    v.act_T = (const int64_t*)(base + o_aT); v.act_kmask = (const uint32_t*)(base + o_amask);
    v.act_param = (const uint32_t*)(base + o_aparam); v.act_pin = (const int32_t*)(base + o_apin);
    v.act_service = svc ? (const int32_t*)(base + o_asvc) : nullptr;
    v.restore = svc ? (const int64_t*)(base + o_rest) : nullptr;
    v.cache_slots = svc ? d->cache_slots : 0;
    v.queue_prefix = (d->flags & TG_TRACE_QUEUE_PREFIX) ? 1 : 0;
    v.gpu_pooled = pooled ? 1 : 0;
    v.cache_per_gpu = svc && (d->flags & TG_TRACE_CACHE_PER_GPU) ? 1 : 0;
    v.act_quota = d->act_quota_mask ? (const uint64_t*)(base + o_aquota) : nullptr;
    v.node_aux = aux ? (const int32_t*)(base + o_naux) : nullptr;
    v.act_aux = aux ? (const int32_t*)(base + o_aaux) : nullptr;
    v.numa_cores = d->numa_cores;
    v.order_cost = d->order_policy == TG_ORDER_COST ? 1 : 0;
    v.kind_cap = v.order_cost ? (const int32_t*)(base + o_kcap) : nullptr;
    v.speedup = (const uint32_t*)(base + o_speed);
  } catch (const std::bad_alloc&) {
    delete t;
    return TG_E_NOMEM;
  }
  *out = t;
  return TG_OK;
}

extern "C" void tg_free_trace(tg_trace* t) {
  if (!t) return;
  if (t->d_arena) (void)hipFree(t->d_arena);
  delete t;
}

extern "C" int tg_replay_workspace_bytes(const tg_trace* t, size_t* bytes) {
  if (!t || !bytes) return TG_E_INVALID_ARG;
  *bytes = carve(t->dev, nullptr, nullptr);
  return TG_OK;
}

extern "C" int tg_replay_trace_part(const tg_trace* t, const tg_replay_out* out, void* d_ws, size_t ws_bytes, int restart, int n_ticks,
                                    void* hip_stream) {
  if (n_ticks < 1) return TG_E_INVALID_ARG;
  if (!t || !out || !out->start_us || !out->finish_us || !out->units || !out->node || !out->mean_act_us ||
      !out->p99_act_us || !out->n_started || !out->n_ticks || (t->dev.numa_cores && !out->core_set))
    return TG_E_INVALID_ARG;
  if (!d_ws || ((uintptr_t)d_ws & 255) || ws_bytes < carve(t->dev, nullptr, nullptr)) return TG_E_WORKSPACE;
  hipStream_t s = (hipStream_t)hip_stream;
  const TgTraceDev& T = t->dev;
  ReplayWs W;
  carve(T, (char*)d_ws, &W);
  TgNodeLdsPlan plan;
  ReplayLds LD;
  size_t lds;
  const int fit = replay_layout(t->mx, T.K, &LD, &plan, &lds);
  if (fit != TG_OK) return fit;
  auto kernel = T.order_cost ? (T.queue_prefix ? tg_replay_kernel<true, true> : tg_replay_kernel<false, true>)
                             : (T.queue_prefix ? tg_replay_kernel<true, false> : tg_replay_kernel<false, false>);
  TG_HIP_CHECK(hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  const size_t total = (size_t)T.S * T.A * T.K;
  if (restart) {                                                  // durations and places stay in the workspace for the calls that go on
    hipLaunchKernelGGL(tg_trace_dur_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, T, W.dur);
    if (T.order_cost)
      hipLaunchKernelGGL(tg_trace_key_kernel, dim3((unsigned)(((size_t)T.S * T.A + 255) / 256)), dim3(256), 0, s, T, W.dur, W.okey, W.okey0);
  }
  hipLaunchKernelGGL(kernel, dim3(T.S), dim3(kThreads), lds, s, T, W, *out, LD, plan, restart ? 1 : 0, n_ticks);
  return hipGetLastError() == hipSuccess ? TG_OK : TG_E_HIP;
}

extern "C" int tg_replay_trace(const tg_trace* t, const tg_replay_out* out, void* d_ws, size_t ws_bytes, void* hip_stream) {
  if (!t) return TG_E_INVALID_ARG;
  return tg_replay_trace_part(t, out, d_ws, ws_bytes, 1, t->dev.max_ticks, hip_stream);
}

extern "C" int tg_replay_capacity(const tg_trace_desc* d, int64_t* cap) {
  if (!d || !cap || !d->node_type || !d->node_cap) return TG_E_INVALID_ARG;
  if (d->S < 1 || d->A < 1 || d->M < 1 || d->K < 1 || d->K > TG_MAX_K) return TG_E_INVALID_ARG;
  if (d->A > TG_MAX_ACTIONS || d->M > 65535) return TG_E_RANGE;
  TraceMaxima mx;
  const int err = trace_maxima(d, &mx);
  if (err != TG_OK) return err;
  TgNodeLdsPlan plan;
  ReplayLds LD;
  size_t lds;
  const int fit = replay_layout(mx, d->K, &LD, &plan, &lds);
  if (fit != TG_OK) return fit;
  // lists in the workspace: one slice of A entries per scenario each (waiting list per kind, running set,
  // candidate order, waiting-pinned order)
  cap[TG_REPLAY_CAP_WAIT_CPU] = cap[TG_REPLAY_CAP_WAIT_GPU] = cap[TG_REPLAY_CAP_WAIT_API] = d->A;
  cap[TG_REPLAY_CAP_RUNNING] = d->A;
  cap[TG_REPLAY_CAP_CAND_NODE] = cap[TG_REPLAY_CAP_CAND_STEP] = cap[TG_REPLAY_CAP_PINNED_WAIT_STEP] = d->A;
  // per-node tables of a wavefront, from the byte ranges of the plan itself
  const int64_t choice_bytes = plan.off_F - plan.off_choice - 16;
  const int64_t rows_tables = std::min<int64_t>({plan.cand_rows,                                     // durations, minimum option
                                                 plan.off_rowbest - plan.off_q0,
                                                 (plan.off_rowarg - plan.off_rowbest) / 8 - 1,       // best totals of rows 0..m
                                                 (plan.off_sel - plan.off_rowarg) / 4 - 1,
                                                 2 * (int64_t)plan.sel_stride});                     // allocation rows, 4 bits each
  const int64_t rows_cpu = mx.max_cap_cpu > 0 ? choice_bytes / std::max(tg_choice_stride(mx.max_cap_cpu), 1) : 0;
  const int64_t rows_gpu = choice_bytes / ((int64_t)mx.max_chunk_states * 2);
  cap[TG_REPLAY_CAP_CAND_CPU_ELASTIC] = std::min(rows_tables, rows_cpu);
  cap[TG_REPLAY_CAP_CAND_GPU_ELASTIC] = std::min(rows_tables, rows_gpu);
  cap[TG_REPLAY_CAP_BUSY_UNITS] = LD.busy_slots;
  cap[TG_REPLAY_CAP_HEAP_ENTRIES] = std::min(plan.heap_slots, 4 * TG_WAVE);                          // LDS staging; register heap
  const int64_t dp_bytes = plan.off_choice - plan.off_dp;
  cap[TG_REPLAY_CAP_CHUNK_STATES] = std::min<int64_t>({mx.max_chunk_states, plan.dp_width, dp_bytes / 16, 512});   // rows; 9-bit state keys
  // a row of Alg. 3's table as the kernel stores it: 64-bit cells, or 32-bit cells behind 64 sentinels
  cap[TG_REPLAY_CAP_DP_CELLS] = std::min<int64_t>({plan.dp_width, dp_bytes / 16, dp_bytes / 8 - 2 - TG_WAVE});
  cap[TG_REPLAY_CAP_NODES_CPU] = LD.pool_nodes[0];
  cap[TG_REPLAY_CAP_NODES_GPU] = LD.pool_nodes[1];
  cap[TG_REPLAY_CAP_NODES_API] = LD.pool_nodes[2];
  return TG_OK;
}
