// Internal definitions shared by the HIP sources of libtangram (not part of the C interface).
#ifndef TG_INTERNAL_H_
#define TG_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <vector>

#include "tg.h"

#define TG_WAVE 64
#define TG_SCORE_CHUNK 512  // entries of the score tensor per workgroup (4 KB): 128 lanes x 2 pairs

// Packed device copy of a problem.  Passed to kernels by value; all pointers are device memory.
struct TgDev {
  int B, N, M, K, n_classes, n_tasks, depth, has_busy;
  int k_list[TG_MAX_K];
  int type_k[4];
  // nodes [B*M]
  const uint8_t* node_type;
  const int32_t* node_cap;
  const int32_t* node_free;
  const int64_t* node_backlog;
  const uint32_t* node_chunks;    // four 8-bit counts of free chunks (sizes 1,2,4,8), GPU nodes
  const int32_t* node_busy_off;   // [B*M+1]
  const int64_t* node_busy_rel;
  const int32_t* node_rank;       // rank of the node among the nodes of its kind in its snapshot
  // actions [B*N]
  const uint8_t* act_type;
  const uint8_t* act_model;
  const uint8_t* act_static;      // 1: statically infeasible (no option, bad pin, minimum above every node)
  const int64_t* act_T;
  const int64_t* act_age;
  const uint32_t* act_kmask;      // effective mask: limited to the kind's options, lowest bit only if non-elastic
  const uint32_t* act_param;
  const int32_t* act_pin;         // node index or -1
  const int32_t* act_pin_rank;    // rank of the pinned node among the nodes of its kind, -1: free or statically infeasible
  const int32_t* act_task;
  const int32_t* node_aux;        // [B*M] second resource left on the node, or nullptr: no second resource
  const int32_t* act_aux;         // [B*N] what an unpinned action needs of it (nullptr together with node_aux)
  // services (Sec. 5.3): all nullptr when the problem has none
  const int32_t* act_service;     // [B*N] service id or -1
  const uint64_t* node_resident;  // [B*M] services resident on the node, one bit each
  const int64_t* restore;         // [TG_MAX_SERVICES] restore time per service
  const uint64_t* row_svc;        // [B*N] kind-grouped: restore time | (service + 1) << 48 of the row's action
  const uint64_t* node_res_k;     // [B*M] kind-grouped copy of node_resident (same order as node_word)
  const uint32_t* node_chunks_real;  // [B*M] pooled GPUs: every node's own free chunks (node_chunks holds the pool's at its first node), else nullptr
  const uint64_t* act_quota;      // [B*N] further quotas of an API action (ranks among the snapshot's API nodes), or nullptr
  const uint64_t* node_cores;     // [B*M*4] bitmap of the free cores of CPU nodes, or nullptr: no core topology
  int numa_cores;                 // cores per NUMA domain (power of two, 4..64) when node_cores is given
  const uint32_t* speedup;        // [n_classes*K]
  // grouping by resource kind, per snapshot
  const int32_t* tact_idx;        // [B*N] action ids grouped by kind, FCFS inside a group
  const int32_t* tact_off;        // [B*4] group starts (entry 3 = N)
  const int32_t* tnode_idx;       // [B*M] node ids grouped by kind
  const int32_t* tnode_off;       // [B*4]
  // kind-grouped views used by the score kernel
  const struct TgRowRec* row_rec; // [B*N] kind-grouped: what Eq. 1 needs of an action
  const int32_t* row_pin;         // [B*N] kind-grouped: rank of the pinned node inside the kind, -1 free, -2 matches nothing
  const uint64_t* node_word;      // [B*M] kind-grouped: backlog | (options admitted by the capacity) << 48
};

// Kind-grouped copy of the fields of an action that Eq. 1 reads (16 bytes, one load).
struct TgRowRec {
  int64_t T;
  uint32_t param;
  uint16_t kmask;
  uint8_t model, pad_;
};

// One dense block of the score tensor: actions of one kind x nodes of that kind x options.
struct TgBlock {
  int64_t cost_off;   // first entry of the block in the tensor
  int64_t entries;    // rows * M_t * K_t  (< 2^31)
  int32_t rows, M_t, K_t, b, t;
  int32_t a_off;      // b*N + first action of the kind in the kind-grouped order
  int32_t n_off;      // b*M + first node of the kind in the kind-grouped order
};

// What the score kernel needs of one block, and the three blocks of a snapshot in one record
// that a workgroup reads with a single uniform load.
struct TgScoreKind {
  int64_t cost_off;   // first entry of the block in the tensor
  double inv_lr;      // 1 / (M_t * K_t)
  int32_t entries;    // rows * M_t * K_t, 0: no such block
  int32_t a_off, n_off;   // as TgBlock
  uint16_t M_t, K_t;
  uint32_t magic_k;   // floor(2^20 / K_t) + 1: x / K_t == (x * magic_k) >> 20 for x < 2^17
  int32_t rows;       // actions of the kind
};
static_assert(sizeof(TgScoreKind) == 40, "three of them and eight more bytes make a snapshot's record");
struct TgScoreSnap {
  TgScoreKind kind[3];
  int32_t chunks;     // workgroups that cover the three blocks
  int32_t pad_;
};
static_assert(sizeof(TgScoreSnap) == 128, "one record per snapshot, read as two 64-byte scalar loads");

// One launch of the score kernel: snapshots first .. first + n_snaps of the record array on a
// grid of max_chunks x n_snaps workgroups.
struct TgScoreLaunch {
  int first, n_snaps, max_chunks;
};

struct tg_problem {
  TgDev dev;
  void* d_arena;
  size_t arena_bytes;
  TgBlock* d_blocks;       // inside the arena
  int n_blocks;
  const TgScoreSnap* d_score_snaps;          // inside the arena, in launch order
  std::vector<TgScoreLaunch> score_launches; // usually one: all snapshots in index order
  int64_t n_candidates;
  // tg_assign runs the node classes side by side: two side streams (default priority) forked
  // from and joined back into the caller's stream with events
  hipStream_t side_stream[2];
  hipEvent_t ev_fork, ev_join[2];
  // tg_step writes the score tensor on a third stream next to the assignment
  hipStream_t score_stream;
  hipEvent_t ev_score_fork, ev_score_done;
  int order_policy;        // TG_ORDER_*
  int queue_prefix;        // 1: one admitted prefix of the whole queue instead of one per pool
  int max_actions_of_kind; // largest N_t over all snapshots and kinds
  int max_nodes_of_kind;   // largest M_t over all snapshots and kinds
  int max_nodes_not_cpu;   // the same over the GPU and API kinds only
  int64_t backlog_spread;  // largest (max - min) backlog over the nodes of one kind in one snapshot
  int max_free_cpu;        // largest node_free over CPU nodes
  int max_heap;            // largest free + busy over CPU and GPU nodes
  size_t nodes_free_gt16, nodes_free_gt64;   // bounds on the nodes that can hold more than 16 / 64 candidates: nodes with as many free
                                             // units (for 64 also: no more than a 65th of the actions of the node's kind)
  int max_free_gpu, max_chunk_states;
  int64_t* d_score_dur;    // [B*N*(K+1)] scratch of tg_score_candidates: getDur per (kind-grouped row, option), then the row's pin; every call
                           // writes the same values, so calls that overlap do not disturb each other
};

// the unit counts k_list[0..8), one byte each
__host__ __device__ static inline uint64_t tg_pack_k(const int* k_list) {
  uint64_t w = 0;
  for (int q = 0; q < TG_MAX_K; ++q) w |= (uint64_t)(uint32_t)k_list[q] << (8 * q);
  return w;
}

__host__ __device__ static inline int tg_chunk_level(int k) { return k <= 1 ? 0 : (k <= 2 ? 1 : (k <= 4 ? 2 : 3)); }

#ifdef __HIPCC__
// Eq. 1 in integer microseconds: ceil(num / den) with num < 2^62 and 2^10 <= den < 2^27.
// A double-precision reciprocal gives the quotient to within a few units; the remainder test
// makes it exact.
__device__ static inline int64_t tg_ceil_div(uint64_t num, uint32_t den) {
  // reciprocal: the hardware estimate refined by two Newton steps (any small error is removed below)
  const double dd = (double)den;
  double inv = __builtin_amdgcn_rcp(dd);
  inv = __builtin_fma(__builtin_fma(-dd, inv, 1.0), inv, inv);
  inv = __builtin_fma(__builtin_fma(-dd, inv, 1.0), inv, inv);
  uint64_t q = (uint64_t)((double)num * inv);
  int64_t r = (int64_t)(num - q * (uint64_t)den);
  while (r < 0) { --q; r += den; }
  while (r >= (int64_t)den) { ++q; r -= den; }
  return (int64_t)(q + (r > 0));
}

// getDur(k_list[q]) of one action (Eq. 1); the caller has checked that option q is allowed.
__device__ static inline int64_t tg_duration(int model, int64_t T, uint32_t param, int k, uint32_t speedup) {
  if (model == TG_MODEL_NONE) return T;
  int64_t d;
  if (model == TG_MODEL_AMDAHL) {
    const uint32_t w = (1000000u - param) * (uint32_t)k + param;   // < 2^26
    d = tg_ceil_div((uint64_t)T * w, 1000000u * (uint32_t)k);
  } else {
    d = tg_ceil_div((uint64_t)T << 16, speedup);
  }
  return d < 1 ? 1 : d;
}

// Largest free chunk size (1,2,4,8 or 0) of a packed count word.
__device__ static inline int tg_chunk_largest(uint32_t c) {
  if (c >> 24) return 8;
  if ((c >> 16) & 0xff) return 4;
  if ((c >> 8) & 0xff) return 2;
  return (c & 0xff) ? 1 : 0;
}

// Best fit with split (Sec. 5.3): take the smallest free chunk of level >= level(k); a larger
// chunk leaves one free chunk of every size from k up to half of it.  Caller checked the fit.
__device__ static inline uint32_t tg_chunk_take(uint32_t c, int k) {
  const int a = tg_chunk_level(k);
  for (int b = a; b < 4; ++b)
    if ((c >> (8 * b)) & 0xff) {
      c -= 1u << (8 * b);
      for (int x = a; x < b; ++x) c += 1u << (8 * x);
      return c;
    }
  return c;
}
#endif

#define TG_HIP_CHECK(expr)                       \
  do {                                           \
    hipError_t e_ = (expr);                      \
    if (e_ != hipSuccess) return TG_E_HIP;       \
  } while (0)

// kernels' launchers (defined in the .hip files)
int tg_launch_score(const tg_problem* p, int64_t* d_cost, hipStream_t s);

#endif  // TG_INTERNAL_H_
