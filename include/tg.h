/*
 * tg.h - C interface of the action-level elastic scheduling step of ARL-Tangram
 * (arXiv 2603.13019), batched over independent cluster snapshots and run on one AMD
 * MI355X (gfx950) by hand-written HIP kernels.
 *
 * One scheduling step (Sec. 4.2, Alg. 1; Alg. 2-4 in App. A-B) takes the waiting queue W of
 * actions in first-come order and the resource status R, and returns the selected actions
 * with their resource units.  Here R is a set of nodes of three kinds (Sec. 5): CPU nodes
 * (cores, scheduled per node, trajectories may be pinned to a node, Sec. 5.2), GPU nodes
 * (buddy chunks of 1/2/4/8 GPUs, Sec. 5.3) and API quotas (Sec. 5.1).
 *
 * Conventions
 *   - All times are int64 microseconds relative to the snapshot instant.  TG_INF marks a
 *     candidate that does not exist.
 *   - Every function returns TG_OK (0) or a negative TG_E_* code; on an error nothing has
 *     been written to any output and nothing has been launched.
 *   - "host" pointers are ordinary CPU memory, read only during the call.  "device" pointers
 *     are HIP device memory owned by the caller (the Python binding allocates it with
 *     PyTorch).  Kernels are enqueued on `hip_stream` (a hipStream_t, NULL = default stream);
 *     no entry point synchronises except tg_build_problem / tg_build_trace (which return after
 *     their host-to-device copies have completed).  Results are valid once the caller has
 *     synchronised the stream.
 *   - A tg_problem / tg_trace is immutable after it is built and owns only its packed device
 *     copy of the inputs (plus, for a tg_problem, a scratch array of one int64 per (action, option)
 *     into which every tg_score_candidates / tg_step call writes the same durations, and three internal
 *     streams and their events on which tg_assign and tg_step run part of their work, forked from and
 *     joined back into `hip_stream`).  No other entry point allocates device memory.  Launches that use the same tg_problem may
 *     be in flight together (each with its own outputs and workspace), but the host calls that
 *     enqueue them must not overlap: one thread at a time per tg_problem.
 *   - Index of an action inside its snapshot == its first-come rank == its action id.
 */
#ifndef TG_H_
#define TG_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TG_INF INT64_MAX

enum { TG_OK = 0, TG_E_INVALID_ARG = -1, TG_E_RANGE = -2, TG_E_ELASTICITY = -3, TG_E_WORKSPACE = -4,
       TG_E_HIP = -5, TG_E_NOMEM = -6, TG_E_STATIC_WS = -7 };

/* resource kinds (Sec. 5) and elasticity models of an action (Sec. 4.1, Eq. 1) */
enum { TG_TYPE_CPU = 0, TG_TYPE_GPU = 1, TG_TYPE_API = 2, TG_N_TYPES = 3 };
enum { TG_MODEL_NONE = 0,   /* elasticity unknown: runs for T_ori on its minimum units (Alg. 1)        */
       TG_MODEL_AMDAHL = 1, /* E(k) = 1/((1-p)k+p), p = act_param in parts per million             */
       TG_MODEL_TABLE = 2   /* E(k)*k = speedup_q16[act_param][q] / 65536                           */ };
/* why an action was not selected in this step */
enum { TG_SELECTED = 0,
       TG_DEFER_PREFIX = 1,     /* behind the first action of its pool that did not fit (Alg. 1)  */
       TG_DEFER_EVICTED = 2,    /* admitted, then evicted by the greedy tail eviction (Alg. 1)      */
       TG_DEFER_INFEASIBLE = 3  /* no allowed unit count fits any node it may use, or bad pin        */ };

/* Order in which tg_assign visits the waiting queue of a pool.  The paper schedules first come
 * first served and notes that its algorithm works with other orderings (Sec. 4.2); TG_ORDER_COST
 * is one: ascending least estimated ACT (Eq. 2) over the action's candidates - the smallest
 * finite entry of its row of the score tensor -, equal keys in FCFS order.  The admitted
 * prefix, the per-node candidate lists and the eviction tail of Alg. 1 all follow that order. */
enum { TG_ORDER_FCFS = 0, TG_ORDER_COST = 1 };

/* limits checked by tg_build_problem / tg_build_trace */
enum { TG_MAX_K = 8, TG_MAX_UNIT = 64, TG_MAX_CPU_UNITS = 256, TG_MAX_GPU_UNITS = 64,
       TG_MAX_CHUNK_STATES = 512, TG_MAX_DEPTH = 4,
       TG_MAX_ACTIONS = 131072,      /* N, actions per snapshot / A, actions per scenario          */
       TG_MAX_NODES_OF_KIND = 4096,  /* nodes of one resource kind in one snapshot               */
       TG_MAX_SERVICES = 64 };
#define TG_T_ORI_LIMIT (1ll << 36)  /* 1 <= T_ori < 2^36 us                                      */
#define TG_TIME_LIMIT (1ll << 40)   /* backlog, age, busy release times in [0, 2^40)              */
#define TG_SUM_T_LIMIT (1ll << 44)  /* sum of T_ori over one snapshot / scenario                  */

typedef struct tg_problem tg_problem; /* opaque */
typedef struct tg_trace tg_trace;     /* opaque */

/*
 * B snapshots, each with N queued actions (W of Alg. 1, FCFS order) and M nodes (R of Alg. 1).
 * All arrays are host memory.  Node arrays have B*M entries (M with nodes_shared), action arrays
 * B*N entries, snapshot-major.
 */
typedef struct {
  int32_t B, N, M, K;
  int32_t n_classes; /* rows of speedup_q16                                                     */
  int32_t n_tasks;   /* act_task values are in [0, n_tasks); segment key of the per-task sums    */
  int32_t depth;     /* options tried for the first waiting action in Alg. 2's estimate; 2 in the paper's runs */
  int32_t order_policy; /* TG_ORDER_FCFS (0) or TG_ORDER_COST */
  const int32_t *k_list;  /* [K] ascending unit counts (the discrete sets of Sec. 4.1), 1..TG_MAX_UNIT */
  const int32_t *type_k;  /* [3] type t may use k_list[0 .. type_k[t]); GPU entries must be 1,2,4,8; API <= 1 */
  const uint32_t *speedup_q16; /* [n_classes*K] round(65536*E(k_q)*k_q); nondecreasing in q, in [65536, 65536*k_q] */
  /* nodes */
  const uint8_t *node_type;        /* TG_TYPE_*                                                  */
  const int32_t *node_cap;         /* units the node has (cores, GPUs, bucket size)              */
  const int32_t *node_free;        /* units free for this step (<= cap); API: whole tokens available */
  const int64_t *node_backlog_us;  /* time at which the free units become usable (queueing part of Eq. 2) */
  const uint8_t *node_chunks;      /* [B*M*4] free chunks of 1,2,4,8 GPUs on GPU nodes; NULL: binary split of node_free */
  const int32_t *node_busy_off;    /* [B*M+1] or NULL: CSR offsets into node_busy_rel_us         */
  const int64_t *node_busy_rel_us; /* release time of every unit held by a running action (executing queue of Alg. 2) */
  /* actions */
  const uint8_t *act_type;        /* TG_TYPE_*: the key elasticity resource (Sec. 4.1)           */
  const uint8_t *act_model;       /* TG_MODEL_*; API actions must be TG_MODEL_NONE               */
  const int64_t *act_t_ori_us;    /* T_ori of Eq. 1: duration on one unit                        */
  const int64_t *act_age_us;      /* time already spent queueing (added to the reported ACT only); may be NULL */
  const uint32_t *act_kmask;      /* bit q set <=> k_list[q] is an allowed unit count            */
  const uint32_t *act_param;      /* Amdahl: parallel fraction in ppm (<= 10^6); table: class id */
  const int32_t *act_pin_node;    /* node index inside the snapshot, or negative = free to choose (Sec. 5.2) */
  const int32_t *act_task;        /* may be NULL (all zero)                                      */
  /* Second, co-constrained component of the cost vector (Sec. 4.1), e.g. memory next to CPU cores
   * (Sec. 5.2): an action that is free to choose its node (act_pin_node < 0) is only admitted to a
   * node that has act_aux left of node_aux_free, and takes it; an action pinned to a node belongs
   * to a trajectory whose share was taken when it was placed and is not charged again.
   * Both arrays or neither (NULL, NULL = no second resource); values >= 0. */
  const int32_t *node_aux_free;   /* [B*M] */
  const int32_t *act_aux;         /* [B*N] */
  /* Long-lived services under evict-on-execution (Sec. 5.3): an action that calls service s runs
   * at once on a node where s is resident in device memory; elsewhere the service is restored
   * from host memory first, which delays the action by restore_us[s] on that node.  The delay is
   * part of every estimate (score tensor, node choice, visiting-order key), of the durations
   * DPArrange and the completion heap see on that node, and of the reported ACT.
   * All three arrays or none (then n_services is ignored). */
  const int32_t *act_service;     /* [B*N] service id in [0, n_services), or negative: none     */
  const uint64_t *node_resident;  /* [B*M] bit s set <=> service s is resident on the node       */
  const int64_t *restore_us;      /* [n_services] in [0, 2^36)                                   */
  /* Core topology of the CPU nodes (Sec. 5.2: the manager names the cores an action runs on and
   * prefers cores of one NUMA domain).  Cores [d*numa_cores, (d+1)*numa_cores) of a node form its
   * domain d.  node_core_free: per node four 64-bit words, bit c%64 of word c/64 set <=> core c is
   * free; on CPU nodes exactly node_free bits, none at or above node_cap; ignored on other nodes.
   * NULL: no topology (then numa_cores must be 0 and tg_assign_out.core_set NULL). */
  const uint64_t *node_core_free; /* [B*M*4] */
  /* Several quotas per action (Sec. 4.1: an action may query several websites, each with its own
   * quota, every one a component of its cost vector).  An API action pinned to a quota also
   * takes one token of every API node whose rank r (the r-th API node of its snapshot in index
   * order, r < 64) is set in act_quota_mask[i]; it is admitted only if all of them have a token
   * left, otherwise it does not fit and waits like any pinned action that does not fit.  The
   * estimates (Eq. 2) use the pinned node only.  Bits must be clear for actions that are not of
   * kind API or not pinned to an API node, for the action's own node and at or above the number
   * of API nodes.  node_used and units_used count these tokens.  NULL: none. */
  const uint64_t *act_quota_mask; /* [B*N] */
  int32_t n_services;             /* 1..TG_MAX_SERVICES                                          */
  int32_t numa_cores;             /* 4, 8, 16, 32 or 64 with node_core_free                      */
  /* 1: the GPU nodes of a snapshot form one pool (Sec. 5.3 and Alg. 4: the GPU manager schedules
   * the cluster as a whole and the state counts the free chunks of every size wherever they are).
   * Admission, DPArrange, the eviction loop and the completion heap then see one resource with the
   * chunks, units and running actions of all GPU nodes; every selected action gets the smallest
   * free chunk of the cluster that holds it, on the lowest-numbered node that has one, and `node`
   * reports that node; node_obj holds the pool's objective at the first GPU node.  Needs per
   * snapshot: GPU nodes of 8 units, at most TG_MAX_GPU_UNITS units together, one common
   * node_backlog_us, no GPU action pinned, no services (else TG_E_INVALID_ARG), and pooled chunk
   * counts within TG_MAX_CHUNK_STATES (else TG_E_RANGE).  0: every node on its own. */
  int32_t gpu_pooled;
  /* 1: Alg. 1 as printed - the admitted candidates are the longest prefix of the whole waiting
   * queue (in visiting order: FCFS rank, or with TG_ORDER_COST the key and then the FCFS rank,
   * over all kinds of resource together) that the resources accommodate: the first action that
   * does not fit, and every action behind it, waits (TG_DEFER_PREFIX), whatever its kind.
   * 0: one such prefix per pool - a misfit closes the queue of its own kind of resource, or of its
   * node if it is pinned (the managers of Sec. 5.2 schedule their resources independently). */
  int32_t queue_prefix;
  /* 1: one node table for all snapshots (the same cluster seen at B instants' queues, R of Alg. 1 given once):
   * every node array then has M entries ([M*4] for node_chunks and node_core_free, node_busy_off [M+1]) instead
   * of B*M, and node indices (act_pin_node) mean the same node in every snapshot.  The builder writes the table
   * out per snapshot, so device memory and every result are as with B identical tables.  0: node arrays [B*M]. */
  int32_t nodes_shared;
  int32_t reserved_;              /* 0 */
} tg_problem_desc;

/* Per-snapshot result of tg_assign.  Only mean_act_us and util are floating point. */
typedef struct {
  int64_t sum_act_us; /* sum of ACT over selected actions (Eq. 2)                               */
  int32_t n_selected, n_prefix, n_evicted, n_infeasible;
  int64_t units_used[3], units_free[3]; /* per resource kind                                    */
  double mean_act_us;                   /* sum_act_us / n_selected, 0 if none                    */
  double util[3];                       /* units_used / units_free, 0 if no free unit            */
} tg_summary;

/* Device output buffers of tg_assign ([B*N] unless noted); optional ones may be NULL. */
typedef struct {
  int32_t *node;         /* chosen node, -1 if not selected                                    */
  int32_t *units;        /* allocated units k_i, 0 if not selected                              */
  int64_t *act_us;       /* age + backlog[node] + getDur(k_i), -1 if not selected               */
  uint8_t *defer_reason; /* TG_SELECTED / TG_DEFER_*                                            */
  tg_summary *summary;   /* [B]                                                                 */
  int32_t *node_used;    /* [B*M] units handed out per node; optional                           */
  int64_t *task_sum_us;  /* [B*n_tasks] sum of ACT per task; optional                           */
  int64_t *node_obj;     /* [B*M] final approximated objective (Alg. 2) of nodes that ran the eviction loop, else -1; optional */
  /* [B*N*4] the cores of every selected CPU action as a bitmap laid out like node_core_free, zero
   * for all other actions; optional, needs a problem built with node_core_free.  The selected
   * actions of a node take their cores one after the other in visiting order: if a domain has
   * `units` free cores, from the domain with the fewest free cores that still has them (lowest
   * domain on ties); otherwise whole domains, the one with the most free cores first (lowest on
   * ties), which spans the fewest domains; inside a domain the lowest-numbered free cores. */
  uint64_t *core_set;
} tg_assign_out;

/*
 * Formulation (Sec. 4.1): validates the description, normalises every action to (kind, T_ori,
 * allowed-unit mask, elasticity model and parameter, pin, FCFS rank), groups actions and nodes
 * by resource kind and copies the packed arrays to the device.
 * Errors: TG_E_INVALID_ARG (null pointer, bad count, unknown kind/model, k_list not ascending,
 * free > cap, chunk counts that do not add up to node_free, ...), TG_E_RANGE (a time or size outside the
 * limits above), TG_E_ELASTICITY (speedup table decreasing, above 65536*k or below 65536;
 * Amdahl fraction above 10^6; class id out of range), TG_E_HIP, TG_E_NOMEM.
 */
int tg_build_problem(const tg_problem_desc *desc, void *hip_stream, tg_problem **out);
void tg_free_problem(tg_problem *p);

/* Number of (action, node, unit-option) candidates of the score tensor and its size in bytes. */
int tg_num_candidates(const tg_problem *p, int64_t *count, int64_t *bytes);

/* Device workspace tg_assign needs for this problem. */
int tg_assign_workspace_bytes(const tg_problem *p, size_t *bytes);

/*
 * Score (Eq. 1 inside Eq. 2): estimated completion time of every type-compatible candidate,
 *   cost[b][t][i][j][q] = node_backlog_us[j] + getDur_i(k_list[q])
 * or TG_INF when k_list[q] is not allowed for action i, exceeds node j's capacity, or the
 * action is pinned to another node.  Layout: for snapshot b = 0..B-1, for kind t = 0..2, a dense
 * block [actions of kind t in FCFS order][nodes of kind t in index order][type_k[t]], q fastest.
 * d_cost: device, tg_num_candidates() int64 values, 16-byte aligned, written completely.
 */
int tg_score_candidates(const tg_problem *p, int64_t *d_cost, void *hip_stream);

/*
 * Assign (Alg. 1 per resource pool): admission in visiting order (FCFS unless the problem was
 * built with TG_ORDER_COST) at minimum units with node choice by least
 * estimated completion time (ties: smaller node index), then per node DPArrange (Alg. 3; Alg. 4's
 * chunk states on GPU nodes) inside the greedy tail eviction on the approximated objective
 * (Alg. 2), then per-snapshot summaries.
 * d_cost: NULL, or a tensor written by tg_score_candidates for this problem; when given, the
 * node choice reads its estimates from the tensor instead of recomputing them (same result);
 * with TG_ORDER_COST the estimates are always recomputed (the tensor's rows are in FCFS order).
 * d_ws/ws_bytes: device workspace of at least tg_assign_workspace_bytes(), 256-byte aligned.
 * Errors: TG_E_INVALID_ARG, TG_E_WORKSPACE, TG_E_HIP.
 */
int tg_assign(const tg_problem *p, const int64_t *d_cost, const tg_assign_out *out, void *d_ws, size_t ws_bytes,
              void *hip_stream);

/*
 * tg_assign for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, results
 * and errors as tg_assign, but the workspace is an array of TG_STATIC_WS_BYTES in the library's own
 * device data (every GPU the library runs on holds one copy until the process ends); the call
 * allocates nothing.  A problem whose tg_assign_workspace_bytes() exceeds TG_STATIC_WS_BYTES is
 * refused with TG_E_STATIC_WS before anything is launched (workload 2, B = 256 x N = 1024, needs
 * 15 MB).  All calls on one GPU share that GPU's array: it keeps the previous call's contents (the
 * kernels clear what they need cleared), and two calls in flight on the same GPU at the same time
 * race - the caller orders them on one stream or with events.
 */
#define TG_STATIC_WS_BYTES (32u << 20)
int tg_assign_static(const tg_problem *p, const int64_t *d_cost, const tg_assign_out *out, void *hip_stream);

/*
 * One whole step in one call: tg_score_candidates and tg_assign for the same problem.  The assignment
 * recomputes its estimates and does not read the tensor.  The score kernels run on a second stream: a tensor
 * of 2^29 candidates (4 GB) or more is written first and the assignment follows (side by side the two only
 * slow each other down); a smaller one is written next to the first, light kernels of the assignment
 * (durations, admission, lists) and the per-node stage (DPArrange, eviction) follows when it is written;
 * everything is forked from and joined back into `hip_stream`.  Same arguments, results and errors as the
 * two calls (d_cost must not be NULL unless the problem has no candidate); everything is complete once
 * `hip_stream` has been synchronised.  What can fail without a launch (argument checks, kernel
 * attributes) is done before the fork.
 * tg_step runs the score kernels on a stream of the problem's own; tg_step_on on the caller's
 * `score_stream` (a hipStream_t other than `hip_stream`, e.g. to bracket them with events of its own).
 */
int tg_step(const tg_problem *p, int64_t *d_cost, const tg_assign_out *out, void *d_ws, size_t ws_bytes, void *hip_stream);
int tg_step_on(const tg_problem *p, int64_t *d_cost, const tg_assign_out *out, void *d_ws, size_t ws_bytes, void *hip_stream,
               void *score_stream);

/*
 * S independent arrival traces replayed against their own clusters.  Every tick_us of simulated
 * time: finished actions release their units, quotas refill (micro-tokens, capped at the bucket
 * size node_cap), arrived actions join the waiting queue in arrival order, one scheduling step
 * (as tg_assign, backlog 0, completion heap seeded with the running actions) selects actions,
 * which start at the tick and run for exactly getDur(k) (after the restore delay of their
 * service, if any).  Action arrays have S*A entries and
 * must be sorted by arrival within a scenario; node arrays have S*M entries.
 */
/* tg_trace_desc.flags: every step admits one prefix of the whole waiting queue (as queue_prefix
 * of tg_problem_desc) instead of one prefix per pool */
enum { TG_TRACE_QUEUE_PREFIX = 1,
       /* the GPU nodes of a scenario form one pool of chunks in every step (as gpu_pooled in tg_problem_desc): the step
        * names the node whose chunk a selected action takes - the smallest free chunk of the cluster that holds it, on the
        * lowest-numbered node that has one - and `node` reports that node.  Needs: no GPU action pinned, no services, no
        * second resource (TG_E_INVALID_ARG), at most 5 GPU nodes per scenario (the pooled chunk counts of more could pass
        * TG_MAX_CHUNK_STATES: TG_E_RANGE). */
       TG_TRACE_GPU_POOLED = 2,
       /* Sec. 5.3 with the cache on the GPU instead of the node (ignored without services): every GPU of a GPU node
        * keeps up to cache_slots services of its own, least recently used out first.  An action finds its service
        * resident when every GPU of the block it is given caches it; afterwards every GPU of the block does.  The
        * allocation takes from the lowest level that has a free chunk, as always; among that level's free chunks the
        * first that holds an aligned block of the action's size caching the service gives that block, otherwise the
        * first chunk gives its first block.  The step keeps its view per node - a service counts as resident where any
        * GPU of the node caches it - so the delay an action really pays (none or restore_us) is known once it has its
        * GPUs and is never less than the step assumed. */
       TG_TRACE_CACHE_PER_GPU = 4 };
typedef struct {
  int32_t S, A, M, K, n_classes, depth;
  int32_t max_ticks; /* the replay of a scenario stops after this many ticks                    */
  uint32_t flags;    /* TG_TRACE_QUEUE_PREFIX | _GPU_POOLED | _CACHE_PER_GPU or 0; other bits clear  */
  int64_t tick_us;   /* rescheduling period                                                     */
  const int32_t *k_list, *type_k;
  const uint32_t *speedup_q16;
  const uint8_t *node_type;
  const int32_t *node_cap;          /* CPU: cores (all free at time 0); GPU: must be 8; API: bucket size (burst) */
  const int32_t *quota_rate;        /* tokens per second (API nodes)                              */
  const int64_t *quota_tok0_micro;  /* tokens at time 0, in millionths                            */
  const int64_t *arrival_us;        /* nondecreasing within a scenario, in [0, 2^40)              */
  const uint8_t *act_type, *act_model;
  const int64_t *act_t_ori_us;
  const uint32_t *act_kmask, *act_param;
  const int32_t *act_pin_node;
  /* Services of GPU actions (Sec. 5.3), both arrays or neither: every node keeps up to cache_slots
   * services resident in device memory, none at time 0.  An action whose service was not resident
   * on its node when the tick began is delayed by restore_us[service] (the step of that tick
   * estimated with the same residency); starting an action makes its service resident and the
   * most recently used one, evicting the least recently used (smaller id on ties) when the node
   * already holds cache_slots others.  Only actions of kind GPU may call a service. */
  const int32_t *act_service;       /* [S*A] service id in [0, n_services), or negative: none    */
  const int64_t *restore_us;        /* [n_services] in [0, 2^36)                                 */
  int32_t n_services;               /* 1..TG_MAX_SERVICES                                        */
  int32_t cache_slots;              /* 1..TG_MAX_SERVICES                                        */
  /* Several quotas per action as in tg_problem_desc.act_quota_mask (ranks among the API nodes of
   * the scenario): the action starts only in a tick in which every named quota holds a whole
   * token, and takes one from each.  NULL: none. */
  const uint64_t *act_quota_mask;   /* [S*A] */
  /* Second, co-constrained resource (Sec. 4.1, 5.2), the node_aux_free / act_aux of a tg_problem_desc;
   * both arrays or neither: an action that is free to choose its node (act_pin_node < 0) starts
   * only on a node that has act_aux of the resource left and holds it from its start to its
   * finish; pinned actions hold none (the share of their trajectory is not part of a trace).
   * Values >= 0. */
  const int32_t *node_aux;          /* [S*M] what every node has of it                           */
  const int32_t *act_aux;           /* [S*A]                                                     */
  /* Named cores (Sec. 5.2) as numa_cores / core_set of a step: 4, 8, 16, 32 or 64 cores per NUMA
   * domain, all cores of every CPU node free at time 0; a CPU action gets its cores by the rule of
   * tg_assign_out.core_set in the step that selects it and keeps them until it finishes;
   * tg_replay_out.core_set is then required.  0: cores are not named. */
  int32_t numa_cores;
  int32_t order_policy;             /* TG_ORDER_FCFS (0), or TG_ORDER_COST: every tick's step visits the waiting queue by least
                                     * estimated ACT (equal keys by arrival), and the actions it selects start in that order.
                                     * With services the estimate of a GPU action counts the restore time unless a node it
                                     * may run on has the service resident when the tick begins, so its place moves with
                                     * the caches */
} tg_trace_desc;

/* Device outputs of tg_replay_trace. */
typedef struct {
  int64_t *start_us;  /* [S*A] tick at which the action started, -1 if it never did             */
  int64_t *finish_us; /* [S*A] start + getDur(units), -1                                         */
  int32_t *units;     /* [S*A]                                                                   */
  int32_t *node;      /* [S*A]                                                                   */
  double *mean_act_us; /* [S] mean of finish - arrival over started actions                      */
  int64_t *p99_act_us; /* [S] nearest-rank 99th percentile of the same, -1 if none started        */
  int32_t *n_started;  /* [S]                                                                    */
  int32_t *n_ticks;    /* [S] ticks simulated                                                    */
  uint64_t *core_set;  /* [S*A*4] cores of every started CPU action, as tg_assign_out.core_set; needed with
                          numa_cores > 0 (written completely), ignored otherwise                */
} tg_replay_out;

/*
 * tg_build_trace validates and packs a trace description like tg_build_problem does a problem
 * (same error codes; also TG_E_INVALID_ARG for arrivals that are not sorted, a GPU node that does
 * not have 8 GPUs, more tokens than the bucket holds, an unknown flag) and returns after its copy
 * to the device; the trace owns only that copy.  tg_replay_trace runs the replay of all S
 * scenarios: one launch computing Eq. 1 for every action, one persistent workgroup per scenario
 * (Sec. 4.2's step every tick, see above); all outputs are written completely.  d_ws: device
 * workspace of at least tg_replay_workspace_bytes(), 256-byte aligned, used by one replay at a
 * time.  Errors: TG_E_INVALID_ARG (a null output, core_set missing with numa_cores > 0),
 * TG_E_WORKSPACE, TG_E_RANGE (the node tables of a scenario do not fit the LDS of a compute
 * unit), TG_E_HIP.
 */
int tg_build_trace(const tg_trace_desc *desc, void *hip_stream, tg_trace **out);
void tg_free_trace(tg_trace *t);
int tg_replay_workspace_bytes(const tg_trace *t, size_t *bytes);
int tg_replay_trace(const tg_trace *t, const tg_replay_out *out, void *d_ws, size_t ws_bytes, void *hip_stream);
/*
 * The replay in pieces: a run can stop after any number of ticks and go on later, e.g. to look at the schedule in
 * between.  restart != 0: every scenario starts at time 0 (tg_replay_trace is restart = 1 with max_ticks ticks);
 * restart == 0: every scenario goes on where the last call on this workspace and these output buffers stopped -
 * both hold the whole state and must not have been touched in between (a workspace that does not carry the mark of
 * an earlier call on a trace of this shape is refused on the device: n_ticks of every scenario becomes -1 and nothing
 * else is written).  n_ticks >= 1: ticks of simulated time this
 * call advances every unfinished scenario by (never past max_ticks).  After every call the outputs are those of a
 * replay whose max_ticks is the tick reached: start / finish / units / node of the actions started so far, n_ticks
 * the tick reached (or the tick after the last start, if everything has started), the statistics over the actions
 * started so far.  Errors as tg_replay_trace; TG_E_INVALID_ARG for n_ticks < 1.
 */
int tg_replay_trace_part(const tg_trace *t, const tg_replay_out *out, void *d_ws, size_t ws_bytes, int restart, int n_ticks,
                         void *hip_stream);

/*
 * Capacities of the replay's buffers, for checking on the host (Sec. 4.2's step works on lists and
 * tables whose sizes change from tick to tick; the replay kernel sizes its local-memory blocks and
 * workspace slices once per trace).  tg_replay_capacity reads only the host arrays of `desc`
 * (node_type, node_cap and the scalar fields), touches no device and fills cap[TG_REPLAY_N_CAPS]
 * (host) with the largest value each quantity may take in a step of a scenario of this trace for
 * every index of the kernel to stay inside its block:
 *   WAIT_CPU / WAIT_GPU / WAIT_API   length of a kind's waiting list
 *   RUNNING                          running CPU and GPU actions
 *   CAND_CPU_ELASTIC / _GPU_ELASTIC  candidates on one CPU / GPU node that has an elastic candidate (rows of the
 *                                    duration, choice, best-total and allocation tables)
 *   CAND_NODE                        candidates on any one node (a quota's are bounded by its list only)
 *   CAND_STEP / PINNED_WAIT_STEP     candidates, and waiting actions pinned to a node, over all nodes of a step
 *   BUSY_UNITS                       units of the running actions of a node that has candidates
 *   HEAP_ENTRIES                     those plus the node's free units (Alg. 2's completion heap)
 *   CHUNK_STATES                     states of Alg. 4's table on one GPU node
 *   DP_CELLS                         cells of a row of Alg. 3's table: free units of a CPU node + 1
 *   NODES_CPU / _GPU / _API          nodes of a kind in one scenario
 * Errors: TG_E_INVALID_ARG, TG_E_RANGE (same conditions as tg_build_trace for the fields it reads, and a
 * scenario whose tables do not fit the local memory of a compute unit).
 */
enum { TG_REPLAY_CAP_WAIT_CPU = 0, TG_REPLAY_CAP_WAIT_GPU, TG_REPLAY_CAP_WAIT_API, TG_REPLAY_CAP_RUNNING,
       TG_REPLAY_CAP_CAND_CPU_ELASTIC, TG_REPLAY_CAP_CAND_GPU_ELASTIC, TG_REPLAY_CAP_CAND_NODE, TG_REPLAY_CAP_CAND_STEP,
       TG_REPLAY_CAP_PINNED_WAIT_STEP, TG_REPLAY_CAP_BUSY_UNITS, TG_REPLAY_CAP_HEAP_ENTRIES, TG_REPLAY_CAP_CHUNK_STATES,
       TG_REPLAY_CAP_DP_CELLS, TG_REPLAY_CAP_NODES_CPU, TG_REPLAY_CAP_NODES_GPU, TG_REPLAY_CAP_NODES_API,
       TG_REPLAY_N_CAPS };
int tg_replay_capacity(const tg_trace_desc *desc, int64_t *cap);

const char *tg_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* TG_H_ */
