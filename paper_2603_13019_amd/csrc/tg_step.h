// Wavefront-level building blocks of one scheduling step, shared by tg_assign (one snapshot
// per launch slot) and tg_replay_trace (one step per tick inside a persistent workgroup).
//
//   tg_place_pool      Alg. 1's admission of a queue prefix for one resource kind: in visiting order, at minimum units,
//                      with node choice by least estimated completion time (Eq. 2), node table in
//                      registers (pools of up to 1024 nodes) or LDS
//   tg_node_schedule   the rest of Alg. 1 for one node: DPArrange (Alg. 3; Alg. 4 chunk states on GPU
//                      nodes), completion-heap estimate (Alg. 2), greedy tail eviction
//
// Both are executed by ONE wavefront (64 lanes) with uniform control flow; `__syncthreads()`
// is only used by callers whose workgroup is that single wavefront, the functions themselves
// order their LDS traffic with tg_wave_sync().
#ifndef TG_STEP_H_
#define TG_STEP_H_

#include <type_traits>

#include "tg_internal.h"

#define TG_PAD INT64_MAX            // heap slot beyond the heap size
#define TG_MARK (INT64_MAX - 1)     // heap slot popped by the action being inserted

// All lanes of a wavefront run in lockstep and the LDS executes one wavefront's accesses in
// order; this only keeps the compiler from moving LDS accesses across the point where one
// lane's write must be seen by the others (no wait on outstanding global memory traffic).
__device__ static inline void tg_wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}

// Wavefront-wide unsigned 64-bit minimum, broadcast to all lanes.  Data-parallel-primitive
// moves inside the rows of 16 lanes (shift right by 1, 2, 4, 8: lane 15 of a row then holds the
// row's minimum because min is idempotent), then row 0 -> 1 and 2 -> 3 (broadcast of lane 15),
// then rows 0-1 -> 2-3 (broadcast of lane 31); lane 63 ends with the minimum of all 64.
__device__ static inline uint64_t tg_wave_min_u64(uint64_t v) {
  uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
#define TG_DPP_MIN_STEP(CTRL, ROWMASK)                                                                        \
  {                                                                                                           \
    const uint32_t lo2 = (uint32_t)__builtin_amdgcn_update_dpp((int)lo, (int)lo, CTRL, ROWMASK, 0xf, false);  \
    const uint32_t hi2 = (uint32_t)__builtin_amdgcn_update_dpp((int)hi, (int)hi, CTRL, ROWMASK, 0xf, false);  \
    const uint64_t w = (uint64_t)hi2 << 32 | lo2, c = (uint64_t)hi << 32 | lo;                                \
    if (w < c) { lo = lo2; hi = hi2; }                                                                        \
  }
  TG_DPP_MIN_STEP(0x111, 0xf) TG_DPP_MIN_STEP(0x112, 0xf) TG_DPP_MIN_STEP(0x114, 0xf) TG_DPP_MIN_STEP(0x118, 0xf)
  TG_DPP_MIN_STEP(0x142, 0xa) TG_DPP_MIN_STEP(0x143, 0xc)
#undef TG_DPP_MIN_STEP
  lo = (uint32_t)__builtin_amdgcn_readlane((int)lo, 63);
  hi = (uint32_t)__builtin_amdgcn_readlane((int)hi, 63);
  return (uint64_t)hi << 32 | lo;
}

// 32-bit variant: the minimum rides on the data-parallel-primitive move itself.
__device__ static inline uint32_t tg_wave_min_u32(uint32_t v) {
#define TG_DPP_MIN32_STEP(CTRL, ROWMASK)                                                                  \
  {                                                                                                       \
    const uint32_t w = (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)v, CTRL, ROWMASK, 0xf, false);      \
    v = w < v ? w : v;   /* lanes without a source see the identity of min */                             \
  }
  TG_DPP_MIN32_STEP(0x111, 0xf) TG_DPP_MIN32_STEP(0x112, 0xf) TG_DPP_MIN32_STEP(0x114, 0xf) TG_DPP_MIN32_STEP(0x118, 0xf)
  TG_DPP_MIN32_STEP(0x142, 0xa) TG_DPP_MIN32_STEP(0x143, 0xc)
#undef TG_DPP_MIN32_STEP
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Inclusive prefix sum across the wavefront on data-parallel-primitive moves: shifts by 1, 2, 4,
// 8 inside the rows of 16 lanes (lanes without a source add 0), then the total of row 0 into
// row 1 and of row 2 into row 3, then the total of rows 0-1 into rows 2-3.
__device__ static inline int tg_wave_scan_i32(int v) {
#define TG_DPP_ADD_STEP(CTRL, ROWMASK) v += __builtin_amdgcn_update_dpp(0, v, CTRL, ROWMASK, 0xf, false);
  TG_DPP_ADD_STEP(0x111, 0xf) TG_DPP_ADD_STEP(0x112, 0xf) TG_DPP_ADD_STEP(0x114, 0xf) TG_DPP_ADD_STEP(0x118, 0xf)
  TG_DPP_ADD_STEP(0x142, 0xa) TG_DPP_ADD_STEP(0x143, 0xc)
#undef TG_DPP_ADD_STEP
  return v;
}

__device__ static inline int tg_wave_sum_i32(int v) { return __builtin_amdgcn_readlane(tg_wave_scan_i32(v), TG_WAVE - 1); }

__device__ static inline int64_t tg_readlane_i64(int64_t v, int l) {
  const int lo = __builtin_amdgcn_readlane((int)(uint32_t)v, l);
  const int hi = __builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), l);
  return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

// Wavefront-wide 64-bit sum (same moves as the prefix sum above, both halves), in every lane.
__device__ static inline int64_t tg_wave_sum_i64(int64_t x) {
  uint64_t v = (uint64_t)x;
#define TG_DPP_ADD64_STEP(CTRL, ROWMASK)                                                                                  \
  {                                                                                                                       \
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, CTRL, ROWMASK, 0xf, false);            \
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), CTRL, ROWMASK, 0xf, false);    \
    v += (uint64_t)hi << 32 | lo;                                                                                         \
  }
  TG_DPP_ADD64_STEP(0x111, 0xf) TG_DPP_ADD64_STEP(0x112, 0xf) TG_DPP_ADD64_STEP(0x114, 0xf) TG_DPP_ADD64_STEP(0x118, 0xf)
  TG_DPP_ADD64_STEP(0x142, 0xa) TG_DPP_ADD64_STEP(0x143, 0xc)
#undef TG_DPP_ADD64_STEP
  return tg_readlane_i64((int64_t)v, TG_WAVE - 1);
}

// ---------------------------------------------------------------------------- placement
struct TgPoolLds {
  int64_t* back;     // [nodes] backlog
  int64_t* dur;      // [64*TG_MAX_K] duration rows of the 64 actions being processed
  int32_t* lim;      // [nodes] CPU/API: units left; GPU: packed counts of free chunks
  int32_t* cnt;      // [nodes] actions admitted to the node so far
  int32_t* dcnt;     // [nodes] waiting actions pinned to the node
  int32_t* aux;      // [nodes] second resource left on the node (only read when the actions carry a demand)
  uint64_t* res;     // [nodes] services resident on the node (only read when the actions call services)
  int32_t* k;        // [TG_MAX_K] unit counts
  uint8_t* closed;   // [nodes] the node's pool is closed (a pinned action did not fit)
  uint8_t* fit;      // [65] bit q set <=> k_list[q] <= min(units, 64)
};

__host__ __device__ static inline size_t tg_pool_lds_bytes(int nodes) {
  const size_t n = (size_t)((nodes + 7) & ~7);
  return n * 8 * 2 + 64 * TG_MAX_K * 8 + n * 4 * 4 + TG_MAX_K * 4 + n + 72;
}

__device__ static inline void tg_pool_lds_carve(unsigned char* smem, int nodes, TgPoolLds* S) {
  const size_t n = (size_t)((nodes + 7) & ~7);
  S->back = reinterpret_cast<int64_t*>(smem);
  S->res = reinterpret_cast<uint64_t*>(S->back + n);
  S->dur = S->back + 2 * n;
  S->lim = reinterpret_cast<int32_t*>(S->dur + 64 * TG_MAX_K);
  S->cnt = S->lim + n;
  S->dcnt = S->cnt + n;
  S->aux = S->dcnt + n;
  S->k = S->aux + n;
  S->closed = reinterpret_cast<uint8_t*>(S->k + TG_MAX_K);
  S->fit = S->closed + n;
}

struct TgPlaceIo {
  // per-action inputs, indexed by the action's id inside its snapshot / scenario
  const uint32_t* act_kmask;
  const uint8_t* act_static;
  const int32_t* act_pin;
  const int32_t* act_aux;      // demand for the node's second resource (charged to unpinned actions), or nullptr
  const int32_t* act_service;  // service the action calls (-1: none), or nullptr: no services
  const int64_t* restore;      // [service] restore time where the service is not resident (Sec. 5.3)
  const uint64_t* act_quota;   // further quotas of a pinned action (ranks < 64 inside this pool), or nullptr (Sec. 4.1)
  const int32_t* act_pin_rank; // rank of the action's pinned node inside its pool, -1: free or statically infeasible; or
                               // nullptr: derive it from act_pin and node_rank
  const int32_t* node_rank;    // node id -> rank inside this pool
  const int32_t* nodes;        // rank -> node id
  const int64_t* dur;          // [id*K + q]
  const int64_t* cost;         // optional block of the score tensor for this pool
  int cost_row_len;
  int K, Kt;
  // outputs
  int32_t* out_node; int32_t* out_units; int64_t* out_act; uint8_t* out_reason; int32_t* slot;
};

// Admission with the node table in registers: node r = lane + 64*s is slot s of its lane
// (Mt <= 64*R).  A lone wavefront is bound by the number of instructions it issues per action,
// so the loop is kept short: backlog (32-bit offsets where the pool's range allows), units
// left, the options those units admit (zero for a closed node) and the list lengths never
// leave the register file; what the loop needs of an action travels in one packed word and its
// result goes back into the action's lane as one word; an action pinned to a node has a
// single candidate and is handled with scalar code; with R = 1 the smallest rank among equal
// estimates is simply the lowest lane.  Same decisions as the LDS variant below.
template <int R, bool AUX, bool GPU>
__device__ static inline void tg_place_pool_regs(const TgPoolLds& S, const TgPlaceIo& io, const int32_t* acts, int Nt,
                                                 int Mt, int lane) {
  // the sizes are the same in every lane: keep the loop control on scalars
  Nt = __builtin_amdgcn_readfirstlane(Nt);
  Mt = __builtin_amdgcn_readfirstlane(Mt);
  bool pool_closed = false;
  tg_wave_sync();
  for (int u = lane; u <= TG_MAX_UNIT; u += TG_WAVE) {
    uint32_t f = 0;
    for (int q = 0; q < io.Kt; ++q) f |= (S.k[q] <= u ? 1u : 0u) << q;
    S.fit[u] = (uint8_t)f;
  }
  tg_wave_sync();
  uint32_t back32[R];                                             // backlog above the pool's smallest
  int32_t limv[R], cntv[R], dcntv[R];
  int32_t auxv[R];                                                // second resource left (Sec. 4.1's cost vector)
  uint64_t resv[R];                                               // services resident on the node (Sec. 5.3)
  const bool has_aux = AUX && io.act_aux, has_svc = AUX && io.act_service;   // AUX: the extended variant
  const bool has_x = AUX && io.act_quota;                         // actions that draw on several quotas (Sec. 4.1)
  uint32_t fitv[R];                                               // options that fit into the units left; 0: closed
  uint64_t closed[R];                                             // wavefront-uniform copies of the closed flags
  int64_t bmin = TG_INF, bmax = 0;
  auto fit_of = [&](int32_t lim) {
    const int u = GPU ? tg_chunk_largest((uint32_t)lim) : lim;
    return (uint32_t)S.fit[u < TG_MAX_UNIT ? u : TG_MAX_UNIT];
  };
  // the same table across the lanes (lane u: what fits into u units), for lookups with a
  // wavefront-uniform argument in the admission loop: one lane read instead of an LDS round trip
  const uint32_t fit_tab = S.fit[lane];
  const uint32_t fit_full = (uint32_t)__builtin_amdgcn_readfirstlane((int)S.fit[TG_MAX_UNIT]);
  auto fit_of_uniform = [&](int32_t lim) {
    const int u = GPU ? tg_chunk_largest((uint32_t)lim) : lim;
    return u >= TG_MAX_UNIT ? fit_full : (uint32_t)__builtin_amdgcn_readlane((int)fit_tab, u);
  };
#pragma unroll
  for (int s = 0; s < R; ++s) {
    const int r = lane + TG_WAVE * s;
    const bool have = r < Mt;
    const bool shut = have && S.closed[r] != 0;
    const int64_t bk = have ? S.back[r] : 0;
    limv[s] = have ? S.lim[r] : 0;
    fitv[s] = have && !shut ? fit_of(limv[s]) : 0u;
    cntv[s] = 0; dcntv[s] = 0;
    auxv[s] = has_aux && have ? S.aux[r] : INT32_MAX;
    resv[s] = has_svc && have ? S.res[r] : 0ull;
    closed[s] = __ballot(shut);
    if (have) { bmin = bk < bmin ? bk : bmin; bmax = bk > bmax ? bk : bmax; }
  }
  bmin = (int64_t)tg_wave_min_u64((uint64_t)bmin);
  bmax = (int64_t)~tg_wave_min_u64(~(uint64_t)bmax);
#pragma unroll
  for (int s = 0; s < R; ++s) { const int r = lane + TG_WAVE * s; back32[s] = r < Mt ? (uint32_t)(S.back[r] - bmin) : 0u; }   // meaningful where the range fits
  // result word of an action: rank + 1 (13 bits) | list slot (17 bits) | reason (2 bits)
  auto pack_res = [](int rank, int slot, int reason) { return (uint32_t)(rank + 1) | (uint32_t)slot << 13 | (uint32_t)reason << 30; };
  // What the loop needs of 64 actions is fetched one chunk ahead (and the action ids two chunks
  // ahead), lane l taking action base+l with its row of durations, so that the two dependent
  // global-memory round trips of a chunk run behind the admission of the chunk before it.
  struct Stage {
    int id, aux, svc, pin;
    int64_t x;
    uint32_t mask, stat;
    int64_t d[TG_MAX_K];
  };
  auto fetch_id = [&](int base) { return base + lane < Nt ? acts[base + lane] : 0; };
  auto fetch = [&](int base, int id, Stage& st) {
    st.id = id; st.aux = 0; st.svc = -1; st.pin = -1; st.x = 0; st.mask = 0; st.stat = 0;
#pragma unroll
    for (int q = 0; q < TG_MAX_K; ++q) st.d[q] = TG_INF;
    if (base + lane < Nt) {
      if (has_x) st.x = (int64_t)io.act_quota[id];
      if (has_aux) st.aux = io.act_aux[id];
      if (has_svc) st.svc = io.act_service[id];
      st.mask = io.act_kmask[id]; st.stat = io.act_static[id] ? 1u : 0u;
      st.pin = io.act_pin_rank ? io.act_pin_rank[id] : io.act_pin[id];
#pragma unroll
      for (int q = 0; q < TG_MAX_K; ++q) if (q < io.K) st.d[q] = io.dur[(size_t)id * io.K + q];
    }
  };
  // restore times across the lanes (lane s: service s), read with a uniform index in the loop
  const int64_t rest_tab = has_svc ? io.restore[lane] : 0;
  const int64_t rest_max = has_svc ? (int64_t)~tg_wave_min_u64(~(uint64_t)rest_tab) : 0;
  int next_id = fetch_id(0);
  Stage cur;
  fetch(0, next_id, cur);
  next_id = fetch_id(TG_WAVE);
  for (int base = 0; base < Nt; base += TG_WAVE) {
    const int cnt = min(TG_WAVE, Nt - base);
    // lane l holds action base+l: its inputs now (mask | static << 8 | minimum units << 9 |
    // (pinned rank + 1) << 16), its result after the loop
    const int my_id = cur.id, my_aux = cur.aux, my_svc = cur.svc;
    const int64_t my_x = cur.x;
    uint32_t my_w = 0, my_res = 0;
    if (lane < cnt) {
      const uint32_t mask = cur.mask, stat = cur.stat;
      int pr = cur.pin;
      if (!io.act_pin_rank) pr = pr >= 0 && !stat ? io.node_rank[pr] : -1;
      const uint32_t kmin = mask ? (uint32_t)S.k[__builtin_ctz(mask)] : 0u;
      my_w = (mask & 0xffu) | stat << 8 | kmin << 9 | (uint32_t)(pr + 1) << 16;
    }
    tg_wave_sync();                                  // previous chunk's readers are done with S.dur
    int64_t dmax = 0;
    if (lane < cnt) {
#pragma unroll
      for (int q = 0; q < TG_MAX_K; ++q)
        if (q < io.K) {
          const int64_t d = cur.d[q];
          S.dur[lane * io.K + q] = d;
          if (d != TG_INF && d > dmax) dmax = d;
        }
    }
    Stage nxt;                                       // in flight while this chunk is admitted
    fetch(base + TG_WAVE, next_id, nxt);
    next_id = fetch_id(base + 2 * TG_WAVE);
    dmax = (int64_t)~tg_wave_min_u64(~(uint64_t)dmax);
    if (has_svc) dmax += rest_max;                   // bound on duration + restore delay
    // every estimate of the chunk fits in 32 bits above the smallest backlog (durations included)
    const bool narrow = Mt > 0 && (bmax + dmax - bmin) < 0xfffffff0ll;
    const uint32_t* dur32 = reinterpret_cast<const uint32_t*>(S.dur);   // low words
    tg_wave_sync();
    for (int l = 0; l < cnt; ++l) {
      const uint32_t w = (uint32_t)__builtin_amdgcn_readlane((int)my_w, l);
      const uint32_t mask = w & 0xffu;
      const int kmin = (int)(w >> 9 & 0x7fu), pr = (int)(w >> 16) - 1;
      if (!AUX && narrow && !pool_closed && (w & 0xffff0100u) == 0) {
        // the common case in straight-line code: feasible, free to choose its node, 32-bit estimates
        uint32_t b32 = 0xffffffffu, brank = 0xffffffffu;
#pragma unroll
        for (int s = 0; s < R; ++s) {                 // ascending rank, strict <: the smaller rank wins ties
          const uint32_t ok = mask & fitv[s];         // allowed options that still fit
          const int qs = 31 - __builtin_clz(ok | 1u); // the largest of them
          const uint32_t d = dur32[2 * (l * io.K + qs)];   // read by every lane (option 0 where nothing fits): no branch
          const uint32_t e32 = ok ? back32[s] + d : 0xffffffffu;
          if (R > 1) { if (e32 < b32) { b32 = e32; brank = (uint32_t)(lane + TG_WAVE * s); } }
          else b32 = e32;
        }
        const uint32_t emin = tg_wave_min_u32(b32);
        int rank;
        if (R == 1) {
          const uint64_t who = __ballot(b32 == emin);
          rank = emin == 0xffffffffu ? -1 : __ffsll((unsigned long long)who) - 1;
        } else rank = (int)tg_wave_min_u32(b32 == emin ? brank : 0xffffffffu);     // -1: nobody fits
        uint32_t res = pack_res(-1, 0, TG_DEFER_PREFIX);
        if (rank < 0) pool_closed = true;
        else {
          const int rl = rank & 63;
          int slot = 0;
#pragma unroll
          for (int s = 0; s < R; ++s) {
            if ((rank >> 6) != s) continue;
            slot = __builtin_amdgcn_readlane(cntv[s], rl);
            const int32_t lim_old = __builtin_amdgcn_readlane(limv[s], rl);
            const int32_t lim_new = GPU ? (int32_t)tg_chunk_take((uint32_t)lim_old, kmin) : lim_old - kmin;
            const uint32_t fit_new = fit_of_uniform(lim_new);
            const bool me = lane == rl;
            cntv[s] = me ? slot + 1 : cntv[s];
            limv[s] = me ? lim_new : limv[s];
            fitv[s] = me ? fit_new : fitv[s];
          }
          res = pack_res(rank, slot, TG_SELECTED);
        }
        my_res = lane == l ? res : my_res;
        continue;
      }
      const int aux = has_aux && pr < 0 ? __builtin_amdgcn_readlane(my_aux, l) : 0;   // pinned: already charged
      const int svc = has_svc ? __builtin_amdgcn_readlane(my_svc, l) : -1;
      const int64_t rest = has_svc && svc >= 0 ? tg_readlane_i64(rest_tab, svc) : 0;
      const uint64_t more = has_x && pr >= 0 ? (uint64_t)tg_readlane_i64(my_x, l) : 0ull;   // ranks are lanes of slot 0
      uint32_t res;
      int take_rank = -1;                                          // node that admits the action
      if (w & 0x100u) {
        res = pack_res(-1, 0, TG_DEFER_INFEASIBLE);
      } else if (pr >= 0) {
        // pinned: one candidate, decided on scalars
        const int pl = pr & 63;
        uint64_t cw = 0;
        uint32_t f = 0;
        int dslot = 0;
#pragma unroll
        for (int s = 0; s < R; ++s) {
          if ((pr >> 6) != s) continue;
          cw = closed[s];
          f = (uint32_t)__builtin_amdgcn_readlane((int)fitv[s], pl);
          dslot = __builtin_amdgcn_readlane(dcntv[s], pl);
        }
        const bool open = !pool_closed && !(cw >> pl & 1ull);
        // every further quota must have a token left as well
        const bool more_ok = !AUX || more == 0 || (more & ~__ballot(limv[0] >= 1)) == 0;
        if (open && (mask & f) != 0 && more_ok) {
          take_rank = pr;
          res = 0;
        } else {
          if (open) {                                              // did not fit: the node's pool closes
#pragma unroll
            for (int s = 0; s < R; ++s) {
              if ((pr >> 6) != s) continue;
              closed[s] |= 1ull << pl;
              if (lane == pl) fitv[s] = 0;
            }
          }
#pragma unroll
          for (int s = 0; s < R; ++s) if ((pr >> 6) == s && lane == pl) ++dcntv[s];
          res = pack_res(-1, dslot, TG_DEFER_PREFIX);
        }
      } else if (pool_closed) {
        res = pack_res(-1, 0, TG_DEFER_PREFIX);
      } else {
        int rank;
        if (narrow) {
          uint32_t b32 = 0xffffffffu, brank = 0xffffffffu;
#pragma unroll
          for (int s = 0; s < R; ++s) {               // ascending rank, strict <: the smaller rank wins ties
            const uint32_t ok = !AUX || auxv[s] >= aux ? mask & fitv[s] : 0u;   // allowed options that still fit
            const int qs = 31 - __builtin_clz(ok | 1u);            // the largest of them
            uint32_t e32 = ok ? back32[s] + dur32[2 * (l * io.K + qs)] : 0xffffffffu;
            if (AUX && ok && svc >= 0 && !(resv[s] >> svc & 1ull)) e32 += (uint32_t)rest;   // restore first
            if (R > 1) { if (e32 < b32) { b32 = e32; brank = (uint32_t)(lane + TG_WAVE * s); } }
            else b32 = e32;
          }
          const uint32_t emin = tg_wave_min_u32(b32);
          if (R == 1) rank = emin == 0xffffffffu ? -1 : __ffsll((unsigned long long)__ballot(b32 == emin)) - 1;
          else rank = (int)tg_wave_min_u32(b32 == emin ? brank : 0xffffffffu);     // 0xffffffff: nobody fits
        } else {
          uint64_t b64 = ~0ull;
#pragma unroll
          for (int s = 0; s < R; ++s) {
            const uint32_t ok = !AUX || auxv[s] >= aux ? mask & fitv[s] : 0u;
            const int qs = 31 - __builtin_clz(ok | 1u);
            const int r = lane + TG_WAVE * s;                     // 64-bit estimates: backlog from the LDS table
            int64_t e = S.back[r < Mt ? r : 0] + S.dur[l * io.K + qs];
            if (AUX && svc >= 0 && !(resv[s] >> svc & 1ull)) e += rest;
            const uint64_t key = (uint64_t)e << 12 | (uint32_t)r;
            if (ok && key < b64) b64 = key;
          }
          b64 = tg_wave_min_u64(b64);
          rank = b64 == ~0ull ? -1 : (int)(b64 & 0xfff);
        }
        rank = __builtin_amdgcn_readfirstlane(rank);
        if (rank < 0) { pool_closed = true; res = pack_res(-1, 0, TG_DEFER_PREFIX); }
        else { take_rank = rank; res = 0; }
      }
      if (take_rank >= 0) {
        const int rl = take_rank & 63;
        int slot = 0;
#pragma unroll
        for (int s = 0; s < R; ++s) {
          if ((take_rank >> 6) != s) continue;
          slot = __builtin_amdgcn_readlane(cntv[s], rl);
          const int32_t lim_old = __builtin_amdgcn_readlane(limv[s], rl);      // the node's new state on scalars
          const int32_t lim_new = GPU ? (int32_t)tg_chunk_take((uint32_t)lim_old, kmin) : lim_old - kmin;
          const uint32_t fit_new = fit_of_uniform(lim_new);
          const bool me = lane == rl;                            // selects, no branch: one lane changes
          cntv[s] = me ? slot + 1 : cntv[s];
          if (AUX) auxv[s] = me ? auxv[s] - aux : auxv[s];
          limv[s] = me ? lim_new : limv[s];
          fitv[s] = me ? fit_new : fitv[s];
        }
        if (AUX && more != 0 && (more >> lane & 1ull)) {           // one token of every further quota
          limv[0] -= 1;
          if (!(closed[0] >> lane & 1ull)) fitv[0] = fit_of(limv[0]);
        }
        res = pack_res(take_rank, slot, TG_SELECTED);
      }
      if (lane == l) my_res = res;
    }
    if (lane < cnt) {
      const int res_rank = (int)(my_res & 0x1fffu) - 1, res_slot = (int)(my_res >> 13 & 0x1ffffu), res_reason = (int)(my_res >> 30);
      io.out_node[my_id] = res_rank >= 0 ? io.nodes[res_rank] : -1;
      io.out_reason[my_id] = (uint8_t)res_reason;
      io.slot[my_id] = res_slot;
      if (res_reason != TG_SELECTED) { io.out_units[my_id] = 0; if (io.out_act) io.out_act[my_id] = -1; }
    }
    cur = nxt;
  }
#pragma unroll
  for (int s = 0; s < R; ++s) {
    const int r = lane + TG_WAVE * s;
    if (r < Mt) { S.cnt[r] = cntv[s]; S.dcnt[r] = dcntv[s]; }
  }
  tg_wave_sync();
}

// Wavefront-wide OR of a small bit mask (data-parallel-primitive moves as in the minima above).
__device__ static inline uint32_t tg_wave_or_u32(uint32_t v) {
#define TG_DPP_OR_STEP(CTRL, ROWMASK) v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROWMASK, 0xf, false);
  TG_DPP_OR_STEP(0x111, 0xf) TG_DPP_OR_STEP(0x112, 0xf) TG_DPP_OR_STEP(0x114, 0xf) TG_DPP_OR_STEP(0x118, 0xf)
  TG_DPP_OR_STEP(0x142, 0xa) TG_DPP_OR_STEP(0x143, 0xc)
#undef TG_DPP_OR_STEP
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Admission of a pool in rounds instead of action by action - same decisions as the serial loop.
//
// Within one step the units left on a node only shrink and closed nodes stay closed, so for a
// given action the estimate of every node only rises (or the node drops out) as earlier actions
// are admitted.  Hence: if all 64 actions of a chunk decide at once on the table as it stands
// (lane = action), the decision of an action is the serial one as long as, after the admissions
// of the actions before it, (a) it is pinned and still fits its node, or (b) it is free and the
// node it chose still offers it the same largest option - every other node can only have become
// worse, and ties went to the smaller index already.  A round therefore decides all remaining
// actions of the chunk, finds for each the units taken from its node by the earlier ones (exact
// prefix sums per node), commits the longest prefix of actions whose decisions hold, and the next
// round starts at the first one that does not.  The first action of a round sees the true table,
// so every round commits at least one action; an action that closes something (a pinned action
// that does not fit closes its node, a free one with no candidate closes the pool) ends its round.
// On GPU nodes a chunk taken from a node changes its state in a way sums do not describe, so there
// only the first action of a round that touches a node is committed.
//
// The estimate of a free action on a node depends on the node only through its backlog and
// through which options still fit (a prefix of the option list: its "class"), so an action
// minimises over one representative per class - the node with the smallest (backlog, rank) - in
// at most K steps, instead of over all nodes; the representatives are recomputed only for
// classes whose membership changed.
//
// Needs: no second resource / services / further quotas, estimates recomputed (no score tensor),
// Mt <= 64 R, and all backlogs of the pool within 2^31 of the smallest (`bmin`).  The LDS arrays
// aux / res of S, unused without those options, serve as per-node counters.
template <int R, bool GPU>
__device__ static inline void tg_place_pool_rounds(const TgPoolLds& S, const TgPlaceIo& io, const int32_t* acts, int Nt,
                                                   int Mt, int lane) {
  enum { kNone = 0, kInfeasible, kPrefix, kWait, kMisfit, kNoFit, kAdmit };
  Nt = __builtin_amdgcn_readfirstlane(Nt);
  Mt = __builtin_amdgcn_readfirstlane(Mt);
  const int Kt = __builtin_amdgcn_readfirstlane(io.Kt);
  tg_wave_sync();
  for (int u = lane; u <= TG_MAX_UNIT; u += TG_WAVE) {
    uint32_t f = 0;
    for (int q = 0; q < Kt; ++q) f |= (S.k[q] <= u ? 1u : 0u) << q;
    S.fit[u] = (uint8_t)f;
  }
  int32_t* win_a = S.aux;                                         // admitted this round, per node
  int32_t* win_w = reinterpret_cast<int32_t*>(S.res);             // put on the waiting list this round, per node
  int64_t bmin = TG_INF;
  for (int r = lane; r < Mt; r += TG_WAVE) { win_a[r] = 0; win_w[r] = 0; const int64_t b = S.back[r]; bmin = b < bmin ? b : bmin; }
  bmin = (int64_t)tg_wave_min_u64((uint64_t)bmin);
  tg_wave_sync();
  auto fit_of = [&](int32_t lim) {
    const int u = GPU ? tg_chunk_largest((uint32_t)lim) : lim;
    return (uint32_t)S.fit[u < 0 ? 0 : u < TG_MAX_UNIT ? u : TG_MAX_UNIT];
  };
  uint32_t back32[R];
  int cls[R];                                                     // options that fit into what the node has left; 0: closed or full
#pragma unroll
  for (int s = 0; s < R; ++s) { const int r = lane + TG_WAVE * s; back32[s] = r < Mt ? (uint32_t)(S.back[r] - bmin) : 0u; cls[s] = -1; }
  uint64_t rep[TG_MAX_K + 1];                                     // per class: (backlog offset << 12 | rank) of its best node, ~0: empty
#pragma unroll
  for (int c = 0; c <= TG_MAX_K; ++c) rep[c] = ~0ull;
  bool pool_closed = false;
  auto pack_res = [](int rank, int slot, int reason) { return (uint32_t)(rank + 1) | (uint32_t)slot << 13 | (uint32_t)reason << 30; };
  const uint64_t lt_mask = (1ull << lane) - 1ull;

  struct Stage {
    int id, pin;
    uint32_t mask, stat;
    int64_t d[TG_MAX_K];
  };
  auto fetch_id = [&](int base) { return base + lane < Nt ? acts[base + lane] : 0; };
  auto fetch = [&](int base, int id, Stage& st) {
    st.id = id; st.pin = -1; st.mask = 0; st.stat = 0;
#pragma unroll
    for (int q = 0; q < TG_MAX_K; ++q) st.d[q] = TG_INF;
    if (base + lane < Nt) {
      st.mask = io.act_kmask[id]; st.stat = io.act_static[id] ? 1u : 0u;
      st.pin = io.act_pin_rank ? io.act_pin_rank[id] : io.act_pin[id];
#pragma unroll
      for (int q = 0; q < TG_MAX_K; ++q) if (q < io.K) st.d[q] = io.dur[(size_t)id * io.K + q];
    }
  };
  int next_id = fetch_id(0);
  Stage cur;
  fetch(0, next_id, cur);
  next_id = fetch_id(TG_WAVE);
  for (int base = 0; base < Nt; base += TG_WAVE) {
    const int cnt = min(TG_WAVE, Nt - base);
    const int my_id = cur.id;
    uint32_t mask = 0, stat = 0;
    int kmin = 0, pr = -1;
    if (lane < cnt) {
      mask = cur.mask & 0xffu; stat = cur.stat;
      pr = cur.pin;
      if (!io.act_pin_rank) pr = pr >= 0 && !stat ? io.node_rank[pr] : -1;
      kmin = mask ? S.k[__builtin_ctz(mask)] : 0;
    }
    tg_wave_sync();                                  // the previous chunk's readers are done with S.dur
    if (lane < cnt) {
#pragma unroll
      for (int q = 0; q < TG_MAX_K; ++q) if (q < io.K) S.dur[lane * io.K + q] = cur.d[q];
    }
    Stage nxt;                                       // in flight while this chunk is admitted
    fetch(base + TG_WAVE, next_id, nxt);
    next_id = fetch_id(base + 2 * TG_WAVE);
    tg_wave_sync();
    uint32_t my_res = 0;
    int f0 = 0;                                      // first action of the chunk that is not committed yet
    while (f0 < cnt) {
      // ---- the table as it stands: class of every node, representatives of the classes that changed
      uint32_t dirty = 0;
#pragma unroll
      for (int s = 0; s < R; ++s) {
        const int r = lane + TG_WAVE * s;
        int c = 0;
        if (r < Mt && !S.closed[r]) c = __builtin_popcount(fit_of(S.lim[r]));
        if (c != cls[s]) { dirty |= (cls[s] >= 0 ? 1u << cls[s] : 0u) | 1u << c; cls[s] = c; }
      }
      dirty = tg_wave_or_u32(dirty);
#pragma unroll
      for (int c = 1; c <= TG_MAX_K; ++c) {
        if (!(dirty >> c & 1u)) continue;
        uint64_t key = ~0ull;
#pragma unroll
        for (int s = 0; s < R; ++s) {
          const uint64_t k2 = (uint64_t)back32[s] << 12 | (uint32_t)(lane + TG_WAVE * s);
          if (cls[s] == c && k2 < key) key = k2;
        }
        rep[c] = tg_wave_min_u64(key);
      }
      // ---- every remaining action decides on this table
      const bool active = lane >= f0 && lane < cnt;
      int dec = kNone, node = -1;
      if (active) {
        if (stat) dec = kInfeasible;
        else if (pr >= 0) {
          const bool fits = (mask & fit_of(S.lim[pr])) != 0;
          if (pool_closed || S.closed[pr]) dec = kWait;
          else if (fits) { dec = kAdmit; node = pr; }
          else dec = kMisfit;
        } else if (pool_closed) dec = kPrefix;
        else {
          uint64_t best = ~0ull;
#pragma unroll
          for (int c = 1; c <= TG_MAX_K; ++c) {
            if (rep[c] == ~0ull) continue;                        // the same in all lanes
            const uint32_t ok = mask & ((1u << c) - 1u);
            if (ok == 0) continue;
            const uint64_t e = (rep[c] >> 12) + (uint64_t)S.dur[lane * io.K + (31 - __builtin_clz(ok))];
            const uint64_t key = e << 12 | (rep[c] & 0xfffull);
            best = key < best ? key : best;
          }
          if (best == ~0ull) dec = kNoFit;
          else { dec = kAdmit; node = (int)(best & 0xfffull); }
        }
      }
      // ---- for actions that enter a list: how many of the earlier ones enter the same list, and the units they take
      const bool waits = dec == kWait || dec == kMisfit;
      const bool listed = dec == kAdmit || waits;
      const int lkey = dec == kAdmit ? node : waits ? pr + 4096 : -1;   // list identity
      int32_t* win = dec == kAdmit ? win_a + node : win_w + (waits ? pr : 0);
      if (listed) atomicAdd(win, 1);
      tg_wave_sync();
      const int shared = listed ? *win : 0;
      tg_wave_sync();
      if (listed) *win = 0;
      int rank = 0, before = 0;
      for (uint64_t todo = __ballot(shared > 1); todo;) {
        const int k0 = __builtin_amdgcn_readlane(lkey, __builtin_ctzll(todo));
        const bool in = lkey == k0;
        const uint64_t m = __ballot(in);
        if (in) rank = __popcll(m & lt_mask);
        if (!GPU && k0 < 4096) {                                  // units taken from the node by the earlier ones
          const int inc = tg_wave_scan_i32(in ? kmin : 0);
          if (in) before = inc - kmin;
        }
        todo &= ~m;
      }
      // ---- which decisions hold after the earlier actions of the round
      bool valid = true;
      int lim_n = 0;
      if (dec == kAdmit) {
        lim_n = S.lim[node];
        if (GPU) valid = rank == 0;
        else {
          const uint32_t fo = mask & fit_of(lim_n), fn = mask & fit_of(lim_n - before);
          valid = fn != 0 && (pr >= 0 || (31 - __builtin_clz(fn)) == (31 - __builtin_clz(fo | 1u)));
        }
      }
      const uint64_t bad = __ballot(active && !valid), ends = __ballot(dec == kMisfit || dec == kNoFit);
      int f = cnt;
      if (bad) f = __builtin_ctzll(bad);
      if (ends) f = min(f, __builtin_ctzll(ends) + 1);
      // ---- commit actions f0 .. f-1
      const bool commit = active && lane < f;
      int slot = 0;
      if (commit && dec == kAdmit) slot = S.cnt[node] + rank;
      if (commit && waits) slot = S.dcnt[pr] + rank;
      tg_wave_sync();                                             // every list length read before any is changed
      if (commit) {
        if (dec == kAdmit) {
          atomicAdd(&S.cnt[node], 1);
          if (GPU) S.lim[node] = (int32_t)tg_chunk_take((uint32_t)lim_n, kmin);
          else atomicSub(&S.lim[node], kmin);
          my_res = pack_res(node, slot, TG_SELECTED);
        } else if (waits) {
          atomicAdd(&S.dcnt[pr], 1);
          if (dec == kMisfit) S.closed[pr] = 1;
          my_res = pack_res(-1, slot, TG_DEFER_PREFIX);
        } else my_res = pack_res(-1, 0, dec == kInfeasible ? TG_DEFER_INFEASIBLE : TG_DEFER_PREFIX);
      }
      if (__ballot(commit && dec == kNoFit)) pool_closed = true;
      tg_wave_sync();
      f0 = f;
    }
    if (lane < cnt) {
      const int res_rank = (int)(my_res & 0x1fffu) - 1, res_slot = (int)(my_res >> 13 & 0x1ffffu), res_reason = (int)(my_res >> 30);
      io.out_node[my_id] = res_rank >= 0 ? io.nodes[res_rank] : -1;
      io.out_reason[my_id] = (uint8_t)res_reason;
      io.slot[my_id] = res_slot;
      if (res_reason != TG_SELECTED) { io.out_units[my_id] = 0; if (io.out_act) io.out_act[my_id] = -1; }
    }
    cur = nxt;
  }
  tg_wave_sync();
}

// The loop specialised on whether the pool's units are buddy chunks (GPU) or plain counts.
template <int R, bool AUX>
__device__ static inline void tg_place_pool_regs_kind(const TgPoolLds& S, const TgPlaceIo& io, const int32_t* acts, int Nt,
                                                      int Mt, bool gpu, int lane) {
  if (gpu) tg_place_pool_regs<R, AUX, true>(S, io, acts, Nt, Mt, lane);
  else tg_place_pool_regs<R, AUX, false>(S, io, acts, Nt, Mt, lane);
}

// Admission of the pool's `Nt` actions (ids acts[0..Nt) in FCFS order) onto its `Mt` nodes.
// On return S.cnt / S.dcnt hold the list lengths per node and every action has its reason,
// node (-1 if deferred) and list slot written.
// MAXR: the widest register variant the caller wants compiled in (0: none, 1, 4 or 16 slots per
// lane); MAXR_EXT: the same for the extended variant, taken when the caller passes a second
// resource (io.act_aux), services (io.act_service) or further quotas (io.act_quota).  Pools no
// compiled variant takes use the LDS table below; LDS_TABLE = false leaves that path out for
// callers whose pools always fit a compiled variant (the register allocation of a kernel is
// shared by everything inlined into it, so a kernel does better with only the variants it runs).
template <int MAXR = 4, int MAXR_EXT = 0, bool LDS_TABLE = true>
__device__ static inline void tg_place_pool(const TgPoolLds& S, const TgPlaceIo& io, const int32_t* acts, int Nt,
                                            int Mt, bool gpu, int lane) {
  if (!io.cost && Mt <= 16 * TG_WAVE) {
    const int slots = Mt <= TG_WAVE ? 1 : Mt <= 4 * TG_WAVE ? 4 : 16;
    const bool ext = io.act_aux || io.act_service || io.act_quota;
    if constexpr (MAXR_EXT >= 1) {
      if (ext && slots <= MAXR_EXT) {
        if (slots == 1) tg_place_pool_regs_kind<1, true>(S, io, acts, Nt, Mt, gpu, lane);
        if constexpr (MAXR_EXT >= 4) { if (slots == 4) tg_place_pool_regs_kind<4, true>(S, io, acts, Nt, Mt, gpu, lane); }
        if constexpr (MAXR_EXT >= 16) { if (slots == 16) tg_place_pool_regs_kind<16, true>(S, io, acts, Nt, Mt, gpu, lane); }
        return;
      }
    }
    if constexpr (MAXR >= 1) {
      if (!ext && slots <= MAXR) {
        if (slots == 1) tg_place_pool_regs_kind<1, false>(S, io, acts, Nt, Mt, gpu, lane);
        if constexpr (MAXR >= 4) { if (slots == 4) tg_place_pool_regs_kind<4, false>(S, io, acts, Nt, Mt, gpu, lane); }
        if constexpr (MAXR >= 16) { if (slots == 16) tg_place_pool_regs_kind<16, false>(S, io, acts, Nt, Mt, gpu, lane); }
        return;
      }
    }
  }
  if constexpr (!LDS_TABLE) return;
  bool pool_closed = false;
  // which options fit into `units` units, for units = 0..64 (every unit count is <= 64)
  tg_wave_sync();
  for (int u = lane; u <= TG_MAX_UNIT; u += TG_WAVE) {
    uint32_t f = 0;
    for (int q = 0; q < io.Kt; ++q) f |= (S.k[q] <= u ? 1u : 0u) << q;
    S.fit[u] = (uint8_t)f;
  }
  // range of the backlogs: with the largest duration of a chunk it tells whether the chunk's
  // estimates fit in 32 bits above the smallest backlog (then the argmin runs on 32-bit keys)
  int64_t bmin = TG_INF, bmax = 0;
  for (int r = lane; r < Mt; r += TG_WAVE) { const int64_t b = S.back[r]; bmin = b < bmin ? b : bmin; bmax = b > bmax ? b : bmax; }
  bmin = (int64_t)tg_wave_min_u64((uint64_t)bmin);
  bmax = (int64_t)~tg_wave_min_u64(~(uint64_t)bmax);
  for (int base = 0; base < Nt; base += TG_WAVE) {
    const int cnt = min(TG_WAVE, Nt - base);
    // lane l holds action base+l: its inputs now, its result after the loop (one global
    // round trip per 64 actions instead of one per action)
    int my_id = 0, my_pr = -1, my_aux = 0, my_svc = -1;
    int64_t my_rest = 0;
    uint32_t my_mask = 0, my_static = 0;
    int64_t my_x = 0;
    if (lane < cnt) {
      my_id = acts[base + lane];
      if (io.act_quota) my_x = (int64_t)io.act_quota[my_id];
      my_mask = io.act_kmask[my_id]; my_static = io.act_static[my_id];
      const int pin = io.act_pin[my_id];
      if (pin >= 0 && !my_static) my_pr = io.node_rank[pin];
      if (io.act_aux) my_aux = io.act_aux[my_id];
      if (io.act_service) { my_svc = io.act_service[my_id]; if (my_svc >= 0) my_rest = io.restore[my_svc]; }
    }
    int res_rank = -1, res_slot = 0, res_reason = TG_SELECTED;
    tg_wave_sync();                                  // previous chunk's readers are done with S.dur
    int64_t dmax = 0;
    for (int x = lane; x < cnt * io.K; x += TG_WAVE) {
      const int a = x / io.K, q = x - a * io.K;
      const int64_t d = io.dur[(size_t)acts[base + a] * io.K + q];
      S.dur[x] = d;
      if (d != TG_INF && d > dmax) dmax = d;
    }
    dmax = (int64_t)~tg_wave_min_u64(~(uint64_t)dmax);
    if (io.act_service) dmax += (int64_t)~tg_wave_min_u64(~(uint64_t)my_rest);   // bound on duration + restore delay
    const bool narrow = !io.cost && Mt > 0 && (bmax + dmax - bmin) < 0xfffffff0ll;
    tg_wave_sync();
    for (int l = 0; l < cnt; ++l) {
      const uint32_t mask = (uint32_t)__builtin_amdgcn_readlane((int)my_mask, l);
      const int pr = __builtin_amdgcn_readlane(my_pr, l);
      const int stat = __builtin_amdgcn_readlane((int)my_static, l);
      const int aux = io.act_aux && pr < 0 ? __builtin_amdgcn_readlane(my_aux, l) : 0;   // pinned: already charged
      const int svc = io.act_service ? __builtin_amdgcn_readlane(my_svc, l) : -1;
      const int64_t rest = io.act_service ? tg_readlane_i64(my_rest, l) : 0;
      const uint64_t more = io.act_quota && pr >= 0 ? (uint64_t)tg_readlane_i64(my_x, l) : 0ull;   // further quotas, ranks < 64
      int reason = TG_SELECTED, rank = -1, slot = 0;
      if (stat) {
        reason = TG_DEFER_INFEASIBLE;
      } else if (pool_closed || (pr >= 0 && S.closed[pr])) {
        reason = TG_DEFER_PREFIX;
      } else {
        const int kmin = S.k[__builtin_ctz(mask)];
        // every further quota must have a token left as well, else the action does not fit
        const bool more_ok = more == 0 || (more & ~__ballot(lane < Mt && S.lim[lane < Mt ? lane : 0] >= 1)) == 0;
        const int r_lo = pr >= 0 ? pr : lane, r_hi = !more_ok ? 0 : pr >= 0 ? (lane == 0 ? pr + 1 : 0) : Mt;
        // this lane's best node: least estimate, smallest rank on ties (ranks ascend in the loop)
        uint32_t b32 = 0xffffffffu, brank = 0xffffffffu;
        uint64_t b64 = ~0ull;
        for (int r = r_lo; r < r_hi; r += TG_WAVE) {
          if (S.closed[r]) continue;
          if (aux > 0 && S.aux[r] < aux) continue;                                    // second resource exhausted
          const int lim = gpu ? tg_chunk_largest((uint32_t)S.lim[r]) : S.lim[r];
          const uint32_t ok = mask & S.fit[lim < TG_MAX_UNIT ? lim : TG_MAX_UNIT];   // allowed options that still fit
          if (ok == 0) continue;                                                      // not even the minimum units
          const int qs = 31 - __builtin_clz(ok);                                      // the largest of them
          const int64_t delay = svc >= 0 && !(S.res[r] >> svc & 1ull) ? rest : 0;     // restore the service first
          if (narrow) {
            const uint32_t e = (uint32_t)(S.back[r] + S.dur[l * io.K + qs] + delay - bmin);
            if (e < b32) { b32 = e; brank = (uint32_t)r; }
          } else {
            const int64_t e = io.cost ? io.cost[(size_t)(base + l) * io.cost_row_len + r * io.Kt + qs]
                                      : S.back[r] + S.dur[l * io.K + qs] + delay;
            const uint64_t key = (uint64_t)e << 12 | (uint32_t)r;
            b64 = key < b64 ? key : b64;
          }
        }
        if (narrow) {
          const uint32_t emin = tg_wave_min_u32(b32);
          rank = (int)tg_wave_min_u32(b32 == emin ? brank : 0xffffffffu);             // 0xffffffff: nobody fits
        } else {
          b64 = tg_wave_min_u64(b64);
          rank = b64 == ~0ull ? -1 : (int)(b64 & 0xfff);
        }
        if (rank < 0) {
          reason = TG_DEFER_PREFIX;
          if (pr >= 0) { if (lane == 0) S.closed[pr] = 1; } else pool_closed = true;
        } else {
          slot = S.cnt[rank];
          if (lane == 0) {
            S.cnt[rank] = slot + 1;
            if (aux > 0) S.aux[rank] -= aux;
            S.lim[rank] = gpu ? (int32_t)tg_chunk_take((uint32_t)S.lim[rank], kmin) : S.lim[rank] - kmin;
          }
          if (more >> lane & 1ull) S.lim[lane] -= 1;              // one token of every further quota
        }
      }
      if (reason == TG_DEFER_PREFIX && pr >= 0) {
        slot = S.dcnt[pr];
        if (lane == 0) S.dcnt[pr] = slot + 1;
      }
      if (lane == l) { res_rank = rank; res_slot = slot; res_reason = reason; }
      tg_wave_sync();
    }
    if (lane < cnt) {
      io.out_node[my_id] = res_rank >= 0 ? io.nodes[res_rank] : -1;
      io.out_reason[my_id] = (uint8_t)res_reason;
      io.slot[my_id] = res_slot;
      if (res_reason != TG_SELECTED) { io.out_units[my_id] = 0; if (io.out_act) io.out_act[my_id] = -1; }
    }
  }
  tg_wave_sync();
}

// Whole-queue prefix (Alg. 1 as printed): how many actions of a pool's list come before place
// `lim` of the whole queue's visiting order.  The list ascends in that order (gkey: the places
// under TG_ORDER_COST, else the action id is the place), so the count is found by bisection.
__device__ static inline int tg_prefix_len(const int32_t* acts, int Nt, const uint64_t* gkey, uint64_t lim) {
  int lo = 0, hi = Nt;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    const int id = acts[mid];
    const uint64_t k = gkey ? gkey[id] : (uint64_t)id;
    if (k < lim) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// The actions acts[n_adm .. Nt) lie behind the end of the admitted prefix: they wait (or can
// never run), and those pinned to a node join its waiting list behind the ones tg_place_pool
// has put there.
__device__ static inline void tg_place_tail(const TgPoolLds& S, const TgPlaceIo& io, const int32_t* acts, int n_adm, int Nt,
                                            int lane) {
  for (int base = n_adm; base < Nt; base += TG_WAVE) {
    const int cnt = min(TG_WAVE, Nt - base);
    int id = 0, pr = -1, stat = 1;
    if (lane < cnt) {
      id = acts[base + lane];
      stat = (int)io.act_static[id];
      const int pin = io.act_pin[id];
      if (pin >= 0 && !stat) pr = io.node_rank[pin];
    }
    int slot = 0;
    for (uint64_t pinned = __ballot(pr >= 0); pinned; pinned &= pinned - 1) {   // one after the other: the lists keep the visiting order
      const int l = __builtin_ctzll(pinned);
      const int r = __builtin_amdgcn_readlane(pr, l);
      const int s = S.dcnt[r];
      if (lane == l) slot = s;
      tg_wave_sync();
      if (lane == 0) S.dcnt[r] = s + 1;
      tg_wave_sync();
    }
    if (lane < cnt) {
      io.out_node[id] = -1;
      io.out_reason[id] = (uint8_t)(stat ? TG_DEFER_INFEASIBLE : TG_DEFER_PREFIX);
      io.slot[id] = slot; io.out_units[id] = 0;
      if (io.out_act) io.out_act[id] = -1;
    }
  }
  tg_wave_sync();
}

// List extents per node after tg_place_pool: exclusive scan of the per-node counts in rank
// order, starting at `a0` (the pool's first slot in the order arrays).
__device__ static inline void tg_pool_extents(const TgPoolLds& S, const int32_t* nodes, int Mt, int a0, int32_t* nl_off,
                                              int32_t* nl_cnt, int32_t* dl_off, int32_t* dl_cnt, int lane) {
  int run = a0, drun = a0;
  for (int base = 0; base < Mt; base += TG_WAVE) {
    const int r = base + lane;
    const int c = r < Mt ? S.cnt[r] : 0, dc = r < Mt ? S.dcnt[r] : 0;
    const int inc = tg_wave_scan_i32(c), dinc = tg_wave_scan_i32(dc);
    if (r < Mt) {
      const int g = nodes[r];
      nl_off[g] = run + inc - c; nl_cnt[g] = c;
      dl_off[g] = drun + dinc - dc; dl_cnt[g] = dc;
    }
    run += __builtin_amdgcn_readlane(inc, TG_WAVE - 1);
    drun += __builtin_amdgcn_readlane(dinc, TG_WAVE - 1);
  }
}

// ---------------------------------------------------------------------------- per node
// Choice table of the units DP: 4 bits per cell (option index, 0xf: unreachable); byte p of a
// row holds cells 2p+1 (low) and 2p+2 (high); cell 0 is unreachable in every row but the empty
// one and is not stored.
__host__ __device__ static inline int tg_choice_stride(int n) { return (n + 1) >> 1; }
__device__ static inline int tg_sel_get(const uint8_t* row, int x) {   // allocation table: candidate x of a row
  const int b = row[x >> 1];
  return x & 1 ? b >> 4 : b & 0xf;
}
__device__ static inline int tg_choice_get(const uint8_t* row, int j) {
  const int b = row[(j - 1) >> 1];
  return (j - 1) & 1 ? b >> 4 : b & 0xf;
}

struct TgNodeLdsPlan {
  int off_cdur, off_dp, off_choice, off_heap, off_rowbest, off_rowarg, off_sel, off_k;
  int dp_width;     // entries per DP row
  int sel_stride;   // bytes per row of the allocation table (two candidates per byte)
  int sel_rows;     // prefix lengths backtracked per batch (<= 64)
  int off_F;        // objectives of one round of evaluations + flags
  int off_q0;       // minimum-unit option of every candidate
  int cand_rows;    // candidates the per-candidate tables hold.  Nodes whose actions are elastic never have more (a
                    // candidate takes at least one of the node's free units); a quota may, its actions are never elastic
  int heap_slots;   // heap entries
  int off_wd, off_wu, wait_slots;   // minimum-unit duration and unit count of the first waiting actions pinned to the node
  int total;        // bytes per wavefront
};

// LDS layout of one wavefront for CPU and GPU nodes with at most `m_cap` candidates (m never
// exceeds the node's free units either).  Quotas can hold more candidates than that: their
// actions are not elastic, so they need none of the tables.
__host__ static inline TgNodeLdsPlan tg_node_lds_plan(int max_free_cpu, int max_free_gpu, int max_states, int max_heap, int K,
                                                      int m_cap = 1 << 30, int sel_rows = TG_WAVE,
                                                      int wait_slots = TG_WAVE) {
  TgNodeLdsPlan p;
  const int m_cpu = max_free_cpu < m_cap ? max_free_cpu : m_cap, m_gpu = max_free_gpu < m_cap ? max_free_gpu : m_cap;
  const int mmax = (m_cpu > m_gpu ? m_cpu : m_gpu) + 1;
  const int width = (max_free_cpu + 1 > max_states ? max_free_cpu + 1 : max_states);
  size_t choice = (size_t)m_cpu * tg_choice_stride(max_free_cpu);
  if ((size_t)m_gpu * max_states * 2 > choice) choice = (size_t)m_gpu * max_states * 2;
  size_t off = 0;
  auto take = [&](size_t b) { const size_t r = off; off += (b + 15) & ~size_t(15); return (int)r; };
  p.cand_rows = mmax;
  p.off_cdur = take((size_t)mmax * K * 8);
  const size_t dp64 = (size_t)width * 2 * 8, dp32 = (size_t)(width + 2 + TG_WAVE) * 2 * 4;   // 32-bit rows carry sentinels
  size_t dp = dp64 > dp32 ? dp64 : dp32;
  p.heap_slots = (max_heap + 2) & ~1;
  const size_t heap = (size_t)p.heap_slots * 8;
  // the wavefront fills the DP rows first and stages heaps only afterwards: one block serves both
  if (heap > dp) dp = heap;
  p.off_dp = take(dp);
  p.off_choice = take(choice + 16);
  p.off_heap = p.off_dp;
  p.off_F = take(5 * 8);
  p.off_q0 = take((size_t)mmax);
  p.off_rowbest = take((size_t)(mmax + 1) * 8);
  p.off_rowarg = take((size_t)(mmax + 1) * 4);
  p.sel_stride = (mmax + 1) >> 1;               // 4 bits per candidate
  p.off_sel = take((size_t)p.sel_stride * sel_rows);    // allocations of sel_rows consecutive prefix lengths
  p.sel_rows = sel_rows;
  p.off_k = take(TG_MAX_K * 4);
  p.wait_slots = wait_slots;
  p.off_wd = take((size_t)wait_slots * 8);
  p.off_wu = take((size_t)wait_slots);
  p.dp_width = width;
  p.total = (int)off;
  return p;
}

struct TgNodeIn {
  int type, cap, free_units;
  int64_t backlog;
  uint32_t chunks;
  int m; const int32_t* clist;       // admitted actions of the node, FCFS
  int nd; const int32_t* dlist;      // waiting actions pinned to the node, FCFS
  int n_busy; const int64_t* busy;   // release times of the units of running actions (global memory), or
  int busy_lds_off;                  // >= 0: the list sits at this byte offset of the wavefront's LDS block instead
  const uint8_t* act_model; const uint32_t* act_kmask; const int64_t* dur;
  int K, depth;
  uint64_t kword;                    // the unit counts k_list[0..8), one byte each
  // services (Sec. 5.3); act_service == nullptr: none
  const int32_t* act_service; const int64_t* restore;
  uint64_t resident;                 // services resident on this node, one bit each
};

// Delay of an action on this node: the restore time of its service where the service is not
// resident in the node's device memory (Sec. 5.3), else nothing.
__device__ static inline int64_t tg_restore_delay(const TgNodeIn& in, int id) {
  if (!in.act_service) return 0;
  const int sv = in.act_service[id];
  return sv >= 0 && !(in.resident >> sv & 1ull) ? in.restore[sv] : 0;
}

struct TgNodeOut {
  int32_t* node; int32_t* units; int64_t* act; uint8_t* reason;
  const int64_t* age;
};

// Waiting actions pinned to the node, as Alg. 2 sees them: duration on the minimum units and
// that unit count (0: can never run here, left out) of the first `slots` of them, in LDS.
struct TgWaitLds {
  const int64_t* d; const uint8_t* u; int slots;
};

// ---------------------------------------------------------------------------- Alg. 2 heaps
// The completion heap of Alg. 2 (one entry per unit of the node: when it frees) lives in the
// registers of the wavefront.  An action that takes u units removes the u earliest entries,
// starts when the last of them frees and puts u copies of its finish time back.
//
// TgHeapSorted<NS>: 32-bit times, kept sorted ascending across the wavefront (element
// s*64 + lane sits in h[s]; unused positions hold the pad value at the end).  The u earliest
// entries are then simply the first u, and re-inserting a finish time is a shift by one lane
// (a single data-parallel-primitive move per 64 entries) followed by a max and a min - instead
// of a wavefront-wide minimum per unit.
// The initial entries are sorted once per estimate by a bitonic network.
template <int NS>
struct TgHeapSorted {
  typedef uint32_t V;
  static constexpr int kSlots = NS;
  static constexpr uint32_t kPad = 0xffffffffu;

  __device__ static inline void load(V (&h)[NS], const int64_t* s_heap, int H, int64_t lo, int lane) {
#pragma unroll
    for (int s = 0; s < NS; ++s) { const int idx = lane + TG_WAVE * s; h[s] = idx < H ? (V)(uint64_t)(s_heap[idx] - lo) : kPad; }
#pragma unroll
    for (int k = 2; k <= TG_WAVE * NS; k <<= 1) {
#pragma unroll
      for (int j = k >> 1; j > 0; j >>= 1) {
        if (j >= TG_WAVE) {                                       // partner in another slot of the same lane
#pragma unroll
          for (int s = 0; s < NS; ++s) {
            const int t = s ^ (j >> 6);
            if (t > s) {
              const bool asc = ((s * TG_WAVE) & k) == 0;
              const V lo2 = h[s] < h[t] ? h[s] : h[t], hi2 = h[s] < h[t] ? h[t] : h[s];
              h[s] = asc ? lo2 : hi2; h[t] = asc ? hi2 : lo2;
            }
          }
        } else {                                                  // partner lane ^ j of the same slot
#pragma unroll
          for (int s = 0; s < NS; ++s) {
            const V o = (V)__shfl_xor((int)h[s], j);
            const int idx = s * TG_WAVE + lane;
            const bool keep_min = ((idx & j) == 0) == ((idx & k) == 0);
            const V lo2 = h[s] < o ? h[s] : o, hi2 = h[s] < o ? o : h[s];
            h[s] = keep_min ? lo2 : hi2;
          }
        }
      }
    }
  }

  // One unit leaves and one copy of `fin` (later than the u earliest entries) enters: with
  // sh[i] = h[i+1], the new sorted sequence is min(sh[i], max(h[i], fin)) - below the insertion
  // point the entries move down one place, at it max() yields fin, above it nothing changes.
  // Repeating the step u times removes the u earliest entries and inserts u copies.
  __device__ static inline V take(V (&h)[NS], int u, V dd, int lane) {
    const V fin = (V)__builtin_amdgcn_readlane((int)h[0], u - 1) + dd;   // u <= 64; starts when its last unit frees
    for (int c = 0; c < u; ++c) {
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const V nxt = s + 1 < NS ? (V)__builtin_amdgcn_readlane((int)h[s + 1 < NS ? s + 1 : s], 0) : kPad;
        const V sh = (V)__builtin_amdgcn_update_dpp((int)nxt, (int)h[s], 0x130, 0xf, 0xf, false);   // lane i <- lane i+1, lane 63 <- nxt
        const V hi = h[s] > fin ? h[s] : fin;
        h[s] = sh < hi ? sh : hi;
      }
    }
    return fin;
  }

  // The same action on D heaps at once (the depths of Alg. 2 side by side): one loop over its units, the D
  // independent chains inside it, so that their dependent instructions overlap.
  template <int D>
  __device__ static inline void take_all(V (&h)[D][NS], int u, V dd, int lane, uint64_t (&obj)[D]) {
    V fin[D];
#pragma unroll
    for (int k = 0; k < D; ++k) fin[k] = (V)__builtin_amdgcn_readlane((int)h[k][0], u - 1) + dd;
    for (int c = 0; c < u; ++c) {
#pragma unroll
      for (int k = 0; k < D; ++k)
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          const V nxt = s + 1 < NS ? (V)__builtin_amdgcn_readlane((int)h[k][s + 1 < NS ? s + 1 : s], 0) : kPad;
          const V sh = (V)__builtin_amdgcn_update_dpp((int)nxt, (int)h[k][s], 0x130, 0xf, 0xf, false);
          const V hi = h[k][s] > fin[k] ? h[k][s] : fin[k];
          h[k][s] = sh < hi ? sh : hi;
        }
    }
#pragma unroll
    for (int k = 0; k < D; ++k) obj[k] += (uint64_t)fin[k];
  }
};

// TgHeapWide: 64-bit times, unsorted, four slots per lane; a unit is found by a wavefront-wide
// minimum.  Only nodes whose times do not fit in 32 bits above their earliest one use it.
struct TgHeapWide {
  typedef uint64_t V;
  static constexpr int kSlots = 4;
  static constexpr uint64_t kPad = ~0ull, kMark = ~0ull - 1;

  __device__ static inline void load(V (&h)[4], const int64_t* s_heap, int H, int64_t, int lane) {
#pragma unroll
    for (int s = 0; s < 4; ++s) { const int idx = lane + TG_WAVE * s; h[s] = idx < H ? (V)s_heap[idx] : kPad; }
  }

  __device__ static inline V take(V (&h)[4], int u, V dd, int lane) {
    V start = 0;
    for (int c = 0; c < u; ++c) {                                 // pop the u earliest units
      V lm = h[0];
      int ls = 0;
#pragma unroll
      for (int s = 1; s < 4; ++s) if (h[s] < lm) { lm = h[s]; ls = s; }
      const V wm = tg_wave_min_u64(lm);
      const int owner = __ffsll((unsigned long long)__ballot(lm == wm)) - 1;
      if (lane == owner) {
#pragma unroll
        for (int s = 0; s < 4; ++s) if (s == ls) h[s] = kMark;
      }
      start = wm;
    }
    const V fin = start + dd;                                     // starts when its last unit frees
#pragma unroll
    for (int s = 0; s < 4; ++s) if (h[s] == kMark) h[s] = fin;
    return fin;
  }

  template <int D>
  __device__ static inline void take_all(V (&h)[D][4], int u, V dd, int lane, uint64_t (&obj)[D]) {
#pragma unroll
    for (int k = 0; k < D; ++k) obj[k] += (uint64_t)take(h[k], u, dd, lane);
  }
};

// Alg. 2 estimate(): insert the waiting actions one after the other into the completion heap
// (`H` entries staged in s_heap).  All but the first action use their minimum units; the first
// tries its d-th smallest option for d = 1..depth.  The evicted tail C[L:] is read from LDS
// (s_cdur, s_q0); only actions pinned to the node that never got in come from global memory.
//
// tg_estimate_run simulates D consecutive depths d0 .. d0+D-1 side by side on D heaps: they
// differ only in the option of the first action, and a lone wavefront is bound by the latency
// of its dependent instructions, so independent heaps overlap.  ok[k] is false when depth
// d0+k does not exist (the first action has fewer usable options).  Times are offsets from
// `lo` (0 with TgHeapWide).
template <typename HP, int D>
__device__ static inline void tg_estimate_run(const TgNodeIn& in, const TgWaitLds& W, const int64_t* s_heap,
                                              const int64_t* s_cdur, const uint8_t* s_q0, const int32_t* s_k, int H, int L,
                                              int lane, int64_t lo, int d0, int64_t* obj_out, bool* ok_out) {
  typedef typename HP::V V;
  const int n_tail = in.m - L, n_ac = n_tail + in.nd;
  V hv[D][HP::kSlots];
  HP::load(hv[0], s_heap, H, lo, lane);
#pragma unroll
  for (int k = 1; k < D; ++k)
#pragma unroll
    for (int s = 0; s < HP::kSlots; ++s) hv[k][s] = hv[0][s];
  uint64_t obj[D];                                              // sums of finish-time offsets (wavefront-uniform)
  bool ok[D];
#pragma unroll
  for (int k = 0; k < D; ++k) { obj[k] = 0; ok[k] = true; }
  int n_done = 0;
  bool first = true;
  for (int base = 0; base < n_ac && ok[0]; base += TG_WAVE) {
    const int cnt = min(TG_WAVE, n_ac - base);
    int my_u = 0;
    bool my_ok = false;
    V my_d = 0;
    if (lane < cnt) {
      const int x = base + lane;
      if (x < n_tail) {                                         // evicted candidate: everything is in LDS
        const int q0 = s_q0[L + x];
        my_u = s_k[q0]; my_ok = true; my_d = (V)(uint64_t)s_cdur[(L + x) * in.K + q0];
      } else if (x - n_tail < W.slots) {                        // staged when the node was set up
        my_u = W.u[x - n_tail]; my_ok = my_u != 0; my_d = (V)(uint64_t)W.d[x - n_tail];
      } else {
        const int id = in.dlist[x - n_tail];
        const uint32_t mask = in.act_kmask[id];
        const int q0 = __builtin_ctz(mask | 0x80000000u);
        my_u = s_k[q0 & (TG_MAX_K - 1)];
        my_ok = mask != 0 && q0 < TG_MAX_K && my_u <= H;        // can never run on this node: left out
        if (my_ok) my_d = (V)(uint64_t)(in.dur[(size_t)id * in.K + q0] + tg_restore_delay(in, id));
      }
    }
    uint64_t todo = __ballot(my_ok);                            // the chunk's actions that take part, FCFS = ascending lane
    auto lane_d = [&](int l) -> V {
      if (sizeof(V) == 4) return (V)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)my_d, l);
      return (V)(uint64_t)tg_readlane_i64((int64_t)(uint64_t)my_d, l);
    };
    if (first && todo) {
      // the very first action tries its d-th smallest usable option, d = d0 + k
      first = false;
      const int l = __ffsll((unsigned long long)todo) - 1;
      todo &= todo - 1;
      const int x = base + l;
      int id = -1, xx = 0;
      uint32_t mask = 0;
      if (x < n_tail) xx = L + x;
      else { id = in.dlist[x - n_tail]; mask = in.act_kmask[id]; }
      int u[D];
      V dd[D];
#pragma unroll
      for (int k = 0; k < D; ++k) {
        u[k] = __builtin_amdgcn_readlane(my_u, l);
        dd[k] = lane_d(l);
        const int d = d0 + k;
        if (d == 1) continue;                                   // the minimum-unit option
        int seen = 0, qd = -1;
        for (int q = 0; q < in.K; ++q) {
          const bool allowed = id < 0 ? s_cdur[xx * in.K + q] != TG_INF : (mask >> q & 1u) != 0;
          if (allowed && s_k[q] <= H && ++seen == d) { qd = q; break; }
        }
        qd = __builtin_amdgcn_readfirstlane(qd);
        if (qd < 0) { ok[k] = false; continue; }                // simulated with the minimum option, result unused
        u[k] = __builtin_amdgcn_readfirstlane(s_k[qd]);
        const int64_t t = id < 0 ? s_cdur[xx * in.K + qd] : in.dur[(size_t)id * in.K + qd] + tg_restore_delay(in, id);
        if (sizeof(V) == 4) dd[k] = (V)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)t);
        else dd[k] = (V)(uint64_t)tg_readlane_i64(t, 0);
      }
      if (!ok[0]) break;
#pragma unroll
      for (int k = 0; k < D; ++k) obj[k] += (uint64_t)HP::take(hv[k], u[k], dd[k], lane);
      ++n_done;
    }
    while (todo) {                                              // everybody else on the minimum units
      const int l = __ffsll((unsigned long long)todo) - 1;
      todo &= todo - 1;
      const int u = __builtin_amdgcn_readlane(my_u, l);
      const V dd = lane_d(l);
      HP::template take_all<D>(hv, u, dd, lane, obj);
      ++n_done;
    }
  }
#pragma unroll
  for (int k = 0; k < D; ++k) { obj_out[k] = (int64_t)obj[k] + lo * n_done; ok_out[k] = ok[k]; }
}

// N32: every time of this node fits in 32 bits above `lo` (checked by the caller).
template <bool N32>
__device__ static inline int64_t tg_estimate(const TgNodeIn& in, const TgWaitLds& W, const int64_t* s_heap,
                                             const int64_t* s_cdur, const uint8_t* s_q0, const int32_t* s_k, int H, int L,
                                             int lane, int64_t lo) {
  if (in.m - L + in.nd == 0) return 0;
  int64_t best = TG_INF;
  for (int d0 = 1; d0 <= in.depth; d0 += 2) {
    int64_t obj[2] = {TG_INF, TG_INF};
    bool ok[2] = {false, false};
    const bool two = d0 < in.depth;
#define TG_RUN(HP)                                                                                             \
  {                                                                                                            \
    if (two) tg_estimate_run<HP, 2>(in, W, s_heap, s_cdur, s_q0, s_k, H, L, lane, N32 ? lo : 0, d0, obj, ok); \
    else tg_estimate_run<HP, 1>(in, W, s_heap, s_cdur, s_q0, s_k, H, L, lane, N32 ? lo : 0, d0, obj, ok);     \
  }
    if (!N32) TG_RUN(TgHeapWide)
    else if (H <= TG_WAVE) TG_RUN(TgHeapSorted<1>)
    else if (H <= 2 * TG_WAVE) TG_RUN(TgHeapSorted<2>)
    else TG_RUN(TgHeapSorted<4>)
#undef TG_RUN
    if (!ok[0]) break;                                          // no d-th option: larger depths do not exist either
    best = obj[0] < best ? obj[0] : best;
    if (!two) break;
    if (!ok[1]) break;
    best = obj[1] < best ? obj[1] : best;
  }
  return best;
}

// Alg. 3 with the basic operator (state = units used), all prefixes at once: row i of the table
// holds the best totals of C[:i]; per row the choice of every cell, the best total over
// used <= n and its smallest argument are kept.  V = uint32_t when every total of the node
// fits in 32 bits (the caller checks the sum of the longest durations), else int64_t.

template <typename V>
__device__ static inline void tg_dp_units(V* prev, V* cur, const int64_t* s_cdur, uint8_t* s_choice, int64_t* s_rowbest,
                                          int32_t* s_rowarg, int m, int n, int K, uint64_t kword, int lane) {
  typedef typename std::make_unsigned<V>::type UV;
  const V kInf = std::is_same<V, uint32_t>::value ? (V)0xffffffffu : (V)TG_INF;
  const int stride = tg_choice_stride(n);
  for (int j = lane; j <= n; j += TG_WAVE) prev[j] = j == 0 ? (V)0 : kInf;
  if (lane == 0) { s_rowbest[0] = 0; s_rowarg[0] = 0; }
  V tq[TG_MAX_K];                                                 // durations of candidate i, same for all lanes
  auto load_tq = [&](int i) {                                     // unconditional reads (index clamped), masked after
#pragma unroll
    for (int q = 0; q < TG_MAX_K; ++q) {
      const int64_t t = s_cdur[(i - 1) * K + (q < K ? q : K - 1)];
      tq[q] = (q >= K || t == TG_INF) ? kInf : (V)t;
    }
  };
  load_tq(1);
  tg_wave_sync();
  for (int i = 1; i <= m; ++i) {
    V tc[TG_MAX_K];
#pragma unroll
    for (int q = 0; q < TG_MAX_K; ++q) tc[q] = tq[q];
    if (i < m) load_tq(i + 1);                                    // next row's durations arrive while this row is computed
    if (lane == 0) cur[0] = kInf;                                 // every candidate takes a unit
    V bv = kInf;                                                  // this lane's best cell, smallest j on ties
    uint32_t bj = 0xffffffffu;
    // Two adjacent cells per pass and every read of the previous row issued unconditionally
    // (index clamped, result masked): the reads of a pass overlap instead of costing one LDS
    // round trip per option.
    for (int j = 2 * lane + 1; j <= n; j += 2 * TG_WAVE) {
      const int j2 = j + 1;
      const bool have2 = j2 <= n;
      V pa[TG_MAX_K], pb[TG_MAX_K];
#pragma unroll
      for (int q = 0; q < TG_MAX_K; ++q) {
        const int kq = (int)(kword >> (8 * q) & 0xff);
        pa[q] = prev[j >= kq ? j - kq : 0];
        pb[q] = prev[have2 && j2 >= kq ? j2 - kq : 0];
      }
      V besta = kInf, bestb = kInf;
      int qa = 0xf, qb = 0xf;
#pragma unroll
      for (int q = 0; q < TG_MAX_K; ++q) {                        // ascending k, strict <: fewer units win ties
        const int kq = (int)(kword >> (8 * q) & 0xff);
        const V ca = (V)((UV)pa[q] + (UV)tc[q]), cb = (V)((UV)pb[q] + (UV)tc[q]);   // masked below where a term is infinite
        const bool ta = tc[q] != kInf && j >= kq && pa[q] != kInf && ca < besta;
        const bool tb = tc[q] != kInf && j2 >= kq && pb[q] != kInf && cb < bestb;
        besta = ta ? ca : besta; qa = ta ? q : qa;
        bestb = tb ? cb : bestb; qb = tb ? q : qb;
      }
      cur[j] = besta;
      if (besta < bv) { bv = besta; bj = (uint32_t)j; }
      if (have2) {
        cur[j2] = bestb;
        if (bestb < bv) { bv = bestb; bj = (uint32_t)j2; }
      }
      s_choice[(size_t)(i - 1) * stride + (j >> 1)] = (uint8_t)(qa | (have2 ? qb : 0xf) << 4);
    }
    // best over used <= n, fewest units on ties
    if (std::is_same<V, uint32_t>::value) {
      const uint32_t vmin = tg_wave_min_u32((uint32_t)bv);
      const uint32_t jmin = tg_wave_min_u32((uint32_t)bv == vmin ? bj : 0xffffffffu);
      if (lane == 0) { s_rowbest[i] = (int64_t)vmin; s_rowarg[i] = (int)(jmin & 511); }
    } else {
      const uint64_t key = bv == kInf ? ~0ull : ((uint64_t)bv << 9 | (bj & 511));
      const uint64_t rb = tg_wave_min_u64(key);
      if (lane == 0) { s_rowbest[i] = (int64_t)(rb >> 9); s_rowarg[i] = (int)(rb & 511); }
    }
    V* tmp = prev; prev = cur; cur = tmp;
    tg_wave_sync();
  }
}

// The same table for nodes whose totals stay below 2^30 (the caller checks the sum of the
// longest durations): 32-bit cells with kDpInf32 = 2^30 standing for "unreachable", so that
// "previous cell + duration" needs no validity test - an unreachable term keeps the sum at or
// above 2^30 without wrapping, and 64 unreachable sentinel cells below cell 0 stand in for the
// cells j - k < 0.  An option then costs an add, a compare, a select and a min per cell.  KK is
// the number of options.  prev / cur point at cell 0 of two rows laid out by the caller.
constexpr uint32_t kDpInf32 = 0x40000000u;

template <int KK>
__device__ static inline void tg_dp_units32(uint32_t* prev, uint32_t* cur, const int64_t* s_cdur, uint8_t* s_choice,
                                            int64_t* s_rowbest, int32_t* s_rowarg, int m, int n, uint64_t kword, int lane) {
  const int stride = tg_choice_stride(n);
  for (int j = lane - TG_WAVE; j <= n + 1; j += TG_WAVE) { prev[j] = j == 0 ? 0u : kDpInf32; cur[j] = kDpInf32; }
  if (lane == 0) { s_rowbest[0] = 0; s_rowarg[0] = 0; }
  uint32_t tq[KK];                                                // durations of candidate i, same for all lanes
  auto load_tq = [&](int i) {
#pragma unroll
    for (int q = 0; q < KK; ++q) {
      const int64_t t = s_cdur[(i - 1) * KK + q];
      tq[q] = t == TG_INF ? kDpInf32 : (uint32_t)t;
    }
  };
  load_tq(1);
  tg_wave_sync();
  for (int i = 1; i <= m; ++i) {
    uint32_t tc[KK];
#pragma unroll
    for (int q = 0; q < KK; ++q) tc[q] = tq[q];
    if (i < m) load_tq(i + 1);                                    // next row's durations arrive while this row is computed
    uint32_t bv = kDpInf32, bj = 0xffffffffu;                     // this lane's best cell, smallest j on ties
    for (int j = 2 * lane + 1; j <= n; j += 2 * TG_WAVE) {        // cells j and j+1 (cell n+1 is scratch)
      uint32_t pa[KK], pb[KK];
#pragma unroll
      for (int q = 0; q < KK; ++q) {
        const int kq = (int)(kword >> (8 * q) & 0xff);
        pa[q] = prev[j - kq];
        pb[q] = prev[j + 1 - kq];
      }
      uint32_t besta = kDpInf32, bestb = kDpInf32, qa = 0xf, qb = 0xf;
#pragma unroll
      for (int q = 0; q < KK; ++q) {                              // ascending k, strict <: fewer units win ties
        const uint32_t ca = pa[q] + tc[q], cb = pb[q] + tc[q];
        qa = ca < besta ? (uint32_t)q : qa; besta = ca < besta ? ca : besta;
        qb = cb < bestb ? (uint32_t)q : qb; bestb = cb < bestb ? cb : bestb;
      }
      const bool have2 = j + 1 <= n;
      cur[j] = besta;
      cur[j + 1] = bestb;
      s_choice[(size_t)(i - 1) * stride + (j >> 1)] = (uint8_t)(qa | qb << 4);
      if (besta < bv) { bv = besta; bj = (uint32_t)j; }
      if (have2 && bestb < bv) { bv = bestb; bj = (uint32_t)(j + 1); }
    }
    // best over used <= n, fewest units on ties.  With one pass per row (n <= 128) the cells ascend with the lanes:
    // the smallest argument is that of the lowest lane that holds the minimum.
    const uint32_t vmin = tg_wave_min_u32(bv);
    uint32_t jmin;
    if (n <= 2 * TG_WAVE) {
      const uint64_t at_min = __ballot(bv == vmin);
      jmin = (uint32_t)__builtin_amdgcn_readlane((int)bj, __builtin_ctzll(at_min));
    } else {
      jmin = tg_wave_min_u32(bv == vmin ? bj : 0xffffffffu);
    }
    if (lane == 0) { s_rowbest[i] = (int64_t)vmin; s_rowarg[i] = (int)(jmin & 511); cur[0] = kDpInf32; }
    uint32_t* tmp = prev; prev = cur; cur = tmp;
    tg_wave_sync();
  }
}

// the k lowest set bits of m (1 <= k <= popcount(m)): binary descent to the k-th set bit
__device__ static inline uint64_t tg_lowest_bits(uint64_t m, int k) {
  if (k <= 4) {                                                   // the usual case: peel the bits off one by one
    uint64_t rest = m;
    for (int x = 0; x < k; ++x) rest &= rest - 1;
    return m ^ rest;
  }
  int pos = 0, r = k;
#pragma unroll
  for (int w = 32; w >= 1; w >>= 1) {
    const int c = __popcll((m >> pos) & ((1ull << w) - 1));
    if (r > c) { pos += w; r -= c; }
  }
  return m & ((2ull << pos) - 1);
}

// One allocation of k cores on a CPU node (Sec. 5.2: the cores of an action are named, one NUMA
// domain where possible).  Lane d holds the free cores of domain d in the low bits of `dm` (0 for
// lanes beyond the node's domains).  If a domain has k free cores: the one with the fewest that
// still has them (lowest domain on ties), its lowest-numbered free cores; otherwise whole domains,
// the one with the most free cores first (lowest on ties), until k cores are found.  Returns the
// bits this lane gives and clears them in `dm`; *one_domain tells whether a single lane gave all.
__device__ static inline uint64_t tg_take_cores(uint64_t& dm, int k, int lane, bool* one_domain) {
  int cnt = __popcll(dm);
  uint64_t take = 0;
  const uint32_t fit = tg_wave_min_u32(cnt >= k ? (uint32_t)cnt << 8 | (uint32_t)lane : 0xffffffffu);   // key = (free cores, domain)
  *one_domain = fit != 0xffffffffu;
  if (*one_domain) {
    if (lane == (int)(fit & 0xff)) take = tg_lowest_bits(dm, k);
  } else {
    int left = k;
    while (left > 0) {
      const uint32_t big = tg_wave_min_u32(cnt > 0 ? (uint32_t)(64 - cnt) << 8 | (uint32_t)lane : 0xffffffffu);
      if (big == 0xffffffffu) break;                              // cannot happen: a node hands out at most its free cores
      const int have = 64 - (int)(big >> 8), t = have < left ? have : left;
      if (lane == (int)(big & 0xff)) { take = tg_lowest_bits(dm, t); cnt -= t; }
      left -= t;
    }
  }
  dm ^= take;
  return take;
}

// A node with one candidate and nobody waiting for it needs no table and no heap: DPArrange over
// one action is its fastest allowed option that fits (equal durations: fewer units on counted
// resources; on GPU nodes the option that leaves the smaller chunk state, as the chunk DP ends in
// the smallest state among the best), the eviction loop has nothing to evict and the estimate of
// an empty queue is 0.  Same results as tg_node_schedule, lane q looks at option q.
__device__ static inline int64_t tg_node_single(const TgNodeIn& in, const TgNodeOut& out, int lane, int* used_units) {
  const int K = in.K;
  const int id = in.clist[0];
  const uint32_t mask = in.act_kmask[id];
  const bool elastic = in.act_model[id] != TG_MODEL_NONE;
  const int64_t delay = tg_restore_delay(in, id);
  const int my_k = (int)(in.kword >> (8 * (lane & (TG_MAX_K - 1))) & 0xff);
  uint64_t key = ~0ull;
  if (lane < K && (mask >> lane & 1u) && (elastic || lane == __builtin_ctz(mask))) {
    const int64_t d = in.dur[(size_t)id * K + lane];
    if (!elastic) key = (uint64_t)(d + delay) << 12;              // runs on its minimum units (Alg. 1)
    else if (d != TG_INF && my_k <= in.cap) {
      if (in.type == TG_TYPE_GPU) {
        if (my_k <= tg_chunk_largest(in.chunks)) {
          const int r0 = max((int)(in.chunks & 0xff), 1) + 1, r1 = max((int)(in.chunks >> 8 & 0xff), 1) + 1,
                    r2 = max((int)(in.chunks >> 16 & 0xff), 1) + 1;
          const uint32_t c = tg_chunk_take(in.chunks, my_k);
          const int code = (int)(c & 0xff) + r0 * ((int)(c >> 8 & 0xff) + r1 * ((int)(c >> 16 & 0xff) + r2 * (int)(c >> 24)));
          key = (uint64_t)(d + delay) << 12 | (uint32_t)code;
        }
      } else if (my_k <= in.free_units) key = (uint64_t)(d + delay) << 12 | (uint32_t)my_k;
    }
  }
  const uint64_t best = tg_wave_min_u64(key);                       // admission has made sure that the minimum units fit
  const int q = __builtin_ctzll(__ballot(key == best));
  const int k = (int)(in.kword >> (8 * q) & 0xff);
  const int64_t d = (int64_t)(best >> 12);
  if (lane == 0) {
    out.units[id] = k;
    if (out.act) out.act[id] = (out.age ? out.age[id] : 0) + in.backlog + d;
  }
  *used_units = k;
  return elastic ? d + in.backlog : -1;
}

// One node, scheduled by one wavefront (no workgroup barrier anywhere): the DPArrange table for
// all prefixes, then the greedy rule of Alg. 1 - evict from the tail while the approximated
// objective of Alg. 2 drops.  Returns the final approximated objective (or -1 when the node
// holds no elastic action and everything simply runs on its minimum units).  `smem` is the
// wavefront's LDS block laid out by `plan`.
__device__ static inline int64_t tg_node_schedule(unsigned char* smem, const TgNodeLdsPlan& plan, const TgNodeIn& in,
                                                  const TgNodeOut& out, int lane, int* used_units) {
  int64_t* s_cdur = reinterpret_cast<int64_t*>(smem + plan.off_cdur);
  int64_t* s_dp = reinterpret_cast<int64_t*>(smem + plan.off_dp);
  uint8_t* s_choice = smem + plan.off_choice;
  uint16_t* s_choice16 = reinterpret_cast<uint16_t*>(smem + plan.off_choice);
  int64_t* s_heap = reinterpret_cast<int64_t*>(smem + plan.off_heap);
  int64_t* s_rowbest = reinterpret_cast<int64_t*>(smem + plan.off_rowbest);
  int32_t* s_rowarg = reinterpret_cast<int32_t*>(smem + plan.off_rowarg);
  uint8_t* s_sel = smem + plan.off_sel;                           // [sel_rows][sel_stride] option of candidate x for L = top - l
  int32_t* s_k = reinterpret_cast<int32_t*>(smem + plan.off_k);
  int64_t* s_F = reinterpret_cast<int64_t*>(smem + plan.off_F);   // [1] elastic? [2] time origin [3] 32-bit times? [4] 32-bit DP?
  uint8_t* s_q0 = smem + plan.off_q0;                             // minimum-unit option of candidate x
  int64_t* s_wd = reinterpret_cast<int64_t*>(smem + plan.off_wd);
  uint8_t* s_wu = smem + plan.off_wu;
  const TgWaitLds W = {s_wd, s_wu, plan.wait_slots};
  const int m = in.m, K = in.K, U = in.free_units;
  const bool gpu = in.type == TG_TYPE_GPU;

  const uint64_t kword = in.kword;                                // unit counts, one byte each
  auto k_of = [&](int q) { return (int)(kword >> (8 * q) & 0xff); };

  tg_wave_sync();
  {
    if (lane < TG_MAX_K) s_k[lane] = k_of(lane);
    // lane = candidate: its elasticity model and its row of durations as this node sees them
    // (options above the node's capacity removed, restore delay added) in two dependent round
    // trips per 64 candidates
    int el = 0;
    for (int x = lane; x < m; x += TG_WAVE) {
      const int id = in.clist[x];
      el |= in.act_model[id] != TG_MODEL_NONE;
      const int64_t delay = tg_restore_delay(in, id);
      int64_t row[TG_MAX_K];
#pragma unroll
      for (int q = 0; q < TG_MAX_K; ++q) row[q] = q < K ? in.dur[(size_t)id * K + q] : TG_INF;
#pragma unroll
      for (int q = 0; q < TG_MAX_K; ++q)
        if (q < K) {
          int64_t d = row[q];
          if (k_of(q) > in.cap) d = TG_INF;
          else if (d != TG_INF) d += delay;
          if (x < plan.cand_rows) s_cdur[x * K + q] = d;            // a quota with more candidates: nothing elastic, rows unused
        }
    }
    const int any_el = __any(el);
    if (lane == 0) s_F[1] = any_el ? 1 : 0;
  }
  tg_wave_sync();
  if (s_F[1] == 0) {                                             // Alg. 1: no elastic action in the group, nothing to scale
    int used = 0;
    {
      for (int x = lane; x < m; x += TG_WAVE) {
        const int id = in.clist[x];
        const int q0 = __builtin_ctz(in.act_kmask[id]);
        out.units[id] = k_of(q0);
        used += k_of(q0);
        if (out.act) out.act[id] = (out.age ? out.age[id] : 0) + in.backlog + tg_restore_delay(in, id) + in.dur[(size_t)id * K + q0];
      }
      used = tg_wave_sum_i32(used);
    }
    *used_units = used;
    return -1;
  }

  int stride = 0;                                                 // entries per choice row
  {
    tg_wave_sync();                                               // the rows staged above
    // minimum-unit option of every candidate, and the range all times of this node's estimates
    // stay in: above `lo`, below the latest initial release plus every waiting duration
    {
      int64_t sumd = 0, sumc = 0, maxd = 0, bmin = in.backlog, bmax = 0;
      for (int x = lane; x < m; x += TG_WAVE) {
        int q0 = 0;
        while (q0 < K - 1 && s_cdur[x * K + q0] == TG_INF) ++q0;
        s_q0[x] = (uint8_t)q0;
        const int64_t d = s_cdur[x * K + q0];
        sumc += d; maxd = d > maxd ? d : maxd;
      }
      for (int y = lane; y < in.nd; y += TG_WAVE) {
        const int id = in.dlist[y];
        const uint32_t mask = in.act_kmask[id];
        const int q0 = __builtin_ctz(mask | 0x80000000u);
        const int u = k_of(q0 & (TG_MAX_K - 1));
        const bool runs = mask != 0 && q0 < TG_MAX_K && u <= U + in.n_busy;   // else it can never run on this node
        int64_t d = 0;
        if (mask) { d = in.dur[(size_t)id * K + __builtin_ctz(mask)] + tg_restore_delay(in, id); sumd += d; }
        if (y < plan.wait_slots) { s_wd[y] = runs ? d : 0; s_wu[y] = runs ? (uint8_t)u : 0; }
      }
      for (int c = lane; c < in.n_busy; c += TG_WAVE) {
        const int64_t b = in.busy_lds_off >= 0 ? reinterpret_cast<const int64_t*>(smem + in.busy_lds_off)[c] : in.busy[c];
        bmin = b < bmin ? b : bmin; bmax = b > bmax ? b : bmax;
      }
      sumd = tg_wave_sum_i64(sumd); sumc = tg_wave_sum_i64(sumc);
      sumd += sumc;
      maxd = (int64_t)~tg_wave_min_u64(~(uint64_t)maxd);
      bmax = (int64_t)~tg_wave_min_u64(~(uint64_t)bmax);
      bmin = (int64_t)tg_wave_min_u64((uint64_t)bmin);
      const int64_t top_t = in.backlog + maxd > bmax ? in.backlog + maxd : bmax;
      if (lane == 0) {
        s_F[2] = bmin;
        s_F[3] = (top_t + sumd - bmin) < 0xfffffff0ll ? 1 : 0;   // estimates in 32 bits
        s_F[4] = sumc < (int64_t)kDpInf32 ? 1 : 0;               // DP totals below the 32-bit "unreachable" mark
      }
      tg_wave_sync();
    }

    // ---- DPArrange over all prefixes at once: row i holds the best totals of C[:i] --------
    if (!gpu) {
      int sm = 0;                                                 // End(S): sum of the largest options
      for (int a = lane; a < m; a += TG_WAVE) {
        int kmax = 0;
        for (int q = 0; q < K; ++q) if (s_cdur[a * K + q] != TG_INF) kmax = k_of(q);
        sm += kmax;
      }
      sm = tg_wave_sum_i32(sm);
      const int n = min(U, sm);
      stride = tg_choice_stride(n);
      if (s_F[4] != 0) {
        uint32_t* r0 = reinterpret_cast<uint32_t*>(s_dp) + TG_WAVE;               // cell 0 of the two rows
        uint32_t* r1 = r0 + plan.dp_width + 2 + TG_WAVE;
        switch (K) {
#define TG_DP32(KK) case KK: tg_dp_units32<KK>(r0, r1, s_cdur, s_choice, s_rowbest, s_rowarg, m, n, kword, lane); break;
          TG_DP32(1) TG_DP32(2) TG_DP32(3) TG_DP32(4) TG_DP32(5) TG_DP32(6) TG_DP32(7) TG_DP32(8)
#undef TG_DP32
        }
      } else
        tg_dp_units<int64_t>(s_dp, s_dp + plan.dp_width, s_cdur, s_choice, s_rowbest, s_rowarg, m, n, K, kword, lane);
    } else {
      // Alg. 4: state = counts of free chunks (1,2,4,8), mixed-radix encoded; a transition takes
      // the smallest chunk that holds k GPUs and splits it.  Forward relaxation with a packed
      // 64-bit key (value | source state | option) so that ties resolve to the smallest source
      // state, then the smallest option, independent of lane timing.
      const int n0 = max((int)(in.chunks & 0xff), 1), n1 = max((int)(in.chunks >> 8 & 0xff), 1),
                n2 = max((int)(in.chunks >> 16 & 0xff), 1), n3 = max((int)(in.chunks >> 24), 1);
      const int r0 = n0 + 1, r1 = n1 + 1, r2 = n2 + 1;
      const int S = r0 * r1 * r2 * (n3 + 1);
      stride = S;
      uint64_t* prev = reinterpret_cast<uint64_t*>(s_dp);
      uint64_t* cur = prev + plan.dp_width;
      const int s_start = (int)(in.chunks & 0xff) + r0 * ((int)(in.chunks >> 8 & 0xff) + r1 * ((int)(in.chunks >> 16 & 0xff) + r2 * (int)(in.chunks >> 24)));
      for (int s = lane; s < S; s += TG_WAVE) prev[s] = s == s_start ? 0ull : ~0ull;
      if (lane == 0) { s_rowbest[0] = 0; s_rowarg[0] = s_start; }
      tg_wave_sync();
      for (int i = 1; i <= m; ++i) {
        for (int s = lane; s < S; s += TG_WAVE) cur[s] = ~0ull;
        tg_wave_sync();
        for (int s = lane; s < S; s += TG_WAVE) {
          const uint64_t kp = prev[s];
          if (kp == ~0ull) continue;
          const uint64_t v = kp >> 12;
          int rest = s;
          const uint32_t c0 = rest % r0; rest /= r0;
          const uint32_t c1 = rest % r1; rest /= r1;
          const uint32_t c2 = rest % r2; rest /= r2;
          const uint32_t c = c0 | c1 << 8 | c2 << 16 | (uint32_t)rest << 24;
          const int largest = tg_chunk_largest(c);
          for (int q = 0; q < K; ++q) {
            const int64_t t = s_cdur[(i - 1) * K + q];
            const int kq = k_of(q);
            if (t == TG_INF || kq > largest) continue;
            const uint32_t c2n = tg_chunk_take(c, kq);
            const int s2 = (int)(c2n & 0xff) + r0 * ((int)(c2n >> 8 & 0xff) + r1 * ((int)(c2n >> 16 & 0xff) + r2 * (int)(c2n >> 24)));
            const uint64_t key = (v + (uint64_t)t) << 12 | (uint64_t)s << 3 | (uint64_t)q;
            atomicMin(reinterpret_cast<unsigned long long*>(&cur[s2]), (unsigned long long)key);
          }
        }
        tg_wave_sync();
        uint64_t rb = ~0ull;
        for (int s = lane; s < S; s += TG_WAVE) {
          const uint64_t k2 = cur[s];
          s_choice16[(size_t)(i - 1) * stride + s] = (uint16_t)(k2 & 0xfff);
          if (k2 != ~0ull) { const uint64_t key = (k2 >> 12) << 9 | (uint32_t)s; rb = key < rb ? key : rb; }
        }
        rb = tg_wave_min_u64(rb);
        if (lane == 0) { s_rowbest[i] = (int64_t)(rb >> 9); s_rowarg[i] = (int)(rb & 511); }
        uint64_t* tmp = prev; prev = cur; cur = tmp;
        tg_wave_sync();
      }
    }
  }

  // ---- Alg. 2: objective of keeping the first L candidates ---------------------------------
  const int H = U + in.n_busy;
  tg_wave_sync();                                                     // wavefront 0's tables are complete
  const int64_t t_lo = s_F[2];
  const bool narrow = s_F[3] != 0;
  // Allocations of up to 64 consecutive prefix lengths at once: lane l of wavefront 0 walks the
  // choice table back from the best end state of C[:top-l]; evaluations only look them up.
  int top = 0;                                                     // longest prefix the allocation table covers
  auto backtrack_batch = [&](int new_top) {
    top = new_top;
    tg_wave_sync();                                                   // nobody still reads the old table
    const int Lm = top - lane;
    if (lane < plan.sel_rows && Lm >= 1) {
      int st = s_rowarg[Lm];
      uint8_t* row = s_sel + (size_t)lane * plan.sel_stride;
      int hold = 0;                                                // option of the odd candidate of the current byte
      for (int i = Lm; i >= 1; --i) {
        int q;
        if (!gpu) { q = tg_choice_get(s_choice + (size_t)(i - 1) * stride, st); st -= k_of(q); }
        else { const int c = s_choice16[(size_t)(i - 1) * stride + st]; q = c & 7; st = c >> 3; }
        if ((i - 1) & 1) hold = q;
        else { row[(i - 1) >> 1] = (uint8_t)(q | hold << 4); hold = 0; }
      }
    }
    tg_wave_sync();
  };
  auto objective = [&](int L) -> int64_t {                         // one wavefront, table covers L
    const uint8_t* sel = s_sel + (size_t)(top - L) * plan.sel_stride;
    int pos = 0;                                                   // units handed out so far
    for (int base = 0; base < L; base += TG_WAVE) {
      const int x = base + lane;
      const int q = x < L ? tg_sel_get(sel, x) : 0, kq = x < L ? k_of(q) : 0;
      const int inc = tg_wave_scan_i32(kq);                        // inclusive scan of the unit counts
      if (x < L) {                                                 // k_i entries at backlog + dur_i(k_i)
        const int64_t fin = in.backlog + s_cdur[x * K + q];
        for (int c = 0; c < kq; ++c) s_heap[pos + inc - kq + c] = fin;
      }
      pos += __builtin_amdgcn_readlane(inc, TG_WAVE - 1);
    }
    for (int c = pos + lane; c < U; c += TG_WAVE) s_heap[c] = in.backlog;   // units left idle
    if (in.busy_lds_off >= 0) {
      const int64_t* bl = reinterpret_cast<const int64_t*>(smem + in.busy_lds_off);
      for (int c = lane; c < in.n_busy; c += TG_WAVE) s_heap[U + c] = bl[c];
    } else {
      for (int c = lane; c < in.n_busy; c += TG_WAVE) s_heap[U + c] = in.busy[c];
    }
    tg_wave_sync();
    const int64_t approx = narrow ? tg_estimate<true>(in, W, s_heap, s_cdur, s_q0, s_k, H, L, lane, t_lo)
                                  : tg_estimate<false>(in, W, s_heap, s_cdur, s_q0, s_k, H, L, lane, 0);
    tg_wave_sync();
    return s_rowbest[L] + (int64_t)L * in.backlog + approx;
  };

  // ---- Alg. 1's eviction loop: evict from the tail while the objective drops ----------------
  // (one call site for the objective: inlined twice it costs the replay kernel its second wavefront per SIMD)
  int L = m;                                                       // accepted length
  int64_t obj = 0;
  for (int Lc = m; Lc >= 1; --Lc) {
    if (Lc > top || Lc <= top - plan.sel_rows) backtrack_batch(Lc);
    const int64_t f = objective(Lc);
    if (Lc < m && f >= obj) break;                                 // a tie stops the eviction
    obj = f;
    L = Lc;
  }
  if (L > top || L <= top - plan.sel_rows) backtrack_batch(L);
  int used = 0;
  {
    const uint8_t* sel = s_sel + (size_t)(top - L) * plan.sel_stride;
    for (int x = lane; x < m; x += TG_WAVE) {
      const int id = in.clist[x];
      if (x < L) {
        const int q = tg_sel_get(sel, x);
        out.units[id] = k_of(q);
        used += k_of(q);
        if (out.act) out.act[id] = (out.age ? out.age[id] : 0) + in.backlog + s_cdur[x * K + q];
      } else {
        out.node[id] = -1; out.units[id] = 0; out.reason[id] = TG_DEFER_EVICTED;
        if (out.act) out.act[id] = -1;
      }
    }
    used = tg_wave_sum_i32(used);
  }
  *used_units = used;
  tg_wave_sync();
  return obj;
}

#endif  // TG_STEP_H_
