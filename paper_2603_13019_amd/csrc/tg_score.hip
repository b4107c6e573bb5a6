// tg_score_candidates: estimated completion time of every (action, node, unit option)
// candidate - Eq. 1 (duration on k units) inside Eq. 2 (queueing + execution) of the paper -
// written as one dense int64 tensor.
//
// Two kernels.  tg_score_dur_kernel evaluates Eq. 1 once per (action, option) into a scratch
// array of the problem (0.6 % of the tensor's size).  tg_score_kernel then is a pure write
// stream (8 bytes per candidate; its inputs are ~0.1 byte per candidate and come from cache).
// On this memory system such a stream runs fastest as short-lived workgroups that each write
// 4 KB and are dispatched in address order, so that the chip as a whole writes one moving window
// of a few MB; what a workgroup does before its stores must then stay short, because nothing
// amortises it - which is why the divisions of Eq. 1 are not done here:
//   * a workgroup is 128 lanes (up to 16 resident per compute unit) and owns 512 consecutive
//     entries of one (snapshot, kind) block; each lane stores two 16-byte pairs;
//   * the launch is a grid (chunk, snapshot): the three blocks of a snapshot sit in one
//     128-byte record, read with one uniform load; a comparison of the chunk index with the
//     blocks' chunk counts picks the block - no per-workgroup lookup table, and workgroups are
//     dispatched in the order of the tensor.  Snapshots of unequal size leave some workgroups
//     of the grid without a chunk (they exit at once); very unequal snapshots are launched in
//     groups of similar size;
//   * after that one load everything a lane needs - node word, duration and pin of each of its
//     four entries - is fetched in a single further round trip; no LDS, no barrier.
#include <cstddef>

#include "tg_internal.h"

namespace {

#ifndef TG_SCORE_PAIRS
#define TG_SCORE_PAIRS 4
#endif
constexpr int kPairs = TG_SCORE_PAIRS;                  // 16-byte pairs every lane stores
constexpr int kThreads = TG_SCORE_CHUNK / (2 * kPairs);
constexpr int kWaveSpan = 2 * TG_WAVE * kPairs;         // entries per wavefront
constexpr int kWaveRows = kPairs <= 2 ? 2 : 3;          // rows of 256 entries or more that span can touch
static_assert(kThreads % TG_WAVE == 0 && (kPairs == 2 || kPairs == 4), "whole wavefronts, two or four pairs per lane");

// The few fields of a problem the kernels read (a short argument list: its loads are the first
// thing every workgroup waits for).
struct ScoreArgs {
  const TgScoreSnap* snaps;       // this launch's snapshots
  const TgRowRec* row_rec;
  const int32_t* row_pin;
  const uint64_t* node_word;
  const uint64_t* row_svc;        // SVC only
  const uint64_t* node_res_k;     // SVC only
  const uint32_t* speedup;
  int64_t* dur;                   // [rows * (K + 1)] per kind-grouped row: getDur per option (TG_INF where not allowed), then the row's pin
  int64_t* cost;
  uint64_t kword;                 // unit counts, one byte each
  int K;                          // options per row of the speedup table; a row of dur has one slot more
  uint32_t magic_K1;              // floor(2^32 / (K + 1)) + 1
  int N, M;                       // actions and nodes per snapshot
};

// x / d for x < 2^31, with inv = 1.0 / d: the product is within 2^-21 of the true quotient, so
// its integer part is the quotient or one below; the remainder test makes it exact.
__device__ inline uint32_t div_u31(uint32_t x, uint32_t d, double inv) {
  uint32_t q = (uint32_t)((double)x * inv);
  const uint32_t r = x - q * d;
  if (r >= d) q += (int32_t)r < 0 ? -1 : 1;
  return q;
}

// Eq. 1 for every (row, option), rows in kind-grouped order; one lane per pair.  The three
// elasticity models are three (numerator, denominator) pairs of the same rounded-up division,
// so the lanes of a wavefront do not diverge on the model.  A row of the scratch array holds
// the K durations and, in a last slot, the row's pin - so that a score workgroup fetches all it
// needs of its rows with one load.  The kernel also reads every node word once: the score
// kernel's workgroups are too short-lived to wait for memory, and what was read just before
// them is still in the memory-side cache when they ask for it.
__global__ __launch_bounds__(256) void tg_score_dur_kernel(const ScoreArgs A) {
  const uint32_t x = blockIdx.x * 256u + threadIdx.x;                     // slot inside the snapshot
  const TgScoreKind& first = A.snaps[blockIdx.y].kind[0];                 // its rows and nodes start where those of its first kind do
  const uint32_t K1 = (uint32_t)A.K + 1u;
  if (x >= (uint32_t)A.N * K1) return;
  uint32_t r = __umulhi(x, A.magic_K1);                                   // x / (K + 1), at most one too large
  if (r * K1 > x) --r;
  const int q = (int)(x - r * K1);
  const size_t g = (size_t)first.a_off + r;
  const uint64_t warm = x < (uint32_t)A.M ? A.node_word[(size_t)first.n_off + x] : 0ull;   // never all ones (the options are counted in 4 bits)
  int64_t out;
  if (q == A.K) out = __builtin_nontemporal_load(A.row_pin + g);
  else {
    // read once: kept out of the caches the score kernel's inputs should stay in
    const int64_t T = __builtin_nontemporal_load(&A.row_rec[g].T);
    const uint64_t rest = __builtin_nontemporal_load(reinterpret_cast<const uint64_t*>(&A.row_rec[g].param));
    const uint32_t param = (uint32_t)rest, kmask = (uint32_t)(rest >> 32) & 0xffffu, model = (uint32_t)(rest >> 48) & 0xffu;
    const bool amdahl = model == TG_MODEL_AMDAHL, table = model == TG_MODEL_TABLE;
    const uint32_t k = (uint32_t)(A.kword >> (8 * q) & 0xff);
    const uint32_t sp = A.speedup[table ? param * (uint32_t)A.K + (uint32_t)q : 0u];
    const uint32_t w = (1000000u - param) * k + param;                   // < 2^26
    const uint64_t num = amdahl ? (uint64_t)T * w : table ? (uint64_t)T << 16 : (uint64_t)T;
    const uint32_t den = amdahl ? 1000000u * k : table ? sp : 1u;
    const int64_t d = tg_ceil_div(num, den);
    out = (kmask >> q & 1u) ? (d < 1 ? 1 : d) : TG_INF;
  }
  A.dur[g * K1 + (uint32_t)q] = warm == ~0ull ? 0 : out;
}

// v of lane `src` (any lane may ask for any lane's value)
__device__ inline int64_t lane_pick64(int64_t v, int src) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_bpermute(src * 4, (int)(uint32_t)v);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_bpermute(src * 4, (int)(uint32_t)((uint64_t)v >> 32));
  return (int64_t)((uint64_t)hi << 32 | lo);
}

constexpr int kKindWords = sizeof(TgScoreKind) / 4;   // cost_off, inv_lr, entries, a_off, n_off, M_t | K_t << 16, magic_k, rows
static_assert(kKindWords == 10 && offsetof(TgScoreKind, entries) == 16 && offsetof(TgScoreKind, M_t) == 28 &&
              offsetof(TgScoreKind, K_t) == 30 && offsetof(TgScoreKind, rows) == 36, "the kernel reads the record word by word");

// One chunk (number x) of 512 entries of the block whose record words are k.  FAST: see tg_score_kernel.
template <bool SVC, bool FAST>
__device__ inline void score_chunk(const ScoreArgs& A, const uint32_t (&k)[kKindWords], int x) {
  const int64_t cost_off = (int64_t)((uint64_t)k[1] << 32 | k[0]);
  const double inv_lr = __builtin_bit_cast(double, (uint64_t)k[3] << 32 | k[2]);
  const int n = (int)k[4], a_off = (int)k[5], n_off = (int)k[6], row_last = (int)k[9] - 1;
  const int Mt = (int)(k[7] & 0xffffu), K = (int)(k[7] >> 16);
  const uint32_t mk = k[8];
  const uint32_t Lr = (uint32_t)(Mt * K);
  // Lanes own adjacent pairs aligned to 16 bytes in the whole tensor: when the block starts at
  // an odd entry the chunks are shifted down by one and entry -1 does not exist.
  const int odd = (int)(cost_off & 1);
  const int e0 = x * TG_SCORE_CHUNK - odd;                                // may be -1
  const int e1 = min(n, e0 + TG_SCORE_CHUNK);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int w0 = e0 + wave * kWaveSpan;                                   // first pair of this wavefront
  if (w0 >= e1) return;                                                   // nothing left for it in the block
  const int f0 = w0 < 0 ? 0 : w0;                                         // its first existing entry
  // the wavefront's first entry: its row, node and option - the same in all lanes, kept in scalar registers
  const int row0 = __builtin_amdgcn_readfirstlane((int)div_u31((uint32_t)f0, Lr, inv_lr));
  const uint32_t col0 = (uint32_t)f0 - (uint32_t)row0 * Lr;               // place of entry f0 in its row
  const int j0 = (int)((col0 * mk) >> 20), q0 = (int)col0 - j0 * K;       // col0 / K: exact for col0 < 2^17

  const uint64_t* words = A.node_word + n_off;
  const uint64_t* resk = SVC ? A.node_res_k + n_off : nullptr;
  const int K1 = A.K + 1;                                                // slots per row of dur: the options, then the pin
  const int64_t* dur = A.dur + (size_t)a_off * K1;
  const uint64_t* rsvc = SVC ? A.row_svc + a_off : nullptr;
  // FAST: the wavefront's entries lie in two rows.  Lane z < 2 (K + 1) fetches slot z % (K + 1) of row z / (K + 1)
  // (durations, then the pin); every lane then picks what its entries need out of those lanes' registers (one data
  // exchange inside the wavefront instead of loads per entry).
  int64_t dv = 0;
  uint64_t sv2 = 0;
  if (FAST) {
    const int r = lane >= 2 * K1 ? 2 : lane >= K1 ? 1 : 0;
    const int rd = min(row0 + r, row_last), rp = min(row0 + min(lane, kWaveRows - 1), row_last);
    if (lane < kWaveRows * K1) dv = dur[(size_t)rd * K1 + (lane - r * K1)];
    if (SVC && lane < kWaveRows) sv2 = rsvc[rp];
  }

  // values of all pairs first, then the stores back to back (nothing is waited for between them)
  int64_t v[kPairs][2];
#pragma unroll
  for (int i = 0; i < kPairs; ++i) {
    const int p = w0 + i * 128 + 2 * lane;
    const int pa = min(max(p, 0), n - 1);                                 // coordinates are taken inside the block
    int row, j, q;
    if (FAST) {
      // (node, option) of the entry from those of the wavefront's first entry: the offset is below 512, so the
      // division by K is a 24-bit multiplication (full rate); at most kWaveRows - 1 row ends are crossed
      const uint32_t t = (uint32_t)q0 + (uint32_t)(pa - f0);
      const uint32_t ja = __umul24(t, mk) >> 20;                          // t / K: exact for t < 2^17
      q = (int)(t - __umul24(ja, (uint32_t)K));
      j = j0 + (int)ja;
      row = row0;
#pragma unroll
      for (int w = 1; w < kWaveRows; ++w) {
        const bool wrap = j >= Mt;
        j -= wrap ? Mt : 0;
        row += wrap ? 1 : 0;
      }
    } else {
      row = (int)div_u31((uint32_t)pa, Lr, inv_lr);
      const uint32_t col = (uint32_t)pa - (uint32_t)row * Lr;
      j = (int)((col * mk) >> 20);                                        // col / K: exact for col < 2^17
      q = (int)col - j * K;
    }
    // the second entry of the pair is one step on - unless entry p = -1 does not exist: then entry 0 is the second
    const bool step = p >= 0;
    const bool wq = step && q + 1 == K, wj = wq && j + 1 == Mt;
    const int q2 = wq ? 0 : q + (step ? 1 : 0), j2 = wj ? 0 : j + (wq ? 1 : 0);
    const int row2 = min(row + (wj ? 1 : 0), row_last);                   // an entry past the end is not stored
    const int rows[2] = {row, row2}, js[2] = {j, j2}, qs[2] = {q, q2};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint64_t nw, res = 0, sw = 0;
      int64_t d;
      int pin;
      if (FAST) {
        const int rl = rows[h] - row0, base = (int)__umul24((uint32_t)rl, (uint32_t)K1);
        nw = *reinterpret_cast<const uint64_t*>(reinterpret_cast<const char*>(words) + ((uint32_t)js[h] << 3));   // 32-bit offset from a uniform base
        d = lane_pick64(dv, base + qs[h]); pin = __builtin_amdgcn_ds_bpermute((base + A.K) * 4, (int)(uint32_t)dv);
        if (SVC) { res = resk[js[h]]; sw = (uint64_t)lane_pick64((int64_t)sv2, rl); }
      } else {
        nw = words[js[h]]; d = dur[(size_t)rows[h] * K1 + qs[h]]; pin = (int)dur[(size_t)rows[h] * K1 + A.K];
        if (SVC) { res = resk[js[h]]; sw = rsvc[rows[h]]; }
      }
      const bool ok = (d != TG_INF) & (qs[h] < (int)(nw >> 48)) & ((pin == -1) | (pin == js[h]));   // no short cut: no load waits for another
      int64_t val = ok ? (int64_t)(nw & 0xffffffffffffull) + d : TG_INF;
      if (SVC && ok) {
        const int sv = (int)(sw >> 48);                                    // service + 1, 0: none
        if (sv && !(res >> (sv - 1) & 1ull)) val += (int64_t)(sw & 0xffffffffffffull);
      }
      v[i][h] = val;
    }
  }
  int64_t* out = A.cost + cost_off;
#pragma unroll
  for (int i = 0; i < kPairs; ++i) {
    const int p = w0 + i * 128 + 2 * lane;
    const bool ok0 = p >= 0 && p < e1, ok1 = p + 1 < e1;
    if (ok0 && ok1) {
      int64_t __attribute__((ext_vector_type(2))) pv = {v[i][0], v[i][1]};
      __builtin_nontemporal_store(pv, reinterpret_cast<int64_t __attribute__((ext_vector_type(2)))*>(out + p));
    } else {
      if (ok0) __builtin_nontemporal_store(v[i][0], out + p);
      if (ok1) __builtin_nontemporal_store(v[i][1], out + p + 1);
    }
  }
}

// SVC: the problem has services (Sec. 5.3): an entry whose action calls a service that is not
// resident on the node carries the service's restore time on top of Eq. 2.
template <bool SVC>
__global__ __launch_bounds__(kThreads) void tg_score_kernel(const ScoreArgs A) {
  // one uniform 128-byte load (the records are never written while a problem exists: constant
  // address space, scalar loads); every word stays in a scalar register
  typedef const __attribute__((address_space(4))) uint32_t* ConstWords;
  ConstWords src = (ConstWords)(A.snaps + blockIdx.y);
  uint32_t w[3 * kKindWords];
#pragma unroll
  for (int i = 0; i < 3 * kKindWords; ++i) w[i] = src[i];
  int x = (int)blockIdx.x;
  int c[3];
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    const int entries = (int)w[t * kKindWords + 4], odd = (int)(w[t * kKindWords] & 1u);
    c[t] = entries ? (entries + odd + TG_SCORE_CHUNK - 1) / TG_SCORE_CHUNK : 0;
  }
  int t = 0;
  if (x >= c[0]) { x -= c[0]; t = 1; if (x >= c[1]) { x -= c[1]; t = 2; if (x >= c[2]) return; } }
  // the chosen block's words, picked out of the record in registers (no second load)
  uint32_t k[kKindWords];
#pragma unroll
  for (int i = 0; i < kKindWords; ++i) k[i] = t == 0 ? w[i] : t == 1 ? w[kKindWords + i] : w[2 * kKindWords + i];
  // Rows of 256 entries or more: the 256 entries of a wavefront lie in two rows, whose durations and pins a
  // few lanes fetch for all.  Other blocks (few nodes: a small part of any tensor) load them per entry.
  const int Mt = (int)(k[7] & 0xffffu), K = (int)(k[7] >> 16);
  if (Mt * K >= TG_SCORE_CHUNK / 2) score_chunk<SVC, true>(A, k, x);
  else score_chunk<SVC, false>(A, k, x);
}

}  // namespace

int tg_launch_score(const tg_problem* p, int64_t* d_cost, hipStream_t s) {
  if (p->score_launches.empty()) return TG_OK;
  const bool svc = p->dev.act_service != nullptr;
  ScoreArgs a;
  a.row_rec = p->dev.row_rec; a.row_pin = p->dev.row_pin; a.node_word = p->dev.node_word;
  a.row_svc = p->dev.row_svc; a.node_res_k = p->dev.node_res_k; a.speedup = p->dev.speedup;
  a.dur = p->d_score_dur; a.cost = d_cost; a.kword = tg_pack_k(p->dev.k_list); a.K = p->dev.K;
  a.magic_K1 = (uint32_t)((1ull << 32) / (uint32_t)(a.K + 1)) + 1u;
  a.N = p->dev.N; a.M = p->dev.M;
  // Slabs of snapshots, each first through tg_score_dur_kernel and then through tg_score_kernel: the durations of a
  // slab (about 24 MB) are read while they are still in the memory-side cache, whatever ran before the call and
  // whatever runs next to it.
  const size_t per_snap = (size_t)a.N * (a.K + 1) * 8;
  const int slab = (int)std::max<size_t>(1, std::min<size_t>(65535, (24u << 20) / std::max<size_t>(per_snap, 1)));
  const unsigned dur_x = (unsigned)(((size_t)a.N * (a.K + 1) + 255) / 256);
  for (const TgScoreLaunch& g : p->score_launches)
    for (int s0 = 0; s0 < g.n_snaps; s0 += slab) {
      const int n = std::min(slab, g.n_snaps - s0);
      a.snaps = p->d_score_snaps + g.first + s0;
      hipLaunchKernelGGL(tg_score_dur_kernel, dim3(dur_x, (unsigned)n, 1), dim3(256), 0, s, a);
      const dim3 grid((unsigned)g.max_chunks, (unsigned)n, 1);
      if (svc) hipLaunchKernelGGL(tg_score_kernel<true>, grid, dim3(kThreads), 0, s, a);
      else hipLaunchKernelGGL(tg_score_kernel<false>, grid, dim3(kThreads), 0, s, a);
    }
  return hipGetLastError() == hipSuccess ? TG_OK : TG_E_HIP;
}

extern "C" int tg_score_candidates(const tg_problem* p, int64_t* d_cost, void* hip_stream) {
  if (!p || (!d_cost && p->n_candidates) || ((uintptr_t)d_cost & 15)) return TG_E_INVALID_ARG;
  return tg_launch_score(p, d_cost, (hipStream_t)hip_stream);
}
