// Formulation stage (Sec. 4.1 of the paper): validate a problem description, normalise every
// action and node, group them by resource kind and ship one packed copy to the device.
#include <algorithm>
#include <cstring>
#include <cstdlib>
#include <new>
#include <vector>

#include "tg_internal.h"

namespace {

// Host staging buffer laid out exactly like the device arena.
struct Arena {
  std::vector<char> host;
  size_t add(size_t bytes) {
    size_t off = (host.size() + 255) & ~size_t(255);
    host.resize(off + bytes, 0);
    return off;
  }
  template <class T> T* at(size_t off) { return reinterpret_cast<T*>(host.data() + off); }
};

bool is_pow2_le8(int k) { return k == 1 || k == 2 || k == 4 || k == 8; }

int check_tables(int K, int n_classes, const int32_t* k_list, const int32_t* type_k, const uint32_t* speedup) {
  if (K < 1 || K > TG_MAX_K || !k_list || !type_k || n_classes < 0) return TG_E_INVALID_ARG;
  for (int q = 0; q < K; ++q) {
    if (k_list[q] < 1 || k_list[q] > TG_MAX_UNIT) return TG_E_INVALID_ARG;
    if (q && k_list[q] <= k_list[q - 1]) return TG_E_INVALID_ARG;
  }
  for (int t = 0; t < TG_N_TYPES; ++t)
    if (type_k[t] < 0 || type_k[t] > K) return TG_E_INVALID_ARG;
  if (type_k[TG_TYPE_API] > 1) return TG_E_INVALID_ARG;
  for (int q = 0; q < type_k[TG_TYPE_GPU]; ++q)
    if (!is_pow2_le8(k_list[q])) return TG_E_INVALID_ARG;
  if (n_classes > 0) {
    if (!speedup) return TG_E_INVALID_ARG;
    for (int c = 0; c < n_classes; ++c)
      for (int q = 0; q < K; ++q) {
        const uint32_t s = speedup[c * K + q];
        if (s < 65536u || s > 65536u * (uint32_t)k_list[q]) return TG_E_ELASTICITY;  // 1/k <= E(k) <= 1
        if (q && s < speedup[c * K + q - 1]) return TG_E_ELASTICITY;                 // E(k) k must not shrink
      }
  }
  return TG_OK;
}

int chunk_states(const uint8_t c[4]) {
  int s = 1;
  for (int x = 0; x < 4; ++x) s *= (std::max<int>(c[x], 1) + 1);
  return s;
}

}  // namespace

extern "C" const char* tg_strerror(int code) {
  switch (code) {
    case TG_OK: return "ok";
    case TG_E_INVALID_ARG: return "invalid argument";
    case TG_E_RANGE: return "value outside the supported range";
    case TG_E_ELASTICITY: return "elasticity description violates 0 < E(k) <= 1 or E(k) k nondecreasing";
    case TG_E_WORKSPACE: return "workspace missing, misaligned or too small";
    case TG_E_HIP: return "HIP runtime call failed";
    case TG_E_NOMEM: return "out of memory";
    case TG_E_STATIC_WS: return "the problem needs more workspace than the library's static buffer holds";
    default: return "unknown error";
  }
}

namespace {

// Pooled GPUs (Sec. 5.3, Alg. 4): the first GPU node of every snapshot stands for the pool.  The
// folded description gives it the units, chunks and running actions of all GPU nodes of the
// snapshot and leaves the others with nothing to hand out, so admission, DPArrange, eviction and
// the completion heap run on one resource without knowing about the mode; `real_chunks` keeps
// every node's own chunks for the kernel that hands out the real chunks afterwards.
struct PoolFold {
  std::vector<int32_t> cap, free_, busy_off;
  std::vector<uint8_t> chunks;
  std::vector<int64_t> busy_rel;
  std::vector<uint32_t> real_chunks;
};

int fold_gpu_pool(const tg_problem_desc* d, PoolFold* f) {
  const int B = d->B, N = d->N, M = d->M;
  const size_t nN = (size_t)B * M;
  if (d->act_service) return TG_E_INVALID_ARG;
  for (size_t g = 0; g < (size_t)B * N; ++g)
    if (d->act_type[g] == TG_TYPE_GPU && d->act_pin_node[g] >= 0) return TG_E_INVALID_ARG;
  f->cap.assign(d->node_cap, d->node_cap + nN);
  f->free_.assign(d->node_free, d->node_free + nN);
  f->chunks.assign(nN * 4, 0);
  f->real_chunks.assign(nN, 0);
  f->busy_off.assign(nN + 1, 0);
  std::vector<std::vector<int64_t>> busy(nN);
  for (int b = 0; b < B; ++b) {
    long pool = -1;
    for (int j = 0; j < M; ++j) {
      const size_t g = (size_t)b * M + j;
      if (d->node_busy_off) {
        const int lo = d->node_busy_off[g], hi = d->node_busy_off[g + 1];
        if (lo < 0 || hi < lo || (hi > lo && !d->node_busy_rel_us)) return TG_E_INVALID_ARG;
        busy[g].assign(d->node_busy_rel_us + lo, d->node_busy_rel_us + hi);
      }
      if (d->node_type[g] != TG_TYPE_GPU) continue;
      const int fr = d->node_free[g];
      if (d->node_cap[g] != 8 || fr < 0 || fr > 8 || (int)busy[g].size() > 8 - fr) return TG_E_INVALID_ARG;
      uint8_t ch[4];
      if (d->node_chunks) std::memcpy(ch, d->node_chunks + g * 4, 4);
      else { ch[3] = (uint8_t)(fr / 8); ch[2] = (fr >> 2) & 1; ch[1] = (fr >> 1) & 1; ch[0] = fr & 1; }
      if (ch[0] + 2 * ch[1] + 4 * ch[2] + 8 * ch[3] != fr) return TG_E_INVALID_ARG;
      f->real_chunks[g] = ch[0] | ch[1] << 8 | ch[2] << 16 | (uint32_t)ch[3] << 24;
      if (pool < 0) {
        pool = (long)g;
        std::memcpy(&f->chunks[g * 4], ch, 4);
        continue;
      }
      if (d->node_backlog_us[g] != d->node_backlog_us[pool]) return TG_E_INVALID_ARG;   // a pool has one queueing term
      if (f->cap[pool] + 8 > TG_MAX_GPU_UNITS) return TG_E_RANGE;
      f->cap[pool] += 8; f->free_[pool] += fr; f->free_[g] = 0;
      for (int x = 0; x < 4; ++x) f->chunks[(size_t)pool * 4 + x] += ch[x];
      busy[pool].insert(busy[pool].end(), busy[g].begin(), busy[g].end());
      busy[g].clear();
    }
  }
  for (size_t g = 0; g < nN; ++g) {
    f->busy_off[g + 1] = f->busy_off[g] + (int32_t)busy[g].size();
    f->busy_rel.insert(f->busy_rel.end(), busy[g].begin(), busy[g].end());
  }
  return TG_OK;
}

}  // namespace

namespace {
int build_problem(const tg_problem_desc* desc, void* hip_stream, tg_problem** out);

// nodes_shared: the description holds one node table for all snapshots.  The per-snapshot tables
// the rest of the builder (and every kernel) works on are written out on the host: B copies.
struct SharedNodes {
  std::vector<uint8_t> type, chunks;
  std::vector<int32_t> cap, free_, busy_off, aux;
  std::vector<int64_t> backlog, busy_rel;
  std::vector<uint64_t> resident, cores;
};

template <class T>
const T* tile(const T* src, size_t per, int B, std::vector<T>* dst) {
  if (!src) return nullptr;
  dst->resize(per * B);
  for (int b = 0; b < B; ++b) std::copy(src, src + per, dst->begin() + (size_t)b * per);
  return dst->data();
}
}  // namespace

extern "C" int tg_build_problem(const tg_problem_desc* desc, void* hip_stream, tg_problem** out) {
  if (!desc || !out) return TG_E_INVALID_ARG;
  *out = nullptr;
  if (desc->nodes_shared != 0 && desc->nodes_shared != 1) return TG_E_INVALID_ARG;
  if (desc->reserved_ != 0) return TG_E_INVALID_ARG;
  if (!desc->nodes_shared) return build_problem(desc, hip_stream, out);
  const int B = desc->B, M = desc->M;
  if (B < 1 || M < 1 || (int64_t)B * M >= (1ll << 31)) return B < 1 || M < 1 ? TG_E_INVALID_ARG : TG_E_RANGE;
  try {
    SharedNodes sn;
    tg_problem_desc d = *desc;
    d.nodes_shared = 0;
    d.node_type = tile(desc->node_type, M, B, &sn.type);
    d.node_cap = tile(desc->node_cap, M, B, &sn.cap);
    d.node_free = tile(desc->node_free, M, B, &sn.free_);
    d.node_backlog_us = tile(desc->node_backlog_us, M, B, &sn.backlog);
    d.node_chunks = tile(desc->node_chunks, (size_t)M * 4, B, &sn.chunks);
    d.node_aux_free = tile(desc->node_aux_free, M, B, &sn.aux);
    d.node_resident = tile(desc->node_resident, M, B, &sn.resident);
    d.node_core_free = tile(desc->node_core_free, (size_t)M * 4, B, &sn.cores);
    if (desc->node_busy_off) {                                    // CSR of one table -> CSR of B tables
      const int32_t* off = desc->node_busy_off;
      if (off[0] != 0) return TG_E_INVALID_ARG;
      for (int j = 0; j < M; ++j) if (off[j + 1] < off[j]) return TG_E_INVALID_ARG;
      const int64_t per = off[M];
      if (per * B >= (1ll << 31)) return TG_E_RANGE;
      if (per > 0 && !desc->node_busy_rel_us) return TG_E_INVALID_ARG;
      sn.busy_off.resize((size_t)B * M + 1);
      for (int b = 0; b < B; ++b)
        for (int j = 0; j < M; ++j) sn.busy_off[(size_t)b * M + j] = (int32_t)(b * per + off[j]);
      sn.busy_off[(size_t)B * M] = (int32_t)(B * per);
      d.node_busy_off = sn.busy_off.data();
      d.node_busy_rel_us = per > 0 ? tile(desc->node_busy_rel_us, (size_t)per, B, &sn.busy_rel) : desc->node_busy_rel_us;
    }
    return build_problem(&d, hip_stream, out);
  } catch (const std::bad_alloc&) { return TG_E_NOMEM; }
}

namespace {
int build_problem(const tg_problem_desc* desc, void* hip_stream, tg_problem** out) {
  if (desc->gpu_pooled != 0 && desc->gpu_pooled != 1) return TG_E_INVALID_ARG;
  if (desc->queue_prefix != 0 && desc->queue_prefix != 1) return TG_E_INVALID_ARG;
  tg_problem_desc folded = *desc;
  PoolFold fold;
  if (desc->gpu_pooled) {
    if (desc->B < 1 || desc->N < 1 || desc->M < 1 || (int64_t)desc->B * desc->N >= (1ll << 31) || (int64_t)desc->B * desc->M >= (1ll << 31))
      return TG_E_INVALID_ARG;
    if (!desc->node_type || !desc->node_cap || !desc->node_free || !desc->node_backlog_us || !desc->act_type || !desc->act_pin_node)
      return TG_E_INVALID_ARG;
    try {
      const int rc = fold_gpu_pool(desc, &fold);
      if (rc) return rc;
    } catch (const std::bad_alloc&) { return TG_E_NOMEM; }
    folded.node_cap = fold.cap.data(); folded.node_free = fold.free_.data(); folded.node_chunks = fold.chunks.data();
    folded.node_busy_off = desc->node_busy_off ? fold.busy_off.data() : nullptr;
    folded.node_busy_rel_us = desc->node_busy_off ? fold.busy_rel.data() : nullptr;
  }
  const tg_problem_desc* d = &folded;
  const int B = d->B, N = d->N, M = d->M, K = d->K;
  if (B < 1 || N < 1 || M < 1 || d->n_tasks < 1) return TG_E_INVALID_ARG;
  if (d->order_policy != TG_ORDER_FCFS && d->order_policy != TG_ORDER_COST) return TG_E_INVALID_ARG;
  if (d->depth < 1 || d->depth > TG_MAX_DEPTH) return TG_E_INVALID_ARG;
  if ((int64_t)B * N >= (1ll << 31) || (int64_t)B * M >= (1ll << 31) || N > TG_MAX_ACTIONS) return TG_E_RANGE;
  int rc = check_tables(K, d->n_classes, d->k_list, d->type_k, d->speedup_q16);
  if (rc) return rc;
  if (!d->node_type || !d->node_cap || !d->node_free || !d->node_backlog_us) return TG_E_INVALID_ARG;
  if (!d->act_type || !d->act_model || !d->act_t_ori_us || !d->act_kmask || !d->act_param || !d->act_pin_node)
    return TG_E_INVALID_ARG;
  if (d->node_busy_off && !d->node_busy_rel_us && d->node_busy_off[(size_t)B * M] > 0) return TG_E_INVALID_ARG;
  if ((d->node_aux_free == nullptr) != (d->act_aux == nullptr)) return TG_E_INVALID_ARG;
  const bool svc = d->act_service != nullptr;
  if (svc != (d->node_resident != nullptr) || svc != (d->restore_us != nullptr)) return TG_E_INVALID_ARG;
  if (svc) {
    if (d->n_services < 1 || d->n_services > TG_MAX_SERVICES) return TG_E_INVALID_ARG;
    for (int s = 0; s < d->n_services; ++s) if (d->restore_us[s] < 0 || d->restore_us[s] >= TG_T_ORI_LIMIT) return TG_E_RANGE;
    for (size_t g = 0; g < (size_t)B * N; ++g) if (d->act_service[g] >= d->n_services) return TG_E_INVALID_ARG;
    if (d->n_services < 64)
      for (size_t g = 0; g < (size_t)B * M; ++g) if (d->node_resident[g] >> d->n_services) return TG_E_INVALID_ARG;
  }
  if (d->node_core_free) {
    const int nc = d->numa_cores;
    if (nc < 4 || nc > 64 || (nc & (nc - 1))) return TG_E_INVALID_ARG;
    for (size_t g = 0; g < (size_t)B * M; ++g) {
      if (d->node_type[g] != TG_TYPE_CPU) continue;
      const int cap = d->node_cap[g];
      if (cap < 0 || cap > TG_MAX_CPU_UNITS) continue;       // reported by the node checks below
      int bits = 0;
      for (int w = 0; w < 4; ++w) {
        const uint64_t m = d->node_core_free[g * 4 + w];
        const int lim = cap - 64 * w;                          // cores of this word below the capacity
        if (lim < 64 && (m >> (lim < 0 ? 0 : lim))) return TG_E_INVALID_ARG;
        bits += __builtin_popcountll(m);
      }
      if (bits != d->node_free[g]) return TG_E_INVALID_ARG;
    }
  } else if (d->numa_cores != 0) return TG_E_INVALID_ARG;
  if (d->act_aux) {
    for (size_t g = 0; g < (size_t)B * M; ++g) if (d->node_aux_free[g] < 0) return TG_E_INVALID_ARG;
    for (size_t g = 0; g < (size_t)B * N; ++g) if (d->act_aux[g] < 0) return TG_E_INVALID_ARG;
  }

  const size_t nN = (size_t)B * M, nA = (size_t)B * N;
  tg_problem* p = new (std::nothrow) tg_problem();                  // value-initialised: every plain member is zero
  if (!p) return TG_E_NOMEM;
  Arena ar;
  try {
    // ---------------- nodes
    const size_t o_ntype = ar.add(nN), o_ncap = ar.add(nN * 4), o_nfree = ar.add(nN * 4), o_nback = ar.add(nN * 8),
                 o_nchunk = ar.add(nN * 4), o_nboff = ar.add((nN + 1) * 4), o_nrank = ar.add(nN * 4),
                 o_tnidx = ar.add(nN * 4), o_tnoff = ar.add((size_t)B * 4 * 4);
    const size_t o_asvc = ar.add(svc ? nA * 4 : 0), o_nres = ar.add(svc ? nN * 8 : 0), o_rest = ar.add(svc ? TG_MAX_SERVICES * 8 : 0),
                 o_rowsvc = ar.add(svc ? nA * 8 : 0), o_nresk = ar.add(svc ? nN * 8 : 0);
    if (svc) {
      for (size_t g = 0; g < nA; ++g) ar.at<int32_t>(o_asvc)[g] = d->act_service[g] < 0 ? -1 : d->act_service[g];
      std::memcpy(ar.at<uint64_t>(o_nres), d->node_resident, nN * 8);
      std::memcpy(ar.at<int64_t>(o_rest), d->restore_us, (size_t)d->n_services * 8);
    }
    const size_t o_naux = ar.add(d->act_aux ? nN * 4 : 0), o_aaux = ar.add(d->act_aux ? nA * 4 : 0);
    if (d->act_aux) {
      std::memcpy(ar.at<int32_t>(o_naux), d->node_aux_free, nN * 4);
      std::memcpy(ar.at<int32_t>(o_aaux), d->act_aux, nA * 4);
    }
    const size_t o_nchreal = ar.add(d->gpu_pooled ? nN * 4 : 0);
    if (d->gpu_pooled) std::memcpy(ar.at<uint32_t>(o_nchreal), fold.real_chunks.data(), nN * 4);
    const size_t o_aquota = ar.add(d->act_quota_mask ? nA * 8 : 0);
    if (d->act_quota_mask) std::memcpy(ar.at<uint64_t>(o_aquota), d->act_quota_mask, nA * 8);
    const size_t o_ncores = ar.add(d->node_core_free ? nN * 32 : 0);
    if (d->node_core_free) std::memcpy(ar.at<uint64_t>(o_ncores), d->node_core_free, nN * 32);
    const size_t n_busy = d->node_busy_off ? (size_t)d->node_busy_off[nN] : 0;
    const size_t o_nbrel = ar.add(std::max<size_t>(n_busy, 1) * 8);
    std::vector<int> max_cap((size_t)B * 3, -1);
    int max_other = 0;                                            // most GPU nodes or quotas of a snapshot
    int max_kind = 0, max_free_cpu = 0, max_heap = 0, max_free_gpu = 0, max_states = 1;
    size_t free_gt16 = 0, free_gt64 = 0, nodes_by_actions_gt64 = 0;
    int64_t backlog_spread = 0;
    for (int b = 0; b < B; ++b) {
      int cnt[3] = {0, 0, 0};
      int64_t bl_lo[3] = {TG_INF, TG_INF, TG_INF}, bl_hi[3] = {0, 0, 0};
      for (int j = 0; j < M; ++j) {
        const size_t g = (size_t)b * M + j;
        const int t = d->node_type[g], cap = d->node_cap[g], fr = d->node_free[g];
        if (t >= TG_N_TYPES || cap < 0 || fr < 0 || fr > cap) { delete p; return TG_E_INVALID_ARG; }
        if ((t == TG_TYPE_CPU && cap > TG_MAX_CPU_UNITS) || (t == TG_TYPE_GPU && cap > TG_MAX_GPU_UNITS)) { delete p; return TG_E_RANGE; }
        const int64_t bl = d->node_backlog_us[g];
        if (bl < 0 || bl >= TG_TIME_LIMIT) { delete p; return TG_E_RANGE; }
        bl_lo[t] = std::min(bl_lo[t], bl); bl_hi[t] = std::max(bl_hi[t], bl);
        int nb = 0;
        if (d->node_busy_off) {
          nb = d->node_busy_off[g + 1] - d->node_busy_off[g];
          if (nb < 0 || d->node_busy_off[0] != 0) { delete p; return TG_E_INVALID_ARG; }
          if (nb > 0 && (t == TG_TYPE_API || nb > cap - fr)) { delete p; return TG_E_INVALID_ARG; }
          for (int x = 0; x < nb; ++x) {
            const int64_t r = d->node_busy_rel_us[d->node_busy_off[g] + x];
            if (r < 0 || r >= TG_TIME_LIMIT) { delete p; return TG_E_RANGE; }
          }
        }
        uint8_t ch[4] = {0, 0, 0, 0};
        if (t == TG_TYPE_GPU) {
          if (d->node_chunks) std::memcpy(ch, d->node_chunks + g * 4, 4);
          else { ch[3] = (uint8_t)(fr / 8); ch[2] = (fr >> 2) & 1; ch[1] = (fr >> 1) & 1; ch[0] = fr & 1; }
          if (ch[0] + 2 * ch[1] + 4 * ch[2] + 8 * ch[3] != fr) { delete p; return TG_E_INVALID_ARG; }
          if (chunk_states(ch) > TG_MAX_CHUNK_STATES) { delete p; return TG_E_RANGE; }
          max_states = std::max(max_states, chunk_states(ch));
          max_free_gpu = std::max(max_free_gpu, fr);
        }
        if (t == TG_TYPE_CPU) max_free_cpu = std::max(max_free_cpu, fr);
        if (t != TG_TYPE_API) max_heap = std::max(max_heap, fr + nb);
        free_gt16 += fr > 16; free_gt64 += fr > 64;
        ar.at<uint8_t>(o_ntype)[g] = (uint8_t)t;
        ar.at<int32_t>(o_ncap)[g] = cap;
        ar.at<int32_t>(o_nfree)[g] = fr;
        ar.at<int64_t>(o_nback)[g] = bl;
        ar.at<uint32_t>(o_nchunk)[g] = ch[0] | ch[1] << 8 | ch[2] << 16 | (uint32_t)ch[3] << 24;
        ar.at<int32_t>(o_nboff)[g] = d->node_busy_off ? d->node_busy_off[g] : 0;
        ar.at<int32_t>(o_nrank)[g] = cnt[t]++;
        max_cap[(size_t)b * 3 + t] = std::max(max_cap[(size_t)b * 3 + t], cap);
      }
      int32_t* off = ar.at<int32_t>(o_tnoff) + (size_t)b * 4;
      off[0] = 0; off[1] = cnt[0]; off[2] = cnt[0] + cnt[1]; off[3] = M;
      int fill[3] = {off[0], off[1], off[2]};
      for (int j = 0; j < M; ++j) {
        const int t = d->node_type[(size_t)b * M + j];
        ar.at<int32_t>(o_tnidx)[(size_t)b * M + fill[t]++] = j;
      }
      for (int t = 0; t < 3; ++t) max_kind = std::max(max_kind, cnt[t]);
      max_other = std::max({max_other, cnt[TG_TYPE_GPU], cnt[TG_TYPE_API]});
      for (int t = 0; t < 3; ++t) if (cnt[t]) backlog_spread = std::max(backlog_spread, bl_hi[t] - bl_lo[t]);
      if (max_kind > TG_MAX_NODES_OF_KIND) { delete p; return TG_E_RANGE; }
    }
    ar.at<int32_t>(o_nboff)[nN] = (int32_t)n_busy;
    if (n_busy) std::memcpy(ar.at<int64_t>(o_nbrel), d->node_busy_rel_us, n_busy * 8);

    // ---------------- actions
    int max_acts_kind = 0;
    const size_t o_atype = ar.add(nA), o_amodel = ar.add(nA), o_astat = ar.add(nA), o_aT = ar.add(nA * 8),
                 o_aage = ar.add(nA * 8), o_amask = ar.add(nA * 4), o_aparam = ar.add(nA * 4), o_apin = ar.add(nA * 4),
                 o_atask = ar.add(nA * 4), o_taidx = ar.add(nA * 4), o_taoff = ar.add((size_t)B * 4 * 4),
                 o_apinrank = ar.add(nA * 4);
    for (int b = 0; b < B; ++b) {
      int cnt[3] = {0, 0, 0};
      int64_t sumT = 0;
      for (int i = 0; i < N; ++i) {
        const size_t g = (size_t)b * N + i;
        const int t = d->act_type[g], model = d->act_model[g];
        if (t >= TG_N_TYPES || model > TG_MODEL_TABLE) { delete p; return TG_E_INVALID_ARG; }
        if (t == TG_TYPE_API && model != TG_MODEL_NONE) { delete p; return TG_E_INVALID_ARG; }
        const int64_t T = d->act_t_ori_us[g], age = d->act_age_us ? d->act_age_us[g] : 0;
        if (T < 1 || T >= TG_T_ORI_LIMIT || age < 0 || age >= TG_TIME_LIMIT) { delete p; return TG_E_RANGE; }
        sumT += T;
        const uint32_t param = d->act_param[g];
        if (model == TG_MODEL_AMDAHL && param > 1000000u) { delete p; return TG_E_ELASTICITY; }
        if (model == TG_MODEL_TABLE && param >= (uint32_t)d->n_classes) { delete p; return TG_E_ELASTICITY; }
        const int task = d->act_task ? d->act_task[g] : 0;
        if (task < 0 || task >= d->n_tasks) { delete p; return TG_E_INVALID_ARG; }
        uint32_t mask = d->act_kmask[g] & ((1u << d->type_k[t]) - 1u);
        if (model == TG_MODEL_NONE) mask &= (~mask + 1u);            // minimum units only
        int pin = d->act_pin_node[g];
        if (pin < 0) pin = -1;
        bool infeasible = mask == 0;
        if (!infeasible) {
          const int kmin = d->k_list[__builtin_ctz(mask)];
          if (pin >= 0) infeasible = pin >= M || d->node_type[(size_t)b * M + pin] != t || kmin > d->node_cap[(size_t)b * M + pin];
          else infeasible = kmin > max_cap[(size_t)b * 3 + t];
        }
        if (d->act_quota_mask && d->act_quota_mask[g]) {             // further quotas: a pinned API action names other API nodes
          const uint64_t more = d->act_quota_mask[g];
          const int32_t* tn = ar.at<int32_t>(o_tnoff) + (size_t)b * 4;
          const int n_api = tn[3] - tn[2];
          const bool pinned_api = t == TG_TYPE_API && pin >= 0 && pin < M && d->node_type[(size_t)b * M + pin] == TG_TYPE_API;
          if (!pinned_api || (n_api < 64 && (more >> n_api)) || (more >> ar.at<int32_t>(o_nrank)[(size_t)b * M + pin] & 1ull)) {
            delete p;
            return TG_E_INVALID_ARG;
          }
        }
        if (pin >= M) pin = M;                                       // any out-of-range pin: matches no node
        ar.at<uint8_t>(o_atype)[g] = (uint8_t)t;
        ar.at<uint8_t>(o_amodel)[g] = (uint8_t)model;
        ar.at<uint8_t>(o_astat)[g] = infeasible;
        ar.at<int64_t>(o_aT)[g] = T;
        ar.at<int64_t>(o_aage)[g] = age;
        ar.at<uint32_t>(o_amask)[g] = mask;
        ar.at<uint32_t>(o_aparam)[g] = param;
        ar.at<int32_t>(o_apin)[g] = pin;
        ar.at<int32_t>(o_apinrank)[g] = pin >= 0 && !infeasible ? ar.at<int32_t>(o_nrank)[(size_t)b * M + pin] : -1;
        ar.at<int32_t>(o_atask)[g] = task;
        ++cnt[t];
      }
      if (sumT >= TG_SUM_T_LIMIT) { delete p; return TG_E_RANGE; }
      for (int t = 0; t < 3; ++t) max_acts_kind = std::max(max_acts_kind, cnt[t]);
      for (int t = 0; t < 3; ++t) nodes_by_actions_gt64 += (size_t)cnt[t] / 65;   // a node with more than 64 candidates needs 65 actions of its kind
      int32_t* off = ar.at<int32_t>(o_taoff) + (size_t)b * 4;
      off[0] = 0; off[1] = cnt[0]; off[2] = cnt[0] + cnt[1]; off[3] = N;
      int fill[3] = {off[0], off[1], off[2]};
      for (int i = 0; i < N; ++i) {
        const int t = d->act_type[(size_t)b * N + i];
        ar.at<int32_t>(o_taidx)[(size_t)b * N + fill[t]++] = i;
      }
    }
    const size_t o_speed = ar.add(std::max<size_t>((size_t)d->n_classes * K, 1) * 4);
    if (d->n_classes) std::memcpy(ar.at<uint32_t>(o_speed), d->speedup_q16, (size_t)d->n_classes * K * 4);

    // ---------------- blocks of the score tensor and the score kernel's work split
    const size_t o_blocks = ar.add((size_t)B * 3 * sizeof(TgBlock));
    const size_t o_rowrec = ar.add(nA * sizeof(TgRowRec)), o_rowpin = ar.add(nA * 4), o_nword = ar.add(nN * 8);
    const size_t o_snaps = ar.add((size_t)B * sizeof(TgScoreSnap));
    int64_t total = 0;
    std::vector<int32_t> snap_chunks((size_t)B, 0);
    for (int b = 0; b < B; ++b)
      for (int t = 0; t < 3; ++t) {
        TgBlock& k = ar.at<TgBlock>(o_blocks)[(size_t)b * 3 + t];
        const int32_t* ta = ar.at<int32_t>(o_taoff) + (size_t)b * 4;
        const int32_t* tn = ar.at<int32_t>(o_tnoff) + (size_t)b * 4;
        k.b = b; k.t = t; k.rows = ta[t + 1] - ta[t]; k.M_t = tn[t + 1] - tn[t]; k.K_t = d->type_k[t];
        k.a_off = (int32_t)((size_t)b * N + ta[t]); k.n_off = (int32_t)((size_t)b * M + tn[t]);
        k.entries = (int64_t)k.rows * k.M_t * k.K_t;
        if (k.entries >= (1ll << 31) - (1 << 20)) { delete p; return TG_E_RANGE; }   // 32-bit indices inside a block
        const uint32_t lr = (uint32_t)(k.M_t * k.K_t);
        k.cost_off = total;
        total += k.entries;
        TgScoreKind& sk = ar.at<TgScoreSnap>(o_snaps)[b].kind[t];
        sk.cost_off = k.cost_off; sk.inv_lr = lr ? 1.0 / (double)lr : 0.0; sk.entries = (int32_t)k.entries;
        sk.a_off = k.a_off; sk.n_off = k.n_off; sk.M_t = (uint16_t)k.M_t; sk.K_t = (uint16_t)k.K_t;
        sk.magic_k = k.K_t ? (1u << 20) / (uint32_t)k.K_t + 1u : 0u; sk.rows = k.rows;
        if (k.entries) {
          snap_chunks[b] += (int32_t)((k.entries + (k.cost_off & 1) + TG_SCORE_CHUNK - 1) / TG_SCORE_CHUNK);
        }
        if (t == 2) ar.at<TgScoreSnap>(o_snaps)[b].chunks = snap_chunks[b];
        // kind-grouped views: row of every action, pin rank per row, node word per rank
        for (int r = 0; r < k.rows; ++r) {
          const int i = ar.at<int32_t>(o_taidx)[(size_t)b * N + ta[t] + r];
          const size_t g = (size_t)b * N + i;
          TgRowRec& rr = ar.at<TgRowRec>(o_rowrec)[(size_t)b * N + ta[t] + r];
          rr.T = ar.at<int64_t>(o_aT)[g]; rr.param = ar.at<uint32_t>(o_aparam)[g];
          rr.kmask = (uint16_t)ar.at<uint32_t>(o_amask)[g]; rr.model = ar.at<uint8_t>(o_amodel)[g]; rr.pad_ = 0;
          const int pin = ar.at<int32_t>(o_apin)[g];
          int pr = -1;
          if (pin >= 0) pr = (pin < M && d->node_type[(size_t)b * M + pin] == t) ? ar.at<int32_t>(o_nrank)[(size_t)b * M + pin] : -2;
          ar.at<int32_t>(o_rowpin)[(size_t)b * N + ta[t] + r] = pr;
          if (svc) {
            const int sv = ar.at<int32_t>(o_asvc)[g];
            ar.at<uint64_t>(o_rowsvc)[(size_t)b * N + ta[t] + r] = sv < 0 ? 0ull : (uint64_t)d->restore_us[sv] | (uint64_t)(sv + 1) << 48;
          }
        }
        for (int r = 0; r < k.M_t; ++r) {
          const size_t g = (size_t)b * M + ar.at<int32_t>(o_tnidx)[(size_t)b * M + tn[t] + r];
          uint64_t qmax = 0;
          while ((int)qmax < k.K_t && d->k_list[qmax] <= d->node_cap[g]) ++qmax;
          ar.at<uint64_t>(o_nword)[(size_t)b * M + tn[t] + r] = (uint64_t)d->node_backlog_us[g] | qmax << 48;
          if (svc) ar.at<uint64_t>(o_nresk)[(size_t)b * M + tn[t] + r] = d->node_resident[g];
        }
      }
    // The score kernel runs on a grid (chunk, snapshot) as wide as the largest snapshot of the launch: one launch
    // over all snapshots in index order (workgroups then start in the order of the tensor) unless that leaves more
    // than an eighth of the grid without a chunk; then the snapshots are sorted by size and launched in groups
    // inside which the same bound holds.
    std::vector<TgScoreLaunch> launches;
    auto add_launch = [&](int first, int count, int max_chunks) {     // the grid's second dimension holds at most 65535 snapshots
      for (int x = 0; x < count; x += 65535) launches.push_back({first + x, std::min(65535, count - x), max_chunks});
    };
    {
      int64_t sum = 0;
      int mx = 0;
      for (int b = 0; b < B; ++b) { sum += snap_chunks[b]; mx = std::max(mx, snap_chunks[b]); }
      const int64_t slack = 4096;
      if (mx > 0 && (int64_t)mx * B <= sum + sum / 8 + slack) add_launch(0, B, mx);
      else if (mx > 0) {
        std::vector<int> order((size_t)B);
        for (int b = 0; b < B; ++b) order[b] = b;
        std::stable_sort(order.begin(), order.end(), [&](int a, int c) { return snap_chunks[a] > snap_chunks[c]; });
        std::vector<TgScoreSnap> sorted((size_t)B);
        for (int x = 0; x < B; ++x) sorted[x] = ar.at<TgScoreSnap>(o_snaps)[order[x]];
        std::memcpy(ar.at<TgScoreSnap>(o_snaps), sorted.data(), (size_t)B * sizeof(TgScoreSnap));
        int first = 0;
        while (first < B && sorted[first].chunks > 0) {
          const int gmax = sorted[first].chunks;
          int64_t gsum = 0;
          int x = first;
          while (x < B && sorted[x].chunks > 0) {                   // extend while the group's grid stays mostly full
            const int64_t s2 = gsum + sorted[x].chunks, cnt = x - first + 1;
            if ((int64_t)gmax * cnt > s2 + s2 / 8 + slack) break;
            gsum = s2; ++x;
          }
          add_launch(first, x - first, gmax);
          first = x;
        }
      }
    }

    // ---------------- ship
    p->arena_bytes = ar.host.size();
    if (nA * (size_t)(K + 1) >= (1ull << 31)) { delete p; return TG_E_RANGE; }  // the slots of the score scratch are indexed in 32 bits
    if (hipMalloc(&p->d_arena, p->arena_bytes) != hipSuccess) { delete p; return TG_E_NOMEM; }
    if (hipMalloc((void**)&p->d_score_dur, std::max<size_t>(nA * (K + 1), 1) * 8) != hipSuccess) { (void)hipFree(p->d_arena); delete p; return TG_E_NOMEM; }
    hipStream_t s = (hipStream_t)hip_stream;
    if (hipMemcpyAsync(p->d_arena, ar.host.data(), ar.host.size(), hipMemcpyHostToDevice, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) {
      (void)hipFree(p->d_arena); (void)hipFree(p->d_score_dur); delete p; return TG_E_HIP;
    }
    bool ok = hipEventCreateWithFlags(&p->ev_fork, hipEventDisableTiming) == hipSuccess;
    for (int i = 0; i < 2 && ok; ++i)
      ok = hipStreamCreateWithFlags(&p->side_stream[i], hipStreamNonBlocking) == hipSuccess &&
           hipEventCreateWithFlags(&p->ev_join[i], hipEventDisableTiming) == hipSuccess;
    ok = ok && hipStreamCreateWithFlags(&p->score_stream, hipStreamNonBlocking) == hipSuccess &&
         hipEventCreateWithFlags(&p->ev_score_fork, hipEventDisableTiming) == hipSuccess &&
         hipEventCreateWithFlags(&p->ev_score_done, hipEventDisableTiming) == hipSuccess;
    if (!ok) { tg_free_problem(p); return TG_E_HIP; }
    char* base = (char*)p->d_arena;
    TgDev& v = p->dev;
    v.B = B; v.N = N; v.M = M; v.K = K; v.n_classes = d->n_classes; v.n_tasks = d->n_tasks; v.depth = d->depth;
    v.has_busy = n_busy > 0;
    for (int q = 0; q < TG_MAX_K; ++q) v.k_list[q] = q < K ? d->k_list[q] : 0;
    for (int t = 0; t < 3; ++t) v.type_k[t] = d->type_k[t];
    v.type_k[3] = 0;
    v.node_type = (const uint8_t*)(base + o_ntype); v.node_cap = (const int32_t*)(base + o_ncap);
    v.node_free = (const int32_t*)(base + o_nfree); v.node_backlog = (const int64_t*)(base + o_nback);
    v.node_chunks = (const uint32_t*)(base + o_nchunk); v.node_busy_off = (const int32_t*)(base + o_nboff);
    v.node_busy_rel = (const int64_t*)(base + o_nbrel); v.node_rank = (const int32_t*)(base + o_nrank);
    v.act_type = (const uint8_t*)(base + o_atype); v.act_model = (const uint8_t*)(base + o_amodel);
    v.act_static = (const uint8_t*)(base + o_astat); v.act_T = (const int64_t*)(base + o_aT);
    v.act_age = (const int64_t*)(base + o_aage); v.act_kmask = (const uint32_t*)(base + o_amask);
    v.act_param = (const uint32_t*)(base + o_aparam); v.act_pin = (const int32_t*)(base + o_apin);
    v.act_pin_rank = (const int32_t*)(base + o_apinrank);
    v.act_service = svc ? (const int32_t*)(base + o_asvc) : nullptr;
    v.node_resident = svc ? (const uint64_t*)(base + o_nres) : nullptr;
    v.restore = svc ? (const int64_t*)(base + o_rest) : nullptr;
    v.row_svc = svc ? (const uint64_t*)(base + o_rowsvc) : nullptr;
    v.node_res_k = svc ? (const uint64_t*)(base + o_nresk) : nullptr;
    v.node_chunks_real = d->gpu_pooled ? (const uint32_t*)(base + o_nchreal) : nullptr;
    v.act_quota = d->act_quota_mask ? (const uint64_t*)(base + o_aquota) : nullptr;
    v.node_cores = d->node_core_free ? (const uint64_t*)(base + o_ncores) : nullptr;
    v.numa_cores = d->node_core_free ? d->numa_cores : 0;
    v.node_aux = d->act_aux ? (const int32_t*)(base + o_naux) : nullptr;
    v.act_aux = d->act_aux ? (const int32_t*)(base + o_aaux) : nullptr;
    v.act_task = (const int32_t*)(base + o_atask); v.speedup = (const uint32_t*)(base + o_speed);
    v.tact_idx = (const int32_t*)(base + o_taidx); v.tact_off = (const int32_t*)(base + o_taoff);
    v.tnode_idx = (const int32_t*)(base + o_tnidx); v.tnode_off = (const int32_t*)(base + o_tnoff);
    v.row_rec = (const TgRowRec*)(base + o_rowrec); v.row_pin = (const int32_t*)(base + o_rowpin);
    v.node_word = (const uint64_t*)(base + o_nword);
    p->d_blocks = (TgBlock*)(base + o_blocks);
    p->d_score_snaps = (const TgScoreSnap*)(base + o_snaps);
    p->score_launches = launches;
    p->n_blocks = B * 3;
    p->n_candidates = total;
    p->max_nodes_of_kind = max_kind;
    p->max_nodes_not_cpu = max_other;
    p->backlog_spread = backlog_spread;
    p->order_policy = d->order_policy; p->queue_prefix = d->queue_prefix; p->max_actions_of_kind = max_acts_kind;
    p->max_free_cpu = max_free_cpu;
    p->max_heap = max_heap;
    p->nodes_free_gt16 = free_gt16; p->nodes_free_gt64 = std::min(free_gt64, nodes_by_actions_gt64);
    p->max_free_gpu = max_free_gpu;
    p->max_chunk_states = max_states;

  } catch (const std::bad_alloc&) {
    tg_free_problem(p);
    return TG_E_NOMEM;
  }
  *out = p;
  return TG_OK;
}
}  // namespace

extern "C" void tg_free_problem(tg_problem* p) {
  if (!p) return;
  if (p->d_arena) (void)hipFree(p->d_arena);
  if (p->d_score_dur) (void)hipFree(p->d_score_dur);
  for (int i = 0; i < 2; ++i) {
    if (p->side_stream[i]) (void)hipStreamDestroy(p->side_stream[i]);
    if (p->ev_join[i]) (void)hipEventDestroy(p->ev_join[i]);
  }
  if (p->ev_fork) (void)hipEventDestroy(p->ev_fork);
  if (p->score_stream) (void)hipStreamDestroy(p->score_stream);
  if (p->ev_score_fork) (void)hipEventDestroy(p->ev_score_fork);
  if (p->ev_score_done) (void)hipEventDestroy(p->ev_score_done);
  delete p;
}

extern "C" int tg_num_candidates(const tg_problem* p, int64_t* count, int64_t* bytes) {
  if (!p) return TG_E_INVALID_ARG;
  if (count) *count = p->n_candidates;
  if (bytes) *bytes = p->n_candidates * 8;
  return TG_OK;
}
