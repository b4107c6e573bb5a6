// tg_score_candidates: estimated completion time of every (action, node, unit option)
// candidate - Eq. 1 (duration on k units) inside Eq. 2 (queueing + execution) of the paper -
// written as one dense int64 tensor.
//
// The kernel is a pure write stream (8 bytes per candidate, inputs are ~0.1 byte per
// candidate), so it is organised around 16-byte fully coalesced stores:
//   * a workgroup (256 lanes) owns one contiguous span of 4096 entries of one (snapshot, kind)
//     block; one table lookup tells it which;
//   * it evaluates Eq. 1 once per (row, option) of its span into LDS from kind-grouped 16-byte
//     action records, and stages the node words (backlog | options the capacity admits) and the
//     pin ranks of its rows - all prepared at build time, so the dependent-load chain before
//     the first store is three loads deep;
//   * then every lane walks the span in 8 steps of 512 entries, two adjacent entries (one
//     16-byte non-temporal store) per lane and step, keeping its (row, node, option)
//     coordinates by mixed-radix increments.
#include "tg_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kStep = 2 * kThreads;

// SVC: the problem has services (Sec. 5.3): an entry whose action calls a service that is not
// resident on the node carries the service's restore time on top of Eq. 2.
template <bool SVC>
__global__ __launch_bounds__(kThreads) void tg_score_kernel(TgDev P, const TgBlock* __restrict__ blocks,
                                                            const int32_t* __restrict__ wg_block, int lds_nodes,
                                                            int dur_slots, int row_slots, int64_t* __restrict__ cost) {
  extern __shared__ __align__(16) unsigned char smem[];
  int64_t* s_dur = reinterpret_cast<int64_t*>(smem);                    // [dur_slots]
  uint64_t* s_node = reinterpret_cast<uint64_t*>(s_dur + dur_slots);     // [lds_nodes]
  uint64_t* s_res = s_node + lds_nodes;                                  // [lds_nodes]  services resident on the node   (SVC)
  uint64_t* s_rsvc = s_res + (SVC ? lds_nodes : 0);                      // [row_slots]  restore time | (service+1) << 48 (SVC)
  int32_t* s_pin = reinterpret_cast<int32_t*>(s_rsvc + (SVC ? ((row_slots + 1) & ~1) : 0));   // [row_slots]

  const int wg = blockIdx.x;
  const TgBlock blk = blocks[wg_block[wg]];
  const int K = blk.K_t, Mt = blk.M_t;
  const uint32_t Lr = (uint32_t)(Mt * K);
  // Every block has fewer than 2^31 entries, so all index arithmetic is 32-bit.  Lanes own
  // adjacent pairs aligned to 16 bytes in the whole tensor: when the block starts at an odd
  // entry the spans are shifted down by one and entry -1 does not exist.
  const int n = (int)blk.entries;
  const int odd = (int)(blk.cost_off & 1);
  const int e0 = (wg - blk.wg_off) * TG_SCORE_SPAN - odd;              // may be -1
  const int e1 = min(n, e0 + TG_SCORE_SPAN);
  const int f0 = e0 < 0 ? 0 : e0;                                       // first existing entry
  const int row0 = (int)((uint32_t)f0 / Lr), row1 = (int)((uint32_t)(e1 - 1) / Lr);
  const int nrows = row1 - row0 + 1;
  // node window: a single partial row needs only the nodes it touches
  int j0 = 0, j1 = Mt - 1;
  if (nrows == 1) { j0 = (int)(((uint32_t)f0 - (uint32_t)row0 * Lr) / (uint32_t)K); j1 = (int)(((uint32_t)(e1 - 1) - (uint32_t)row0 * Lr) / (uint32_t)K); }

  const TgRowRec* recs = P.row_rec + blk.a_off + row0;
  const int32_t* pins = P.row_pin + blk.a_off + row0;
  const uint64_t* words = P.node_word + blk.n_off;
  const int tid = threadIdx.x;

  for (int x = tid; x < nrows * K; x += kThreads) {
    const int r = x / K, q = x - r * K;
    const TgRowRec rec = recs[r];
    int64_t d = TG_INF;
    if (rec.kmask >> q & 1u) {
      const uint32_t sp = rec.model == TG_MODEL_TABLE ? P.speedup[rec.param * P.K + q] : 0u;
      d = tg_duration(rec.model, rec.T, rec.param, P.k_list[q], sp);
    }
    s_dur[x] = d;
  }
  for (int r = tid; r < nrows; r += kThreads) s_pin[r] = pins[r];
  for (int j = j0 + tid; j <= j1; j += kThreads) s_node[j - j0] = words[j];
  if (SVC) {
    for (int r = tid; r < nrows; r += kThreads) s_rsvc[r] = P.row_svc[blk.a_off + row0 + r];
    for (int j = j0 + tid; j <= j1; j += kThreads) s_res[j - j0] = P.node_res_k[blk.n_off + j];
  }
  __syncthreads();

  int64_t* out = cost + blk.cost_off;
  // coordinates of this lane's first entry, and of a step of 512 entries, in radix (row, Mt, K)
  int e = e0 + 2 * tid;
  const uint32_t ec = (uint32_t)(e < 0 ? 0 : e);
  int row = (int)(ec / Lr);
  const uint32_t col = ec - (uint32_t)row * Lr;
  int j = (int)(col / (uint32_t)K), q = (int)(col - (uint32_t)j * (uint32_t)K);
  if (e < 0 && --q < 0) {                                              // step back to the entry before the block
    q = K - 1;
    if (--j < 0) { j = Mt - 1; --row; }
  }
  const int srow = (int)((uint32_t)kStep / Lr), srem = kStep - srow * (int)Lr, sj = srem / K, sq = srem - sj * K;

  for (; e < e1; e += kStep) {
    int64_t v[2];
    int rr = row, jj = j, qq = q;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      if (h == 1) {
        if (++qq == K) { qq = 0; if (++jj == Mt) { jj = 0; ++rr; } }
      }
      int64_t val = TG_INF;
      if (e + h >= 0 && e + h < e1) {
        const uint64_t nw = s_node[jj - j0];
        const int64_t d = s_dur[(rr - row0) * K + qq];
        const int pin = s_pin[rr - row0];
        const bool ok = d != TG_INF && qq < (int)(nw >> 48) && (pin == -1 || pin == jj);
        if (ok) val = (int64_t)(nw & 0xffffffffffffull) + d;
        if (SVC && ok) {
          const uint64_t sw = s_rsvc[rr - row0];
          const int sv = (int)(sw >> 48);                                // service + 1, 0: none
          if (sv && !(s_res[jj - j0] >> (sv - 1) & 1ull)) val += (int64_t)(sw & 0xffffffffffffull);
        }
      }
      v[h] = val;
    }
    if (e >= 0 && e + 1 < e1) {
      int64_t __attribute__((ext_vector_type(2))) pv = {v[0], v[1]};
      __builtin_nontemporal_store(pv, reinterpret_cast<int64_t __attribute__((ext_vector_type(2)))*>(out + e));
    } else {
      if (e >= 0) __builtin_nontemporal_store(v[0], out + e);
      if (e + 1 < e1) __builtin_nontemporal_store(v[1], out + e + 1);
    }
    // advance by one step
    q += sq; if (q >= K) { q -= K; ++j; }
    j += sj; if (j >= Mt) { j -= Mt; ++row; }
    row += srow;
  }
}

}  // namespace

int tg_launch_score(const tg_problem* p, int64_t* d_cost, hipStream_t s) {
  if (p->score_wgs == 0) return TG_OK;
  const bool svc = p->dev.act_service != nullptr;
  const size_t lds = (size_t)p->score_dur_slots * 8 + (size_t)p->score_lds_nodes * 8 + (size_t)p->score_row_slots * 4 +
                     (svc ? (size_t)p->score_lds_nodes * 8 + (size_t)((p->score_row_slots + 1) & ~1) * 8 : 0);
  if (svc)
    hipLaunchKernelGGL(tg_score_kernel<true>, dim3(p->score_wgs), dim3(kThreads), lds, s, p->dev, p->d_blocks, p->d_wg_block,
                       p->score_lds_nodes, p->score_dur_slots, p->score_row_slots, d_cost);
  else
    hipLaunchKernelGGL(tg_score_kernel<false>, dim3(p->score_wgs), dim3(kThreads), lds, s, p->dev, p->d_blocks, p->d_wg_block,
                       p->score_lds_nodes, p->score_dur_slots, p->score_row_slots, d_cost);
  return hipGetLastError() == hipSuccess ? TG_OK : TG_E_HIP;
}

extern "C" int tg_score_candidates(const tg_problem* p, int64_t* d_cost, void* hip_stream) {
  if (!p || (!d_cost && p->n_candidates) || ((uintptr_t)d_cost & 15)) return TG_E_INVALID_ARG;
  return tg_launch_score(p, d_cost, (hipStream_t)hip_stream);
}
