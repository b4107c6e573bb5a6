// Score kernel: estimated completion time of every (action, node, unit option) candidate,
// Eq. 1 (duration on k units) inside Eq. 2 (queueing + execution) of the paper, written as one
// dense int64 tensor.  The kernel is a pure write stream (8 bytes per candidate, inputs are
// ~0.1 byte per candidate), so it is organised around 16-byte fully coalesced stores:
//   * a workgroup owns one contiguous span of one (snapshot, kind) block of the tensor;
//   * it first evaluates Eq. 1 once per (row, option) of its span into LDS, together with the
//     node words (backlog | number of options the node's capacity admits) it needs;
//   * then every lane walks the span in steps of 512 entries, two adjacent entries per lane
//     and step, keeping its (row, node, option) coordinates by mixed-radix increments.
#include "tg_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kDurSlots = 2048;        // (row, option) durations per workgroup
constexpr int kRowSlots = 2048;        // rows per workgroup

__global__ __launch_bounds__(kThreads) void tg_score_kernel(TgDev P, const TgBlock* __restrict__ blocks, int n_blocks,
                                                            int lds_nodes, int64_t* __restrict__ cost) {
  extern __shared__ __align__(16) unsigned char smem[];
  int64_t* s_dur = reinterpret_cast<int64_t*>(smem);                    // [kDurSlots]
  uint64_t* s_node = reinterpret_cast<uint64_t*>(s_dur + kDurSlots);     // [lds_nodes]
  int32_t* s_pin = reinterpret_cast<int32_t*>(s_node + lds_nodes);       // [kRowSlots]

  // which block does this workgroup work on (uniform binary search over the block table)
  int lo = 0, hi = n_blocks - 1;
  const int wg = blockIdx.x;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (blocks[mid].wg_off <= wg) lo = mid; else hi = mid - 1;
  }
  const TgBlock blk = blocks[lo];
  const int K = blk.K_t, Mt = blk.M_t, b = blk.b, t = blk.t;
  const int Lr = Mt * K;
  const int64_t e0 = (int64_t)(wg - blk.wg_off) * blk.span;
  const int64_t e1 = min(blk.entries, e0 + (int64_t)blk.span);
  if (e0 >= e1) return;
  const int row0 = (int)(e0 / Lr), row1 = (int)((e1 - 1) / Lr);
  const int nrows = row1 - row0 + 1;
  // node window: a single partial row needs only the nodes it touches
  int j0 = 0, j1 = Mt - 1;
  if (nrows == 1) { j0 = (int)(e0 - (int64_t)row0 * Lr) / K; j1 = (int)(e1 - 1 - (int64_t)row0 * Lr) / K; }

  const int32_t* acts = P.tact_idx + (size_t)b * P.N + P.tact_off[b * 4 + t];
  const int32_t* nodes = P.tnode_idx + (size_t)b * P.M + P.tnode_off[b * 4 + t];
  const size_t abase = (size_t)b * P.N, nbase = (size_t)b * P.M;
  const int tid = threadIdx.x;

  for (int x = tid; x < nrows * K; x += kThreads) {
    const int r = x / K, q = x - r * K;
    const size_t g = abase + acts[row0 + r];
    int64_t d = TG_INF;
    if (P.act_kmask[g] >> q & 1u) {
      const int model = P.act_model[g];
      const uint32_t param = P.act_param[g];
      const uint32_t sp = model == TG_MODEL_TABLE ? P.speedup[param * P.K + q] : 0u;
      d = tg_duration(model, P.act_T[g], param, P.k_list[q], sp);
    }
    s_dur[x] = d;
  }
  for (int r = tid; r < nrows; r += kThreads) {
    const size_t g = abase + acts[row0 + r];
    const int pin = P.act_pin[g];
    int pr = -1;                                                     // -1: free to choose
    if (pin >= 0) pr = (pin < P.M && P.node_type[nbase + pin] == t) ? P.node_rank[nbase + pin] : -2;
    s_pin[r] = pr;
  }
  for (int j = j0 + tid; j <= j1; j += kThreads) {
    const size_t g = nbase + nodes[j];
    const int cap = P.node_cap[g];
    int qmax = 0;
    while (qmax < K && P.k_list[qmax] <= cap) ++qmax;
    s_node[j - j0] = (uint64_t)P.node_backlog[g] | (uint64_t)qmax << 48;
  }
  __syncthreads();

  // pairs of adjacent entries; a pair never straddles a 16-byte boundary of the tensor
  const int odd = (int)((blk.cost_off + e0) & 1);
  int64_t* out = cost + blk.cost_off;
  // coordinates of this lane's first entry, and of a step of 512 entries, in radix (row, Mt, K)
  int64_t e = e0 - odd + 2 * tid;
  const int64_t ec = e < e0 ? e0 : e;                                // only the lane holding e0-1 differs
  int row = (int)(ec / Lr);
  const int col = (int)(ec - (int64_t)row * Lr);
  int j = col / K, q = col - j * K;
  if (e < e0 && --q < 0) {                                           // step back to the entry before the span
    q = K - 1;
    if (--j < 0) { j = Mt - 1; --row; }
  }
  const int srow = 512 / Lr, srem = 512 - srow * Lr, sj = srem / K, sq = srem - sj * K;

  for (; e < e1; e += 512) {
    int64_t v[2];
    int rr = row, jj = j, qq = q;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      if (h == 1) {
        if (++qq == K) { qq = 0; if (++jj == Mt) { jj = 0; ++rr; } }
      }
      int64_t val = TG_INF;
      if (e + h >= e0 && e + h < e1) {
        const uint64_t nw = s_node[jj - j0];
        const int64_t d = s_dur[(rr - row0) * K + qq];
        const int pin = s_pin[rr - row0];
        const bool ok = d != TG_INF && qq < (int)(nw >> 48) && (pin == -1 || pin == jj);
        if (ok) val = (int64_t)(nw & 0xffffffffffffull) + d;
      }
      v[h] = val;
    }
    if (e >= e0 && e + 1 < e1) {
      int64_t __attribute__((ext_vector_type(2))) pv = {v[0], v[1]};
      __builtin_nontemporal_store(pv, reinterpret_cast<int64_t __attribute__((ext_vector_type(2)))*>(out + e));
    } else {
      if (e >= e0) __builtin_nontemporal_store(v[0], out + e);
      if (e + 1 < e1) __builtin_nontemporal_store(v[1], out + e + 1);
    }
    // advance by 512 entries
    q += sq; if (q >= K) { q -= K; ++j; }
    j += sj; if (j >= Mt) { j -= Mt; ++row; }
    row += srow;
  }
}

}  // namespace

int tg_launch_score(const tg_problem* p, int64_t* d_cost, hipStream_t s) {
  if (p->score_wgs == 0) return TG_OK;
  const size_t lds = (size_t)kDurSlots * 8 + (size_t)p->score_lds_nodes * 8 + (size_t)kRowSlots * 4;
  hipLaunchKernelGGL(tg_score_kernel, dim3(p->score_wgs), dim3(kThreads), lds, s, p->dev, p->d_blocks, p->n_blocks,
                     p->score_lds_nodes, d_cost);
  return hipGetLastError() == hipSuccess ? TG_OK : TG_E_HIP;
}

extern "C" int tg_score_candidates(const tg_problem* p, int64_t* d_cost, void* hip_stream) {
  if (!p || (!d_cost && p->n_candidates) || ((uintptr_t)d_cost & 15)) return TG_E_INVALID_ARG;
  return tg_launch_score(p, d_cost, (hipStream_t)hip_stream);
}
