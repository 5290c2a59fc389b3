// Host-side planning arithmetic of the asynchronous reconfiguration algorithm
// (paper Alg. 1): phase 1 (intermediate configuration, KV budget, feasibility),
// phase 3 (which layers each GPU adds and where their KV comes from), phase 4's
// convergence predicate and phase 5 (layers to delete, post-commit budget).
// Pure host code: no device work, no allocation.  Layer ranges are inclusive
// [first, last]; a GPU with no layers has last < first.
#include <math.h>

#include "pipelive.h"

namespace {

inline bool in_range(int32_t l, int32_t first, int32_t last) { return l >= first && l <= last; }
inline int32_t range_len(int32_t first, int32_t last) { return last >= first ? last - first + 1 : 0; }

// |[a0,a1] U [b0,b1]|
inline int32_t union_len(int32_t a0, int32_t a1, int32_t b0, int32_t b1) {
  const int32_t la = range_len(a0, a1), lb = range_len(b0, b1);
  if (la == 0) return lb;
  if (lb == 0) return la;
  const int32_t lo = a0 > b0 ? a0 : b0, hi = a1 < b1 ? a1 : b1;
  return la + lb - range_len(lo, hi);
}

}  // namespace

extern "C" {

int32_t pipelive_plan_reconfig(int32_t num_gpus, const int32_t *cur_first, const int32_t *cur_last,
                               const int32_t *tgt_first, const int32_t *tgt_last,
                               const double *mem_bytes, double util, double weight_bytes_per_layer,
                               double block_bytes_per_layer, int64_t blocks_in_use,
                               int64_t cur_blocks, pipelive_reconfig_plan_t *plan, int32_t *mig,
                               int32_t max_mig, int32_t *del, int32_t max_del) {
  if (num_gpus <= 0 || !cur_first || !cur_last || !tgt_first || !tgt_last || !mem_bytes || !plan)
    return PIPELIVE_E_INVAL;
  if (max_mig < 0 || max_del < 0 || (max_mig > 0 && !mig) || (max_del > 0 && !del))
    return PIPELIVE_E_INVAL;
  pipelive_reconfig_plan_t out;
  out.feasible = 0;
  out.need_shrink = 0;
  out.n_mig = 0;
  out.n_del = 0;
  // phase 1: B_shrink = min_i MaxBlocks(i, |C_cur[i] U C_tgt[i]|); phase 5: B_new over C_tgt
  int64_t b_shrink = -1, b_new = -1;
  for (int i = 0; i < num_gpus; ++i) {
    const int32_t n_tmp = union_len(cur_first[i], cur_last[i], tgt_first[i], tgt_last[i]);
    const int32_t n_tgt = range_len(tgt_first[i], tgt_last[i]);
    if (n_tmp > 0) {
      const int64_t b = pipelive_max_blocks(mem_bytes[i], util, n_tmp, weight_bytes_per_layer, block_bytes_per_layer);
      if (b_shrink < 0 || b < b_shrink) b_shrink = b;
    }
    if (n_tgt > 0) {
      const int64_t b = pipelive_max_blocks(mem_bytes[i], util, n_tgt, weight_bytes_per_layer, block_bytes_per_layer);
      if (b_new < 0 || b < b_new) b_new = b;
    }
  }
  out.b_shrink = b_shrink < 0 ? 0 : b_shrink;
  out.b_new = b_new < 0 ? 0 : b_new;
  out.feasible = blocks_in_use <= out.b_shrink ? 1 : 0;
  out.need_shrink = out.b_shrink < cur_blocks ? 1 : 0;
  // phase 3: every layer a GPU gains comes from the GPU that owns it now
  int32_t rc = PIPELIVE_OK;
  for (int dst = 0; dst < num_gpus; ++dst) {
    for (int32_t l = tgt_first[dst]; l <= tgt_last[dst]; ++l) {
      if (in_range(l, cur_first[dst], cur_last[dst])) continue;
      int src = -1;
      for (int j = 0; j < num_gpus; ++j)
        if (in_range(l, cur_first[j], cur_last[j])) src = j;
      if (src < 0) return PIPELIVE_E_RANGE;  // target asks for a layer nobody holds
      if (out.n_mig < max_mig) {
        mig[3 * out.n_mig + 0] = src;
        mig[3 * out.n_mig + 1] = dst;
        mig[3 * out.n_mig + 2] = l;
      } else {
        rc = PIPELIVE_E_NOSPACE;
      }
      ++out.n_mig;
    }
  }
  // phase 5: M_del(i) = (C_cur[i] U C_tgt[i]) \ C_tgt[i]
  for (int i = 0; i < num_gpus; ++i) {
    for (int32_t l = cur_first[i]; l <= cur_last[i]; ++l) {
      if (in_range(l, tgt_first[i], tgt_last[i])) continue;
      if (out.n_del < max_del) {
        del[2 * out.n_del + 0] = i;
        del[2 * out.n_del + 1] = l;
      } else {
        rc = PIPELIVE_E_NOSPACE;
      }
      ++out.n_del;
    }
  }
  *plan = out;
  return rc;
}

int32_t pipelive_converged(int64_t t_sched, const int64_t *t_applied, int32_t n, int64_t tau) {
  if (n < 0 || (n > 0 && !t_applied)) return PIPELIVE_E_INVAL;
  for (int i = 0; i < n; ++i)
    if (t_sched - t_applied[i] >= tau) return 0;
  return 1;
}

double pipelive_kv_utilization(const int32_t *ctx_lens, int64_t n, int32_t block_tokens) {
  if (!ctx_lens || n <= 0 || block_tokens <= 0) return 1.0;
  int64_t tokens = 0, slots = 0;
  for (int64_t s = 0; s < n; ++s) {
    const int64_t c = ctx_lens[s] > 0 ? ctx_lens[s] : 0;
    tokens += c;
    slots += (c + block_tokens - 1) / block_tokens * block_tokens;
  }
  return slots == 0 ? 1.0 : (double)tokens / (double)slots;
}

int64_t pipelive_stacked_block_tokens(size_t phys_block_bytes, int32_t stack_k,
                                      size_t token_bytes_per_layer) {
  if (stack_k <= 0 || token_bytes_per_layer == 0) return 0;
  return (int64_t)(phys_block_bytes / ((size_t)stack_k * token_bytes_per_layer));
}

}  // extern "C"
