// The adaptive tiling step (Section 4.2, "Adaptive Scheduling and Tiling") as the tilers call it; see vdc_sched.cpp.
#pragma once
#include <cstdint>

#include "../../include/vdcores.h"

namespace vdc {

// span (the time the last lane ends) and work (the sum of the items' costs, waiting left out) of one operator whose K
// range is cut into S ranges (tail = T > 0: of its last T row blocks only), on C cores of V compute cores
void sched_op_cost(const vdc_sched_op &op, int64_t S, int64_t tail, int64_t C, int64_t V, const vdc_cost_model &cm, int64_t &span, int64_t &work);

// parts[o], tails[o] (0: all row blocks cut, T: the last T only) = the decomposition of operator o once no dominant critical path is left or the best gain is marginal.
// pred_begin / preds: the operator DAG (predecessors of o: preds[pred_begin[o] .. pred_begin[o + 1]), all below o); both
// may be null (no edges).  log (may be null): 5 words per look at the graph (path cost, average per lane, refined
// operator or -1, its new S, gain); *n_looks: capacity on entry, looks taken on return.
int sched_adaptive(const vdc_sched_op *ops, int32_t n_ops, const int32_t *pred_begin, const int32_t *preds, int64_t C, int64_t V,
                   const vdc_cost_model &cm, int32_t threshold_pct, int32_t min_gain_pct, int32_t *parts, int32_t *tails, int64_t *log,
                   int32_t *n_looks);

// The cost model the tilers use when the caller gives none: nanoseconds on this GPU for tiles of tile_bytes.
vdc_cost_model sched_default_cost(int32_t tile_bytes);

constexpr int32_t kSchedThresholdPct = 10, kSchedMinGainPct = 3;

}  // namespace vdc
