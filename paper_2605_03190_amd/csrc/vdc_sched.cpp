// The adaptive tiling step of the uop generator (Section 4.2, "Adaptive Scheduling and Tiling").  Host code only.
//
// The operators of a graph are scheduled onto the virtual cores, every operator in the coarsest of its decompositions;
// then, while the longest path through the operator DAG costs more than the average per core by more than a threshold (a
// dominant critical path), the operator on that path whose finer tiling shortens it most is given that tiling, until the
// best gain is marginal or nothing finer is left.
//
// An operator here is a matvec: n_blocks row blocks, a K range of nk tile steps.  Its decompositions cut the K range of
// every row block into S = 1 .. max_parts ranges (range s = steps [nk s / S, nk (s + 1) / S)); the work items, in the
// order (range, row block), are dealt in contiguous shares: core c takes items [NI c / C, NI (c + 1) / C) and deals them
// to its compute cores in turn.  The items of all ranges but the last store partial sums and signal a depId, the item of
// the last range adds them to its own (join_group of them per extra step, behind a load that waits for the depId).  With
// surplus = T the builder also offers every cut for the last T row blocks alone: the others stay whole and are dealt first.  Costs are integers: a tile
// step, an item (its output region and store), a joining step, a dependency edge (from the end of the producing
// item to the moment the joining item can use the result).  A compute core is a lane and works through its items in order;
// a joining item does its own steps first and waits then.
#include <algorithm>
#include <cstdint>
#include <map>
#include <utility>
#include <vector>

#include "../../include/vdcores.h"
#include "vdc_sched.h"

namespace vdc {

void sched_op_cost(const vdc_sched_op &op, int64_t S, int64_t tail, int64_t C, int64_t V, const vdc_cost_model &cm, int64_t &span, int64_t &work) {
    const int64_t NB = op.n_blocks, nk = op.nk;
    const int64_t T = S > 1 ? (tail > 0 ? tail : NB) : 0;      // row blocks that are cut; the first NB - T stay whole and are dealt first
    const int64_t NW = NB - T, NI = T * S;
    std::vector<int64_t> lane_t((size_t)(C * V), 0), finish((size_t)NI, 0);
    work = 0;
    for (int64_t c = 0; c < C; c++) {
        const int64_t b0 = NW * c / C, b1 = NW * (c + 1) / C;
        for (int64_t b = b0; b < b1; b++) {
            lane_t[(size_t)(c * V + (b - b0) % V)] += nk * cm.step + cm.item;
            work += nk * cm.step + cm.item;
        }
    }
    for (int64_t c = 0; c < C; c++) {
        const int64_t i0 = NI * c / C, i1 = NI * (c + 1) / C;
        for (int64_t i = i0; i < i1; i++) {
            const int64_t s = i / T, rb = i % T;
            const int64_t own = (nk * (s + 1) / S - nk * s / S) * cm.step;
            int64_t &lt = lane_t[(size_t)(c * V + (i - i0) % V)];
            if (s < S - 1) {
                lt += own + cm.item;
                work += own + cm.item;
            } else {
                int64_t ready = 0;
                for (int64_t sp = 0; sp < S - 1; sp++) ready = std::max(ready, finish[(size_t)(sp * T + rb)]);
                const int64_t G = op.join_group > 0 ? op.join_group : 1, joins = (S - 1 + G - 1) / G;
                lt = std::max(lt + own, ready + cm.edge) + joins * cm.join + cm.item;
                work += own + joins * cm.join + cm.item;
            }
            finish[(size_t)i] = lt;
        }
    }
    span = 0;
    for (int64_t t : lane_t) span = std::max(span, t);
}

int sched_adaptive(const vdc_sched_op *ops, int32_t n_ops, const int32_t *pred_begin, const int32_t *preds, int64_t C, int64_t V,
                   const vdc_cost_model &cm, int32_t threshold_pct, int32_t min_gain_pct, int32_t *parts, int32_t *tails, int64_t *log,
                   int32_t *n_looks) {
    if (n_ops < 0 || C < 1 || V < 1 || threshold_pct < 0 || min_gain_pct < 0 || cm.step < 1 || cm.item < 0 || cm.join < 0 || cm.edge < 0)
        return VDC_EINVAL;
    for (int32_t o = 0; o < n_ops; o++) {
        if (ops[o].n_blocks < 1 || ops[o].nk < 1 || ops[o].max_parts < 1 || ops[o].max_parts > ops[o].nk || ops[o].join_group < 0) return VDC_EINVAL;
        if (ops[o].surplus < 0 || ops[o].surplus >= ops[o].n_blocks || (ops[o].surplus > 0 && !tails)) return VDC_EINVAL;
        if (ops[o].n_blocks * (int64_t)ops[o].max_parts > (int64_t)1 << 24) return VDC_EINVAL;       // the cost of a decomposition walks its items
        if (pred_begin)
            for (int32_t e = pred_begin[o]; e < pred_begin[o + 1]; e++)
                if (preds[e] < 0 || preds[e] >= o) return VDC_EINVAL;                                 // a topological order
    }
    // a decomposition: S in the low half, 1 in bit 32 when only the surplus blocks are cut
    std::map<std::pair<int32_t, int64_t>, std::pair<int64_t, int64_t>> memo;
    auto oc = [&](int32_t o, int32_t S, bool surplus) -> const std::pair<int64_t, int64_t> & {
        const int64_t key = (int64_t)S | ((int64_t)(surplus && S > 1) << 32);
        auto it = memo.find({o, key});
        if (it == memo.end()) {
            int64_t span, work;
            sched_op_cost(ops[o], S, surplus ? ops[o].surplus : 0, C, V, cm, span, work);
            it = memo.emplace(std::make_pair(o, key), std::make_pair(span, work)).first;
        }
        return it->second;
    };
    const int32_t cap = (log && n_looks) ? *n_looks : 0;
    int32_t looks = 0;
    auto note = [&](int64_t pc, int64_t avg, int64_t o, int64_t S, int64_t gain) {
        if (looks < cap) {
            int64_t *l = log + (size_t)looks * 5;
            l[0] = pc; l[1] = avg; l[2] = o; l[3] = S; l[4] = gain;
        }
        looks++;
    };
    std::vector<char> sur((size_t)n_ops, 0);
    for (int32_t o = 0; o < n_ops; o++) parts[o] = 1;
    std::vector<int64_t> spans((size_t)n_ops), dist((size_t)n_ops);
    std::vector<int32_t> via((size_t)n_ops), path;
    for (;;) {
        int64_t total = 0;
        for (int32_t o = 0; o < n_ops; o++) {
            spans[(size_t)o] = oc(o, parts[o], sur[(size_t)o]).first;
            total += oc(o, parts[o], sur[(size_t)o]).second;
        }
        const int64_t avg = total / (C * V);
        // the longest path; ties go to the predecessor and to the sink with the lowest index
        int64_t pc = 0;
        int32_t end = -1;
        for (int32_t o = 0; o < n_ops; o++) {
            int64_t best = 0;
            int32_t arg = -1;
            if (pred_begin)
                for (int32_t e = pred_begin[o]; e < pred_begin[o + 1]; e++)
                    if (dist[(size_t)preds[e]] > best) { best = dist[(size_t)preds[e]]; arg = preds[e]; }
            dist[(size_t)o] = best + spans[(size_t)o];
            via[(size_t)o] = arg;
            if (end < 0 || dist[(size_t)o] > pc) { pc = dist[(size_t)o]; end = o; }
        }
        path.clear();
        for (int32_t o = end; o >= 0; o = via[(size_t)o]) path.push_back(o);
        std::reverse(path.begin(), path.end());
        if (pc * 100 <= avg * (100 + (int64_t)threshold_pct)) {
            note(pc, avg, -1, 0, 0);
            break;
        }
        // among the operators on the path and their finer decompositions (the surplus blocks alone before all blocks)
        int64_t gain = 0;
        int32_t go = -1, gs = 0;
        bool gsur = false;
        for (int32_t o : path)
            for (int32_t S = parts[o] + 1; S <= ops[o].max_parts; S++)
                for (int k = ops[o].surplus > 0 ? 0 : 1; k < 2; k++) {
                    const int64_t g = spans[(size_t)o] - oc(o, S, k == 0).first;
                    if (g > gain) { gain = g; go = o; gs = S; gsur = k == 0; }
                }
        if (gain <= 0 || gain * 100 < pc * (int64_t)min_gain_pct) {
            note(pc, avg, -1, 0, gain);
            break;
        }
        note(pc, avg, go, gs, gain);
        parts[go] = gs;
        sur[(size_t)go] = gsur;
    }
    if (tails)
        for (int32_t o = 0; o < n_ops; o++) tails[o] = sur[(size_t)o] ? (int32_t)ops[o].surplus : 0;
    if (n_looks) *n_looks = looks;
    return VDC_OK;
}

// Nanoseconds on an MI355X, fitted to whole runs of dense matvecs under every cut the builder offers, of all row blocks and
// of the surplus alone (sched_bench): a compute core streams tiles of 16 KB at its share (1 / 512) of 6.3 TB/s and smaller
// tiles at what the per-tile cost leaves of it (8 KB: 62 %, 4 KB: 37 % of the memory's peak); an item costs the refill of
// the pipeline when a compute core moves to another row block, its row sums and its store; a joining step is a tile step
// whose uops the front end cannot replay; a dependency edge, where a joining item has to wait it out, is a store written
// through at device scope and waited for, the counter, the waiting load's next look at it after its back-off, a read past
// the L2 and the joining step's own way through the pipeline.
vdc_cost_model sched_default_cost(int32_t tile_bytes) {
    vdc_cost_model cm;
    cm.step = 510 + tile_bytes / 20;
    cm.item = 1500;
    cm.join = cm.step + 1200;
    cm.edge = 16000;
    return cm;
}

}  // namespace vdc

extern "C" int vdc_schedule(vdc_executor *ex, const vdc_sched_op *ops, int32_t n_ops, const int32_t *pred_begin, const int32_t *preds,
                            const vdc_cost_model *cost, int32_t tile_bytes, int32_t *parts, int32_t *tails, int64_t *log, int32_t *n_looks) {
    vdc_config cfg;
    if (!ex || (n_ops > 0 && (!ops || !parts)) || (pred_begin && !preds && n_ops > 0 && pred_begin[n_ops] > 0) || (log && !n_looks) ||
        vdc_get_config(ex, &cfg) != VDC_OK)
        return VDC_EINVAL;
    if (!cost && (tile_bytes < 256 || tile_bytes > 32768)) return VDC_EINVAL;
    const vdc_cost_model cm = cost ? *cost : vdc::sched_default_cost(tile_bytes);
    return vdc::sched_adaptive(ops, n_ops, pred_begin, preds, cfg.n_cores, cfg.vcc_per_core, cm, cfg.sched_threshold_pct, cfg.sched_min_gain_pct,
                               parts, tails, log, n_looks);
}
