// The lowering steps of the uop generator (Section 4.2, "Dependency Graph Lowering" and "Dynamic Data Placement and
// Fusion") for graphs whose addresses are literals, and the placement step in the form that also works on looped
// streams.  Host code only.
//
//   place     a store and the load that reads exactly what it wrote, neighbours on one compute core, nobody else
//             reading the data, the tensor marked temporary: store.local / load.local, the data stays in local memory
//   flows     the loads of a compute core from one tensor are a chain of their own (a load that waits for another core
//             stalls only its chain); chains get virtual flows, stores and local pairs the compute core's store flow
//   order     slots are allocated in program order, so the way a memory core's stream interleaves its compute cores'
//             uops can over-commit the pool: the stream is checked by the validator's data-free run, and on deadlock it
//             is merged again one consumption group at a time, round-robin over the compute cores
//   deps      every load with producers waits for one depId that all of them signal (counted); a wait that an earlier
//             load on the same flow of the same core already made is dropped (in-order execution implies it)
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <map>
#include <set>
#include <string>
#include <vector>

#include "../../include/vdcores.h"
#include "vdc_isa.h"

using namespace vdc;

namespace {

struct Node {
    vdc_graph_memop in;
    Desc desc;
    bool local = false, device = false;
    int32_t vflow = 0;
    int32_t dep_wait = -1, dep_count = 0, dep_signal = -1;
    int64_t seq = 0;
};

bool same_desc(const Desc &a, const Desc &b) { return !memcmp(&a, &b, sizeof(Desc)); }

struct Lowering {
    const vdc_config &cfg;
    std::vector<Node> nodes;
    std::vector<std::pair<int64_t, int64_t>> edges;
    std::vector<std::vector<int64_t>> seqs;      // [core * V + vcc] -> node indices in the order the compute core takes the regions
    std::vector<std::vector<int64_t>> order;     // [core] -> the memory core's stream
    std::vector<Desc> descs_out;

    uint32_t desc_index(const Desc &d) {
        for (size_t i = 0; i < descs_out.size(); i++)
            if (same_desc(descs_out[i], d)) return (uint32_t)i;
        descs_out.push_back(d);
        return (uint32_t)descs_out.size() - 1;
    }

    int place(uint32_t temp_mask, int32_t geom_tensor) {
        std::map<int64_t, int> n_out, n_in;
        for (auto &e : edges) { n_out[e.first]++; n_in[e.second]++; }
        std::vector<std::pair<int64_t, int64_t>> kept;
        int done = 0;
        for (auto &e : edges) {
            Node &s = nodes[(size_t)e.first], &l = nodes[(size_t)e.second];
            const auto &seq = seqs[(size_t)(s.in.core * cfg.vcc_per_core + s.in.vcc)];
            const auto is = std::find(seq.begin(), seq.end(), e.first);
            const bool neighbours = is != seq.end() && is + 1 != seq.end() && *(is + 1) == e.second;
            const bool ok = s.in.core == l.in.core && s.in.vcc == l.in.vcc && s.in.op == OP_STORE && l.in.op == OP_LOAD &&
                            s.desc.tensor < 32 && ((temp_mask >> s.desc.tensor) & 1u) && n_out[e.first] == 1 && n_in[e.second] == 1 &&
                            s.in.offset == l.in.offset && s.in.rows == l.in.rows && same_desc(s.desc, l.desc) && neighbours;
            if (!ok) { kept.push_back(e); continue; }
            s.local = l.local = true;
            // the region keeps its slots from the store's allocation; the load allocates nothing and touches no memory
            Desc box = s.desc;
            box.tensor = (uint32_t)geom_tensor;
            box.row_bytes = box.lds_pitch;
            s.desc = l.desc = box;
            s.in.offset = l.in.offset = 0;
            s.in.rows = l.in.rows = (int32_t)box.box_rows;
            l.in.nslots = 0;
            if (l.in.group == s.in.group) l.in.group = s.in.group + 1;
            done++;
        }
        edges.swap(kept);
        return done;
    }

    void flows() {
        const int V = cfg.vcc_per_core;
        for (size_t q = 0; q < seqs.size(); q++) {
            const int v = (int)(q % (size_t)V);
            std::vector<uint32_t> chains;
            for (int64_t i : seqs[q]) {
                Node &m = nodes[(size_t)i];
                if (m.in.op == OP_STORE || m.local) { m.vflow = 2 * V + v; continue; }
                size_t c = std::find(chains.begin(), chains.end(), m.desc.tensor) - chains.begin();
                if (c == chains.size()) chains.push_back(m.desc.tensor);
                m.vflow = 2 * v + (int)std::min<size_t>(c, 1);
            }
        }
    }

    // per core: the nodes in the order they were written down
    void default_order() {
        order.assign((size_t)cfg.n_cores, {});
        std::vector<int64_t> all(nodes.size());
        for (size_t i = 0; i < nodes.size(); i++) all[i] = (int64_t)i;
        std::stable_sort(all.begin(), all.end(), [&](int64_t a, int64_t b) { return nodes[(size_t)a].seq < nodes[(size_t)b].seq; });
        for (int64_t i : all) order[(size_t)nodes[(size_t)i].in.core].push_back(i);
    }

    void merged_order() {
        const int V = cfg.vcc_per_core;
        for (int c = 0; c < cfg.n_cores; c++) {
            std::vector<size_t> at((size_t)V, 0);
            std::vector<int64_t> merged;
            for (;;) {
                bool any = false;
                for (int v = 0; v < V; v++) {
                    const auto &s = seqs[(size_t)(c * V + v)];
                    size_t &a = at[(size_t)v];
                    if (a >= s.size()) continue;
                    any = true;
                    const int32_t grp = nodes[(size_t)s[a]].in.group;
                    while (a < s.size() && nodes[(size_t)s[a]].in.group == grp) merged.push_back(s[a++]);
                }
                if (!any) break;
            }
            order[(size_t)c] = merged;
        }
    }

    // returns 0, or a VDC_E* code; stats: depIds, waits kept, waits dropped
    int deps(int32_t *n_ids, int32_t *kept, int32_t *dropped) {
        std::map<int64_t, std::vector<int64_t>> prods;
        for (auto &e : edges) prods[e.second].push_back(e.first);
        std::map<std::set<int64_t>, int32_t> ids;
        std::map<int64_t, int32_t> by_store;
        *kept = *dropped = 0;
        for (int c = 0; c < cfg.n_cores; c++) {
            std::map<int32_t, std::set<int32_t>> waited;
            for (int64_t i : order[(size_t)c]) {
                auto it = prods.find(i);
                if (it == prods.end()) continue;
                Node &m = nodes[(size_t)i];
                std::set<int64_t> key(it->second.begin(), it->second.end());
                auto f = ids.find(key);
                if (f == ids.end()) {
                    const int32_t id = (int32_t)ids.size();
                    if (id >= cfg.n_dep_ids) return VDC_EINVAL;
                    f = ids.emplace(key, id).first;
                    for (int64_t s : key) {
                        auto b = by_store.emplace(s, id);
                        if (b.first->second != id) return VDC_EPROGRAM;   // a store cannot signal two depIds
                        nodes[(size_t)s].dep_signal = id;
                        nodes[(size_t)s].device = true;
                    }
                }
                m.device = true;        // the data was written during this run, by whoever
                if (key.size() > 255) return VDC_EINVAL;
                auto &seen = waited[m.vflow];
                if (seen.count(f->second)) { (*dropped)++; continue; }
                seen.insert(f->second);
                m.dep_wait = f->second;
                m.dep_count = (int32_t)key.size();
                (*kept)++;
            }
        }
        *n_ids = (int32_t)ids.size();
        return VDC_OK;
    }

    void assemble(const Word *comp, const uint32_t *comp_begin, std::vector<Word> &words, std::vector<uint32_t> &sb) {
        const int V = cfg.vcc_per_core;
        descs_out.clear();
        words.clear();
        sb.assign(1, 0);
        for (int c = 0; c < cfg.n_cores; c++) {
            for (int64_t i : order[(size_t)c]) {
                const Node &m = nodes[(size_t)i];
                uint32_t flags = F_SEND | (m.in.nt ? F_NT : 0u);
                if (m.in.op == OP_STORE) flags |= F_RECV;
                if (m.local) flags |= F_LOCAL;
                uint32_t dep_id = 0, dep_count = 0;
                if (m.dep_wait >= 0) { flags |= F_DEP_RECV; dep_id = (uint32_t)m.dep_wait; dep_count = (uint32_t)m.dep_count; }
                if (m.dep_signal >= 0) { flags |= F_DEP_SEND; dep_id = (uint32_t)m.dep_signal; }
                if (m.device && !m.local) flags |= F_DEVICE;
                words.push_back(encode((uint32_t)m.in.op, flags, (uint32_t)m.vflow, (uint32_t)m.in.vcc, 0, (uint32_t)m.in.nslots, (uint32_t)m.in.rows,
                                       dep_id, m.in.offset, desc_index(m.desc), dep_count));
            }
            words.push_back(encode(OP_HALT, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0));
            sb.push_back((uint32_t)words.size());
            for (int v = 0; v < V; v++) {
                const uint32_t q = (uint32_t)(c * V + v);
                for (uint32_t j = comp_begin[q]; j < comp_begin[q + 1]; j++)
                    if (decode(comp[j]).opcode != OP_HALT) words.push_back(comp[j]);
                words.push_back(encode(OP_HALT, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0));
                sb.push_back((uint32_t)words.size());
            }
        }
        if (descs_out.empty()) descs_out.push_back(Desc{0, 1, 16, 16, 0, 0, 0, 0});
    }
};

}  // namespace

extern "C" {

int vdc_graph_lower(vdc_executor *ex, const vdc_graph_memop *ops, int64_t n_ops, const int64_t *edges, int64_t n_edges,
                    const void *comp_uops, const uint32_t *comp_begin, const void *descs, int32_t n_descs, uint32_t temp_tensors,
                    int32_t geom_tensor, const int64_t *tensor_bytes, int32_t n_tensors, void *uops_out, int64_t *n_uops,
                    uint32_t *stream_begin, void *descs_out, int32_t *n_descs_out, int32_t *stats) {
    if (!ex || !ops || n_ops < 1 || (n_edges > 0 && !edges) || n_edges < 0 || !comp_uops || !comp_begin || !descs || n_descs < 1 ||
        !tensor_bytes || n_tensors < 1 || n_tensors > kMaxTensors || !n_uops || !n_descs_out || geom_tensor < 0 || geom_tensor >= n_tensors)
        return VDC_EINVAL;
    vdc_config cfg;
    int rc = vdc_get_config(ex, &cfg);
    if (rc != VDC_OK) return rc;
    const int V = cfg.vcc_per_core;
    Lowering lw{cfg};
    lw.nodes.resize((size_t)n_ops);
    lw.seqs.assign((size_t)(cfg.n_cores * V), {});
    for (int64_t i = 0; i < n_ops; i++) {
        const vdc_graph_memop &o = ops[i];
        if ((o.op != (int32_t)OP_LOAD && o.op != (int32_t)OP_STORE) || o.core < 0 || o.core >= cfg.n_cores || o.vcc < 0 || o.vcc >= V ||
            o.desc < 0 || o.desc >= n_descs || o.rows < 1 || o.rows > 65535 || o.nslots < 1 || o.nslots > cfg.n_slots || o.offset < 0)
            return VDC_EINVAL;
        Node &n = lw.nodes[(size_t)i];
        n.in = o;
        n.desc = ((const Desc *)descs)[o.desc];
        n.seq = i;
        lw.seqs[(size_t)(o.core * V + o.vcc)].push_back(i);
    }
    for (int64_t e = 0; e < n_edges; e++) {
        const int64_t s = edges[2 * e], l = edges[2 * e + 1];
        if (s < 0 || s >= n_ops || l < 0 || l >= n_ops || ops[s].op != (int32_t)OP_STORE || ops[l].op != (int32_t)OP_LOAD) return VDC_EINVAL;
        lw.edges.push_back({s, l});
    }
    int32_t st[5] = {0, 0, 0, 0, 0};     // pairs placed, stream reordered, depIds, waits kept, waits dropped
    st[0] = lw.place(temp_tensors, geom_tensor);
    lw.flows();
    lw.default_order();
    std::vector<Word> words;
    std::vector<uint32_t> sb;
    // the order as written: does it run to its end under in-order allocation?  (Dependencies are not embedded yet: this
    // asks about the slots alone.)
    lw.assemble((const Word *)comp_uops, comp_begin, words, sb);
    char msg[128];
    rc = vdc_program_validate(ex, words.data(), (int64_t)words.size(), sb.data(), lw.descs_out.data(), (int32_t)lw.descs_out.size(), tensor_bytes,
                              n_tensors, msg, (int32_t)sizeof msg);
    if (rc == VDC_EPROGRAM && strstr(msg, "deadlock")) {
        lw.merged_order();
        st[1] = 1;
    } else if (rc != VDC_OK) {
        return rc;
    }
    rc = lw.deps(&st[2], &st[3], &st[4]);
    if (rc != VDC_OK) return rc;
    lw.assemble((const Word *)comp_uops, comp_begin, words, sb);
    rc = vdc_program_validate(ex, words.data(), (int64_t)words.size(), sb.data(), lw.descs_out.data(), (int32_t)lw.descs_out.size(), tensor_bytes,
                              n_tensors, msg, (int32_t)sizeof msg);
    if (rc != VDC_OK) return rc;         // also: the merged order over-commits the slots as well
    if (stats) memcpy(stats, st, sizeof st);
    const int64_t cap_w = *n_uops;
    const int32_t cap_d = *n_descs_out;
    *n_uops = (int64_t)words.size();
    *n_descs_out = (int32_t)lw.descs_out.size();
    bool fits = true;
    if (uops_out) { if (cap_w >= (int64_t)words.size()) memcpy(uops_out, words.data(), words.size() * sizeof(Word)); else fits = false; }
    if (descs_out) { if (cap_d >= (int32_t)lw.descs_out.size()) memcpy(descs_out, lw.descs_out.data(), lw.descs_out.size() * sizeof(Desc)); else fits = false; }
    if (stream_begin) memcpy(stream_begin, sb.data(), sb.size() * sizeof(uint32_t));
    return fits ? VDC_OK : VDC_EINVAL;
}

}  // extern "C"

namespace vdc {

// The placement step on bytecode that may contain loops (the operators' own tilers write looped streams): in every
// memory core's stream, a STORE directly followed by a LOAD of the same compute core that moves the same box of a
// temporary tensor from the same address expression (literal part, accumulator, dynamic flag) with no dependency flags
// becomes store.local / load.local.  The pair may stand inside a loop: both halves see the same accumulator value on
// every trip.  Descriptors are appended as needed.  Returns the number of pairs rewritten.
int place_local_in_streams(const vdc_config &cfg, std::vector<Word> &words, const std::vector<uint32_t> &sb, std::vector<Desc> &descs,
                           uint32_t temp_mask, uint32_t geom_tensor) {
    const int V = cfg.vcc_per_core;
    int done = 0;
    auto desc_index = [&](const Desc &d) {
        for (size_t i = 0; i < descs.size(); i++)
            if (!memcmp(&descs[i], &d, sizeof d)) return (uint32_t)i;
        descs.push_back(d);
        return (uint32_t)descs.size() - 1;
    };
    for (int c = 0; c < cfg.n_cores; c++) {
        const uint32_t b = sb[(size_t)c * (1 + V)], e = sb[(size_t)c * (1 + V) + 1];
        for (uint32_t i = b; i + 1 < e; i++) {
            const Fields s = decode(words[i]), l = decode(words[i + 1]);
            if (s.opcode != OP_STORE || l.opcode != OP_LOAD || s.desc >= descs.size() || l.desc >= descs.size()) continue;
            const Desc ds = descs[s.desc], dl = descs[l.desc];
            const uint32_t plain = F_SEND | F_RECV | F_DYNAMIC | F_NT;
            if ((s.flags & ~plain) || (l.flags & ~plain) || !(s.flags & F_SEND) || !(s.flags & F_RECV) || !(l.flags & F_SEND) || (l.flags & F_RECV)) continue;
            if (ds.tensor >= 32 || !((temp_mask >> ds.tensor) & 1u) || memcmp(&ds, &dl, sizeof ds)) continue;
            if (s.vcc != l.vcc || s.imm != l.imm || s.size != l.size || ((s.flags ^ l.flags) & F_DYNAMIC) || ((s.flags & F_DYNAMIC) && s.acc != l.acc)) continue;
            Desc box = ds;
            box.tensor = geom_tensor;
            box.row_bytes = box.lds_pitch;
            const uint32_t di = desc_index(box);
            words[i] = encode(OP_STORE, F_SEND | F_RECV | F_LOCAL, s.vflow, s.vcc, 0, s.nslots, box.box_rows, 0, 0, di, 0);
            words[i + 1] = encode(OP_LOAD, F_SEND | F_LOCAL, s.vflow, s.vcc, 0, 0, box.box_rows, 0, 0, di, 0);
            done++;
            i++;
        }
    }
    return done;
}

}  // namespace vdc
