// Host side of the library: executor life cycle, program validation (a data-free walk of the whole uop
// graph, the generator-side check of Section 4.2 "Dependency Graph Lowering"), the matvec tiler (the slice of
// the uop generator of Section 4.2 that the matvec operator needs) and the C ABI declared in vdcores.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <deque>
#include <memory>
#include <new>
#include <string>
#include <chrono>
#include <thread>
#include <vector>

#include "../../include/vdcores.h"
#include "vdc_isa.h"
#include "vdc_kernel.h"
#include "vdc_sched.h"

using namespace vdc;

struct vdc_program {
    vdc_executor *ex = nullptr;
    Word *d_words = nullptr;
    uint32_t *d_stream_begin = nullptr;
    Desc *d_descs = nullptr;
    int32_t n_descs = 0;
    int32_t n_tensors = 0;
    int64_t tensor_bytes[kMaxTensors] = {0};
    bool uses_dep = false;
    uint32_t max_dep_id = 0;
    uint32_t loaded_tensors = 0;   // bit t: some LOAD reads tensor t (its base must be 16-byte aligned: 128-bit loads)
    uint32_t ops = 0;              // families of compute uops the program uses (OPS_*): picks the kernel variant
    void *d_workspace = nullptr;   // matvec programs that split K: the [I | 0] tile and the partial results
    int32_t placement = 0;         // which roles share a SIMD, see vdc_program_set_placement
};

// The operators cache the programs they build.  A key is the operator's kind followed by everything the uop graph
// depends on (shapes, tile size, segment offsets, ...), as one vector of 64-bit words, looked up by hash and then by
// content.  The cache is bounded: beyond kProgramCacheCap entries the least recently used program is destroyed (after a
// device synchronisation, inside vdc_program_destroy), so a caller whose shapes change on every call (decode attention
// with growing contexts) pays a rebuild per call but does not grow device memory without limit.
constexpr size_t kProgramCacheCap = 64;
struct CachedProgram {
    uint64_t hash;
    std::vector<int64_t> key;
    vdc_program *prog;
    uint64_t last_use;
};
enum ProgramKind : int64_t { PK_MATVEC = 1, PK_CHAIN = 2, PK_ATTN = 3, PK_STREAM = 4 };

struct vdc_executor {
    vdc_config cfg{};
    int cu_count = 0;
    size_t lds_limit = 0;
    uint32_t *d_dep = nullptr;
    uint32_t *d_status = nullptr;
    uint32_t *h_status = nullptr;  // pinned
#if defined(VDC_PROFILE) || defined(VDC_PROFILE_WAITS)
    unsigned long long *d_prof = nullptr;
#endif
    std::vector<vdc_program *> programs;
    std::vector<CachedProgram> cache;
    uint64_t use_clock = 0;
    // for vdc_matvec_noalloc, all obtained at vdc_create: this device's static scratch array, a pinned staging buffer
    // for the program image, and the event that tells when the last copy out of it has been done
    unsigned char *scratch = nullptr;
    unsigned char *h_stage = nullptr;
    hipEvent_t stage_done = nullptr;
    bool stage_pending = false;
    // the resident form (vdc_resident_*): the mailbox in pinned host memory, the device words behind it, the stream the
    // grid runs on, graphs posted so far
    volatile uint32_t *r_mailbox = nullptr;
    uint32_t *r_dev = nullptr;
    hipStream_t r_stream = nullptr;
    uint32_t r_posted = 0;
    bool r_up = false;             // vdc_resident_start has been called and vdc_resident_stop has not
};

// What the static scratch array of each device holds right now (it is shared by every executor on that device and keeps
// its content from call to call): the key of the uploaded program and what a run needs to know about it.
struct ScratchImage {
    std::vector<int64_t> key;      // empty: nothing valid
    int32_t n_descs = 0, n_tensors = 0, placement = 0;
    int64_t tensor_bytes[kMaxTensors] = {0};
    bool uses_dep = false;
    uint32_t max_dep_id = 0, loaded_tensors = 0, ops = 0;
    size_t off_sb = 0, off_descs = 0, off_words = 0, off_ws = 0;   // byte offsets from the start of the array
    bool has_ws = false;
};
static ScratchImage g_scratch_image[64];

namespace vdc {
int place_local_in_streams(const vdc_config &cfg, std::vector<Word> &words, const std::vector<uint32_t> &sb, std::vector<Desc> &descs,
                           uint32_t temp_mask, uint32_t geom_tensor);
}

namespace {

int hip_fail(hipError_t) { return VDC_EDEVICE; }
#define HIP_TRY(x)                                \
    do {                                          \
        hipError_t e_ = (x);                      \
        if (e_ != hipSuccess) return hip_fail(e_); \
    } while (0)

bool is_pow2(int64_t x) { return x > 0 && (x & (x - 1)) == 0; }

uint64_t key_hash(const std::vector<int64_t> &k) {   // FNV-1a over the words
    uint64_t h = 1469598103934665603ull;
    for (int64_t w : k) {
        h ^= (uint64_t)w;
        h *= 1099511628211ull;
    }
    return h;
}

vdc_program *cache_find(vdc_executor *ex, const std::vector<int64_t> &key) {
    const uint64_t h = key_hash(key);
    for (CachedProgram &c : ex->cache)
        if (c.hash == h && c.key == key) {
            c.last_use = ++ex->use_clock;
            return c.prog;
        }
    return nullptr;
}

// Adds a program; evicts the least recently used one first when the cache is full.
void cache_insert(vdc_executor *ex, std::vector<int64_t> key, vdc_program *prog) {
    if (ex->cache.size() >= kProgramCacheCap) {
        size_t lru = 0;
        for (size_t i = 1; i < ex->cache.size(); i++)
            if (ex->cache[i].last_use < ex->cache[lru].last_use) lru = i;
        vdc_program *victim = ex->cache[lru].prog;
        ex->cache.erase(ex->cache.begin() + (long)lru);
        (void)vdc_program_destroy(victim);     // waits for the device, then frees the program's device memory
    }
    const uint64_t h = key_hash(key);
    ex->cache.push_back({h, std::move(key), prog, ++ex->use_clock});
}

// The factor on the scores: the caller's, or (scale <= 0) the usual d^(-1/2).  False for a value that is not a number.
bool attn_scale_resolve(float &scale, int32_t d) {
    if (scale != scale || d < 1) return false;
    if (scale <= 0.0f) scale = 1.0f / std::sqrt((float)d);
    return true;
}

int64_t float_bits(float x) {
    uint32_t b;
    memcpy(&b, &x, 4);
    return (int64_t)b;
}

// ------------------------------------------------------------------------------------------------------------
// Validation: run the abstract machine without data.  Every core's front end walks its stream in program order,
// allocating slots from the same first-fit mask as the device; loads complete at once; a compute core consumes
// its tickets in order and returns regions; a store completes when its region comes back.  Cores take turns
// until all streams are at HALT.  A full sweep without progress is a deadlock: in-order execution cannot finish,
// which is the situation the paper's generator must exclude before a program reaches the device.
// ------------------------------------------------------------------------------------------------------------
struct SeqH {
    uint32_t pc = 0, begin = 0, end = 0;
    std::vector<std::pair<uint32_t, uint32_t>> loops;  // (start, trips left)
    int64_t acc[kNumAcc] = {0};
    bool halted = false;
};

struct SentMsg {
    uint32_t slot, nslots, rows, row_bytes, box_rows, lds_pitch;
    bool is_store;
    bool is_local = false;        // the region of a store.local
    uint32_t unit = 0;            // the store unit a STORE sits on
};

struct VccH {
    SeqH s;
    std::deque<SentMsg> m2c;      // delivered, in ticket order (loads complete at once in this model)
    // running MATVEC
    bool in_uop = false;
    uint32_t left = 0, B = 0, R = 0, lpr = 0;
    uint32_t xspan = 0, xstep = 0;   // MATVEC with a vector tile over several steps: steps per tile, steps done on the one held
    uint32_t rowspan = 0;            // MATVEC over several row blocks: how many
    bool holds_x = false;
    int phase = 0;                // MATVEC: 0 expect a, 1 expect b, 2 expect out, 3 expect a vector tile over several steps; ROPE: 10 expect values, 11 expect angles, 12 expect out;
                                  // DROP: 20; FILL: 21; COPY: 22 expect in, 23 expect out;
                                  // ATTN: 30 expect q, 31 expect K tile, 32 expect V tile, 34 expect the partial rows to join, 33 expect out; ATTN_MERGE: 40 expect rows, 41 expect out;
                                  // MATVEC over several row blocks: 50 expect out, 51 expect the vector tile, 52 expect a matrix tile
    SentMsg q{};
    uint32_t chunks = 0;
    uint32_t join = 0;             // attn: partial rows of other items joined behind the last pair
    SentMsg a{}, b{};
};

struct CoreH {
    SeqH vmc;
    std::vector<VccH> vcc;
    uint32_t mask = 0;
    std::deque<SentMsg> stores_waiting;  // STOREs whose region has not come back yet (only counted)
    std::deque<SentMsg> parked[2];       // per store unit: regions a store.local took back, waiting for their load.local
};

struct Validator {
    const vdc_config &cfg;
    const Word *words;
    int64_t n_words;
    const uint32_t *sb;
    const Desc *descs;
    int32_t n_descs;
    const int64_t *tensor_bytes;
    int32_t n_tensors;
    std::string err;
    bool uses_dep = false;
    uint32_t max_dep = 0;
    uint32_t loaded_tensors = 0;
    uint32_t ops = 0;              // OPS_* families of the compute uops met
    bool big_regions = false;      // some memory uop's region takes more than one slot
    std::vector<uint32_t> dep;
    int64_t steps = 0;

    bool fail(const std::string &m) {
        if (err.empty()) err = m;
        return false;
    }

    // the store unit a STORE or a local memory uop goes to: its flow, modulo the number of units
    uint32_t stu_of(const Fields &f) const { return f.vflow & (uint32_t)(cfg.n_stu - 1); }

    int first_fit(uint32_t mask, uint32_t n) const {
        for (int p = 0; p + (int)n <= cfg.n_slots; p++) {
            uint64_t bits = ((n >= 64 ? ~0ull : ((1ull << n) - 1ull)) << p);
            if (((uint64_t)mask & bits) == 0) return p;
        }
        return -1;
    }

    // control uops; returns 1 handled, 2 halt, 0 not control, -1 error
    int control(SeqH &s, const Fields &f) {
        switch (f.opcode) {
            case OP_HALT:
                if (!s.loops.empty()) { fail("HALT inside a loop"); return -1; }
                s.halted = true;
                return 2;
            case OP_LOOP:
                if (f.imm < 1 || f.imm > 0xFFFFFFFFll || (int)s.loops.size() >= kMaxLoopDepth) { fail("bad LOOP"); return -1; }
                s.loops.push_back({s.pc + 1, (uint32_t)f.imm});
                s.pc++;
                return 1;
            case OP_REPEAT:
                if (s.loops.empty()) { fail("REPEAT without LOOP"); return -1; }
                if (__builtin_add_overflow(s.acc[f.acc], f.imm, &s.acc[f.acc])) { fail("accumulator overflow"); return -1; }
                if (--s.loops.back().second > 0) s.pc = s.loops.back().first;
                else { s.loops.pop_back(); s.pc++; }
                return 1;
            case OP_ADD:
                if (__builtin_add_overflow(s.acc[f.acc], f.imm, &s.acc[f.acc])) { fail("accumulator overflow"); return -1; }
                s.pc++;
                return 1;
            case OP_SET:
                s.acc[f.acc] = f.imm;
                s.pc++;
                return 1;
            case OP_CONTINUE_IF: {
                if (s.loops.empty()) { fail("CONTINUE_IF outside a loop"); return -1; }
                // `size` words on stands the REPEAT of the innermost loop; what lies between closes every loop it opens
                int depth = 0;
                bool ok = f.size >= 1 && (uint64_t)s.pc + f.size < (uint64_t)s.end;
                for (uint32_t q = s.pc + 1; ok && q < s.pc + f.size; q++) {
                    const uint32_t op = decode(words[q]).opcode;
                    depth += op == OP_LOOP ? 1 : (op == OP_REPEAT ? -1 : 0);
                    if (depth < 0) ok = false;
                }
                if (!ok || depth != 0 || decode(words[s.pc + f.size]).opcode != OP_REPEAT) { fail("CONTINUE_IF does not point at the REPEAT of its loop"); return -1; }
                if (s.acc[f.acc] < f.imm) s.pc++;
                else { s.loops.pop_back(); s.pc += f.size + 1; }
                return 1;
            }
            default:
                return 0;
        }
    }

    bool fetch(SeqH &s, Fields &f) {
        if (s.pc >= s.end) return fail("stream runs past its end without HALT");
        f = decode(words[s.pc]);
        return true;
    }

    // one front-end step of core c; returns 1 progress, 0 blocked, -1 error
    int cfu_step(CoreH &c) {
        SeqH &s = c.vmc;
        if (s.halted) return 0;
        Fields f;
        if (!fetch(s, f)) return -1;
        int k = control(s, f);
        if (k < 0) return -1;
        if (k > 0) return 1;
        if (f.opcode != OP_LOAD && f.opcode != OP_STORE) { fail("opcode not valid on a memory core"); return -1; }
        if ((int)f.desc >= n_descs) { fail("descriptor index out of range"); return -1; }
        const Desc &d = descs[f.desc];
        const bool is_load = f.opcode == OP_LOAD;
        const bool local = (f.flags & F_LOCAL) != 0;
        if (f.nslots > 1) big_regions = true;
        if (local) {
            // store.local / load.local: no memory access.  The load names no region of its own: it hands on the oldest
            // region a store.local of this core has taken back.
            if ((f.flags & (F_DYNAMIC | F_DEP_SEND | F_DEP_RECV | F_NT | F_DEVICE)) || f.imm != 0 || !(f.flags & F_SEND) || (!is_load && !(f.flags & F_RECV)) ||
                (is_load && (f.flags & F_RECV))) { fail("malformed local memory uop"); return -1; }
            if ((int)f.vcc >= cfg.vcc_per_core) { fail("vcc out of range"); return -1; }
            if (d.box_rows < 1 || d.box_rows > 65535 || d.lds_pitch < 4 || d.lds_pitch > 65535 || d.row_bytes < 4 || d.row_bytes > d.lds_pitch ||
                f.size < 1 || f.size > d.box_rows) { fail("bad descriptor box"); return -1; }
        }
        if (local && is_load) {
            if (f.nslots != 0) { fail("load.local allocates nothing: nslots must be 0"); return -1; }
            if (c.parked[stu_of(f)].empty()) return 0;
            SentMsg m = c.parked[stu_of(f)].front();
            c.parked[stu_of(f)].pop_front();
            if ((uint64_t)d.box_rows * d.lds_pitch > (uint64_t)m.nslots * cfg.slot_bytes) { fail("load.local: the region is smaller than the box it is handed on as"); return -1; }
            m.rows = f.size; m.row_bytes = d.row_bytes; m.box_rows = d.box_rows; m.lds_pitch = d.lds_pitch; m.is_store = false; m.is_local = false;
            c.vcc[f.vcc].m2c.push_back(m);
            s.pc++;
            return 1;
        }
        const uint64_t gpitch = (uint64_t)d.gpitch_lo | ((uint64_t)d.gpitch_hi << 32);
        if ((int)d.tensor >= n_tensors) { fail("tensor id out of range"); return -1; }
        if (is_load) loaded_tensors |= 1u << d.tensor;
        if (d.box_rows < 1 || d.box_rows > 65535 || d.lds_pitch < 4 || d.lds_pitch > 65535 || d.row_bytes < 4 ||
            d.row_bytes > d.lds_pitch) { fail("bad descriptor box"); return -1; }
        if (is_load ? (d.lds_pitch % 16 || d.row_bytes % 16 || gpitch % 16) : (d.lds_pitch % 4 || d.row_bytes % 4 || gpitch % 4)) {
            fail("descriptor alignment"); return -1;
        }
        if (f.size < 1 || f.size > d.box_rows) { fail("rows exceed the descriptor box"); return -1; }
        const uint64_t box_bytes = (uint64_t)d.box_rows * d.lds_pitch;
        const uint32_t need = (uint32_t)((box_bytes + cfg.slot_bytes - 1) / cfg.slot_bytes);
        if (f.nslots != need || need < 1 || (int)need > cfg.n_slots) { fail("nslots does not match the descriptor box"); return -1; }
        if ((int)f.vcc >= cfg.vcc_per_core) { fail("vcc out of range"); return -1; }
        if (is_load && !(f.flags & F_SEND)) { fail("LOAD without SEND would never be released"); return -1; }
        if (!is_load && !(f.flags & F_RECV)) { fail("STORE without RECV has no data to write"); return -1; }
        // with two store units each receives the c2m queue of one compute core (unit i: VCC i)
        if (!is_load && stu_of(f) != (f.vcc & (uint32_t)(cfg.n_stu - 1))) { fail("STORE on another store unit than its compute core's"); return -1; }
        if (is_load && (f.flags & F_RECV)) { fail("LOAD with RECV is not defined"); return -1; }
        if (f.flags & (F_DEP_SEND | F_DEP_RECV)) {
            if ((int)f.dep_id >= cfg.n_dep_ids) { fail("depId out of range"); return -1; }
            uses_dep = true;
            max_dep = std::max(max_dep, f.dep_id);
        }
        int64_t eff = f.imm;
        if ((f.flags & F_DYNAMIC) && __builtin_add_overflow(eff, s.acc[f.acc], &eff)) { fail("effective address overflows"); return -1; }
        if (eff < 0 || (eff % (is_load ? 16 : 4)) != 0) { fail("effective address negative or misaligned"); return -1; }
        // the last byte the box touches, in arithmetic that cannot wrap: a pitch of 2^63 must not pass as zero
        if (!local) {
            const uint64_t tb = tensor_bytes[d.tensor] > 0 ? (uint64_t)tensor_bytes[d.tensor] : 0ull;
            uint64_t span = 0, last = 0;
            if (__builtin_mul_overflow((uint64_t)(f.size - 1), gpitch, &span) || __builtin_add_overflow((uint64_t)eff, span, &last) ||
                __builtin_add_overflow(last, (uint64_t)d.row_bytes, &last) || last > tb) { fail("memory uop reaches beyond its tensor"); return -1; }
        }
        // a DEP_RECV whose counter is not there yet blocks its unit, not the front end; in this in-order model the
        // front end waits as well, which is conservative
        if ((f.flags & F_DEP_RECV) && dep[f.dep_id] < std::max<uint32_t>(1u, f.dep_count)) return 0;
        int slot = first_fit(c.mask, f.nslots);
        if (slot < 0) return 0;
        c.mask |= (uint32_t)(((f.nslots >= 32 ? 0xFFFFFFFFull : ((1ull << f.nslots) - 1ull)) << slot));
        SentMsg m{(uint32_t)slot, f.nslots, f.size, d.row_bytes, d.box_rows, d.lds_pitch, !is_load, local, stu_of(f)};
        if (f.flags & F_SEND) c.vcc[f.vcc].m2c.push_back(m);
        if (!is_load) {
            if (!(f.flags & F_SEND)) { fail("STORE with RECV but without SEND: nothing hands its region to a compute core"); return -1; }
            c.stores_waiting.push_back(m);
            if (f.flags & F_DEP_SEND) dep[f.dep_id]++;   // counted at issue: the store itself cannot block
        } else if (f.flags & F_DEP_SEND) {
            dep[f.dep_id]++;
        }
        s.pc++;
        return 1;
    }

    void release(CoreH &c, const SentMsg &m) {
        c.mask &= ~(uint32_t)(((m.nslots >= 32 ? 0xFFFFFFFFull : ((1ull << m.nslots) - 1ull)) << m.slot));
    }

    // a produced region returns to its STORE: written back and freed, or (store.local) kept for the load.local
    bool store_returns(CoreH &c, const SentMsg &m) {
        for (auto it = c.stores_waiting.begin(); it != c.stores_waiting.end(); ++it)
            if (it->slot == m.slot && it->nslots == m.nslots) {
                const bool local = it->is_local;
                const uint32_t unit = it->unit;
                c.stores_waiting.erase(it);
                if (local) c.parked[unit].push_back(m); else release(c, m);
                return true;
            }
        return fail("a compute uop's output region has no STORE");
    }

    int vcc_step(CoreH &c, VccH &v) {
        if (!v.in_uop) {
            if (v.s.halted) return 0;
            Fields f;
            if (!fetch(v.s, f)) return -1;
            int k = control(v.s, f);
            if (k < 0) return -1;
            if (k > 0) return 1;
            ops |= f.opcode == OP_MATVEC ? (matvec_rowspan(f) >= 2 ? (OPS_MATVEC | OPS_ROWS) : OPS_MATVEC)
                   : f.opcode == OP_ROPE ? OPS_ROPE
                   : (f.opcode == OP_ATTN || f.opcode == OP_ATTN_MERGE) ? OPS_ATTN
                   : (f.opcode == OP_DROP || f.opcode == OP_COPY || f.opcode == OP_FILL) ? OPS_STREAM : 0u;
            if (f.opcode == OP_ROPE) {
                v.B = (uint32_t)f.imm & 0xFFu;
                v.R = (uint32_t)(f.imm >> 8) & 0xFFFFu;
                if (!rope_geometry_ok(v.B, v.R)) { fail("rope geometry not supported"); return -1; }
                v.phase = 10;
                v.in_uop = true;
                return 1;
            }
            if (f.opcode == OP_DROP || f.opcode == OP_COPY || f.opcode == OP_FILL) {
                if (f.size < 1) { fail("stream uop over zero regions"); return -1; }
                v.chunks = f.opcode == OP_COPY ? (uint32_t)f.imm & 0xFFFFu : f.opcode == OP_FILL ? (uint32_t)(f.imm >> 32) & 0xFFFFu : 0u;
                if (f.opcode != OP_DROP && (v.chunks < 1 || v.chunks > kMaxStreamChunks)) { fail("stream uop: bad byte count"); return -1; }
                v.left = f.size;
                v.phase = f.opcode == OP_DROP ? 20 : f.opcode == OP_FILL ? 21 : 22;
                v.in_uop = true;
                return 1;
            }
            if (f.opcode == OP_ATTN || f.opcode == OP_ATTN_MERGE) {
                v.lpr = (uint32_t)f.imm & 0xFFu;
                v.R = f.opcode == OP_ATTN ? (uint32_t)(f.imm >> 8) & 0xFFu : 16u;     // a merge has no tile rows: any supported value
                if (!attn_geometry_ok(v.lpr, v.R)) { fail("attn geometry not supported"); return -1; }
                if (f.size < 1 || (f.opcode == OP_ATTN_MERGE && f.size > kAttnMaxPartials)) { fail("attn: bad size"); return -1; }
                v.join = f.opcode == OP_ATTN ? attn_join(f) : 0u;
                if (v.join > kAttnMaxPartials) { fail("attn: too many partial rows to join"); return -1; }
                v.left = f.size;
                v.phase = f.opcode == OP_ATTN ? 30 : 40;
                v.in_uop = true;
                return 1;
            }
            if (f.opcode != OP_MATVEC) { fail("opcode not valid on a compute core"); return -1; }
            v.B = (uint32_t)f.imm & 0xFFu;
            v.R = (uint32_t)(f.imm >> 8) & 0xFFFFu;
            v.lpr = (uint32_t)(f.imm >> 24) & 0xFFFFu;
            if (!matvec_geometry_ok(v.B, v.R, v.lpr, nullptr, nullptr)) { fail("matvec geometry not supported"); return -1; }
            v.xspan = matvec_xspan(f.imm);
            if (v.xspan >= 2 && (v.xspan > kMaxXspan || v.lpr > 64 || !matvec_xspan_ok(v.B, v.R, v.lpr))) { fail("matvec: a vector tile over several steps needs at most 8 steps, rows inside one wave, and one vector or a geometry the compute uop has with several"); return -1; }
            if (f.size < 1) { fail("matvec over zero tiles"); return -1; }
            v.rowspan = matvec_rowspan(f);
            if (v.rowspan >= 2 && (f.size != 1 || v.xspan >= 2 || v.lpr > 64 || v.rowspan > kMaxRowspan || v.B > kMaxRowspanB)) {
                fail("matvec over several row blocks needs one tile step per block, a vector tile of its own, rows inside one wave, at most 16 blocks and at most 4 vectors"); return -1;
            }
            if ((uint64_t)v.B * v.R * std::max(1u, v.rowspan) * 4 > (uint64_t)cfg.slot_bytes * cfg.n_slots) { fail("matvec output too large"); return -1; }
            v.left = v.rowspan >= 2 ? v.rowspan : f.size;
            v.phase = v.rowspan >= 2 ? 50 : (v.xspan >= 2 ? 3 : 0);
            v.holds_x = false;
            v.in_uop = true;
            return 1;
        }
        if (v.m2c.empty()) return 0;
        SentMsg m = v.m2c.front();
        v.m2c.pop_front();
        if (v.phase >= 50) {
            // MATVEC over several row blocks: the output region first, then the vector tile, then one matrix tile per block
            if (v.phase == 50) {
                if (!m.is_store || m.rows != v.B || m.lds_pitch != v.rowspan * v.R * 4 || m.row_bytes > v.rowspan * v.R * 4) { fail("matvec: output region does not match the uop"); return -1; }
                v.q = m; v.phase = 51;
            } else if (v.phase == 51) {
                if (m.is_store || m.box_rows != v.B || m.rows != v.B || m.lds_pitch != v.lpr * 16) { fail("matvec: vector tile does not match the uop"); return -1; }
                v.b = m; v.phase = 52;
            } else {
                if (m.is_store || m.box_rows != v.R || m.lds_pitch != v.lpr * 16) { fail("matvec: matrix tile does not match the uop"); return -1; }
                release(c, m);
                if (--v.left == 0) {
                    release(c, v.b);
                    if (!store_returns(c, v.q)) return -1;
                    v.in_uop = false;
                    v.s.pc++;
                }
            }
            return 1;
        }
        if (v.phase >= 30) {
            const uint32_t row = v.lpr * 16, prow = row + 16;     // bytes of a key / value row, of a partial row
            switch (v.phase) {
                case 30:
                    if (m.is_store || m.rows != 1 || m.row_bytes != row) { fail("attn: the query tile is not one row of d values"); return -1; }
                    v.q = m; v.phase = 31;
                    break;
                case 31:
                    if (m.is_store || m.box_rows != v.R || m.lds_pitch != row || m.row_bytes != row) { fail("attn: key tile does not match the uop"); return -1; }
                    v.a = m; v.phase = 32;
                    break;
                case 32:
                    if (m.is_store || m.box_rows != v.R || m.lds_pitch != row || m.row_bytes != row || m.rows != v.a.rows) { fail("attn: value tile does not match the key tile"); return -1; }
                    release(c, v.a);
                    release(c, m);
                    if (--v.left == 0) { release(c, v.q); v.phase = v.join ? 34 : 33; } else v.phase = 31;
                    break;
                case 34:
                    if (m.is_store || m.rows != v.join || m.row_bytes != prow || m.lds_pitch != prow) { fail("attn: the tile behind the last pair is not the partial rows to join"); return -1; }
                    release(c, m);
                    v.phase = 33;
                    break;
                case 33:
                    // a partial row (o, m, l, 0, 0) of a context that other items share, or the finished row of d values of a
                    // context the uop saw all of or joined the rest of
                    if (!m.is_store || m.rows != 1 || (m.row_bytes != prow && m.row_bytes != row) || (v.join && m.row_bytes != row)) { fail("attn: the output region is neither a partial row nor a result row"); return -1; }
                    if (!store_returns(c, m)) return -1;
                    v.in_uop = false; v.s.pc++;
                    break;
                case 40:
                    if (m.is_store || m.rows != v.left || m.row_bytes != prow || m.lds_pitch != prow) { fail("attn_merge: the tile is not `size` partial rows"); return -1; }
                    v.a = m; v.phase = 41;
                    break;
                default:
                    if (!m.is_store || m.rows != 1 || m.row_bytes != row) { fail("attn_merge: the output region is not one row of d values"); return -1; }
                    release(c, v.a);
                    if (!store_returns(c, m)) return -1;
                    v.in_uop = false; v.s.pc++;
                    break;
            }
            return 1;
        }
        if (v.phase >= 20) {
            const uint64_t need = (uint64_t)v.chunks * 16, have = (uint64_t)m.nslots * cfg.slot_bytes;
            if (v.phase == 20 || v.phase == 22) {
                if (m.is_store) { fail("stream uop: expected a loaded region"); return -1; }
                if (need > have) { fail("copy: more bytes than the loaded region holds"); return -1; }
                if (v.phase == 20) release(c, m); else v.a = m;
            } else {
                if (!m.is_store) { fail("stream uop: expected an output region"); return -1; }
                if (need > have) { fail("stream uop: more bytes than the output region holds"); return -1; }
                if (v.phase == 23) release(c, v.a);
                if (!store_returns(c, m)) return -1;
            }
            if (v.phase == 22) { v.phase = 23; return 1; }
            if (v.phase == 23) v.phase = 22;
            if (--v.left == 0) { v.in_uop = false; v.s.pc++; }
            return 1;
        }
        if (v.phase >= 10) {
            if (v.phase < 12) {
                if (m.is_store || m.rows != v.B || m.box_rows != v.B || m.lds_pitch != v.R * 4) { fail("rope: input tile does not match the uop"); return -1; }
                if (v.phase == 10) v.a = m; else v.b = m;
                v.phase++;
            } else {
                if (!m.is_store || m.rows != v.B || m.lds_pitch != v.R * 4 || m.row_bytes > v.R * 4) { fail("rope: output region does not match the uop"); return -1; }
                release(c, v.a);
                release(c, v.b);
                if (!store_returns(c, m)) return -1;
                v.in_uop = false;
                v.s.pc++;
            }
            return 1;
        }
        if (v.phase == 3) {
            // the vector tile of the next min(xspan, left) steps
            const uint32_t need = std::min(v.xspan, v.left);
            const bool ok1 = v.B == 1 && m.lds_pitch == v.lpr * 16 && m.row_bytes == v.lpr * 16 && m.rows >= need;
            // several vectors: B rows of xspan pieces side by side
            const bool okb = v.B > 1 && m.rows == v.B && m.box_rows == v.B && m.lds_pitch == v.xspan * v.lpr * 16 && m.row_bytes >= need * v.lpr * 16 && m.row_bytes <= m.lds_pitch;
            if (m.is_store || !(ok1 || okb)) { fail("matvec: vector tile does not hold the steps it is popped for"); return -1; }
            v.b = m;
            v.holds_x = true;
            v.xstep = 0;
            v.phase = 0;
        } else if (v.phase == 0 && v.xspan >= 2) {
            if (m.is_store || m.box_rows != v.R || m.lds_pitch != v.lpr * 16) { fail("matvec: matrix tile does not match the uop"); return -1; }
            release(c, m);
            v.xstep++;
            v.left--;
            if (v.left == 0 || v.xstep == v.xspan) {
                release(c, v.b);
                v.holds_x = false;
                v.phase = v.left == 0 ? 2 : 3;
            }
        } else if (v.phase == 0) {
            if (m.is_store || m.box_rows != v.R || m.lds_pitch != v.lpr * 16) { fail("matvec: matrix tile does not match the uop"); return -1; }
            v.a = m;
            v.phase = 1;
        } else if (v.phase == 1) {
            if (m.is_store || m.box_rows != v.B || m.rows != v.B || m.lds_pitch != v.lpr * 16) { fail("matvec: vector tile does not match the uop"); return -1; }
            release(c, v.a);
            release(c, m);
            if (--v.left == 0) v.phase = 2; else v.phase = 0;
        } else {
            if (!m.is_store || m.rows != v.B || m.lds_pitch != v.R * 4 || m.row_bytes > v.R * 4) { fail("matvec: output region does not match the uop"); return -1; }
            if (!store_returns(c, m)) return -1;
            v.in_uop = false;
            v.s.pc++;
        }
        return 1;
    }

    bool run() {
        const int V = cfg.vcc_per_core, C = cfg.n_cores;
        dep.assign(cfg.n_dep_ids, 0);
        std::vector<CoreH> cores(C);
        for (int c = 0; c < C; c++) {
            uint32_t base = c * (1 + V);
            for (int k = 0; k <= V; k++) {
                if (sb[base + k] > sb[base + k + 1] || (int64_t)sb[base + k + 1] > n_words) return fail("stream_begin is not a partition of the uops");
            }
            cores[c].vmc.pc = cores[c].vmc.begin = sb[base];
            cores[c].vmc.end = sb[base + 1];
            cores[c].vcc.resize(V);
            for (int v = 0; v < V; v++) {
                cores[c].vcc[v].s.pc = cores[c].vcc[v].s.begin = sb[base + 1 + v];
                cores[c].vcc[v].s.end = sb[base + 2 + v];
            }
        }
        const int64_t step_limit = 400000000;
        std::vector<char> done(C, 0);
        int n_done = 0;
        while (n_done < C) {
            bool progress = false;
            for (int c = 0; c < C; c++) {
                if (done[c]) continue;
                CoreH &core = cores[c];
                // run this core as far as it goes on its own
                for (;;) {
                    bool moved = false;
                    for (;;) {
                        int r = cfu_step(core);
                        if (r < 0) return false;
                        if (r == 0) break;
                        moved = true;
                        if (++steps > step_limit) return fail("program too long to validate");
                    }
                    for (auto &v : core.vcc) {
                        for (;;) {
                            int r = vcc_step(core, v);
                            if (r < 0) return false;
                            if (r == 0) break;
                            moved = true;
                            if (++steps > step_limit) return fail("program too long to validate");
                        }
                    }
                    if (!moved) break;
                    progress = true;
                }
                bool fin = core.vmc.halted;
                for (auto &v : core.vcc) fin = fin && v.s.halted && !v.in_uop && v.m2c.empty();
                if (fin) {
                    if (core.mask != 0 || !core.stores_waiting.empty() || !core.parked[0].empty() || !core.parked[1].empty()) return fail("a core ends with slots still allocated");
                    done[c] = 1;
                    n_done++;
                    progress = true;
                }
            }
            if (!progress) return fail("deadlock under in-order execution (slots over-committed, a missing send, or a depId that is never signalled)");
        }
        return true;
    }
};

// ------------------------------------------------------------------------------------------------------------
// Matvec tiler: rows of M are cut into blocks of R rows (Section 3 tiles the matrix along its row dimension);
// every core gets a contiguous range of blocks and deals them alternately to its compute cores; the K loop
// and the block loop are LOOP/REPEAT nests over dynamic addresses (Section 5).
// Tensors: 0 = M, 1 = X, 2 = Y.
// ------------------------------------------------------------------------------------------------------------
struct Run {        // consecutive row blocks of one segment handled by one core
    int64_t m_off;  // byte offset of the first row in M
    int64_t x_off;  // byte offset of the segment's vector(s) in X
    int64_t y_off;  // byte offset of the first result in Y
    int64_t n_full; // full blocks of R rows
    int32_t tail;   // rows of a final partial block, 0 if none
};

constexpr uint32_t kRopeTempTensor = 4;     // the intermediate O = M X of the fused operator before the placement step

struct Tiler {
    const vdc_config &cfg;
    int64_t K, ld, y_pitch;  // elements
    int32_t B, R, Kt;
    std::vector<std::vector<Word>> streams;
    std::vector<Desc> descs;
    bool nt = true;
    bool rope = false;     // fused form: O = M X stays in local memory and a ROPE uop turns it (tensor 3 = T) before the store
    bool x_span_ok = true; // one vector tile for several steps where the shape allows it
    uint32_t vcc_xspan = 0;
    int rowspan = 0;       // K fits one tile: row blocks per MATVEC (0, 1: one, the uop of the listing)
    int k_unroll = 1;      // measured: 2 saves front-end work but makes every load unit alternate between two static records; slower
    bool k_skew = false;   // measured on cfg5: no gain (the vector tiles are not what the cores wait for)

    uint32_t desc(uint32_t tensor, uint32_t box_rows, uint32_t row_bytes, uint32_t lds_pitch, uint64_t gpitch) {
        Desc d{tensor, box_rows, row_bytes, lds_pitch, (uint32_t)gpitch, (uint32_t)(gpitch >> 32), 0, 0};
        for (size_t i = 0; i < descs.size(); i++)
            if (!memcmp(&descs[i], &d, sizeof d)) return (uint32_t)i;
        descs.push_back(d);
        return (uint32_t)descs.size() - 1;
    }
    uint32_t slots_for(uint64_t bytes) const { return (uint32_t)((bytes + cfg.slot_bytes - 1) / cfg.slot_bytes); }
    std::vector<Word> &vmc(int core) { return streams[core * (1 + cfg.vcc_per_core)]; }
    std::vector<Word> &vcc(int core, int v) { return streams[core * (1 + cfg.vcc_per_core) + 1 + v]; }

    // virtual flows: matrix tiles of compute core v on flow v, vector tiles on flow V + v, stores on flow 2V + v
    uint32_t flow_m(int v) const { return (uint32_t)v; }
    uint32_t flow_x(int v) const { return (uint32_t)(cfg.vcc_per_core + v); }
    uint32_t flow_y(int v) const { return (uint32_t)(2 * cfg.vcc_per_core + v); }

    // What follows the K loop of one row block on the memory core: the store of the result, or, fused with rope
    // (Section 3's running example), store.local + load.local hand the matvec's region on to the ROPE uop of the same
    // compute core, a load brings the (cos, sin) tile, and the store writes what ROPE produced.
    void emit_result(std::vector<Word> &vm, int v, uint32_t flags_dyn, uint32_t acc, int64_t y_off, uint32_t dy, uint32_t rows_valid, uint32_t y_slots) {
        if (rope) {
            // The two operators as they come: O = M X is stored to a temporary tensor (4, shaped like Y) and rope loads it
            // back.  The generator's placement step (place_local_in_streams, Section 4.2) then finds the one-to-one pair
            // and keeps O in local memory; the temporary tensor is never touched.
            const uint32_t d_o = desc(kRopeTempTensor, B, rows_valid * 4, R * 4, (uint64_t)y_pitch * 4);
            const uint32_t d_t = desc(3, B, rows_valid * 4, R * 4, (uint64_t)y_pitch * 4);
            vm.push_back(encode(OP_STORE, F_SEND | F_RECV | flags_dyn, flow_y(v), v, acc, y_slots, B, 0, y_off, d_o, 0));
            vm.push_back(encode(OP_LOAD, F_SEND | flags_dyn, flow_y(v), v, acc, y_slots, B, 0, y_off, d_o, 0));
            vm.push_back(encode(OP_LOAD, F_SEND | flags_dyn, flow_x(v), v, acc, y_slots, B, 0, y_off, d_t, 0));
        }
        vm.push_back(encode(OP_STORE, F_SEND | F_RECV | flags_dyn, flow_y(v), v, acc, y_slots, B, 0, y_off, dy, 0));
    }

    // `count` iterations; in each, every compute core in `vs` takes one block of `rows_valid` rows.
    void emit_blocks(int core, const std::vector<int> &vs, int64_t count, int64_t m_off, int64_t x_off, int64_t y_off,
                     uint32_t rows_valid) {
        auto &vm = vmc(core);
        const int64_t nk_full = K / Kt, ktail = K % Kt;
        const int n = (int)vs.size();
        const uint32_t dm = desc(0, R, Kt * 4, Kt * 4, (uint64_t)ld * 4), dx = desc(1, B, Kt * 4, Kt * 4, (uint64_t)K * 4);
        const uint32_t dmt = ktail ? desc(0, R, (uint32_t)ktail * 4, Kt * 4, (uint64_t)ld * 4) : 0;
        const uint32_t dxt = ktail ? desc(1, B, (uint32_t)ktail * 4, Kt * 4, (uint64_t)K * 4) : 0;
        const uint32_t dy = desc(2, B, rows_valid * 4, R * 4, (uint64_t)y_pitch * 4);
        const uint32_t nk = (uint32_t)(nk_full + (ktail ? 1 : 0));
        const uint32_t m_slots = slots_for((uint64_t)R * Kt * 4), x_slots = slots_for((uint64_t)B * Kt * 4), y_slots = slots_for((uint64_t)B * R * 4);
        const uint32_t m_flags = F_SEND | F_DYNAMIC | (nt ? F_NT : 0);
        // One vector: a vector tile is a small part of a slot, and half of all memory uops only fetch vector tiles.  A
        // vector tile of xspan rows (xspan * Kt floats, still one slot) then serves xspan consecutive steps.
        uint32_t xspan = 0;
        // (Measured: +6 % on 8 KB tiles, where the front end sets the pace; 2 % slower on 16 KB tiles, which memory bounds.)
        if (x_span_ok && count <= 8 && B == 1 && !ktail && Kt <= 256 && nk_full >= 2 && (int64_t)R * Kt * 4 <= 8192)
            for (uint32_t n2 = kMaxXspan; n2 >= 2; n2 >>= 1)
                if (nk_full % n2 == 0 && (uint64_t)n2 * Kt * 4 <= (uint64_t)cfg.slot_bytes) { xspan = n2; break; }
        vcc_xspan = xspan;
        if (count <= 8 && xspan >= 2) {
            const uint32_t dxs = desc(1, xspan, Kt * 4, Kt * 4, (uint64_t)Kt * 4);
            for (int64_t it = 0; it < count; it++) {
                int64_t k0 = (k_skew && nk_full >= 8) ? ((int64_t)core * nk_full / cfg.n_cores) : 0;
                k0 -= k0 % xspan;
                auto sweep = [&](int64_t first, int64_t steps) {
                    if (steps <= 0) return;
                    const int64_t outer = steps / xspan;         // steps is a multiple of xspan
                    vm.push_back(encode(OP_SET, 0, 0, 0, 2, 0, 0, 0, first * Kt * 4, 0, 0));
                    if (outer > 1) vm.push_back(encode(OP_LOOP, 0, 0, 0, 0, 0, 0, 0, outer, 0, 0));
                    for (int i = 0; i < n; i++)
                        vm.push_back(encode(OP_LOAD, F_SEND | F_DYNAMIC, flow_x(vs[i]), vs[i], 2, 1, xspan, 0, x_off, dxs, 0));
                    // two steps per trip: the four matrix tiles of a trip are one batch for the front end and go to four
                    // different load units (the vector tiles' units have little else to do now), one static record each
                    if (xspan > 2) vm.push_back(encode(OP_LOOP, 0, 0, 0, 0, 0, 0, 0, xspan / 2, 0, 0));
                    for (int u = 0; u < 2; u++)
                        for (int i = 0; i < n; i++) {
                            const int64_t blk = it * n + i;
                            vm.push_back(encode(OP_LOAD, m_flags, u ? flow_x(vs[i]) : flow_m(vs[i]), vs[i], 2, m_slots, rows_valid, 0,
                                                m_off + blk * R * ld * 4 + (int64_t)u * Kt * 4, dm, 0));
                        }
                    vm.push_back(encode(xspan > 2 ? OP_REPEAT : OP_ADD, 0, 0, 0, 2, 0, 0, 0, 2 * (int64_t)Kt * 4, 0, 0));
                    if (outer > 1) vm.push_back(encode(OP_REPEAT, 0, 0, 0, 7, 0, 0, 0, 0, 0, 0));
                };
                sweep(k0, nk_full - k0);
                sweep(0, k0);
                for (int i = 0; i < n; i++) emit_result(vm, vs[i], 0, 0, y_off + (it * n + i) * R * 4, dy, rows_valid, y_slots);
            }
        } else if (count <= 8 && B > 1 && (cfg.issue_flags & 2) && !ktail && nk_full >= 4 && nk_full % 2 == 0 && Kt <= 256 &&
                   matvec_xspan_ok((uint32_t)B, (uint32_t)R, (uint32_t)Kt / 4) && (uint64_t)B * 2 * Kt * 4 <= (uint64_t)cfg.slot_bytes) {
            // Several vectors whose tile fills half a slot at most: a vector tile holds the pieces of two steps (B rows of
            // two pieces side by side, one slot), so a trip of two steps is one vector tile and two matrix tiles per compute
            // core: a slot less per step in flight and three memory uops instead of four.  On request only (measured on
            // 32768 x 65536 with eight vectors: 63 % of the HBM peak against 85 % step by step with 16 KB tiles, 51 % against
            // 62 % with 8 KB tiles, whose uops all take one slot: the fewer uops do not make up for what the compute uop's
            // second pop and the kept tile cost per step).
            vcc_xspan = 2;
            const uint32_t dx2 = desc(1, B, 2 * Kt * 4, 2 * Kt * 4, (uint64_t)K * 4);
            for (int64_t it = 0; it < count; it++) {
                vm.push_back(encode(OP_SET, 0, 0, 0, 2, 0, 0, 0, 0, 0, 0));
                vm.push_back(encode(OP_LOOP, 0, 0, 0, 0, 0, 0, 0, nk_full / 2, 0, 0));
                for (int i = 0; i < n; i++)
                    vm.push_back(encode(OP_LOAD, F_SEND | F_DYNAMIC, flow_x(vs[i]), vs[i], 2, 1, B, 0, x_off, dx2, 0));
                for (int u = 0; u < 2; u++)
                    for (int i = 0; i < n; i++) {
                        const int64_t blk = it * n + i;
                        vm.push_back(encode(OP_LOAD, m_flags, u ? flow_x(vs[i]) : flow_m(vs[i]), vs[i], 2, m_slots, rows_valid, 0,
                                            m_off + blk * R * ld * 4 + (int64_t)u * Kt * 4, dm, 0));
                    }
                vm.push_back(encode(OP_REPEAT, 0, 0, 0, 2, 0, 0, 0, 2 * (int64_t)Kt * 4, 0, 0));
                for (int i = 0; i < n; i++) emit_result(vm, vs[i], 0, 0, y_off + (it * n + i) * R * 4, dy, rows_valid, y_slots);
            }
        } else if (count <= 8) {
            // Few iterations: the block loop is unrolled, every block's addresses are literals plus ONE accumulator
            // (2: the offset along K, shared by the matrix and the vector tiles), so that the K loop costs a single
            // control uop per trip.
            for (int64_t it = 0; it < count; it++) {
                vm.push_back(encode(OP_SET, 0, 0, 0, 2, 0, 0, 0, 0, 0, 0));
                auto tile_pairs = [&](uint32_t d_m, uint32_t d_x, int64_t koff) {
                    for (int i = 0; i < n; i++) {
                        const int v = vs[i];
                        const int64_t blk = it * n + i;
                        vm.push_back(encode(OP_LOAD, m_flags, flow_m(v), v, 2, m_slots, rows_valid, 0, m_off + blk * R * ld * 4 + koff, d_m, 0));
                        vm.push_back(encode(OP_LOAD, F_SEND | F_DYNAMIC, flow_x(v), v, 2, x_slots, B, 0, x_off + koff, d_x, 0));
                    }
                };
                // U K steps per trip.  (Two per trip halve the front end's fixed cost per uop, but a batch is only
                // published when all of it is allocated, and the longer wait for the first tiles costs more.)
                // Every core starts its sweep over K at a different tile (and wraps around): cores that run in step
                // would otherwise all ask the L2 for the same vector tile at the same moment.
                const int64_t k0 = (k_skew && nk_full >= 8) ? ((int64_t)core * nk_full / cfg.n_cores) : 0;
                // k_unroll K steps per loop trip: one control uop per k_unroll steps (the front end still dispatches
                // at most kBatch memory uops at a time, see the kernel)
                auto sweep = [&](int64_t first, int64_t steps) {
                    if (steps <= 0) return;
                    vm.push_back(encode(OP_SET, 0, 0, 0, 2, 0, 0, 0, first * Kt * 4, 0, 0));
                    const int64_t U = steps >= 2 * k_unroll ? k_unroll : 1, trips = steps / U, rest = steps % U;
                    if (trips > 1) vm.push_back(encode(OP_LOOP, 0, 0, 0, 0, 0, 0, 0, trips, 0, 0));
                    for (int64_t uu = 0; uu < U; uu++) tile_pairs(dm, dx, uu * Kt * 4);
                    vm.push_back(encode(trips > 1 ? OP_REPEAT : OP_ADD, 0, 0, 0, 2, 0, 0, 0, U * (int64_t)Kt * 4, 0, 0));
                    for (int64_t uu = 0; uu < rest; uu++) {
                        tile_pairs(dm, dx, 0);
                        vm.push_back(encode(OP_ADD, 0, 0, 0, 2, 0, 0, 0, (int64_t)Kt * 4, 0, 0));
                    }
                };
                sweep(k0, nk_full - k0);
                if (ktail) tile_pairs(dmt, dxt, 0);      // acc 2 is at the end of the last full tile here
                sweep(0, k0);
                for (int i = 0; i < n; i++) emit_result(vm, vs[i], 0, 0, y_off + (it * n + i) * R * 4, dy, rows_valid, y_slots);
            }
        } else if (nk == 1) {
            // One tile per row block (K fits a tile): no loop over K.  One accumulator runs over the matrix tiles and one
            // over the results; the compute cores are told apart by the literal part of the address, the vector tile's
            // address is a literal.  Two control uops per trip, and the memory uops of a trip stand together.
            vm.push_back(encode(OP_SET, 0, 0, 0, 0, 0, 0, 0, m_off, 0, 0));
            vm.push_back(encode(OP_SET, 0, 0, 0, 3, 0, 0, 0, y_off, 0, 0));
            vm.push_back(encode(OP_LOOP, 0, 0, 0, 0, 0, 0, 0, count, 0, 0));
            for (int i = 0; i < n; i++) {
                const int v = vs[i];
                vm.push_back(encode(OP_LOAD, m_flags, flow_m(v), v, 0, m_slots, rows_valid, 0, (int64_t)i * R * ld * 4, nk_full ? dm : dmt, 0));
                vm.push_back(encode(OP_LOAD, F_SEND, flow_x(v), v, 0, x_slots, B, 0, x_off, nk_full ? dx : dxt, 0));
            }
            for (int i = 0; i < n; i++) emit_result(vm, vs[i], F_DYNAMIC, 3, (int64_t)i * R * 4, dy, rows_valid, y_slots);
            vm.push_back(encode(OP_ADD, 0, 0, 0, 3, 0, 0, 0, (int64_t)n * R * 4, 0, 0));
            vm.push_back(encode(OP_REPEAT, 0, 0, 0, 0, 0, 0, 0, (int64_t)n * R * ld * 4, 0, 0));
        } else {
            // accumulators: 0,1 matrix offset of compute core 0,1; 2 vector offset; 3,4 result offset of compute core 0,1
            for (int i = 0; i < n; i++) {
                vm.push_back(encode(OP_SET, 0, 0, 0, vs[i], 0, 0, 0, m_off + (int64_t)i * R * ld * 4, 0, 0));
                vm.push_back(encode(OP_SET, 0, 0, 0, 3 + vs[i], 0, 0, 0, y_off + (int64_t)i * R * 4, 0, 0));
            }
            vm.push_back(encode(OP_SET, 0, 0, 0, 2, 0, 0, 0, x_off, 0, 0));
            vm.push_back(encode(OP_LOOP, 0, 0, 0, 0, 0, 0, 0, count, 0, 0));
            auto tile_pairs = [&](uint32_t d_m, uint32_t d_x) {
                for (int i = 0; i < n; i++) {
                    const int v = vs[i];
                    vm.push_back(encode(OP_LOAD, m_flags, flow_m(v), v, v, m_slots, rows_valid, 0, 0, d_m, 0));
                    vm.push_back(encode(OP_LOAD, F_SEND | F_DYNAMIC, flow_x(v), v, 2, x_slots, B, 0, 0, d_x, 0));
                }
            };
            if (nk_full > 0) {
                if (nk_full > 1) vm.push_back(encode(OP_LOOP, 0, 0, 0, 0, 0, 0, 0, nk_full, 0, 0));
                tile_pairs(dm, dx);
                for (int i = 0; i < n; i++) vm.push_back(encode(OP_ADD, 0, 0, 0, vs[i], 0, 0, 0, (int64_t)Kt * 4, 0, 0));
                vm.push_back(encode(nk_full > 1 ? OP_REPEAT : OP_ADD, 0, 0, 0, 2, 0, 0, 0, (int64_t)Kt * 4, 0, 0));
            }
            if (ktail) tile_pairs(dmt, dxt);
            for (int i = 0; i < n; i++) emit_result(vm, vs[i], F_DYNAMIC, 3 + vs[i], 0, dy, rows_valid, y_slots);
            for (int i = 0; i < n; i++) {
                vm.push_back(encode(OP_ADD, 0, 0, 0, vs[i], 0, 0, 0, (int64_t)n * R * ld * 4 - nk_full * Kt * 4, 0, 0));
                vm.push_back(encode(OP_ADD, 0, 0, 0, 3 + vs[i], 0, 0, 0, (int64_t)n * R * 4, 0, 0));
            }
            vm.push_back(encode(OP_REPEAT, 0, 0, 0, 2, 0, 0, 0, -nk_full * Kt * 4, 0, 0));
        }
        for (int i = 0; i < n; i++) {
            auto &vc = vcc(core, vs[i]);
            if (count > 1) vc.push_back(encode(OP_LOOP, 0, 0, 0, 0, 0, 0, 0, count, 0, 0));
            vc.push_back(encode(OP_MATVEC, 0, 0, 0, 0, 0, nk, 0, matvec_imm(B, R, Kt / 4, vcc_xspan), 0, 0));
            if (rope) vc.push_back(encode(OP_ROPE, 0, 0, 0, 0, 0, 1, 0, rope_imm(B, R), 0, 0));
            if (count > 1) vc.push_back(encode(OP_REPEAT, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0));
        }
    }

    // One K range [kt0, kt1) (in tiles; the last range also takes the K tail) of one row block per compute core in
    // `vs`.  Every range but the last stores its partial sums to the workspace (tensor 3) and signals its row block's depId.
    // The workspace keeps the S - 1 partial results of a cut row block (counted from rb0, the first of them) side by side,
    // [row block - rb0][B][S - 1][R], so that G =
    // Kt / R of them are one vector tile ([B] rows of G R values).  The last range then adds them, G per extra tile step:
    // the matrix tile is [I I .. I | 0] (G unit matrices, from the workspace) and the vector tile holds G partial results
    // (the rest of its row reads as zero), fetched with a load that waits for the depId (Section 4.1: a load with an
    // inter-memory-uop dependency), and stores to Y.  The order of the additions is fixed by the program.
    void emit_split(int core, const std::vector<int> &vs, const std::vector<int64_t> &rbs, int s, int S, int64_t kt0, int64_t kt1,
                    int64_t rows_total, int64_t rb0, int64_t p_base) {
        auto &vm = vmc(core);
        const int64_t nk_all = K / Kt, ktail = K % Kt;
        const int n = (int)vs.size();
        const int64_t full = std::min(kt1, nk_all) - kt0;            // full tiles of this range
        const bool with_tail = ktail && kt1 > nk_all;
        const uint32_t m_slots = slots_for((uint64_t)R * Kt * 4), x_slots = slots_for((uint64_t)B * Kt * 4), y_slots = slots_for((uint64_t)B * R * 4);
        const uint32_t m_flags = F_SEND | F_DYNAMIC | (nt ? F_NT : 0);
        const uint32_t dx = desc(1, B, Kt * 4, Kt * 4, (uint64_t)K * 4);
        const uint32_t dxt = ktail ? desc(1, B, (uint32_t)ktail * 4, Kt * 4, (uint64_t)K * 4) : 0;
        const int64_t G = Kt / R, prow = (int64_t)(S - 1) * R;       // partial results per join step; values per row of a block's partial results
        const int64_t nq = (S - 1 + G - 1) / G;                      // join steps
        const uint32_t d_id = desc(3, R, Kt * 4, Kt * 4, (uint64_t)Kt * 4);                    // [I I .. I | 0]
        const uint32_t d_ps = desc(3, B, R * 4, R * 4, (uint64_t)prow * 4);                    // partial result store
        vm.push_back(encode(OP_SET, 0, 0, 0, 2, 0, 0, 0, kt0 * Kt * 4, 0, 0));
        std::vector<uint32_t> rows_valid(n);
        for (int i = 0; i < n; i++) rows_valid[i] = (uint32_t)std::min<int64_t>(R, rows_total - rbs[i] * R);
        auto tile_pairs = [&](bool tail) {
            for (int i = 0; i < n; i++) {
                const int v = vs[i];
                const uint32_t d_m = tail ? desc(0, R, (uint32_t)ktail * 4, Kt * 4, (uint64_t)ld * 4) : desc(0, R, Kt * 4, Kt * 4, (uint64_t)ld * 4);
                vm.push_back(encode(OP_LOAD, m_flags, flow_m(v), v, 2, m_slots, rows_valid[i], 0, rbs[i] * R * ld * 4, d_m, 0));
                vm.push_back(encode(OP_LOAD, F_SEND | F_DYNAMIC, flow_x(v), v, 2, x_slots, B, 0, 0, tail ? dxt : dx, 0));
            }
        };
        if (full > 0) {
            if (full > 1) vm.push_back(encode(OP_LOOP, 0, 0, 0, 0, 0, 0, 0, full, 0, 0));
            tile_pairs(false);
            vm.push_back(encode(full > 1 ? OP_REPEAT : OP_ADD, 0, 0, 0, 2, 0, 0, 0, (int64_t)Kt * 4, 0, 0));
        }
        if (with_tail) tile_pairs(true);
        if (s == S - 1) {
            // Every partial result of row block rb signals depId rb; the first load of them waits until all S - 1 have
            // (one round trip to the counter per joining item, not one per partial result), the others follow it on the same
            // load unit and need no wait of their own.  All are read at device scope: the waiting unit then needs no
            // acquire, which would empty its whole L2.
            for (int64_t q = 0; q < nq; q++)
                for (int i = 0; i < n; i++) {
                    const int v = vs[i];
                    const int64_t g = std::min<int64_t>(G, S - 1 - q * G);                     // partial results of this step
                    const uint32_t d_pl = desc(3, B, (uint32_t)(g * R * 4), Kt * 4, (uint64_t)prow * 4);
                    vm.push_back(encode(OP_LOAD, F_SEND, flow_m(v), v, 0, m_slots, R, 0, 0, d_id, 0));
                    vm.push_back(encode(OP_LOAD, F_SEND | F_DEVICE | (q == 0 ? F_DEP_RECV : 0u), flow_x(v), v, 0, x_slots, B, q == 0 ? (uint32_t)(rbs[i] - rb0) : 0u,
                                        p_base + ((rbs[i] - rb0) * B * prow + q * G * R) * 4, d_pl, q == 0 ? (uint32_t)(S - 1) : 0u));
                }
        }
        for (int i = 0; i < n; i++) {
            const int v = vs[i];
            if (s < S - 1) {
                vm.push_back(encode(OP_STORE, F_SEND | F_RECV | F_DEP_SEND, flow_y(v), v, 0, y_slots, B, (uint32_t)(rbs[i] - rb0),
                                    p_base + ((rbs[i] - rb0) * B * prow + (int64_t)s * R) * 4, d_ps, 0));
            } else {
                const uint32_t dy = desc(2, B, rows_valid[i] * 4, R * 4, (uint64_t)y_pitch * 4);
                vm.push_back(encode(OP_STORE, F_SEND | F_RECV, flow_y(v), v, 0, y_slots, B, 0, rbs[i] * R * 4, dy, 0));
            }
            const uint32_t nk = (uint32_t)(full + (with_tail ? 1 : 0) + (s == S - 1 ? nq : 0));
            vcc(core, v).push_back(encode(OP_MATVEC, 0, 0, 0, 0, 0, nk, 0, matvec_imm(B, R, Kt / 4), 0, 0));
        }
    }

    // K fits one tile and there are many row blocks per compute core: a MATVEC covers up to `rowspan` consecutive blocks of
    // a segment, which share the segment's vector tile and one STORE (the uop's tile is tall, its I/O blocks keep the
    // configured size).  Per group: the STORE first (the compute core holds the output region throughout), the vector
    // tile, the matrix tiles; groups alternate between the compute cores; every address is a literal.
    void emit_core_rows(int core, const std::vector<Run> &runs) {
        const int V = cfg.vcc_per_core;
        auto &vm = vmc(core);
        const uint32_t kbytes = (uint32_t)K * 4;
        const uint32_t dm = desc(0, R, kbytes, Kt * 4, (uint64_t)ld * 4), dx = desc(1, B, kbytes, Kt * 4, (uint64_t)K * 4);
        const uint32_t m_slots = slots_for((uint64_t)R * Kt * 4), x_slots = slots_for((uint64_t)B * Kt * 4);
        const uint32_t m_flags = F_SEND | (nt ? F_NT : 0);
        int g = 0;
        for (const Run &r : runs) {
            const int64_t blocks = r.n_full + (r.tail ? 1 : 0), rows_run = r.n_full * R + r.tail;
            for (int64_t done = 0; done < blocks;) {
                const int64_t nb = std::min<int64_t>(rowspan, blocks - done);
                const int64_t rows_valid = std::min<int64_t>(nb * R, rows_run - done * R);
                const int v = g++ % V;
                const uint32_t dy = desc(2, B, (uint32_t)rows_valid * 4, (uint32_t)(nb * R * 4), (uint64_t)y_pitch * 4);
                const uint32_t y_slots = slots_for((uint64_t)B * nb * R * 4);
                if (nb >= 2) vm.push_back(encode(OP_STORE, F_SEND | F_RECV, flow_y(v), v, 0, y_slots, B, 0, r.y_off + done * R * 4, dy, 0));
                if (nb >= 2) vm.push_back(encode(OP_LOAD, F_SEND, flow_x(v), v, 0, x_slots, B, 0, r.x_off, dx, 0));
                for (int64_t j = 0; j < nb; j++) {
                    const uint32_t rv = (uint32_t)std::min<int64_t>(R, rows_valid - j * R);
                    // the matrix tiles of a compute core take turns on its two flows: with four load units every unit then
                    // carries a quarter of them (a load unit's cost is per uop: two units alone set the pace on 8 KB tiles)
                    vm.push_back(encode(OP_LOAD, m_flags, (j & 1) ? flow_x(v) : flow_m(v), v, 0, m_slots, rv, 0, r.m_off + (done + j) * R * ld * 4, dm, 0));
                }
                if (nb < 2) {      // a single block: the uop of the listing (matrix tile, vector tile, then the output region)
                    vm.push_back(encode(OP_LOAD, F_SEND, flow_x(v), v, 0, x_slots, B, 0, r.x_off, dx, 0));
                    vm.push_back(encode(OP_STORE, F_SEND | F_RECV, flow_y(v), v, 0, y_slots, B, 0, r.y_off + done * R * 4, dy, 0));
                }
                vcc(core, v).push_back(encode(OP_MATVEC, 0, 0, 0, 0, 0, 1, 0, matvec_imm(B, R, Kt / 4), nb >= 2 ? (uint32_t)nb : 0u, 0));
                done += nb;
            }
        }
    }

    void emit_core(int core, const std::vector<Run> &runs) {
        if (rowspan >= 2) return emit_core_rows(core, runs);
        const int V = cfg.vcc_per_core;
        int next_v = 0;
        for (const Run &r : runs) {
            int64_t left = r.n_full, m = r.m_off, y = r.y_off;
            const int64_t blk_m = (int64_t)R * ld * 4, blk_y = (int64_t)R * 4;
            if (V == 2) {
                if (next_v == 1 && left > 0) {  // re-align so that the paired loop starts on compute core 0
                    emit_blocks(core, {1}, 1, m, r.x_off, y, R);
                    m += blk_m; y += blk_y; left--; next_v = 0;
                }
                if (left >= 2) {
                    emit_blocks(core, {0, 1}, left / 2, m, r.x_off, y, R);
                    m += (left / 2) * 2 * blk_m; y += (left / 2) * 2 * blk_y; left -= (left / 2) * 2;
                }
                if (left == 1) {
                    emit_blocks(core, {next_v}, 1, m, r.x_off, y, R);
                    m += blk_m; y += blk_y; next_v ^= 1;
                }
                if (r.tail) {
                    emit_blocks(core, {next_v}, 1, m, r.x_off, y, (uint32_t)r.tail);
                    next_v ^= 1;
                }
            } else {
                if (left > 0) emit_blocks(core, {0}, left, m, r.x_off, y, R);
                m += left * blk_m; y += left * blk_y;
                if (r.tail) emit_blocks(core, {0}, 1, m, r.x_off, y, (uint32_t)r.tail);
            }
        }
    }
};

// Rows per matrix tile for a tile of tile_bytes: keep a tile row inside one wave (at most 64 chunks of 16 bytes,
// no cross-wave reduction), keep at least 512 contiguous bytes per row when K allows, and prefer at least 4 rows
// per right-hand vector so that the vector tiles (which come from the L2, not from HBM) stay a small part of the
// LDS fill traffic.
bool choose_tile(const vdc_config &cfg, int64_t K, int32_t B, int32_t tile_bytes, int32_t &R, int32_t &Kt) {
    const int32_t chunks = tile_bytes / 16;
    if (tile_bytes != 2048 && tile_bytes != 4096 && tile_bytes != 8192 && tile_bytes != 16384) return false;
    int32_t lpr;
    if (cfg.tile_rows > 0) {
        if (chunks % cfg.tile_rows) return false;
        lpr = chunks / cfg.tile_rows;
    } else {
        lpr = 64;
        while (lpr > 32 && chunks / lpr < 4 * B) lpr >>= 1;
        while (lpr > 1 && (int64_t)lpr * 4 >= 2 * K) lpr >>= 1;   // no tile much wider than a row
    }
    if (lpr < 1 || chunks % lpr) return false;
    R = chunks / lpr;
    Kt = lpr * 4;
    return matvec_geometry_ok((uint32_t)B, (uint32_t)R, (uint32_t)lpr, nullptr, nullptr);
}

// K of a dense matrix may be cut into S ranges: every (range, row block) pair is then a work item; the partial sums travel
// from range to range through a workspace and depId signals (Section 4.1, inter-memory-uop dependencies).  S == 1: no cut.
// S is the tiling the adaptive step of the generator chooses for the operator (Section 4.2, "Adaptive Scheduling and
// Tiling"): a matrix with fewer row blocks than compute cores, or with a number of row blocks that leaves some cores one
// block more than others, is a dominant critical path, and cutting K is the finer decomposition that removes it.
struct SplitPlan {
    int S = 1, S_max = 1;
    int64_t NB = 0, T = 0;                         // row blocks; how many of them (the last T) are cut
    int64_t ident_floats = 0, bytes = 0;           // workspace: the tile [I I .. I | 0], then the partial results [T][B][S - 1][R]
};

// The finest cut the builder offers for a shape: the joining step multiplies by an [I | 0] tile, so a tile must be at least
// as wide as it is tall; every range keeps at least four tile steps; one depId per cut row block; a core's
// stream of items stays short (the cut is for shapes with few blocks per compute core: with many the deal is even enough).
int split_max_parts(const vdc_config &cfg, int64_t NB, int64_t nk, int32_t R, int32_t Kt, bool ragged, int64_t &surplus) {
    surplus = 0;
    if (ragged || (R & 3) || R > Kt) return 1;
    const int64_t lanes = (int64_t)cfg.n_cores * cfg.vcc_per_core;
    // more row blocks than compute cores and some left over when they go round: those alone may be cut as well
    if (NB > lanes && NB % lanes) surplus = NB % lanes;
    const int64_t cut = surplus ? surplus : NB;                                 // the fewest blocks a cut may apply to
    if (cut > (int64_t)cfg.n_dep_ids) return 1;                                 // one depId per cut row block
    int64_t S = std::min<int64_t>(16, nk / 4);
    S = std::min<int64_t>(S, std::max<int64_t>(1, 8 * lanes / cut));           // at most eight items of cut blocks per compute core
    if (S < 2) surplus = 0;
    return (int)std::max<int64_t>(S, 1);
}

SplitPlan plan_split(const vdc_config &cfg, int64_t rows, int64_t K, int32_t B, int32_t R, int32_t Kt, int32_t tile_bytes, bool ragged) {
    SplitPlan sp;
    sp.NB = (rows + R - 1) / R;
    const int64_t nk = (K + Kt - 1) / Kt;
    int64_t surplus = 0;
    sp.S_max = split_max_parts(cfg, sp.NB, nk, R, Kt, ragged, surplus);
    if (sp.S_max < 2) return sp;
    int32_t S = 1, tail = 0;
    if (cfg.sched_force_parts > 0) {
        S = std::min<int32_t>(cfg.sched_force_parts % 100, sp.S_max);
        tail = cfg.sched_force_parts > 100 ? (int32_t)surplus : 0;
    } else {
        const vdc_sched_op op{sp.NB, nk, sp.S_max, Kt / R, surplus};       // a joining step adds Kt / R partial results
        if (sched_adaptive(&op, 1, nullptr, nullptr, cfg.n_cores, cfg.vcc_per_core, sched_default_cost(tile_bytes), cfg.sched_threshold_pct,
                           cfg.sched_min_gain_pct, &S, &tail, nullptr, nullptr) != VDC_OK) S = 1;
    }
    if (S < 2) return sp;
    sp.T = tail > 0 ? tail : sp.NB;
    if (sp.T > (int64_t)cfg.n_dep_ids || sp.T * S > ((int64_t)1 << 20)) return sp;   // (a cut of all blocks the builder cannot write: left whole)
    sp.S = S;
    sp.ident_floats = (int64_t)R * Kt;
    sp.bytes = (sp.ident_floats + (int64_t)(S - 1) * B * sp.T * R) * 4;
    return sp;
}

// K fits one tile: with at least two groups of row blocks per compute core a MATVEC covers several blocks, as many as keep
// its output region inside one slot, at most 8 (0: the form is not used).  nb: row blocks in all.
int rowspan_for(const vdc_config &cfg, int64_t nb, int64_t K, int32_t B, int32_t R, int32_t Kt) {
    if (K > Kt || Kt > 256 || B > (int32_t)kMaxRowspanB) return 0;
    int64_t G = std::min<int64_t>(8, nb / ((int64_t)cfg.n_cores * cfg.vcc_per_core * 2));
    G = std::min<int64_t>(G, (int64_t)cfg.slot_bytes / ((int64_t)B * R * 4));
    return G >= 2 ? (int)G : 0;
}

// Which roles share a SIMD (vdc_program_set_placement) for a matvec program: measured per form of the graph.
int matvec_placement(const vdc_config &cfg, int64_t rows, int64_t K, int32_t B, int32_t tile_bytes, bool rope) {
    int R = 0, Kt = 0;
    if (!choose_tile(cfg, K, B, tile_bytes, R, Kt)) return 0;
    if (!rope && K <= Kt) {
        // one tile per row block.  MATVECs over several row blocks: the compute waves set the pace (placement 2).  One
        // tile, one MATVEC and one STORE per row block: the front end and the store unit do (placement 1), if there are
        // enough blocks to matter
        if (rowspan_for(cfg, (rows + R - 1) / R, K, B, R, Kt) >= 2) return 2;
        return rows / R >= 8 * (int64_t)cfg.n_cores * cfg.vcc_per_core ? 1 : 0;
    }
    // long sweeps over K: the front end's loop is the busiest wave; it gets a SIMD with one compute wave only
    return K / Kt >= 16 ? 2 : 0;
}

int build_matvec(const vdc_config &cfg, int64_t rows, int64_t K, int64_t ld, int32_t B, int32_t tile_bytes,
                 const int64_t *row_off, int32_t n_seg, std::vector<Word> &words, std::vector<uint32_t> &sb,
                 std::vector<Desc> &descs, bool rope = false) {
    int32_t R = 0, Kt = 0;
    if (!choose_tile(cfg, K, B, tile_bytes, R, Kt)) return VDC_EINVAL;
    if ((uint64_t)((K + Kt - 1) / Kt) > 65535) return VDC_EINVAL;
    const int C = cfg.n_cores, V = cfg.vcc_per_core;
    Tiler t{cfg, K, ld, row_off ? 0 : rows, B, R, Kt};
    t.rope = rope;
    if (rope && (row_off || (rows & 3) || (R & 3) || !rope_geometry_ok((uint32_t)B, (uint32_t)R))) return VDC_EINVAL;
    t.streams.resize((size_t)C * (1 + V));
    // global list of row blocks, segment by segment; core c takes blocks [c*NB/C, (c+1)*NB/C)
    struct Seg { int64_t row0, len, first_block, n_blocks; };
    std::vector<Seg> segs;
    int64_t nb = 0;
    if (row_off) {
        for (int s = 0; s < n_seg; s++) {
            int64_t len = row_off[s + 1] - row_off[s];
            int64_t n = (len + R - 1) / R;
            segs.push_back({row_off[s], len, nb, n});
            nb += n;
        }
    } else {
        segs.push_back({0, rows, 0, (rows + R - 1) / R});
        nb = segs[0].n_blocks;
    }
    const SplitPlan sp = rope ? SplitPlan{} : plan_split(cfg, rows, K, B, R, Kt, tile_bytes, row_off != nullptr);
    if (!rope && sp.S == 1) t.rowspan = rowspan_for(cfg, nb, K, B, R, Kt);
    // whole row blocks: the first nw of the global list, core c takes blocks [c*nw/C, (c+1)*nw/C)
    auto deal_whole = [&](int64_t nw) {
        size_t si = 0;
        for (int c = 0; c < C; c++) {
            int64_t b0 = nw * c / C, b1 = nw * (c + 1) / C;
            std::vector<Run> runs;
            while (b0 < b1) {
                while (si < segs.size() && segs[si].first_block + segs[si].n_blocks <= b0) si++;
                const Seg &sg = segs[si];
                int64_t e = std::min(b1, sg.first_block + sg.n_blocks);
                int64_t lb0 = b0 - sg.first_block, lb1 = e - sg.first_block;   // local block range in the segment
                int64_t r0 = lb0 * R, r1 = std::min(sg.len, lb1 * R);
                Run r;
                r.m_off = (sg.row0 + r0) * ld * 4;
                r.x_off = row_off ? (int64_t)si * K * 4 : 0;
                r.y_off = (sg.row0 + r0) * 4;
                r.n_full = (r1 - r0) / R;
                r.tail = (int32_t)((r1 - r0) % R);
                runs.push_back(r);
                b0 = e;
            }
            t.emit_core(c, runs);
        }
    };
    if (sp.S > 1) {
        // The last T row blocks are cut (all of them, or the surplus that is left when the others go round the compute
        // cores evenly: those stay whole and come first in every core's stream).  Items of the cut blocks in the order
        // (range, row block); core c takes items [c*NI/C, (c+1)*NI/C).  Only items of the last range wait, and only for
        // items of earlier ranges, which earlier positions of the same or of earlier cores hold: no cycles.
        const int64_t NW = sp.NB - sp.T, NI = sp.T * sp.S, nk = (K + Kt - 1) / Kt;
        if (NW > 0) deal_whole(NW);
        for (int c = 0; c < C; c++) {
            int64_t i0 = NI * c / C, i1 = NI * (c + 1) / C;
            int next_v = 0;
            while (i0 < i1) {
                const int s0 = (int)(i0 / sp.T);
                std::vector<int> vs{V == 2 ? next_v : 0};
                std::vector<int64_t> rbs{NW + i0 % sp.T};
                if (V == 2 && i0 + 1 < i1 && (int)((i0 + 1) / sp.T) == s0) { vs = {0, 1}; rbs.push_back(NW + (i0 + 1) % sp.T); }
                else next_v ^= 1;
                t.emit_split(c, vs, rbs, s0, sp.S, nk * s0 / sp.S, nk * (s0 + 1) / sp.S, rows, NW, sp.ident_floats * 4);
                i0 += (int64_t)vs.size();
            }
        }
    } else {
        deal_whole(nb);
    }
    words.clear();
    sb.assign(1, 0);
    for (auto &s : t.streams) {
        words.insert(words.end(), s.begin(), s.end());
        words.push_back(encode(OP_HALT, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0));
        sb.push_back((uint32_t)words.size());
    }
    descs = t.descs;
    if (descs.empty()) descs.push_back(Desc{0, 1, 16, 16, 0, 0, 0, 0});
    if (rope) {
        // dynamic data placement: every row block's store of O and the load behind it become store.local / load.local
        const int placed = place_local_in_streams(cfg, words, sb, descs, 1u << kRopeTempTensor, 2u);
        int64_t stores_left = 0;
        for (const Word &w : words) {
            const Fields f = decode(w);
            if ((f.opcode == OP_LOAD || f.opcode == OP_STORE) && !(f.flags & F_LOCAL) && f.desc < descs.size() && descs[f.desc].tensor == kRopeTempTensor) stores_left++;
        }
        if (placed < 1 || stores_left != 0) return VDC_EPROGRAM;     // the intermediate would have to exist in memory
    }
    if (descs.size() > 256) return VDC_EINVAL;
    return VDC_OK;
}

// A chain of matvec operators in ONE uop graph (Section 3: operators are composed through their memory uops, not through
// kernel boundaries; Section 4.1, "Encoding dependency in uop"): Y_0 = M_0 X, Y_l = M_l Y_(l-1).  dims[0] = K_0,
// dims[l + 1] = rows of M_l.  Tensors: 0 = W, the matrices back to back (M_l is [dims[l + 1]][dims[l]], row-major);
// 1 and 2 = A, the activations back to back (X as [B][dims[0]], then every Y_l as [B][dims[l + 1]]), read as tensor 1
// and written as tensor 2.  Every layer is tiled like a single matvec (choose_tile) and its row blocks are dealt to the
// cores in contiguous ranges.  The vector tile kt of layer l + 1 is a range of rows of Y_l.  Vector tiles are taken in
// groups of G (at most 32, and at most 255 producing row blocks): the row blocks of layer l inside a group's rows signal
// the group's depId with their stores (written through at device scope), and on a core's first pass over the vector
// tiles of a layer the first load of every group waits for it, so a layer starts on a group of tiles as soon as that
// group is complete, not when the layer before it has ended.  (A wait costs a round trip to the counter: one per
// tile made a pass over K three times longer.)  Later row blocks of the same core and layer need no wait: their
// loads follow the waiting ones on the same load unit.  All vector tiles of layers after the first are read at device
// scope.  Within a stream a layer's uops precede the next layer's, and layer 0 waits for nothing: by induction over
// the layers no wait can last forever (Section 4.3, "Avoiding Deadlock").
struct ChainLayer {
    int64_t K, rows, w_off, x_off, y_off;
    int32_t R, Kt, R_prev, Kt_next;
    int32_t G, G_next;           // vector tiles per dependency group: of this layer, of the next
    int64_t rows_prev;
    int32_t dep_in, dep_out;     // first depId of this layer's vector tiles / of its outputs; -1: none
};

int build_chain(const vdc_config &cfg, const int64_t *dims, int32_t L, int32_t B, int32_t tile_bytes, std::vector<Word> &words,
                std::vector<uint32_t> &sb, std::vector<Desc> &descs, int64_t &w_bytes, int64_t &a_bytes) {
    if (!dims || L < 1 || L > 64 || B < 1 || B > 8) return VDC_EINVAL;
    for (int l = 0; l <= L; l++)
        if (dims[l] < 4 || (dims[l] & 3)) return VDC_EINVAL;
    const int C = cfg.n_cores, V = cfg.vcc_per_core;
    std::vector<ChainLayer> ly((size_t)L);
    int64_t w = 0, a = 0;
    int32_t dep = 0;
    for (int l = 0; l < L; l++) {
        ChainLayer &c = ly[(size_t)l];
        c.K = dims[l]; c.rows = dims[l + 1];
        if (!choose_tile(cfg, c.K, B, tile_bytes, c.R, c.Kt)) return VDC_EINVAL;
        if ((uint64_t)((c.K + c.Kt - 1) / c.Kt) > 65535) return VDC_EINVAL;
        c.w_off = w; c.x_off = a; c.y_off = a + (int64_t)B * c.K * 4;
        w += c.rows * c.K * 4;
        a += (int64_t)B * c.K * 4;
    }
    a += (int64_t)B * dims[L] * 4;
    w_bytes = w; a_bytes = a;
    for (int l = 0; l < L; l++) {
        ChainLayer &c = ly[(size_t)l];
        c.dep_in = -1; c.dep_out = -1; c.Kt_next = 0; c.R_prev = 0; c.rows_prev = 0; c.G = 1; c.G_next = 1;
        if (l > 0) {
            c.dep_in = ly[(size_t)l - 1].dep_out; c.R_prev = ly[(size_t)l - 1].R; c.rows_prev = ly[(size_t)l - 1].rows;
            c.G = ly[(size_t)l - 1].G_next;
        }
        if (l + 1 < L) {
            c.Kt_next = ly[(size_t)l + 1].Kt;
            if (c.Kt_next % c.R) return VDC_EINVAL;                       // a row block must lie inside one vector tile of the next layer
            const int32_t per_tile = c.Kt_next / c.R;
            if (per_tile > 255) return VDC_EINVAL;
            c.G_next = std::max(1, std::min(32, 255 / per_tile));
            c.dep_out = dep;
            dep += (int32_t)((c.rows + (int64_t)c.Kt_next * c.G_next - 1) / ((int64_t)c.Kt_next * c.G_next));
        }
    }
    if (dep > cfg.n_dep_ids) return VDC_EINVAL;
    Tiler t{cfg, 0, 0, 0, B, 1, 4};
    t.streams.resize((size_t)C * (1 + V));
    for (int l = 0; l < L; l++) {
        const ChainLayer &c = ly[(size_t)l];
        const int64_t NB = (c.rows + c.R - 1) / c.R, nk_full = c.K / c.Kt, ktail = c.K % c.Kt;
        const uint32_t nk = (uint32_t)(nk_full + (ktail ? 1 : 0));
        const uint32_t R = (uint32_t)c.R, Kt = (uint32_t)c.Kt;
        const uint32_t dm = t.desc(0, R, Kt * 4, Kt * 4, (uint64_t)c.K * 4), dx = t.desc(1, (uint32_t)B, Kt * 4, Kt * 4, (uint64_t)c.K * 4);
        const uint32_t dmt = ktail ? t.desc(0, R, (uint32_t)ktail * 4, Kt * 4, (uint64_t)c.K * 4) : 0;
        const uint32_t dxt = ktail ? t.desc(1, (uint32_t)B, (uint32_t)ktail * 4, Kt * 4, (uint64_t)c.K * 4) : 0;
        const uint32_t m_slots = t.slots_for((uint64_t)R * Kt * 4), x_slots = t.slots_for((uint64_t)B * Kt * 4), y_slots = t.slots_for((uint64_t)B * R * 4);
        const uint32_t x_flags = l > 0 ? (uint32_t)F_DEVICE : 0u;
        for (int core = 0; core < C; core++) {
            const int64_t b0 = NB * core / C, b1 = NB * (core + 1) / C;
            auto &vm = t.vmc(core);
            bool first = true;
            for (int64_t b = b0; b < b1; b += V) {
                const int n = (int)std::min<int64_t>(V, b1 - b);
                auto rows_valid = [&](int64_t blk) { return (uint32_t)std::min<int64_t>(R, c.rows - blk * R); };
                auto pairs = [&](uint32_t d_m, uint32_t d_x, uint32_t xf, uint32_t dep_id, uint32_t dep_count) {
                    for (int i = 0; i < n; i++) {
                        const int64_t blk = b + i;
                        vm.push_back(encode(OP_LOAD, F_SEND | F_DYNAMIC | F_NT, t.flow_m(i), i, 2, m_slots, rows_valid(blk), 0, c.w_off + blk * R * c.K * 4, d_m, 0));
                        vm.push_back(encode(OP_LOAD, F_SEND | F_DYNAMIC | xf, t.flow_x(i), i, 2, x_slots, (uint32_t)B, dep_id, c.x_off, d_x, dep_count));
                    }
                };
                if (first && l > 0) {
                    // the core's first pass over this layer's vector tiles: the first tile of every group waits for the row
                    // blocks of the layer before that produce the group; the rest of the group follows it on the same load
                    // unit.  One accumulator (2) runs along K.
                    for (uint32_t kt0 = 0; kt0 < nk; kt0 += (uint32_t)c.G) {
                        const uint32_t kt1 = std::min<uint32_t>(nk, kt0 + (uint32_t)c.G);
                        const int64_t in_group = std::min<int64_t>((int64_t)Kt * c.G, c.rows_prev - (int64_t)kt0 * Kt);
                        const uint32_t producers = (uint32_t)((in_group + c.R_prev - 1) / c.R_prev);
                        const bool first_is_tail = ktail && kt0 == nk - 1;
                        vm.push_back(encode(OP_SET, 0, 0, 0, 2, 0, 0, 0, (int64_t)kt0 * Kt * 4, 0, 0));
                        pairs(first_is_tail ? dmt : dm, first_is_tail ? dxt : dx, F_DEVICE | F_DEP_RECV, (uint32_t)(c.dep_in + (int32_t)(kt0 / (uint32_t)c.G)), producers);
                        vm.push_back(encode(OP_ADD, 0, 0, 0, 2, 0, 0, 0, (int64_t)Kt * 4, 0, 0));
                        const int64_t full = std::min<int64_t>(kt1, nk_full) - (int64_t)(kt0 + 1);
                        if (full > 0) {
                            if (full > 1) vm.push_back(encode(OP_LOOP, 0, 0, 0, 0, 0, 0, 0, full, 0, 0));
                            pairs(dm, dx, F_DEVICE, 0, 0);
                            vm.push_back(encode(full > 1 ? OP_REPEAT : OP_ADD, 0, 0, 0, 2, 0, 0, 0, (int64_t)Kt * 4, 0, 0));
                        }
                        if (ktail && kt1 == nk && !first_is_tail) pairs(dmt, dxt, F_DEVICE, 0, 0);
                    }
                } else {
                    // one accumulator (2) runs along K for the matrix and the vector tiles of the row blocks of this step
                    vm.push_back(encode(OP_SET, 0, 0, 0, 2, 0, 0, 0, 0, 0, 0));
                    if (nk_full > 0) {
                        if (nk_full > 1) vm.push_back(encode(OP_LOOP, 0, 0, 0, 0, 0, 0, 0, nk_full, 0, 0));
                        pairs(dm, dx, x_flags, 0, 0);
                        vm.push_back(encode(nk_full > 1 ? OP_REPEAT : OP_ADD, 0, 0, 0, 2, 0, 0, 0, (int64_t)Kt * 4, 0, 0));
                    }
                    if (ktail) pairs(dmt, dxt, x_flags, 0, 0);
                }
                first = false;
                for (int i = 0; i < n; i++) {
                    const int64_t blk = b + i;
                    const uint32_t dy = t.desc(2, (uint32_t)B, rows_valid(blk) * 4, R * 4, (uint64_t)c.rows * 4);
                    const bool sig = c.dep_out >= 0;
                    vm.push_back(encode(OP_STORE, F_SEND | F_RECV | (sig ? (uint32_t)(F_DEP_SEND | F_DEVICE) : 0u), t.flow_y(i), i, 0, y_slots, (uint32_t)B,
                                        sig ? (uint32_t)(c.dep_out + (int32_t)(blk * R / ((int64_t)c.Kt_next * c.G_next))) : 0u, c.y_off + blk * R * 4, dy, 0));
                    t.vcc(core, i).push_back(encode(OP_MATVEC, 0, 0, 0, 0, 0, nk, 0, matvec_imm((uint32_t)B, R, Kt / 4), 0, 0));
                }
            }
        }
    }
    words.clear();
    sb.assign(1, 0);
    for (auto &st : t.streams) {
        words.insert(words.end(), st.begin(), st.end());
        words.push_back(encode(OP_HALT, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0));
        sb.push_back((uint32_t)words.size());
    }
    descs = t.descs;
    if (descs.empty()) descs.push_back(Desc{0, 1, 16, 16, 0, 0, 0, 0});
    if (descs.size() > 256) return VDC_EINVAL;
    return VDC_OK;
}

// Memory uops with no arithmetic behind them (Section 6.3, "Memory virtual core overhead"): the byte range
// [0, bytes) in blocks of tile_bytes.  mode 0: every block is loaded (tensor 0) and dropped; mode 1: every block of
// tensor 0 is written with copies of `value`; mode 2: every block is loaded from tensor 0, moved to an output region and
// stored to the same place in tensor 1.  Compute core (c, v) takes a contiguous run of blocks; the memory core's
// stream walks the runs of its compute cores side by side, two blocks of each per loop trip, with one accumulator
// as the running offset (Section 5, "Dynamic address generation").  What is left of the range after the last whole block
// goes to the last compute core: whole rows of it as one short block, the rest as a block of one short row.
int build_stream(const vdc_config &cfg, int32_t mode, int64_t bytes, uint32_t value, int32_t tile_bytes, std::vector<Word> &words,
                 std::vector<uint32_t> &sb, std::vector<Desc> &descs) {
    if (mode < 0 || mode > 2 || bytes < 16 || (bytes & 15) || !is_pow2(tile_bytes) || tile_bytes < 256 ||
        (uint32_t)tile_bytes > kMaxStreamChunks * 16u) return VDC_EINVAL;
    const int C = cfg.n_cores, V = cfg.vcc_per_core;
    Tiler t{cfg, 0, 0, 0, 1, 1, 4};
    t.streams.resize((size_t)C * (1 + V));
    const uint32_t row_bytes = (uint32_t)std::min(tile_bytes, 1024), box_rows = (uint32_t)tile_bytes / row_bytes;
    const uint32_t nslots = t.slots_for((uint64_t)tile_bytes);
    if ((int64_t)nslots * (mode == 2 ? 2 : 1) > cfg.n_slots) return VDC_EINVAL;
    const uint32_t d_in = mode != 1 ? t.desc(0, box_rows, row_bytes, row_bytes, row_bytes) : 0;
    const uint32_t d_out = mode != 0 ? t.desc(mode == 1 ? 0 : 1, box_rows, row_bytes, row_bytes, row_bytes) : 0;
    auto emit_block = [&](std::vector<Word> &vm, int v, int j, bool dyn, int64_t off, uint32_t din, uint32_t dout, uint32_t ns, uint32_t rows) {
        const uint32_t fd = dyn ? F_DYNAMIC : 0;
        if (mode != 1) vm.push_back(encode(OP_LOAD, F_SEND | F_NT | fd, (j & 1) ? t.flow_x(v) : t.flow_m(v), v, 0, ns, rows, 0, off, din, 0));
        if (mode != 0) vm.push_back(encode(OP_STORE, F_SEND | F_RECV | fd, t.flow_y(v), v, 0, ns, rows, 0, off, dout, 0));
    };
    auto emit_uop = [&](std::vector<Word> &vc, int64_t n, uint32_t chunks) {
        for (; n > 0; n -= 65535) {
            const uint32_t k = (uint32_t)std::min<int64_t>(n, 65535);
            vc.push_back(mode == 0 ? encode(OP_DROP, 0, 0, 0, 0, 0, k, 0, 0, 0, 0)
                         : mode == 1 ? encode(OP_FILL, 0, 0, 0, 0, 0, k, 0, fill_imm(value, chunks), 0, 0)
                                     : encode(OP_COPY, 0, 0, 0, 0, 0, k, 0, copy_imm(chunks), 0, 0));
        }
    };
    const int64_t NBk = bytes / tile_bytes, U = (int64_t)C * V;
    for (int c = 0; c < C; c++) {
        std::vector<Word> &vm = t.vmc(c);
        int64_t n[2] = {0, 0}, s0[2] = {0, 0};
        for (int v = 0; v < V; v++) {
            const int64_t u = (int64_t)c * V + v;
            n[v] = NBk / U + (u < NBk % U ? 1 : 0);
            s0[v] = u * (NBk / U) + std::min(u, NBk % U);
        }
        const int64_t common = V == 2 ? std::min(n[0], n[1]) : n[0];
        // blocks per compute core and trip: eight memory uops per trip, as many as the front end dispatches at once
        const int64_t J = (mode == 2 ? 4 : 8) / V;
        const int64_t trips = common / J;
        if (trips > 0xFFFFFFFFll) return VDC_EINVAL;
        if (trips > 0) {
            vm.push_back(encode(OP_SET, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0));
            vm.push_back(encode(OP_LOOP, 0, 0, 0, 0, 0, 0, 0, trips, 0, 0));
            for (int j = 0; j < (int)J; j++)
                for (int v = 0; v < V; v++) emit_block(vm, v, j, true, (s0[v] + j) * tile_bytes, d_in, d_out, nslots, box_rows);
            vm.push_back(encode(OP_REPEAT, 0, 0, 0, 0, 0, 0, 0, J * tile_bytes, 0, 0));
        }
        for (int64_t i = J * trips; i < std::max(n[0], n[1]); i++)
            for (int v = 0; v < V; v++)
                if (i < n[v]) emit_block(vm, v, (int)(i & 1), false, (s0[v] + i) * tile_bytes, d_in, d_out, nslots, box_rows);
        for (int v = 0; v < V; v++) emit_uop(t.vcc(c, v), n[v], (uint32_t)tile_bytes / 16u);
    }
    // the rest of the range
    int64_t off = NBk * tile_bytes;
    const int64_t rest_rows = (bytes - off) / row_bytes;
    std::vector<Word> &vm = t.vmc(C - 1);
    if (rest_rows > 0) {
        emit_block(vm, V - 1, 0, false, off, d_in, d_out, nslots, (uint32_t)rest_rows);
        emit_uop(t.vcc(C - 1, V - 1), 1, (uint32_t)(rest_rows * row_bytes / 16));
        off += rest_rows * row_bytes;
    }
    if (off < bytes) {
        const uint32_t rb = (uint32_t)(bytes - off);
        const uint32_t di = mode != 1 ? t.desc(0, 1, rb, rb, rb) : 0, dout = mode != 0 ? t.desc(mode == 1 ? 0 : 1, 1, rb, rb, rb) : 0;
        emit_block(vm, V - 1, 1, false, off, di, dout, t.slots_for(rb), 1);
        emit_uop(t.vcc(C - 1, V - 1), 1, rb / 16u);
    }
    words.clear();
    sb.assign(1, 0);
    for (auto &st : t.streams) {
        words.insert(words.end(), st.begin(), st.end());
        words.push_back(encode(OP_HALT, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0));
        sb.push_back((uint32_t)words.size());
    }
    descs = t.descs;
    return VDC_OK;
}

// Decode attention, one query per request, over ragged contexts (Section 6.2, "Dynamic Attention Length"), as a uop
// graph.  Tensors: 0 = K, 1 = V ([rows][d], the contexts back to back), 2 = Q ([n_seg][d]), 3 = O ([n_seg][d]),
// 4 = W, the partial rows ([n_items][d + 4]).  A context is cut into tiles of R rows.  The tiles of all contexts, in
// order, are dealt to the compute cores in equal contiguous shares, and an item is a run of tiles of one context on one
// compute core: LOAD the query row, `n` x {LOAD key tile, LOAD value tile}, one STORE.  A context that lies inside one
// share is one item whose ATTN uop is handed a region of d values and writes the request's result itself.  A context
// that crosses shares is cut where they meet.  Its first item stands last in its compute core's list and the others
// first in theirs (or alone): the others store partial rows and signal the request's depId; the first loads those
// partial rows behind its last pair (a load.dep that waits for all of them: by then they have long been written), its
// ATTN uop joins them to its own running state and writes the result.  No partial row of the item that finishes the
// request goes through memory, and nothing is left to do after a core's last tile but one STORE.  A context longer than
// kAttnMaxPartials + 1 shares is cut into that many equal items instead.  In every memory stream all items that signal
// stand before the first load that waits: a waiting load never stands in front of a producer (Section 4.3, "Avoiding
// Deadlock").  The memory core's stream takes the steps of its compute cores in turn.
int build_attn(const vdc_config &cfg, const int64_t *row_off, int32_t n_seg, int32_t d, float scale, int32_t tile_bytes,
               std::vector<Word> &words, std::vector<uint32_t> &sb, std::vector<Desc> &descs, int64_t &n_items) {
    if (!row_off || n_seg < 1 || n_seg > cfg.n_dep_ids || (d != 128 && d != 64) || row_off[0] != 0) return VDC_EINVAL;
    if (tile_bytes != 4096 && tile_bytes != 8192 && tile_bytes != 16384) return VDC_EINVAL;
    const uint32_t lpr = (uint32_t)d / 4, R = (uint32_t)tile_bytes / ((uint32_t)d * 4), row = (uint32_t)d * 4, prow = row + 16;
    if (!attn_geometry_ok(lpr, R)) return VDC_EINVAL;
    const int C = cfg.n_cores, V = cfg.vcc_per_core;
    const int64_t units = (int64_t)C * V;
    constexpr int64_t kMaxPieces = (int64_t)kAttnMaxPartials + 1;
    int64_t NT = 0;
    for (int s = 0; s < n_seg; s++) {
        const int64_t L = row_off[s + 1] - row_off[s];
        if (L < 1) return VDC_EINVAL;
        const int64_t T = (L + R - 1) / R;
        if ((T + kMaxPieces - 1) / kMaxPieces > 65535) return VDC_EINVAL;
        NT += T;
    }
    Tiler t{cfg, 0, 0, 0, 1, 1, 4};
    t.streams.resize((size_t)C * (1 + V));
    uint32_t scale_bits;
    memcpy(&scale_bits, &scale, 4);
    const uint32_t kv_slots = t.slots_for((uint64_t)tile_bytes), q_slots = t.slots_for(row), w_slots = t.slots_for(prow);
    const uint32_t d_k = t.desc(0, R, row, row, row), d_v = t.desc(1, R, row, row, row), d_q = t.desc(2, 1, row, row, row);
    const uint32_t d_o = t.desc(3, 1, row, row, row), d_w = t.desc(4, 1, prow, prow, prow);
    // per compute core: groups of memory uops that are dispatched together; signals: the group belongs to an item that
    // signals a depId; waits: the group holds a load that waits for one
    struct Group { std::vector<Word> uops; bool signals, waits; };
    std::vector<std::vector<Group>> steps((size_t)units);
    // share u holds the tiles [u * NT / units, (u + 1) * NT / units) of the sequence of all tiles
    auto share_of = [&](int64_t g) { return std::min(units - 1, ((g + 1) * units - 1) / NT); };
    auto share_end = [&](int64_t u) { return (u + 1) * NT / units; };
    int64_t item = 0, tiles_before = 0;
    for (int s = 0; s < n_seg; s++) {
        const int64_t L = row_off[s + 1] - row_off[s], T = (L + R - 1) / R;
        // the cuts of the context: where shares meet, or equal items when that would be too many partial rows
        std::vector<int64_t> cuts{0};
        for (int64_t t0 = 0; t0 < T;) {
            const int64_t u = share_of(tiles_before + t0);
            const int64_t t1 = std::min(T, std::max(t0 + 1, share_end(u) - tiles_before));
            cuts.push_back(t1);
            t0 = t1;
        }
        if ((int64_t)cuts.size() - 1 > kMaxPieces) {
            const int64_t chunk = (T + kMaxPieces - 1) / kMaxPieces;
            cuts.assign(1, 0);
            for (int64_t t0 = 0; t0 < T; t0 += chunk) cuts.push_back(std::min(T, t0 + chunk));
        }
        const uint32_t others = (uint32_t)cuts.size() - 2;      // items of the context besides the first
        if (others > kAttnMaxPartials) return VDC_EINVAL;
        const int64_t first_partial = item;
        for (size_t ci = 0; ci + 1 < cuts.size(); ci++) {
            const int64_t t0 = cuts[ci], t1 = cuts[ci + 1];
            const int64_t u = share_of(tiles_before + t0);
            const int v = (int)(u % V);
            const bool finishes = ci == 0, signals = !finishes;
            auto &st = steps[(size_t)u];
            st.push_back({{encode(OP_LOAD, F_SEND, t.flow_x(v), v, 0, q_slots, 1, 0, (int64_t)s * row, d_q, 0)}, signals, false});
            for (int64_t ti = t0; ti < t1; ti++) {
                const int64_t r0 = row_off[s] + ti * R;
                const uint32_t rv = (uint32_t)std::min<int64_t>(R, row_off[s + 1] - r0);
                st.push_back({{encode(OP_LOAD, F_SEND | F_NT, t.flow_m(v), v, 0, kv_slots, rv, 0, r0 * row, d_k, 0),
                               encode(OP_LOAD, F_SEND | F_NT, t.flow_x(v), v, 0, kv_slots, rv, 0, r0 * row, d_v, 0)}, signals, false});
            }
            if (finishes) {
                std::vector<Word> g;
                if (others > 0) {
                    const uint32_t d_t = t.desc(4, others, prow, prow, prow);
                    const uint32_t t_slots = t.slots_for((uint64_t)others * prow);
                    if ((int)(t_slots + q_slots) > cfg.n_slots) return VDC_EINVAL;
                    g.push_back(encode(OP_LOAD, F_SEND | F_DEP_RECV, t.flow_x(v), v, 0, t_slots, others, (uint32_t)s, first_partial * prow, d_t, others));
                }
                g.push_back(encode(OP_STORE, F_SEND | F_RECV, t.flow_y(v), v, 0, q_slots, 1, 0, (int64_t)s * row, d_o, 0));
                st.push_back({g, false, others > 0});
            } else {
                st.push_back({{encode(OP_STORE, F_SEND | F_RECV | F_DEP_SEND, t.flow_y(v), v, 0, w_slots, 1, (uint32_t)s, item * prow, d_w, 0)}, true, false});
                item++;
            }
            t.vcc((int)(u / V), v).push_back(encode(OP_ATTN, 0, 0, 0, 0, 0, (uint32_t)(t1 - t0), 0, attn_imm(lpr, R, scale_bits), finishes ? others : 0u, 0));
        }
        tiles_before += T;
    }
    n_items = std::max<int64_t>(item, 1);       // the workspace is never empty
    for (int c = 0; c < C; c++) {
        // the steps of the core's compute cores in turn, each list at its own pace, so that they end together (the
        // lists of a core differ in length when contexts are uneven; strict alternation left one compute core alone
        // at the end).  A group with a waiting load goes out only when every group of the core's signalling items has.
        std::vector<size_t> at((size_t)V, 0);
        auto signals_left = [&]() {
            for (int v = 0; v < V; v++) {
                const auto &l = steps[(size_t)c * V + v];
                for (size_t i = at[(size_t)v]; i < l.size(); i++)
                    if (l[i].signals) return true;
            }
            return false;
        };
        for (;;) {
            int pick = -1;
            double best = 2.0;
            bool held = false;
            for (int v = 0; v < V; v++) {
                const auto &l = steps[(size_t)c * V + v];
                if (at[(size_t)v] >= l.size()) continue;
                if (l[at[(size_t)v]].waits && signals_left()) { held = true; continue; }
                const double prog = (double)at[(size_t)v] / (double)l.size();
                if (prog < best) { best = prog; pick = v; }
            }
            if (pick < 0) {
                if (held) return VDC_EINVAL;      // cannot happen: a list's signalling items stand before its waiting load
                break;
            }
            const auto &g = steps[(size_t)c * V + pick][at[(size_t)pick]++];
            t.vmc(c).insert(t.vmc(c).end(), g.uops.begin(), g.uops.end());
        }
    }
    words.clear();
    sb.assign(1, 0);
    for (auto &st : t.streams) {
        words.insert(words.end(), st.begin(), st.end());
        words.push_back(encode(OP_HALT, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0));
        sb.push_back((uint32_t)words.size());
    }
    descs = t.descs;
    if (descs.size() > 256) return VDC_EINVAL;
    return VDC_OK;
}

int resolve_config(vdc_config &c, int cu_count, size_t lds_limit) {
    if (c.sched_threshold_pct < 0 || c.sched_threshold_pct > 1000 || c.sched_min_gain_pct < 0 || c.sched_min_gain_pct > 100 ||
        c.sched_force_parts < 0 || (c.sched_force_parts > 16 && (c.sched_force_parts < 101 || c.sched_force_parts > 116))) return VDC_EINVAL;
    if (c.sched_threshold_pct == 0) c.sched_threshold_pct = kSchedThresholdPct;
    if (c.sched_min_gain_pct == 0) c.sched_min_gain_pct = kSchedMinGainPct;
    if (c.issue_batch < 0 || c.issue_batch > 8 || (c.issue_flags & ~3)) return VDC_EINVAL;
    if (c.issue_batch == 0) c.issue_batch = 8;
    if (c.n_cores == 0) c.n_cores = cu_count;
    if (c.vcc_per_core == 0) c.vcc_per_core = 2;
    if (c.threads_per_eu == 0) c.threads_per_eu = 128;
    if (c.slot_bytes == 0) c.slot_bytes = 8192;
    if (c.n_ldu == 0) c.n_ldu = 4;
    if (c.n_stu == 0) c.n_stu = 1;
    if (c.n_dep_ids == 0) c.n_dep_ids = 4096;
    if (c.watchdog_spins == 0) c.watchdog_spins = 1 << 22;
    if (c.n_cores < 1 || c.n_cores > cu_count) return VDC_EINVAL;   // all cores must be co-resident
    if (c.vcc_per_core < 1 || c.vcc_per_core > 2 || c.threads_per_eu != 128) return VDC_EINVAL;
    if (!is_pow2(c.slot_bytes) || c.slot_bytes < 1024 || c.slot_bytes > 16384) return VDC_EINVAL;
    if ((c.n_ldu != 1 && c.n_ldu != 2 && c.n_ldu != 4) || (c.n_stu != 1 && c.n_stu != 2)) return VDC_EINVAL;   // at most 11 waves per core
    if (c.n_stu > c.vcc_per_core) return VDC_EINVAL;   // a store unit serves at least one compute core
    if (c.n_dep_ids < 1 || c.n_dep_ids > 65536 || c.watchdog_spins < 1 || c.tile_rows < 0) return VDC_EINVAL;
    const size_t ctl = lds_control_bytes();
    if (c.n_slots == 0) {
        size_t fit = (lds_limit - ctl) / (size_t)c.slot_bytes;
        c.n_slots = (int32_t)std::min<size_t>(fit, 32);
    }
    if (c.n_slots < 1 || c.n_slots > 32) return VDC_EINVAL;
    if (lds_bytes_needed(c.n_slots, c.slot_bytes) > lds_limit) return VDC_EINVAL;
    return VDC_OK;
}

// The kernel parameters of one run of `prog` on `tensor_bases`, and the waves per core it wants.
int prepare_params(vdc_executor *ex, const vdc_program *prog, void *const *tensor_bases, int32_t n_tensors, uint32_t *trace,
                   uint32_t *trace_count, int32_t trace_cap, uint32_t *dep_table, uint32_t *finished, KParams &p, uint32_t &n_waves) {
    if (!ex || !prog || prog->ex != ex || !tensor_bases || n_tensors != prog->n_tensors) return VDC_EINVAL;
    if (ex->cfg.device == -1) return VDC_EINVAL;
    p = KParams{};
    p.words = prog->d_words;
    p.stream_begin = prog->d_stream_begin;
    p.descs = prog->d_descs;
    p.n_descs = (uint32_t)prog->n_descs;
    for (int i = 0; i < n_tensors; i++) {
        // tiles are loaded in 16-byte units, results stored in units of 4 bytes or more
        const uintptr_t align = ((prog->loaded_tensors >> i) & 1u) ? 15u : 3u;
        if (!tensor_bases[i] || ((uintptr_t)tensor_bases[i] & align)) return VDC_EINVAL;
        p.tensors[i] = (char *)tensor_bases[i];
    }
    p.dep = dep_table ? dep_table : ex->d_dep;
    p.status = ex->d_status;
    p.seq_table = ex->d_status + ST_WORDS + 4;
    p.trace = trace;
    p.trace_count = trace_count;
    p.trace_cap = (uint32_t)trace_cap;
    p.n_slots = ex->cfg.n_slots;
    p.slot_bytes = ex->cfg.slot_bytes;
    p.n_ldu = ex->cfg.n_ldu;
    p.n_stu = ex->cfg.n_stu;
    p.V = ex->cfg.vcc_per_core;
    p.watchdog = (uint32_t)ex->cfg.watchdog_spins;
    p.issue_batch = (uint32_t)ex->cfg.issue_batch;
    p.no_replay = (uint32_t)(ex->cfg.issue_flags & 1);
    // Wave w of a workgroup runs on SIMD w % 4.  Placement 0 takes the roles in wave order (front end, load units, store
    // unit, compute waves): with the default ten waves every SIMD then holds one compute wave.  Placement 1, for graphs
    // bound by the front end and the store unit, keeps those two away from the compute waves: SIMD 0 = front end + load
    // units 0, 1; SIMD 1 = store unit + load units 2, 3; SIMDs 2 and 3 = one wave of each compute core.
    p.wave_roles = 0xFEDCBA9876543210ull;
    n_waves = 1u + p.n_ldu + p.n_stu + 2u * p.V;
    constexpr int kForcePlacement = -1;      // experiments only
    const int placement = kForcePlacement >= 0 ? kForcePlacement : prog->placement;
    const bool default_units = ex->cfg.n_ldu == 4 && ex->cfg.n_stu == 1 && ex->cfg.vcc_per_core == 2;
    if (placement == 1 && default_units)
        p.wave_roles = 0xFEDCBA0000000000ull | 0x4298317650ull;
    // Placement 2: twelve waves, two of which leave at once (position 15), so that the hardware's round-robin puts the
    // front end on a SIMD with one compute wave and nothing else, the store unit likewise, and two load units (one of
    // matrix tiles, one of vector tiles) with one compute wave on each of the other two SIMDs.
#ifdef VDC_PROFILE
    const bool room_for_twelve = false;      // the observer wave of profiling builds takes the twelfth place
#else
    const bool room_for_twelve = true;
#endif
    if (placement == 2 && default_units && room_for_twelve) {
        p.wave_roles = 0xFFFFF98F74365210ull;    // wave 0..11: CFU, LDU0, LDU1, STU, VCC0.0, LDU2, LDU3, VCC0.1, idle, VCC1.0, VCC1.1, idle
        n_waves = 12u;
    }
    // (With two store units, eleven waves, the like of it was measured and is no gain over the wave order: not taken.)
#if defined(VDC_PROFILE) || defined(VDC_PROFILE_WAITS)
    if (!ex->d_prof && hipMalloc(&ex->d_prof, 8 * (16 * 8 * (size_t)ex->cfg.n_cores + 2 * 65536 + 8)) != hipSuccess) return VDC_ENOMEM;
    p.prof = ex->d_prof;
#endif
    // the depId counters are zero between runs: the core that finishes last clears the ones its program used
    p.finished = finished ? finished : ex->d_status + ST_WORDS + 3;
    p.n_dep_used = prog->uses_dep ? prog->max_dep_id + 1 : 0;
    return VDC_OK;
}

int run_program(vdc_executor *ex, const vdc_program *prog, void *const *tensor_bases, int32_t n_tensors, uint32_t *trace,
                uint32_t *trace_count, int32_t trace_cap, hipStream_t stream, uint32_t *dep_table = nullptr, uint32_t *finished = nullptr) {
    KParams p;
    uint32_t n_waves = 0;
    int rc = prepare_params(ex, prog, tensor_bases, n_tensors, trace, trace_count, trace_cap, dep_table, finished, p, n_waves);
    if (rc != VDC_OK) return rc;
    if (ex->r_up) return VDC_ESTATE;      // the resident grid holds every compute unit: a launch would only wait for it
    HIP_TRY(hipSetDevice(ex->cfg.device));
    if (trace_count) HIP_TRY(launch_clear(trace_count, (uint32_t)(ex->cfg.n_cores * (1 + ex->cfg.vcc_per_core)), stream));
    HIP_TRY(launch_executor(p, (uint32_t)ex->cfg.n_cores, n_waves, prog->ops, stream));
    return VDC_OK;
}

// Stop the resident grid, wait for it to leave and give its resources back.
int resident_down(vdc_executor *ex) {
    if (!ex->r_up) return VDC_OK;
    __atomic_store_n(&ex->r_mailbox[MB_STOP], 1u, __ATOMIC_RELEASE);
    hipError_t e = hipStreamSynchronize(ex->r_stream);      // every wait of the grid is bounded: this returns
    (void)hipStreamDestroy(ex->r_stream);
    (void)hipFree(ex->r_dev);
    (void)hipHostFree((void *)ex->r_mailbox);
    ex->r_stream = nullptr; ex->r_dev = nullptr; ex->r_mailbox = nullptr;
    ex->r_up = false;
    return e == hipSuccess ? VDC_OK : VDC_EDEVICE;
}

}  // namespace

extern "C" {

int vdc_create(vdc_executor **out, const vdc_config *cfg_in) {
    if (!out) return VDC_EINVAL;
    *out = nullptr;
    vdc_config cfg{};
    if (cfg_in) cfg = *cfg_in;
    if (cfg.device == -1) {
        // host-only executor: builds and validates programs, owns no device resources and cannot run
        int rc = resolve_config(cfg, cfg.n_cores > 0 ? cfg.n_cores : 256, 163840);
        if (rc != VDC_OK) return rc;
        vdc_executor *h = new (std::nothrow) vdc_executor();
        if (!h) return VDC_ENOMEM;
        h->cfg = cfg;
        h->cu_count = cfg.n_cores;
        h->lds_limit = 163840;
        *out = h;
        return VDC_OK;
    }
    int ndev = 0;
    HIP_TRY(hipGetDeviceCount(&ndev));
    if (cfg.device < 0 || cfg.device >= ndev) return VDC_EINVAL;
    HIP_TRY(hipSetDevice(cfg.device));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, cfg.device));
    int lds_max = 0;
    HIP_TRY(hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, cfg.device));
    int rc = resolve_config(cfg, prop.multiProcessorCount, (size_t)lds_max);
    if (rc != VDC_OK) return rc;
    std::unique_ptr<vdc_executor> ex(new (std::nothrow) vdc_executor());
    if (!ex) return VDC_ENOMEM;
    ex->cfg = cfg;
    ex->cu_count = prop.multiProcessorCount;
    ex->lds_limit = (size_t)lds_max;
    if (hipMalloc(&ex->d_dep, sizeof(uint32_t) * cfg.n_dep_ids) != hipSuccess) return VDC_ENOMEM;
    // status words, four words for vdc_raw_stream's sink and the finished-cores count, then the table of sequence numbers
    if (hipMalloc(&ex->d_status, sizeof(uint32_t) * (ST_WORDS + 4 + kSeqTableWords)) != hipSuccess) { (void)hipFree(ex->d_dep); return VDC_ENOMEM; }
    if (hipHostMalloc(&ex->h_status, sizeof(uint32_t) * ST_WORDS) != hipSuccess) { (void)hipFree(ex->d_dep); (void)hipFree(ex->d_status); return VDC_ENOMEM; }
    hipError_t e = hipMemset(ex->d_dep, 0, sizeof(uint32_t) * cfg.n_dep_ids);
    if (e == hipSuccess) e = hipMemset(ex->d_status, 0, sizeof(uint32_t) * (ST_WORDS + 4));   // the last four words: the sink of vdc_raw_stream
    if (e == hipSuccess) {
        std::vector<uint32_t> seq(kSeqTableWords);
        for (uint32_t i = 0; i < kSeqTableWords; i++) seq[i] = i;
        e = hipMemcpy(ex->d_status + ST_WORDS + 4, seq.data(), sizeof(uint32_t) * kSeqTableWords, hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = prepare_executor_kernels(lds_bytes_needed(cfg.n_slots, cfg.slot_bytes));
    // set-up for the entry point that may not allocate: the address of this device's static scratch array (the device
    // is current here), a pinned staging buffer and an event
    void *scratch_ptr = nullptr;
    if (e == hipSuccess) e = scratch_address(cfg.device, &scratch_ptr);
    ex->scratch = (unsigned char *)scratch_ptr;
    if (e == hipSuccess) e = hipHostMalloc((void **)&ex->h_stage, kScratchBytes);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ex->stage_done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        (void)hipFree(ex->d_dep);
        (void)hipFree(ex->d_status);
        (void)hipHostFree(ex->h_status);
        if (ex->h_stage) (void)hipHostFree(ex->h_stage);
        if (ex->stage_done) (void)hipEventDestroy(ex->stage_done);
        return VDC_EDEVICE;
    }
    *out = ex.release();
    return VDC_OK;
}

int vdc_destroy(vdc_executor *ex) {
    if (!ex) return VDC_EINVAL;
    if (ex->cfg.device == -1) {
        delete ex;
        return VDC_OK;
    }
    (void)hipSetDevice(ex->cfg.device);
    (void)resident_down(ex);
    (void)hipDeviceSynchronize();
    for (vdc_program *p : ex->programs) {
        (void)hipFree(p->d_words);
        (void)hipFree(p->d_stream_begin);
        (void)hipFree(p->d_descs);
        (void)hipFree(p->d_workspace);
        delete p;
    }
    (void)hipFree(ex->d_dep);
    (void)hipFree(ex->d_status);
    (void)hipHostFree(ex->h_status);
    (void)hipHostFree(ex->h_stage);
    (void)hipEventDestroy(ex->stage_done);
    delete ex;
    return VDC_OK;
}

int vdc_get_config(const vdc_executor *ex, vdc_config *cfg) {
    if (!ex || !cfg) return VDC_EINVAL;
    *cfg = ex->cfg;
    return VDC_OK;
}

int vdc_program_create(vdc_executor *ex, const void *uops, int64_t n_uops, const uint32_t *stream_begin, const void *descs,
                       int32_t n_descs, const int64_t *tensor_bytes, int32_t n_tensors, vdc_program **out) {
    if (out) *out = nullptr;
    if (!ex || !uops || n_uops < 1 || n_uops > 0x7FFFFFFF || !stream_begin || !descs || n_descs < 1 || n_descs > 256 ||
        !tensor_bytes || n_tensors < 0 || n_tensors > kMaxTensors || !out)
        return VDC_EINVAL;
    if (ex->cfg.device == -1) return VDC_EINVAL;
    if (ex->r_up) return VDC_ESTATE;      // it allocates device memory, which may wait for the resident grid to leave
    const int n_streams = ex->cfg.n_cores * (1 + ex->cfg.vcc_per_core);
    if (stream_begin[0] != 0 || (int64_t)stream_begin[n_streams] != n_uops) return VDC_EPROGRAM;
    Validator val{ex->cfg, (const Word *)uops, n_uops, stream_begin, (const Desc *)descs, n_descs, tensor_bytes, n_tensors};
    if (!val.run()) return VDC_EPROGRAM;
    std::unique_ptr<vdc_program> p(new (std::nothrow) vdc_program());
    if (!p) return VDC_ENOMEM;
    p->ex = ex;
    p->n_descs = n_descs;
    p->n_tensors = n_tensors;
    for (int i = 0; i < n_tensors; i++) p->tensor_bytes[i] = tensor_bytes[i];
    p->uses_dep = val.uses_dep;
    p->max_dep_id = val.max_dep;
    p->loaded_tensors = val.loaded_tensors;
    p->ops = val.ops | (val.big_regions ? 0u : OPS_ONE_SLOT);
    HIP_TRY(hipSetDevice(ex->cfg.device));
    const size_t wb = (size_t)n_uops * sizeof(Word), sbb = (size_t)(n_streams + 1) * 4, db = (size_t)std::max(n_descs, 1) * sizeof(Desc);   // never an empty table: the front end reads entry 0 for uops without one
    if (hipMalloc(&p->d_words, wb) != hipSuccess) return VDC_ENOMEM;
    if (hipMalloc(&p->d_stream_begin, sbb) != hipSuccess) { (void)hipFree(p->d_words); return VDC_ENOMEM; }
    if (hipMalloc(&p->d_descs, db) != hipSuccess) { (void)hipFree(p->d_words); (void)hipFree(p->d_stream_begin); return VDC_ENOMEM; }
    hipError_t e = hipMemcpy(p->d_words, uops, wb, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(p->d_stream_begin, stream_begin, sbb, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(p->d_descs, 0, db);
    if (e == hipSuccess && n_descs > 0) e = hipMemcpy(p->d_descs, descs, (size_t)n_descs * sizeof(Desc), hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(p->d_words); (void)hipFree(p->d_stream_begin); (void)hipFree(p->d_descs); return VDC_EDEVICE; }
    ex->programs.push_back(p.get());
    *out = p.release();
    return VDC_OK;
}

int vdc_program_validate(vdc_executor *ex, const void *uops, int64_t n_uops, const uint32_t *stream_begin, const void *descs,
                         int32_t n_descs, const int64_t *tensor_bytes, int32_t n_tensors, char *msg, int32_t msg_cap) {
    if (msg && msg_cap > 0) msg[0] = 0;
    if (!ex || !uops || n_uops < 1 || n_uops > 0x7FFFFFFF || !stream_begin || !descs || n_descs < 1 || n_descs > 256 ||
        !tensor_bytes || n_tensors < 0 || n_tensors > kMaxTensors)
        return VDC_EINVAL;
    const int n_streams = ex->cfg.n_cores * (1 + ex->cfg.vcc_per_core);
    Validator val{ex->cfg, (const Word *)uops, n_uops, stream_begin, (const Desc *)descs, n_descs, tensor_bytes, n_tensors};
    bool ok = stream_begin[0] == 0 && (int64_t)stream_begin[n_streams] == n_uops;
    if (!ok) val.err = "stream_begin does not cover the uops";
    ok = ok && val.run();
    if (!ok && msg && msg_cap > 0) {
        strncpy(msg, val.err.c_str(), (size_t)msg_cap - 1);
        msg[msg_cap - 1] = 0;
    }
    return ok ? VDC_OK : VDC_EPROGRAM;
}

int vdc_program_destroy(vdc_program *prog) {
    if (!prog) return VDC_EINVAL;
    vdc_executor *ex = prog->ex;
    if (ex->r_up) return VDC_ESTATE;      // a resident grid may still be reading it, and its memory must not be handed out again
    (void)hipSetDevice(ex->cfg.device);
    (void)hipDeviceSynchronize();
    ex->programs.erase(std::remove(ex->programs.begin(), ex->programs.end(), prog), ex->programs.end());
    for (auto it = ex->cache.begin(); it != ex->cache.end();)
        it = (it->prog == prog) ? ex->cache.erase(it) : it + 1;
    (void)hipFree(prog->d_words);
    (void)hipFree(prog->d_stream_begin);
    (void)hipFree(prog->d_descs);
    (void)hipFree(prog->d_workspace);
    delete prog;
    return VDC_OK;
}

int vdc_run(vdc_executor *ex, const vdc_program *prog, void *const *tensor_bases, int32_t n_tensors, void *hip_stream) {
    return run_program(ex, prog, tensor_bases, n_tensors, nullptr, nullptr, 0, (hipStream_t)hip_stream);
}

int vdc_run_traced(vdc_executor *ex, const vdc_program *prog, void *const *tensor_bases, int32_t n_tensors, uint32_t *trace,
                   uint32_t *trace_count, int32_t trace_cap, void *hip_stream) {
    if (!trace || !trace_count || trace_cap < 1) return VDC_EINVAL;
    return run_program(ex, prog, tensor_bases, n_tensors, trace, trace_count, trace_cap, (hipStream_t)hip_stream);
}

int vdc_resident_start(vdc_executor *ex, int32_t idle_ms) {
    if (!ex || ex->cfg.device == -1 || idle_ms < 0) return VDC_EINVAL;
    if (ex->r_up) return VDC_ESTATE;
    HIP_TRY(hipSetDevice(ex->cfg.device));
    HIP_TRY(hipDeviceSynchronize());
    const size_t mb_words = MB_JOBS + (size_t)kResidentJobs * kResidentJobWords;
    void *mb = nullptr;
    if (hipHostMalloc(&mb, mb_words * 4, hipHostMallocCoherent) != hipSuccess) return VDC_ENOMEM;
    memset(mb, 0, mb_words * 4);
    hipError_t e = hipMalloc(&ex->r_dev, RD_WORDS * 4);
    if (e == hipSuccess) e = hipMemset(ex->r_dev, 0, RD_WORDS * 4);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&ex->r_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e == hipSuccess) {
        ex->r_mailbox = (volatile uint32_t *)mb;
        ex->r_mailbox[MB_STATE] = 1u;
        ResidentParams rp{};
        rp.mailbox = (uint32_t *)mb;
        rp.dev = ex->r_dev;
        rp.status = ex->d_status;
        // the watcher looks about every four microseconds (a nap and two reads of host memory)
        const uint64_t polls = (uint64_t)(idle_ms ? idle_ms : 1000) * 250u;
        rp.idle_polls = (uint32_t)std::min<uint64_t>(polls, 1u << 30);
        rp.backstop_polls = (uint32_t)std::min<uint64_t>((uint64_t)rp.idle_polls * 16u + (1u << 22), 0xFFFFFFF0u);
        e = launch_resident(rp, (uint32_t)ex->cfg.n_cores, 1u + (uint32_t)ex->cfg.n_ldu + (uint32_t)ex->cfg.n_stu + 2u * (uint32_t)ex->cfg.vcc_per_core,
                            lds_bytes_needed(ex->cfg.n_slots, ex->cfg.slot_bytes), ex->r_stream);
    }
    if (e != hipSuccess) {
        if (ex->r_stream) (void)hipStreamDestroy(ex->r_stream);
        (void)hipFree(ex->r_dev);
        (void)hipHostFree(mb);
        ex->r_stream = nullptr; ex->r_dev = nullptr; ex->r_mailbox = nullptr;
        return VDC_EDEVICE;
    }
    ex->r_posted = 0;
    ex->r_up = true;
    return VDC_OK;
}

int vdc_resident_submit(vdc_executor *ex, const vdc_program *prog, void *const *tensor_bases, int32_t n_tensors, uint32_t *ticket) {
    if (!ex || !ticket) return VDC_EINVAL;
    if (!ex->r_up) return VDC_ESTATE;
    KParams p;
    uint32_t n_waves = 0;
    int rc = prepare_params(ex, prog, tensor_bases, n_tensors, nullptr, nullptr, 0, nullptr, nullptr, p, n_waves);
    if (rc != VDC_OK) return rc;
#if defined(VDC_PROFILE) || defined(VDC_PROFILE_WAITS)
    return VDC_EINVAL;
#endif
    // The resident grid has one wave per unit and no more: on two of a compute unit's four SIMDs that leaves registers for
    // a wave of another kernel (the small copy kernels of the runtime among them), which twelve waves per core would
    // not.  A program that asks for the twelve-wave placement runs in wave order instead; results do not depend on it.
    const uint32_t r_waves = 1u + p.n_ldu + p.n_stu + 2u * p.V;
    if (n_waves > r_waves) p.wave_roles = 0xFEDCBA9876543210ull;
    for (uint32_t w = r_waves; w < 16u; w++) p.wave_roles |= 0xFull << (4u * w);
    // room in the mailbox: at most kResidentJobs graphs posted and not complete
    const uint32_t seq = ex->r_posted + 1u;
    for (;;) {
        if (__atomic_load_n(&ex->r_mailbox[MB_STATE], __ATOMIC_ACQUIRE) == 2u) return VDC_ESTATE;      // the grid has left
        if (seq - __atomic_load_n(&ex->r_mailbox[MB_DONE], __ATOMIC_ACQUIRE) <= kResidentJobs) break;
        std::this_thread::yield();
    }
    uint32_t img[kResidentJobWords] = {0};
    static_assert(sizeof(KParams) <= sizeof(img), "a graph's parameter block fits one mailbox entry");
    memcpy(img, &p, sizeof(KParams));
    volatile uint32_t *slot = ex->r_mailbox + MB_JOBS + (seq % kResidentJobs) * kResidentJobWords;
    for (uint32_t i = 0; i < kResidentJobWords; i++) slot[i] = img[i];
    __atomic_store_n(&ex->r_mailbox[MB_TAIL], seq, __ATOMIC_RELEASE);
    ex->r_posted = seq;
    *ticket = seq;
    return VDC_OK;
}

int vdc_resident_wait(vdc_executor *ex, uint32_t ticket, int32_t timeout_ms, uint32_t *info) {
    if (!ex || ticket == 0 || timeout_ms < 0) return VDC_EINVAL;
    if (!ex->r_up || ticket > ex->r_posted) return VDC_ESTATE;
    const auto t0 = std::chrono::steady_clock::now();
    for (;;) {
        if ((int32_t)(__atomic_load_n(&ex->r_mailbox[MB_DONE], __ATOMIC_ACQUIRE) - ticket) >= 0) break;
        if (__atomic_load_n(&ex->r_mailbox[MB_STATE], __ATOMIC_ACQUIRE) == 2u) {
            // the grid has left; a graph it completed on its way out still counts
            if ((int32_t)(__atomic_load_n(&ex->r_mailbox[MB_DONE], __ATOMIC_ACQUIRE) - ticket) >= 0) break;
            return VDC_ESTATE;
        }
        if (std::chrono::duration_cast<std::chrono::milliseconds>(std::chrono::steady_clock::now() - t0).count() > timeout_ms) return VDC_ETIMEOUT;
        std::this_thread::yield();
    }
    const volatile uint32_t *st = ex->r_mailbox + MB_STATUS;
    if (info) { info[0] = st[ST_CORE]; info[1] = st[ST_ROLE]; info[2] = st[ST_PC]; info[3] = st[ST_DETAIL]; }
    if (st[ST_ABORT] == 0) return VDC_OK;
    const int code = -(int)st[ST_CODE];
    return code ? code : VDC_EDEVICE;
}

int vdc_resident_state(vdc_executor *ex, uint32_t *completed) {
    if (!ex) return VDC_EINVAL;
    if (completed) *completed = ex->r_up ? __atomic_load_n(&ex->r_mailbox[MB_DONE], __ATOMIC_ACQUIRE) : 0u;
    if (!ex->r_up) return 0;
    return __atomic_load_n(&ex->r_mailbox[MB_STATE], __ATOMIC_ACQUIRE) == 2u ? 2 : 1;
}

int vdc_resident_stop(vdc_executor *ex) {
    if (!ex || ex->cfg.device == -1) return VDC_EINVAL;
    if (!ex->r_up) return VDC_ESTATE;
    HIP_TRY(hipSetDevice(ex->cfg.device));
    const bool aborted = ex->r_mailbox[MB_STATUS + ST_ABORT] != 0u;
    int rc = resident_down(ex);
    if (rc == VDC_OK && aborted) {
        // a graph that ended in an error may have left depId counters and the count of finished cores anywhere
        HIP_TRY(launch_clear(ex->d_dep, (uint32_t)ex->cfg.n_dep_ids, nullptr));
        HIP_TRY(launch_clear(ex->d_status + ST_WORDS + 3, 1u, nullptr));
        HIP_TRY(launch_clear(ex->d_status, ST_WORDS, nullptr));
        HIP_TRY(hipDeviceSynchronize());
    }
    return rc;
}

int vdc_sync_status(vdc_executor *ex, void *hip_stream, uint32_t *info) {
    if (!ex || ex->cfg.device == -1) return VDC_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(hipSetDevice(ex->cfg.device));
    HIP_TRY(hipMemcpyAsync(ex->h_status, ex->d_status, sizeof(uint32_t) * ST_WORDS, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if (info) {
        info[0] = ex->h_status[ST_CORE];
        info[1] = ex->h_status[ST_ROLE];
        info[2] = ex->h_status[ST_PC];
        info[3] = ex->h_status[ST_DETAIL];
    }
    if (ex->h_status[ST_ABORT] == 0) return VDC_OK;
    int code = -(int)ex->h_status[ST_CODE];
    // an aborted run may have left depId counters and the count of finished cores anywhere: start the next one clean
    HIP_TRY(launch_clear(ex->d_dep, (uint32_t)ex->cfg.n_dep_ids, s));
    HIP_TRY(launch_clear(ex->d_status + ST_WORDS + 3, 1u, s));
    HIP_TRY(launch_clear(ex->d_status, ST_WORDS, s));
    HIP_TRY(hipStreamSynchronize(s));
    return code ? code : VDC_EDEVICE;
}

// Initial content of the workspace (tensor 3) of a matvec program that splits K: the tile [I I .. I | 0] (R rows of Kt
// floats, Kt / R unit matrices side by side), then the partial results, zero.  Empty when the program does not split.
static void workspace_init(const vdc_config &cfg, int64_t rows, int64_t K, int32_t B, int32_t tile_bytes, bool ragged, std::vector<float> &ws) {
    ws.clear();
    int32_t R = 0, Kt = 0;
    if (!choose_tile(cfg, K, B, tile_bytes, R, Kt)) return;
    const SplitPlan sp = plan_split(cfg, rows, K, B, R, Kt, tile_bytes, ragged);
    if (sp.S < 2) return;
    ws.assign((size_t)(sp.bytes / 4), 0.0f);
    for (int g = 0; g < Kt / R; g++)
        for (int r = 0; r < R; r++) ws[(size_t)r * Kt + (size_t)g * R + r] = 1.0f;
}

static int matvec_common(vdc_executor *ex, const float *M, int64_t rows, int64_t K, int64_t ld, const float *X, float *Y,
                         int32_t B, int32_t tile_bytes, const int64_t *row_off, int32_t n_seg, void *hip_stream,
                         const float *T = nullptr, bool rope = false) {
    if (!ex || ex->cfg.device == -1 || !M || !X || !Y || rows < 1 || K < 4 || (K & 3) || ld < K || (ld & 3) || B < 1 || B > 8) return VDC_EINVAL;
    if (((uintptr_t)M & 15u) || ((uintptr_t)X & 15u) || ((uintptr_t)Y & 3u)) return VDC_EINVAL;
    if (rope && (!T || ((uintptr_t)T & 15u) || row_off)) return VDC_EINVAL;
    std::vector<int64_t> key{PK_MATVEC, rows, K, ld, B, tile_bytes, row_off ? n_seg : -1, rope ? 1 : 0};
    if (row_off) key.insert(key.end(), row_off, row_off + n_seg + 1);
    vdc_program *prog = cache_find(ex, key);
    if (!prog) {
        std::vector<Word> words;
        std::vector<uint32_t> sb;
        std::vector<Desc> descs;
        int rc = build_matvec(ex->cfg, rows, K, ld, B, tile_bytes, row_off, n_seg, words, sb, descs, rope);
        if (rc != VDC_OK) return rc;
        const int64_t x_rows = row_off ? n_seg : B;
        std::vector<float> ws;
        if (!rope) workspace_init(ex->cfg, rows, K, B, tile_bytes, row_off != nullptr, ws);
        int64_t tb[4] = {((rows - 1) * ld + K) * 4, x_rows * K * 4, (int64_t)B * rows * 4, rope ? (int64_t)B * rows * 4 : (int64_t)ws.size() * 4};
        rc = vdc_program_create(ex, words.data(), (int64_t)words.size(), sb.data(), descs.data(), (int32_t)descs.size(), tb,
                                (ws.empty() && !rope) ? 3 : 4, &prog);
        if (rc != VDC_OK) return rc;
        if (!ws.empty()) {
            if (hipMalloc(&prog->d_workspace, ws.size() * 4) != hipSuccess) { vdc_program_destroy(prog); return VDC_ENOMEM; }
            if (hipMemcpy(prog->d_workspace, ws.data(), ws.size() * 4, hipMemcpyHostToDevice) != hipSuccess) { vdc_program_destroy(prog); return VDC_EDEVICE; }
        }
        prog->placement = matvec_placement(ex->cfg, rows, K, B, tile_bytes, rope);
        cache_insert(ex, std::move(key), prog);
    }
    void *bases[4] = {(void *)M, (void *)X, (void *)Y, rope ? (void *)T : prog->d_workspace};
    return vdc_run(ex, prog, bases, (rope || prog->d_workspace) ? 4 : 3, hip_stream);
}

int vdc_matvec(vdc_executor *ex, const float *M, int64_t rows, int64_t K, int64_t ld, const float *X, float *Y, int32_t B,
               int32_t tile_bytes, void *hip_stream) {
    return matvec_common(ex, M, rows, K, ld, X, Y, B, tile_bytes, nullptr, 0, hip_stream);
}

// vdc_matvec for callers that cannot allocate.  Nothing here calls hipMalloc, hipFree or an allocating library routine:
// the program image goes from the executor's pinned staging buffer into the device's static scratch array with an
// asynchronous copy on the caller's stream, and the kernels read it there.  A program that is already in the array
// (same executor configuration, same shape) is not built or copied again.
int vdc_matvec_noalloc(vdc_executor *ex, const float *M, int64_t rows, int64_t K, int64_t ld, const float *X, float *Y, int32_t B,
                       int32_t tile_bytes, void *hip_stream) {
    if (!ex || ex->cfg.device == -1 || !M || !X || !Y || rows < 1 || K < 4 || (K & 3) || ld < K || (ld & 3) || B < 1 || B > 8) return VDC_EINVAL;
    if (((uintptr_t)M & 15u) || ((uintptr_t)X & 15u) || ((uintptr_t)Y & 3u)) return VDC_EINVAL;
    const int dev = ex->cfg.device;
    if (dev < 0 || dev >= 64 || !ex->scratch || !ex->h_stage) return VDC_EINVAL;
    hipStream_t stream = (hipStream_t)hip_stream;
    HIP_TRY(hipSetDevice(dev));
    const vdc_config &c = ex->cfg;
    std::vector<int64_t> key{PK_MATVEC, rows, K, ld, B, tile_bytes, c.n_cores, c.vcc_per_core, c.slot_bytes, c.n_slots, c.n_ldu, c.n_stu,
                             c.n_dep_ids, c.tile_rows, c.issue_batch, c.issue_flags};
    ScratchImage &img = g_scratch_image[dev];
    auto up = [](size_t x) { return (x + 255u) & ~(size_t)255u; };
    if (img.key != key) {
        std::vector<Word> words;
        std::vector<uint32_t> sb;
        std::vector<Desc> descs;
        int rc = build_matvec(c, rows, K, ld, B, tile_bytes, nullptr, 0, words, sb, descs, false);
        if (rc != VDC_OK) return rc;
        std::vector<float> ws;
        workspace_init(c, rows, K, B, tile_bytes, false, ws);
        ScratchImage n;
        n.n_descs = (int32_t)descs.size();
        n.n_tensors = ws.empty() ? 3 : 4;
        n.tensor_bytes[0] = ((rows - 1) * ld + K) * 4;
        n.tensor_bytes[1] = (int64_t)B * K * 4;
        n.tensor_bytes[2] = (int64_t)B * rows * 4;
        n.tensor_bytes[3] = (int64_t)ws.size() * 4;
        n.off_sb = kScratchDepBytes;
        n.off_descs = n.off_sb + up(sb.size() * 4);
        n.off_words = n.off_descs + up(descs.size() * sizeof(Desc));
        n.off_ws = n.off_words + up(words.size() * sizeof(Word));
        n.has_ws = !ws.empty();
        const size_t end = n.off_ws + up(ws.size() * 4);
        if (end > kScratchBytes) return VDC_ETOOBIG;
        Validator val{c, words.data(), (int64_t)words.size(), sb.data(), descs.data(), n.n_descs, n.tensor_bytes, n.n_tensors};
        if (!val.run()) return VDC_EPROGRAM;
        n.uses_dep = val.uses_dep;
        n.max_dep_id = val.max_dep;
        n.loaded_tensors = val.loaded_tensors;
        n.ops = val.ops | (val.big_regions ? 0u : OPS_ONE_SLOT);
        if (n.uses_dep && ((size_t)n.max_dep_id + 2) * 4 > kScratchDepBytes) return VDC_ETOOBIG;
        n.placement = matvec_placement(c, rows, K, B, tile_bytes, false);   // the same choice of role placement as vdc_matvec makes
        // the staging buffer may still be the source of the copy of an earlier call
        if (ex->stage_pending) HIP_TRY(hipEventSynchronize(ex->stage_done));
        ex->stage_pending = false;
        unsigned char *h = ex->h_stage;
        memcpy(h + n.off_sb, sb.data(), sb.size() * 4);
        memcpy(h + n.off_descs, descs.data(), descs.size() * sizeof(Desc));
        memcpy(h + n.off_words, words.data(), words.size() * sizeof(Word));
        if (n.has_ws) memcpy(h + n.off_ws, ws.data(), ws.size() * 4);
        img.key.clear();      // whatever the array held is being replaced from here on
        HIP_TRY(hipMemcpyAsync(ex->scratch + kScratchDepBytes, h + kScratchDepBytes, end - kScratchDepBytes, hipMemcpyHostToDevice, stream));
        HIP_TRY(hipEventRecord(ex->stage_done, stream));
        ex->stage_pending = true;
        n.key = key;
        img = n;
    }
    // The array keeps what the last call left: the depId counters a run starts from, and the count of finished cores,
    // are put to zero by a small fill kernel (an aborted run, or a run of another executor, may have left them anywhere).
    uint32_t *dep = (uint32_t *)ex->scratch;
    uint32_t *finished = dep + kScratchDepBytes / 4 - 1;
    if (img.uses_dep) {
        HIP_TRY(launch_clear(dep, img.max_dep_id + 1u, stream));
        HIP_TRY(launch_clear(finished, 1u, stream));
    }
    vdc_program prog;
    prog.ex = ex;
    prog.d_words = (Word *)(ex->scratch + img.off_words);
    prog.d_stream_begin = (uint32_t *)(ex->scratch + img.off_sb);
    prog.d_descs = (Desc *)(ex->scratch + img.off_descs);
    prog.n_descs = img.n_descs;
    prog.n_tensors = img.n_tensors;
    for (int i = 0; i < kMaxTensors; i++) prog.tensor_bytes[i] = img.tensor_bytes[i];
    prog.uses_dep = img.uses_dep;
    prog.max_dep_id = img.max_dep_id;
    prog.loaded_tensors = img.loaded_tensors;
    prog.ops = img.ops;
    prog.placement = img.placement;
    void *bases[4] = {(void *)M, (void *)X, (void *)Y, img.has_ws ? (void *)(ex->scratch + img.off_ws) : nullptr};
    return run_program(ex, &prog, bases, img.n_tensors, nullptr, nullptr, 0, stream, dep, finished);
}

int vdc_matvec_rope(vdc_executor *ex, const float *M, int64_t rows, int64_t K, int64_t ld, const float *X, const float *T, float *Y,
                    int32_t B, int32_t tile_bytes, void *hip_stream) {
    return matvec_common(ex, M, rows, K, ld, X, Y, B, tile_bytes, nullptr, 0, hip_stream, T, true);
}

int vdc_matvec_ragged(vdc_executor *ex, const float *M, const int64_t *row_off, int32_t n_seg, int64_t K, const float *X,
                      float *Y, int32_t tile_bytes, void *hip_stream) {
    if (!row_off || n_seg < 1 || row_off[0] != 0) return VDC_EINVAL;
    for (int s = 0; s < n_seg; s++)
        if (row_off[s + 1] < row_off[s]) return VDC_EINVAL;
    return matvec_common(ex, M, row_off[n_seg], K, K, X, Y, 1, tile_bytes, row_off, n_seg, hip_stream);
}

static int matvec_program_common(vdc_executor *ex, int64_t rows, int64_t K, int64_t ld, int32_t B, int32_t tile_bytes,
                                 const int64_t *row_off, int32_t n_seg, void *uops, int64_t *n_uops, uint32_t *stream_begin, void *descs,
                                 int32_t *n_descs, bool rope);

int vdc_matvec_program(vdc_executor *ex, int64_t rows, int64_t K, int64_t ld, int32_t B, int32_t tile_bytes,
                       const int64_t *row_off, int32_t n_seg, void *uops, int64_t *n_uops, uint32_t *stream_begin, void *descs,
                       int32_t *n_descs) {
    return matvec_program_common(ex, rows, K, ld, B, tile_bytes, row_off, n_seg, uops, n_uops, stream_begin, descs, n_descs, false);
}

int vdc_matvec_rope_program(vdc_executor *ex, int64_t rows, int64_t K, int64_t ld, int32_t B, int32_t tile_bytes, void *uops,
                            int64_t *n_uops, uint32_t *stream_begin, void *descs, int32_t *n_descs) {
    return matvec_program_common(ex, rows, K, ld, B, tile_bytes, nullptr, 0, uops, n_uops, stream_begin, descs, n_descs, true);
}

static int matvec_program_common(vdc_executor *ex, int64_t rows, int64_t K, int64_t ld, int32_t B, int32_t tile_bytes,
                                 const int64_t *row_off, int32_t n_seg, void *uops, int64_t *n_uops, uint32_t *stream_begin, void *descs,
                                 int32_t *n_descs, bool rope) {
    if (!ex || !n_uops || !n_descs || rows < 1 || K < 4 || (K & 3) || ld < K || (ld & 3) || B < 1 || B > 8) return VDC_EINVAL;
    if (row_off) {
        if (n_seg < 1 || row_off[0] != 0 || row_off[n_seg] != rows || B != 1 || ld != K) return VDC_EINVAL;
        for (int s = 0; s < n_seg; s++)
            if (row_off[s + 1] < row_off[s]) return VDC_EINVAL;
    }
    std::vector<Word> words;
    std::vector<uint32_t> sb;
    std::vector<Desc> ds;
    int rc = build_matvec(ex->cfg, rows, K, ld, B, tile_bytes, row_off, n_seg, words, sb, ds, rope);
    if (rc != VDC_OK) return rc;
    const int64_t cap_w = *n_uops;
    const int32_t cap_d = *n_descs;
    *n_uops = (int64_t)words.size();
    *n_descs = (int32_t)ds.size();
    bool fits = true;
    if (uops) { if (cap_w >= (int64_t)words.size()) memcpy(uops, words.data(), words.size() * sizeof(Word)); else fits = false; }
    if (descs) { if (cap_d >= (int32_t)ds.size()) memcpy(descs, ds.data(), ds.size() * sizeof(Desc)); else fits = false; }
    if (stream_begin) memcpy(stream_begin, sb.data(), sb.size() * sizeof(uint32_t));
    return fits ? VDC_OK : VDC_EINVAL;
}

int vdc_matvec_workspace(vdc_executor *ex, int64_t rows, int64_t K, int64_t ld, int32_t B, int32_t tile_bytes, void *init,
                         int64_t *bytes) {
    if (!ex || !bytes || rows < 1 || K < 4 || (K & 3) || ld < K || (ld & 3) || B < 1 || B > 8) return VDC_EINVAL;
    std::vector<float> ws;
    workspace_init(ex->cfg, rows, K, B, tile_bytes, false, ws);
    const int64_t cap = *bytes;
    *bytes = (int64_t)ws.size() * 4;
    if (init && !ws.empty()) {
        if (cap < *bytes) return VDC_EINVAL;
        memcpy(init, ws.data(), ws.size() * 4);
    }
    return VDC_OK;
}

int vdc_matvec_tiling(vdc_executor *ex, int64_t rows, int64_t K, int32_t B, int32_t tile_bytes, int64_t *out) {
    if (!ex || !out || rows < 1 || K < 4 || (K & 3) || B < 1 || B > 8) return VDC_EINVAL;
    int32_t R = 0, Kt = 0;
    if (!choose_tile(ex->cfg, K, B, tile_bytes, R, Kt)) return VDC_EINVAL;
    const SplitPlan sp = plan_split(ex->cfg, rows, K, B, R, Kt, tile_bytes, false);
    out[0] = R; out[1] = Kt; out[2] = sp.NB; out[3] = (K + Kt - 1) / Kt; out[4] = sp.S_max; out[5] = sp.S;
    out[6] = sp.S > 1 && sp.T < sp.NB ? sp.T : 0;
    return VDC_OK;
}

int vdc_matvec_chain(vdc_executor *ex, const float *W, float *A, const int64_t *dims, int32_t L, int32_t B, int32_t tile_bytes,
                     void *hip_stream) {
    if (!ex || ex->cfg.device == -1 || !W || !A || !dims || L < 1 || ((uintptr_t)W & 15u) || ((uintptr_t)A & 15u)) return VDC_EINVAL;
    std::vector<int64_t> key{PK_CHAIN, B, tile_bytes, L};
    key.insert(key.end(), dims, dims + L + 1);
    vdc_program *prog = cache_find(ex, key);
    if (!prog) {
        std::vector<Word> words;
        std::vector<uint32_t> sb;
        std::vector<Desc> descs;
        int64_t w_bytes = 0, a_bytes = 0;
        int rc = build_chain(ex->cfg, dims, L, B, tile_bytes, words, sb, descs, w_bytes, a_bytes);
        if (rc != VDC_OK) return rc;
        int64_t tb[3] = {w_bytes, a_bytes, a_bytes};
        rc = vdc_program_create(ex, words.data(), (int64_t)words.size(), sb.data(), descs.data(), (int32_t)descs.size(), tb, 3, &prog);
        if (rc != VDC_OK) return rc;
        cache_insert(ex, std::move(key), prog);
    }
    void *bases[3] = {(void *)W, (void *)A, (void *)A};
    return vdc_run(ex, prog, bases, 3, hip_stream);
}

int vdc_matvec_chain_program(vdc_executor *ex, const int64_t *dims, int32_t L, int32_t B, int32_t tile_bytes, void *uops, int64_t *n_uops,
                             uint32_t *stream_begin, void *descs, int32_t *n_descs) {
    if (!ex || !n_uops || !n_descs) return VDC_EINVAL;
    std::vector<Word> words;
    std::vector<uint32_t> sb;
    std::vector<Desc> ds;
    int64_t w_bytes = 0, a_bytes = 0;
    int rc = build_chain(ex->cfg, dims, L, B, tile_bytes, words, sb, ds, w_bytes, a_bytes);
    if (rc != VDC_OK) return rc;
    const int64_t cap_w = *n_uops;
    const int32_t cap_d = *n_descs;
    *n_uops = (int64_t)words.size();
    *n_descs = (int32_t)ds.size();
    bool fits = true;
    if (uops) { if (cap_w >= (int64_t)words.size()) memcpy(uops, words.data(), words.size() * sizeof(Word)); else fits = false; }
    if (descs) { if (cap_d >= (int32_t)ds.size()) memcpy(descs, ds.data(), ds.size() * sizeof(Desc)); else fits = false; }
    if (stream_begin) memcpy(stream_begin, sb.data(), sb.size() * sizeof(uint32_t));
    return fits ? VDC_OK : VDC_EINVAL;
}

int vdc_attn_decode(vdc_executor *ex, const float *Q, const float *K, const float *V, const int64_t *row_off, int32_t n_seg,
                    int32_t d, float scale, float *O, int32_t tile_bytes, void *hip_stream) {
    if (!ex || ex->cfg.device == -1 || !Q || !K || !V || !O || !row_off || n_seg < 1) return VDC_EINVAL;
    if (((uintptr_t)Q & 15u) || ((uintptr_t)K & 15u) || ((uintptr_t)V & 15u) || ((uintptr_t)O & 15u)) return VDC_EINVAL;
    if (!attn_scale_resolve(scale, d)) return VDC_EINVAL;
    std::vector<int64_t> key{PK_ATTN, d, float_bits(scale), tile_bytes, n_seg};
    key.insert(key.end(), row_off, row_off + n_seg + 1);
    vdc_program *prog = cache_find(ex, key);
    if (!prog) {
        std::vector<Word> words;
        std::vector<uint32_t> sb;
        std::vector<Desc> descs;
        int64_t n_items = 0;
        int rc = build_attn(ex->cfg, row_off, n_seg, d, scale, tile_bytes, words, sb, descs, n_items);
        if (rc != VDC_OK) return rc;
        const int64_t rows = row_off[n_seg], row = (int64_t)d * 4;
        int64_t tb[5] = {rows * row, rows * row, n_seg * row, n_seg * row, n_items * (row + 16)};   // n_items >= 1
        rc = vdc_program_create(ex, words.data(), (int64_t)words.size(), sb.data(), descs.data(), (int32_t)descs.size(), tb, 5, &prog);
        if (rc != VDC_OK) return rc;
        if (hipMalloc(&prog->d_workspace, (size_t)tb[4]) != hipSuccess) { vdc_program_destroy(prog); return VDC_ENOMEM; }
        cache_insert(ex, std::move(key), prog);
    }
    void *bases[5] = {(void *)K, (void *)V, (void *)Q, (void *)O, prog->d_workspace};
    return vdc_run(ex, prog, bases, 5, hip_stream);
}

int vdc_attn_decode_program(vdc_executor *ex, const int64_t *row_off, int32_t n_seg, int32_t d, float scale, int32_t tile_bytes,
                            void *uops, int64_t *n_uops, uint32_t *stream_begin, void *descs, int32_t *n_descs, int64_t *n_items) {
    if (!ex || !n_uops || !n_descs || !n_items) return VDC_EINVAL;
    if (!attn_scale_resolve(scale, d)) return VDC_EINVAL;
    std::vector<Word> words;
    std::vector<uint32_t> sb;
    std::vector<Desc> ds;
    int rc = build_attn(ex->cfg, row_off, n_seg, d, scale, tile_bytes, words, sb, ds, *n_items);
    if (rc != VDC_OK) return rc;
    const int64_t cap_w = *n_uops;
    const int32_t cap_d = *n_descs;
    *n_uops = (int64_t)words.size();
    *n_descs = (int32_t)ds.size();
    bool fits = true;
    if (uops) { if (cap_w >= (int64_t)words.size()) memcpy(uops, words.data(), words.size() * sizeof(Word)); else fits = false; }
    if (descs) { if (cap_d >= (int32_t)ds.size()) memcpy(descs, ds.data(), ds.size() * sizeof(Desc)); else fits = false; }
    if (stream_begin) memcpy(stream_begin, sb.data(), sb.size() * sizeof(uint32_t));
    return fits ? VDC_OK : VDC_EINVAL;
}

int vdc_program_set_placement(vdc_program *prog, int32_t placement) {
    if (!prog || placement < 0 || placement > 2) return VDC_EINVAL;
    prog->placement = placement;
    return VDC_OK;
}

int vdc_stream(vdc_executor *ex, int32_t mode, const void *src, void *dst, int64_t bytes, uint32_t value, int32_t tile_bytes,
               void *hip_stream) {
    if (!ex || ex->cfg.device == -1 || mode < 0 || mode > 2) return VDC_EINVAL;
    if ((mode != 1 && (!src || ((uintptr_t)src & 15u))) || (mode != 0 && (!dst || ((uintptr_t)dst & 15u)))) return VDC_EINVAL;
    if (mode != 1) value = 0;
    std::vector<int64_t> key{PK_STREAM, mode, bytes, (int64_t)value, tile_bytes};
    vdc_program *prog = cache_find(ex, key);
    if (!prog) {
        std::vector<Word> words;
        std::vector<uint32_t> sb;
        std::vector<Desc> descs;
        int rc = build_stream(ex->cfg, mode, bytes, value, tile_bytes, words, sb, descs);
        if (rc != VDC_OK) return rc;
        int64_t tb[2] = {bytes, bytes};
        rc = vdc_program_create(ex, words.data(), (int64_t)words.size(), sb.data(), descs.data(), (int32_t)descs.size(), tb,
                                mode == 2 ? 2 : 1, &prog);
        if (rc != VDC_OK) return rc;
        // a store per block: bound by the store unit and the front end (copies of 32 KB blocks by the load units again)
        prog->placement = (mode == 1 || (mode == 2 && tile_bytes < 32768)) ? 1 : 0;
        cache_insert(ex, std::move(key), prog);
    }
    void *bases[2] = {mode == 1 ? dst : (void *)src, dst};
    return vdc_run(ex, prog, bases, mode == 2 ? 2 : 1, hip_stream);
}

int vdc_raw_stream(vdc_executor *ex, int32_t mode, const void *src, void *dst, int64_t bytes, uint32_t value, void *hip_stream) {
    if (!ex || ex->cfg.device == -1 || mode < 0 || mode > 2 || bytes < 16 || (bytes & 15)) return VDC_EINVAL;
    if ((mode != 1 && (!src || ((uintptr_t)src & 15u))) || (mode != 0 && (!dst || ((uintptr_t)dst & 15u)))) return VDC_EINVAL;
    HIP_TRY(hipSetDevice(ex->cfg.device));
    HIP_TRY(launch_raw_stream(mode, src, dst, (uint64_t)bytes, value, ex->d_status + ST_WORDS, ex->cu_count * 8, (hipStream_t)hip_stream));
    return VDC_OK;
}

int vdc_stream_program(vdc_executor *ex, int32_t mode, int64_t bytes, uint32_t value, int32_t tile_bytes, void *uops, int64_t *n_uops,
                       uint32_t *stream_begin, void *descs, int32_t *n_descs) {
    if (!ex || !n_uops || !n_descs) return VDC_EINVAL;
    std::vector<Word> words;
    std::vector<uint32_t> sb;
    std::vector<Desc> ds;
    int rc = build_stream(ex->cfg, mode, bytes, mode == 1 ? value : 0, tile_bytes, words, sb, ds);
    if (rc != VDC_OK) return rc;
    const int64_t cap_w = *n_uops;
    const int32_t cap_d = *n_descs;
    *n_uops = (int64_t)words.size();
    *n_descs = (int32_t)ds.size();
    bool fits = true;
    if (uops) { if (cap_w >= (int64_t)words.size()) memcpy(uops, words.data(), words.size() * sizeof(Word)); else fits = false; }
    if (descs) { if (cap_d >= (int32_t)ds.size()) memcpy(descs, ds.data(), ds.size() * sizeof(Desc)); else fits = false; }
    if (stream_begin) memcpy(stream_begin, sb.data(), sb.size() * sizeof(uint32_t));
    return fits ? VDC_OK : VDC_EINVAL;
}

int vdc_debug_alloc(vdc_executor *ex, const uint32_t *masks, const int32_t *nslots, int32_t n_slots, int32_t *pos, int32_t n,
                    void *hip_stream) {
    if (!ex || ex->cfg.device == -1 || !masks || !nslots || !pos || n < 1 || n_slots < 1 || n_slots > 32) return VDC_EINVAL;
    HIP_TRY(hipSetDevice(ex->cfg.device));
    HIP_TRY(launch_debug_alloc(masks, nslots, n_slots, pos, n, (hipStream_t)hip_stream));
    return VDC_OK;
}

#if defined(VDC_PROFILE) || defined(VDC_PROFILE_WAITS)
int vdc_prof_events(vdc_executor *ex, unsigned long long *out) {   // 2 * 65536 + 1 words: the observer's log, then its count
    return hipMemcpy(out, ex->d_prof + 16 * 8 * (size_t)ex->cfg.n_cores, 8 * (2 * 65536 + 1), hipMemcpyDeviceToHost) == hipSuccess ? 0 : VDC_EDEVICE;
}
int vdc_prof_read(vdc_executor *ex, unsigned long long *out) {
    return hipMemcpy(out, ex->d_prof, 8 * 16 * 8 * (size_t)ex->cfg.n_cores, hipMemcpyDeviceToHost) == hipSuccess ? 0 : VDC_EDEVICE;
}
#endif

const char *vdc_strerror(int code) {
    switch (code) {
        case VDC_OK: return "ok";
        case VDC_EINVAL: return "invalid argument";
        case VDC_ENOMEM: return "out of memory";
        case VDC_EPROGRAM: return "malformed uop program";
        case VDC_EDEVICE: return "HIP error";
        case VDC_EDEADLOCK: return "device watchdog: a unit waited past the spin limit";
        case VDC_ELEAK: return "run ended with local-memory slots still allocated";
        case VDC_ESTATE: return "the call does not fit the executor's state (resident grid up, not up, or already gone)";
        case VDC_ETIMEOUT: return "the graph was not complete within the time given";
        case VDC_ETOOBIG: return "the uop program and its workspace do not fit the static scratch of the entry point that allocates nothing";
        default: return "unknown error";
    }
}

}  // extern "C"
