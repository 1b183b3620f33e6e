// The on-GPU executor: persistent virtual cores for CDNA4 (gfx950), one workgroup per compute unit.
//
// Section 4.3 of the paper ("GPU Executor") describes, for Hopper, one virtual memory core (VMC) per SM
// built from a control-flow unit (CFU) feeding parallel load units (LDU) and store units (STU), two
// virtual compute cores (VCC) of 128 threads, FIFO dependency queues between them, TMA for the tile
// copies and mbarrier for blocking waits.  CDNA4 has neither TMA nor mbarrier, so the roles map to
// wave64 wavefronts of one workgroup as follows:
//
//   wave 0                      CFU   fetch / decode / control uops / address generation / slot allocation /
//                                     dispatch by virtual flow / receiver of the c2m queues
//   waves 1 .. n_ldu (<= 2)     LDU   direct-to-LDS 128-bit loads (global_load_lds_dwordx4), several tiles in
//                                     flight per unit, completion observed with s_waitcnt vmcnt(N), then the
//                                     region is delivered into its m2c ticket
//   next n_stu waves            STU   waits for the produced region, LDS -> global, frees the slots, signals depId
//   next 2 * V waves            VCC   v = 0..V-1, two waves (128 threads) each: the compute uop handlers
//
// All queues live in LDS.  A waiter polls an LDS word with s_sleep back-off (no hardware de-scheduling
// exists); every poll loop counts its iterations and raises VDC_EDEADLOCK at the watchdog limit, and every
// loop also leaves when another unit or core has raised an error, so the grid always drains.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vdc_isa.h"
#include "vdc_kernel.h"

namespace vdc {

// ------------------------------------------------------------------------------------------------
// LDS layout: [0, n_slots * slot_bytes) the slots, then the control block.
// ------------------------------------------------------------------------------------------------
constexpr int kUQ = 8;         // records per unit queue (CFU -> LDU/STU)
constexpr int kM2C = 32;       // m2c ring entries per VCC (>= slots, so a delivery never finds it full)
constexpr int kC2M = 64;       // c2m ring entries per VCC
constexpr int kMbox = 32;      // produced regions waiting for their STORE, per VCC
constexpr int kMaxUnits = 4;   // n_ldu + n_stu
constexpr int kMaxV = 2;
constexpr int kMaxInflight = 4;  // tiles one LDU keeps in flight
constexpr int kMaxVm = 56;       // outstanding load instructions one LDU allows itself (vmcnt holds 63)

struct UnitRec {  // a memory uop after the front end (48 bytes)
    uint32_t gaddr_lo, gaddr_hi;
    uint32_t gpitch_lo, gpitch_hi;
    uint32_t lds_off;    // byte offset of the region in LDS
    uint32_t rows_box;   // valid rows | box_rows << 16
    uint32_t rb_pitch;   // valid row_bytes | lds_pitch << 16
    uint32_t w0;         // first word of the uop: opcode, flags, vflow, vcc, acc, nslots
    uint32_t ticket;     // m2c position when SEND
    uint32_t slot;
    uint32_t dep;        // depId | dep_count << 16
    uint32_t pc;
};

struct Ctl {
    uint32_t mask;                 // slot availability: bit set = in use (Section 4.3: 32-bit mask in shared memory)
    uint32_t abort;                // set when any unit of this core gives up
    uint32_t cfu_halted;
    uint32_t vcc_done;             // VCC waves that reached HALT
    uint32_t c2m_tail[kMaxV];      // next c2m position, taken with an atomic add by the pushing wave
    uint32_t mbox_tail[kMaxV];
    uint32_t mbox_head[kMaxV];
    uint32_t red_flag[kMaxV];      // cross-wave reduction hand-shake of a VCC
    uint32_t red_ack[kMaxV];
    uint32_t uq_tail[kMaxUnits];
    uint32_t uq_head[kMaxUnits];
    uint32_t pad0[2];
    uint64_t m2c[kMaxV][kM2C];     // low: slot | nslots << 6 | rows << 12; high: (ticket + 1) & 0xffff | row_bytes << 16
    uint64_t c2m[kMaxV][kC2M];     // low: kind | slot << 1 | nslots << 7; high: position + 1
    uint32_t m2c_done[kMaxV][kM2C];  // how many of the two waves of the VCC are done with the entry
    uint32_t mbox[kMaxV][kMbox];
    UnitRec uq[kMaxUnits][kUQ];
    float red[kMaxV][64];
};

size_t lds_control_bytes() { return (sizeof(Ctl) + 255) & ~(size_t)255; }
size_t lds_bytes_needed(uint32_t n_slots, uint32_t slot_bytes) {
    return (size_t)n_slots * slot_bytes + lds_control_bytes();
}

extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

typedef __attribute__((address_space(3))) unsigned char lds_byte;
typedef __attribute__((address_space(3))) volatile uint32_t lds_vu32;
typedef __attribute__((address_space(3))) volatile uint64_t lds_vu64;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define DEV __device__ __forceinline__

DEV lds_byte *lds0() { return (lds_byte *)smem; }
DEV f32x4 lds_ld128(uint32_t off) { return *(const __attribute__((address_space(3))) f32x4 *)(lds0() + off); }
DEV void lds_st128(uint32_t off, u32x4 v) { *(__attribute__((address_space(3))) u32x4 *)(lds0() + off) = v; }
DEV float lds_ldf(uint32_t off) { return *(const __attribute__((address_space(3))) float *)(lds0() + off); }
DEV void lds_stf(uint32_t off, float v) { *(__attribute__((address_space(3))) float *)(lds0() + off) = v; }
DEV uint32_t lds_ld32(uint32_t off) { return *(const __attribute__((address_space(3))) uint32_t *)(lds0() + off); }

DEV void compiler_barrier() { asm volatile("" ::: "memory"); }
DEV void lds_wait() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
DEV uint32_t uni(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }
DEV uint64_t uni64(uint64_t x) {
    return (uint64_t)uni((uint32_t)x) | ((uint64_t)uni((uint32_t)(x >> 32)) << 32);
}

// Program memory is read-only while a run is in flight: read it through the constant address space so that
// uniform addresses become scalar loads.
typedef const __attribute__((address_space(4))) uint32_t *cptr32;
DEV uint32_t cload(const void *p, uint32_t idx) { return uni(((cptr32)(uintptr_t)p)[idx]); }

struct Ctx {
    const KParams *p;
    __attribute__((address_space(3))) Ctl *ctl;
    uint32_t core, lane, role, unit;  // unit: LDU/STU index in the unit queues, or VCC index
    uint32_t stream_pc0;              // first word of this unit's stream (CFU, VCC)
    uint32_t pc;                      // current word (for error reports)
    uint32_t spins_limit;
};

// ------------------------------------------------------------------------------------------------
// Errors and waiting
// ------------------------------------------------------------------------------------------------
DEV void raise_error(Ctx &c, int code, uint32_t detail) {
    if (c.lane == 0) {
        uint32_t *st = c.p->status;
        if (atomicCAS(&st[ST_ABORT], 0u, 1u) == 0u) {
            st[ST_CODE] = (uint32_t)(-code);
            st[ST_CORE] = c.core;
            st[ST_ROLE] = c.role | (c.unit << 8);
            st[ST_PC] = c.pc - c.stream_pc0;
            st[ST_DETAIL] = detail;
            __threadfence();
        }
        ((lds_vu32 *)&c.ctl->abort)[0] = 1u;
    }
}

struct Spin {
    uint32_t n = 0;
};

// One back-off step of a poll loop.  Returns false when the unit must give up (error raised somewhere,
// or the watchdog limit is reached, in which case this unit raises VDC_EDEADLOCK).
DEV bool spin_step(Ctx &c, Spin &s, uint32_t detail) {
    __builtin_amdgcn_s_sleep(1);
    s.n++;
    if ((s.n & 31u) == 0u) {
        if (uni(((lds_vu32 *)&c.ctl->abort)[0])) return false;
        if ((s.n & 1023u) == 0u) {
            uint32_t g = uni(__hip_atomic_load(&c.p->status[ST_ABORT], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            if (g) return false;
        }
        if (s.n >= c.spins_limit) {
            raise_error(c, -5 /* VDC_EDEADLOCK */, detail);
            return false;
        }
    }
    return true;
}

// ------------------------------------------------------------------------------------------------
// Register state of a stream: pc, loop stack, accumulators (Section 4.1: "a lightweight register machine")
// ------------------------------------------------------------------------------------------------
// Indexed state (accumulators, loop stack) is kept in a "lane register file": one vector register whose lane i
// holds entry i, read with v_readlane and written with v_writelane under a wave-uniform index.  Nothing of a
// unit's register state lives in memory.
DEV uint32_t rf_get(uint32_t v, uint32_t idx) { return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)idx); }
DEV uint32_t rf_set(uint32_t v, uint32_t idx, uint32_t x) {
    x = uni(x);
    idx = uni(idx);
    // one scalar register operand per vector instruction on this target: the lane select goes through M0;
    // the nops keep the required distance between the scalar writes and the lane access
    asm("s_mov_b32 m0, %2\n\ts_nop 3\n\tv_writelane_b32 %0, %1, m0" : "+v"(v) : "s"(x), "s"(idx));
    return v;
}

struct Seq {
    uint32_t pc, depth;
    uint32_t rf_lo, rf_hi;   // lanes 0..7: accumulator i (low, high word); lanes 8..11: loop level d (body start, trips left)
};

DEV void seq_init(Seq &s, uint32_t pc) {
    s.pc = pc;
    s.depth = 0;
    s.rf_lo = 0;
    s.rf_hi = 0;
}

DEV int64_t seq_acc(const Seq &s, uint32_t a) {
    return (int64_t)((uint64_t)rf_get(s.rf_lo, a) | ((uint64_t)rf_get(s.rf_hi, a) << 32));
}

DEV void seq_acc_set(Seq &s, uint32_t a, int64_t v) {
    s.rf_lo = rf_set(s.rf_lo, a, (uint32_t)(uint64_t)v);
    s.rf_hi = rf_set(s.rf_hi, a, (uint32_t)((uint64_t)v >> 32));
}

DEV Word fetch(const KParams *p, uint32_t pc) {
    Word w;
    w.w0 = cload(p->words, pc * 4 + 0);
    w.w1 = cload(p->words, pc * 4 + 1);
    w.w2 = cload(p->words, pc * 4 + 2);
    w.w3 = cload(p->words, pc * 4 + 3);
    return w;
}

// Control uops (run on every kind of core).  Returns 1 if handled, 2 for HALT, 0 if `f` is not a control uop.
// The host validated nesting and trip counts, so the stack cannot overflow here.
DEV int seq_control(Seq &s, const Fields &f) {
    switch (f.opcode) {
        case OP_HALT:
            return 2;
        case OP_LOOP: {
            s.rf_lo = rf_set(s.rf_lo, 8u + s.depth, s.pc + 1u);
            s.rf_hi = rf_set(s.rf_hi, 8u + s.depth, (uint32_t)f.imm);
            s.depth++;
            s.pc++;
            return 1;
        }
        case OP_REPEAT: {
            seq_acc_set(s, f.acc, seq_acc(s, f.acc) + f.imm);
            const uint32_t lvl = 8u + s.depth - 1u;
            const uint32_t left = rf_get(s.rf_hi, lvl) - 1u;
            s.rf_hi = rf_set(s.rf_hi, lvl, left);
            if (left > 0) {
                s.pc = rf_get(s.rf_lo, lvl);
            } else {
                s.depth--;
                s.pc++;
            }
            return 1;
        }
        case OP_ADD:
            seq_acc_set(s, f.acc, seq_acc(s, f.acc) + f.imm);
            s.pc++;
            return 1;
        case OP_SET:
            seq_acc_set(s, f.acc, f.imm);
            s.pc++;
            return 1;
        default:
            return 0;
    }
}

DEV void trace_put(Ctx &c, uint32_t stream, uint32_t &count, uint32_t pc_rel, uint32_t info, uint64_t v) {
    if (c.lane == 0) {
        if (count < c.p->trace_cap) {
            uint32_t *t = c.p->trace + ((size_t)stream * c.p->trace_cap + count) * 4;
            t[0] = pc_rel;
            t[1] = info;
            t[2] = (uint32_t)v;
            t[3] = (uint32_t)(v >> 32);
        }
        c.p->trace_count[stream] = count + 1;
    }
    count++;
}

// ------------------------------------------------------------------------------------------------
// SIMT slot allocator (Section 4.3): lane p probes position p; a wave vote takes the first free run.
// ------------------------------------------------------------------------------------------------
DEV int slot_find(uint32_t mask, uint32_t n, uint32_t n_slots, uint32_t lane) {
    // positions at or beyond n_slots count as busy
    uint64_t busy = (uint64_t)mask | (~0ull << n_slots);
    uint64_t ones = (n >= 64) ? ~0ull : ((1ull << n) - 1ull);
    bool ok = lane < 32u && ((busy >> lane) & ones) == 0ull;
    uint64_t vote = __ballot(ok);
    if (vote == 0ull) return -1;
    return (int)__builtin_ctzll(vote);
}

__global__ void debug_alloc_kernel(const uint32_t *masks, const int32_t *nslots, int32_t n_slots, int32_t *pos, int32_t n) {
    uint32_t lane = threadIdx.x & 63u;
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        int p = slot_find(masks[i], (uint32_t)nslots[i], (uint32_t)n_slots, lane);
        if (lane == 0) pos[i] = p;
    }
}

__global__ void clear_kernel(uint32_t *p, uint32_t n) {
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// ------------------------------------------------------------------------------------------------
// Queue primitives
// ------------------------------------------------------------------------------------------------
DEV void m2c_deliver(Ctx &c, uint32_t v, uint32_t ticket, uint32_t slot, uint32_t nslots, uint32_t rows, uint32_t row_bytes) {
    if (c.lane == 0) {
        uint64_t e = (uint64_t)(slot | (nslots << 6) | (rows << 12)) |
                     ((uint64_t)(((ticket + 1u) & 0xFFFFu) | (row_bytes << 16)) << 32);
        ((lds_vu64 *)&c.ctl->m2c[v][ticket & (kM2C - 1)])[0] = e;
    }
}

struct Msg {
    uint32_t slot, nslots, rows, row_bytes;
};

// pop_wait of the listing: block until ticket `head` of m2c[v] has been delivered.
DEV bool m2c_pop_wait(Ctx &c, uint32_t v, uint32_t head, Msg &m) {
    lds_vu64 *e = (lds_vu64 *)&c.ctl->m2c[v][head & (kM2C - 1)];
    const uint32_t want = (head + 1u) & 0xFFFFu;
    Spin s;
    for (;;) {
        uint64_t x = uni64(e[0]);
        uint32_t hi = (uint32_t)(x >> 32);
        if ((hi & 0xFFFFu) == want) {
            uint32_t lo = (uint32_t)x;
            m.slot = lo & 63u;
            m.nslots = (lo >> 6) & 63u;
            m.rows = lo >> 12;
            m.row_bytes = hi >> 16;
            compiler_barrier();
            return true;
        }
        if (!spin_step(c, s, 0x100u | v)) return false;
    }
}

// push to c2m[v]: the two waves of a VCC both call this when they are done with ticket `head`; the second
// one to arrive sends the message (kind 0 = used region to recycle, 1 = produced region).
DEV void c2m_push_when_both_done(Ctx &c, uint32_t v, uint32_t head, const Msg &m, uint32_t kind) {
    compiler_barrier();
    if (c.lane == 0) {
        __attribute__((address_space(3))) uint32_t *done =
            (__attribute__((address_space(3))) uint32_t *)&c.ctl->m2c_done[v][head & (kM2C - 1)];
        uint32_t old = __hip_atomic_fetch_add(done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (old == 1u) {
            __hip_atomic_store(done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            uint32_t pos = __hip_atomic_fetch_add((__attribute__((address_space(3))) uint32_t *)&c.ctl->c2m_tail[v], 1u,
                                                  __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            uint64_t e = (uint64_t)(kind | (m.slot << 1) | (m.nslots << 7)) | ((uint64_t)(pos + 1u) << 32);
            ((lds_vu64 *)&c.ctl->c2m[v][pos & (kC2M - 1)])[0] = e;
        }
    }
    compiler_barrier();
}

DEV void slots_free(Ctx &c, uint32_t slot, uint32_t nslots) {
    if (c.lane == 0) {
        uint32_t bits = (nslots >= 32u ? 0xFFFFFFFFu : ((1u << nslots) - 1u)) << slot;
        __hip_atomic_fetch_and((__attribute__((address_space(3))) uint32_t *)&c.ctl->mask, ~bits, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_WORKGROUP);
    }
}

// ------------------------------------------------------------------------------------------------
// CFU: the front end of the virtual memory core
// ------------------------------------------------------------------------------------------------
struct CfuState {
    uint32_t c2m_head0, c2m_head1;
    uint32_t mbox_tail0, mbox_tail1;
    uint32_t ticket0, ticket1;
    uint32_t uq_tail_rf;   // lane u: records pushed to unit u
};

DEV uint32_t uq_tail_get(const CfuState &st, uint32_t u) { return rf_get(st.uq_tail_rf, u); }
DEV void uq_tail_inc(CfuState &st, uint32_t u) { st.uq_tail_rf = rf_set(st.uq_tail_rf, u, rf_get(st.uq_tail_rf, u) + 1u); }

// Receiver of one c2m queue: used regions go back to the pool, produced regions to the STORE waiting for them.
DEV void cfu_drain_one(Ctx &c, uint32_t v, uint32_t &c2m_head, uint32_t &mbox_tail) {
    for (;;) {
        uint64_t x = uni64(((lds_vu64 *)&c.ctl->c2m[v][c2m_head & (kC2M - 1)])[0]);
        if ((uint32_t)(x >> 32) != c2m_head + 1u) break;
        c2m_head++;
        uint32_t lo = (uint32_t)x;
        uint32_t slot = (lo >> 1) & 63u, nslots = (lo >> 7) & 63u;
        if ((lo & 1u) == 0u) {
            slots_free(c, slot, nslots);
        } else {
            if (c.lane == 0) {
                ((lds_vu32 *)&c.ctl->mbox[v][mbox_tail & (kMbox - 1)])[0] = slot | (nslots << 6);
                ((lds_vu32 *)&c.ctl->mbox_tail[v])[0] = mbox_tail + 1u;
            }
            mbox_tail++;
        }
    }
}

DEV void cfu_drain(Ctx &c, CfuState &st) {
    cfu_drain_one(c, 0u, st.c2m_head0, st.mbox_tail0);
    if (c.p->V > 1u) cfu_drain_one(c, 1u, st.c2m_head1, st.mbox_tail1);
}

DEV void cfu_main(Ctx &c) {
    const bool TRACE = c.p->trace != nullptr;
    const KParams *p = c.p;
    const uint32_t stream = c.core * (1u + p->V);
    Seq s;
    seq_init(s, cload(p->stream_begin, stream));
    c.stream_pc0 = s.pc;
    CfuState st = {0, 0, 0, 0, 0, 0, 0};
    uint32_t trace_n = 0;
    const uint32_t slot_shift = __builtin_ctz(p->slot_bytes);
    bool ok = true;

    while (ok) {
        c.pc = s.pc;
        Word w = fetch(p, s.pc);
        Fields f = decode(w);
        int ctl = seq_control(s, f);
        if (ctl == 2) break;
        if (ctl == 1) continue;
        // ---- a memory uop: address generation, slot allocation in program order, dispatch by virtual flow ----
        const uint32_t dbase = f.desc * 8u;
        const uint32_t d_tensor = cload(p->descs, dbase + 0), d_box = cload(p->descs, dbase + 1);
        const uint32_t d_rowb = cload(p->descs, dbase + 2), d_pitch = cload(p->descs, dbase + 3);
        const uint32_t d_gp_lo = cload(p->descs, dbase + 4), d_gp_hi = cload(p->descs, dbase + 5);
        const bool is_load = f.opcode == OP_LOAD;
        const uint32_t unit = is_load ? (f.vflow % p->n_ldu) : (p->n_ldu + f.vflow % p->n_stu);
        int64_t eff = f.imm + ((f.flags & F_DYNAMIC) ? seq_acc(s, f.acc) : 0);

        // room in the unit's queue
        Spin sp;
        for (;;) {
            cfu_drain(c, st);
            uint32_t head = uni(((lds_vu32 *)&c.ctl->uq_head[unit])[0]);
            if (uq_tail_get(st, unit) - head < (uint32_t)kUQ) break;
            if (!spin_step(c, sp, 0x200u | unit)) { ok = false; break; }
        }
        if (!ok) break;
        // in-order allocation: stall right here until the request fits
        int slot;
        for (;;) {
            uint32_t mask = uni(((lds_vu32 *)&c.ctl->mask)[0]);
            slot = slot_find(mask, f.nslots, p->n_slots, c.lane);
            if (slot >= 0) break;
            cfu_drain(c, st);
            if (!spin_step(c, sp, 0x300u | f.nslots)) { ok = false; break; }
        }
        if (!ok) break;
        if (c.lane == 0) {
            uint32_t bits = (f.nslots >= 32u ? 0xFFFFFFFFu : ((1u << f.nslots) - 1u)) << slot;
            __hip_atomic_fetch_or((__attribute__((address_space(3))) uint32_t *)&c.ctl->mask, bits, __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        uint32_t ticket = 0xFFFFFFFFu;
        if (f.flags & F_SEND) {
            if (f.vcc == 0u) ticket = st.ticket0++;
            else ticket = st.ticket1++;
        }
        if (TRACE) trace_put(c, stream, trace_n, s.pc - c.stream_pc0, f.opcode | (f.desc << 8) | (f.size << 16), (uint64_t)eff);
        if (!is_load && (f.flags & F_SEND)) {
            // the empty output region goes to the compute core at once; the store unit only waits for it to return
            m2c_deliver(c, f.vcc, ticket, (uint32_t)slot, f.nslots, f.size, d_rowb);
        }
        // hand the decoded uop to its unit
        {
            // the tensor table sits in the kernel arguments: a uniform index makes this a scalar load
            const uint64_t base = uni64((uint64_t)(uintptr_t)p->tensors[d_tensor & (kMaxTensors - 1)]);
            uint64_t gaddr = base + (uint64_t)eff;
            const uint32_t tail = uq_tail_get(st, unit);
            uint32_t idx = tail & (kUQ - 1);
            if (c.lane == 0) {
                uint32_t off = (uint32_t)((size_t)&c.ctl->uq[unit][idx] - (size_t)lds0());
                u32x4 a = {(uint32_t)gaddr, (uint32_t)(gaddr >> 32), d_gp_lo, d_gp_hi};
                u32x4 b = {(uint32_t)slot << slot_shift, f.size | (d_box << 16), d_rowb | (d_pitch << 16), w.w0};
                u32x4 d = {ticket, (uint32_t)slot, f.dep_id | (f.dep_count << 16), s.pc - c.stream_pc0};
                lds_st128(off, a);
                lds_st128(off + 16, b);
                lds_st128(off + 32, d);
                compiler_barrier();
                ((lds_vu32 *)&c.ctl->uq_tail[unit])[0] = tail + 1u;
            }
            uq_tail_inc(st, unit);
        }
        s.pc++;
    }

    // HALT (or error): no more dispatches.  Keep receiving c2m until the units and the compute cores are done.
    if (c.lane == 0) ((lds_vu32 *)&c.ctl->cfu_halted)[0] = 1u;
    Spin sp;
    while (ok) {
        cfu_drain(c, st);
        bool done = uni(((lds_vu32 *)&c.ctl->vcc_done)[0]) == 2u * p->V;
        for (uint32_t u = 0; u < p->n_ldu + p->n_stu; u++)
            done = done && (uni(((lds_vu32 *)&c.ctl->uq_head[u])[0]) == uq_tail_get(st, u));
        if (done) break;
        if (!spin_step(c, sp, 0x400u)) ok = false;
    }
    if (ok) {
        cfu_drain(c, st);
        lds_wait();
        uint32_t mask = uni(((lds_vu32 *)&c.ctl->mask)[0]);
        if (mask != 0u) raise_error(c, -6 /* VDC_ELEAK */, mask);
    }
}

// ------------------------------------------------------------------------------------------------
// LDU: tile loads, global -> LDS, without going through registers
// ------------------------------------------------------------------------------------------------
DEV void wait_vmcnt_le(uint32_t n) {
#define VDC_VM_CASE(k) \
    case k:            \
        asm volatile("s_waitcnt vmcnt(" #k ")" ::: "memory"); \
        break;
    switch (n) {
        VDC_VM_CASE(0) VDC_VM_CASE(1) VDC_VM_CASE(2) VDC_VM_CASE(3) VDC_VM_CASE(4) VDC_VM_CASE(5) VDC_VM_CASE(6) VDC_VM_CASE(7)
        VDC_VM_CASE(8) VDC_VM_CASE(9) VDC_VM_CASE(10) VDC_VM_CASE(11) VDC_VM_CASE(12) VDC_VM_CASE(13) VDC_VM_CASE(14)
        VDC_VM_CASE(15) VDC_VM_CASE(16) VDC_VM_CASE(17) VDC_VM_CASE(18) VDC_VM_CASE(19) VDC_VM_CASE(20) VDC_VM_CASE(21)
        VDC_VM_CASE(22) VDC_VM_CASE(23) VDC_VM_CASE(24) VDC_VM_CASE(25) VDC_VM_CASE(26) VDC_VM_CASE(27) VDC_VM_CASE(28)
        VDC_VM_CASE(29) VDC_VM_CASE(30) VDC_VM_CASE(31) VDC_VM_CASE(32) VDC_VM_CASE(33) VDC_VM_CASE(34) VDC_VM_CASE(35)
        VDC_VM_CASE(36) VDC_VM_CASE(37) VDC_VM_CASE(38) VDC_VM_CASE(39) VDC_VM_CASE(40) VDC_VM_CASE(41) VDC_VM_CASE(42)
        VDC_VM_CASE(43) VDC_VM_CASE(44) VDC_VM_CASE(45) VDC_VM_CASE(46) VDC_VM_CASE(47) VDC_VM_CASE(48) VDC_VM_CASE(49)
        VDC_VM_CASE(50) VDC_VM_CASE(51) VDC_VM_CASE(52) VDC_VM_CASE(53) VDC_VM_CASE(54) VDC_VM_CASE(55) VDC_VM_CASE(56)
        default:
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            break;
    }
#undef VDC_VM_CASE
}

DEV void load_lds_b128(uint32_t lds_addr_wave, const char *gptr, bool nt) {
    // LDS address = M0 + lane * 16 (wave-uniform base in M0, one 16-byte chunk per active lane)
    lds_addr_wave = uni(lds_addr_wave);
    if (nt)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(lds_addr_wave), "v"(gptr) : "memory");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr_wave), "v"(gptr) : "memory");
}

struct Inflight {   // what an LDU must do once the loads of a tile have landed
    uint32_t w0, ticket, dep;
    uint32_t slot_ninstr;   // slot | load instructions << 8
    uint32_t rows_rb;       // valid rows | valid row_bytes << 16
};

DEV bool dep_wait(Ctx &c, uint32_t dep) {
    uint32_t id = dep & 0xFFFFu, need = dep >> 16;
    if (need == 0u) need = 1u;
    Spin s;
    for (;;) {
        uint32_t v = uni(__hip_atomic_load(&c.p->dep[id], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT));
        if (v >= need) return true;
        if (!spin_step(c, s, 0x500u | id)) return false;
    }
}

DEV void dep_signal(Ctx &c, uint32_t dep) {
    if (c.lane == 0) {
        __hip_atomic_fetch_add(&c.p->dep[dep & 0xFFFFu], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
}

DEV void ldu_retire(Ctx &c, const Inflight &t) {
    const uint32_t flags = (t.w0 >> 8) & 0xFFu, vcc = (t.w0 >> 20) & 3u, nslots = (t.w0 >> 25) & 63u;
    lds_wait();   // zero fill of this tile (ds_write) is done as well
    if (flags & F_SEND) m2c_deliver(c, vcc, t.ticket, t.slot_ninstr & 0xFFu, nslots, t.rows_rb & 0xFFFFu, t.rows_rb >> 16);
    if (flags & F_DEP_SEND) dep_signal(c, t.dep);
}

DEV void ldu_main(Ctx &c) {
    const KParams *p = c.p;
    const uint32_t u = c.unit;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds0();
    // tiles in flight: a ring in a lane register file (lane k = entry k), oldest at fl_head
    uint32_t fl_w0 = 0, fl_ticket = 0, fl_dep = 0, fl_sn = 0, fl_rr = 0;
    uint32_t fl_head = 0;
    uint32_t n_fl = 0;
    uint32_t vm_out = 0;      // load instructions issued and not yet known complete
    uint32_t head = 0;
    Spin sp;
    bool ok = true;
    while (ok) {
        uint32_t tail = uni(((lds_vu32 *)&c.ctl->uq_tail[u])[0]);
        compiler_barrier();
        bool have = tail != head;
        uint32_t ni = 0;
        UnitRec r;
        if (have) {
            uint32_t off = (uint32_t)((size_t)&c.ctl->uq[u][head & (kUQ - 1)] - (size_t)lds0());
            f32x4 a = lds_ld128(off), b = lds_ld128(off + 16), d = lds_ld128(off + 32);
            r.gaddr_lo = uni(__float_as_uint(a.x)); r.gaddr_hi = uni(__float_as_uint(a.y));
            r.gpitch_lo = uni(__float_as_uint(a.z)); r.gpitch_hi = uni(__float_as_uint(a.w));
            r.lds_off = uni(__float_as_uint(b.x)); r.rows_box = uni(__float_as_uint(b.y));
            r.rb_pitch = uni(__float_as_uint(b.z)); r.w0 = uni(__float_as_uint(b.w));
            r.ticket = uni(__float_as_uint(d.x)); r.slot = uni(__float_as_uint(d.y));
            r.dep = uni(__float_as_uint(d.z)); r.pc = uni(__float_as_uint(d.w));
            uint32_t chunks = (r.rows_box >> 16) * ((r.rb_pitch >> 16) >> 4);
            ni = (chunks + 63u) >> 6;
        }
        // retire the oldest tile when nothing can be issued on top of what is in flight
        bool can_issue = have && n_fl < (uint32_t)kMaxInflight && (vm_out + ni <= (uint32_t)kMaxVm || n_fl == 0);
        if (!can_issue) {
            if (n_fl > 0) {
                const uint32_t k = fl_head & (kMaxInflight - 1);
                Inflight o = {rf_get(fl_w0, k), rf_get(fl_ticket, k), rf_get(fl_dep, k), rf_get(fl_sn, k), rf_get(fl_rr, k)};
                wait_vmcnt_le(vm_out - (o.slot_ninstr >> 8));
                vm_out -= o.slot_ninstr >> 8;
                ldu_retire(c, o);
                fl_head++;
                n_fl--;
                sp.n = 0;
                continue;
            }
            if (!have) {
                if (uni(((lds_vu32 *)&c.ctl->cfu_halted)[0]) && uni(((lds_vu32 *)&c.ctl->uq_tail[u])[0]) == head) break;
                if (!spin_step(c, sp, 0x600u | u)) ok = false;
                continue;
            }
        }
        // ---- issue the loads of record r ----
        c.pc = c.stream_pc0 + r.pc;
        const uint32_t flags = (r.w0 >> 8) & 0xFFu;
        if (flags & F_DEP_RECV) {
            // an unresolved dependency blocks this unit, and only this unit (Section 4.3).  Whatever is already in
            // flight is delivered first: the awaited signal may depend on it
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            vm_out = 0;
            for (; n_fl > 0; n_fl--, fl_head++) {
                const uint32_t k = fl_head & (kMaxInflight - 1);
                Inflight o = {rf_get(fl_w0, k), rf_get(fl_ticket, k), rf_get(fl_dep, k), rf_get(fl_sn, k), rf_get(fl_rr, k)};
                ldu_retire(c, o);
            }
            if (!dep_wait(c, r.dep)) { ok = false; break; }
        }
        const uint32_t rows = r.rows_box & 0xFFFFu, box_rows = r.rows_box >> 16;
        const uint32_t row_bytes = r.rb_pitch & 0xFFFFu, lds_pitch = r.rb_pitch >> 16;
        const uint32_t cpr = lds_pitch >> 4;                 // 16-byte chunks per row of the box
        const uint32_t vcr = row_bytes >> 4;                 // valid chunks per row
        const uint32_t total = box_rows * cpr;
        const uint64_t gaddr = (uint64_t)r.gaddr_lo | ((uint64_t)r.gaddr_hi << 32);
        const uint64_t gpitch = (uint64_t)r.gpitch_lo | ((uint64_t)r.gpitch_hi << 32);
        const bool nt = (flags & F_NT) != 0;
        uint32_t row = c.lane / cpr, col = c.lane % cpr;
        const uint32_t drow = 64u / cpr, dcol = 64u % cpr;
        const bool full = rows == box_rows && vcr == cpr && (total & 63u) == 0u;
        for (uint32_t i = 0; i < ni; i++) {
            const uint32_t q = i * 64u + c.lane;
            const char *g = (const char *)(uintptr_t)(gaddr + (uint64_t)row * gpitch + (uint64_t)col * 16u);
            const uint32_t dst = lds_base + r.lds_off + i * 1024u;
            if (full) {
                load_lds_b128(dst, g, nt);
            } else {
                const bool inside = q < total;
                const bool valid = inside && row < rows && col < vcr;
                if (valid) load_lds_b128(dst, g, nt);
                if (inside && !valid) {
                    u32x4 z = {0u, 0u, 0u, 0u};
                    lds_st128(r.lds_off + q * 16u, z);       // the box outside the valid tile reads as zero
                }
            }
            row += drow;
            col += dcol;
            if (col >= cpr) { col -= cpr; row++; }
        }
        {
            const uint32_t k = (fl_head + n_fl) & (kMaxInflight - 1);
            fl_w0 = rf_set(fl_w0, k, r.w0);
            fl_ticket = rf_set(fl_ticket, k, r.ticket);
            fl_dep = rf_set(fl_dep, k, r.dep);
            fl_sn = rf_set(fl_sn, k, r.slot | (ni << 8));
            fl_rr = rf_set(fl_rr, k, rows | (row_bytes << 16));
        }
        n_fl++;
        vm_out += ni;
        head++;
        if (c.lane == 0) ((lds_vu32 *)&c.ctl->uq_head[u])[0] = head;
        sp.n = 0;
    }
    // never leave with loads in flight: their LDS destination belongs to this workgroup only while it lives
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (ok) {
        for (; n_fl > 0; n_fl--, fl_head++) {
            const uint32_t k = fl_head & (kMaxInflight - 1);
            Inflight o = {rf_get(fl_w0, k), rf_get(fl_ticket, k), rf_get(fl_dep, k), rf_get(fl_sn, k), rf_get(fl_rr, k)};
            ldu_retire(c, o);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// STU: produced region -> global memory
// ------------------------------------------------------------------------------------------------
DEV void stu_main(Ctx &c) {
    const KParams *p = c.p;
    const uint32_t u = c.unit;
    uint32_t head = 0;
    uint32_t mbox_head[kMaxV] = {0, 0};
    Spin sp;
    bool ok = true;
    while (ok) {
        uint32_t tail = uni(((lds_vu32 *)&c.ctl->uq_tail[u])[0]);
        if (tail == head) {
            if (uni(((lds_vu32 *)&c.ctl->cfu_halted)[0]) && uni(((lds_vu32 *)&c.ctl->uq_tail[u])[0]) == head) break;
            if (!spin_step(c, sp, 0x700u | u)) ok = false;
            continue;
        }
        sp.n = 0;
        compiler_barrier();
        uint32_t off = (uint32_t)((size_t)&c.ctl->uq[u][head & (kUQ - 1)] - (size_t)lds0());
        f32x4 a = lds_ld128(off), b = lds_ld128(off + 16), d = lds_ld128(off + 32);
        const uint64_t gaddr = (uint64_t)uni(__float_as_uint(a.x)) | ((uint64_t)uni(__float_as_uint(a.y)) << 32);
        const uint64_t gpitch = (uint64_t)uni(__float_as_uint(a.z)) | ((uint64_t)uni(__float_as_uint(a.w)) << 32);
        const uint32_t lds_off = uni(__float_as_uint(b.x)), rows = uni(__float_as_uint(b.y)) & 0xFFFFu;
        const uint32_t rb_pitch = uni(__float_as_uint(b.z)), w0 = uni(__float_as_uint(b.w));
        const uint32_t slot = uni(__float_as_uint(d.y)), dep = uni(__float_as_uint(d.z));
        c.pc = c.stream_pc0 + uni(__float_as_uint(d.w));
        const uint32_t flags = (w0 >> 8) & 0xFFu, vcc = (w0 >> 20) & 3u, nslots = (w0 >> 25) & 63u;
        if (flags & F_DEP_RECV) {
            if (!dep_wait(c, dep)) { ok = false; break; }
        }
        if (flags & F_RECV) {
            // wait for the compute core to hand the region back as "produced"
            uint32_t mh = vcc == 0u ? mbox_head[0] : mbox_head[1];
            Spin s2;
            for (;;) {
                if (uni(((lds_vu32 *)&c.ctl->mbox_tail[vcc])[0]) != mh) break;
                if (!spin_step(c, s2, 0x800u | vcc)) { ok = false; break; }
            }
            if (!ok) break;
            uint32_t got = uni(((lds_vu32 *)&c.ctl->mbox[vcc][mh & (kMbox - 1)])[0]);
            if (got != (slot | (nslots << 6))) {
                raise_error(c, -3 /* VDC_EPROGRAM */, 0x900u | got);
                ok = false;
                break;
            }
            if (vcc == 0u) mbox_head[0]++; else mbox_head[1]++;
            compiler_barrier();
        }
        const uint32_t row_words = (rb_pitch & 0xFFFFu) >> 2, lds_pitch = rb_pitch >> 16;
        const uint32_t total = rows * row_words;
        for (uint32_t i = c.lane; i < total; i += 64u) {
            uint32_t rr = i / row_words, cc = i % row_words;
            float v = lds_ldf(lds_off + rr * lds_pitch + cc * 4u);
            *(float *)(uintptr_t)(gaddr + (uint64_t)rr * gpitch + (uint64_t)cc * 4u) = v;
        }
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        slots_free(c, slot, nslots);
        if (flags & F_DEP_SEND) {
            __threadfence();
            dep_signal(c, dep);
        }
        head++;
        if (c.lane == 0) ((lds_vu32 *)&c.ctl->uq_head[u])[0] = head;
    }
}

// ------------------------------------------------------------------------------------------------
// VCC: compute uop handlers
// ------------------------------------------------------------------------------------------------
struct VccState {
    uint32_t head;     // next m2c ticket to pop
    uint32_t red_seq;  // cross-wave reductions done so far
    uint32_t wv;       // which of the two waves of the execution unit this is
    uint32_t t;        // thread index inside the execution unit, 0..127
};

DEV float dot4(f32x4 m, f32x4 x, float acc) {
    acc = __builtin_fmaf(m.x, x.x, acc);
    acc = __builtin_fmaf(m.y, x.y, acc);
    acc = __builtin_fmaf(m.z, x.z, acc);
    acc = __builtin_fmaf(m.w, x.w, acc);
    return acc;
}

// The matvec compute uop (listing in Section 4.1).  A matrix tile is NF passes of 128 chunks of 16 bytes.
//   J == 0: a tile row has lpr <= 64 chunks and lies inside one wave: thread t always sees columns
//           4*(t % lpr) .. +3 and, in pass i, row i * (128 / lpr) + t / lpr.
//   J >= 1: a tile row has 128 * J chunks: pass i holds chunks (i % J) * 128 + t of row i / J.
// The vector tile is [B][4 * lpr] floats with the same row pitch.
template <int B, int NF, int J>
DEV bool matvec_uop(Ctx &c, VccState &vs, uint32_t size, uint32_t R, uint32_t lpr) {
    const KParams *p = c.p;
    const uint32_t v = c.unit;
    const uint32_t slot_shift = __builtin_ctz(p->slot_bytes);
    constexpr int NACC = (J == 0) ? NF : NF / (J == 0 ? 1 : J);
    constexpr int NX = (J == 0) ? 1 : J;
    float acc[NACC][B];                      // alloc_registers(NCREGS)
#pragma unroll
    for (int i = 0; i < NACC; i++)
#pragma unroll
        for (int b = 0; b < B; b++) acc[i][b] = 0.0f;
    const uint32_t t = vs.t;
    const uint32_t c4 = (J == 0) ? (t & (lpr - 1u)) : t;
    const uint32_t pitch = lpr * 16u;

    for (uint32_t it = 0; it < size; it++) {
        Msg ma, mb;
        if (!m2c_pop_wait(c, v, vs.head, ma)) return false;         // a = m2c.pop_wait()
        if (!m2c_pop_wait(c, v, vs.head + 1u, mb)) return false;    // b = m2c.pop_wait()
        const uint32_t a_off = ma.slot << slot_shift, b_off = mb.slot << slot_shift;
        f32x4 xv[NX][B];
#pragma unroll
        for (int j = 0; j < NX; j++)
#pragma unroll
            for (int b = 0; b < B; b++) xv[j][b] = lds_ld128(b_off + (uint32_t)b * pitch + ((uint32_t)j * 128u + c4) * 16u);
        f32x4 m[NF];
#pragma unroll
        for (int i = 0; i < NF; i++) m[i] = lds_ld128(a_off + ((uint32_t)i * 128u + t) * 16u);
#pragma unroll
        for (int i = 0; i < NF; i++) {
            constexpr int JJ = (J == 0) ? 1 : J;
            const int ai = (J == 0) ? i : i / JJ;
            const int xi = (J == 0) ? 0 : i % JJ;
#pragma unroll
            for (int b = 0; b < B; b++) acc[ai][b] = dot4(m[i], xv[xi][b], acc[ai][b]);   // matvec_tile_accumulate
        }
        // all LDS reads of both tiles have returned once their values were used; hand the regions back
        c2m_push_when_both_done(c, v, vs.head, ma, 0u);              // c2m.push(a, b)
        c2m_push_when_both_done(c, v, vs.head + 1u, mb, 0u);
        vs.head += 2u;
    }

    Msg mo;
    if (!m2c_pop_wait(c, v, vs.head, mo)) return false;              // c_shared = m2c.pop_wait()
    const uint32_t o_off = mo.slot << slot_shift;
    if (J == 0) {
        const uint32_t lsh = __builtin_ctz(lpr);
        const uint32_t rpp = 128u >> lsh;
#pragma unroll
        for (int i = 0; i < NF; i++)
#pragma unroll
            for (int b = 0; b < B; b++) {
                float x = acc[i][b];
                for (uint32_t s = lpr >> 1; s > 0u; s >>= 1) x += __shfl_xor(x, (int)s, 64);
                if (c4 == 0u) lds_stf(o_off + ((uint32_t)b * R + (uint32_t)i * rpp + (t >> lsh)) * 4u, x);   // copy(c, c_shared)
            }
    } else {
        float mine = 0.0f;
#pragma unroll
        for (int r = 0; r < NACC; r++)
#pragma unroll
            for (int b = 0; b < B; b++) {
                float x = acc[r][b];
#pragma unroll
                for (int s = 32; s > 0; s >>= 1) x += __shfl_xor(x, s, 64);
                mine = (c.lane == (uint32_t)(r * B + b)) ? x : mine;
            }
        // the two waves of the execution unit each hold half of every row sum
        const uint32_t red_off = (uint32_t)((size_t)&c.ctl->red[v][0] - (size_t)lds0());
        Spin s;
        if (vs.wv == 1u) {
            while (uni(((lds_vu32 *)&c.ctl->red_ack[v])[0]) != vs.red_seq)
                if (!spin_step(c, s, 0xA00u)) return false;
            lds_stf(red_off + c.lane * 4u, mine);
            lds_wait();
            if (c.lane == 0) ((lds_vu32 *)&c.ctl->red_flag[v])[0] = vs.red_seq + 1u;
        } else {
            while (uni(((lds_vu32 *)&c.ctl->red_flag[v])[0]) != vs.red_seq + 1u)
                if (!spin_step(c, s, 0xB00u)) return false;
            compiler_barrier();
            mine += lds_ldf(red_off + c.lane * 4u);
            if (c.lane < (uint32_t)(NACC * B)) {
                uint32_t r = c.lane / (uint32_t)B, b = c.lane % (uint32_t)B;
                lds_stf(o_off + (b * R + r) * 4u, mine);
            }
            lds_wait();
            if (c.lane == 0) ((lds_vu32 *)&c.ctl->red_ack[v])[0] = vs.red_seq + 1u;
        }
        vs.red_seq++;
    }
    lds_wait();
    c2m_push_when_both_done(c, v, vs.head, mo, 1u);                   // push the produced region
    vs.head += 1u;
    return true;
}

template <int B>
DEV bool matvec_dispatch_b(Ctx &c, VccState &vs, uint32_t size, uint32_t R, uint32_t lpr, uint32_t nf, uint32_t j) {
#define VDC_MV(NF_, J_) \
    if (nf == NF_ && j == J_) return matvec_uop<B, NF_, J_>(c, vs, size, R, lpr);
    VDC_MV(1, 0) VDC_MV(2, 0) VDC_MV(4, 0) VDC_MV(8, 0)
    VDC_MV(1, 1) VDC_MV(2, 1) VDC_MV(4, 1) VDC_MV(8, 1)
    if constexpr (B * 2 <= 16) { VDC_MV(2, 2) VDC_MV(4, 2) VDC_MV(8, 2) }
    if constexpr (B * 4 <= 16) { VDC_MV(4, 4) VDC_MV(8, 4) }
    if constexpr (B * 8 <= 16) { VDC_MV(8, 8) }
#undef VDC_MV
    raise_error(c, -3 /* VDC_EPROGRAM */, 0xC00u);
    return false;
}

DEV bool matvec_dispatch(Ctx &c, VccState &vs, const Fields &f) {
    const uint32_t B = (uint32_t)f.imm & 0xFFu, R = (uint32_t)(f.imm >> 8) & 0xFFFFu, lpr = (uint32_t)(f.imm >> 24) & 0xFFFFu;
    const uint32_t nf = (R * lpr) >> 7;
    const uint32_t j = lpr <= 64u ? 0u : lpr >> 7;
    switch (B) {
        case 1: return matvec_dispatch_b<1>(c, vs, f.size, R, lpr, nf, j);
        case 2: return matvec_dispatch_b<2>(c, vs, f.size, R, lpr, nf, j);
        case 3: return matvec_dispatch_b<3>(c, vs, f.size, R, lpr, nf, j);
        case 4: return matvec_dispatch_b<4>(c, vs, f.size, R, lpr, nf, j);
        case 5: return matvec_dispatch_b<5>(c, vs, f.size, R, lpr, nf, j);
        case 6: return matvec_dispatch_b<6>(c, vs, f.size, R, lpr, nf, j);
        case 7: return matvec_dispatch_b<7>(c, vs, f.size, R, lpr, nf, j);
        case 8: return matvec_dispatch_b<8>(c, vs, f.size, R, lpr, nf, j);
        default:
            raise_error(c, -3 /* VDC_EPROGRAM */, 0xD00u);
            return false;
    }
}

// The control-flow unit of a VCC runs on the execution unit's own threads (Section 4.3, "Virtual Compute Core"):
// each of its two waves decodes the stream, runs control uops itself and then yields to the uop handler.
DEV void vcc_main(Ctx &c, uint32_t wv) {
    const bool TRACE = c.p->trace != nullptr;
    const KParams *p = c.p;
    const uint32_t stream = c.core * (1u + p->V) + 1u + c.unit;
    Seq s;
    seq_init(s, cload(p->stream_begin, stream));
    c.stream_pc0 = s.pc;
    VccState vs;
    vs.head = 0; vs.red_seq = 0; vs.wv = wv; vs.t = wv * 64u + c.lane;
    uint32_t trace_n = 0;
    bool ok = true;
    while (ok) {
        c.pc = s.pc;
        Word w = fetch(p, s.pc);
        Fields f = decode(w);
        int ctl = seq_control(s, f);
        if (ctl == 2) break;
        if (ctl == 1) continue;
        if (TRACE && wv == 0u) trace_put(c, stream, trace_n, s.pc - c.stream_pc0, f.opcode | (f.size << 16), (uint64_t)f.imm);
        if (f.opcode == OP_MATVEC) {
            ok = matvec_dispatch(c, vs, f);
        } else {
            raise_error(c, -3 /* VDC_EPROGRAM */, 0xE00u | f.opcode);
            ok = false;
        }
        s.pc++;
    }
    if (c.lane == 0)
        __hip_atomic_fetch_add((__attribute__((address_space(3))) uint32_t *)&c.ctl->vcc_done, 1u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_WORKGROUP);
}

// ------------------------------------------------------------------------------------------------
// The persistent kernel: every wave takes its role and runs it to the end of the uop graph
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(512) vdc_executor_kernel(const KParams p) {
    const uint32_t wave = uni(threadIdx.x >> 6);
    Ctx c;
    c.p = &p;
    c.core = blockIdx.x;
    c.lane = threadIdx.x & 63u;
    c.ctl = (__attribute__((address_space(3))) Ctl *)(lds0() + p.n_slots * p.slot_bytes);
    c.spins_limit = p.watchdog;
    c.stream_pc0 = 0;
    c.pc = 0;
    // the control block starts at zero (slots need no initialisation)
    {
        const uint32_t words = (uint32_t)(sizeof(Ctl) / 4);
        lds_vu32 *z = (lds_vu32 *)c.ctl;
        for (uint32_t i = threadIdx.x; i < words; i += blockDim.x) z[i] = 0u;
    }
    __syncthreads();   // the only workgroup barrier: before the roles diverge

    if (wave == 0u) {
        c.role = ROLE_CFU; c.unit = 0;
        cfu_main(c);
    } else if (wave <= p.n_ldu) {
        c.role = ROLE_LDU; c.unit = wave - 1u;
        c.stream_pc0 = cload(p.stream_begin, c.core * (1u + p.V));
        ldu_main(c);
    } else if (wave <= p.n_ldu + p.n_stu) {
        c.role = ROLE_STU; c.unit = wave - 1u;
        c.stream_pc0 = cload(p.stream_begin, c.core * (1u + p.V));
        stu_main(c);
    } else {
        const uint32_t k = wave - 1u - p.n_ldu - p.n_stu;
        c.role = ROLE_VCC; c.unit = k >> 1;
        vcc_main(c, k & 1u);
    }
}

hipError_t prepare_executor_kernels(size_t lds_bytes) {
    return hipFuncSetAttribute((const void *)vdc_executor_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
}

hipError_t launch_executor(const KParams &p, uint32_t n_cores, bool traced, hipStream_t stream) {
    const uint32_t waves = 1u + p.n_ldu + p.n_stu + 2u * p.V;
    const size_t lds = lds_bytes_needed(p.n_slots, p.slot_bytes);
    (void)traced;   // tracing is switched by p.trace
    hipLaunchKernelGGL(vdc_executor_kernel, dim3(n_cores), dim3(waves * 64u), lds, stream, p);
    return hipGetLastError();
}

hipError_t launch_clear(uint32_t *ptr, uint32_t n, hipStream_t stream) {
    hipLaunchKernelGGL(clear_kernel, dim3((n + 255u) / 256u), dim3(256), 0, stream, ptr, n);
    return hipGetLastError();
}

hipError_t launch_debug_alloc(const uint32_t *masks, const int32_t *nslots, int32_t n_slots, int32_t *pos, int32_t n,
                              hipStream_t stream) {
    int blocks = n < 1024 ? (n > 0 ? n : 1) : 1024;
    hipLaunchKernelGGL(debug_alloc_kernel, dim3(blocks), dim3(64), 0, stream, masks, nslots, n_slots, pos, n);
    return hipGetLastError();
}

}  // namespace vdc
