// The on-GPU executor: persistent virtual cores for CDNA4 (gfx950), one workgroup per compute unit.
//
// Section 4.3 of the paper ("GPU Executor") describes, for Hopper, one virtual memory core (VMC) per SM
// built from a control-flow unit (CFU) feeding parallel load units (LDU) and store units (STU), two
// virtual compute cores (VCC) of 128 threads, FIFO dependency queues between them, TMA for the tile
// copies and mbarrier for blocking waits.  CDNA4 has neither TMA nor mbarrier, so the roles map to
// wave64 wavefronts of one workgroup as follows:
//
//   wave 0                      CFU   fetch / decode / control uops / address generation / slot allocation /
//                                     dispatch by virtual flow
//   waves 1 .. n_ldu (<= 4)     LDU   direct-to-LDS 128-bit loads (global_load_lds_dwordx4), several tiles in
//                                     flight per unit, completion observed with s_waitcnt vmcnt(N), then the
//                                     region is delivered into its m2c ticket
//   next n_stu (1 or 2) waves   STU   receiver of the c2m queues (two units: one compute core each); waits for the
//                                     produced region, LDS -> global, frees the slots, signals depId; store.local /
//                                     load.local
//   next 2 * V waves            VCC   v = 0..V-1, two waves (128 threads) each: the compute uop handlers
//
// All queues live in LDS.  A waiter polls LDS with s_sleep back-off (no hardware de-scheduling exists);
// every poll loop counts its iterations and raises VDC_EDEADLOCK at the watchdog limit, and every loop also
// leaves when another unit or core has raised an error, so the grid always drains.
//
// What keeps the per-uop cost low (the paper's Section 4.3 asks for SIMT parallelism inside each unit):
//   * a unit reads everything it must look at (queue heads, its next record, the slot mask, the abort flag)
//     with ONE gathered LDS read, each lane fetching a different word, and one wait;
//   * uop words are fetched 64 at a time into a register window (one lane per word) and picked with v_readlane;
//     descriptors live in a register file of the same kind; no indexed state lives in memory;
//   * the slot mask is one scalar register in the front end: "first run of n free slots" is n - 1 shift-and-and
//     steps and a count-trailing-zeros, and a batch of up to four memory uops is allocated in one straight-line pass;
//   * nothing on the hot paths branches per lane: stores by single lanes are exec-masked LDS instructions, and a
//     compute core that is done with a used region clears its bits in the slot mask itself, with one LDS atomic.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <type_traits>

#include "vdc_isa.h"
#include "vdc_kernel.h"

namespace vdc {

// Instrumentation for throw-away profiling builds; the product build compiles none of it.  -DVDC_PROFILE adds an
// observer wave (see observer_main).
#if defined(VDC_PROFILE) || defined(VDC_PROFILE_WAITS)
static __device__ __forceinline__ unsigned long long prof_now() {
    unsigned long long t;
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t)::"memory");
    return t;
}
#endif

// ------------------------------------------------------------------------------------------------
// LDS layout: [0, n_slots * slot_bytes) the slots, then the control block.
// ------------------------------------------------------------------------------------------------
#define DEV_EARLY __device__ __forceinline__
constexpr int kUQ = 8;         // records per unit queue (CFU -> LDU/STU)
constexpr int kBatch = 4;      // memory uops the front end dispatches at once (a batch is published in one piece: more is later)
constexpr int kBatchOnes = 8;  // ... when every uop of the batch takes one slot: the lanes then allocate side by side
constexpr int kBatchWide = 6;  // ... when the batch is the whole body of a loop that is replayed (a trip of two steps: a vector
                               // tile and two matrix tiles per compute core)
constexpr int kM2C = 32;       // m2c ring entries per VCC (>= slots, so a delivery never finds it full)
constexpr int kC2M = 64;       // c2m ring entries per VCC
constexpr int kMbox = 32;      // produced regions waiting for their STORE, per VCC
constexpr int kMaxUnits = 8;   // n_ldu + n_stu
constexpr int kMaxV = 2;
constexpr int kRecWords = 4;
constexpr int kStatWords = 8;
constexpr int kWin = 64;        // uops in the decoded window
// A unit that polls takes issue slots from the compute wave on its SIMD (every vector instruction of a wave64 holds the
// SIMD's ALU for four cycles, whatever it computes), so a unit that has found nothing to do several times in a row
// looks less often: units of 64 cycles between two looks, and the idle looks after which the longer pause applies.
constexpr int kStuIdleNap = 8;
constexpr uint32_t kStuIdleAfter = 4;
constexpr int kCfuPrio = 3, kLduPrio = 2, kStuPrio = 2;

struct UnitRec {  // the per-execution part of a memory uop after the front end (16 bytes)
    uint32_t gaddr_lo, gaddr_hi;   // effective global address
    uint32_t info;                 // slot [5:0] | window lane [11:6] | table [12]
    uint32_t ticket;               // m2c position when SEND
};

// One m2c entry (16 bytes).  The payload is written by the front end when it dispatches the sending uop (it knows the
// slot, the shape and the ticket); `ready` says that the region may be used.  For a loaded tile `ready` is written by the
// memory system itself: the load unit issues, behind the tile's direct-to-LDS loads, one more direct-to-LDS load of four
// bytes that brings the expected sequence number from a small table in global memory into this word.  Loads of one wave
// return in the order they were issued, so the word changes only after the whole tile is in place, and the load unit
// never has to wait for a tile or come back to it: the copy completes, and announces itself, without a wave, as a
// copy engine with a completion object would do it.  The sequence number of ticket t is (t / kM2C mod kSeqRounds) + 1: never
// zero, and different from the one the same ring position carried kM2C tickets earlier.
struct M2cEnt {
    uint32_t lo;      // slot | nslots << 6 | rows << 12
    uint32_t hi;      // (ticket + 1) & 0xffff | row_bytes << 16
    uint32_t ready;   // the ticket's sequence number once the region may be used
    uint32_t rsv;
};
constexpr uint32_t kSeqRounds = 2048;   // the table in global memory holds 0 .. kSeqRounds, word i = i
static_assert(kSeqTableWords > kSeqRounds, "the table holds every sequence number");
DEV_EARLY uint32_t m2c_seq(uint32_t ticket) { return ((ticket / (uint32_t)kM2C) & (kSeqRounds - 1u)) + 1u; }

struct StatRec {  // the static part, written for all 64 uops of a window at once when it is decoded (32 bytes)
    uint32_t gp_lo, gp_hi;   // bytes between rows in global memory
    uint32_t rows_box;       // valid rows | box_rows << 16
    uint32_t rb_pitch;       // valid row_bytes | lds_pitch << 16
    uint32_t w0;             // first word of the uop: opcode, flags, vflow, vcc, acc, nslots
    uint32_t dep;            // depId | dep_count << 16
    uint32_t pc;             // stream-relative pc
    uint32_t rsv;
};

struct Ctl {
    // --- polled together by the CFU with one gathered LDS read: keep these ten words contiguous ---
    uint32_t uq_head[kMaxUnits];   // records picked up by each unit
    uint32_t mask;                 // slot availability: bit set = in use (Section 4.3: 32-bit mask in shared memory).  In the
                                   // variants built with VDC_WAVE_MASKS a slot is in use while its bit stands in this
                                   // word or in mask1: the two waves of a compute core each clear one of them when they
                                   // are done with a region (no count of the waves, no answer to wait for), whoever
                                   // else frees clears both, the front end sets both
    uint32_t abort;                // set when any unit of this core gives up
    // ---
    uint32_t cfu_halted;
    uint32_t vcc_done;             // VCC waves that reached HALT
    uint32_t uq_tail[kMaxUnits];   // records pushed to each unit
    uint32_t uq_done[kMaxUnits];   // records completed by each unit (store units)
    uint32_t stu_left;             // store units that have finished
    uint32_t rsv0[kMaxV - 1];
    uint32_t red_flag[kMaxV];      // cross-wave reduction hand-shake of a VCC
    uint32_t red_ack[kMaxV];
    uint32_t win_gen;              // number of windows the front end has decoded so far
    uint32_t mask1;                // see mask
    M2cEnt m2c[kMaxV][kM2C];       // see M2cEnt
    uint64_t c2m[kMaxV][kC2M];     // low: kind | slot << 1 | nslots << 7; high: position + 1
    UnitRec uq[kMaxUnits][kUQ];
    StatRec stat[2][kWin];         // two tables: the window being executed and the previous one
    float red[kMaxV][64];
    uint32_t arrive[kMaxV][32];    // per group of tickets: how many of a VCC's two waves are done with it (counts up, odd -> even)
#ifdef VDC_PROFILE
    uint32_t phase[16];            // profiling builds: what each wave is doing right now (see observer_main)
#endif
};
static_assert(offsetof(Ctl, mask) == offsetof(Ctl, uq_head) + 4 * kMaxUnits && offsetof(Ctl, abort) == offsetof(Ctl, mask) + 4, "poll block");
static_assert(sizeof(M2cEnt) == 16 && offsetof(Ctl, m2c) % 16 == 0 && offsetof(Ctl, c2m) % 8 == 0 && offsetof(Ctl, uq) % 16 == 0 && offsetof(Ctl, stat) % 16 == 0, "alignment");
static_assert(sizeof(UnitRec) == 4 * kRecWords && sizeof(StatRec) == 4 * kStatWords, "record size");
#define CTL_OFF(field) ((uint32_t)offsetof(Ctl, field))
#ifdef VDC_PROFILE_SECTIONS
#define SEC_BEGIN(c) ((c).w_mark = prof_now())
#define SEC_END(c, i) do { const unsigned long long t_ = prof_now(); (c).w_sec[i] += t_ - (c).w_mark; (c).w_mark = t_; } while (0)
#else
#define SEC_BEGIN(c)
#define SEC_END(c, i)
#endif
#if defined(VDC_PROFILE) && defined(VDC_PROFILE_PHASES)
#define PHASE(c, w, id) do { if ((c).lane == 0) lds_vst32((c).ctl + CTL_OFF(phase) + (w) * 4u, (id)); reconverge(); } while (0)
#define OBS(c, w, v)
#elif defined(VDC_PROFILE)
#define PHASE(c, w, id)
#define OBS(c, w, v) lds_st32_lanes(1ull, (c).ctl + CTL_OFF(phase) + (w) * 4u, (v))
#else
#define PHASE(c, w, id)
#define OBS(c, w, v)
#endif

// The build compiles this file once per variant of the executor kernel (-DVDC_PART=i: nothing but that variant, see the
// end of the file) and once for everything else (-DVDC_SPLIT), all in parallel; without either macro it is one unit.
#ifndef VDC_PART
size_t lds_control_bytes() { return (sizeof(Ctl) + 255) & ~(size_t)255; }
size_t lds_bytes_needed(uint32_t n_slots, uint32_t slot_bytes) {
    return (size_t)n_slots * slot_bytes + lds_control_bytes();
}
#endif

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
// volatile accesses to the control words: every call is one LDS instruction, never cached or merged
DEV uint32_t lds_vld32(uint32_t off) { return ((lds_vu32 *)(lds0() + off))[0]; }
DEV uint64_t lds_vld64(uint32_t off) { return ((lds_vu64 *)(lds0() + off))[0]; }
DEV void lds_vst32(uint32_t off, uint32_t v) { ((lds_vu32 *)(lds0() + off))[0] = v; }
DEV void lds_vst64(uint32_t off, uint64_t v) { ((lds_vu64 *)(lds0() + off))[0] = v; }

DEV void compiler_barrier() { asm volatile("" ::: "memory"); }
// LDS stores by a wave-uniform set of lanes without control flow: the execution mask is narrowed for the one
// instruction and restored.  A branch costs this target about as much as four scalar instructions, taken or not, and
// a per-lane "if" also makes the compiler restructure every loop around it; the hot loops therefore avoid both.
DEV void lds_st32_lanes(uint64_t lanes, uint32_t off, uint32_t v) {
    uint64_t saved;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, %1\n\tds_write_b32 %2, %3\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved) : "s"(lanes), "v"(off), "v"(v) : "memory");
}
DEV void lds_st64_lanes(uint64_t lanes, uint32_t off, uint64_t v) {
    uint64_t saved;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, %1\n\tds_write_b64 %2, %3\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved) : "s"(lanes), "v"(off), "v"(v) : "memory");
}
DEV void lds_st128_lanes(uint64_t lanes, uint32_t off, u32x4 v) {
    uint64_t saved;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, %1\n\tds_write_b128 %2, %3\n\ts_nop 0\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved) : "s"(lanes), "v"(off), "v"(v) : "memory");
}
DEV void lds_and32_lanes(uint64_t lanes, uint32_t off, uint32_t v) {
    uint64_t saved;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, %1\n\tds_and_b32 %2, %3\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved) : "s"(lanes), "v"(off), "v"(v) : "memory");
}
// The same for a 16-byte store to global memory.  The two scalar instructions behind the store are the wait states
// this target asks for between a store of more than 8 bytes and a vector instruction that overwrites its data
// registers; the compiler cannot see into the block to add them itself.
DEV void gst128_lanes(uint64_t lanes, uint64_t addr, f32x4 v) {
    uint64_t saved;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, %1\n\tglobal_store_dwordx4 %2, %3, off\n\ts_nop 0\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved) : "s"(lanes), "v"(addr), "v"(v) : "memory");
}
// The same store at device scope (sc1): it is written through, so that once it has completed (vmcnt) every compute
// unit of the device reads the new data from memory, whichever L2 it sits behind.  A store that is followed by a
// depId signal uses this form; the alternative, a release fence, writes back the whole L2 of the signalling side.
DEV void gst128_lanes_device(uint64_t lanes, uint64_t addr, f32x4 v) {
    uint64_t saved;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, %1\n\tglobal_store_dwordx4 %2, %3, off sc1\n\ts_nop 0\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved) : "s"(lanes), "v"(addr), "v"(v) : "memory");
}
// LDS atomic add by lane 0 alone; returns the value before the add, wave-uniform.
DEV uint32_t lds_add_rtn_lane0(uint32_t off, uint32_t v) {
    uint64_t saved;
    uint32_t r;
    asm volatile("s_mov_b64 %1, exec\n\ts_mov_b64 exec, 1\n\tds_add_rtn_u32 %0, %2, %3\n\ts_mov_b64 exec, %1\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(r), "=&s"(saved) : "v"(off), "v"(v) : "memory");
    return __builtin_amdgcn_readfirstlane(r);
}
DEV void lds_or32_lanes(uint64_t lanes, uint32_t off, uint32_t v) {
    uint64_t saved;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, %1\n\tds_or_b32 %2, %3\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved) : "s"(lanes), "v"(off), "v"(v) : "memory");
}
// Placed right after every "if (lane == 0) { ... }" block: an opaque statement at the point where the lanes meet
// again, so that the optimiser cannot fold that join into later joins (which would make later, wave-uniform values
// look as if they depended on the per-lane branch).
// The wave barrier is a convergent operation (so it is never cloned into the arms of the branch) and emits no code.
DEV void reconverge() { __builtin_amdgcn_wave_barrier(); }
DEV void lds_wait() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
DEV uint32_t uni(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }
DEV uint64_t uni64(uint64_t x) {
    return (uint64_t)uni((uint32_t)x) | ((uint64_t)uni((uint32_t)(x >> 32)) << 32);
}

// Program memory is read-only while a run is in flight: read it through the constant address space so that
// uniform addresses become scalar loads.
typedef const __attribute__((address_space(4))) uint32_t *cptr32;
DEV uint32_t cload(const void *p, uint32_t idx) { return uni(((cptr32)(uintptr_t)p)[idx]); }

// Indexed state (accumulators, loop stack, descriptors, the uop window, queue snapshots) is kept in "lane
// register files": a vector register whose lane i holds entry i, read with v_readlane and written with
// v_writelane under a wave-uniform index.  Nothing of a unit's register state lives in memory.
DEV uint32_t rf_get(uint32_t v, uint32_t idx) { return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)idx); }
DEV uint32_t rf_set(uint32_t v, uint32_t idx, uint32_t x) {
    x = uni(x);
    idx = uni(idx);
    // one scalar register operand per vector instruction on this target: the lane select goes through M0;
    // the nops keep the required distance between the scalar writes and the lane access
    asm("s_mov_b32 m0, %2\n\ts_nop 3\n\tv_writelane_b32 %0, %1, m0" : "+v"(v) : "s"(x), "s"(idx));
    return v;
}

struct Ctx {
    const KParams *p;
    uint32_t ctl;                     // byte offset of the control block in LDS
    uint32_t core, lane, role, unit;  // unit: LDU/STU index in the unit queues, or VCC index
    uint32_t stream_pc0;              // first word of this unit's stream
    uint32_t pc;                      // current word (for error reports)
    uint32_t spins_limit;
#ifdef VDC_PROFILE_WAITS
    unsigned long long w_wait = 0, w_spins = 0, w_vm = 0, w_t0 = 0, w_last = 0;   // profiling builds: cycles this wave spent waiting
    unsigned long long w_sec[4] = {0, 0, 0, 0}, w_mark = 0;                           // and in sections of its loop
#endif
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
        lds_vst32(c.ctl + CTL_OFF(abort), 1u);
    }
    reconverge();
}

struct Spin {
    uint32_t n = 0;
};

// One back-off step of a poll loop.  `aborted` is the core's abort word as the caller's poll saw it.  Returns
// false when the unit must give up: an error was raised somewhere, or the watchdog limit is reached, in which
// case this unit raises VDC_EDEADLOCK.
template <int NAP = 1>
DEV bool spin_step(Ctx &c, Spin &s, uint32_t aborted, uint32_t detail) {
    if (aborted) return false;
#ifdef VDC_PROFILE_WAITS
#ifdef VDC_PROFILE_WAIT_CYCLES
    {   // time between consecutive failed looks of one wait (s.n is zero at its first)
        const unsigned long long t = prof_now();
        if (s.n != 0u) c.w_wait += t - c.w_last;
        c.w_last = t;
    }
#endif
    c.w_spins++;
#endif
    __builtin_amdgcn_s_sleep(NAP);
    s.n++;
    if ((s.n & 255u) == 0u) {
        uint32_t g = uni(__hip_atomic_load(&c.p->status[ST_ABORT], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        if (g) return false;
    }
    if (s.n >= c.spins_limit) {
        raise_error(c, -5 /* VDC_EDEADLOCK */, detail);
        return false;
    }
    return true;
}

// ------------------------------------------------------------------------------------------------
// Register state of a stream: pc, loop stack, accumulators (Section 4.1 models every core as a small register machine),
// and the uop window
// ------------------------------------------------------------------------------------------------
struct Seq {
    uint32_t pc, depth, end;
    uint32_t rf_lo, rf_hi;   // lanes 0..7: accumulator i (low, high word); lanes 8..11: loop level d (body start, trips left)
    uint32_t win_base;       // the window holds words win_base .. win_base + 63 (lane l = word win_base + l)
    u32x4 win;
};

DEV void seq_refill(Ctx &c, Seq &s) {
    uint32_t idx = s.pc + c.lane;
    if (idx >= s.end) idx = s.end - 1u;     // the stream's HALT
    s.win = ((const u32x4 *)c.p->words)[idx];
    s.win_base = s.pc;
}

DEV void seq_init(Ctx &c, Seq &s, uint32_t pc, uint32_t end) {
    s.pc = pc;
    s.end = end;
    s.depth = 0;
    s.rf_lo = 0;
    s.rf_hi = 0;
    seq_refill(c, s);
}

DEV int64_t seq_acc(const Seq &s, uint32_t a) {
    return (int64_t)((uint64_t)rf_get(s.rf_lo, a) | ((uint64_t)rf_get(s.rf_hi, a) << 32));
}

DEV void seq_acc_set(Seq &s, uint32_t a, int64_t v) {
    s.rf_lo = rf_set(s.rf_lo, a, (uint32_t)(uint64_t)v);
    s.rf_hi = rf_set(s.rf_hi, a, (uint32_t)((uint64_t)v >> 32));
}

// Instruction fetch: 64 words per global load (one per lane), then v_readlane per uop.  Loop bodies of up to 64
// uops run entirely out of the window.
DEV Word fetch(Ctx &c, Seq &s) {
    uint32_t k = s.pc - s.win_base;
    if (k >= 64u) {
        seq_refill(c, s);
        k = 0;
    }
    Word w;
    w.w0 = rf_get(s.win.x, k);
    w.w1 = rf_get(s.win.y, k);
    w.w2 = rf_get(s.win.z, k);
    w.w3 = rf_get(s.win.w, k);
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
        case OP_CONTINUE_IF:
            // the loop goes on while the register is below the bound; otherwise it is left: drop its frame, go on behind
            // its REPEAT (the host checked that `size` words on is that REPEAT)
            if (seq_acc(s, f.acc) < f.imm) {
                s.pc++;
            } else {
                s.depth--;
                s.pc += f.size + 1u;
            }
            return 1;
        default:
            return 0;
    }
}

// A note that holds for every "if (lane == 0) { ... }" block in this file: a wave-uniform value that is used both
// inside such a block and after it is computed BEFORE the block.  Otherwise the optimiser may compute it once in
// each arm and merge the two copies behind the branch, and a value merged behind a divergent branch counts as
// divergent: the loops around it would then be compiled with per-lane masks instead of scalar branches.
DEV void trace_put(Ctx &c, uint32_t stream, uint32_t &count, uint32_t pc_rel, uint32_t info, uint64_t v) {
    const uint32_t next = uni(count + 1u);
    if (c.lane == 0) {
        if (count < c.p->trace_cap) {
            uint32_t *t = c.p->trace + ((size_t)stream * c.p->trace_cap + count) * 4;
            t[0] = pc_rel;
            t[1] = info;
            t[2] = (uint32_t)v;
            t[3] = (uint32_t)(v >> 32);
        }
        c.p->trace_count[stream] = next;
    }
    reconverge();
    count = next;
}

// ------------------------------------------------------------------------------------------------
// Slot allocator (Section 4.3): first fit on the bitmask, lowest position first.
// ------------------------------------------------------------------------------------------------
// `busy` has a set bit for every taken position and for every position at or beyond n_slots; everything is
// wave-uniform, so this runs on the scalar unit: f ends with bit p set iff positions p .. p + n - 1 are all free, and
// the lowest such p wins.  (The vote of 32 probing lanes that the paper describes computes the same position.)
DEV int slot_find(uint64_t busy, uint32_t n) {
    if (n == 0u) return 0;          // nothing to allocate (load.local)
    uint64_t f = ~busy;
    for (uint32_t i = 1; i < n; i++) f &= f >> 1;
    if (f == 0ull) return -1;
    return (int)__builtin_ctzll(f);
}
DEV uint64_t slots_beyond(uint32_t n_slots) { return n_slots >= 64u ? 0ull : (~0ull << n_slots); }

#ifndef VDC_PART
__global__ void debug_alloc_kernel(const uint32_t *masks, const int32_t *nslots, int32_t n_slots, int32_t *pos, int32_t n) {
    uint32_t lane = threadIdx.x & 63u;
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        int p = slot_find((uint64_t)uni(masks[i]) | slots_beyond((uint32_t)n_slots), uni((uint32_t)nslots[i]));
        if (lane == 0) pos[i] = p;
    }
}

__global__ void clear_kernel(uint32_t *p, uint32_t n) {
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}
#endif

// ------------------------------------------------------------------------------------------------
// Queue primitives
// ------------------------------------------------------------------------------------------------
DEV uint32_t slot_bits(uint32_t slot, uint32_t nslots) {
    return (nslots >= 32u ? 0xFFFFFFFFu : ((1u << nslots) - 1u)) << slot;
}

DEV void m2c_deliver(Ctx &c, uint32_t v, uint32_t ticket, uint32_t slot, uint32_t nslots, uint32_t rows, uint32_t row_bytes) {
    // payload and sequence number in one 16-byte store: a reader sees all of it or none
    const u32x4 e = {slot | (nslots << 6) | (rows << 12), ((ticket + 1u) & 0xFFFFu) | (row_bytes << 16), m2c_seq(ticket), 0u};
    lds_st128_lanes(1ull, c.ctl + CTL_OFF(m2c) + (v * kM2C + (ticket & (kM2C - 1))) * (uint32_t)sizeof(M2cEnt), e);
}

#ifdef VDC_WAVE_MASKS
// lanes 0 and 1: the two words of the slot mask
DEV uint32_t mask_words(Ctx &c) { return c.ctl + (c.lane == 1u ? CTL_OFF(mask1) : CTL_OFF(mask)); }
#endif

DEV void slots_free(Ctx &c, uint32_t slot, uint32_t nslots) {
#ifdef VDC_WAVE_MASKS
    if (c.lane < 2u) {
        __hip_atomic_fetch_and((__attribute__((address_space(3))) uint32_t *)(lds0() + mask_words(c)),
                               ~slot_bits(slot, nslots), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    reconverge();
    return;
#endif
    if (c.lane == 0) {
        __hip_atomic_fetch_and((__attribute__((address_space(3))) uint32_t *)(lds0() + c.ctl + CTL_OFF(mask)),
                               ~slot_bits(slot, nslots), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    reconverge();
}

// ------------------------------------------------------------------------------------------------
// CFU: the front end of the virtual memory core
// ------------------------------------------------------------------------------------------------
struct CfuState {
    uint32_t ticket0, ticket1;
    uint32_t uq_tail_rf;   // lane u: records pushed to unit u
    uint32_t mark_rf0;     // lane u: uq_tail[u] when the window that used stat table 0 was left
    uint32_t mark_rf1;     //         ... stat table 1
    uint32_t n_refill;
};

// One gathered read of what the front end looks at: lanes 0..7 = uq_head[0..7], lane 8 = slot mask, lane 9 = abort.
constexpr uint32_t kPollMask = kMaxUnits, kPollAbort = kMaxUnits + 1;
#ifdef VDC_WAVE_MASKS
// ... and lane 63 = the slot mask's second word, which lane 8 takes in: a slot is in use while either word says so
constexpr uint32_t kPollMask1 = 63;
DEV uint32_t cfu_poll(Ctx &c) {
    const uint32_t l = c.lane < kPollAbort ? c.lane : kPollAbort;
    const uint32_t v = lds_vld32(c.lane == kPollMask1 ? c.ctl + CTL_OFF(mask1) : c.ctl + CTL_OFF(uq_head) + l * 4u);
    return c.lane == kPollMask ? v | rf_get(v, kPollMask1) : v;
}
#else
DEV uint32_t cfu_poll(Ctx &c) {
    const uint32_t l = c.lane < kPollAbort ? c.lane : kPollAbort;
    return lds_vld32(c.ctl + CTL_OFF(uq_head) + l * 4u);
}
#endif

// The decoded uop window of the front end: lane l describes word win_base + l.  Decoding (field extraction,
// descriptor lookup, flow -> unit mapping, tensor base + literal address) is done for 64 uops at once, one per
// lane, when the window is (re)filled; executing a uop then only picks its lane with v_readlane.  The fields a
// load/store unit needs but the front end does not (row pitch, box, flags, depId) go straight from the decoding
// lane into a table in LDS; the per-execution record handed to the unit only names the table entry.
struct DecWin {
    uint32_t base;       // first word in the window
    uint32_t ctl;        // opcode [7:0] | flags [15:8] | unit [18:16] | vcc [19] | acc [22:20] | nslots [28:23] | tensor [31:29]
    uint32_t a_lo, a_hi; // memory uop: tensor base + literal offset; control uop: the immediate
    uint32_t aux;        // valid rows [15:0] | valid row_bytes [31:16]   (for the early hand-over of an output region, and the trace)
    uint32_t desc;       // descriptor index (trace only)
    // What dispatching needs of each uop, worked out for all 64 lanes when the window is decoded:
    uint32_t dynacc;     // the accumulator a memory uop's address moves with (8: none)
    uint32_t rank;       // window lanes below this one whose uop goes to the same unit
    uint32_t srank;      // window lanes below this one whose uop sends to the same compute core
    uint32_t um_lo, um_hi;   // all window lanes whose uop goes to the same unit as this one's (0: not a memory uop)
    uint32_t tm_lo, tm_hi;   // all window lanes whose uop sends to the same compute core (0: this one does not send)
    uint32_t uu_lo, uu_hi;   // in lane u: the window lanes whose uop goes to unit u
    uint32_t nsp_lo, nsp_hi; // byte j: nslots of the uop j lanes further on (j = 0..7), 0 beyond the window
    uint32_t uq_off;     // where the unit's ring of records starts in LDS
    uint32_t m2c_off;    // where the compute core's m2c ring starts
    uint32_t e_lo, e_hi; // a uop that sends: its m2c entry without slot and ticket
    uint32_t e_sel;      // all ones for a STORE that sends (its empty region is ready at once), else 0
    uint32_t info;       // the record's info word without the slot: window lane << 6 | table << 12
    uint64_t mem;        // wave-uniform: lanes that hold memory uops
    uint64_t t0, t1;     // wave-uniform: lanes whose uop sends to compute core 0 / 1
    uint64_t ones;       // wave-uniform: lanes that hold a memory uop of exactly one slot
};

// What moves while the window is executed, per lane, for the uop that lane holds.  A memory uop's effective address
// changes only when a control uop changes its accumulator; its position in its unit's ring and its m2c ticket are
// fixed as long as execution runs straight through the window (every uop passed is dispatched, so "records pushed so
// far" and "lanes passed so far" grow together), and move by a constant per lane whenever a loop jumps back: by the
// number of uops of the loop body that go to the same unit / send to the same compute core.  Keeping the three up to
// date costs a few masked vector additions per control uop; dispatching a batch then needs no gather and no
// population count per lane.
struct CfuLive {
    uint32_t g_lo, g_hi;  // effective global address if the uop were dispatched now
    uint32_t pos;         // position in the unit's ring when the pc reaches this lane in sequence
    uint32_t tick;        // m2c ticket likewise (0xffffffff and never moved: the uop does not send)
    // the last loop that jumped back inside the window: its body, and what it adds per trip
    uint32_t loop_key;    // body start lane | REPEAT lane << 8 | windows decoded so far << 16
    uint32_t dpos, dtick;
};

// The descriptor table as the front end keeps it: lane l holds the six words it needs of descriptor l (programs rarely
// have more than a handful; beyond 64 the table is read from memory as before).  It is fetched once, at the same time as
// the stream's bounds, so decoding a window costs one trip to memory (the uops) instead of two dependent ones.
struct DescRegs {
    uint32_t w[6];
    bool all;        // every descriptor of the program is in the lanes
};

DEV DescRegs desc_regs_load(Ctx &c) {
    const KParams *p = c.p;
    DescRegs r;
    const uint32_t nd = p->n_descs ? p->n_descs : 1u;
    const uint32_t *dp = (const uint32_t *)(p->descs + (c.lane < nd ? c.lane : nd - 1u));
#pragma unroll
    for (int k = 0; k < 6; k++) r.w[k] = dp[k];
    r.all = p->n_descs <= 64u;
    return r;
}

// The words of the window that starts at pc: lane l = word pc + l, the stream's HALT beyond its end.
DEV u32x4 cfu_window_words(const KParams *p, uint32_t lane, uint32_t pc, uint32_t end) {
    uint32_t idx = pc + lane;
    if (idx >= end) idx = end - 1u;             // the stream's HALT
    return ((const u32x4 *)p->words)[idx];
}

// `fetched`: the window's words if the caller has asked for them already (cfu_window_words), else null.
DEV bool cfu_refill(Ctx &c, DecWin &d, CfuLive &lv, CfuState &st, const DescRegs &dr, uint32_t acc_rf_lo, uint32_t acc_rf_hi, uint32_t pc, uint32_t end,
                    const u32x4 *fetched = nullptr) {
    const KParams *p = c.p;
    const u32x4 raw = fetched ? *fetched : cfu_window_words(p, c.lane, pc, end);
    const uint32_t idx = pc + c.lane < end ? pc + c.lane : end - 1u;    // the word this lane holds
    Word w = {raw.x, raw.y, raw.z, raw.w};
    const Fields f = decode(w);
    const bool is_mem = f.opcode == OP_LOAD || f.opcode == OP_STORE;
    const uint32_t di = (is_mem && f.desc < p->n_descs) ? f.desc : 0u;
    uint32_t d_tensor, d_box, d_rowb, d_pitch, d_gplo, d_gphi;
    if (dr.all) {
        d_tensor = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(di * 4u), (int)dr.w[0]);
        d_box = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(di * 4u), (int)dr.w[1]);
        d_rowb = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(di * 4u), (int)dr.w[2]);
        d_pitch = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(di * 4u), (int)dr.w[3]);
        d_gplo = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(di * 4u), (int)dr.w[4]);
        d_gphi = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(di * 4u), (int)dr.w[5]);
    } else {
        const uint32_t *dp = (const uint32_t *)(p->descs + di);
        d_tensor = dp[0]; d_box = dp[1]; d_rowb = dp[2]; d_pitch = dp[3]; d_gplo = dp[4]; d_gphi = dp[5];
    }
    uint64_t tbase = 0;
#pragma unroll
    for (int t = 0; t < kMaxTensors; t++) tbase = ((d_tensor & (kMaxTensors - 1)) == (uint32_t)t) ? (uint64_t)(uintptr_t)p->tensors[t] : tbase;
    // loads go to the load unit of their flow (n_ldu is 1, 2 or 4); stores, and the load.local that hands a kept
    // region on, to the store unit of their flow (n_stu is 1 or 2)
    const uint32_t unit = (f.opcode == OP_LOAD && !(f.flags & F_LOCAL)) ? (f.vflow & (p->n_ldu - 1u)) : p->n_ldu + (f.vflow & (p->n_stu - 1u));
    const uint64_t a = (uint64_t)f.imm + (is_mem ? tbase : 0ull);
    d.base = pc;
    d.ctl = f.opcode | (f.flags << 8) | (unit << 16) | ((f.vcc & 1u) << 19) | (f.acc << 20) | (f.nslots << 23) | ((d_tensor & 7u) << 29);
    d.a_lo = (uint32_t)a;
    d.a_hi = (uint32_t)(a >> 32);
    d.aux = f.size | (d_rowb << 16);
    d.desc = f.desc;
    const bool send = is_mem && (f.flags & F_SEND) != 0u;
    {
        const uint64_t lt = (1ull << c.lane) - 1ull;
        const uint32_t n_units = p->n_ldu + p->n_stu;
        uint64_t my_um = 0, uu = 0;
        for (uint32_t u = 0; u < n_units; u++) {
            const uint64_t b = __ballot(is_mem && unit == u);
            my_um = (is_mem && unit == u) ? b : my_um;
            uu = c.lane == u ? b : uu;
        }
        d.mem = uni64(__ballot(is_mem));
        d.t0 = uni64(__ballot(send && (f.vcc & 1u) == 0u));
        d.t1 = uni64(__ballot(send && (f.vcc & 1u) == 1u));
        d.ones = uni64(__ballot(is_mem && f.nslots == 1u));
        const uint64_t tm = send ? ((f.vcc & 1u) ? d.t1 : d.t0) : 0ull;
        d.um_lo = (uint32_t)my_um; d.um_hi = (uint32_t)(my_um >> 32);
        d.tm_lo = (uint32_t)tm; d.tm_hi = (uint32_t)(tm >> 32);
        d.rank = (uint32_t)__builtin_popcountll(my_um & lt);
        d.srank = (uint32_t)__builtin_popcountll(tm & lt);
        d.uu_lo = (uint32_t)uu; d.uu_hi = (uint32_t)(uu >> 32);
        uint64_t nsp = 0;
#pragma unroll
        for (uint32_t j = 0; j < 8u; j++) {
            const uint32_t o = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(((c.lane + j) & 63u) * 4u), (int)f.nslots);
            nsp |= (uint64_t)((c.lane + j < (uint32_t)kWin) ? (o & 0xFFu) : 0u) << (8u * j);
        }
        d.nsp_lo = (uint32_t)nsp; d.nsp_hi = (uint32_t)(nsp >> 32);
    }
    d.dynacc = (is_mem && (f.flags & F_DYNAMIC)) ? f.acc : 8u;
    d.uq_off = c.ctl + CTL_OFF(uq) + unit * kUQ * (uint32_t)sizeof(UnitRec);
    d.m2c_off = c.ctl + CTL_OFF(m2c) + (f.vcc & 1u) * kM2C * (uint32_t)sizeof(M2cEnt);
    d.e_sel = (send && f.opcode == OP_STORE) ? 0xFFFFFFFFu : 0u;
    d.e_lo = (f.nslots << 6) | (f.size << 12);
    d.e_hi = d_rowb << 16;
    d.info = (c.lane << 6) | ((st.n_refill & 1u) << 12);
    // the moving values, as of now: the pc stands at the window's first lane
    {
        const uint32_t acc_lo = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((f.acc & 7u) * 4u), (int)acc_rf_lo);
        const uint32_t acc_hi = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((f.acc & 7u) * 4u), (int)acc_rf_hi);
        const uint32_t tail = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(unit * 4u), (int)st.uq_tail_rf);
        const uint64_t g = a + (d.dynacc < 8u ? ((uint64_t)acc_lo | ((uint64_t)acc_hi << 32)) : 0ull);
        lv.g_lo = (uint32_t)g;
        lv.g_hi = (uint32_t)(g >> 32);
        lv.pos = tail + d.rank;
        lv.tick = send ? ((f.vcc & 1u) ? st.ticket1 : st.ticket0) + d.srank : 0xFFFFFFFFu;
        lv.loop_key = 0xFFFFFFFFu;
        lv.dpos = 0;
        lv.dtick = 0;
    }
    // The table this window writes was last used two windows ago.  Its records may still sit in a unit's queue:
    // wait until every unit has picked up everything that was dispatched from that window.
    const uint32_t t = st.n_refill & 1u;
    const uint32_t filled = st.uq_tail_rf;
    if (t == 0u) st.mark_rf1 = filled; else st.mark_rf0 = filled;     // the window being left used the other table
    const uint32_t mark = t == 0u ? st.mark_rf0 : st.mark_rf1;
    Spin sp;
    for (;;) {
        const uint32_t snap = cfu_poll(c);
        const bool behind = c.lane < (uint32_t)kMaxUnits && (int32_t)(snap - mark) < 0;
        if (__ballot(behind) == 0ull) break;
        if (!spin_step(c, sp, rf_get(snap, kPollAbort), 0x250u)) return false;
    }
    const uint32_t off = c.ctl + CTL_OFF(stat) + (t * kWin + c.lane) * (uint32_t)sizeof(StatRec);
    u32x4 s0 = {d_gplo, d_gphi, f.size | (d_box << 16), d_rowb | (d_pitch << 16)};
    u32x4 s1 = {w.w0, f.dep_id | (f.dep_count << 16), idx - c.stream_pc0, 0u};
    lds_st128(off, s0);
    lds_st128(off + 16, s1);
    compiler_barrier();
    st.n_refill = uni(st.n_refill + 1u);
    if (c.lane == 0) lds_vst32(c.ctl + CTL_OFF(win_gen), st.n_refill);   // units drop what they remember of older windows
    reconverge();
    return true;
}

DEV uint32_t lanes_below(uint64_t m, uint32_t lane) {   // how many bits of m are set below `lane`
    return (uint32_t)__builtin_popcountll(m & ((1ull << lane) - 1ull));
}

// What dispatching needs besides the window: constants of the run and the trace cursor.
struct CfuEnv {
    uint32_t n_units, stream;
    uint64_t unit_lanes, busy_hi;
    bool trace;
    uint32_t trace_n;
};

// In-order first fit for a batch of up to four uops that take at most three slots each (Section 4.3: the first free
// location, lowest position; the same function as slot_find, uop by uop, every later uop seeing the slots of the earlier
// ones as taken).  nsp32: byte j = slots of the j-th uop; lim: how many uops to try; occ32: bit set = slot taken (every
// position beyond the pool is marked taken, the pool has at most 32 slots, so 32-bit arithmetic is enough).  Stops at
// the first uop that does not fit.  Returns the number that fit; pack: byte j = first slot of the j-th; bits: all slots
// taken.  Straight-line code for the scalar unit, no branch: a branch costs this front end as much as five scalar
// instructions, taken or not, and the allocation is the busiest scalar code of the whole executor.
DEV uint32_t cfu_alloc4(uint32_t occ32, uint32_t nsp32, uint32_t lim, uint32_t &pack_out, uint32_t &bits_out) {
    static_assert(kBatch <= 4 && kMaxSlots <= 32, "the packed slot counts and positions of a batch are 32 bits here");
    uint32_t got, alloc, pack, ok, ns, f, g, h, pos, pb, b, v;
#define VDC_ALLOC_STEP(I, BFE)                                                                                  \
    "s_bfe_u32 %[ns], %[nsp], " BFE "\n\t"      /* slots of uop I */                                              \
    "s_not_b32 %[f], %[occ]\n\t"                                                                                 \
    "s_lshr_b32 %[g], %[f], 1\n\t"                                                                               \
    "s_and_b32 %[g], %[g], %[f]\n\t"            /* starts of runs of two free slots */                           \
    "s_lshr_b32 %[h], %[f], 2\n\t"                                                                               \
    "s_and_b32 %[h], %[h], %[g]\n\t"            /* of three */                                                   \
    "s_cmp_eq_u32 %[ns], 2\n\t"                                                                                  \
    "s_cselect_b32 %[f], %[g], %[f]\n\t"                                                                         \
    "s_cmp_eq_u32 %[ns], 3\n\t"                                                                                  \
    "s_cselect_b32 %[f], %[h], %[f]\n\t"                                                                         \
    "s_cmp_eq_u32 %[ns], 0\n\t"                                                                                  \
    "s_cselect_b32 %[f], 1, %[f]\n\t"           /* nothing to allocate (load.local): position 0, no bits */     \
    "s_ff1_i32_b32 %[pos], %[f]\n\t"                                                                             \
    "s_lshl_b32 %[pb], %[pos], " #I " * 8\n\t"                                                                   \
    "s_bfm_b32 %[b], %[ns], %[pos]\n\t"                                                                          \
    "s_cmp_lg_u32 %[f], 0\n\t"                                                                                   \
    "s_cselect_b32 %[v], %[ok], 0\n\t"          /* fits, and every uop before it did */                          \
    "s_cmp_gt_u32 %[lim], " #I "\n\t"                                                                            \
    "s_cselect_b32 %[ok], %[v], 0\n\t"          /* and it is one of those to try */                              \
    "s_cmp_lg_u32 %[ok], 0\n\t"                                                                                  \
    "s_cselect_b32 %[b], %[b], 0\n\t"                                                                            \
    "s_cselect_b32 %[pb], %[pb], 0\n\t"                                                                          \
    "s_or_b32 %[occ], %[occ], %[b]\n\t"                                                                          \
    "s_or_b32 %[alloc], %[alloc], %[b]\n\t"                                                                      \
    "s_or_b32 %[pack], %[pack], %[pb]\n\t"                                                                       \
    "s_add_u32 %[got], %[got], %[ok]\n\t"
    asm volatile(
        "s_mov_b32 %[got], 0\n\t"
        "s_mov_b32 %[alloc], 0\n\t"
        "s_mov_b32 %[pack], 0\n\t"
        "s_mov_b32 %[ok], 1\n\t"
        VDC_ALLOC_STEP(0, "0x20000")
        VDC_ALLOC_STEP(1, "0x20008")
        VDC_ALLOC_STEP(2, "0x20010")
        VDC_ALLOC_STEP(3, "0x20018")
        : [got] "=&s"(got), [alloc] "=&s"(alloc), [pack] "=&s"(pack), [ok] "=&s"(ok), [occ] "+s"(occ32), [ns] "=&s"(ns), [f] "=&s"(f),
          [g] "=&s"(g), [h] "=&s"(h), [pos] "=&s"(pos), [pb] "=&s"(pb), [b] "=&s"(b), [v] "=&s"(v)
        : [nsp] "s"(nsp32), [lim] "s"(lim)
        : "scc");
#undef VDC_ALLOC_STEP
    pack_out = pack;
    bits_out = alloc;
    return got;
}

// The same in-order first fit for a batch of up to six uops (the body of a replayed loop): slot counts and first slots
// of the fifth and sixth uop stand in the low bytes of a second word.
DEV uint32_t cfu_alloc6(uint32_t occ32, uint32_t nsp_lo, uint32_t nsp_hi, uint32_t lim, uint32_t &pack_lo_out, uint32_t &pack_hi_out,
                        uint32_t &bits_out) {
    static_assert(kBatchWide <= 6 && kMaxSlots <= 32, "six steps, two words of packed slot counts and positions");
    uint32_t got, alloc, pack, packh, ok, ns, f, g, h, pos, pb, b, v;
#define VDC_ALLOC_STEP(I, BYTE, BFE, NSP, PACK)                                                                  \
    "s_bfe_u32 %[ns], %[" NSP "], " BFE "\n\t"  /* slots of uop I */                                              \
    "s_not_b32 %[f], %[occ]\n\t"                                                                                 \
    "s_lshr_b32 %[g], %[f], 1\n\t"                                                                               \
    "s_and_b32 %[g], %[g], %[f]\n\t"            /* starts of runs of two free slots */                           \
    "s_lshr_b32 %[h], %[f], 2\n\t"                                                                               \
    "s_and_b32 %[h], %[h], %[g]\n\t"            /* of three */                                                   \
    "s_cmp_eq_u32 %[ns], 2\n\t"                                                                                  \
    "s_cselect_b32 %[f], %[g], %[f]\n\t"                                                                         \
    "s_cmp_eq_u32 %[ns], 3\n\t"                                                                                  \
    "s_cselect_b32 %[f], %[h], %[f]\n\t"                                                                         \
    "s_cmp_eq_u32 %[ns], 0\n\t"                                                                                  \
    "s_cselect_b32 %[f], 1, %[f]\n\t"           /* nothing to allocate: position 0, no bits */                   \
    "s_ff1_i32_b32 %[pos], %[f]\n\t"                                                                             \
    "s_lshl_b32 %[pb], %[pos], " #BYTE " * 8\n\t"                                                                \
    "s_bfm_b32 %[b], %[ns], %[pos]\n\t"                                                                          \
    "s_cmp_lg_u32 %[f], 0\n\t"                                                                                   \
    "s_cselect_b32 %[v], %[ok], 0\n\t"          /* fits, and every uop before it did */                          \
    "s_cmp_gt_u32 %[lim], " #I "\n\t"                                                                            \
    "s_cselect_b32 %[ok], %[v], 0\n\t"          /* and it is one of those to try */                              \
    "s_cmp_lg_u32 %[ok], 0\n\t"                                                                                  \
    "s_cselect_b32 %[b], %[b], 0\n\t"                                                                            \
    "s_cselect_b32 %[pb], %[pb], 0\n\t"                                                                          \
    "s_or_b32 %[occ], %[occ], %[b]\n\t"                                                                          \
    "s_or_b32 %[alloc], %[alloc], %[b]\n\t"                                                                      \
    "s_or_b32 %[" PACK "], %[" PACK "], %[pb]\n\t"                                                               \
    "s_add_u32 %[got], %[got], %[ok]\n\t"
    asm volatile(
        "s_mov_b32 %[got], 0\n\t"
        "s_mov_b32 %[alloc], 0\n\t"
        "s_mov_b32 %[pack], 0\n\t"
        "s_mov_b32 %[packh], 0\n\t"
        "s_mov_b32 %[ok], 1\n\t"
        VDC_ALLOC_STEP(0, 0, "0x20000", "nsp", "pack")
        VDC_ALLOC_STEP(1, 1, "0x20008", "nsp", "pack")
        VDC_ALLOC_STEP(2, 2, "0x20010", "nsp", "pack")
        VDC_ALLOC_STEP(3, 3, "0x20018", "nsp", "pack")
        VDC_ALLOC_STEP(4, 0, "0x20000", "nsph", "packh")
        VDC_ALLOC_STEP(5, 1, "0x20008", "nsph", "packh")
        : [got] "=&s"(got), [alloc] "=&s"(alloc), [pack] "=&s"(pack), [packh] "=&s"(packh), [ok] "=&s"(ok), [occ] "+s"(occ32), [ns] "=&s"(ns),
          [f] "=&s"(f), [g] "=&s"(g), [h] "=&s"(h), [pos] "=&s"(pos), [pb] "=&s"(pb), [b] "=&s"(b), [v] "=&s"(v)
        : [nsp] "s"(nsp_lo), [nsph] "s"(nsp_hi), [lim] "s"(lim)
        : "scc");
#undef VDC_ALLOC_STEP
    pack_lo_out = pack;
    pack_hi_out = packh;
    bits_out = alloc;
    return got;
}

// Publish n uops of the batch that starts at window lane k: mark the slots, hand the empty region of a STORE that
// sends to its compute core, write the unit records and then the new ring tails (one piece: a unit sees all or
// nothing), advance the front end's counters.  pos_pack: byte j = first slot of the j-th uop.
DEV void cfu_publish_lanes(Ctx &c, const DecWin &d, const CfuLive &lv, CfuState &st, CfuEnv &env, uint32_t pc, uint32_t k, uint32_t n,
                           uint32_t slot_vec, uint32_t alloc_bits) {
    const KParams *p = c.p;
    const uint64_t my_uu = (uint64_t)d.uu_lo | ((uint64_t)d.uu_hi << 32);
    const uint64_t bm = ((1ull << n) - 1ull) << k;
    const uint32_t add_vec = (uint32_t)__builtin_popcountll(my_uu & bm);                     // lane u: records this batch pushes to unit u
    const uint32_t new_t0 = st.ticket0 + (uint32_t)__builtin_popcountll(d.t0 & bm), new_t1 = st.ticket1 + (uint32_t)__builtin_popcountll(d.t1 & bm);
    const uint32_t new_tails = st.uq_tail_rf + add_vec;     // lane u = unit u
    if (__builtin_expect(env.trace, 0)) {
        const uint64_t my_gaddr = (uint64_t)lv.g_lo | ((uint64_t)lv.g_hi << 32);
        const bool inb = ((bm >> c.lane) & 1ull) != 0ull;
        const uint32_t tidx = env.trace_n + (c.lane - k);
        uint64_t tb = 0;
#pragma unroll
        for (int t = 0; t < kMaxTensors; t++) tb = ((d.ctl >> 29) == (uint32_t)t) ? (uint64_t)(uintptr_t)p->tensors[t] : tb;
        if (inb && tidx < p->trace_cap) {
            const uint64_t eff = my_gaddr - tb;
            u32x4 tr = {pc + (c.lane - k) - c.stream_pc0, (d.ctl & 0xFFu) | (d.desc << 8) | ((d.aux & 0xFFFFu) << 16), (uint32_t)eff, (uint32_t)(eff >> 32)};
            *(u32x4 *)(p->trace + ((size_t)env.stream * p->trace_cap + tidx) * 4) = tr;
        }
        reconverge();
        if (c.lane == 0) p->trace_count[env.stream] = env.trace_n + n;
        reconverge();
        env.trace_n += n;
    }
    // the slots are marked taken before anything that names them is published: whoever frees them later (an atomic
    // and on the same word) then always finds the bits set
#ifdef VDC_WAVE_MASKS
    lds_or32_lanes(3ull, mask_words(c), alloc_bits);
#else
    lds_or32_lanes(1ull, c.ctl + CTL_OFF(mask), alloc_bits);
#endif
    // every uop that sends: the payload of its m2c entry.  A STORE that sends: the empty output region goes to the compute
    // core at once (the entry is ready), the store unit only waits for it to return; for a LOAD the entry becomes ready
    // when the tile has landed
    const u32x4 e = {slot_vec | d.e_lo, ((lv.tick + 1u) & 0xFFFFu) | d.e_hi, m2c_seq(lv.tick) & d.e_sel, 0u};
    lds_st128_lanes((d.t0 | d.t1) & bm, d.m2c_off + (lv.tick & (kM2C - 1)) * (uint32_t)sizeof(M2cEnt), e);
    u32x4 rec = {lv.g_lo, lv.g_hi, slot_vec | d.info, lv.tick};
    lds_st128_lanes(bm, d.uq_off + (lv.pos & (kUQ - 1)) * (uint32_t)sizeof(UnitRec), rec);
    lds_st32_lanes(env.unit_lanes, c.ctl + CTL_OFF(uq_tail) + c.lane * 4u, new_tails);     // after the records
    st.uq_tail_rf = new_tails;
    st.ticket0 = new_t0;
    st.ticket1 = new_t1;
}

DEV void cfu_publish(Ctx &c, const DecWin &d, const CfuLive &lv, CfuState &st, CfuEnv &env, uint32_t pc, uint32_t k, uint32_t n,
                     uint64_t pos_pack, uint32_t alloc_bits) {
    const uint32_t slot_vec = (uint32_t)(pos_pack >> (((c.lane - k) & 7u) * 8u)) & 0xFFu;   // lane (k + j): first slot of the j-th uop
    cfu_publish_lanes(c, d, lv, st, env, pc, k, n, slot_vec, alloc_bits);
}

// First fit for n uops of one slot each, all at once: the j-th uop of the batch takes the j-th free slot from the bottom,
// which is what n first fits one after the other give (Section 4.3 lets the lanes of the unit probe the mask side by
// side; here lane l looks at slot l).  free32: bit set = slot free; n <= the number of free slots.  Lane l, if its slot
// is among the n lowest free ones, sends l to the lane of the uop that gets it (lane k + rank, rank = free slots below
// l) through the cross-lane network; every other lane sends to lane k - 1, which no uop of the batch occupies.
// Returns, in lane k + j, the slot of the j-th uop; bits: the n slots taken.
DEV uint32_t cfu_alloc_ones(Ctx &c, uint32_t free32, uint32_t n, uint32_t k, uint32_t &bits) {
    const uint32_t rank = __builtin_amdgcn_mbcnt_lo(free32, 0u);
    const bool take = c.lane < 32u && ((free32 >> (c.lane & 31u)) & 1u) != 0u && rank < n;
    bits = (uint32_t)__ballot(take);
    const uint32_t dst = take ? k + rank : (k + 63u) & 63u;
    return (uint32_t)__builtin_amdgcn_ds_permute((int)(dst * 4u), (int)c.lane);
}

// Dispatch a run of up to nmax <= kBatchOnes consecutive memory uops of one slot each, starting at window lane k: as
// many of them as there are free slots right now (at least one), provided every unit's ring has room for its share;
// when some ring has not, only the first uop, if its unit has room.  In order, lowest slots first, published in one
// piece.  Returns how many were dispatched, or 0 when the run was aborted.
DEV uint32_t cfu_dispatch_ones(Ctx &c, const DecWin &d, const CfuLive &lv, CfuState &st, CfuEnv &env, uint32_t pc, uint32_t k, uint32_t nmax,
                               uint32_t unit_k) {
    const uint64_t my_uu = (uint64_t)d.uu_lo | ((uint64_t)d.uu_hi << 32);
    const uint32_t busy32 = (uint32_t)env.busy_hi;
    Spin sp;
    PHASE(c, 0u, 3u);
    for (;;) {
        const uint32_t snap = cfu_poll(c);
        const uint32_t free32 = ~(rf_get(snap, kPollMask) | busy32);
        const uint32_t nfree = (uint32_t)__builtin_popcount(free32);
        uint32_t n = nfree < nmax ? nfree : nmax;
        const uint32_t used = st.uq_tail_rf - snap;          // lane u: records unit u has not picked up yet
        const uint32_t add = (uint32_t)__builtin_popcountll(my_uu & (((1ull << n) - 1ull) << k));
        const bool over = __ballot(c.lane < env.n_units && used + add > (uint32_t)kUQ) != 0ull;
        const bool first_full = __ballot(c.lane == unit_k && used >= (uint32_t)kUQ) != 0ull;
        n = over ? (n < 1u ? n : 1u) : n;
        n = first_full ? 0u : n;
        if (n > 0u) {
            uint32_t bits;
            const uint32_t slot_vec = cfu_alloc_ones(c, free32, n, k, bits);
            PHASE(c, 0u, 6u);
            cfu_publish_lanes(c, d, lv, st, env, pc, k, n, slot_vec, bits);
            return n;
        }
        PHASE(c, 0u, first_full ? 0u : 5u);
        if (!spin_step(c, sp, rf_get(snap, kPollAbort), 0x300u | 1u | (first_full ? 0x80u : 0u))) return 0u;
    }
}

// Dispatch the run of consecutive memory uops that starts at window lane k as one batch, lane (k + j) working on the
// j-th of them: every lane already holds its uop's effective address, ring position and ticket (CfuLive); only the
// slot allocation walks the batch in program order (in-order allocation, Section 4.3), on the scalar unit.  nmax = uops
// in the run (at most kBatch), nsp = their slot counts (a byte each), unit_k = the unit of the first.  Waits until at
// least the first uop has its slots and its unit has room; returns how many were dispatched (they are published in
// one piece), or 0 when the run was aborted.
DEV uint32_t cfu_dispatch(Ctx &c, const DecWin &d, const CfuLive &lv, CfuState &st, CfuEnv &env, uint32_t pc, uint32_t k, uint32_t nmax,
                          uint64_t nsp, uint32_t unit_k) {
    const bool small_regions = (nsp & 0xFCFCFCFCFCFCFCFCull) == 0ull;    // every uop of the batch takes at most 3 slots
    uint64_t pos_pack = 0;       // byte j: first slot of the j-th uop of the batch
    uint32_t alloc_bits = 0;
    uint32_t n = 0;
    Spin sp;
    PHASE(c, 0u, 3u);
    SEC_END(c, 3);
    for (;;) {
        const uint32_t snap = cfu_poll(c);
#ifdef VDC_PROFILE_SECTIONS
        { const uint32_t snap_ = snap; asm volatile("s_waitcnt lgkmcnt(0)" :: "v"(snap_) : "memory"); }
#endif
        SEC_END(c, 1);   // the look at the queues and the slot mask
        // room in the unit queues?  A batch adds at most kBatch records to a ring: when some ring has fewer free
        // places than that, only the batch's first uop is tried, if its unit has room at all.
        const uint32_t used = st.uq_tail_rf - snap;          // lane u: records unit u has not picked up yet
        const bool over = __ballot(c.lane < env.n_units && used > (uint32_t)(kUQ - kBatch)) != 0ull;
        const bool first_full = __ballot(c.lane == unit_k && used >= (uint32_t)kUQ) != 0ull;
        uint32_t lim = over ? 1u : nmax;
        lim = first_full ? 0u : lim;
        // slots, uop by uop in program order: first fit, lowest position (Section 4.3)
        uint64_t occ = (uint64_t)rf_get(snap, kPollMask) | env.busy_hi;
        uint32_t got = 0;
        alloc_bits = 0;
        pos_pack = 0;
        if (__builtin_expect(small_regions, 1)) {
            // the same first fit for regions of at most 3 slots as a loop that leaves at the first uop that does not
            // fit: a look that finds no room, the usual case while this path waits, costs a dozen instructions
            uint32_t sh, ns, pos, pb, bits32, pack32 = 0, f, g, occ32 = (uint32_t)occ;
            const uint32_t nsp32 = (uint32_t)nsp;
            asm volatile(
                "s_mov_b32 %[got], 0\n\t"
                "s_mov_b32 %[alloc], 0\n\t"
                "s_cmp_eq_u32 %[lim], 0\n\t"
                "s_cbranch_scc1 2f\n"
                "1:\n\t"
                "s_lshl_b32 %[sh], %[got], 3\n\t"
                "s_lshr_b32 %[ns], %[nsp], %[sh]\n\t"
                "s_and_b32 %[ns], %[ns], 3\n\t"
                "s_not_b32 %[f], %[occ]\n\t"
                "s_cmp_eq_u32 %[ns], 1\n\t"
                "s_cbranch_scc1 3f\n\t"
                "s_lshr_b32 %[g], %[f], 1\n\t"
                "s_and_b32 %[g], %[g], %[f]\n\t"
                "s_lshr_b32 %[f], %[f], 2\n\t"
                "s_and_b32 %[f], %[f], %[g]\n\t"
                "s_cmp_eq_u32 %[ns], 2\n\t"
                "s_cselect_b32 %[f], %[g], %[f]\n\t"
                "s_cmp_eq_u32 %[ns], 0\n\t"
                "s_cselect_b32 %[f], 1, %[f]\n"      // nothing to allocate (load.local): position 0, no bits
                "3:\n\t"
                "s_cmp_eq_u32 %[f], 0\n\t"
                "s_cbranch_scc1 2f\n\t"
                "s_ff1_i32_b32 %[pos], %[f]\n\t"
                "s_bfm_b32 %[b32], %[ns], %[pos]\n\t"
                "s_or_b32 %[occ], %[occ], %[b32]\n\t"
                "s_or_b32 %[alloc], %[alloc], %[b32]\n\t"
                "s_lshl_b32 %[pb], %[pos], %[sh]\n\t"
                "s_or_b32 %[pack], %[pack], %[pb]\n\t"
                "s_add_u32 %[got], %[got], 1\n\t"
                "s_cmp_lt_u32 %[got], %[lim]\n\t"
                "s_cbranch_scc1 1b\n"
                "2:"
                : [got] "=&s"(got), [alloc] "=&s"(alloc_bits), [pack] "+s"(pack32), [occ] "+s"(occ32), [sh] "=&s"(sh), [ns] "=&s"(ns),
                  [pos] "=&s"(pos), [pb] "=&s"(pb), [b32] "=&s"(bits32), [f] "=&s"(f), [g] "=&s"(g)
                : [nsp] "s"(nsp32), [lim] "s"(lim)
                : "scc");
            pos_pack = pack32;
        } else {
            for (; got < lim; got++) {
                const uint32_t ns = (uint32_t)(nsp >> (8u * got)) & 0xFFu;
                const int pos = slot_find(occ, ns);
                if (pos < 0) break;
                const uint64_t bits = ((1ull << ns) - 1ull) << (uint32_t)pos;
                occ |= bits;
                alloc_bits |= (uint32_t)bits;
                pos_pack |= (uint64_t)(uint32_t)pos << (8u * got);
            }
        }
        n = got;
        SEC_END(c, 2);   // the allocation
        if (got > 0u) break;
        PHASE(c, 0u, (first_full || over) ? 0u : ((uint32_t)__builtin_popcountll(~occ) >= ((uint32_t)nsp & 0xFFu) ? 4u : 5u));
        if (!spin_step(c, sp, rf_get(snap, kPollAbort), 0x300u | ((uint32_t)nsp & 0x3Fu) | (first_full ? 0x80u : 0u))) return 0u;
    }
    PHASE(c, 0u, 6u);
    cfu_publish(c, d, lv, st, env, pc, k, n, pos_pack, alloc_bits);
    return n;
}

// What the front end needs from memory before it can decode anything: the bounds of its stream, the first window's words
// (a second, dependent trip) and the descriptors.
struct CfuStart {
    uint32_t pc, end;
    u32x4 words;
    DescRegs dr;
};

DEV CfuStart cfu_start_fetch(Ctx &c) {
    const KParams *p = c.p;
    CfuStart f;
    f.dr = desc_regs_load(c);                     // in flight together with the stream's bounds
    const uint32_t stream = c.core * (1u + p->V);
    f.pc = cload(p->stream_begin, stream);
    f.end = cload(p->stream_begin, stream + 1u);
    f.words = cfu_window_words(p, c.lane, f.pc, f.end);
    return f;
}

DEV void cfu_main(Ctx &c, const CfuStart &start) {
    const KParams *p = c.p;
    const uint32_t n_slots = p->n_slots, n_ldu = p->n_ldu, n_units = p->n_ldu + p->n_stu;
    Seq s;
    const DescRegs dr = start.dr;
    CfuEnv env;
    env.n_units = n_units;
    env.stream = c.core * (1u + p->V);
    env.unit_lanes = (1ull << n_units) - 1ull;
    env.busy_hi = slots_beyond(n_slots);
    env.trace = p->trace != nullptr;
    env.trace_n = 0;
    s.pc = start.pc;
    s.end = start.end;
    s.depth = 0; s.rf_lo = 0; s.rf_hi = 0; s.win_base = 0; s.win = u32x4{0u, 0u, 0u, 0u};
    c.stream_pc0 = s.pc;
    CfuState st = {0, 0, 0, 0, 0, 0};
    DecWin d;
    CfuLive lv;
    bool ok = cfu_refill(c, d, lv, st, dr, s.rf_lo, s.rf_hi, s.pc, s.end, &start.words);

    // The innermost loop frame is kept in scalars (top_start, top_left); outer frames wait in lanes 8.. of the
    // register file.  Accumulators are updated by a masked vector add, so that a control uop never moves a value
    // from the vector to the scalar side and back.
    uint32_t top_start = 0, top_left = 0;
    SEC_BEGIN(c);
    while (ok) {
        c.pc = s.pc;
        PHASE(c, 0u, 1u);
        SEC_END(c, 3);       // whatever lies between two sections: the post part of a batch, loop top
        uint32_t k = s.pc - d.base;
        if (__builtin_expect(k >= (uint32_t)kWin, 0)) {
            PHASE(c, 0u, 7u);
            if (!cfu_refill(c, d, lv, st, dr, s.rf_lo, s.rf_hi, s.pc, s.end)) { ok = false; break; }
            k = 0;
        }
        const uint32_t ctlw = rf_get(d.ctl, k);
        const uint32_t opcode = ctlw & 0xFFu;
        if (opcode < (uint32_t)OP_LOAD) {
            // ---- control uops ----
            const uint32_t imm_lo = rf_get(d.a_lo, k), imm_hi = rf_get(d.a_hi, k);
            if (__builtin_expect(opcode <= (uint32_t)OP_LOOP, 0)) {
                if (opcode == (uint32_t)OP_HALT) break;
                if (s.depth > 0u) {
                    s.rf_lo = rf_set(s.rf_lo, 7u + s.depth, top_start);
                    s.rf_hi = rf_set(s.rf_hi, 7u + s.depth, top_left);
                }
                top_start = s.pc + 1u;
                top_left = imm_lo;
                s.depth++;
                s.pc++;
                continue;
            }
            const uint32_t j = (ctlw >> 20) & 7u;
            if (__builtin_expect(opcode == (uint32_t)OP_CONTINUE_IF, 0)) {
                const int64_t cur = (int64_t)((uint64_t)rf_get(s.rf_lo, j) | ((uint64_t)rf_get(s.rf_hi, j) << 32));
                const int64_t bound = (int64_t)((uint64_t)imm_lo | ((uint64_t)imm_hi << 32));
                if (cur < bound) {
                    s.pc++;
                } else {
                    // the loop is left: the uops between here and its REPEAT are skipped, not dispatched, so every lane's
                    // ring position and ticket move back by what the skipped lanes would have pushed (a jump out of the
                    // window decodes a new one and starts from the counters)
                    const uint32_t dist = rf_get(d.aux, k) & 0xFFFFu;
                    if (k + dist < (uint32_t)kWin) {
                        const uint64_t skipped = ((1ull << (k + dist + 1u)) - 1ull) & ~((1ull << (k + 1u)) - 1ull);
                        lv.pos -= (uint32_t)__builtin_popcountll(((uint64_t)d.um_lo | ((uint64_t)d.um_hi << 32)) & skipped);
                        lv.tick -= (uint32_t)__builtin_popcountll(((uint64_t)d.tm_lo | ((uint64_t)d.tm_hi << 32)) & skipped);
                    }
                    s.pc += dist + 1u;
                    s.depth--;
                    if (s.depth > 0u) {
                        top_start = rf_get(s.rf_lo, 7u + s.depth);
                        top_left = rf_get(s.rf_hi, 7u + s.depth);
                    }
                }
                continue;
            }
            // REPEAT, ADD, SET: the accumulator, and the address of every memory uop of the window that moves with it
            const uint64_t imm = (uint64_t)imm_lo | ((uint64_t)imm_hi << 32);
            const bool me = c.lane == j, mine = d.dynacc == j;
            {
                const bool set = opcode == (uint32_t)OP_SET;
                const uint64_t cur = (uint64_t)s.rf_lo | ((uint64_t)s.rf_hi << 32);
                const uint64_t nv = set ? imm : cur + imm;
                s.rf_lo = me ? (uint32_t)nv : s.rf_lo;
                s.rf_hi = me ? (uint32_t)(nv >> 32) : s.rf_hi;
                const uint64_t g = (set ? ((uint64_t)d.a_lo | ((uint64_t)d.a_hi << 32)) : ((uint64_t)lv.g_lo | ((uint64_t)lv.g_hi << 32))) + imm;
                lv.g_lo = mine ? (uint32_t)g : lv.g_lo;
                lv.g_hi = mine ? (uint32_t)(g >> 32) : lv.g_hi;
            }
            const bool rep = opcode == (uint32_t)OP_REPEAT;
            const uint32_t left = rep ? top_left - 1u : top_left;
            const bool back = rep && left > 0u;
            bool replay = false;
            uint32_t sl = 0;
            if (back) {
                // the loop jumps back: inside the window every lane's ring position and ticket move by what the body
                // dispatches to its unit / sends to its compute core (worked out once per loop); a jump out of the
                // window decodes a new one at the top of the loop above
                sl = top_start - d.base;
                if (sl <= k) {
                    const uint32_t key = sl | (k << 8) | (st.n_refill << 16);
                    if (__builtin_expect(key != lv.loop_key, 0)) {
                        const uint64_t body = (k >= 63u ? ~0ull : ((1ull << (k + 1u)) - 1ull)) & ~((1ull << sl) - 1ull);
                        lv.dpos = (uint32_t)__builtin_popcountll(((uint64_t)d.um_lo | ((uint64_t)d.um_hi << 32)) & body);
                        lv.dtick = (uint32_t)__builtin_popcountll(((uint64_t)d.tm_lo | ((uint64_t)d.tm_hi << 32)) & body);
                        lv.loop_key = key;
                    }
                    lv.pos += lv.dpos;
                    lv.tick += lv.dtick;
                    // a body that is nothing but one batch of memory uops is replayed below without decoding anything
                    const uint32_t n0 = k - sl;
                    const uint64_t body0 = (1ull << n0) - 1ull;
                    replay = n0 >= 1u && n0 <= p->issue_batch && p->no_replay == 0u && (~(d.mem >> sl) & body0) == 0ull &&
                             (n0 <= (uint32_t)kBatchWide || (n0 <= (uint32_t)kBatchOnes && (~(d.ones >> sl) & body0) == 0ull));
                }
            }
            s.pc = back ? top_start : s.pc + 1u;
            top_left = left;
            if (__builtin_expect(rep && left == 0u, 0)) {
                s.depth--;
                if (s.depth > 0u) {
                    top_start = rf_get(s.rf_lo, 7u + s.depth);
                    top_left = rf_get(s.rf_hi, 7u + s.depth);
                }
            }
            SEC_END(c, 0);   // a control uop
            if (!replay) continue;
            // ---- loop replay: the rest of the trips of a loop whose body is one batch followed by this REPEAT.  Every
            // trip is the batch and then, fused, what the REPEAT does: the accumulator and the addresses that move with
            // it advance by the immediate, positions and tickets by the body's counts.  A batch that could only be
            // dispatched in part (slots, room in a ring) ends the replay; the general path above takes over from there.
            {
                const uint32_t n0 = k - sl;
                const uint64_t nsp_r = (uint64_t)rf_get(d.nsp_lo, sl) | ((uint64_t)rf_get(d.nsp_hi, sl) << 32);
                const uint32_t nsp32 = (uint32_t)nsp_r & (n0 >= 4u ? 0xFFFFFFFFu : ((1u << (8u * n0)) - 1u));
                const bool ones = n0 >= 2u && (~(d.ones >> sl) & ((1ull << n0) - 1ull)) == 0ull;   // one slot each: the wide allocation
                const uint32_t nsp_hi32 = n0 > 4u ? (uint32_t)(nsp_r >> 32) & ((1u << (8u * (n0 - 4u))) - 1u) : 0u;   // n0 <= 6 where it is used
                const bool wide = n0 > (uint32_t)kBatch;     // five or six uops that are not all of one slot: the longer allocation
                const bool fast = (ones || (n0 <= (uint32_t)kBatchWide && ((nsp32 | nsp_hi32) & 0xFCFCFCFCu) == 0u)) && !env.trace;   // regions of at most three slots, no trace
                const uint32_t dg_lo = mine ? imm_lo : 0u, dg_hi = mine ? imm_hi : 0u;
                const uint32_t da_lo = me ? imm_lo : 0u, da_hi = me ? imm_hi : 0u;
                // what a whole batch publishes is the same on every trip
                const uint64_t bm0 = ((1ull << n0) - 1ull) << sl;
                const uint32_t add0 = (uint32_t)__builtin_popcountll(((uint64_t)d.uu_lo | ((uint64_t)d.uu_hi << 32)) & bm0);
                const uint32_t dt0 = (uint32_t)__builtin_popcountll(d.t0 & bm0), dt1 = (uint32_t)__builtin_popcountll(d.t1 & bm0);
                const uint64_t send0 = (d.t0 | d.t1) & bm0;
                const uint32_t jsh = ((c.lane - sl) & 7u) * 8u;
                const uint32_t busy32 = (uint32_t)env.busy_hi;
                const uint32_t need0 = ones ? n0 : (nsp32 & 0xFFu) + ((nsp32 >> 8) & 0xFFu) + ((nsp32 >> 16) & 0xFFu) + (nsp32 >> 24) +
                                                   (nsp_hi32 & 0xFFu) + ((nsp_hi32 >> 8) & 0xFFu);
                // lanes whose look at the queues can forbid a whole batch: a unit whose ring has no room for its share, or
                // the abort word (the lanes from kPollAbort on all read it)
#ifdef VDC_WAVE_MASKS
                const uint32_t room_need = c.lane < env.n_units ? (uint32_t)kUQ - add0 : (c.lane >= kPollAbort && c.lane != kPollMask1 ? 0u : 0xFFFFFFFFu);
#else
                const uint32_t room_need = c.lane < env.n_units ? (uint32_t)kUQ - add0 : (c.lane >= kPollAbort ? 0u : 0xFFFFFFFFu);
#endif
                bool done = false;
                // one trip without a branch but the two that end the loop: look, allocate the whole batch, publish it,
                // and do what the REPEAT does
                auto trips = [&](auto kind_tag) __attribute__((always_inline)) {
                    constexpr bool ONES = decltype(kind_tag)::value == 1, WIDE = decltype(kind_tag)::value == 2;
                    for (;;) {
                        SEC_END(c, 3);
                        const uint32_t snap = cfu_poll(c);
#ifdef VDC_PROFILE_SECTIONS
                        { const uint32_t snap_ = snap; asm volatile("s_waitcnt lgkmcnt(0)" :: "v"(snap_) : "memory"); }
#endif
                        SEC_END(c, 1);
                        // lane u: records unit u has not picked up yet; from kPollAbort on: minus the abort word
                        const uint32_t used = st.uq_tail_rf - snap;
                        const bool crowded = __ballot(used > room_need) != 0ull;
                        const uint32_t occ32 = rf_get(snap, kPollMask) | busy32;
                        // fewer free slots than the batch takes in all: nothing to try here (the general path waits)
                        if (crowded || (uint32_t)__builtin_popcount(~occ32) < need0) break;
                        uint32_t slot_vec, bits;
                        if (ONES) {
                            slot_vec = cfu_alloc_ones(c, ~occ32, n0, sl, bits);
                        } else if (WIDE) {
                            uint32_t pack_lo, pack_hi;
                            const uint32_t got = cfu_alloc6(occ32, nsp32, nsp_hi32, n0, pack_lo, pack_hi, bits);
                            const uint64_t pack64 = (uint64_t)pack_lo | ((uint64_t)pack_hi << 32);
                            if (got != n0) {
                                if (got != 0u) {
                                    cfu_publish(c, d, lv, st, env, s.pc, sl, got, pack64, bits);
                                    s.pc += got;
                                }
                                break;
                            }
                            slot_vec = (uint32_t)(pack64 >> jsh) & 0xFFu;
                        } else {
                            uint32_t pack32;
                            const uint32_t got = cfu_alloc4(occ32, nsp32, n0, pack32, bits);
                            if (got != n0) {
                                // not all of it fits right now: publish what did and let the general path wait for the rest
                                if (got != 0u) {
                                    cfu_publish(c, d, lv, st, env, s.pc, sl, got, pack32, bits);
                                    s.pc += got;
                                }
                                break;
                            }
                            slot_vec = (pack32 >> jsh) & 0xFFu;
                        }
                        SEC_END(c, 2);
#ifdef VDC_WAVE_MASKS
                        lds_or32_lanes(3ull, mask_words(c), bits);
#else
                        lds_or32_lanes(1ull, c.ctl + CTL_OFF(mask), bits);
#endif
                        const u32x4 e = {slot_vec | d.e_lo, ((lv.tick + 1u) & 0xFFFFu) | d.e_hi, m2c_seq(lv.tick) & d.e_sel, 0u};
                        lds_st128_lanes(send0, d.m2c_off + (lv.tick & (kM2C - 1)) * (uint32_t)sizeof(M2cEnt), e);
                        u32x4 rec = {lv.g_lo, lv.g_hi, slot_vec | d.info, lv.tick};
                        lds_st128_lanes(bm0, d.uq_off + (lv.pos & (kUQ - 1)) * (uint32_t)sizeof(UnitRec), rec);
                        st.uq_tail_rf += add0;
                        lds_st32_lanes(env.unit_lanes, c.ctl + CTL_OFF(uq_tail) + c.lane * 4u, st.uq_tail_rf);     // after the records
                        st.ticket0 += dt0;
                        st.ticket1 += dt1;
                        // the REPEAT
                        const uint64_t a2 = ((uint64_t)s.rf_lo | ((uint64_t)s.rf_hi << 32)) + ((uint64_t)da_lo | ((uint64_t)da_hi << 32));
                        s.rf_lo = (uint32_t)a2; s.rf_hi = (uint32_t)(a2 >> 32);
                        const uint64_t g2 = ((uint64_t)lv.g_lo | ((uint64_t)lv.g_hi << 32)) + ((uint64_t)dg_lo | ((uint64_t)dg_hi << 32));
                        lv.g_lo = (uint32_t)g2; lv.g_hi = (uint32_t)(g2 >> 32);
                        top_left--;
                        if (top_left == 0u) { done = true; break; }
                        lv.pos += lv.dpos;
                        lv.tick += lv.dtick;
                    }
                };
                if (fast) {
                    if (ones) trips(std::integral_constant<int, 1>{});
                    else if (wide) trips(std::integral_constant<int, 2>{});
                    else trips(std::integral_constant<int, 0>{});
                }
                if (done) {
                    s.pc = top_start + n0 + 1u;          // past the REPEAT: the loop is done
                    s.depth--;
                    if (s.depth > 0u) {
                        top_start = rf_get(s.rf_lo, 7u + s.depth);
                        top_left = rf_get(s.rf_hi, 7u + s.depth);
                    }
                }
            }
            continue;
        }
        // ---- memory uops: the run of consecutive memory uops that starts here is one batch ----
        PHASE(c, 0u, 2u);
        const uint64_t not_mem = ~(d.mem >> k);                 // bit j clear = word k + j is a memory uop
        uint32_t nmax = (uint32_t)__builtin_ctzll(not_mem | (1ull << 63));
        nmax = nmax > (uint32_t)kBatch ? (uint32_t)kBatch : nmax;
        nmax = nmax > (uint32_t)kWin - k ? (uint32_t)kWin - k : nmax;
        nmax = nmax > p->issue_batch ? p->issue_batch : nmax;
        nmax = nmax < 1u ? 1u : nmax;
        // a run of uops of one slot each goes the wide way
        uint32_t run1 = (uint32_t)__builtin_ctzll(~(d.ones >> k) | (1ull << 63));
        run1 = run1 > (uint32_t)kBatchOnes ? (uint32_t)kBatchOnes : run1;
        run1 = run1 > (uint32_t)kWin - k ? (uint32_t)kWin - k : run1;
        run1 = run1 > p->issue_batch ? p->issue_batch : run1;
        if (run1 >= 2u) {
            const uint32_t n1 = cfu_dispatch_ones(c, d, lv, st, env, s.pc, k, run1, (ctlw >> 16) & 7u);
            if (n1 == 0u) { ok = false; break; }
            s.pc += n1;
            continue;
        }
        const uint64_t nsp = (uint64_t)rf_get(d.nsp_lo, k) | ((uint64_t)rf_get(d.nsp_hi, k) << 32);   // slot counts of the batch
        const uint32_t n = cfu_dispatch(c, d, lv, st, env, s.pc, k, nmax, nsp, (ctlw >> 16) & 7u);
        if (n == 0u) { ok = false; break; }
        s.pc += n;
    }

    // HALT (or error): no more dispatches.  The store unit goes on receiving c2m; wait until every unit is done with
    // what it was given.
    if (c.lane == 0) lds_vst32(c.ctl + CTL_OFF(cfu_halted), 1u);
    reconverge();
    Spin sp;
    while (ok) {
        const uint32_t snap = cfu_poll(c);
        bool done = true;
        for (uint32_t u = 0; u < n_ldu; u++) done = done && (rf_get(snap, u) == rf_get(st.uq_tail_rf, u));
        for (uint32_t u = n_ldu; u < n_units; u++)
            done = done && (uni(lds_vld32(c.ctl + CTL_OFF(uq_done) + u * 4u)) == rf_get(st.uq_tail_rf, u));
        if (done) break;
        if (!spin_step(c, sp, rf_get(snap, kPollAbort), 0x400u)) ok = false;
    }
}

// ------------------------------------------------------------------------------------------------
// LDU: tile loads, global -> LDS, without going through registers
// ------------------------------------------------------------------------------------------------
DEV void load_lds_b128(uint32_t lds_addr_wave, const char *gptr, bool nt, bool device) {
    // LDS address = M0 + lane * 16 (wave-uniform base in M0, one 16-byte chunk per active lane)
    lds_addr_wave = uni(lds_addr_wave);
    if (device)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off sc1" ::"s"(lds_addr_wave), "v"(gptr) : "memory");
    else if (nt)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(lds_addr_wave), "v"(gptr) : "memory");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr_wave), "v"(gptr) : "memory");
}

// Is the dependency there?  One relaxed look at the counter.
DEV bool dep_ready(Ctx &c, uint32_t dep) {
    uint32_t id = dep & 0xFFFFu, need = (dep >> 16) & 0xFFu;
    if (need == 0u) need = 1u;
    return uni(__hip_atomic_load(&c.p->dep[id], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) >= need;
}

// Wait for it.  The counter is polled relaxed.  `acquire`: once it is there, one acquire at device scope (an invalidate
// of this side's caches), for a load that reads through the caches; a load at device scope does not need it.
DEV bool dep_wait(Ctx &c, uint32_t dep, bool acquire) {
    Spin s;
    for (;;) {
        if (dep_ready(c, dep)) {
            if (acquire) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            return true;
        }
        if (!spin_step(c, s, uni(lds_vld32(c.ctl + CTL_OFF(abort))), 0x500u | (dep & 0xFFFFu))) return false;
    }
}

// `written_through`: the data the signal covers was stored at device scope and has completed, so the counter needs no
// release semantics of its own; otherwise the increment is a release at device scope (an L2 write-back).
DEV void dep_signal(Ctx &c, uint32_t dep, bool written_through) {
    if (c.lane == 0) {
        if (written_through) __hip_atomic_fetch_add(&c.p->dep[dep & 0xFFFFu], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else __hip_atomic_fetch_add(&c.p->dep[dep & 0xFFFFu], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
    reconverge();
}

// The static part of a record: lanes 0..7 = the StatRec the record's info word points at.
DEV uint32_t stat_fetch(Ctx &c, uint32_t info) {
    const uint32_t base = c.ctl + CTL_OFF(stat) + (((info >> 12) & 1u) * kWin + ((info >> 6) & 63u)) * (uint32_t)sizeof(StatRec);
    return lds_vld32(base + (c.lane & 7u) * 4u);
}

// Everything about a LOAD that does not change from one execution to the next, derived once from its static record
// and kept for the two uops a unit saw last (a loop body alternates between very few).
struct LduEnt {
    uint32_t key;               // table | window lane, 0xffffffff = empty
    uint32_t val;               // the static record itself: lanes 0..7
    uint32_t ni;                // load instructions per tile
    uint32_t bits;              // 1 NT | 2 SEND | 4 DEP_SEND | 8 DEP_RECV | 16 fast path | 32 DEVICE | lanes of a last, partial instruction << 8 | chunks of zeros behind the run << 14
    uint32_t step_lo, step_hi;  // fast path: address step per load instruction
    uint32_t m2c_ready;         // LDS byte offset of the ready word of entry 0 of the compute core's m2c ring
    uint32_t off_lo, off_hi;    // fast path, per lane: offset of the lane's first chunk from the tile address
};

DEV void ldu_derive(Ctx &c, LduEnt &e, uint32_t key, uint32_t info) {
    e.key = key;
    e.val = stat_fetch(c, info);
    const uint64_t gpitch = (uint64_t)rf_get(e.val, 0) | ((uint64_t)rf_get(e.val, 1) << 32);
    const uint32_t rows_box = rf_get(e.val, 2), rb_pitch = rf_get(e.val, 3), w0 = rf_get(e.val, 4);
    const uint32_t rows = rows_box & 0xFFFFu, box_rows = rows_box >> 16, row_bytes = rb_pitch & 0xFFFFu, lds_pitch = rb_pitch >> 16;
    const uint32_t cpr = lds_pitch >> 4, vcr = row_bytes >> 4, total = box_rows * cpr;
    const uint32_t flags = (w0 >> 8) & 0xFFu, vcc = (w0 >> 20) & 3u;
    e.ni = (total + 63u) >> 6;
    const bool pow2 = (cpr & (cpr - 1u)) == 0u && cpr <= 64u;
    // a box whose rows follow each other without a gap, in memory as in the region, is one run of `total` chunks whatever
    // its row length: 64 chunks per instruction, and a last instruction of `tail` lanes
    // (a box with fewer valid rows than it has: the valid rows are the run, the rest of the box is filled with zeros)
    const bool contig = gpitch == (uint64_t)lds_pitch && row_bytes == lds_pitch && rows <= box_rows && total - rows * cpr < 2048u;
    const uint32_t run = rows * cpr, tail = contig ? (run & 63u) : 0u, zeros = contig ? total - run : 0u;
    const bool fast = (pow2 && rows == box_rows && vcr == cpr && (total & 63u) == 0u) || contig;
    if (contig) e.ni = (run + 63u) >> 6;
    e.bits = ((flags & F_NT) ? 1u : 0u) | ((flags & F_SEND) ? 2u : 0u) | ((flags & F_DEP_SEND) ? 4u : 0u) |
             ((flags & F_DEP_RECV) ? 8u : 0u) | (fast ? 16u : 0u) | ((flags & F_DEVICE) ? 32u : 0u) | (tail << 8) | (zeros << 14);
    uint32_t sh = 0, drow = 0;
    if (pow2) { sh = __builtin_ctz(cpr); drow = 64u >> sh; }
    const uint64_t step = contig ? 1024ull : (uint64_t)drow * gpitch;
    e.step_lo = (uint32_t)step;
    e.step_hi = (uint32_t)(step >> 32);
    e.m2c_ready = c.ctl + CTL_OFF(m2c) + vcc * kM2C * (uint32_t)sizeof(M2cEnt) + (uint32_t)offsetof(M2cEnt, ready);
    const uint64_t off = contig ? (uint64_t)c.lane * 16u : (uint64_t)(c.lane >> sh) * gpitch + (uint64_t)(c.lane & (cpr - 1u)) * 16u;
    e.off_lo = (uint32_t)off;
    e.off_hi = (uint32_t)(off >> 32);
}

// A load unit pops its ring in order, issues the direct-to-LDS loads of the tile and, behind them, the four-byte load
// that makes the tile's m2c entry ready when everything before it has landed (see M2cEnt).  It never waits for a tile:
// as many tiles are in flight as there are slots for them, and a tile is delivered the moment it is complete.
DEV void ldu_main(Ctx &c) {
    const uint32_t u = c.unit;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds0();
    const uint32_t slot_shift = __builtin_ctz(c.p->slot_bytes);
    const uint64_t seq_table = (uint64_t)(uintptr_t)c.p->seq_table;
    uint32_t head = 0;
    // an upper bound of the wave's outstanding load instructions (the hardware counter holds 63)
    uint32_t vm_bound = 0;
    // Keys are (table, window lane); both entries are dropped whenever the front end has decoded a new window,
    // which the poll sees in the same snapshot as any record dispatched from it.  `cur` is the entry of the uop
    // the unit handled last, with its wave-uniform fields in scalar registers.
    LduEnt e0 = {}, e1 = {}, cur = {};
    e0.key = e1.key = cur.key = 0xFFFFFFFFu;
    uint32_t seen_gen = 0;
    // what the poll reads: lane 0 = uq_tail[u], lanes 1..4 = the record at `head`, lane 5 = cfu_halted,
    // lane 6 = abort, lane 7.. = win_gen
    uint32_t poll_off = c.ctl + CTL_OFF(win_gen);
    poll_off = c.lane == 6u ? c.ctl + CTL_OFF(abort) : poll_off;
    poll_off = c.lane == 5u ? c.ctl + CTL_OFF(cfu_halted) : poll_off;
    poll_off = c.lane <= 4u ? c.ctl + CTL_OFF(uq) + u * kUQ * (uint32_t)sizeof(UnitRec) + (c.lane - 1u) * 4u : poll_off;
    poll_off = c.lane == 0u ? c.ctl + CTL_OFF(uq_tail) + u * 4u : poll_off;
    const uint32_t poll_rec = (c.lane >= 1u && c.lane <= 4u) ? (uint32_t)sizeof(UnitRec) : 0u;
    Spin sp;
    bool ok = true;
    SEC_BEGIN(c);
    while (ok) {
        PHASE(c, 1u + u, 1u);
        SEC_END(c, 3);
        const uint32_t snap = lds_vld32(poll_off + poll_rec * (head & (kUQ - 1)));
#ifdef VDC_PROFILE_SECTIONS
        { const uint32_t snap_ = snap; asm volatile("s_waitcnt lgkmcnt(0)" :: "v"(snap_) : "memory"); }
#endif
        SEC_END(c, 0);
        if (rf_get(snap, 0) == head) {
            // nothing to do
            if (rf_get(snap, 5) && uni(lds_vld32(c.ctl + CTL_OFF(uq_tail) + u * 4u)) == head) break;
            PHASE(c, 1u + u, 5u);
            if (!spin_step(c, sp, rf_get(snap, 6), 0x600u | u)) ok = false;
            continue;
        }
        const uint32_t gen = rf_get(snap, 7);
        if (__builtin_expect(gen != seen_gen, 0)) {
            seen_gen = gen;
            e0.key = e1.key = cur.key = 0xFFFFFFFFu;
        }
        const uint32_t info = rf_get(snap, 3);
        const uint32_t key = (info >> 6) & 0x7Fu;
        if (key != cur.key) {
            if (((key >> 2) ^ key) & 1u) {   // two entries: loop bodies alternate between lanes 1, 2 or 4 apart
                if (e1.key != key) ldu_derive(c, e1, key, info);
                cur = e1;
            } else {
                if (e0.key != key) ldu_derive(c, e0, key, info);
                cur = e0;
            }
            cur.ni = uni(cur.ni); cur.bits = uni(cur.bits); cur.key = uni(cur.key);
            cur.step_lo = uni(cur.step_lo); cur.step_hi = uni(cur.step_hi); cur.m2c_ready = uni(cur.m2c_ready);
        }
        SEC_END(c, 1);
        // ---- issue the loads of the record ----
        PHASE(c, 1u + u, 2u);
        const uint32_t ni = cur.ni, val = cur.val, bits = cur.bits;
        const uint64_t gaddr = (uint64_t)rf_get(snap, 1) | ((uint64_t)rf_get(snap, 2) << 32);
        const uint32_t ticket = rf_get(snap, 4), slot = info & 63u, lds_off = slot << slot_shift;
        if (__builtin_expect((bits & 8u) != 0u, 0)) {
            // an unresolved dependency blocks this unit, and only this unit (Section 4.3); what it has in flight
            // completes by itself meanwhile.  A dependency that is already there costs one look at its counter.
            c.pc = c.stream_pc0 + rf_get(val, 6);
            if (!dep_wait(c, rf_get(val, 5), (bits & 32u) == 0u)) { ok = false; break; }
        }
        // the counter of outstanding loads must not run over: make room first when this tile might
        if (__builtin_expect(vm_bound + ni + 1u > 60u, 0)) {
            if (ni + 1u > 44u) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); vm_bound = 0; }
            else { asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); vm_bound = 16; }
        }
        SEC_END(c, 2);
        if ((bits & 0xFFFFFF10u) == 0x10u) {
            // the usual case: whole tile, a power-of-two row of at most 64 chunks (or any gap-free run of whole
            // instructions).  Every instruction moves 64 / cpr whole rows, so the per-lane address just advances by a
            // uniform step
            const uint64_t off = (uint64_t)cur.off_lo | ((uint64_t)cur.off_hi << 32);
            const uint64_t step = (uint64_t)cur.step_lo | ((uint64_t)cur.step_hi << 32);
            uint32_t dst = lds_base + lds_off;
            // Four instructions per trip, straight-line: back to back they issue about four times faster than one per
            // loop trip (a taken branch costs about as much as one of these loads)
#define VDC_LOAD4(NT)                                                                                              \
    asm volatile("s_mov_b32 m0, %[dst]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[g], off" NT "\n\t"                   \
                 "s_add_u32 m0, m0, 0x400\n\tv_lshl_add_u64 %[g], %[g], 0, %[step]\n\tglobal_load_lds_dwordx4 %[g], off" NT "\n\t" \
                 "s_add_u32 m0, m0, 0x400\n\tv_lshl_add_u64 %[g], %[g], 0, %[step]\n\tglobal_load_lds_dwordx4 %[g], off" NT "\n\t" \
                 "s_add_u32 m0, m0, 0x400\n\tv_lshl_add_u64 %[g], %[g], 0, %[step]\n\tglobal_load_lds_dwordx4 %[g], off" NT "\n\t" \
                 "v_lshl_add_u64 %[g], %[g], 0, %[step]"                                                           \
                 : [g] "+v"(ga) : [dst] "s"(dst), [step] "s"(step) : "memory", "scc")
#define VDC_LOAD_TILE(NT)                                                                                          \
    for (; i + 4u <= ni; i += 4u) {                                                                                \
        VDC_LOAD4(NT);                                                                                             \
        dst += 4096u;                                                                                              \
        if (__builtin_expect((i & 31u) == 28u && i + 4u < ni, 0)) asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); \
    }                                                                                                              \
    for (; i < ni; i++) {                                                                                          \
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" NT ::"s"(dst), "v"(ga) : "memory"); \
        dst += 1024u;                                                                                              \
        ga += step;                                                                                                \
    }
            uint64_t ga = gaddr + off;
            uint32_t i = 0;
            if (bits & 32u) {
                // device scope: the tile may have been written by another core during this run
                VDC_LOAD_TILE(" sc1")
            } else if (bits & 1u) {
                VDC_LOAD_TILE(" nt")
            } else {
                VDC_LOAD_TILE("")
            }
#undef VDC_LOAD_TILE
#undef VDC_LOAD4
        } else if (bits & 16u) {
            // a gap-free run that ends inside an instruction (a query row, a few partial rows, the last tile of a context),
            // and the rows of the box that the tensor does not have: those read as zero
            const uint32_t tail = (bits >> 8) & 63u, zeros = bits >> 14, nfull = tail ? ni - 1u : ni;
            const bool nt = (bits & 1u) != 0u, device = (bits & 32u) != 0u;
            uint64_t ga = gaddr + ((uint64_t)cur.off_lo | ((uint64_t)cur.off_hi << 32));
            uint32_t dst = lds_base + lds_off;
            for (uint32_t i = 0; i < nfull; i++) {
                load_lds_b128(dst, (const char *)(uintptr_t)ga, nt, device);
                dst += 1024u;
                ga += 1024u;
                if ((i & 31u) == 31u && i + 1u < ni) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
            }
            if (tail != 0u) {
                if (c.lane < tail) load_lds_b128(dst, (const char *)(uintptr_t)ga, nt, device);
                reconverge();
            }
            if (zeros != 0u) {
                // ordinary LDS writes of this wave: in place before the completing load is issued
                const uint32_t z0 = lds_off + (nfull * 64u + tail) * 16u;
                const u32x4 z = {0u, 0u, 0u, 0u};
                for (uint32_t i = c.lane; i < zeros; i += 64u) lds_st128(z0 + i * 16u, z);
                lds_wait();
            }
        } else {
            const uint64_t gpitch = (uint64_t)rf_get(val, 0) | ((uint64_t)rf_get(val, 1) << 32);
            const uint32_t rows_box = rf_get(val, 2), rb_pitch = rf_get(val, 3);
            const uint32_t rows = rows_box & 0xFFFFu, box_rows = rows_box >> 16;
            const uint32_t cpr = (rb_pitch >> 16) >> 4;          // 16-byte chunks per row of the box
            const uint32_t vcr = (rb_pitch & 0xFFFFu) >> 4;      // valid chunks per row
            const uint32_t total = box_rows * cpr;
            const bool nt = (bits & 1u) != 0u;
            uint32_t row = c.lane / cpr, col = c.lane % cpr;
            const uint32_t drow = 64u / cpr, dcol = 64u % cpr;
            for (uint32_t i = 0; i < ni; i++) {
                const uint32_t q = i * 64u + c.lane;
                const char *g = (const char *)(uintptr_t)(gaddr + (uint64_t)row * gpitch + (uint64_t)col * 16u);
                const uint32_t dst = lds_base + lds_off + i * 1024u;
                const bool inside = q < total;
                const bool valid = inside && row < rows && col < vcr;
                if (valid) load_lds_b128(dst, g, nt, (bits & 32u) != 0u);
                if (inside && !valid) {
                    u32x4 z = {0u, 0u, 0u, 0u};
                    lds_st128(lds_off + q * 16u, z);             // the box outside the valid tile reads as zero
                }
                row += drow;
                col += dcol;
                if (col >= cpr) { col -= cpr; row++; }
                if ((i & 31u) == 31u && i + 1u < ni) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
            }
            // the zero fill is an ordinary LDS write of this wave: it must be in place before the completing load is
            // even issued
            lds_wait();
        }
        vm_bound += ni + 1u;
        PHASE(c, 1u + u, 6u);
        if (__builtin_expect((bits & 4u) != 0u, 0)) {
            // A load that signals does so once its data has landed and before it delivers: once the tile is delivered the
            // compute core may finish and the core may leave, and the core that leaves last puts the counters back to
            // zero; no signal may come after that.
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            vm_bound = 0;
            dep_signal(c, rf_get(val, 5), false);
        }
        // the completing load: the entry's sequence number, fetched behind the tile
        {
            const uint32_t rdst = lds_base + cur.m2c_ready + (ticket & (kM2C - 1)) * (uint32_t)sizeof(M2cEnt);
            const uint64_t fa = seq_table + (uint64_t)m2c_seq(ticket) * 4u;
            const uint64_t lanes = (bits & 2u) ? 1ull : 0ull;
            uint64_t saved;
            asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, %1\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %3, off\n\ts_mov_b64 exec, %0"
                         : "=&s"(saved) : "s"(lanes), "s"(rdst), "v"(fa) : "memory");
        }
        head++;
        OBS(c, 1u + u, head);
        lds_st32_lanes(1ull, c.ctl + CTL_OFF(uq_head) + u * 4u, head);
        sp.n = 0;
    }
    // never leave with loads in flight: their LDS destination belongs to this workgroup only while it lives
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// ------------------------------------------------------------------------------------------------
// STU: receiver of the c2m queues, and produced region -> global memory
// ------------------------------------------------------------------------------------------------
// lanes 0,1 = next c2m entry of the unit's first VCC `ring0` (low, high), lanes 2,3 = of VCC 1 (looked at only by a unit
// that serves both), lane 4 = uq_tail[u], lanes 5..8 = the record at `head`, lane 9 = cfu_halted, lane 10 = abort,
// lane 11 = vcc_done, lane 12 = slot mask, lane 13 = win_gen
// Each lane's offset is a fixed part plus its share of the three positions that move (the record at `head`, the next
// message of each c2m queue): worked out once, three multiply-adds per look.
struct StuPoll {
    uint32_t base, k_rec, k_e0, k_e1;   // per lane: fixed offset, and bytes per step of head / c2m_head0 / c2m_head1
};
DEV StuPoll stu_poll_init(Ctx &c, uint32_t u, uint32_t ring0) {
    StuPoll p;
    const uint32_t e0 = c.ctl + CTL_OFF(c2m) + ring0 * kC2M * 8u, e1 = c.ctl + CTL_OFF(c2m) + kC2M * 8u;
    const uint32_t rec = c.ctl + CTL_OFF(uq) + u * kUQ * (uint32_t)sizeof(UnitRec);
    uint32_t off = c.ctl + CTL_OFF(mask);
    off = c.lane == 13u ? c.ctl + CTL_OFF(win_gen) : off;
    off = c.lane == 11u ? c.ctl + CTL_OFF(vcc_done) : off;
    off = c.lane == 10u ? c.ctl + CTL_OFF(abort) : off;
    off = c.lane == 9u ? c.ctl + CTL_OFF(cfu_halted) : off;
    off = c.lane <= 8u ? rec + (c.lane - 5u) * 4u : off;
    off = c.lane == 4u ? c.ctl + CTL_OFF(uq_tail) + u * 4u : off;
    off = c.lane < 4u ? e1 + (c.lane - 2u) * 4u : off;
    off = c.lane < 2u ? e0 + c.lane * 4u : off;
    p.base = off;
    p.k_rec = (c.lane >= 5u && c.lane <= 8u) ? (uint32_t)sizeof(UnitRec) : 0u;
    p.k_e0 = c.lane < 2u ? 8u : 0u;
    p.k_e1 = (c.lane >= 2u && c.lane < 4u) ? 8u : 0u;
    return p;
}
DEV uint32_t stu_poll(const StuPoll &p, uint32_t head, uint32_t c2m_head0, uint32_t c2m_head1) {
    return lds_vld32(p.base + p.k_rec * (head & (kUQ - 1)) + p.k_e0 * (c2m_head0 & (kC2M - 1)) + p.k_e1 * (c2m_head1 & (kC2M - 1)));
}

// Take the next message of one c2m queue out of the snapshot: a used region goes back to the pool (Section 4.3:
// "recycled"), a produced region is kept for the STORE that waits for it ("written back").
DEV bool stu_receive(Ctx &c, uint32_t lo, uint32_t hi, uint32_t &c2m_head, uint32_t &box_rf, uint32_t &box_tail) {
    if (hi != c2m_head + 1u) return false;
    c2m_head++;
    const uint32_t slot = (lo >> 1) & 63u, nslots = (lo >> 7) & 63u;
    if ((lo & 1u) == 0u) {
        slots_free(c, slot, nslots);
    } else {
        box_rf = rf_set(box_rf, box_tail & (kMbox - 1), slot | (nslots << 6));
        box_tail++;
    }
    return true;
}

DEV void stu_main(Ctx &c) {
    const uint32_t u = c.unit;
    const uint32_t V = c.p->V;
    // One store unit receives the c2m queues of all compute cores; two take one compute core each (unit i: VCC i), and
    // a STORE or a local uop must then sit on the unit of its compute core.
    const bool split = c.p->n_stu == 2u;
    const uint32_t ring0 = split ? u - c.p->n_ldu : 0u, n_rings = split ? 1u : V;
    const uint32_t slot_shift = __builtin_ctz(c.p->slot_bytes);
    uint32_t head = 0, done = 0;
    uint32_t c2m_head0 = 0, c2m_head1 = 0;
    uint32_t box_rf0 = 0, box_rf1 = 0;              // produced regions waiting for their STORE: lane (i & 31) = entry i
    uint32_t box_head0 = 0, box_tail0 = 0, box_head1 = 0, box_tail1 = 0;
    bool have = false;                              // a STORE has been picked up and is waiting
    uint32_t r_glo = 0, r_ghi = 0, r_info = 0, r_ticket = 0, stat = 0;
    uint32_t park_rf = 0, park_head = 0, park_tail = 0;   // regions a store.local took back, waiting for their load.local
    // What the unit remembers of the STOREs it has seen, by window lane mod 8 (a loop body alternates between few): lane k =
    // the key (table | window lane) of entry k, the first word of its uop, and whether it is a plain store of one gap-free
    // run of 16-byte chunks (bit 31) with the chunk count.  Dropped when the front end has decoded a new window.
    uint32_t ck_rf = 0xFFFFFFFFu, cw_rf = 0, ci_rf = 0, seen_gen = 0;
    const StuPoll poll = stu_poll_init(c, u, ring0);
    const uint32_t pub_off = c.ctl + (c.lane == 0u ? CTL_OFF(uq_head) : CTL_OFF(uq_done)) + u * 4u;
    Spin sp;
    bool ok = true;
    SEC_BEGIN(c);
    while (ok) {
        PHASE(c, 1u + u, 1u);
        SEC_END(c, 3);
        // the c2m queues carry produced regions only (a compute core frees a used region itself, see vcc_done_with):
        // the poll brings the next entry of each along
        uint32_t snap;
        // ---- The usual STORE, one look each: nothing is held, the next record is a plain store of one gap-free run of
        // 16-byte chunks whose region is the next message of its compute core.  What the unit knows of the uop comes from
        // its register files; every condition is folded into one flag and one branch (a branch costs this target as much
        // as four or five other instructions, taken or not); no second trip to local memory for the static record, no
        // parking of the region, nothing per lane but the run's own reads and writes.
        for (;;) {
            snap = stu_poll(poll, head, c2m_head0, c2m_head1);
            if ((uint32_t)have | (uint32_t)(rf_get(snap, 4) == head)) break;      // an idle look stays short
            const uint32_t info = rf_get(snap, 7), key = (info >> 6) & 0x7Fu, k = key & 7u;
            const uint32_t ci = rf_get(ci_rf, k), w0 = rf_get(cw_rf, k);
            const uint32_t vi = ((w0 >> 20) & 3u) - ring0, vs = vi < n_rings ? vi : 0u;
            const uint32_t lo = rf_get(snap, vs * 2u), hi = rf_get(snap, vs * 2u + 1u), r_lo = rf_get(snap, 5);
            const uint32_t ch = vs == 0u ? c2m_head0 : c2m_head1;
            const uint32_t slot = info & 63u, nslots = (w0 >> 25) & 63u;
            const uint32_t boxed = vs == 0u ? box_head0 ^ box_tail0 : box_head1 ^ box_tail1;   // regions the general path holds go first
            const uint32_t stop = (rf_get(snap, 13) ^ seen_gen) | (rf_get(ck_rf, k) ^ key) |
                                  (~ci >> 31) | (uint32_t)(vi >= n_rings) | (r_lo & 15u) | boxed | (hi ^ (ch + 1u)) |
                                  (lo ^ (1u | (slot << 1) | (nslots << 7))) | rf_get(snap, 10);
            if (stop != 0u) break;
#ifdef VDC_PROFILE_WAITS
            c.w_wait++;
#endif
            const uint64_t gaddr = (uint64_t)r_lo | ((uint64_t)rf_get(snap, 6) << 32);
            const uint32_t total = ci & 0xFFFFu, lds_off = slot << slot_shift;
            head++;
            done++;
            c2m_head0 += vs == 0u ? 1u : 0u;
            c2m_head1 += vs == 0u ? 0u : 1u;
            uint32_t i0 = 0;
            do {
                f32x4 v[4];
                uint64_t on[4];
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const uint32_t i = i0 + (uint32_t)q * 64u + c.lane;
                    const bool in = i < total;
                    on[q] = __ballot(in);
                    v[q] = lds_ld128(lds_off + (in ? i : 0u) * 16u);
                }
#pragma unroll
                for (int q = 0; q < 4; q++) gst128_lanes(on[q], gaddr + (uint64_t)(i0 + (uint32_t)q * 64u + c.lane) * 16u, v[q]);
                i0 += 256u;
            } while (i0 < total);
            // the data is in registers on its way out: the region is free as soon as the reads have returned
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#ifdef VDC_WAVE_MASKS
            lds_and32_lanes(3ull, mask_words(c), ~slot_bits(slot, nslots));
#else
            lds_and32_lanes(1ull, c.ctl + CTL_OFF(mask), ~slot_bits(slot, nslots));
#endif
            lds_st32_lanes(3ull, pub_off, c.lane == 0u ? head : done);         // the record's place in the ring is free, the STORE is done
            sp.n = 0;
        }
        PHASE(c, 1u + u, 2u);
#ifdef VDC_PROFILE_SECTIONS
        { const uint32_t snap_ = snap; asm volatile("s_waitcnt lgkmcnt(0)" :: "v"(snap_) : "memory"); }
#endif
        SEC_END(c, 0);
        // Why the loop above stopped, where that is for this unit to mend: a new window (what is remembered is dropped), a
        // uop seen for the first time (its static record is read, once), a region that is still with the compute core
        // (wait for it here).  Everything else (other kinds of STORE, local uops, nothing to do, leaving) is the
        // general path's, below.
        if (!have && rf_get(snap, 4) != head) {
            const uint32_t gen = rf_get(snap, 13);
            const bool new_window = gen != seen_gen;
            if (__builtin_expect(new_window, 0)) { seen_gen = gen; ck_rf = 0xFFFFFFFFu; }
            const uint32_t info = rf_get(snap, 7), key = (info >> 6) & 0x7Fu, k = key & 7u;
            if (__builtin_expect(rf_get(ck_rf, k) != key, 0)) {
                const uint32_t sr = stat_fetch(c, info);
                const uint32_t gp_lo = rf_get(sr, 0), gp_hi = rf_get(sr, 1), rows = rf_get(sr, 2) & 0xFFFFu, rb_pitch = rf_get(sr, 3), w0s = rf_get(sr, 4);
                const uint32_t rb = rb_pitch & 0xFFFFu, lp = rb_pitch >> 16, fl = (w0s >> 8) & 0xFFu;
                const bool plain = (w0s & 0xFFu) == (uint32_t)OP_STORE && (fl & ~(uint32_t)(F_SEND | F_DYNAMIC | F_NT)) == (uint32_t)F_RECV;
                const bool run = (rb & 15u) == 0u && rb != 0u && (rows == 1u || (gp_hi == 0u && gp_lo == rb && lp == rb));
                const uint32_t chunks = rows * (rb >> 4);
                ck_rf = rf_set(ck_rf, k, key);
                cw_rf = rf_set(cw_rf, k, w0s);
                ci_rf = rf_set(ci_rf, k, (plain && run && chunks != 0u && chunks < 0x10000u ? 0x80000000u : 0u) | (chunks & 0xFFFFu));
                continue;
            }
            const uint32_t ci = rf_get(ci_rf, k), w0 = rf_get(cw_rf, k);
            const uint32_t vi = ((w0 >> 20) & 3u) - ring0;
            if ((ci >> 31) != 0u && vi < n_rings && (rf_get(snap, 5) & 15u) == 0u && (vi == 0u ? box_head0 == box_tail0 : box_head1 == box_tail1)) {
                if (new_window) continue;
                // (a message that is there and is not the region this STORE names is the general path's to report)
                const uint32_t ch = vi == 0u ? c2m_head0 : c2m_head1;
                if (rf_get(snap, vi * 2u + 1u) != ch + 1u) {
                    // wait for that one message and look at nothing else meanwhile: a short look, so that the compute wave
                    // on this SIMD keeps its issue slots
                    PHASE(c, 1u + u, 6u);
                    const uint32_t e_hi = c.ctl + CTL_OFF(c2m) + ((ring0 + vi) * kC2M + (ch & (kC2M - 1))) * 8u + 4u;
                    const uint32_t w_off = c.lane == 0u ? e_hi : c.ctl + CTL_OFF(abort);
                    for (;;) {
                        const uint32_t two = lds_vld32(w_off);
                        if (rf_get(two, 0) == ch + 1u) break;
                        if (!spin_step(c, sp, rf_get(two, 1), 0x780u)) { ok = false; break; }
                    }
                    continue;
                }
            }
        }
        bool moved = stu_receive(c, rf_get(snap, 0), rf_get(snap, 1), c2m_head0, box_rf0, box_tail0);
        if (n_rings > 1u) moved = stu_receive(c, rf_get(snap, 2), rf_get(snap, 3), c2m_head1, box_rf1, box_tail1) || moved;
        if (moved) OBS(c, 5u, c2m_head0 | (c2m_head1 << 16));
        if (!have && rf_get(snap, 4) != head) {
            // pick the next STORE up: from here on its queue entry and its static record may be reused
            PHASE(c, 1u + u, 3u);
            r_glo = rf_get(snap, 5); r_ghi = rf_get(snap, 6); r_info = rf_get(snap, 7); r_ticket = rf_get(snap, 8);
            stat = stat_fetch(c, r_info);
            stat = stat + 0u;
            lds_wait();
            head++;
            lds_st32_lanes(1ull, c.ctl + CTL_OFF(uq_head) + u * 4u, head);
            have = true;
            moved = true;
        }
        SEC_END(c, 1);
        if (have) {
            const uint32_t w0 = rf_get(stat, 4), dep = rf_get(stat, 5);
            const uint32_t flags = (w0 >> 8) & 0xFFu, vcc = (w0 >> 20) & 3u, nslots = (w0 >> 25) & 63u;
            const uint32_t slot = r_info & 63u;
            c.pc = c.stream_pc0 + rf_get(stat, 6);
            bool ready = true;
            const uint32_t vi = vcc - ring0;        // which of this unit's c2m queues
            if ((flags & F_RECV) && vi >= n_rings) {
                // the region would come back on a queue another store unit receives
                raise_error(c, -3 /* VDC_EPROGRAM */, 0x990u | vcc);
                ok = false;
                break;
            }
            if ((flags & F_LOCAL) && (w0 & 0xFFu) == (uint32_t)OP_LOAD) {
                // load.local: the oldest kept region goes to the compute core as a delivered tile
                if (park_head == park_tail) {
                    raise_error(c, -3 /* VDC_EPROGRAM */, 0x980u);
                    ok = false;
                    break;
                }
                const uint32_t got = rf_get(park_rf, park_head & (kMbox - 1));
                park_head++;
                const uint32_t rows = rf_get(stat, 2) & 0xFFFFu, row_bytes = rf_get(stat, 3) & 0xFFFFu;
                m2c_deliver(c, vcc, r_ticket, got & 63u, (got >> 6) & 63u, rows, row_bytes);
                done++;
                lds_st32_lanes(1ull, c.ctl + CTL_OFF(uq_done) + u * 4u, done);
                have = false;
                sp.n = 0;
                continue;
            }
            if (flags & F_DEP_RECV) {
                uint32_t need = (dep >> 16) & 0xFFu;
                if (need == 0u) need = 1u;
                ready = uni(__hip_atomic_load(&c.p->dep[dep & 0xFFFFu], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) >= need;   // the store reads nothing from memory: order alone is needed
            }
            if (ready && (flags & F_RECV)) {
                // wait for the compute core to hand the region back as "produced"
                const uint32_t bh = vi == 0u ? box_head0 : box_head1, bt = vi == 0u ? box_tail0 : box_tail1;
                ready = bh != bt;
                if (ready) {
                    const uint32_t got = rf_get(vi == 0u ? box_rf0 : box_rf1, bh & (kMbox - 1));
                    if (got != (slot | (nslots << 6))) {
                        raise_error(c, -3 /* VDC_EPROGRAM */, 0x900u | got);
                        ok = false;
                        break;
                    }
                    if (vi == 0u) box_head0++; else box_head1++;
                }
            }
            if (ready && (flags & F_LOCAL)) {
                // store.local: nothing is written and nothing is freed; the region waits for its load.local
                park_rf = rf_set(park_rf, park_tail & (kMbox - 1), slot | (nslots << 6));
                park_tail++;
                done++;
                lds_st32_lanes(1ull, c.ctl + CTL_OFF(uq_done) + u * 4u, done);
                have = false;
                moved = true;
            } else if (ready) {
                const uint64_t gaddr = (uint64_t)r_glo | ((uint64_t)r_ghi << 32);
                const uint64_t gpitch = (uint64_t)rf_get(stat, 0) | ((uint64_t)rf_get(stat, 1) << 32);
                const uint32_t rows = rf_get(stat, 2) & 0xFFFFu, rb_pitch = rf_get(stat, 3);
                const uint32_t row_words = (rb_pitch & 0xFFFFu) >> 2, lds_pitch = rb_pitch >> 16;
                const uint32_t lds_off = slot << slot_shift;
                compiler_barrier();
                PHASE(c, 1u + u, 4u);
                SEC_END(c, 2);
                bool through = false;            // stored at device scope (only the 16-byte path does that)
                if (((r_glo | (uint32_t)gpitch | rb_pitch | (rb_pitch >> 16)) & 15u) == 0u) {
                    // whole 16-byte chunks: lane l takes chunks l, l + 64, ... of the box, four at a time.  The lane's
                    // offsets into the region and into memory advance by uniform steps (plus a uniform correction when
                    // the column wraps into the next row): no multiplication or division per chunk, and no branch
                    const uint32_t cpr = (rb_pitch & 0xFFFFu) >> 4, total = rows * cpr;
                    uint32_t rr, cc, dr, dc;
                    if ((cpr & (cpr - 1u)) == 0u) {
                        const uint32_t sh = (uint32_t)__builtin_ctz(cpr);
                        rr = c.lane >> sh; cc = c.lane & (cpr - 1u);
                        dr = 64u >> sh; dc = 64u & (cpr - 1u);
                    } else {
                        rr = c.lane / cpr; cc = c.lane - rr * cpr;
                        dr = 64u / cpr; dc = 64u - dr * cpr;
                    }
                    const uint32_t l_step = dr * lds_pitch + dc * 16u, l_wrap = lds_pitch - cpr * 16u;
                    const uint64_t g_step = (uint64_t)dr * gpitch + (uint64_t)dc * 16u, g_wrap = gpitch - (uint64_t)cpr * 16u;
                    uint32_t loff = lds_off + rr * lds_pitch + cc * 16u;
                    uint64_t goff = gaddr + (uint64_t)rr * gpitch + (uint64_t)cc * 16u;
                    for (uint32_t i0 = 0; i0 < total; i0 += 256u) {
                        f32x4 v[4];
                        uint64_t ga[4];
                        uint64_t on[4];
#pragma unroll
                        for (int q = 0; q < 4; q++) {
                            const bool in = i0 + (uint32_t)q * 64u + c.lane < total;
                            on[q] = __ballot(in);
                            ga[q] = goff;
                            v[q] = lds_ld128(in ? loff : lds_off);
                            cc += dc;
                            const bool wrap = cc >= cpr;
                            cc -= wrap ? cpr : 0u;
                            loff += l_step + (wrap ? l_wrap : 0u);
                            goff += g_step + (wrap ? g_wrap : 0ull);
                        }
                        if (flags & (F_DEP_SEND | F_DEVICE)) {
#pragma unroll
                            for (int q = 0; q < 4; q++) gst128_lanes_device(on[q], ga[q], v[q]);
                        } else {
#pragma unroll
                            for (int q = 0; q < 4; q++) gst128_lanes(on[q], ga[q], v[q]);
                        }
                    }
                    through = true;
                } else {
                    const uint32_t total = rows * row_words;
                    for (uint32_t i = c.lane; i < total; i += 64u) {
                        uint32_t rr = i / row_words, cc = i % row_words;
                        float v = lds_ldf(lds_off + rr * lds_pitch + cc * 4u);
                        *(float *)(uintptr_t)(gaddr + (uint64_t)rr * gpitch + (uint64_t)cc * 4u) = v;
                    }
                }
                // the data is in registers on its way out: the region is free as soon as the reads have returned
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                slots_free(c, slot, nslots);
                if (flags & F_DEP_SEND) {
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    if (!through) __threadfence();
                    dep_signal(c, dep, through);
                }
                done++;
                lds_st32_lanes(1ull, c.ctl + CTL_OFF(uq_done) + u * 4u, done);
                have = false;
                moved = true;
            }
        }
        if (moved) {
            sp.n = 0;
            continue;
        }
        // nothing to do right now.  The store units leave last: the front end has halted, every STORE is written, the
        // compute cores are done and the unit's c2m queues are empty.
        if (!have && rf_get(snap, 9) && rf_get(snap, 11) == 2u * V && uni(lds_vld32(c.ctl + CTL_OFF(uq_tail) + u * 4u)) == head) {
            const uint32_t last = stu_poll(poll, head, c2m_head0, c2m_head1);
            const bool more = rf_get(last, 1) == c2m_head0 + 1u || (n_rings > 1u && rf_get(last, 3) == c2m_head1 + 1u);
            if (!more) break;
            continue;
        }
        PHASE(c, 1u + u, have ? 6u : 5u);
        if (!have && sp.n >= kStuIdleAfter) {
            if (!spin_step<kStuIdleNap>(c, sp, rf_get(snap, 10), 0x700u)) ok = false;
        } else if (!spin_step(c, sp, rf_get(snap, 10), 0x700u | (have ? 0x80u : 0u))) ok = false;
    }
    // The store unit that leaves last is the last of its core to touch a slot or a depId counter (every signal and every
    // wait of the core lies before the last region comes back).
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    if (lds_add_rtn_lane0(c.ctl + CTL_OFF(stu_left), 1u) + 1u != c.p->n_stu) return;
    // After a run that came to its end every slot must be free again.
    if (ok) {
#ifdef VDC_WAVE_MASKS
        const uint32_t mask = uni(lds_vld32(c.ctl + CTL_OFF(mask))) | uni(lds_vld32(c.ctl + CTL_OFF(mask1)));
#else
        const uint32_t mask = uni(lds_vld32(c.ctl + CTL_OFF(mask)));
#endif
        if (mask != 0u) raise_error(c, -6 /* VDC_ELEAK */, mask);
    }
    // The core that leaves last, of all cores, puts the counters the program used back to zero for the next run: no
    // clearing launch between runs, also after a run that was aborted.
    if (c.p->n_dep_used != 0u) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        uint32_t before = 0;
        if (c.lane == 0) before = __hip_atomic_fetch_add(c.p->finished, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        reconverge();
        before = uni(before);
        if (before == gridDim.x - 1u) {
            for (uint32_t i = c.lane; i < c.p->n_dep_used; i += 64u)
                __hip_atomic_store(&c.p->dep[i], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (c.lane == 0) __hip_atomic_store(c.p->finished, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            reconverge();
        }
    }
}

// ------------------------------------------------------------------------------------------------
// VCC: compute uop handlers
// ------------------------------------------------------------------------------------------------
// The two waves of an execution unit pop the same tickets, in the same groups.  A region may go back to the memory
// core only when both are done with it: each wave counts itself in on the group's arrival word, and the one that
// arrives second hands the group's regions back at once.
struct VccState {
    uint32_t head;     // next m2c ticket to pop
    uint32_t group;    // groups of tickets finished so far
    uint32_t c2m_pos;  // produced regions pushed to c2m so far (both waves count alike)
    uint32_t pay0, pay1;   // kind | slot << 1 | nslots << 7 of the tickets popped last
    uint32_t red_seq;  // cross-wave reductions done so far
    uint32_t wv;       // which of the two waves of the execution unit this is
    uint32_t t;        // thread index inside the execution unit, 0..127
};

struct Msg {
    uint32_t slot, nslots, rows, row_bytes;
};

// lanes 0..3 = m2c entry of ticket head (payload low, high, ready word, unused), lanes 4..7 = of ticket head + 1,
// lane 8 = abort
constexpr uint32_t kVccPollAbort = 8;
DEV uint32_t vcc_poll(Ctx &c, uint32_t head) {
    const uint32_t v = c.unit;
    const uint32_t e0 = c.ctl + CTL_OFF(m2c) + (v * kM2C + (head & (kM2C - 1))) * (uint32_t)sizeof(M2cEnt);
    const uint32_t e1 = c.ctl + CTL_OFF(m2c) + (v * kM2C + ((head + 1u) & (kM2C - 1))) * (uint32_t)sizeof(M2cEnt);
    uint32_t off = c.ctl + CTL_OFF(abort);
    off = c.lane < 8u ? e1 + (c.lane - 4u) * 4u : off;
    off = c.lane < 4u ? e0 + c.lane * 4u : off;
    return lds_vld32(off);
}

DEV bool msg_ready(uint32_t snap, uint32_t which, uint32_t ticket, Msg &m) {
    const uint32_t lo = rf_get(snap, which * 4u), hi = rf_get(snap, which * 4u + 1u);
    if (rf_get(snap, which * 4u + 2u) != m2c_seq(ticket)) return false;
    m.slot = lo & 63u;
    m.nslots = (lo >> 6) & 63u;
    m.rows = lo >> 12;
    m.row_bytes = hi >> 16;
    return true;
}

// pop_wait of the listing for `n` (1 or 2) consecutive tickets.  `kind` is what the regions will be pushed back
// as (0 = used, 1 = produced).  While it waits, the first wave keeps returning finished regions.
DEV bool vcc_pop_wait(Ctx &c, VccState &vs, uint32_t n, uint32_t kind, Msg &m0, Msg &m1) {
    Spin s;
    PHASE(c, 6u + c.unit * 2u + vs.wv, 1u);
    for (;;) {
        const uint32_t snap = vcc_poll(c, vs.head);
        const bool r0 = msg_ready(snap, 0, vs.head, m0);
        const bool r1 = n < 2u || msg_ready(snap, 1, vs.head + 1u, m1);
        if (r0 && r1) {
            vs.pay0 = kind | (m0.slot << 1) | (m0.nslots << 7);
            vs.pay1 = kind | (m1.slot << 1) | (m1.nslots << 7);
            compiler_barrier();
            PHASE(c, 6u + c.unit * 2u + vs.wv, 2u);
            OBS(c, 6u + c.unit * 2u + vs.wv, vs.head + n);
            return true;
        }
        if (!spin_step(c, s, rf_get(snap, kVccPollAbort), 0x100u | c.unit)) return false;
    }
}

// Called after the wave has finished reading (or writing) the regions of its last `n` (1 or 2) tickets: c2m.push,
// by whichever of the two waves gets here second.  For a used region the message to the memory core is nothing but
// "these slots are free again", so it is delivered as the LDS atomic that clears the slots' bits in the availability
// mask; a produced region goes through the c2m ring to the store unit, which has a STORE waiting for it.
DEV void vcc_done_with(Ctx &c, VccState &vs, uint32_t n, uint32_t kind) {
    compiler_barrier();
    const uint32_t v = c.unit;
#ifdef VDC_WAVE_MASKS
    if (kind == 0u) {
        // each wave clears its own word of the mask: nothing to wait for, and no count of the waves
        const uint32_t payload = c.lane == 0u ? vs.pay0 : vs.pay1;     // lane j < n: ticket head + j
        lds_and32_lanes((1ull << n) - 1ull, c.ctl + (vs.wv == 1u ? CTL_OFF(mask1) : CTL_OFF(mask)), ~slot_bits((payload >> 1) & 63u, (payload >> 7) & 63u));
        vs.head += n;
        vs.group++;
        compiler_barrier();
        return;
    }
#endif
    const uint32_t before = lds_add_rtn_lane0(c.ctl + CTL_OFF(arrive) + (v * 32u + (vs.group & 31u)) * 4u, 1u);
    if (before & 1u) {
        OBS(c, 10u + v, vs.head + n);
        const uint32_t payload = c.lane == 0u ? vs.pay0 : vs.pay1;     // lane j < n: ticket head + j
        if (kind == 0u) {
            lds_and32_lanes((1ull << n) - 1ull, c.ctl + CTL_OFF(mask), ~slot_bits((payload >> 1) & 63u, (payload >> 7) & 63u));
        } else {
            const uint32_t pos = vs.c2m_pos + c.lane;
            lds_st64_lanes((1ull << n) - 1ull, c.ctl + CTL_OFF(c2m) + (v * kC2M + (pos & (kC2M - 1))) * 8u,
                           (uint64_t)payload | ((uint64_t)(pos + 1u) << 32));
        }
    }
    if (kind != 0u) vs.c2m_pos += n;
    vs.head += n;
    vs.group++;
    compiler_barrier();
}

// A region that was popped earlier and kept (its ticket already counted in vs.head) goes back as used: the same
// arrival protocol as vcc_done_with, with the payload the caller saved at the pop.
DEV void vcc_return_kept(Ctx &c, VccState &vs, uint32_t payload) {
    compiler_barrier();
    const uint32_t v = c.unit;
#ifdef VDC_WAVE_MASKS
    (void)v;
    lds_and32_lanes(1ull, c.ctl + (vs.wv == 1u ? CTL_OFF(mask1) : CTL_OFF(mask)), ~slot_bits((payload >> 1) & 63u, (payload >> 7) & 63u));
    vs.group++;
    compiler_barrier();
    return;
#endif
    const uint32_t before = lds_add_rtn_lane0(c.ctl + CTL_OFF(arrive) + (v * 32u + (vs.group & 31u)) * 4u, 1u);
    if (before & 1u) lds_and32_lanes(1ull, c.ctl + CTL_OFF(mask), ~slot_bits((payload >> 1) & 63u, (payload >> 7) & 63u));
    vs.group++;
    compiler_barrier();
}

// A produced region that was popped earlier and kept (its ticket already counted in vs.head) goes to the store unit: the
// arrival protocol of vcc_done_with, with the payload the caller saved at the pop.
DEV void vcc_push_kept(Ctx &c, VccState &vs, uint32_t payload) {
    compiler_barrier();
    const uint32_t v = c.unit;
    const uint32_t before = lds_add_rtn_lane0(c.ctl + CTL_OFF(arrive) + (v * 32u + (vs.group & 31u)) * 4u, 1u);
    const uint32_t pos = vs.c2m_pos;
    if (before & 1u)
        lds_st64_lanes(1ull, c.ctl + CTL_OFF(c2m) + (v * kC2M + (pos & (kC2M - 1))) * 8u, (uint64_t)payload | ((uint64_t)(pos + 1u) << 32));
    vs.c2m_pos = pos + 1u;
    vs.group++;
    compiler_barrier();
}

// Cross-lane reductions of the compute uops without a trip through the LDS crossbar: data-parallel-primitive (DPP)
// operands move values inside a row of 16 lanes (and from the last lane of a row into the next rows), v_readlane takes
// one value per row of 16 to the scalar side.
template <int CTRL>
DEV float dpp_f32(float x) {   // x as seen through the DPP control CTRL (all rows, all banks)
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}
template <int CTRL, int BANKS>
DEV float dpp_f32_banks(float x, float other) {   // lanes of the quads in BANKS see x through CTRL, the rest see `other`
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, other), __builtin_bit_cast(int, x), CTRL, 0xF, BANKS, false));
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E;            // quad_perm [1,0,3,2], [2,3,0,1]
constexpr int kDppRor4 = 0x124, kDppRor8 = 0x128;          // row_ror:4, row_ror:8
constexpr int kDppShl4 = 0x104, kDppShr4 = 0x114;          // row_shl:4, row_shr:4
constexpr int kDppBcast15 = 0x142, kDppBcast31 = 0x143;    // lane 15 of every row -> the next row; lane 31 -> rows 2 and 3

// Sum of x over each group of `lpr` consecutive lanes (lpr = 1, 2, 4, ..., 64, wave-uniform); the LAST lane of every
// group holds the sum afterwards (for lpr <= 16 every lane does).  Steps that do not apply add zero: no branches.
DEV float lane_group_sum(float x, uint32_t lpr) {
    const float a1 = dpp_f32<kDppXor1>(x);
    x += lpr >= 2u ? a1 : 0.0f;
    const float a2 = dpp_f32<kDppXor2>(x);
    x += lpr >= 4u ? a2 : 0.0f;
    const float a4x = dpp_f32_banks<kDppShl4, 0x5>(x, 0.0f) + dpp_f32_banks<kDppShr4, 0xA>(x, 0.0f);   // lane ^ 4
    const float a4r = dpp_f32<kDppRor4>(x);
    x += lpr == 8u ? a4x : (lpr >= 16u ? a4r : 0.0f);
    const float a8 = dpp_f32<kDppRor8>(x);
    x += lpr >= 16u ? a8 : 0.0f;
    const float a16 = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), kDppBcast15, 0xA, 0xF, false));
    x += lpr >= 32u ? a16 : 0.0f;
    const float a32 = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), kDppBcast31, 0xC, 0xF, false));
    x += lpr >= 64u ? a32 : 0.0f;
    return x;
}


// The same sum for a group size known when the code is compiled: one DPP step per level and nothing else.
template <int LPR>
DEV float lane_group_sum_fixed(float x) {
    if (LPR >= 2) x += dpp_f32<kDppXor1>(x);
    if (LPR >= 4) x += dpp_f32<kDppXor2>(x);
    if (LPR == 8) x += dpp_f32_banks<kDppShl4, 0x5>(x, 0.0f) + dpp_f32_banks<kDppShr4, 0xA>(x, 0.0f);   // lane ^ 4
    if (LPR >= 16) x += dpp_f32<kDppRor4>(x);
    if (LPR >= 16) x += dpp_f32<kDppRor8>(x);
    if (LPR >= 32) x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), kDppBcast15, 0xA, 0xF, false));
    if (LPR >= 64) x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), kDppBcast31, 0xC, 0xF, false));
    return x;
}

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
// xspan >= 2 (B = 1, J = 0): one vector tile of xspan rows serves xspan consecutive steps, row j step j.  It is popped
// before the first matrix tile of those steps, kept while they pass, and handed back after the last (the same
// out-of-order return as the query tile of attn): half the memory uops per step for the front end.
template <int B, int NF, int J, bool SPANS = false>
DEV bool matvec_uop(Ctx &c, VccState &vs, uint32_t size, uint32_t R, uint32_t lpr, uint32_t xspan) {
    static_assert(!SPANS || J == 0, "a vector tile over several steps: rows inside a wave");
    const KParams *p = c.p;
    const uint32_t v = c.unit;
    const uint32_t slot_shift = __builtin_ctz(p->slot_bytes);
    constexpr int JJ = (J == 0) ? 1 : J;
    constexpr int NACC = NF / JJ;
    float acc[NACC][B];                      // the uop's register accumulators, kept over all its tile steps
#pragma unroll
    for (int i = 0; i < NACC; i++)
#pragma unroll
        for (int b = 0; b < B; b++) acc[i][b] = 0.0f;
    const uint32_t t = vs.t;
    const uint32_t c4 = (J == 0) ? (t & (lpr - 1u)) : t;
    const uint32_t pitch = lpr * 16u;
    // a vector tile over several steps with several vectors: B rows of xspan pieces side by side
    const uint32_t xpitch = (SPANS && B > 1) ? xspan * pitch : pitch;

    constexpr bool spans = SPANS;
    uint32_t x_pay = 0, x_base = 0, xs = 0;      // the vector tile that is held, and the step inside it
    for (uint32_t it = 0; it < size; it++) {
        Msg ma, mb;
        uint32_t b_off;
        if (spans) {
            if (xs == 0u) {
                if (it != 0u) vcc_return_kept(c, vs, x_pay);
                if (!vcc_pop_wait(c, vs, 1u, 0u, mb, ma)) return false;
                x_pay = vs.pay0;
                vs.head += 1u;                   // popped; handed back after its last step
                x_base = mb.slot << slot_shift;
            }
            if (!vcc_pop_wait(c, vs, 1u, 0u, ma, mb)) return false;
            b_off = x_base + xs * pitch;
            xs = xs + 1u == xspan ? 0u : xs + 1u;
        } else {
            if (!vcc_pop_wait(c, vs, 2u, 0u, ma, mb)) return false;  // wait for the step's matrix tile and vector tile
            b_off = mb.slot << slot_shift;
        }
        const uint32_t a_off = ma.slot << slot_shift;
        f32x4 xv[JJ][B];
#pragma unroll
        for (int j = 0; j < JJ; j++)
#pragma unroll
            for (int b = 0; b < B; b++) xv[j][b] = lds_ld128(b_off + (uint32_t)b * xpitch + ((uint32_t)j * 128u + c4) * 16u);
        f32x4 m[NF];
#pragma unroll
        for (int i = 0; i < NF; i++) m[i] = lds_ld128(a_off + ((uint32_t)i * 128u + t) * 16u);
#pragma unroll
        for (int i = 0; i < NF; i++) {
            const int ai = (J == 0) ? i : i / JJ;
            const int xi = (J == 0) ? 0 : i % JJ;
#pragma unroll
            for (int b = 0; b < B; b++) acc[ai][b] = dot4(m[i], xv[xi][b], acc[ai][b]);   // the step's partial products
        }
        // every LDS read of both tiles has returned once its value was used: the regions can go back
        vcc_done_with(c, vs, spans ? 1u : 2u, 0u);                   // both regions go back to the memory core as used
    }
    if (spans) vcc_return_kept(c, vs, x_pay);

    Msg mo, unused;
    if (!vcc_pop_wait(c, vs, 1u, 1u, mo, unused)) return false;      // wait for the output region
    const uint32_t o_off = mo.slot << slot_shift;
    if (J == 0) {
        const uint32_t lsh = __builtin_ctz(lpr);
        const uint32_t rpp = 128u >> lsh;
#pragma unroll
        for (int i = 0; i < NF; i++)
#pragma unroll
            for (int b = 0; b < B; b++) {
                const float x = lane_group_sum(acc[i][b], lpr);
                if (c4 == lpr - 1u) lds_stf(o_off + ((uint32_t)b * R + (uint32_t)i * rpp + (t >> lsh)) * 4u, x);   // the row sums go into the region
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
        const uint32_t red_off = c.ctl + CTL_OFF(red) + v * 256u;
        Spin s;
        if (vs.wv == 1u) {
            while (uni(lds_vld32(c.ctl + CTL_OFF(red_ack) + v * 4u)) != vs.red_seq)
                if (!spin_step(c, s, uni(lds_vld32(c.ctl + CTL_OFF(abort))), 0xA00u)) return false;
            lds_stf(red_off + c.lane * 4u, mine);
            lds_wait();
            if (c.lane == 0) lds_vst32(c.ctl + CTL_OFF(red_flag) + v * 4u, vs.red_seq + 1u);
            reconverge();
        } else {
            while (uni(lds_vld32(c.ctl + CTL_OFF(red_flag) + v * 4u)) != vs.red_seq + 1u)
                if (!spin_step(c, s, uni(lds_vld32(c.ctl + CTL_OFF(abort))), 0xB00u)) return false;
            compiler_barrier();
            mine += lds_ldf(red_off + c.lane * 4u);
            if (c.lane < (uint32_t)(NACC * B)) {
                uint32_t r = c.lane / (uint32_t)B, b = c.lane % (uint32_t)B;
                lds_stf(o_off + (b * R + r) * 4u, mine);
            }
            lds_wait();
            if (c.lane == 0) lds_vst32(c.ctl + CTL_OFF(red_ack) + v * 4u, vs.red_seq + 1u);
            reconverge();
        }
        vs.red_seq++;
    }
    lds_wait();
    vcc_done_with(c, vs, 1u, 1u);                                     // the region goes back as produced
    return true;
}

// The matvec uop over `nrb` row blocks of R rows that share one vector tile (K fits one tile; a tile row lies inside one
// wave).  The output region ([B][nrb * R] fp32) is popped first and kept, then the vector tile, which is read into
// registers once; every matrix tile is multiplied, its row sums go straight into the region at the block's rows, and
// the tile goes back; the vector tile goes back after the last block and the region as produced.
template <int B, int NF>
DEV bool matvec_rows_uop(Ctx &c, VccState &vs, uint32_t nrb, uint32_t R, uint32_t lpr) {
    const uint32_t slot_shift = __builtin_ctz(c.p->slot_bytes);
    const uint32_t t = vs.t, c4 = t & (lpr - 1u), pitch = lpr * 16u;
    const uint32_t lsh = __builtin_ctz(lpr), rpp = 128u >> lsh;
    Msg mo, mx, ma, unused;
    if (!vcc_pop_wait(c, vs, 1u, 1u, mo, unused)) return false;       // the output region
    const uint32_t o_pay = vs.pay0;
    vs.head += 1u;                                                     // popped; pushed as produced at the end
    if (!vcc_pop_wait(c, vs, 1u, 0u, mx, unused)) return false;       // the vector tile
    const uint32_t x_pay = vs.pay0;
    vs.head += 1u;                                                     // popped; handed back after the last block
    const uint32_t o_off = mo.slot << slot_shift, x_off = mx.slot << slot_shift;
    f32x4 xv[B];
#pragma unroll
    for (int b = 0; b < B; b++) xv[b] = lds_ld128(x_off + (uint32_t)b * pitch + c4 * 16u);
    const uint32_t opitch = nrb * R;                                   // values per row of the output region
    const uint64_t last_lanes = __ballot(c4 == lpr - 1u);              // the lanes that hold a row's sum after the reduction
    const uint32_t o_lane = o_off + (t >> lsh) * 4u;
    // the row sums of one matrix tile (block j) go straight into the region
    auto block = [&](const f32x4 (&m)[NF], uint32_t j) __attribute__((always_inline)) {
        float r[NF][B];
#pragma unroll
        for (int i = 0; i < NF; i++)
#pragma unroll
            for (int b = 0; b < B; b++) r[i][b] = dot4(m[i], xv[b], 0.0f);
        // the usual tile widths have the reduction without a select per level
        if (lpr == 32u) {
#pragma unroll
            for (int i = 0; i < NF; i++)
#pragma unroll
                for (int b = 0; b < B; b++) r[i][b] = lane_group_sum_fixed<32>(r[i][b]);
        } else if (lpr == 64u) {
#pragma unroll
            for (int i = 0; i < NF; i++)
#pragma unroll
                for (int b = 0; b < B; b++) r[i][b] = lane_group_sum_fixed<64>(r[i][b]);
        } else if (lpr == 16u) {
#pragma unroll
            for (int i = 0; i < NF; i++)
#pragma unroll
                for (int b = 0; b < B; b++) r[i][b] = lane_group_sum_fixed<16>(r[i][b]);
        } else {
#pragma unroll
            for (int i = 0; i < NF; i++)
#pragma unroll
                for (int b = 0; b < B; b++) r[i][b] = lane_group_sum(r[i][b], lpr);
        }
#pragma unroll
        for (int i = 0; i < NF; i++)
#pragma unroll
            for (int b = 0; b < B; b++)
                lds_st32_lanes(last_lanes, o_lane + ((uint32_t)b * opitch + j * R + (uint32_t)i * rpp) * 4u, __builtin_bit_cast(uint32_t, r[i][b]));
    };
    // two blocks at a time while two are left: one look at the queue and one hand-back for both
    for (uint32_t j = 0; j < nrb; j += 2u) {
        const uint32_t n = nrb - j >= 2u ? 2u : 1u;
        Msg mb;
        if (!vcc_pop_wait(c, vs, n, 0u, ma, mb)) return false;
        const uint32_t a_off = ma.slot << slot_shift, b_off = (n == 2u ? mb.slot : ma.slot) << slot_shift;
        f32x4 m0[NF], m1[NF];
#pragma unroll
        for (int i = 0; i < NF; i++) m0[i] = lds_ld128(a_off + ((uint32_t)i * 128u + t) * 16u);
#pragma unroll
        for (int i = 0; i < NF; i++) m1[i] = lds_ld128(b_off + ((uint32_t)i * 128u + t) * 16u);
        block(m0, j);
        if (n == 2u) block(m1, j + 1u);
        vcc_done_with(c, vs, n, 0u);
    }
    vcc_return_kept(c, vs, x_pay);
    lds_wait();
    vcc_push_kept(c, vs, o_pay);
    return true;
}

template <int B>
DEV bool matvec_rows_dispatch_b(Ctx &c, VccState &vs, uint32_t nrb, uint32_t R, uint32_t lpr, uint32_t nf) {
    if (nf == 1u) return matvec_rows_uop<B, 1>(c, vs, nrb, R, lpr);
    if (nf == 2u) return matvec_rows_uop<B, 2>(c, vs, nrb, R, lpr);
    if (nf == 4u) return matvec_rows_uop<B, 4>(c, vs, nrb, R, lpr);
    if (nf == 8u) return matvec_rows_uop<B, 8>(c, vs, nrb, R, lpr);
    raise_error(c, -3 /* VDC_EPROGRAM */, 0xC20u);
    return false;
}

template <int B>
DEV bool matvec_dispatch_b(Ctx &c, VccState &vs, uint32_t size, uint32_t R, uint32_t lpr, uint32_t nf, uint32_t j, uint32_t xspan) {
#define VDC_MV(NF_, J_) \
    if (nf == NF_ && j == J_ && xspan < 2u) return matvec_uop<B, NF_, J_>(c, vs, size, R, lpr, xspan);
    VDC_MV(1, 0) VDC_MV(2, 0) VDC_MV(4, 0) VDC_MV(8, 0)
    VDC_MV(1, 1) VDC_MV(2, 1) VDC_MV(4, 1) VDC_MV(8, 1)
    if constexpr (B * 2 <= 16) { VDC_MV(2, 2) VDC_MV(4, 2) VDC_MV(8, 2) }
    if constexpr (B * 4 <= 16) { VDC_MV(4, 4) VDC_MV(8, 4) }
    if constexpr (B * 8 <= 16) { VDC_MV(8, 8) }
#undef VDC_MV
    if constexpr (B == 8) {
        // several vectors and a vector tile over several steps: the tiles of the largest batch (matvec_xspan_ok)
        if (xspan >= 2u && j == 0u) {
            if (nf == 4u) return matvec_uop<8, 4, 0, true>(c, vs, size, R, lpr, xspan);
            if (nf == 8u) return matvec_uop<8, 8, 0, true>(c, vs, size, R, lpr, xspan);
        }
    }
    if constexpr (B == 1) {
        // the variant that keeps a vector tile over several steps is a code path of its own: the usual one pays nothing
        if (xspan >= 2u && j == 0u) {
            if (nf == 1u) return matvec_uop<1, 1, 0, true>(c, vs, size, R, lpr, xspan);
            if (nf == 2u) return matvec_uop<1, 2, 0, true>(c, vs, size, R, lpr, xspan);
            if (nf == 4u) return matvec_uop<1, 4, 0, true>(c, vs, size, R, lpr, xspan);
            if (nf == 8u) return matvec_uop<1, 8, 0, true>(c, vs, size, R, lpr, xspan);
        }
    }
    raise_error(c, -3 /* VDC_EPROGRAM */, 0xC00u);
    return false;
}

template <uint32_t OPS>
DEV bool matvec_dispatch(Ctx &c, VccState &vs, const Fields &f) {
    const uint32_t B = (uint32_t)f.imm & 0xFFu, R = (uint32_t)(f.imm >> 8) & 0xFFFFu, lpr = (uint32_t)(f.imm >> 24) & 0xFFFFu;
    const uint32_t nf = (R * lpr) >> 7;
    const uint32_t j = lpr <= 64u ? 0u : lpr >> 7;
    const uint32_t xspan = matvec_xspan(f.imm);
    if (xspan >= 2u && (j != 0u || xspan > kMaxXspan || !matvec_xspan_ok(B, R, lpr))) {
        raise_error(c, -3 /* VDC_EPROGRAM */, 0xC10u);
        return false;
    }
    const uint32_t rowspan = matvec_rowspan(f);
    if (rowspan >= 2u) {
        if constexpr ((OPS & OPS_ROWS) == 0u) {
            raise_error(c, -3 /* VDC_EPROGRAM */, 0xC40u);
            return false;
        } else {
        if (j != 0u || f.size != 1u || xspan >= 2u || rowspan > kMaxRowspan || B > kMaxRowspanB) {
            raise_error(c, -3 /* VDC_EPROGRAM */, 0xC30u);
            return false;
        }
        switch (B) {
            case 1: return matvec_rows_dispatch_b<1>(c, vs, rowspan, R, lpr, nf);
            case 2: return matvec_rows_dispatch_b<2>(c, vs, rowspan, R, lpr, nf);
            case 3: return matvec_rows_dispatch_b<3>(c, vs, rowspan, R, lpr, nf);
            case 4: return matvec_rows_dispatch_b<4>(c, vs, rowspan, R, lpr, nf);
            default:
                raise_error(c, -3 /* VDC_EPROGRAM */, 0xD00u);
                return false;
        }
        }
    }
    switch (B) {
        case 1: return matvec_dispatch_b<1>(c, vs, f.size, R, lpr, nf, j, xspan);
        case 2: return matvec_dispatch_b<2>(c, vs, f.size, R, lpr, nf, j, xspan);
        case 3: return matvec_dispatch_b<3>(c, vs, f.size, R, lpr, nf, j, xspan);
        case 4: return matvec_dispatch_b<4>(c, vs, f.size, R, lpr, nf, j, xspan);
        case 5: return matvec_dispatch_b<5>(c, vs, f.size, R, lpr, nf, j, xspan);
        case 6: return matvec_dispatch_b<6>(c, vs, f.size, R, lpr, nf, j, xspan);
        case 7: return matvec_dispatch_b<7>(c, vs, f.size, R, lpr, nf, j, xspan);
        case 8: return matvec_dispatch_b<8>(c, vs, f.size, R, lpr, nf, j, xspan);
        default:
            raise_error(c, -3 /* VDC_EPROGRAM */, 0xD00u);
            return false;
    }
}

// The rope uop of the running example (Section 3): the value tile, the tile of (cos, sin) pairs and the output region
// are all [B][R] fp32, rows back to back, so pair p of the tile lies at byte 8 p of each.  Thread t turns pairs
// t, t + 128, ... (at most four).
DEV bool rope_uop(Ctx &c, VccState &vs, uint32_t B, uint32_t R) {
    const uint32_t slot_shift = __builtin_ctz(c.p->slot_bytes);
    Msg mo, mt;
    if (!vcc_pop_wait(c, vs, 2u, 0u, mo, mt)) return false;
    const uint32_t o_off = mo.slot << slot_shift, t_off = mt.slot << slot_shift;
    const uint32_t pairs = B * R / 2u;
    float rx[4], ry[4];
#pragma unroll
    for (uint32_t q = 0; q < 4u; q++) {
        const uint32_t pr = vs.t + q * 128u;
        rx[q] = 0.0f; ry[q] = 0.0f;
        if (pr < pairs) {
            const float x = lds_ldf(o_off + pr * 8u), y = lds_ldf(o_off + pr * 8u + 4u);
            const float cs = lds_ldf(t_off + pr * 8u), sn = lds_ldf(t_off + pr * 8u + 4u);
            rx[q] = __builtin_fmaf(x, cs, -(y * sn));
            ry[q] = __builtin_fmaf(x, sn, y * cs);
        }
    }
    // the results are in registers, so every read of the two input tiles has returned: they can go back
    vcc_done_with(c, vs, 2u, 0u);
    Msg mout, unused;
    if (!vcc_pop_wait(c, vs, 1u, 1u, mout, unused)) return false;
    const uint32_t out_off = mout.slot << slot_shift;
#pragma unroll
    for (uint32_t q = 0; q < 4u; q++) {
        const uint32_t pr = vs.t + q * 128u;
        if (pr < pairs) {
            lds_stf(out_off + pr * 8u, rx[q]);
            lds_stf(out_off + pr * 8u + 4u, ry[q]);
        }
    }
    lds_wait();
    vcc_done_with(c, vs, 1u, 1u);
    return true;
}

// Compute uops without arithmetic, which leave the memory uops around them as the only work (Section 6.3, "Memory
// virtual core overhead").  A region is at most kStreamPasses * 128 chunks of 16 bytes: thread t moves chunks
// t, t + 128, ...
constexpr uint32_t kStreamPasses = 16;

DEV bool drop_uop(Ctx &c, VccState &vs, uint32_t size) {
    // one region at a time, as the uop is defined: popping two at once would need both resident, which a small pool
    // of slots may not allow
    Msg m, unused;
    for (; size != 0u; size--) {
        if (!vcc_pop_wait(c, vs, 1u, 0u, m, unused)) return false;
        vcc_done_with(c, vs, 1u, 0u);
    }
    return true;
}

DEV bool fill_uop(Ctx &c, VccState &vs, uint32_t size, uint32_t value, uint32_t chunks) {
    const uint32_t slot_shift = __builtin_ctz(c.p->slot_bytes);
    const u32x4 v = u32x4{value, value, value, value};
    Msg mo, unused;
    for (; size != 0u; size--) {
        if (!vcc_pop_wait(c, vs, 1u, 1u, mo, unused)) return false;
        const uint32_t off = mo.slot << slot_shift;
        for (uint32_t ch = vs.t; ch < chunks; ch += 128u) lds_st128(off + ch * 16u, v);
        lds_wait();
        vcc_done_with(c, vs, 1u, 1u);
    }
    return true;
}

DEV bool copy_uop(Ctx &c, VccState &vs, uint32_t size, uint32_t chunks) {
    const uint32_t slot_shift = __builtin_ctz(c.p->slot_bytes);
    Msg mi, mo, unused;
    for (; size != 0u; size--) {
        if (!vcc_pop_wait(c, vs, 1u, 0u, mi, unused)) return false;
        const uint32_t in_off = mi.slot << slot_shift;
        f32x4 r[kStreamPasses];
#pragma unroll
        for (uint32_t q = 0; q < kStreamPasses; q++) {
            const uint32_t ch = vs.t + q * 128u;
            r[q] = lds_ld128(ch < chunks ? in_off + ch * 16u : in_off);
        }
        lds_wait();
        vcc_done_with(c, vs, 1u, 0u);
        if (!vcc_pop_wait(c, vs, 1u, 1u, mo, unused)) return false;
        const uint32_t out_off = mo.slot << slot_shift;
#pragma unroll
        for (uint32_t q = 0; q < kStreamPasses; q++) {
            const uint32_t ch = vs.t + q * 128u;
            if (ch < chunks) *(__attribute__((address_space(3))) f32x4 *)(lds0() + out_off + ch * 16u) = r[q];
        }
        lds_wait();
        vcc_done_with(c, vs, 1u, 1u);
    }
    return true;
}

// Sum over the G = 4 or 8 consecutive lanes that share a key row; every lane of the group gets the sum.
template <int G>
DEV float group_sum(float x) {
    x += dpp_f32<kDppXor1>(x);
    x += dpp_f32<kDppXor2>(x);
    if (G == 8) x += dpp_f32_banks<kDppShl4, 0x5>(x, 0.0f) + dpp_f32_banks<kDppShr4, 0xA>(x, 0.0f);   // lane ^ 4
    return x;
}
// All 64 lanes get the maximum (MAX) or the sum of x over the key rows, x being equal inside each group of G lanes.
template <int G, bool MAX>
DEV float rows_reduce(float x) {
    if (G == 4) {
        const float y = dpp_f32<kDppRor4>(x);
        x = MAX ? __builtin_fmaxf(x, y) : x + y;
    }
    const float z = dpp_f32<kDppRor8>(x);
    x = MAX ? __builtin_fmaxf(x, z) : x + z;
    const float t0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 0));
    const float t1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 16));
    const float t2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 32));
    const float t3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 48));
    return MAX ? __builtin_fmaxf(__builtin_fmaxf(t0, t1), __builtin_fmaxf(t2, t3)) : (t0 + t1) + (t2 + t3);
}

// The attn uop (Section 4.1) for decoding: one query row of d = 4 LPR values (128 or 64) against `size` (key tile, value tile) pairs of
// R rows, FlashAttention-style: a running maximum m of the scores, a running sum l of exp(score - m) and the running
// sums o of exp(score - m) times the value rows.  Both waves of the execution unit compute every score (so m and l
// come out bit-identical in the two waves and no exchange between them is needed): the key tile is taken in NP passes
// of RP <= 16 rows, G = 64 / RP lanes sharing a row.  Wave w then owns columns 64 w .. 64 w + 63 of o, one per lane.
// The query tile is allocated first and handed back last, after every key and value tile: slots return in another
// order than they went out (Section 4.3).  Rows of a short last tile score minus infinity.
template <int R, int LPR>
DEV bool attn_uop(Ctx &c, VccState &vs, uint32_t size, float scale, uint32_t join) {
    constexpr int RP = R > 16 ? 16 : R;            // key rows per pass
    constexpr int NP = R / RP;                     // passes per tile
    constexpr uint32_t G = 64u / (uint32_t)RP;     // lanes per key row: 4 or 8
    constexpr int NC = LPR / (int)G;               // 16-byte chunks of the row per lane: 8 or 4
    constexpr uint32_t ROW = (uint32_t)LPR * 16u;  // bytes per row of a key / value tile (d = 4 LPR values)
    constexpr uint32_t COLS = (uint32_t)LPR * 2u;  // columns of o a wave owns: 64 (one per lane) or 32 (the upper lanes repeat the lower)
    const uint32_t slot_shift = __builtin_ctz(c.p->slot_bytes);
    Msg mq, unused;
    if (!vcc_pop_wait(c, vs, 1u, 0u, mq, unused)) return false;
    const uint32_t q_pay = vs.pay0;
    vs.head += 1u;                                 // popped; handed back at the end
    const uint32_t q_off = mq.slot << slot_shift;
    // lane (row, sub) takes chunks (j G + sub + row) mod LPR of its key rows, j = 0 .. NC - 1: the rotation by the row
    // spreads the lanes of one read over the banks (rows are 256 or 512 bytes apart, so equal columns would all collide)
    const uint32_t sub = c.lane & (G - 1u), row = c.lane / G, rot = sub + row;
    f32x4 qv[NC];
#pragma unroll
    for (int j = 0; j < NC; j++) qv[j] = lds_ld128(q_off + (((uint32_t)j * G + rot) & (uint32_t)(LPR - 1)) * 16u);
    const uint32_t col = vs.wv * COLS + (c.lane & (COLS - 1u));
    float m = -__builtin_inff(), l = 0.0f, o = 0.0f;
    for (uint32_t it = 0; it < size; it++) {
        Msg mk, mv;
        if (!vcc_pop_wait(c, vs, 2u, 0u, mk, mv)) return false;
        const uint32_t k_off = (mk.slot << slot_shift) + row * ROW, v_off = (mv.slot << slot_shift) + col * 4u;
        // the chunk offsets are recomputed per tile (three cheap instructions each): kept across tiles they would
        // take registers that the loads in flight need
        uint32_t rot_t = rot;
        asm volatile("" : "+v"(rot_t));
        float s[NP];
#pragma unroll
        for (int h = 0; h < NP; h++) {
            f32x4 kv[NC];
#pragma unroll
            for (int j = 0; j < NC; j++) kv[j] = lds_ld128(k_off + (uint32_t)h * RP * ROW + (((uint32_t)j * G + rot_t) & (uint32_t)(LPR - 1)) * 16u);
            float s0 = 0.0f, s1 = 0.0f;
#pragma unroll
            for (int j = 0; j < NC; j += 2) {
                s0 = dot4(kv[j], qv[j], s0);
                s1 = dot4(kv[j + 1], qv[j + 1], s1);
            }
            const float x = group_sum<(int)G>(s0 + s1);
            s[h] = (uint32_t)h * RP + row < mk.rows ? x * scale : -__builtin_inff();
            compiler_barrier();      // one pass of key reads in flight at a time: the registers for more are not there
        }
        float tm = s[0];
#pragma unroll
        for (int h = 1; h < NP; h++) tm = __builtin_fmaxf(tm, s[h]);
        const float m_new = __builtin_fmaxf(m, rows_reduce<(int)G, true>(tm));
        float p[NP], ps = 0.0f;
#pragma unroll
        for (int h = 0; h < NP; h++) {
            p[h] = expf(s[h] - m_new);
            ps += p[h];
        }
        ps = rows_reduce<(int)G, false>(ps);
        const float alpha = expf(m - m_new);     // 0 on the first tile
        l = __builtin_fmaf(l, alpha, ps);
        o *= alpha;
#pragma unroll
        for (int r0 = 0; r0 < R; r0 += 8) {
            float vv[8];
#pragma unroll
            for (int r = 0; r < 8; r++) vv[r] = lds_ldf(v_off + (uint32_t)(r0 + r) * ROW);
#pragma unroll
            for (int r = 0; r < 8; r++) {
                const float pr = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, p[(r0 + r) / RP]), ((r0 + r) % RP) * (int)G));
                o = __builtin_fmaf(pr, vv[r], o);
            }
        }
        m = m_new;
        vcc_done_with(c, vs, 2u, 0u);
    }
    vcc_return_kept(c, vs, q_pay);
    if (join != 0u) {
        // The context has `join` <= 64 other items: their partial rows (o, m, l, 0, 0) come as one more tile and are joined
        // to this uop's own state, the same rescaling as from tile to tile.  Lane i takes row i's maximum and sum, so the
        // weights are one exponential per lane; the weighted sum takes one LDS read per row, the weight from the scalar side.
        constexpr uint32_t PROW = ROW + 16u;
        Msg mt;
        if (join > 64u) {
            raise_error(c, -3 /* VDC_EPROGRAM */, 0xE50u);
            return false;
        }
        if (!vcc_pop_wait(c, vs, 1u, 0u, mt, unused)) return false;
        const uint32_t t_off = mt.slot << slot_shift;
        const bool mine = c.lane < join;
        const uint32_t r_off = t_off + (mine ? c.lane : 0u) * PROW + ROW;
        const float mi = mine ? lds_ldf(r_off) : -__builtin_inff(), li = mine ? lds_ldf(r_off + 4u) : 0.0f;
        float M = mi;
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) M = __builtin_fmaxf(M, __shfl_xor(M, s, 64));
        M = __builtin_fmaxf(M, m);
        const float w = mine ? expf(mi - M) : 0.0f, w_own = expf(m - M);
        float ls = w * li;
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) ls += __shfl_xor(ls, s, 64);
        l = __builtin_fmaf(l, w_own, ls);
        o *= w_own;
        for (uint32_t i = 0; i < join; i++) {
            const float wi = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w), (int)i));
            o = __builtin_fmaf(wi, lds_ldf(t_off + i * PROW + col * 4u), o);
        }
        m = M;
        vcc_done_with(c, vs, 1u, 0u);
    }
    Msg mo;
    if (!vcc_pop_wait(c, vs, 1u, 1u, mo, unused)) return false;
    const uint32_t out_off = mo.slot << slot_shift;
    // The region says what is wanted: one row of d values takes the finished result o / l (the uop saw the whole context),
    // a row of d + 4 values the partial row (o, m, l, 0, 0) that an ATTN_MERGE joins with those of the context's other items.
    const bool whole = mo.row_bytes == ROW;
    lds_st32_lanes(COLS == 64u ? ~0ull : 0xFFFFFFFFull, out_off + col * 4u, __builtin_bit_cast(uint32_t, whole ? o / l : o));
    lds_st32_lanes(whole || vs.wv != 0u ? 0ull : 0xFull, out_off + ROW + c.lane * 4u, __builtin_bit_cast(uint32_t, c.lane == 0u ? m : (c.lane == 1u ? l : 0.0f)));
    lds_wait();
    vcc_done_with(c, vs, 1u, 1u);
    return true;
}

// attn_merge: `P` <= 64 partial rows (o[0..d), m, l, 0, 0) of one request become its result; thread t owns column t
// (d = 4 lpr).  Lane i of every wave takes row i's maximum and sum, so the weights exp(m_i - M) are one exponential per
// lane and M and the denominator are reductions over the wave; the weighted sum then takes one LDS read per row, the
// weight coming from the scalar side.
DEV bool attn_merge_uop(Ctx &c, VccState &vs, uint32_t P, uint32_t lpr) {
    const uint32_t D4 = lpr * 16u, PROW = D4 + 16u;
    const uint32_t tcol = vs.t < lpr * 4u ? vs.t : 0u;
    const uint32_t slot_shift = __builtin_ctz(c.p->slot_bytes);
    Msg mt, mo, unused;
    if (P > 64u) {
        raise_error(c, -3 /* VDC_EPROGRAM */, 0xE40u);
        return false;
    }
    if (!vcc_pop_wait(c, vs, 1u, 0u, mt, unused)) return false;
    const uint32_t t_off = mt.slot << slot_shift;
    const bool mine = c.lane < P;
    const uint32_t r_off = t_off + (mine ? c.lane : 0u) * PROW + D4;
    const float mi = mine ? lds_ldf(r_off) : -__builtin_inff(), li = mine ? lds_ldf(r_off + 4u) : 0.0f;
    float M = mi;
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) M = __builtin_fmaxf(M, __shfl_xor(M, s, 64));
    const float w = mine ? expf(mi - M) : 0.0f;
    float den = w * li;
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) den += __shfl_xor(den, s, 64);
    float num = 0.0f;
    for (uint32_t i = 0; i < P; i++) {
        const float wi = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w), (int)i));
        num = __builtin_fmaf(wi, lds_ldf(t_off + i * PROW + tcol * 4u), num);
    }
    const float res = num / den;
    vcc_done_with(c, vs, 1u, 0u);
    if (!vcc_pop_wait(c, vs, 1u, 1u, mo, unused)) return false;
    if (vs.t < lpr * 4u) lds_stf((mo.slot << slot_shift) + vs.t * 4u, res);
    lds_wait();
    vcc_done_with(c, vs, 1u, 1u);
    return true;
}

// The control-flow unit of a VCC runs on the execution unit's own threads (Section 4.3, "Virtual Compute Core"):
// each of its two waves decodes the stream, runs control uops itself and then yields to the uop handler.
// OPS: the compute uops this build of the kernel has handlers for (a program runs on the variant compiled for what it uses:
// the kernel is one function, and every handler in it weighs on the register allocation of all the others).
template <uint32_t OPS>
DEV void vcc_main(Ctx &c, uint32_t wv) {
    const KParams *p = c.p;
    const bool TRACE = p->trace != nullptr;
    const uint32_t stream = c.core * (1u + p->V) + 1u + c.unit;
    Seq s;
    seq_init(c, s, cload(p->stream_begin, stream), cload(p->stream_begin, stream + 1u));
    c.stream_pc0 = s.pc;
    VccState vs;
    vs.head = 0; vs.group = 0; vs.c2m_pos = 0; vs.pay0 = 0; vs.pay1 = 0; vs.red_seq = 0; vs.wv = wv; vs.t = wv * 64u + c.lane;
    uint32_t trace_n = 0;
    bool ok = true;
    while (ok) {
        c.pc = s.pc;
        Word w = fetch(c, s);
        Fields f = decode(w);
        int ctl = seq_control(s, f);
        if (ctl == 2) break;
        if (ctl == 1) continue;
        if (TRACE && wv == 0u) trace_put(c, stream, trace_n, s.pc - c.stream_pc0, f.opcode | (f.size << 16), (uint64_t)f.imm);
        if ((OPS & OPS_MATVEC) != 0u && f.opcode == OP_MATVEC) {
            ok = matvec_dispatch<OPS>(c, vs, f);
        } else if ((OPS & OPS_ROPE) != 0u && f.opcode == OP_ROPE) {
            ok = rope_uop(c, vs, (uint32_t)f.imm & 0xFFu, (uint32_t)(f.imm >> 8) & 0xFFFFu);
        } else if ((OPS & OPS_ATTN) != 0u && f.opcode == OP_ATTN) {
            const uint32_t lpr = (uint32_t)f.imm & 0xFFu, R = (uint32_t)(f.imm >> 8) & 0xFFu, join = attn_join(f);
            const float scale = __builtin_bit_cast(float, (uint32_t)(f.imm >> 16));
            if (lpr == 32u && R == 32u) ok = attn_uop<32, 32>(c, vs, f.size, scale, join);
            else if (lpr == 32u && R == 16u) ok = attn_uop<16, 32>(c, vs, f.size, scale, join);
            else if (lpr == 32u && R == 8u) ok = attn_uop<8, 32>(c, vs, f.size, scale, join);
            else if (lpr == 16u && R == 64u) ok = attn_uop<64, 16>(c, vs, f.size, scale, join);
            else if (lpr == 16u && R == 32u) ok = attn_uop<32, 16>(c, vs, f.size, scale, join);
            else if (lpr == 16u && R == 16u) ok = attn_uop<16, 16>(c, vs, f.size, scale, join);
            else {
                raise_error(c, -3 /* VDC_EPROGRAM */, 0xE00u | f.opcode);
                ok = false;
            }
        } else if ((OPS & OPS_ATTN) != 0u && f.opcode == OP_ATTN_MERGE) {
            ok = attn_merge_uop(c, vs, f.size, (uint32_t)f.imm & 0xFFu);
        } else if ((OPS & OPS_STREAM) != 0u && f.opcode == OP_DROP) {
            ok = drop_uop(c, vs, f.size);
        } else if ((OPS & OPS_STREAM) != 0u && f.opcode == OP_FILL) {
            ok = fill_uop(c, vs, f.size, (uint32_t)f.imm, (uint32_t)(f.imm >> 32) & 0xFFFFu);
        } else if ((OPS & OPS_STREAM) != 0u && f.opcode == OP_COPY) {
            ok = copy_uop(c, vs, f.size, (uint32_t)f.imm & 0xFFFFu);
        } else {
            raise_error(c, -3 /* VDC_EPROGRAM */, 0xE00u | f.opcode);
            ok = false;
        }
        s.pc++;
    }
    compiler_barrier();
    if (c.lane == 0)
        __hip_atomic_fetch_add((__attribute__((address_space(3))) uint32_t *)(lds0() + c.ctl + CTL_OFF(vcc_done)), 1u,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    reconverge();
}

// ------------------------------------------------------------------------------------------------
// The persistent kernel: every wave takes its role and runs it to the end of the uop graph
// ------------------------------------------------------------------------------------------------
#ifdef VDC_PROFILE
// Profiling builds only: an extra wave of core 0 that only reads.  It samples the control words (and the ticket
// halves of the m2c rings) as fast as it can and logs every change with a time stamp: (cycles, word | value << 32).
constexpr uint32_t kObsCap = 1u << 16;
DEV void observer_main(Ctx &c, uint32_t V) {
    if (c.core != 0u) return;
    unsigned long long *log = c.p->prof + (size_t)gridDim.x * 16 * 8;
#ifdef VDC_PROFILE_PHASES
    // statistical profile: sample every wave's phase word as fast as possible; lane w counts how often wave w was
    // seen in each phase
    uint32_t h[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    uint32_t poff = c.ctl + CTL_OFF(phase) + (c.lane & 15u) * 4u;
    poff = c.lane == 16u ? c.ctl + CTL_OFF(abort) : poff;
    poff = c.lane == 17u ? c.ctl + CTL_OFF(cfu_halted) : poff;
    poff = c.lane == 18u ? c.ctl + CTL_OFF(vcc_done) : poff;
    uint32_t it = 0;
    for (; it < (1u << 24); it++) {
        const uint32_t ph = lds_vld32(poff);
#pragma unroll
        for (uint32_t i = 0; i < 8u; i++) h[i] += ph == i ? 1u : 0u;
        if (rf_get(ph, 16) != 0u || (rf_get(ph, 17) != 0u && rf_get(ph, 18) == 2u * V)) break;
    }
    if (c.lane < 16u)
        for (uint32_t i = 0; i < 8u; i++) log[c.lane * 8u + i] = h[i];
    if (c.lane == 0) log[(size_t)kObsCap * 2] = it;
    return;
#endif
    uint32_t prev_a = 0, n = 0;
    const uint32_t off = c.ctl + (c.lane < 36u ? c.lane * 4u : CTL_OFF(phase) + ((c.lane - 36u) & 15u) * 4u);
    for (uint32_t it = 0; it < (1u << 22); it++) {
        const uint32_t a = lds_vld32(off);
        unsigned long long t;
        asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t)::"memory");
        const bool ca = a != prev_a && c.lane < 52u;
        const uint64_t ma = __ballot(ca);
        prev_a = a;
        if (rf_get(a, 9) != 0u || (rf_get(a, 10) != 0u && rf_get(a, 11) == 2u * V)) break;
        if (ma == 0ull) continue;
        if (ca) {
            const uint32_t idx = n + lanes_below(ma, c.lane);
            if (idx < kObsCap) { log[idx * 2] = t; log[idx * 2 + 1] = (unsigned long long)c.lane | ((unsigned long long)a << 32); }
        }
        n = uni(n + (uint32_t)__builtin_popcountll(ma));
    }
    if (c.lane == 0) log[(size_t)kObsCap * 2] = n;
}
#endif

#define VDC_MAX_THREADS 768     // twelve waves: three per SIMD, which leaves each 170 vector registers
// One uop graph on one core, from a zeroed control block to the last unit leaving: every wave of the workgroup calls it.
template <uint32_t OPS>
DEV void run_core(const KParams &p) {
    // The hardware deals the waves of a workgroup round-robin over the four SIMDs of the compute unit, so which roles
    // share a SIMD (and contend for its issue slots) is decided by which wave takes which role: the host chooses.
    const uint32_t wave = uni((uint32_t)(p.wave_roles >> ((threadIdx.x >> 6) * 4u)) & 15u);
    Ctx c;
    c.p = &p;
    c.core = blockIdx.x;
    c.lane = threadIdx.x & 63u;
    c.ctl = p.n_slots * p.slot_bytes;
    c.spins_limit = p.watchdog;
    c.stream_pc0 = 0;
    c.pc = 0;
    // the front end's two trips to memory for its first window start here, so that they overlap the clearing of the
    // control block and the barrier (the wave clears its share once the stream's bounds are there; the words follow)
    CfuStart start = {};
    if (wave == 0u) start = cfu_start_fetch(c);
    // the control block starts at zero (slots need no initialisation)
    {
        const uint32_t words = (uint32_t)(sizeof(Ctl) / 4);
        for (uint32_t i = threadIdx.x; i < words; i += blockDim.x) lds_vst32(c.ctl + i * 4u, 0u);
    }
    // the only workgroup barrier: before the roles diverge.  It orders the clearing stores to local memory alone; the front
    // end's loads from memory stay in flight across it
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    if (wave == 15u) return;   // a wave that is there only to shift the others to another SIMD
#ifdef VDC_PROFILE_WAITS
    c.w_t0 = prof_now();
#endif

    if (wave == 0u) {
        c.role = ROLE_CFU; c.unit = 0;
        // the front end is a long dependent chain of cheap instructions: let it win the issue arbitration against the
        // compute wave that shares its SIMD
        __builtin_amdgcn_s_setprio(kCfuPrio);
        cfu_main(c, start);
    } else if (wave <= p.n_ldu) {
        c.role = ROLE_LDU; c.unit = wave - 1u;
        c.stream_pc0 = cload(p.stream_begin, c.core * (1u + p.V));
        __builtin_amdgcn_s_setprio(kLduPrio);
        ldu_main(c);
    } else if (wave <= p.n_ldu + p.n_stu) {
        c.role = ROLE_STU; c.unit = wave - 1u;
        c.stream_pc0 = cload(p.stream_begin, c.core * (1u + p.V));
        __builtin_amdgcn_s_setprio(kStuPrio);
        stu_main(c);
#ifdef VDC_PROFILE
    } else if (wave == 1u + p.n_ldu + p.n_stu + 2u * p.V) {
        observer_main(c, p.V);
#endif
    } else {
        const uint32_t k = wave - 1u - p.n_ldu - p.n_stu;
        c.role = ROLE_VCC; c.unit = k >> 1;
        vcc_main<OPS>(c, k & 1u);
    }
#ifdef VDC_PROFILE_WAITS
    if (c.lane == 0 && wave < 16u) {
        unsigned long long *o = p.prof + ((size_t)blockIdx.x * 16 + wave) * 8;
        o[0] = c.w_wait; o[1] = c.w_spins; o[2] = c.w_vm; o[3] = prof_now() - c.w_t0;
        o[4] = c.w_sec[0]; o[5] = c.w_sec[1]; o[6] = c.w_sec[2]; o[7] = c.w_sec[3];
    }
#endif
}

template <uint32_t OPS>
__global__ void __launch_bounds__(VDC_MAX_THREADS) vdc_executor_kernel(const KParams p) { run_core<OPS>(p); }

// The variants of the kernel, from few handlers to all; a program runs on the first that has every handler it needs.
#ifdef VDC_PROFILE
constexpr uint32_t kVariants[] = {OPS_ALL};
#elif defined(VDC_SPLIT) || defined(VDC_PART)
// the last three: matvec and stream programs whose regions all take one slot, built with VDC_WAVE_MASKS (see Ctl::mask)
constexpr uint32_t kVariants[] = {OPS_MATVEC, OPS_MATVEC | OPS_ROWS, OPS_MATVEC | OPS_ROPE, OPS_STREAM, OPS_ATTN, OPS_ALL,
                                  OPS_ONE_SLOT | OPS_MATVEC, OPS_ONE_SLOT | OPS_MATVEC | OPS_ROWS, OPS_ONE_SLOT | OPS_STREAM};
#else
constexpr uint32_t kVariants[] = {OPS_MATVEC, OPS_MATVEC | OPS_ROWS, OPS_MATVEC | OPS_ROPE, OPS_STREAM, OPS_ATTN, OPS_ALL};
#endif
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

#ifdef VDC_PART
// A unit of the split build: this variant of the kernel and the function that hands out its address, nothing else.
#define VDC_PART_NAME2(I) vdc_variant_entry_##I
#define VDC_PART_NAME(I) VDC_PART_NAME2(I)
extern "C" const void *VDC_PART_NAME(VDC_PART)() { return (const void *)vdc_executor_kernel<kVariants[VDC_PART]>; }
}  // namespace vdc
#else

// ------------------------------------------------------------------------------------------------
// The resident form (Section 4.3: the virtual cores are launched once and new uop graphs are streamed to them as requests
// arrive).  The grid stays up between graphs.  The first wave of core 0 watches a mailbox in pinned host memory; when
// the host has posted graph number seq it copies the graph's parameter block into device memory and publishes seq in a
// device word that every wave of the grid waits for; every core then runs the graph exactly as a launch of its own
// would, cores count themselves out, and the last one reports the number to the host.  A graph is published only when
// the one before is complete on every core (what a kernel boundary would give), with a release and an acquire at device
// scope around it so that one graph's stores are read by the next on whatever compute unit.
// Every wait has an end of its own: the watcher gives up after idle_polls looks without a new graph or when the host
// says stop, and publishes STOP, at which every wave leaves; the other waves wait for the device word with a much larger
// bound of their own.  When the host goes quiet or dies the grid therefore drains by itself.
// ------------------------------------------------------------------------------------------------
#ifndef VDC_PROFILE
constexpr uint32_t kResidentStop = 0xFFFFFFFFu;
static_assert(sizeof(KParams) <= 4 * kResidentJobWords, "a graph's parameter block fits one mailbox entry");

DEV uint32_t sys_load(const uint32_t *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM); }
DEV uint32_t dev_load(const uint32_t *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// The watcher's part before graph `seq`.  Returns nothing: what it decides is published in the device word.
DEV void resident_watch(const ResidentParams &rp, uint32_t seq, uint32_t lane) {
    uint32_t *dev_tail = rp.dev + RD_TAIL;
    bool stop = false;
    // the graph before must be complete on every core (each of its waits is bounded, so this one ends)
    if (seq > 1u) {
        uint32_t n = 0;
        while (uni(dev_load(rp.dev + RD_DONE)) < seq - 1u) {
            if (++n > rp.backstop_polls) { stop = true; break; }
            __builtin_amdgcn_s_sleep(16);
        }
        // a graph that ended in an error ends the residency
        if (uni(dev_load(rp.status + ST_ABORT)) != 0u) stop = true;
    }
    bool got = false;
    for (uint32_t n = 0; !stop && !got; n++) {
        // MB_TAIL and MB_STOP in one read of host memory (a trip over the host link each)
        const uint64_t both = __hip_atomic_load((const uint64_t *)(rp.mailbox + MB_TAIL), __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM);
        const uint32_t tail = uni((uint32_t)both), quit = uni((uint32_t)(both >> 32));
        if ((int32_t)(tail - seq) >= 0) got = true;
        else if (quit != 0u || n >= rp.idle_polls) stop = true;
        else __builtin_amdgcn_s_sleep(64);
    }
    if (got && !stop) {
        // the graph's parameter block: one word per lane, host memory -> device memory
        const uint32_t w = sys_load(rp.mailbox + MB_JOBS + (seq % kResidentJobs) * kResidentJobWords + lane);
        __hip_atomic_store(rp.dev + RD_JOB + lane, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (lane == 0) __hip_atomic_store(dev_tail, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        reconverge();
    } else {
        if (lane == 0) {
            __hip_atomic_store(rp.mailbox + MB_STATE, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            __hip_atomic_store(dev_tail, kResidentStop, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        reconverge();
    }
}

__global__ void __launch_bounds__(VDC_MAX_THREADS) vdc_resident_kernel(const ResidentParams rp) {
    const uint32_t lane = threadIdx.x & 63u;
    const bool watcher = blockIdx.x == 0u && (threadIdx.x >> 6) == 0u;
    for (uint32_t seq = 1u;; seq++) {
        if (watcher) resident_watch(rp, seq, lane);
        uint32_t t = 0;
        for (uint32_t n = 0;; n++) {
            t = uni(dev_load(rp.dev + RD_TAIL));
            if (t >= seq) break;                              // the graph, or STOP
            if (n >= rp.backstop_polls) { t = kResidentStop; break; }
            __builtin_amdgcn_s_sleep(16);
        }
        if (t == kResidentStop) break;
        // One wave of the core takes the acquire for all of them (it empties the compute unit's vector cache and the
        // stale lines of the L2 behind it; the barrier at the start of the graph orders the other waves behind it), as one
        // wave makes the release at the end: a fence per wave, 2560 of them on the same caches, cost 70 us per graph.
        if ((threadIdx.x >> 6) == 0u) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        // the parameter block into this wave's registers: lane l holds word l
        const uint32_t img = dev_load(rp.dev + RD_JOB + lane);
        KParams jp;
        {
            uint32_t raw[sizeof(KParams) / 4];
#pragma unroll
            for (uint32_t i = 0; i < (uint32_t)(sizeof(KParams) / 4); i++) raw[i] = rf_get(img, i);
            __builtin_memcpy(&jp, raw, sizeof(KParams));
        }
        __builtin_amdgcn_s_setprio(0);                        // whatever role the wave had in the graph before
        run_core<OPS_ALL>(jp);
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");      // this wave's stores have reached the L2
        __syncthreads();                                      // every wave of the core is done with the graph
        if ((threadIdx.x >> 6) == 0u) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");     // and the L2 is written back
        if (threadIdx.x == 0) {
            const uint32_t before = __hip_atomic_fetch_add(rp.dev + RD_CORES, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
            if (before == gridDim.x - 1u) {
                // the last core: the graph is complete.  The host reads results and the status after it has seen the number.
                __hip_atomic_store(rp.dev + RD_CORES, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (dev_load(rp.status + ST_ABORT) != 0u)      // the status words travel only when there is something to report
                    for (uint32_t i = 0; i < (uint32_t)ST_WORDS; i++)
                        __hip_atomic_store(rp.mailbox + MB_STATUS + i, dev_load(rp.status + i), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                __hip_atomic_store(rp.mailbox + MB_DONE, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
                __hip_atomic_store(rp.dev + RD_DONE, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        __syncthreads();
    }
}

hipError_t launch_resident(const ResidentParams &rp, uint32_t n_cores, uint32_t n_waves, size_t lds_bytes, hipStream_t stream) {
    hipError_t e = hipFuncSetAttribute((const void *)vdc_resident_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(vdc_resident_kernel, dim3(n_cores), dim3(n_waves * 64u), lds_bytes, stream, rp);
    return hipGetLastError();
}
#else
hipError_t launch_resident(const ResidentParams &, uint32_t, uint32_t, size_t, hipStream_t) { return hipErrorNotSupported; }
#endif

#if defined(VDC_SPLIT) && !defined(VDC_PROFILE)
// the variants are compiled in units of their own (see the end of the file): each exports the address of its kernel
#define VDC_DECLARE_PART(I) extern "C" const void *vdc_variant_entry_##I();
VDC_DECLARE_PART(0) VDC_DECLARE_PART(1) VDC_DECLARE_PART(2) VDC_DECLARE_PART(3) VDC_DECLARE_PART(4) VDC_DECLARE_PART(5)
VDC_DECLARE_PART(6) VDC_DECLARE_PART(7) VDC_DECLARE_PART(8)
#undef VDC_DECLARE_PART
static_assert(kNumVariants == 9, "one unit per variant");
static const void *variant_entry(int i) {
    switch (i) {
        case 0: return vdc_variant_entry_0();
        case 1: return vdc_variant_entry_1();
        case 2: return vdc_variant_entry_2();
        case 3: return vdc_variant_entry_3();
        case 4: return vdc_variant_entry_4();
        case 6: return vdc_variant_entry_6();
        case 7: return vdc_variant_entry_7();
        case 8: return vdc_variant_entry_8();
        default: return vdc_variant_entry_5();
    }
}
#else
template <int I>
static const void *variant_entry_at(int i) {
    if constexpr (I < kNumVariants) {
        if (i == I) return (const void *)vdc_executor_kernel<kVariants[I]>;
        return variant_entry_at<I + 1>(i);
    } else {
        return nullptr;
    }
}
static const void *variant_entry(int i) { return variant_entry_at<0>(i); }
#endif

hipError_t prepare_executor_kernels(size_t lds_bytes) {
    for (int i = 0; i < kNumVariants; i++) {
        hipError_t e = hipFuncSetAttribute(variant_entry(i), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_executor(const KParams &p, uint32_t n_cores, uint32_t n_waves, uint32_t ops, hipStream_t stream) {
#ifdef VDC_PROFILE
    const uint32_t waves = n_waves + 1u;   // one more: the observer
#else
    const uint32_t waves = n_waves;
#endif
    const size_t lds = lds_bytes_needed(p.n_slots, p.slot_bytes);
    // the first variant that has every handler the program needs; for a program whose regions all take one slot, the first
    // of the variants built for those, if one of them has
    const uint32_t fam = ops & ~OPS_ONE_SLOT;
    int pick = -1;
    if (ops & OPS_ONE_SLOT)
        for (int i = kNumVariants - 1; i >= 0; i--)
            if ((kVariants[i] & OPS_ONE_SLOT) && (fam & ~kVariants[i]) == 0u) pick = i;
    if (pick < 0)
        for (int i = kNumVariants - 1; i >= 0; i--)
            if (!(kVariants[i] & OPS_ONE_SLOT) && (fam & ~kVariants[i]) == 0u) pick = i;
    if (pick < 0) return hipErrorInvalidValue;
    KParams args = p;
    void *kargs[] = {&args};
    return hipLaunchKernel(variant_entry(pick), dim3(n_cores), dim3(waves * 64u), kargs, lds, stream);
}

hipError_t launch_clear(uint32_t *ptr, uint32_t n, hipStream_t stream) {
    hipLaunchKernelGGL(clear_kernel, dim3((n + 255u) / 256u), dim3(256), 0, stream, ptr, n);
    return hipGetLastError();
}

// What the memory uops are measured against (Section 6.3, "Memory virtual core overhead"): the same bytes moved by plain
// 128-bit load and store instructions, no virtual cores.  Every thread walks the range with the grid as its stride,
// four chunks per trip.
template <int MODE>
__global__ void __launch_bounds__(256) raw_stream_kernel(const u32x4 *src, u32x4 *dst, uint64_t chunks, uint32_t value, uint32_t *sink) {
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    const u32x4 fill = u32x4{value, value, value, value};
    uint32_t keep = 0;
    for (; i + 3u * stride < chunks; i += 4u * stride) {
        if (MODE == 1) {
#pragma unroll
            for (int q = 0; q < 4; q++) __builtin_nontemporal_store(fill, &dst[i + q * stride]);
        } else {
            u32x4 v[4];
#pragma unroll
            for (int q = 0; q < 4; q++) v[q] = __builtin_nontemporal_load(&src[i + q * stride]);
#pragma unroll
            for (int q = 0; q < 4; q++) {
                if (MODE == 2) __builtin_nontemporal_store(v[q], &dst[i + q * stride]);
                else keep |= v[q].x ^ v[q].y ^ v[q].z ^ v[q].w;
            }
        }
    }
    for (; i < chunks; i += stride) {
        if (MODE == 1) dst[i] = fill;
        else {
            const u32x4 v = src[i];
            if (MODE == 2) dst[i] = v;
            else keep |= v.x ^ v.y ^ v.z ^ v.w;
        }
    }
    // a read must leave a trace or the compiler drops it: the fold of everything read goes out when a flag in memory,
    // which the host keeps at zero, says so
    if (MODE == 0 && *sink != 0u) sink[1 + (blockIdx.x & 1u)] = keep;
}

hipError_t launch_raw_stream(int mode, const void *src, void *dst, uint64_t bytes, uint32_t value, uint32_t *sink, int blocks, hipStream_t stream) {
    const uint64_t chunks = bytes / 16u;
    if (mode == 0) hipLaunchKernelGGL(raw_stream_kernel<0>, dim3(blocks), dim3(256), 0, stream, (const u32x4 *)src, (u32x4 *)dst, chunks, value, sink);
    else if (mode == 1) hipLaunchKernelGGL(raw_stream_kernel<1>, dim3(blocks), dim3(256), 0, stream, (const u32x4 *)src, (u32x4 *)dst, chunks, value, sink);
    else hipLaunchKernelGGL(raw_stream_kernel<2>, dim3(blocks), dim3(256), 0, stream, (const u32x4 *)src, (u32x4 *)dst, chunks, value, sink);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Static scratch for the entry point that may not allocate (vdc_matvec_noalloc): the uop program, the workspace of a
// split-K program and the depId counters of one run live in this array instead of in allocated memory.  Every GPU holds
// its own copy at its own address for the life of the process.  In host code the array's name is only a stand-in for
// the symbol, not a device address: the address is asked for once per device (hipGetSymbolAddress) and kept; kernels
// and copies are always given that pointer.
// ------------------------------------------------------------------------------------------------
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kScratchBytes];

constexpr int kMaxScratchDevices = 64;
static void *g_scratch_ptr[kMaxScratchDevices] = {nullptr};

hipError_t scratch_address(int device, void **out) {
    *out = nullptr;
    if (device < 0 || device >= kMaxScratchDevices) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[device]) {
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) return e;
        if (cur != device) return hipErrorInvalidDevice;     // the symbol's address is the current device's
        void *ptr = nullptr;
        e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

hipError_t launch_debug_alloc(const uint32_t *masks, const int32_t *nslots, int32_t n_slots, int32_t *pos, int32_t n,
                              hipStream_t stream) {
    int blocks = n < 1024 ? (n > 0 ? n : 1) : 1024;
    hipLaunchKernelGGL(debug_alloc_kernel, dim3(blocks), dim3(64), 0, stream, masks, nslots, n_slots, pos, n);
    return hipGetLastError();
}

}  // namespace vdc
#endif   // VDC_PART
