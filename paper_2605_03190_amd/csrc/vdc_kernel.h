// Interface between the host side of the library and its device code: kernel parameters and launchers.
#ifndef VDC_KERNEL_H
#define VDC_KERNEL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vdc_isa.h"

namespace vdc {

// Words of the device status buffer (global memory, one per executor).
enum StatusWord : int {
    ST_ABORT = 0,   // non-zero once any core has raised an error: every spin loop on the device polls it
    ST_CODE = 1,    // the VDC_E* code (stored negated, i.e. positive)
    ST_CORE = 2,
    ST_ROLE = 3,    // see Role
    ST_PC = 4,      // stream-relative pc of the uop the unit was at
    ST_DETAIL = 5,
    ST_WORDS = 8
};

enum Role : uint32_t { ROLE_CFU = 0, ROLE_LDU = 1, ROLE_STU = 2, ROLE_VCC = 3 };

struct KParams {
    const Word *words;
    const uint32_t *stream_begin;
    const Desc *descs;
    uint32_t n_descs;
    char *tensors[kMaxTensors];
    uint32_t *dep;          // depId counters
    uint32_t *finished;     // cores whose store unit has left (the last one clears the counters the program uses)
    uint32_t n_dep_used;    // depId counters the program uses (0: none)
    uint64_t wave_roles;    // four bits per wave of the workgroup: the position in the role order (front end, load units,
                            // store units, compute waves) that this wave takes
    uint32_t *status;       // ST_WORDS words
    const uint32_t *seq_table;  // kSeqTableWords words, word i = i: where the load units fetch the sequence numbers that
                                // mark a loaded tile ready (the kernel's M2cEnt explains)
    uint32_t *trace;        // optional: n_streams * trace_cap * 4 words
    uint32_t *trace_count;  // optional: n_streams words
    uint32_t trace_cap;
    uint32_t n_slots, slot_bytes, n_ldu, n_stu, V;
    uint32_t watchdog;
    uint32_t issue_batch;   // memory uops the front end dispatches at once at most (1..8)
    uint32_t no_replay;     // the front end decodes and dispatches every trip of a loop through its general path
#if defined(VDC_PROFILE) || defined(VDC_PROFILE_WAITS)
    unsigned long long *prof;   // cores * 8 waves * 8 counters (profiling builds only)
#endif
};

constexpr uint32_t kSeqTableWords = 2052;

// The resident form of the executor: the grid stays up and takes uop graphs from a mailbox in pinned host memory.
// Mailbox (words): MB_TAIL graphs posted so far, MB_STOP non-zero = leave, MB_DONE graphs completed so far, MB_STATE
// 1 = the grid is up, 2 = it has left (or is leaving), MB_STATUS.. the status words after the last completed graph,
// MB_JOBS.. kResidentJobs entries of kResidentJobWords words, graph seq in entry seq % kResidentJobs: its KParams.
// Device words: RD_JOB.. the parameter block of the graph being run, RD_TAIL the graph every wave may start (or STOP),
// RD_CORES cores done with it, RD_DONE graphs completed so far.
enum : uint32_t { MB_TAIL = 0, MB_STOP = 1, MB_DONE = 2, MB_STATE = 3, MB_STATUS = 8, MB_JOBS = 64 };
enum : uint32_t { RD_JOB = 0, RD_TAIL = 64, RD_CORES = 65, RD_DONE = 66, RD_WORDS = 128 };
constexpr uint32_t kResidentJobs = 8, kResidentJobWords = 64;
struct ResidentParams {
    uint32_t *mailbox;        // pinned host memory, MB_JOBS + kResidentJobs * kResidentJobWords words
    uint32_t *dev;            // device memory, RD_WORDS words, zero at the launch
    uint32_t *status;         // the executor's status words
    uint32_t idle_polls;      // looks of the watcher without a new graph before the grid leaves by itself
    uint32_t backstop_polls;  // bound of every other wait between graphs
};
hipError_t launch_resident(const ResidentParams &rp, uint32_t n_cores, uint32_t n_waves, size_t lds_bytes, hipStream_t stream);

// Bytes of dynamic LDS one workgroup needs for n_slots slots of slot_bytes plus the control block.
size_t lds_bytes_needed(uint32_t n_slots, uint32_t slot_bytes);
size_t lds_control_bytes();

// Launch the persistent virtual-core kernel: one workgroup per core.
// The families of compute uops a program uses: the kernel is built in several variants, each with the handlers of some
// families only, and a program is launched on the smallest variant that has all of its own.
enum : uint32_t { OPS_MATVEC = 1, OPS_ROWS = 2, OPS_ROPE = 4, OPS_STREAM = 8, OPS_ATTN = 16, OPS_ALL = 31 };
// beside the families, in a program's `ops`: every region of the program takes one slot (tiles of a slot at most: the
// compute waves' fixed work per tile sets the pace there, and the variants of the kernel built for it pay)
constexpr uint32_t OPS_ONE_SLOT = 0x80000000u;
hipError_t launch_executor(const KParams &p, uint32_t n_cores, uint32_t n_waves, uint32_t ops, hipStream_t stream);
// Raise the kernel's dynamic LDS limit; call once per device before the first launch.
hipError_t prepare_executor_kernels(size_t lds_bytes);
// Zero n words (a fill kernel; safe inside stream capture, unlike a memset node).
hipError_t launch_clear(uint32_t *p, uint32_t n, hipStream_t stream);
hipError_t launch_raw_stream(int mode, const void *src, void *dst, uint64_t bytes, uint32_t value, uint32_t *sink, int blocks,
                             hipStream_t stream);
// The static device array behind the entry point that allocates nothing: kScratchBytes per GPU, laid out as
// [0, kScratchDepBytes) depId counters and the count of finished cores, then the program image (stream_begin,
// descriptors, uops, workspace).  scratch_address gives the array's address on `device`, which must be the current
// device on the first call for it; the address is kept per device.
constexpr size_t kScratchBytes = 256u << 10;
constexpr size_t kScratchDepBytes = 16u << 10;     // 4095 depId counters + the finished-cores word
hipError_t scratch_address(int device, void **out);
hipError_t launch_debug_alloc(const uint32_t *masks, const int32_t *nslots, int32_t n_slots, int32_t *pos, int32_t n,
                              hipStream_t stream);

}  // namespace vdc
#endif
