/*
 * vdcores.h — C ABI of the VDCores executor for AMD MI355X (gfx950).
 *
 * The library runs micro-operation (uop) graphs on persistent "virtual cores":
 * one virtual memory core (VMC) and two virtual compute cores (VCC) per compute
 * unit, connected by the dependency queues m2c / c2m, as described in Sections
 * 3 ("Overview"), 4.1 ("Decoupled Model") and 4.3 ("GPU Executor") of the
 * VDCores paper.  The operator it ships is the paper's running example, the
 * tiled matrix-vector product O = M @ N (Section 3, "Execution Example";
 * Section 4.1, listing of the `matvec` compute uop).
 *
 * Conventions for every entry point
 *   - return value: 0 (VDC_OK) or a negative VDC_E* code; no exceptions, no
 *     global state; vdc_strerror() names a code.
 *   - "device" pointers are HIP device memory owned by the caller; the library
 *     never allocates, frees or copies the caller's tensors.  "host" pointers
 *     are ordinary memory read during the call only.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     vdc_run / vdc_matvec* enqueue work and return without synchronising.
 *   - outputs are overwritten, never accumulated into.
 *   - one executor must not be used from two host threads at once, and two
 *     runs of one executor must not overlap on the device (they share the
 *     depId table and the status buffer): enqueue them on one stream.
 */
#ifndef VDCORES_H
#define VDCORES_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    VDC_OK = 0,
    VDC_EINVAL = -1,    /* null or misaligned pointer, non-positive shape, unsupported size          */
    VDC_ENOMEM = -2,    /* host or device allocation failed                                        */
    VDC_EPROGRAM = -3,  /* the uop program is malformed (found by host-side validation)            */
    VDC_EDEVICE = -4,   /* a HIP call failed                                                       */
    VDC_EDEADLOCK = -5, /* the device watchdog fired: some unit waited longer than the spin limit  */
    VDC_ELEAK = -6,     /* a run ended with local-memory slots still allocated                      */
    VDC_ETOOBIG = -7,   /* vdc_matvec_noalloc: program + workspace exceed the static scratch        */
    VDC_ESTATE = -8,    /* the call does not fit the executor's state (vdc_resident_*)              */
    VDC_ETIMEOUT = -9   /* vdc_resident_wait: the graph was not complete within the time given      */
};

typedef struct vdc_executor vdc_executor; /* opaque, library-owned */
typedef struct vdc_program vdc_program;   /* opaque, library-owned device copy of a uop graph */

/* Deployment constants of the virtual cores.  Zero in any field selects the default, which is the
 * paper's deployment (Table 1 caption: 1 VMC + 2 VCCs per SM/CU, 8 KB slots; Section 4.3: 128
 * threads per execution unit, 32-bit slot mask). */
typedef struct {
    int32_t device;         /* HIP device ordinal; -1 => host-only executor (see vdc_create)           */
    int32_t n_cores;        /* virtual-core triples (workgroups); 0 => one per compute unit           */
    int32_t vcc_per_core;   /* 1 or 2; default 2                                                      */
    int32_t threads_per_eu; /* must be 128 (two wave64) or 0                                          */
    int32_t slot_bytes;     /* local-memory slot size, power of two, 1024..16384; default 8192        */
    int32_t n_slots;        /* slots per core, 1..32; default = as many as fit in the CU's LDS        */
    int32_t n_ldu;          /* load units per VMC: 1, 2 or 4; default 4                                   */
    int32_t n_stu;          /* store units per VMC: 1, 2 or 0 (=1); 2 needs vcc_per_core = 2: unit i  */
                            /* then serves compute core i, and a STORE must be on flow vflow % 2 = vcc */
    int32_t n_dep_ids;      /* size of the global depId table; default 4096                           */
    int32_t watchdog_spins; /* polls before a waiting unit reports VDC_EDEADLOCK; default 1<<22       */
    int32_t tile_rows;      /* tuning knob of the matvec tiler: rows per matrix tile; 0 => automatic  */
    int32_t issue_batch;    /* memory uops the front end dispatches at once at most, 1..8; 0 => 8.  For   */
                            /* measuring the issue path (Section 6.3); no effect on results              */
    int32_t issue_flags;    /* bit 0: the front end does not replay loop bodies, every trip is decoded   */
                            /* and dispatched through its general path (same purpose); bit 1: the matvec */
                            /* tiler gives eight vectors a vector tile over two steps where the shape    */
                            /* allows it (for measuring that form: slower); other bits zero              */
    int32_t sched_threshold_pct; /* adaptive tiling (Section 4.2): a critical path is dominant when it costs more  */
                            /* than (100 + this) % of the average per compute core; 0 => 10                   */
    int32_t sched_min_gain_pct;  /* a finer tiling is taken only if it shortens its operator by at least this many */
                            /* per cent of the path; 0 => 3                                                   */
    int32_t sched_force_parts;   /* 0: adaptive.  n = 1..16: no scheduling, every matvec cuts K into min(n, what it */
                            /* may) ranges; 100 + n: the same cut on the surplus row blocks alone where the   */
                            /* shape has a surplus.  For measuring the cost model; no effect on what is computed */
} vdc_config;

/* Create the executor on cfg->device (Section 4.3: the cores every run launches once as a persistent
 * kernel).  cfg may be NULL (all defaults).  *out is valid only when VDC_OK is returned.
 * With cfg->device == -1 the executor is host-only: it touches no GPU, assumes 160 KB of local memory and
 * cfg->n_cores cores (default 256), and serves only vdc_matvec_program, vdc_program_validate, vdc_get_config
 * and vdc_destroy; every entry point that needs the device returns VDC_EINVAL. */
int vdc_create(vdc_executor **out, const vdc_config *cfg);

/* Destroy the executor and every program created from it.  Waits for the device first. */
int vdc_destroy(vdc_executor *ex);

/* Fill *cfg with the values in effect (defaults resolved, n_cores = the CU count, ...). */
int vdc_get_config(const vdc_executor *ex, vdc_config *cfg);

/* ---- low level: uop graphs (Section 3: one uop stream per virtual core, the streams tied together by dependency edges) ----
 *
 * uops          host, n_uops words of 16 bytes (layout: csrc/vdc_isa.h)
 * stream_begin  host, n_cores*(1+vcc_per_core)+1 offsets into uops; stream index = core*(1+V) for the
 *               VMC of `core`, core*(1+V)+1+v for its VCC v; every stream ends with HALT
 * descs         host, n_descs descriptors of 32 bytes
 * tensor_bytes  host, n_tensors sizes in bytes of the tensors the program addresses (ids 0..n_tensors-1,
 *               at most 8); every memory uop is checked against them
 * The program is validated by walking every stream's control flow on the host: opcodes, loop nesting,
 * tensor bounds and alignment of every executed memory uop, unit and depId ranges, matvec geometry, and
 * the in-order slot demand of the paper's generator-side deadlock check (Section 4.2, "Dependency Graph
 * Lowering").  Anything wrong returns VDC_EPROGRAM and no program. */
int vdc_program_create(vdc_executor *ex, const void *uops, int64_t n_uops, const uint32_t *stream_begin,
                       const void *descs, int32_t n_descs, const int64_t *tensor_bytes, int32_t n_tensors,
                       vdc_program **out);
int vdc_program_destroy(vdc_program *prog);

/* Which units of a core share a SIMD of the compute unit (Section 4.3 maps the virtual cores onto the threads of one
 * thread block; on this GPU a workgroup's waves are dealt round-robin over four SIMDs, and waves on one SIMD contend for
 * its issue slots).  placement 0 (default): every SIMD holds one compute wave next to the memory core's units, best
 * when the compute cores set the pace.  placement 1: the front end and the store unit share their SIMDs with load
 * units only and the compute waves pair up, best for graphs with a store per tile.  placement 2: the workgroup is
 * launched with two more waves that leave at once, which shifts the others so that the front end shares its SIMD with
 * one compute wave and nothing else, the store unit likewise, and the other two SIMDs hold two load units and one
 * compute wave each: best for long loops over K, where the front end is the busiest wave.  No effect on results;
 * applies to the default deployment (4 load units, 1 store unit, 2 compute cores) and is ignored otherwise.  The
 * operators below choose for their own programs.  VDC_EINVAL for another value. */
int vdc_program_set_placement(vdc_program *prog, int32_t placement);

/* The validation of vdc_program_create alone (no device copy is made).  msg (host, may be NULL) receives a
 * NUL-terminated reason of at most msg_cap bytes when the result is VDC_EPROGRAM. */
int vdc_program_validate(vdc_executor *ex, const void *uops, int64_t n_uops, const uint32_t *stream_begin,
                         const void *descs, int32_t n_descs, const int64_t *tensor_bytes, int32_t n_tensors,
                         char *msg, int32_t msg_cap);

/* Run a program (Section 3: submit the uop graph to the on-GPU executors, which run until it finishes).
 * tensor_bases: host array of n_tensors device pointers, each at least as large as declared at
 * vdc_program_create; a tensor that some LOAD reads must be 16-byte aligned, any other 4-byte aligned
 * (VDC_EINVAL otherwise).  Asynchronous on hip_stream. */
int vdc_run(vdc_executor *ex, const vdc_program *prog, void *const *tensor_bases, int32_t n_tensors,
            void *hip_stream);

/* As vdc_run, and every unit also records the uops it executes, in its own program order:
 * trace (device, caller-owned): n_streams * trace_cap records of 4 x uint32
 *        { pc relative to the stream, opcode | desc<<8 | size<<16, low, high }
 *        (low, high) = effective byte offset into the tensor for LOAD/STORE, the uop's imm for MATVEC;
 * trace_count (device): n_streams uint32, the number of records each stream produced (records past
 *        trace_cap are counted but not written).  Only memory and compute uops are recorded. */
int vdc_run_traced(vdc_executor *ex, const vdc_program *prog, void *const *tensor_bases, int32_t n_tensors,
                   uint32_t *trace, uint32_t *trace_count, int32_t trace_cap, void *hip_stream);

/* Wait for hip_stream, then report what the cores wrote into the status buffer: VDC_OK, or the first
 * error a core raised (VDC_EDEADLOCK, VDC_ELEAK, VDC_EPROGRAM for a geometry the device rejected).
 * info (host, may be NULL) receives 4 words: core, role, stream pc, detail.  Clears the status. */
int vdc_sync_status(vdc_executor *ex, void *hip_stream, uint32_t *info);

/* ---- the resident form (Section 4.3: the virtual cores are launched once as a persistent kernel, and the runtime streams
 * new uop graphs to them as requests arrive) ----
 *
 * vdc_resident_start launches the cores on a stream of the library's own and leaves them up: between graphs they watch a
 * mailbox in pinned host memory.  vdc_resident_submit posts one graph (a program and its tensors, as for vdc_run) and
 * returns its ticket (1, 2, ...) without waiting; graphs run one after the other, in the order posted, each complete on
 * every core before the next starts, and one graph's stores are visible to the next: the results are those of as many
 * vdc_run calls on one stream, without a launch per graph.  At most 8 posted graphs may be incomplete (a further
 * submit waits for room).  vdc_resident_wait returns when graph `ticket` is complete: VDC_OK, the error the graph ended
 * in (VDC_EDEADLOCK, VDC_ELEAK, VDC_EPROGRAM; info as for vdc_sync_status), VDC_ETIMEOUT after timeout_ms, or
 * VDC_ESTATE when the cores have left without running it.  vdc_resident_stop tells the cores to leave, waits until they
 * have, and returns the executor to its ordinary state.
 * The cores never wait without a bound: when no graph arrives for idle_ms milliseconds (0: 1000; the bound is counted in
 * looks at the mailbox, so the time is approximate) they leave by themselves, as they do after a graph that ended in an
 * error; a caller that dies therefore leaves no kernel behind.  vdc_resident_state returns 0 (not started), 1 (up) or
 * 2 (the cores have left, or are leaving; vdc_resident_stop is still to be called) and the number of completed graphs.
 * While the cores are resident they hold every compute unit: vdc_run, the operators below, vdc_program_create and
 * vdc_program_destroy return VDC_ESTATE (programs are created before vdc_resident_start; a graph is a program plus
 * the tensors it is posted with, so one program serves any number of requests), other GPU work of the process that
 * needs a compute unit's whole local memory waits for them, and so may calls that allocate or free device or pinned
 * memory: buffers are allocated beforehand.
 * The caller's own streams are not involved: it waits with vdc_resident_wait before it touches a graph's results.  While
 * the cores are up, other GPU work of the process may wait until they have left: anything on the legacy default stream
 * (a blocking hipMemcpy included), and kernels, the runtime's small copies among them, that the runtime queues behind the
 * resident grid.  Results are therefore read after vdc_resident_stop, or a graph writes them where the host can see
 * them (an output tensor in pinned, mapped host memory: the cores' last stores are visible before the ticket is). */
int vdc_resident_start(vdc_executor *ex, int32_t idle_ms);
int vdc_resident_submit(vdc_executor *ex, const vdc_program *prog, void *const *tensor_bases, int32_t n_tensors,
                        uint32_t *ticket);
int vdc_resident_wait(vdc_executor *ex, uint32_t ticket, int32_t timeout_ms, uint32_t *info);
int vdc_resident_state(vdc_executor *ex, uint32_t *completed);
int vdc_resident_stop(vdc_executor *ex);

/* ---- high level: the matvec operator (Section 3, O = M @ N, the matrix cut into tiles along its row dimension) ----
 *
 * Y[b][i] = sum_j M[i*ld + j] * X[b*K + j],  0 <= i < rows, 0 <= b < B, fp32.
 * M, X, Y: device.  K and ld multiples of 4 (rows are moved in 16-byte units), ld >= K, 1 <= B <= 8,
 * M and X 16-byte aligned, Y 4-byte aligned.  tile_bytes = size of one matrix tile (the paper's I/O
 * block): 2048, 4096, 8192 or 16384.  The host tiler turns the call into a uop graph (cached per
 * shape), validates it and runs it.  Asynchronous on hip_stream.
 * The first call for a shape builds and uploads the program (device allocations, a synchronous copy); later calls
 * for the same shape only enqueue kernels, so a caller may capture them in a HIP graph.  The same holds for the
 * other operators below (vdc_matvec_rope, vdc_matvec_ragged, vdc_matvec_chain, vdc_attn_decode, vdc_stream).
 * Cache policy: an executor keeps at most 64 operator programs, keyed by everything the uop graph depends on (shapes,
 * tile size, every segment or context offset).  A call that needs a 65th destroys the least recently used one first,
 * which waits for the device.  A caller whose offsets change on every call (contexts that grow by a token per step)
 * therefore pays a rebuild per call; its memory use stays bounded. */
int vdc_matvec(vdc_executor *ex, const float *M, int64_t rows, int64_t K, int64_t ld, const float *X, float *Y,
               int32_t B, int32_t tile_bytes, void *hip_stream);

/* vdc_matvec for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same result, same kernels as vdc_matvec, but the call performs no
 * allocation of any kind on the device (no hipMalloc, hipFree, or library routine that allocates): the uop program,
 * the workspace of a shape that is also cut along K, the depId counters and the count of finished cores live in a
 * static device array of VDC_NOALLOC_SCRATCH_BYTES that every GPU the library runs on holds until the process ends
 * (its address, a pinned staging buffer and an event are obtained once, in vdc_create).  The program image (stream
 * offsets, descriptors, uops, workspace) must fit VDC_NOALLOC_SCRATCH_BYTES minus the 16 KB of counters, and the
 * program may use at most 4094 depIds: VDC_ETOOBIG otherwise, and nothing is enqueued.
 * The array is shared by all executors and all calls on that GPU and keeps the last call's content: a call with the
 * shape and executor configuration of the one before it reuses the program in place; any other shape is built on the
 * host and copied into the array asynchronously on hip_stream (the call first waits, on the host, for its staging
 * buffer's previous copy); the counters are put to zero by a fill kernel at the start of every call.  Calls that
 * overlap in time on one GPU (different streams, or different executors) race on the array: issue them on one stream.
 * Errors as vdc_matvec, plus VDC_ETOOBIG. */
#define VDC_NOALLOC_SCRATCH_BYTES (256 * 1024)
int vdc_matvec_noalloc(vdc_executor *ex, const float *M, int64_t rows, int64_t K, int64_t ld, const float *X, float *Y,
                       int32_t B, int32_t tile_bytes, void *hip_stream);

/* The running example of Section 3 in its fused form: O = M X as above, then R = rope(O, T), with O never leaving
 * local memory (Section 4.2: a store.local / load.local pair hands the matvec's output region to the rope uop of
 * the same compute core).  T: device, [B][rows] floats: for vector b and the pair of rows (2i, 2i+1), T[b][2i] is the
 * cosine and T[b][2i+1] the sine of the pair's angle;  Y[b][2i] = O[b][2i] cos - O[b][2i+1] sin,
 * Y[b][2i+1] = O[b][2i] sin + O[b][2i+1] cos.  rows must be a multiple of 4; T 16-byte aligned.  Dense only.
 * The tiler writes the two operators as they come (O stored to a temporary tensor, loaded back for rope) and the
 * generator's placement step turns every such pair into store.local / load.local; the temporary never exists. */
int vdc_matvec_rope(vdc_executor *ex, const float *M, int64_t rows, int64_t K, int64_t ld, const float *X,
                    const float *T, float *Y, int32_t B, int32_t tile_bytes, void *hip_stream);

/* Ragged batch: n_seg independent row segments stacked in M (rows row_off[s] .. row_off[s+1]-1, K floats
 * each, contiguous); segment s is multiplied by its own vector X[s][0..K).  Y[i] for every stacked row.
 * row_off: host, n_seg+1 non-decreasing offsets starting at 0.  The tiler splits long segments over the
 * cores (the paper's adaptive scheduling, Section 4.2) so that every core gets the same number of bytes. */
int vdc_matvec_ragged(vdc_executor *ex, const float *M, const int64_t *row_off, int32_t n_seg, int64_t K,
                      const float *X, float *Y, int32_t tile_bytes, void *hip_stream);

/* Emit the uop graph vdc_matvec / vdc_matvec_ragged would run, without running it (for tests and for
 * inspection).  Any output pointer may be NULL; counts are always written.  Buffers are host memory with
 * capacities *n_uops (16-byte words), *n_descs (32-byte descriptors) on entry; on return the needed counts.
 * stream_begin must hold n_cores*(1+vcc_per_core)+1 entries.  Returns VDC_EINVAL if a buffer is too small
 * (counts are still written).  row_off == NULL selects the dense operator (n_seg ignored). */
int vdc_matvec_program(vdc_executor *ex, int64_t rows, int64_t K, int64_t ld, int32_t B, int32_t tile_bytes,
                       const int64_t *row_off, int32_t n_seg, void *uops, int64_t *n_uops,
                       uint32_t *stream_begin, void *descs, int32_t *n_descs);

/* The same for vdc_matvec_rope (tensors 0 = M, 1 = X, 2 = Y, 3 = T). */
int vdc_matvec_rope_program(vdc_executor *ex, int64_t rows, int64_t K, int64_t ld, int32_t B, int32_t tile_bytes,
                            void *uops, int64_t *n_uops, uint32_t *stream_begin, void *descs, int32_t *n_descs);

/* Where the adaptive tiling step finds it worth while (vdc_matvec_tiling; Section 4.2), a dense matrix whose row blocks
 * do not fill the compute cores evenly is also cut along K, all its row blocks or the surplus ones: each (K range,
 * row block) pair is a work item, and the partial sums pass to the item of the last range through a library-owned workspace
 * with depId signals (Section 4.1, dependencies between memory uops; Section 4.3, the global depId queue).  The
 * emitted program then names a fourth tensor, 3 = the workspace.  This call gives its size in *bytes (0: the shape
 * is not split, the program uses tensors 0..2 only) and, if init != NULL, its initial content (host buffer of
 * capacity *bytes on entry).  vdc_matvec allocates and initialises the workspace itself; the call is for running
 * vdc_matvec_program's output elsewhere. */
int vdc_matvec_workspace(vdc_executor *ex, int64_t rows, int64_t K, int64_t ld, int32_t B, int32_t tile_bytes,
                         void *init, int64_t *bytes);

/* A chain of matvec operators as ONE uop graph and one launch (Section 3: operators are composed through their memory
 * uops, with no kernel boundary between them; Section 4.1: a memory uop may depend on one other through a depId):
 *     Y_0 = M_0 X,   Y_l = M_l Y_(l-1),   l = 1 .. L-1.
 * dims (host, L + 1 entries): dims[0] = columns of M_0, dims[l + 1] = rows of M_l; all multiples of 4.
 * W (device, 16-byte aligned): the matrices back to back, M_l as [dims[l + 1]][dims[l]] fp32, row-major.
 * A (device, 16-byte aligned): the activations back to back, X as [B][dims[0]], then every Y_l as [B][dims[l + 1]];
 *   the caller writes X, the run writes every Y_l (all of them stay readable).  1 <= B <= 8, L <= 64.
 * A layer starts on a group of (at most 32) vector tiles as soon as the row blocks of the layer before that produce them
 * have been stored: their stores signal the group's depId and the first load of the group waits for it; nothing waits
 * for a whole layer.  Needs one depId per group of layers 1 .. L-1 (n_dep_ids of the executor).  Asynchronous on hip_stream; programs are
 * cached by (dims, B, tile_bytes).  VDC_EINVAL for shapes the tiler cannot chain. */
int vdc_matvec_chain(vdc_executor *ex, const float *W, float *A, const int64_t *dims, int32_t L, int32_t B,
                     int32_t tile_bytes, void *hip_stream);

/* The uop program vdc_matvec_chain runs (tensors: 0 = W, 1 = A read, 2 = A written), handed out like
 * vdc_matvec_program does. */
int vdc_matvec_chain_program(vdc_executor *ex, const int64_t *dims, int32_t L, int32_t B, int32_t tile_bytes, void *uops,
                             int64_t *n_uops, uint32_t *stream_begin, void *descs, int32_t *n_descs);

/* Decode attention with one query per request over contexts of uneven length (Section 6.2, "Dynamic Attention
 * Length"), run as a uop graph around the attn compute uop (Section 4.1; a FlashAttention-style uop whose slots come
 * back in another order than they were allocated, Section 4.3):
 *     O[s][t] = sum_r p_r V[r][t],  p = softmax_r(scale * sum_j Q[s][j] K[r][j]),  r in [row_off[s], row_off[s + 1])
 * Q [n_seg][d], O [n_seg][d], K and V [row_off[n_seg]][d] (the contexts back to back): device, fp32, row-major,
 * 16-byte aligned, caller-owned; row_off: host, n_seg + 1 offsets, row_off[0] = 0, every request at least one row.
 * d = 128 or 64; tile_bytes in {4096, 8192, 16384} (tile_bytes / (4 d) context rows per key / value tile);
 * n_seg <= n_dep_ids.  scale > 0, or scale <= 0 for the usual d^(-1/2) (computed in fp32 as 1 / sqrtf(d)).
 * The tiles of all contexts, in order, are dealt to the compute cores in equal contiguous shares.  A context inside one
 * share is one item whose attn uop writes the request's result itself.  A context that crosses shares is cut where they
 * meet: its later items leave partial rows (weighted values, running maximum, running sum) in a library-owned workspace
 * and signal the request's depId; its first item loads those rows behind its last tile pair, joins them to its own
 * running state and writes the result (at most 64 partial rows per request; a longer context is cut into 65 equal
 * items).  fp32 arithmetic, exp() of differences to the running maximum only.
 * Asynchronous on hip_stream; programs are cached by (row_off, d, scale, tile_bytes).  Errors: VDC_EINVAL (arguments),
 * VDC_ENOMEM, VDC_EPROGRAM, VDC_EDEVICE. */
int vdc_attn_decode(vdc_executor *ex, const float *Q, const float *K, const float *V, const int64_t *row_off,
                    int32_t n_seg, int32_t d, float scale, float *O, int32_t tile_bytes, void *hip_stream);

/* The uop program vdc_attn_decode runs, handed out like vdc_matvec_program does.  Tensors: 0 = K, 1 = V, 2 = Q, 3 = O,
 * 4 = the workspace of *n_items rows of d + 4 floats (no initial content needed; one row per item that leaves a partial
 * row, at least one). */
int vdc_attn_decode_program(vdc_executor *ex, const int64_t *row_off, int32_t n_seg, int32_t d, float scale,
                            int32_t tile_bytes, void *uops, int64_t *n_uops, uint32_t *stream_begin, void *descs,
                            int32_t *n_descs, int64_t *n_items);

/* Memory uops with nothing to compute behind them (Section 6.3, "Memory virtual core overhead": the cost of the
 * memory core by I/O block size).  The byte range of `bytes` bytes is cut into blocks of tile_bytes, each moved by
 * one memory uop (the rest of the range: one shorter block of whole 1 KB rows, then one of a single short row); the
 * blocks are dealt to the compute cores in contiguous runs, and every compute core runs one uop that only pops and
 * returns regions.
 *   mode 0, read : every block of src is loaded into local memory and dropped; memory is left as it was.
 *   mode 1, fill : every 32-bit word of dst[0, bytes) becomes `value` (filled in local memory, then stored).
 *   mode 2, copy : dst[0, bytes) = src[0, bytes) (loaded, moved to an output region, stored); the ranges must not overlap.
 * src, dst: device, 16-byte aligned, caller-owned; the one the mode does not use is ignored.  bytes >= 16 and a
 * multiple of 16; tile_bytes a power of two, 256 .. 32768, that fits the slots (twice for copy).  Asynchronous on
 * hip_stream; programs are cached by (mode, bytes, value, tile_bytes).  VDC_EINVAL for anything else. */
int vdc_stream(vdc_executor *ex, int32_t mode, const void *src, void *dst, int64_t bytes, uint32_t value,
               int32_t tile_bytes, void *hip_stream);

/* What Section 6.3 measures the memory uops against: the same bytes moved by plain 128-bit load and store
 * instructions of an ordinary grid-stride kernel (no virtual cores, no local memory).  Modes, pointers, bytes and
 * value as for vdc_stream; a read folds what it loads into a word nobody looks at.  Asynchronous on hip_stream. */
int vdc_raw_stream(vdc_executor *ex, int32_t mode, const void *src, void *dst, int64_t bytes, uint32_t value,
                   void *hip_stream);

/* The uop program vdc_stream runs (tensors: 0 = src, or dst for fill; 1 = dst for copy), handed out like
 * vdc_matvec_program does. */
int vdc_stream_program(vdc_executor *ex, int32_t mode, int64_t bytes, uint32_t value, int32_t tile_bytes, void *uops,
                       int64_t *n_uops, uint32_t *stream_begin, void *descs, int32_t *n_descs);

/* ---- the generator's lowering steps (Section 4.2, "Dependency Graph Lowering" and "Dynamic Data Placement and Fusion") ----
 *
 * A uop graph before lowering: memory uops with literal addresses, written down in any order that keeps, per compute
 * core, the order in which that compute core takes their regions (that order is semantics); the compute cores' own
 * streams; and edges (store, load) "this load reads what that store wrote".  No flows, no depIds, no local placement. */
typedef struct {
    int32_t op;       /* 8 = LOAD, 9 = STORE                                                               */
    int32_t core;     /* memory core                                                                       */
    int32_t vcc;      /* compute core that takes (LOAD) or produces (STORE) the region                     */
    int32_t desc;     /* index into the descriptor table handed in                                         */
    int64_t offset;   /* byte offset in the descriptor's tensor                                            */
    int32_t rows;     /* valid rows of the box                                                             */
    int32_t nslots;   /* slots the box takes                                                               */
    int32_t group;    /* consumption group on its compute core: the regions one step of a compute uop holds
                         together carry one number, numbers do not decrease along the compute core's order */
    int32_t nt;       /* non-zero: streaming hint                                                          */
} vdc_graph_memop;

/* Lower a graph to bytecode for vdc_program_create, in the paper's steps:
 *   1. dynamic data placement: an edge whose store and load are neighbours on one compute core, move the same box of a
 *      tensor in `temp_tensors` (bit t = tensor t), and are each other's only producer / consumer becomes store.local /
 *      load.local (the descriptor then names `geom_tensor`: geometry only);
 *   2. virtual flow assignment: the loads of a compute core v from one tensor form a chain; chains take flows 2v, 2v+1
 *      in the order they first appear (further chains share the second); stores and local pairs take flow 2V + v;
 *   3. over-allocation: the stream of every memory core (the uops in the order given) is run without data under in-order
 *      slot allocation; if it deadlocks, every memory core's stream is merged again one consumption group at a time,
 *      round-robin over its compute cores;
 *   4. dependencies: every load with producers waits for one depId that all its producers signal (counted; a store
 *      signals one depId: VDC_EPROGRAM if its consumers do not share their producers), both sides marked device scope;
 *      a wait that an earlier load on the same flow of the same memory core already made is dropped.
 * ops (host, n_ops), edges (host, n_edges pairs of indices into ops: store, load), comp_uops / comp_begin (host: the
 * compute cores' streams, n_cores * vcc_per_core + 1 offsets, compute core (c, v) at index c * V + v; HALTs are added),
 * descs (host, n_descs of 32 bytes), tensor_bytes (host, n_tensors).  Outputs as vdc_matvec_program's (capacities in
 * *n_uops, *n_descs_out on entry, needed counts on return; descriptors are renumbered).  stats (host, may be NULL): 5
 * words: pairs placed, 1 if the streams were reordered, depIds used, waits kept, waits dropped.  The result has passed
 * the validation of vdc_program_create.  Errors: VDC_EINVAL, VDC_EPROGRAM (also: no order this step knows fits the slots). */
int vdc_graph_lower(vdc_executor *ex, const vdc_graph_memop *ops, int64_t n_ops, const int64_t *edges, int64_t n_edges,
                    const void *comp_uops, const uint32_t *comp_begin, const void *descs, int32_t n_descs,
                    uint32_t temp_tensors, int32_t geom_tensor, const int64_t *tensor_bytes, int32_t n_tensors,
                    void *uops_out, int64_t *n_uops, uint32_t *stream_begin, void *descs_out, int32_t *n_descs_out,
                    int32_t *stats);

/* ---- the generator's adaptive tiling step (Section 4.2, "Adaptive Scheduling and Tiling") ----
 *
 * The operators of a graph are scheduled onto the virtual cores in their coarsest decompositions; while the longest path
 * through the operator DAG costs more than the average per compute core by more than the threshold (a dominant critical
 * path), the operator on it whose finer tiling shortens it most takes that tiling, until the best gain is marginal or
 * nothing finer is left.  An operator is a matvec of n_blocks row blocks over nk tile steps of K; decomposition S cuts
 * the K range of every row block into S ranges (range s = steps [nk s / S, nk (s + 1) / S)), the items in the order
 * (range, row block) are dealt in contiguous shares (core c: items [NI c / C, NI (c + 1) / C), to its compute cores in
 * turn), the items of ranges 0 .. S - 2 store partial sums and signal, the item of the last range joins them,
 * join_group of them per extra step. */
typedef struct {
    int64_t n_blocks;   /* row blocks, >= 1                                                                   */
    int64_t nk;         /* tile steps along K per row block, >= 1                                             */
    int32_t max_parts;  /* finest decomposition the operator's builder offers, 1 .. nk                        */
    int32_t join_group; /* partial results that one joining step of the last range adds; 0 => 1                */
    int64_t surplus;    /* T > 0 (T < n_blocks): the builder offers every cut a second time for the last T row  */
                        /* blocks alone; the first n_blocks - T then stay whole and are dealt first, in shares  */
                        /* of their own.  0: no such decompositions                                             */
} vdc_sched_op;

typedef struct {        /* integers in one unit of the caller's choice (the library's own model: nanoseconds) */
    int64_t step;       /* one tile step of a compute core (matrix tile and vector tile loaded and used), >= 1 */
    int64_t item;       /* per work item on top of its steps: output region, row sums, store                  */
    int64_t join;       /* per joining step of an item of the last range                                      */
    int64_t edge;       /* from the end of a producing item to the moment the joining item can use its result */
} vdc_cost_model;

/* parts[o] (host, n_ops) = the decomposition S chosen for operator o, tails[o] (host, n_ops; may be NULL when no operator
 * has a surplus) = 0 when all its row blocks are cut, T when only its surplus is.  ops (host); pred_begin (host, n_ops + 1 offsets
 * into preds) and preds (host): the operators that must have ended before operator o starts, all with indices below o;
 * both may be NULL (no edges).  cost: NULL selects the library's model for tiles of tile_bytes (otherwise tile_bytes is
 * ignored).  Threshold and margin are the executor's (sched_threshold_pct, sched_min_gain_pct).  log (host, may be
 * NULL): 5 words per look at the graph: path cost, average per compute core, refined operator or -1, its new S, gain;
 * *n_looks: capacity in looks on entry, looks taken on return (n_looks may be NULL when log is).  Works on a host-only
 * executor.  VDC_EINVAL for anything malformed (an operator with more than 2^24 items among them). */
int vdc_schedule(vdc_executor *ex, const vdc_sched_op *ops, int32_t n_ops, const int32_t *pred_begin, const int32_t *preds,
                 const vdc_cost_model *cost, int32_t tile_bytes, int32_t *parts, int32_t *tails, int64_t *log, int32_t *n_looks);

/* What the matvec tiler decides for a dense shape (vdc_matvec, vdc_matvec_program): out (host, 7 words) = rows per
 * matrix tile, tile width in floats, row blocks, tile steps along K, the finest K cut the shape allows (1: the tiler
 * has no other decomposition for it), the cut taken, the number of trailing row blocks it is taken on (0: all).
 * Works on a host-only executor. */
int vdc_matvec_tiling(vdc_executor *ex, int64_t rows, int64_t K, int32_t B, int32_t tile_bytes, int64_t *out);

/* Run the slot allocator of the VMC (Section 4.3, "Virtual Memory Core": the first run of contiguous free slots in
 * the availability mask) on n independent (mask, nslots) requests with a pool of n_slots slots:
 * pos[i] = the lowest start of nslots[i] contiguous clear bits of masks[i], or -1.  masks, nslots, pos: device. */
int vdc_debug_alloc(vdc_executor *ex, const uint32_t *masks, const int32_t *nslots, int32_t n_slots, int32_t *pos,
                    int32_t n, void *hip_stream);

const char *vdc_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* VDCORES_H */
