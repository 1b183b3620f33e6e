// Micro-operation (uop) instruction set of the executor: word layout, opcodes, flags, descriptors.
//
// The paper names the fields of the instruction word (Section 4.1: opcode, size, address, flags
// send / recv / dynamic, depId, virtualFlowId; Section 5: accumulator-relative dynamic addresses) but
// gives no widths; this is the layout this library defines.  Shared by the host side (tiler,
// validator) and the device side (decoders in the kernel) of the library.
#ifndef VDC_ISA_H
#define VDC_ISA_H

#include <stdint.h>

#if defined(__HIPCC__) || defined(__HIP__)
#define VDC_HD __host__ __device__ __forceinline__
#else
#define VDC_HD inline
#endif

namespace vdc {

enum Opcode : uint32_t {
    OP_HALT = 0,    // end of stream
    OP_LOOP = 1,    // push (pc + 1, imm trips)
    OP_REPEAT = 2,  // acc[a] += imm; next trip of the innermost loop or fall through
    OP_ADD = 3,     // acc[a] += imm
    OP_SET = 4,     // acc[a] = imm
    OP_CONTINUE_IF = 5,  // continue_if (Section 4.1): while acc[a] < imm nothing happens; otherwise the innermost loop is left:
                         // its frame is dropped and execution goes on behind its REPEAT, which stands `size` words further on
    OP_LOAD = 8,    // VMC: global -> local-memory region
    OP_STORE = 9,   // VMC: local-memory region -> global
    OP_MATVEC = 16, // VCC: the matvec compute uop of the listing in Section 4.1
    OP_ROPE = 17,   // VCC: the rope uop of the running example (Section 3): turn pairs of values by given angles
    // compute uops without arithmetic, for measuring memory uops alone (Section 6.3, "Memory virtual core overhead")
    OP_DROP = 18,   // VCC: pop `size` loaded regions, hand each back as used
    OP_COPY = 19,   // VCC: `size` times: pop a loaded region and an output region, move bytes across, hand both back
    OP_FILL = 20,   // VCC: pop `size` output regions, write one 32-bit word all over each, hand it back as produced
    // decode attention (the attn uop of Section 4.1; FlashAttention-style, slots freed out of order, Section 4.3)
    OP_ATTN = 21,        // VCC: pop the query tile and keep it; `size` times {pop a key tile, pop a value tile, update the
                         // running maximum m, sum l and weighted values o}; hand the query tile back; with a count P in the
                         // descriptor field (attn_join): pop one more tile, the P partial rows of the context's other
                         // items, and join them to (m, l, o); pop the output region: one row of d + 4 values takes the
                         // partial row (o[0..d), m, l, 0, 0), one row of d values the finished result o / l (the form after
                         // a join); hand it back as produced
    OP_ATTN_MERGE = 22   // VCC: pop a tile of `size` such rows of one request and an output region; write
                         // sum_i exp(m_i - M) o_i / sum_i exp(m_i - M) l_i, M = max_i m_i
};

enum Flag : uint32_t {
    F_SEND = 1,      // forward the region to local compute core `vcc` (m2c)
    F_RECV = 2,      // consume a region produced by local compute core `vcc` (c2m)
    F_DYNAMIC = 4,   // address = imm + acc[a]
    F_NT = 8,        // streaming hint for the load path; no semantic effect
    F_DEP_SEND = 16, // after completion: dep[depId] += 1
    F_DEP_RECV = 32, // before starting: wait until dep[depId] >= max(1, dep_count)
    F_DEVICE = 128,  // the access is made at device scope: a LOAD reads past caches that another core's store may have left
                     // stale, a STORE is written through.  For data that one core writes and another reads within a run
                     // (between a DEP_SEND store and the DEP_RECV loads behind it); no effect on the abstract machine
    F_LOCAL = 64     // store.local / load.local (Section 4.2): the region stays in local memory.  A STORE takes the
                     // produced region back and keeps it; the next LOAD with this flag on the same flow hands it to a
                     // compute core again (no allocation: nslots = 0; no memory access)
};

constexpr int kMaxLoopDepth = 4;
constexpr int kNumAcc = 8;
constexpr int kMaxTensors = 8;
constexpr int kMaxSlots = 32;   // 32-bit availability mask (Section 4.3)

struct Word {            // 16 bytes
    uint32_t w0, w1, w2, w3;
};

struct Desc {            // 32 bytes: the 2-D box a memory uop moves
    uint32_t tensor;     // tensor id
    uint32_t box_rows;   // rows of the local-memory box
    uint32_t row_bytes;  // valid bytes per row (multiple of 16 for LOAD, of 4 for STORE)
    uint32_t lds_pitch;  // bytes between rows in local memory (multiple of 16)
    uint32_t gpitch_lo;  // bytes between rows in global memory
    uint32_t gpitch_hi;
    uint32_t rsv0, rsv1;
};

struct Fields {
    uint32_t opcode, flags, vflow, vcc, acc, nslots, size, dep_id, desc, dep_count;
    int64_t imm;
};

VDC_HD Fields decode(const Word &w) {
    Fields f;
    f.opcode = w.w0 & 0xFFu;
    f.flags = (w.w0 >> 8) & 0xFFu;
    f.vflow = (w.w0 >> 16) & 0xFu;
    f.vcc = (w.w0 >> 20) & 0x3u;
    f.acc = (w.w0 >> 22) & 0x7u;
    f.nslots = (w.w0 >> 25) & 0x3Fu;
    f.size = w.w1 & 0xFFFFu;
    f.dep_id = w.w1 >> 16;
    uint64_t q = (uint64_t)w.w2 | ((uint64_t)w.w3 << 32);
    f.imm = (int64_t)(q << 16) >> 16;   // sign-extend 48 bits
    f.desc = (uint32_t)(q >> 48) & 0xFFu;
    f.dep_count = (uint32_t)(q >> 56);
    return f;
}

inline Word encode(uint32_t opcode, uint32_t flags, uint32_t vflow, uint32_t vcc, uint32_t acc, uint32_t nslots,
                   uint32_t size, uint32_t dep_id, int64_t imm, uint32_t desc, uint32_t dep_count) {
    Word w;
    w.w0 = (opcode & 0xFFu) | ((flags & 0xFFu) << 8) | ((vflow & 0xFu) << 16) | ((vcc & 0x3u) << 20) |
           ((acc & 0x7u) << 22) | ((nslots & 0x3Fu) << 25);
    w.w1 = (size & 0xFFFFu) | ((dep_id & 0xFFFFu) << 16);
    uint64_t q = ((uint64_t)imm & 0xFFFFFFFFFFFFull) | ((uint64_t)(desc & 0xFFu) << 48) |
                 ((uint64_t)(dep_count & 0xFFu) << 56);
    w.w2 = (uint32_t)q;
    w.w3 = (uint32_t)(q >> 32);
    return w;
}

// MATVEC imm: B [7:0], R [23:8] (box rows of a matrix tile), lpr [39:24] (16-byte chunks per tile row), xspan [46:40]:
// 0 or 1 = a vector tile per step; n >= 2 (n <= kMaxXspan; B = 1, or matvec_xspan_ok) = one vector tile of n rows serves n consecutive
// steps, row j step j: it is popped before the first matrix tile of those steps and handed back after the last.
constexpr uint32_t kMaxXspan = 8;
// With several vectors (the tile then holds B rows of n pieces side by side) the compute uop has the form for B = 8 and
// tiles of 512 or 1024 chunks whose rows lie inside one wave.
VDC_HD bool matvec_xspan_ok(uint32_t B, uint32_t R, uint32_t lpr) {
    return B == 1u || (B == 8u && lpr <= 64u && (R * lpr == 512u || R * lpr == 1024u));
}
inline int64_t matvec_imm(uint32_t B, uint32_t R, uint32_t lpr, uint32_t xspan = 0) {
    return (int64_t)B | ((int64_t)R << 8) | ((int64_t)lpr << 24) | ((int64_t)xspan << 40);
}
VDC_HD uint32_t matvec_xspan(int64_t imm) { return (uint32_t)(imm >> 40) & 0x7Fu; }
// MATVEC over several row blocks (when K fits one tile): a compute uop names no descriptor, and on a MATVEC the field
// [55:48] counts the row blocks the uop covers: 0 or 1 = the uop of the listing; n >= 2 (n <= kMaxRowspan, size = 1, no
// xspan, lpr <= 64, B <= kMaxRowspanB) = n blocks of R rows that share one vector tile.  The uop pops its output region first and keeps it
// ([B][n * R] fp32, row pitch n * R * 4: one STORE for all the blocks), then the vector tile, then n matrix tiles, block
// j giving rows j * R ..; every matrix tile goes back when it is done, the vector tile after the last, then the region
// as produced.
constexpr uint32_t kMaxRowspan = 16;
constexpr uint32_t kMaxRowspanB = 4;    // vectors a MATVEC over several row blocks takes at most
VDC_HD uint32_t matvec_rowspan(const Fields &f) { return f.desc; }
// A compute uop names no descriptor: on an ATTN the field counts the partial rows of the context's other items that the uop
// joins to its own running state behind its last pair (0: none).
VDC_HD uint32_t attn_join(const Fields &f) { return f.desc; }

// ROPE imm: B [7:0], R [23:8]: the value tile, the tile of (cos, sin) pairs and the output region are all [B][R]
// fp32 with a row pitch of R * 4 bytes; R even, B * R <= 1024
inline int64_t rope_imm(uint32_t B, uint32_t R) { return (int64_t)B | ((int64_t)R << 8); }
inline bool rope_geometry_ok(uint32_t B, uint32_t R) { return B >= 1 && B <= 8 && R >= 2 && (R & 1u) == 0 && B * R <= 1024; }

// COPY imm: chunks [15:0]; FILL imm: value [31:0], chunks [47:32]; a chunk is 16 bytes, counted from the start of the
// region.  1 <= chunks, and the bytes must fit the region (checked against the allocation when the program is created).
inline int64_t copy_imm(uint32_t chunks) { return (int64_t)chunks; }
inline int64_t fill_imm(uint32_t value, uint32_t chunks) { return (int64_t)value | ((int64_t)chunks << 32); }
constexpr uint32_t kMaxStreamChunks = 2048;   // 32 KB: sixteen passes of the 128 threads of an execution unit

// ATTN imm: lpr [7:0] = d / 4 (16-byte chunks per row of a key / value tile), R [15:8] (box rows of those tiles), the bits
// of the fp32 factor on the scores [47:16].  ATTN_MERGE imm: lpr [7:0].  Supported: d = 128 (lpr = 32) with R in {8, 16, 32}
// and d = 64 (lpr = 16) with R in {16, 32, 64} (tiles of 4, 8, 16 KB), at most 64 partial rows per merge.
inline int64_t attn_imm(uint32_t lpr, uint32_t R, uint32_t scale_bits) { return (int64_t)lpr | ((int64_t)R << 8) | ((int64_t)scale_bits << 16); }
inline bool attn_geometry_ok(uint32_t lpr, uint32_t R) {
    return (lpr == 32 && (R == 8 || R == 16 || R == 32)) || (lpr == 16 && (R == 16 || R == 32 || R == 64));
}
constexpr uint32_t kAttnMaxPartials = 64;

// The compute uop works on `threads_per_eu` = 128 threads; a matrix tile is NF passes of 128 chunks of
// 16 bytes.  Supported geometries (anything else is rejected when the program is created):
//   lpr in {1,2,4,...,64}  : a tile row lies inside one wave  (mode J = 0), R*lpr = NF*128
//   lpr = 128*J, J in {1,2,4,8}: a tile row spans J passes of all 128 threads, R*J = NF
//   NF in {1,2,4,8} (tiles of 2, 4, 8, 16 KB), 1 <= B <= 8, and J*B <= 16 (vector registers)
inline bool matvec_geometry_ok(uint32_t B, uint32_t R, uint32_t lpr, uint32_t *nf_out, uint32_t *j_out) {
    if (B < 1 || B > 8 || R < 1 || lpr < 1) return false;
    uint64_t chunks = (uint64_t)R * lpr;
    if (chunks % 128 != 0) return false;
    uint32_t nf = (uint32_t)(chunks / 128);
    if (nf != 1 && nf != 2 && nf != 4 && nf != 8) return false;
    uint32_t j = 0;
    if (lpr <= 64) {
        if (lpr & (lpr - 1)) return false;
    } else {
        if (lpr % 128) return false;
        j = lpr / 128;
        if (j != 1 && j != 2 && j != 4 && j != 8) return false;
        if (j > nf || j * B > 16) return false;
    }
    if (nf_out) *nf_out = nf;
    if (j_out) *j_out = j;
    return true;
}

}  // namespace vdc
#endif
