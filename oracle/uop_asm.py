"""Assembler for micro-operation (uop) programs, oracle side.

Test infrastructure, not product code.  The paper names the fields of the
instruction word (Section 4.1: opcode, size, address, flags send/recv/dynamic,
depId, virtualFlowId) but fixes no widths; the layout used by this build is
restated here from its written description, independently of the product's
encoder, so that tests can build programs without touching product code.

Word (4 x uint32, little endian):
  w0  [7:0] opcode  [15:8] flags  [19:16] vflow  [21:20] vcc  [24:22] acc  [30:25] nslots
  w1  [15:0] size   [31:16] depId
  w2:w3 (64 bit)  [47:0] imm (signed)  [55:48] desc  [63:56] dep_count
Descriptor (8 x uint32): tensor, box_rows, row_bytes, lds_pitch, gpitch_lo, gpitch_hi, 0, 0
"""
import numpy as np

# opcodes
HALT, LOOP, REPEAT, ADD, SET = 0, 1, 2, 3, 4
CONTINUE_IF = 5      # the loop goes on while acc[acc] < imm; otherwise it is left: `size` = distance to its REPEAT
LOAD, STORE = 8, 9
MATVEC = 16
ROPE = 17
DROP, COPY, FILL = 18, 19, 20
ATTN, ATTN_MERGE = 21, 22

# flags
F_SEND, F_RECV, F_DYNAMIC, F_NT, F_DEP_SEND, F_DEP_RECV, F_LOCAL = 1, 2, 4, 8, 16, 32, 64
F_DEVICE = 128     # the access is made at device scope (a hint for real caches; no effect on the abstract machine)

MASK48 = (1 << 48) - 1


def word(opcode, flags=0, vflow=0, vcc=0, acc=0, nslots=0, size=0, dep_id=0, imm=0, desc=0, dep_count=0):
    assert 0 <= opcode < 256 and 0 <= flags < 256 and 0 <= vflow < 16 and 0 <= vcc < 4
    assert 0 <= acc < 8 and 0 <= nslots < 64 and 0 <= size < 65536 and 0 <= dep_id < 65536
    assert -(1 << 47) <= imm < (1 << 47) and 0 <= desc < 256 and 0 <= dep_count < 256
    w0 = opcode | (flags << 8) | (vflow << 16) | (vcc << 20) | (acc << 22) | (nslots << 25)
    w1 = size | (dep_id << 16)
    q = (imm & MASK48) | (desc << 48) | (dep_count << 56)
    return (w0, w1, q & 0xFFFFFFFF, q >> 32)


def descriptor(tensor, box_rows, row_bytes, lds_pitch, gpitch):
    assert 0 <= tensor < 256 and 0 < box_rows < (1 << 20) and 0 < row_bytes <= lds_pitch < 65536 and gpitch >= 0
    return (tensor, box_rows, row_bytes, lds_pitch, gpitch & 0xFFFFFFFF, gpitch >> 32, 0, 0)


def matvec_imm(B, R, lpr, xspan=0):
    """Static geometry of a MATVEC: B vectors, R box rows per matrix tile, lpr 16-byte chunks per tile row; xspan >= 2:
    one vector tile holds the pieces of xspan consecutive steps (B = 1: one per row; B > 1: B rows of xspan pieces)."""
    assert 1 <= B <= 8 and 1 <= R < 65536 and 1 <= lpr < 65536 and 0 <= xspan < 128
    return B | (R << 8) | (lpr << 24) | (xspan << 40)


def rope_imm(B, R):
    """Static geometry of a ROPE: B vectors, R values (R / 2 pairs) per vector in the tile."""
    assert 1 <= B <= 8 and 2 <= R < 65536 and R % 2 == 0
    return B | (R << 8)


def copy_imm(nbytes):
    """COPY: the first nbytes (a multiple of 16) of the loaded region go to the output region."""
    assert nbytes % 16 == 0 and 0 < nbytes // 16 < 65536
    return nbytes // 16


def fill_imm(value, nbytes):
    """FILL: the first nbytes (a multiple of 16) of the output region become copies of the 32-bit word `value`."""
    assert nbytes % 16 == 0 and 0 < nbytes // 16 < 32768 and 0 <= value < (1 << 32)
    return value | ((nbytes // 16) << 32)


def attn_imm(d, R, scale):
    """ATTN: head dimension d (a multiple of 4), R box rows per key / value tile, fp32 scale of the scores."""
    assert d % 4 == 0 and 0 < d // 4 < 256 and 0 < R < 256
    bits = int(np.array([scale], dtype=np.float32).view(np.uint32)[0])
    return (d // 4) | (R << 8) | (bits << 16)


class Program:
    """Per-unit uop streams of n_cores cores, each with one VMC stream and vcc_per_core VCC streams."""

    def __init__(self, n_cores, vcc_per_core=2):
        self.n_cores, self.V = n_cores, vcc_per_core
        self.streams = [[] for _ in range(n_cores * (1 + vcc_per_core))]
        self.descs = []

    def vmc(self, core):
        return self.streams[core * (1 + self.V)]

    def vcc(self, core, v):
        return self.streams[core * (1 + self.V) + 1 + v]

    def desc(self, *a, **k):
        d = descriptor(*a, **k)
        if d in self.descs:
            return self.descs.index(d)
        self.descs.append(d)
        return len(self.descs) - 1

    def finish(self):
        """Terminate every stream with HALT and return (words[n,4] u32, stream_begin[n_streams+1] u32, descs[n,8] u32)."""
        words, begin = [], [0]
        for s in self.streams:
            body = list(s)
            if not body or (body[-1][0] & 0xFF) != HALT:
                body.append(word(HALT))
            words.extend(body)
            begin.append(len(words))
        descs = self.descs if self.descs else [descriptor(0, 1, 4, 4, 0)]
        return (np.array(words, dtype=np.uint32).reshape(-1, 4), np.array(begin, dtype=np.uint32),
                np.array(descs, dtype=np.uint32).reshape(-1, 8))


def dense_matvec_program(rows, K, ld, B, R, Kt, slot_bytes, n_cores, vcc_per_core=2, nt=False, rope=False, xspan=0):
    """A straightforward dense Y = M X program in the form of the paper's listing (Section 4.1):
    row blocks of R rows are dealt round-robin to the (core, vcc) pairs; each row block is one MATVEC
    over ceil(K/Kt) (matrix tile, vector tile) pairs, followed by a send+recv STORE of the result.
    No loops, no accumulators: every address is a literal.  Tensors: 0 = M, 1 = X, 2 = Y.
    xspan >= 2 (K a multiple of Kt): one vector tile serves xspan consecutive steps (B = 1: xspan rows, one piece each;
    B > 1: B rows of xspan pieces side by side); it is loaded before the first matrix tile of those steps.

    rope=True builds the fused form of the running example of Section 3 (O = M @ N; R = rope(O, T)):
    the matvec result never goes to memory; a store.local / load.local pair hands its region on to a
    ROPE uop of the same compute core, which also gets the tile of tensor 3 = T ([B][rows], cos and
    sin interleaved per pair of rows) and writes its result to Y."""
    assert K % 4 == 0 and ld % 4 == 0 and Kt % 4 == 0
    p = Program(n_cores, vcc_per_core)
    lpr = Kt // 4
    nk = -(-K // Kt)
    m_slots = -(-R * Kt * 4 // slot_bytes)
    x_slots = -(-B * Kt * 4 // slot_bytes)
    y_slots = -(-B * R * 4 // slot_bytes)
    nrb = -(-rows // R)
    for rb in range(nrb):
        unit = rb % (n_cores * vcc_per_core)
        core, v = unit // vcc_per_core, unit % vcc_per_core
        r0 = rb * R
        rv = min(R, rows - r0)
        vm = p.vmc(core)
        for kt in range(nk):
            k0 = kt * Kt
            kv = min(Kt, K - k0)
            dm = p.desc(0, R, kv * 4, Kt * 4, ld * 4)
            dx = p.desc(1, B, kv * 4, Kt * 4, K * 4)
            if xspan >= 2 and kt % xspan == 0:
                assert K % Kt == 0
                steps = min(xspan, nk - kt)
                if B == 1:
                    dxs = p.desc(1, xspan, Kt * 4, Kt * 4, Kt * 4)      # xspan pieces of the vector, one per row
                    vm.append(word(LOAD, F_SEND, vflow=2 * v + 1, vcc=v, nslots=-(-xspan * Kt * 4 // slot_bytes), size=steps,
                                   imm=k0 * 4, desc=dxs))
                else:
                    dxs = p.desc(1, B, steps * Kt * 4, xspan * Kt * 4, K * 4)   # B rows, the pieces of the steps side by side
                    vm.append(word(LOAD, F_SEND, vflow=2 * v + 1, vcc=v, nslots=-(-B * xspan * Kt * 4 // slot_bytes), size=B,
                                   imm=k0 * 4, desc=dxs))
            vm.append(word(LOAD, F_SEND | (F_NT if nt else 0), vflow=2 * v, vcc=v, nslots=m_slots, size=rv,
                           imm=(r0 * ld + k0) * 4, desc=dm))
            if xspan < 2:
                vm.append(word(LOAD, F_SEND, vflow=2 * v + 1, vcc=v, nslots=x_slots, size=B, imm=k0 * 4, desc=dx))
        dy = p.desc(2, B, rv * 4, R * 4, rows * 4)
        if rope:
            assert rv % 2 == 0 and (rv * 4) % 16 == 0
            do = p.desc(2, B, R * 4, R * 4, rows * 4)        # geometry of the region that is handed on (no memory access)
            dt = p.desc(3, B, rv * 4, R * 4, rows * 4)
            vm.append(word(STORE, F_SEND | F_RECV | F_LOCAL, vflow=4 + v, vcc=v, nslots=y_slots, size=B, imm=0, desc=do))
            vm.append(word(LOAD, F_SEND | F_LOCAL, vflow=4 + v, vcc=v, nslots=0, size=B, imm=0, desc=do))
            vm.append(word(LOAD, F_SEND, vflow=2 * v + 1, vcc=v, nslots=y_slots, size=B, imm=r0 * 4, desc=dt))
        vm.append(word(STORE, F_SEND | F_RECV, vflow=4 + v, vcc=v, nslots=y_slots, size=B, imm=r0 * 4, desc=dy))
        p.vcc(core, v).append(word(MATVEC, size=nk, imm=matvec_imm(B, R, lpr, xspan)))
        if rope:
            p.vcc(core, v).append(word(ROPE, size=1, imm=rope_imm(B, R)))
    return p


def rowspan_matvec_program(row_off, K, ld, B, R, Kt, slot_bytes, n_cores, span, vcc_per_core=2):
    """Y = M X for a matrix whose K fits one tile (K <= Kt), dense (row_off = [0, rows], B vectors) or ragged
    (row_off = segment bounds, one vector per segment, B = 1), with MATVEC uops that cover up to `span` row blocks each:
    the blocks of a segment are taken `span` at a time; a group is one STORE of all its rows (first, so that the compute
    core holds the output region throughout), one LOAD of the vector tile, one LOAD per matrix tile, and one MATVEC whose
    descriptor field holds the number of blocks.  Groups are dealt round-robin to the (core, vcc) pairs; every address
    is a literal.  Tensors: 0 = M, 1 = X ([B][K] dense, [n_seg][K] ragged), 2 = Y ([B][rows] dense, [rows] ragged)."""
    assert K % 4 == 0 and ld % 4 == 0 and K <= Kt and span >= 2
    ragged = len(row_off) > 2
    assert not ragged or B == 1
    rows = row_off[-1]
    p = Program(n_cores, vcc_per_core)
    lpr = Kt // 4
    dx = p.desc(1, B, K * 4, Kt * 4, K * 4)
    g = 0
    for s in range(len(row_off) - 1):
        r = row_off[s]
        while r < row_off[s + 1]:
            n_rows = min(span * R, row_off[s + 1] - r)
            nb = -(-n_rows // R)
            unit = g % (n_cores * vcc_per_core)
            core, v = unit // vcc_per_core, unit % vcc_per_core
            vm = p.vmc(core)
            if nb == 1:      # a single block: the uop of the listing
                dy = p.desc(2, B, n_rows * 4, R * 4, (0 if ragged else rows) * 4)
                vm.append(word(LOAD, F_SEND, vflow=2 * v, vcc=v, nslots=-(-R * Kt * 4 // slot_bytes), size=n_rows, imm=r * ld * 4,
                               desc=p.desc(0, R, K * 4, Kt * 4, ld * 4)))
                vm.append(word(LOAD, F_SEND, vflow=2 * v + 1, vcc=v, nslots=-(-B * Kt * 4 // slot_bytes), size=B,
                               imm=(s * K * 4 if ragged else 0), desc=dx))
                vm.append(word(STORE, F_SEND | F_RECV, vflow=4 + v, vcc=v, nslots=-(-B * R * 4 // slot_bytes), size=B, imm=r * 4, desc=dy))
                p.vcc(core, v).append(word(MATVEC, size=1, imm=matvec_imm(B, R, lpr)))
            else:
                dy = p.desc(2, B, n_rows * 4, nb * R * 4, (0 if ragged else rows) * 4)
                vm.append(word(STORE, F_SEND | F_RECV, vflow=4 + v, vcc=v, nslots=-(-B * nb * R * 4 // slot_bytes), size=B, imm=r * 4, desc=dy))
                vm.append(word(LOAD, F_SEND, vflow=2 * v + 1, vcc=v, nslots=-(-B * Kt * 4 // slot_bytes), size=B,
                               imm=(s * K * 4 if ragged else 0), desc=dx))
                for j in range(nb):
                    rv = min(R, n_rows - j * R)
                    vm.append(word(LOAD, F_SEND, vflow=2 * v, vcc=v, nslots=-(-R * Kt * 4 // slot_bytes), size=rv,
                                   imm=(r + j * R) * ld * 4, desc=p.desc(0, R, K * 4, Kt * 4, ld * 4)))
                p.vcc(core, v).append(word(MATVEC, size=1, imm=matvec_imm(B, R, lpr), desc=nb))
            r += n_rows
            g += 1
    return p


def looped_matvec_program(rows, K, ld, B, R, Kt, slot_bytes, n_cores, vcc_per_core=2, nt=False):
    """The same product as dense_matvec_program, written the way Section 5 ("Dynamic address
    generation") describes recurring patterns: a LOOP/REPEAT nest whose memory uops carry the
    `dynamic` flag and take their offset from accumulators that control uops advance.
    Requires rows % R == 0, K % Kt == 0 and rows/R divisible by the number of (core, vcc) pairs,
    so that every unit runs the same nest on a contiguous range of row blocks.
    Accumulators: 0 = matrix offset, 1 = vector offset, 2 = result offset."""
    units = n_cores * vcc_per_core
    nrb = rows // R
    assert rows % R == 0 and K % Kt == 0 and nrb % units == 0
    per = nrb // units
    nk = K // Kt
    p = Program(n_cores, vcc_per_core)
    lpr = Kt // 4
    m_slots = -(-R * Kt * 4 // slot_bytes)
    x_slots = -(-B * Kt * 4 // slot_bytes)
    y_slots = -(-B * R * 4 // slot_bytes)
    dm = p.desc(0, R, Kt * 4, Kt * 4, ld * 4)
    dx = p.desc(1, B, Kt * 4, Kt * 4, K * 4)
    dy = p.desc(2, B, R * 4, R * 4, rows * 4)
    for core in range(n_cores):
        vm = p.vmc(core)
        # the two compute cores of a memory core are served one after the other, row block by row block
        for v in range(vcc_per_core):
            first = (core * vcc_per_core + v) * per          # first row block of this unit
            vm.append(word(SET, acc=0, imm=first * R * ld * 4))
            vm.append(word(SET, acc=1, imm=0))
            vm.append(word(SET, acc=2, imm=first * R * 4))
            vm.append(word(LOOP, imm=per))
            vm.append(word(LOOP, imm=nk))
            vm.append(word(LOAD, F_SEND | F_DYNAMIC | (F_NT if nt else 0), vflow=2 * v, vcc=v, acc=0,
                           nslots=m_slots, size=R, imm=0, desc=dm))
            vm.append(word(LOAD, F_SEND | F_DYNAMIC, vflow=2 * v + 1, vcc=v, acc=1, nslots=x_slots, size=B,
                           imm=0, desc=dx))
            vm.append(word(ADD, acc=1, imm=Kt * 4))
            vm.append(word(REPEAT, acc=0, imm=Kt * 4))
            vm.append(word(STORE, F_SEND | F_RECV | F_DYNAMIC, vflow=4 + v, vcc=v, acc=2, nslots=y_slots, size=B,
                           imm=0, desc=dy))
            vm.append(word(ADD, acc=1, imm=-K * 4))
            vm.append(word(ADD, acc=2, imm=R * 4))
            vm.append(word(REPEAT, acc=0, imm=(R * ld - K) * 4))
            vc = p.vcc(core, v)
            vc.append(word(LOOP, imm=per))
            vc.append(word(MATVEC, size=nk, imm=matvec_imm(B, R, lpr)))
            vc.append(word(REPEAT, acc=0, imm=0))
    return p


def stream_program(mode, nbytes, tile_bytes, slot_bytes, n_cores, vcc_per_core=2, value=0, row_bytes=1024):
    """Memory uops with no arithmetic behind them (Section 6.3, "Memory virtual core overhead"): the
    byte range [0, nbytes) is cut into blocks of tile_bytes, dealt round-robin to the (core, vcc) pairs.
    mode "read": every block is loaded and dropped (tensor 0).  mode "fill": every block of tensor 0 is
    written with copies of `value`.  mode "copy": every block of tensor 0 is loaded, moved to an output
    region and stored to the same place in tensor 1.  A block is a box of tile_bytes / row_bytes rows;
    the last block may have fewer rows, and a rest shorter than a row is a block of one short row.
    Every address is a literal."""
    assert mode in ("read", "fill", "copy")
    assert nbytes % 16 == 0 and tile_bytes % row_bytes == 0 and row_bytes % 16 == 0
    p = Program(n_cores, vcc_per_core)
    rows = tile_bytes // row_bytes
    nslots = -(-tile_bytes // slot_bytes)
    blocks = []                                   # (offset, rows, row_bytes of this block)
    off = 0
    while nbytes - off >= row_bytes:
        r = min(rows, (nbytes - off) // row_bytes)
        blocks.append((off, r, row_bytes))
        off += r * row_bytes
    if off < nbytes:
        blocks.append((off, 1, nbytes - off))
    count = {}
    for i, (o, r, rb) in enumerate(blocks):
        unit = i % (n_cores * vcc_per_core)
        core, v = unit // vcc_per_core, unit % vcc_per_core
        vm = p.vmc(core)
        box_rows = rows if rb == row_bytes else 1
        ns = nslots if rb == row_bytes else -(-rb // slot_bytes)
        if mode != "fill":
            d = p.desc(0, box_rows, rb, rb, rb)
            vm.append(word(LOAD, F_SEND | F_NT, vflow=2 * v, vcc=v, nslots=ns, size=r, imm=o, desc=d))
        if mode != "read":
            d = p.desc(0 if mode == "fill" else 1, box_rows, rb, rb, rb)
            vm.append(word(STORE, F_SEND | F_RECV, vflow=4 + v, vcc=v, nslots=ns, size=r, imm=o, desc=d))
        # one compute uop per run of blocks of the same shape
        key = (core, v)
        nb = box_rows * rb
        last = count.get(key)
        if last is not None and last[1] == nb and last[0] < 65535:
            last[0] += 1
        else:
            if last is not None:
                _emit_stream_uop(p, core, v, mode, last, value)
            count[key] = [1, nb]
    for (core, v), last in count.items():
        _emit_stream_uop(p, core, v, mode, last, value)
    return p


def _emit_stream_uop(p, core, v, mode, last, value):
    n, nb = last
    if mode == "read":
        p.vcc(core, v).append(word(DROP, size=n))
    elif mode == "fill":
        p.vcc(core, v).append(word(FILL, size=n, imm=fill_imm(value, nb)))
    else:
        p.vcc(core, v).append(word(COPY, size=n, imm=copy_imm(nb)))


def attn_decode_program(row_off, d, R, slot_bytes, n_cores, vcc_per_core=2, chunk_tiles=4, scale=None, whole=False, join=False):
    """Decode attention with one query per request over ragged contexts (Section 6.2, "Dynamic Attention
    Length"), written as uops.  Tensors: 0 = K and 1 = V ([rows][d], the contexts back to back), 2 = Q
    ([n_seg][d]), 3 = O ([n_seg][d]), 4 = W, the partial rows ([n_items][d + 4]).  A context is cut into tiles of
    R rows and into items of chunk_tiles tiles; items are dealt round-robin to the (core, vcc) pairs.  An item
    loads its query row, its (key tile, value tile) pairs and stores its partial row, signalling the request's
    depId; request s is merged by pair s mod (number of pairs): a load.dep of its partial rows that waits for all
    of them, and the store of the result.  All merges come after all items in every stream, so a waiting load
    never stands in front of a producer.  Every address is a literal.  whole: a context of a single item is not merged;
    its ATTN gets a region of d values and writes the request's result itself (no partial row, no depId).  join: a
    context of several items has no ATTN_MERGE; its first item comes behind all other items of its stream (among the
    merges), loads the partial rows of the context's other items behind its last pair, waiting for all of them, joins
    them to its own state and writes the result."""
    n_seg = len(row_off) - 1
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    p = Program(n_cores, vcc_per_core)
    units = n_cores * vcc_per_core
    kv_slots = -(-R * d * 4 // slot_bytes)
    q_slots = -(-d * 4 // slot_bytes)
    w_slots = -(-(d + 4) * 4 // slot_bytes)
    steps = [[] for _ in range(units)]          # per pair: lists of memory uops dispatched together
    merges = [[] for _ in range(units)]
    finals = [[] for _ in range(units)]         # join: the items that wait for partial rows, behind every other item
    final_uops = [[] for _ in range(units)]
    item = 0                                    # partial rows so far
    dealt = 0                                   # items so far, partial or whole
    n_items = []
    for s in range(n_seg):
        L = int(row_off[s + 1] - row_off[s])
        tiles = -(-L // R)
        first_item = item
        n_cut = -(-tiles // chunk_tiles)
        for t0 in range(0, tiles, chunk_tiles):
            t1 = min(tiles, t0 + chunk_tiles)
            unit = dealt % units
            dealt += 1
            core, v = unit // vcc_per_core, unit % vcc_per_core
            joins = join and n_cut > 1 and t0 == 0          # the item that joins the others' partial rows and writes the result
            mine = finals[unit] if joins else steps[unit]
            dq = p.desc(2, 1, d * 4, d * 4, d * 4)
            mine.append([word(LOAD, F_SEND, vflow=2 * v + 1, vcc=v, nslots=q_slots, size=1, imm=s * d * 4, desc=dq)])
            for t in range(t0, t1):
                r0 = int(row_off[s]) + t * R
                rv = min(R, int(row_off[s + 1]) - r0)
                dk = p.desc(0, R, d * 4, d * 4, d * 4)
                dv = p.desc(1, R, d * 4, d * 4, d * 4)
                mine.append([word(LOAD, F_SEND | F_NT, vflow=2 * v, vcc=v, nslots=kv_slots, size=rv, imm=r0 * d * 4, desc=dk),
                             word(LOAD, F_SEND | F_NT, vflow=2 * v + 1, vcc=v, nslots=kv_slots, size=rv, imm=r0 * d * 4, desc=dv)])
            if joins:
                P = n_cut - 1
                assert P <= 255
                dt = p.desc(4, P, (d + 4) * 4, (d + 4) * 4, (d + 4) * 4)
                do = p.desc(3, 1, d * 4, d * 4, d * 4)
                t_slots = -(-P * (d + 4) * 4 // slot_bytes)
                mine.append([word(LOAD, F_SEND | F_DEP_RECV, vflow=2 * v + 1, vcc=v, nslots=t_slots, size=P, dep_id=s, dep_count=P,
                                  imm=item * (d + 4) * 4, desc=dt),
                             word(STORE, F_SEND | F_RECV, vflow=4 + v, vcc=v, nslots=q_slots, size=1, imm=s * d * 4, desc=do)])
                final_uops[unit].append(word(ATTN, size=t1 - t0, imm=attn_imm(d, R, scale), desc=P))   # the descriptor field of a compute uop: partial rows to join
                continue
            p.vcc(core, v).append(word(ATTN, size=t1 - t0, imm=attn_imm(d, R, scale)))
            if whole and tiles <= chunk_tiles:
                do = p.desc(3, 1, d * 4, d * 4, d * 4)
                steps[unit].append([word(STORE, F_SEND | F_RECV, vflow=4 + v, vcc=v, nslots=q_slots, size=1, imm=s * d * 4, desc=do)])
                continue
            dw = p.desc(4, 1, (d + 4) * 4, (d + 4) * 4, (d + 4) * 4)
            steps[unit].append([word(STORE, F_SEND | F_RECV | F_DEP_SEND, vflow=4 + v, vcc=v, nslots=w_slots, size=1, dep_id=s,
                                     imm=item * (d + 4) * 4, desc=dw)])
            item += 1
        n_items.append((first_item, 0 if join else item - first_item))
    for s in range(n_seg):
        first_item, P = n_items[s]
        if P == 0:
            continue                            # one of the request's items writes the result itself
        assert 1 <= P <= 255
        unit = s % units
        v = unit % vcc_per_core
        dt = p.desc(4, P, (d + 4) * 4, (d + 4) * 4, (d + 4) * 4)
        do = p.desc(3, 1, d * 4, d * 4, d * 4)
        t_slots = -(-P * (d + 4) * 4 // slot_bytes)
        merges[unit].append([word(LOAD, F_SEND | F_DEP_RECV, vflow=2 * v + 1, vcc=v, nslots=t_slots, size=P, dep_id=s, dep_count=P,
                                  imm=first_item * (d + 4) * 4, desc=dt),
                             word(STORE, F_SEND | F_RECV, vflow=4 + v, vcc=v, nslots=q_slots, size=1, imm=s * d * 4, desc=do)])
    for unit in range(units):                   # the compute streams: items first, then merges
        core, v = unit // vcc_per_core, unit % vcc_per_core
        for s in range(n_seg):
            if s % units == unit and n_items[s][1] > 0:
                p.vcc(core, v).append(word(ATTN_MERGE, size=n_items[s][1], imm=d // 4))
    for unit in range(units):
        p.vcc(unit // vcc_per_core, unit % vcc_per_core).extend(final_uops[unit])
    for core in range(n_cores):                 # the memory stream: the pairs' steps in turn
        for lists in (steps, merges, finals):
            mine = [lists[core * vcc_per_core + v] for v in range(vcc_per_core)]
            for i in range(max(len(x) for x in mine)):
                for x in mine:
                    if i < len(x):
                        p.vmc(core).extend(x[i])
    return p, item


def chain_matvec_program(dims, B, R, Kt, slot_bytes, n_cores, vcc_per_core=2):
    """A chain of matvec operators in ONE uop graph: Y_0 = M_0 X, Y_l = M_l Y_(l-1), every layer's tiles waiting only
    for the tiles of the layer before that they read (Section 4.1, "Encoding dependency in uop": a memory uop may depend
    on one other memory uop through a depId; Section 3: operators are composed by their memory uops, not by kernel
    boundaries).  dims = (K_0, rows_0, rows_1, ...): M_l is [dims[l + 1]][dims[l]].  Tensors: 0 = W, the matrices back
    to back; 1 and 2 = A, the activations back to back ([B][dims[0]] = X, then every Y_l as [B][dims[l + 1]]), read as
    tensor 1 and written as tensor 2.  Row blocks of R rows are dealt round-robin to the (core, vcc) pairs, layer after
    layer.  The vector tile kt of layer l + 1 is rows kt Kt .. kt Kt + Kt - 1 of Y_l: the Kt / R row blocks of layer
    l that produce them signal depId (l, kt) with their stores, and every load of that tile waits for all of them.
    Requires Kt % R == 0 and every dim a multiple of Kt.  Every address is a literal."""
    L = len(dims) - 1
    assert Kt % R == 0 and all(d % Kt == 0 for d in dims)
    p = Program(n_cores, vcc_per_core)
    units = n_cores * vcc_per_core
    m_slots = -(-R * Kt * 4 // slot_bytes)
    x_slots = -(-B * Kt * 4 // slot_bytes)
    y_slots = -(-B * R * 4 // slot_bytes)
    w_off = [0]
    a_off = [0]
    for l in range(L):
        w_off.append(w_off[-1] + dims[l + 1] * dims[l] * 4)
        a_off.append(a_off[-1] + B * dims[l] * 4)
    dep_base = [0]
    for l in range(L):
        dep_base.append(dep_base[-1] + dims[l + 1] // Kt)
    for l in range(L):
        K, rows = dims[l], dims[l + 1]
        nk = K // Kt
        dm = p.desc(0, R, Kt * 4, Kt * 4, K * 4)
        dx = p.desc(1, B, Kt * 4, Kt * 4, K * 4)
        dy = p.desc(2, B, R * 4, R * 4, rows * 4)
        for rb in range(rows // R):
            unit = rb % units
            core, v = unit // vcc_per_core, unit % vcc_per_core
            vm = p.vmc(core)
            for kt in range(nk):
                vm.append(word(LOAD, F_SEND | F_NT, vflow=2 * v, vcc=v, nslots=m_slots, size=R, imm=w_off[l] + (rb * R * K + kt * Kt) * 4, desc=dm))
                if l == 0:
                    vm.append(word(LOAD, F_SEND, vflow=2 * v + 1, vcc=v, nslots=x_slots, size=B, imm=kt * Kt * 4, desc=dx))
                else:
                    vm.append(word(LOAD, F_SEND | F_DEP_RECV | F_DEVICE, vflow=2 * v + 1, vcc=v, nslots=x_slots, size=B,
                                   dep_id=dep_base[l - 1] + kt, dep_count=Kt // R, imm=a_off[l] + kt * Kt * 4, desc=dx))
            last = l == L - 1
            vm.append(word(STORE, F_SEND | F_RECV | (0 if last else F_DEP_SEND | F_DEVICE), vflow=4 + v, vcc=v, nslots=y_slots, size=B,
                           dep_id=0 if last else dep_base[l] + rb * R // Kt, imm=a_off[l + 1] + rb * R * 4, desc=dy))
            p.vcc(core, v).append(word(MATVEC, size=nk, imm=matvec_imm(B, R, Kt // 4)))
    return p, w_off, a_off
