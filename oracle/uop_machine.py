"""Sequential CPU interpreter of the decoupled abstract machine.

Test infrastructure, not product code.  It follows the paper's description of the
machine in the paper's order and vocabulary and shares nothing with the HIP path:

* Section 4.1 ("Abstraction of GPU Hardware"): every core is a small register machine
  running its own uop stream: memory and control uops on the virtual memory core (VMC),
  compute and control uops on each virtual compute core (VCC).
* Section 4.1 ("Encoding dependency in uop"): a memory uop forwards its region to a local
  VCC when it carries `send`, consumes a region from a local VCC when it carries `recv`,
  and has at most one dependency on another memory uop, named by `depId`.
* Section 4.1 ("Virtual-flow-based execution") and Section 4.3 ("Parallel virtual flow
  execution"): uops of one virtual flow go to one load/store unit and run in order there;
  different flows may overlap.
* Section 4.3 ("Virtual Memory Core"): a front end (CFU) keeps register state, runs control
  uops and generates addresses, then issues to load units (LDU) and store units (STU);
  local memory is handed out in slots tracked by a 32-bit mask; a request takes the first
  run of contiguous free slots.
* Section 4.3 ("Dependency Resolving"): FIFO queues m2c (VMC to VCC: loaded regions) and
  c2m (VCC to VMC: used or produced regions); a global table indexed by depId between VMCs.
* Section 4.3 ("Avoiding Deadlock"): slots are allocated in program order; everything
  after allocation may complete out of order.
* Section 5 ("Dynamic address generation"): with `dynamic`, the address field is offset by
  an accumulator register that control uops update.
* Section 4.1 names `continue_if` beside `loop` among the control uops that run on every kind of
  core and says no more about it.  Reading taken here: a condition on a register decides whether
  the innermost loop goes on.  While acc[acc] < imm the uop does nothing; otherwise the loop is
  left at once (its frame is dropped, execution continues behind its REPEAT, `size` words on).
* Section 4.1, listing of the `matvec` compute uop: for each of `size` tiles pop a matrix
  tile and a vector tile from m2c, accumulate, push both to c2m; then pop an output
  region, copy the accumulators into it and push it back.
* Section 3 ("Execution Example") and Section 4.2: fused operators keep an intermediate
  result on chip: a store.local takes the produced region back from the compute core but
  writes nothing, and the load.local behind it on the same flow hands the very same region
  to a compute core again.  The `rope` uop of the example turns pairs of values by the
  angles whose cosines and sines a second tile holds.
* Section 6.3 ("Memory virtual core overhead"): memory uops measured without any arithmetic
  behind them.  Three compute uops without arithmetic stand behind the loads and stores
  of that measurement here: `drop` returns every region it pops as used, `fill` writes one
  32-bit word all over every output region it pops, `copy` pops a loaded region and an
  output region and moves the bytes of the first into the second.
* Section 4.1 names an `attn` compute uop (fused attention score computation) and Section 4.3
  ("Virtual Memory Core") says a FlashAttention uop frees slots in another order than they were
  allocated.  `attn` here serves one query over part of a context: it pops the query tile and keeps
  it, then for each of `size` (key tile, value tile) pairs updates a running maximum m, a running
  sum l of exp(score - m) and the sums o of exp(score - m) times the value rows, hands the query
  tile back (the oldest allocation goes back last), and writes (o, m, l) to an output region.
  `attn_merge` pops a tile of such partial rows of one request and an output region and writes
  sum_i exp(m_i - M) o_i / sum_i exp(m_i - M) l_i with M = max_i m_i.

Where the paper is silent this build reads it as follows:
16-byte words, the opcode set below, m2c delivery in program order of the `send` uops
(tickets), and a `kind` tag on c2m messages (recycle / produced).

The interpreter is driven by a scheduler that repeatedly picks one *enabled* action;
"program" order scans the agents round-robin, "random" picks uniformly with a seed.
The machine is deterministic in its results (memory image, per-unit traces) under every
legal schedule; tests check that.
"""
from collections import deque
from dataclasses import dataclass, field

import numpy as np

HALT, LOOP, REPEAT, ADD, SET, CONTINUE_IF = 0, 1, 2, 3, 4, 5
CONTROL_OPS = (HALT, LOOP, REPEAT, ADD, SET, CONTINUE_IF)
LOAD, STORE = 8, 9
MATVEC, ROPE, DROP, COPY, FILL, ATTN, ATTN_MERGE = 16, 17, 18, 19, 20, 21, 22
F_SEND, F_RECV, F_DYNAMIC, F_NT, F_DEP_SEND, F_DEP_RECV, F_LOCAL = 1, 2, 4, 8, 16, 32, 64
F_DEVICE = 128     # a hint for real caches (access at device scope); nothing to do in this machine
KIND_FREE, KIND_DATA = 0, 1
MAX_LOOP_DEPTH = 4
N_ACC = 8


class DeadlockError(RuntimeError):
    pass


class ProgramError(RuntimeError):
    pass


@dataclass
class Uop:
    opcode: int
    flags: int
    vflow: int
    vcc: int
    acc: int
    nslots: int
    size: int
    dep_id: int
    imm: int
    desc: int
    dep_count: int


def decode(w):
    """Split one 4 x uint32 word into its fields: w0 = opcode [7:0], flags [15:8], vflow [19:16], vcc [21:20],
    acc [24:22], nslots [30:25]; w1 = size [15:0], depId [31:16]; w2:w3 = imm [47:0] signed, desc [55:48], dep_count [63:56]."""
    w0, w1, w2, w3 = (int(x) for x in w)
    q = w2 | (w3 << 32)
    imm = q & ((1 << 48) - 1)
    if imm >> 47:
        imm -= 1 << 48
    return Uop(opcode=w0 & 0xFF, flags=(w0 >> 8) & 0xFF, vflow=(w0 >> 16) & 0xF, vcc=(w0 >> 20) & 0x3,
               acc=(w0 >> 22) & 0x7, nslots=(w0 >> 25) & 0x3F, size=w1 & 0xFFFF, dep_id=w1 >> 16,
               imm=imm, desc=(q >> 48) & 0xFF, dep_count=q >> 56)


@dataclass
class Desc:
    tensor: int
    box_rows: int
    row_bytes: int
    lds_pitch: int
    gpitch: int


def decode_desc(d):
    d = [int(x) for x in d]
    return Desc(d[0], d[1], d[2], d[3], d[4] | (d[5] << 32))


def first_fit(mask, n, n_slots):
    """Lowest p such that slots p .. p+n-1 are all free (bit clear) and p+n <= n_slots; -1 if none.
    Section 4.3: every allocator thread probes from its own position and the vote takes the first."""
    for p in range(0, n_slots - n + 1):
        if all(((mask >> (p + i)) & 1) == 0 for i in range(n)):
            return p
    return -1


class _Seq:
    """Register state of one stream: program counter, loop stack, accumulators."""

    def __init__(self, words, begin, end):
        self.words, self.begin, self.end = words, begin, end
        self.pc = begin
        self.loops = []
        self.acc = [0] * N_ACC
        self.halted = False

    def fetch(self):
        if self.pc >= self.end:
            raise ProgramError("stream ran past its end without HALT")
        return decode(self.words[self.pc])

    def control(self, u):
        """Run a control uop; returns True if `u` was one."""
        if u.opcode == HALT:
            if self.loops:
                raise ProgramError("HALT inside a loop")
            self.halted = True
        elif u.opcode == LOOP:
            if u.imm < 1 or len(self.loops) >= MAX_LOOP_DEPTH:
                raise ProgramError("bad LOOP")
            self.loops.append([self.pc + 1, u.imm])
            self.pc += 1
        elif u.opcode == REPEAT:
            if not self.loops:
                raise ProgramError("REPEAT without LOOP")
            self.acc[u.acc] += u.imm
            self.loops[-1][1] -= 1
            if self.loops[-1][1] > 0:
                self.pc = self.loops[-1][0]
            else:
                self.loops.pop()
                self.pc += 1
        elif u.opcode == ADD:
            self.acc[u.acc] += u.imm
            self.pc += 1
        elif u.opcode == SET:
            self.acc[u.acc] = u.imm
            self.pc += 1
        elif u.opcode == CONTINUE_IF:
            # Section 4.1 names continue_if next to loop among the control uops and says no more.  The reading taken
            # here: a condition on a register decides whether the innermost loop goes on.  While acc[acc] < imm the uop
            # does nothing; otherwise the loop is left at once: its frame is dropped and execution continues behind its
            # REPEAT, which stands `size` words further on (the generator knows the distance; the words in between
            # must close every loop they open).
            if not self.loops:
                raise ProgramError("CONTINUE_IF outside a loop")
            depth = 0
            for q in range(self.pc + 1, self.pc + u.size):
                if q >= self.end:
                    break
                op = decode(self.words[q]).opcode
                depth += 1 if op == LOOP else (-1 if op == REPEAT else 0)
                if depth < 0:
                    break
            if u.size < 1 or self.pc + u.size >= self.end or depth != 0 or decode(self.words[self.pc + u.size]).opcode != REPEAT:
                raise ProgramError("CONTINUE_IF does not point at the REPEAT of its loop")
            if self.acc[u.acc] < u.imm:
                self.pc += 1
            else:
                self.loops.pop()
                self.pc += u.size + 1
        else:
            return False
        return True


@dataclass
class Issued:
    """A memory uop after the front end: decoded, address generated, slots allocated."""
    pc: int
    u: Uop
    d: Desc
    offset: int          # byte offset inside the tensor
    slot: int
    ticket: int          # position in m2c[vcc] when SEND, else -1


class Core:
    def __init__(self, m, idx):
        self.m, self.idx = m, idx
        V = m.V
        sb = m.stream_begin
        base = idx * (1 + V)
        self.vmc = _Seq(m.words, int(sb[base]), int(sb[base + 1]))
        self.vccs = [_Seq(m.words, int(sb[base + 1 + v]), int(sb[base + 2 + v])) for v in range(V)]
        self.mask = 0
        self.lmem = np.zeros(m.n_slots * m.slot_bytes, dtype=np.uint8)
        self.ldu = [deque() for _ in range(m.n_ldu)]
        self.stu = [deque() for _ in range(m.n_stu)]
        self.m2c = [dict() for _ in range(V)]        # ticket -> message
        self.m2c_next_ticket = [0] * V
        self.m2c_head = [0] * V
        self.c2m = [deque() for _ in range(V)]
        self.mailbox = [deque() for _ in range(V)]   # produced regions waiting for their STORE
        # regions a store.local took back, waiting for the load.local behind it on the same flow: one queue per store unit
        self.parked = [deque() for _ in range(m.n_stu)]
        self.vcc_run = [None] * V                    # running compute uop (generator) per VCC
        self.vcc_wait = [False] * V
        self.peak_slots = 0
        self.free_log = []                           # (position, n) in the order the regions came back
        self.stats = dict(m2c_push=[0] * V, m2c_pop=[0] * V, c2m_push=[0] * V, c2m_pop=[0] * V)

    # ---- slot pool -------------------------------------------------------------------------
    def alloc(self, n):
        p = first_fit(self.mask, n, self.m.n_slots)
        if p < 0:
            return -1
        bits = ((1 << n) - 1) << p
        assert self.mask & bits == 0
        self.mask |= bits
        self.peak_slots = max(self.peak_slots, bin(self.mask).count("1"))
        return p

    def free(self, p, n):
        bits = ((1 << n) - 1) << p
        if self.mask & bits != bits:
            raise ProgramError("free of slots that are not allocated")
        self.mask &= ~bits
        self.free_log.append((p, n))

    def region(self, slot, nslots):
        sb = self.m.slot_bytes
        return self.lmem[slot * sb:(slot + nslots) * sb]


class Machine:
    def __init__(self, words, stream_begin, descs, tensors, n_cores, vcc_per_core=2, slot_bytes=8192,
                 n_slots=19, n_ldu=2, n_stu=1, n_dep_ids=64, unit_queue_cap=8):
        """tensors: list of numpy arrays (any dtype); they are read and written in place as bytes."""
        self.words = np.asarray(words, dtype=np.uint32).reshape(-1, 4)
        self.stream_begin = np.asarray(stream_begin, dtype=np.uint32)
        self.descs = [decode_desc(d) for d in np.asarray(descs, dtype=np.uint32).reshape(-1, 8)]
        self.tensors = [t.reshape(-1).view(np.uint8) for t in tensors]
        self.n_cores, self.V = n_cores, vcc_per_core
        assert len(self.stream_begin) == n_cores * (1 + vcc_per_core) + 1
        assert 1 <= n_slots <= 32
        self.slot_bytes, self.n_slots = slot_bytes, n_slots
        self.n_ldu, self.n_stu, self.qcap = n_ldu, n_stu, unit_queue_cap
        self.dep = [0] * n_dep_ids
        self.cores = [Core(self, c) for c in range(n_cores)]
        # per-unit traces: (pc relative to the stream, opcode, desc, tensor byte offset, rows)
        self.trace_vmc = [[] for _ in range(n_cores)]
        self.trace_vcc = [[[] for _ in range(vcc_per_core)] for _ in range(n_cores)]
        self.alloc_log = [[] for _ in range(n_cores)]     # (mask before, n, position) per allocation
        self.steps = 0

    # ---- front end of the VMC ----------------------------------------------------------------
    def _cfu_enabled_and_step(self, core, commit):
        s = core.vmc
        if s.halted:
            return False
        u = s.fetch()
        if u.opcode in CONTROL_OPS:
            if commit:
                s.control(u)
            return True
        if u.opcode not in (LOAD, STORE):
            raise ProgramError("opcode %d on a memory core" % u.opcode)
        d = self.descs[u.desc]
        local = bool(u.flags & F_LOCAL)
        load_local = local and u.opcode == LOAD          # hands an existing region on: allocates and reads nothing
        need = 0 if load_local else -(-d.box_rows * d.lds_pitch // self.slot_bytes)
        if u.nslots != need or (u.nslots < 1 and not load_local) or u.nslots > self.n_slots:
            raise ProgramError("nslots does not match the descriptor box")
        if u.size < 1 or u.size > d.box_rows or u.vcc >= self.V:
            raise ProgramError("bad rows or vcc")
        if local and (not u.flags & F_SEND or (u.opcode == STORE and not u.flags & F_RECV) or u.flags & F_DYNAMIC or u.imm):
            raise ProgramError("malformed local memory uop")
        units = core.ldu if (u.opcode == LOAD and not local) else core.stu
        if units is core.stu and not load_local and u.vflow % self.n_stu != u.vcc % self.n_stu:
            # several store units share the compute cores' return queues out between them (unit i: VCC i, i + n_stu, ..)
            raise ProgramError("a STORE sits on another store unit than the one its compute core returns regions to")
        q = units[u.vflow % len(units)]
        if len(q) >= self.qcap:
            return False
        if not load_local and first_fit(core.mask, u.nslots, self.n_slots) < 0:
            return False                      # in-order allocation: the front end stalls here
        if not commit:
            return True
        slot = -1
        if not load_local:
            before = core.mask
            slot = core.alloc(u.nslots)
            self.alloc_log[core.idx].append((before, u.nslots, slot))
        off = u.imm + (s.acc[u.acc] if u.flags & F_DYNAMIC else 0)
        t = self.tensors[d.tensor]
        last = off + (u.size - 1) * d.gpitch + d.row_bytes
        if not local and (off < 0 or last > t.size):
            raise ProgramError("tensor access out of bounds")
        ticket = -1
        if u.flags & F_SEND:
            ticket = core.m2c_next_ticket[u.vcc]
            core.m2c_next_ticket[u.vcc] += 1
        rec = Issued(s.pc - s.begin, u, d, off, slot, ticket)
        self.trace_vmc[core.idx].append((rec.pc, u.opcode, u.desc, off, u.size))
        if u.opcode == STORE and u.flags & F_SEND:
            # the empty output region goes to the compute core at once; the store unit only
            # waits for it to come back
            core.region(slot, u.nslots)[:] = 0
            self._m2c_push(core, u.vcc, ticket, (slot, u.nslots, u.size, d.row_bytes))
        q.append(rec)
        s.pc += 1
        return True

    def _m2c_push(self, core, v, ticket, msg):
        assert ticket not in core.m2c[v]
        core.m2c[v][ticket] = msg
        core.stats["m2c_push"][v] += 1

    # ---- load / store units ------------------------------------------------------------------
    def _unit_enabled_and_step(self, core, q, commit):
        if not q:
            return False
        rec = q[0]
        u, d = rec.u, rec.d
        if u.flags & F_DEP_RECV and self.dep[u.dep_id] < max(1, u.dep_count):
            return False
        if u.opcode == STORE and u.flags & F_RECV and not core.mailbox[u.vcc]:
            return False
        if u.opcode == LOAD and u.flags & F_LOCAL and not core.parked[u.vflow % self.n_stu]:
            return False
        if not commit:
            return True
        q.popleft()
        if u.flags & F_LOCAL:
            if u.opcode == STORE:
                # store.local: take the produced region back, write nothing, keep it allocated
                got = core.mailbox[u.vcc].popleft()
                if got != (rec.slot, u.nslots):
                    raise ProgramError("store received a region it did not allocate")
                core.parked[u.vflow % self.n_stu].append(got)
            else:
                # load.local: the oldest kept region goes to a compute core as a delivered tile
                slot, nslots = core.parked[u.vflow % self.n_stu].popleft()
                self._m2c_push(core, u.vcc, rec.ticket, (slot, nslots, u.size, d.row_bytes))
            if u.flags & F_DEP_SEND:
                self.dep[u.dep_id] += 1
            return True
        t = self.tensors[d.tensor]
        reg = core.region(rec.slot, u.nslots)
        if u.opcode == LOAD:
            reg[:] = 0                        # the part of the box outside the valid tile reads as zero
            for r in range(u.size):
                g = rec.offset + r * d.gpitch
                reg[r * d.lds_pitch:r * d.lds_pitch + d.row_bytes] = t[g:g + d.row_bytes]
            if u.flags & F_SEND:
                self._m2c_push(core, u.vcc, rec.ticket, (rec.slot, u.nslots, u.size, d.row_bytes))
            # a load that is not sent on stays allocated until something frees it; not used here
        else:
            if u.flags & F_RECV:
                slot, nslots = core.mailbox[u.vcc].popleft()
                if (slot, nslots) != (rec.slot, u.nslots):
                    raise ProgramError("store received a region it did not allocate")
            for r in range(u.size):
                g = rec.offset + r * d.gpitch
                t[g:g + d.row_bytes] = reg[r * d.lds_pitch:r * d.lds_pitch + d.row_bytes]
            core.free(rec.slot, u.nslots)
        if u.flags & F_DEP_SEND:
            self.dep[u.dep_id] += 1
        return True

    # ---- c2m receiver of the VMC ---------------------------------------------------------------
    def _drain_enabled_and_step(self, core, v, commit):
        if not core.c2m[v]:
            return False
        if commit:
            kind, slot, nslots = core.c2m[v].popleft()
            core.stats["c2m_pop"][v] += 1
            if kind == KIND_FREE:
                core.free(slot, nslots)
            else:
                core.mailbox[v].append((slot, nslots))
        return True

    # ---- compute cores -------------------------------------------------------------------------
    def _matvec(self, core, v, u):
        """The matvec compute uop (Section 4.1, the matvec listing), as a coroutine that yields wherever it waits for a region."""
        B = u.imm & 0xFF
        R = (u.imm >> 8) & 0xFFFF
        lpr = (u.imm >> 24) & 0xFFFF
        xspan = (u.imm >> 40) & 0x7F
        Kt = lpr * 4
        rowspan = u.desc                                   # a compute uop names no descriptor: on a MATVEC the field counts row blocks
        if rowspan >= 2:
            # The uop's tile is the tiler's to choose (the listing fixes none): when K fits one tile, a MATVEC may cover
            # `rowspan` row blocks of R rows that share one vector tile, each block fetched as an I/O block of its own.
            # Its output region ([B][rowspan * R], one STORE for all the blocks) is allocated first and kept, then the
            # vector tile, then the matrix tiles come and go, block j giving rows j R .. j R + R - 1; the vector tile goes
            # back after the last block and the region goes back as produced.
            if u.size != 1 or xspan >= 2:
                raise ProgramError("matvec over several row blocks: one tile step per block, a vector tile of its own")
            o = yield                                      # the output region
            o_slot, o_n, o_rows, o_rb = o
            if o_rows != B or o_rb > rowspan * R * 4:
                raise ProgramError("matvec: output region does not match the uop")
            b = yield                                      # the vector tile
            b_slot, b_n, b_rows, b_rb = b
            if b_rows != B:
                raise ProgramError("matvec: tile geometry does not match the uop")
            bt = core.region(b_slot, b_n).view(np.float32)[:B * Kt].reshape(B, Kt).astype(np.float64)
            out = core.region(o_slot, o_n).view(np.float32)[:B * rowspan * R].reshape(B, rowspan * R)
            for j in range(rowspan):
                a = yield                                  # the matrix tile of block j
                a_slot, a_n, a_rows, a_rb = a
                if a_rows > R:
                    raise ProgramError("matvec: tile geometry does not match the uop")
                at = core.region(a_slot, a_n).view(np.float32)[:R * Kt].reshape(R, Kt).astype(np.float64)
                out[:, j * R:(j + 1) * R] = (bt @ at.T).astype(np.float32)
                self._c2m_push(core, v, KIND_FREE, a_slot, a_n)
            self._c2m_push(core, v, KIND_FREE, b_slot, b_n)
            self._c2m_push(core, v, KIND_DATA, o_slot, o_n)
            return
        c = np.zeros((B, R), dtype=np.float64)            # the accumulators the uop keeps over all its tile steps
        if xspan >= 2:
            # The tile shape is the tiler's to choose (the listing fixes none): a vector tile may hold the pieces of `xspan`
            # consecutive steps.  With one vector: one piece per row.  With B vectors: B rows of xspan pieces side by
            # side, i.e. the vectors' next xspan * Kt columns as they lie in memory.  It is popped before the first matrix
            # tile it serves, kept while the matrix tiles of its steps come and go, and handed back after the last of them.
            held = None
            for i in range(u.size):
                if i % xspan == 0:
                    if held is not None:
                        self._c2m_push(core, v, KIND_FREE, held[0], held[1])
                    held = yield                           # wait for the vector tile of this and the next xspan - 1 steps
                    need = min(xspan, u.size - i)
                    if B == 1 and (held[2] < need or held[3] != Kt * 4):
                        raise ProgramError("matvec: vector tile does not hold the steps it is popped for")
                    if B > 1 and (held[2] != B or held[3] < need * Kt * 4 or held[3] > xspan * Kt * 4):
                        raise ProgramError("matvec: vector tile does not hold the steps it is popped for")
                a = yield                                  # wait for the matrix tile
                a_slot, a_n, a_rows, a_rb = a
                if a_rows > R:
                    raise ProgramError("matvec: tile geometry does not match the uop")
                at = core.region(a_slot, a_n).view(np.float32)[:R * Kt].reshape(R, Kt).astype(np.float64)
                j = i % xspan
                hv = core.region(held[0], held[1]).view(np.float32)
                if B == 1:
                    bt = hv[j * Kt:(j + 1) * Kt].reshape(1, Kt).astype(np.float64)
                else:
                    bt = hv[:B * xspan * Kt].reshape(B, xspan * Kt)[:, j * Kt:(j + 1) * Kt].astype(np.float64)
                c += bt @ at.T
                self._c2m_push(core, v, KIND_FREE, a_slot, a_n)
            if held is not None:
                self._c2m_push(core, v, KIND_FREE, held[0], held[1])
        for _ in range(u.size if xspan < 2 else 0):
            a = yield                                      # wait for the matrix tile,
            b = yield                                      # then for the vector tile
            a_slot, a_n, a_rows, a_rb = a
            b_slot, b_n, b_rows, b_rb = b
            if b_rows != B or a_rows > R:
                raise ProgramError("matvec: tile geometry does not match the uop")
            at = core.region(a_slot, a_n).view(np.float32)[:R * Kt].reshape(R, Kt).astype(np.float64)
            bt = core.region(b_slot, b_n).view(np.float32)[:B * Kt].reshape(B, Kt).astype(np.float64)
            c += bt @ at.T                                 # every vector against every tile row
            self._c2m_push(core, v, KIND_FREE, a_slot, a_n)   # both regions go back as used
            self._c2m_push(core, v, KIND_FREE, b_slot, b_n)
        o = yield                                          # wait for the output region
        o_slot, o_n, o_rows, o_rb = o
        if o_rows != B or o_rb > R * 4:
            raise ProgramError("matvec: output region does not match the uop")
        out = core.region(o_slot, o_n).view(np.float32)[:B * R].reshape(B, R)
        out[:, :] = c.astype(np.float32)                   # the sums go into the region
        self._c2m_push(core, v, KIND_DATA, o_slot, o_n)    # which goes back as produced, for the write-back

    def _rope(self, core, v, u):
        """The rope compute uop of the running example (Section 3): pop the value tile, the tile of cosines
        and sines and an output region, each [B][R] fp32; turn every pair (2i, 2i + 1) by its angle."""
        B = u.imm & 0xFF
        R = (u.imm >> 8) & 0xFFFF
        o = yield
        t = yield
        out = yield
        if o[2] != B or t[2] != B or out[2] != B or R % 2:
            raise ProgramError("rope: tile geometry does not match the uop")
        ov = core.region(o[0], o[1]).view(np.float32)[:B * R].reshape(B, R).astype(np.float64)
        tv = core.region(t[0], t[1]).view(np.float32)[:B * R].reshape(B, R).astype(np.float64)
        r = np.empty((B, R), dtype=np.float64)
        x, y, c, s = ov[:, 0::2], ov[:, 1::2], tv[:, 0::2], tv[:, 1::2]
        r[:, 0::2] = x * c - y * s
        r[:, 1::2] = x * s + y * c
        core.region(out[0], out[1]).view(np.float32)[:B * R].reshape(B, R)[:, :] = r.astype(np.float32)
        self._c2m_push(core, v, KIND_FREE, o[0], o[1])
        self._c2m_push(core, v, KIND_FREE, t[0], t[1])
        self._c2m_push(core, v, KIND_DATA, out[0], out[1])

    def _drop(self, core, v, u):
        """`size` loaded regions are popped and handed back as used, untouched."""
        for _ in range(u.size):
            a = yield
            self._c2m_push(core, v, KIND_FREE, a[0], a[1])

    def _fill(self, core, v, u):
        """`size` output regions are popped; the first 16 * chunks bytes of each become copies of one 32-bit word."""
        value = u.imm & 0xFFFFFFFF
        nbytes = ((u.imm >> 32) & 0xFFFF) * 16
        for _ in range(u.size):
            o = yield
            reg = core.region(o[0], o[1])
            if nbytes > reg.size:
                raise ProgramError("fill: more bytes than the region holds")
            reg[:nbytes].view(np.uint32)[:] = value
            self._c2m_push(core, v, KIND_DATA, o[0], o[1])

    def _copy(self, core, v, u):
        """`size` times: pop a loaded region and an output region, move the first 16 * chunks bytes across."""
        nbytes = (u.imm & 0xFFFF) * 16
        for _ in range(u.size):
            a = yield
            o = yield
            src, dst = core.region(a[0], a[1]), core.region(o[0], o[1])
            if nbytes > src.size or nbytes > dst.size:
                raise ProgramError("copy: more bytes than a region holds")
            dst[:nbytes] = src[:nbytes]
            self._c2m_push(core, v, KIND_FREE, a[0], a[1])
            self._c2m_push(core, v, KIND_DATA, o[0], o[1])

    def _attn(self, core, v, u):
        """One query over `size` (key tile, value tile) pairs of a context; imm = d/4 [7:0], R [15:8], the bits of
        the fp32 scale [47:16].  The output region says what is written: a region of one row of d + 4 values takes the
        partial row (o[0..d), m, l, 0, 0) of a context that other items share (ATTN_MERGE joins them); a region of one
        row of d values takes the finished result o / l of a context this uop saw all of (Section 4.1 names one attn
        uop; reading: which of the two it produces follows from the region the memory core hands it).  A compute uop names
        no descriptor: on an ATTN the field holds P; P > 0: the context has P other items; behind its last pair the uop takes one more tile, their P partial rows,
        and joins them to its own running state before it writes the result (what ATTN_MERGE does, without the uop's
        own partial row going through memory)."""
        d = (u.imm & 0xFF) * 4
        R = (u.imm >> 8) & 0xFF
        scale = float(np.array([(u.imm >> 16) & 0xFFFFFFFF], dtype=np.uint32).view(np.float32)[0])
        q = yield
        if q[2] != 1 or q[3] != d * 4:
            raise ProgramError("attn: the query tile is not one row of d values")
        qv = core.region(q[0], q[1]).view(np.float32)[:d].astype(np.float64)
        m, l, o = -np.inf, 0.0, np.zeros(d)
        for _ in range(u.size):
            k = yield
            kv = core.region(k[0], k[1]).view(np.float32)[:R * d].reshape(R, d).astype(np.float64)
            rows = k[2]
            if rows < 1 or rows > R or k[3] != d * 4:
                raise ProgramError("attn: key tile geometry does not match the uop")
            score = scale * (kv[:rows] @ qv)
            w = yield
            if w[2] != rows or w[3] != d * 4:
                raise ProgramError("attn: value tile geometry does not match the key tile")
            vv = core.region(w[0], w[1]).view(np.float32)[:R * d].reshape(R, d).astype(np.float64)
            m_new = max(m, float(score.max()))
            p = np.exp(score - m_new)
            alpha = np.exp(m - m_new)                      # 0 on the first tile
            l = l * alpha + p.sum()
            o = o * alpha + p @ vv[:rows]
            m = m_new
            self._c2m_push(core, v, KIND_FREE, k[0], k[1])
            self._c2m_push(core, v, KIND_FREE, w[0], w[1])
        self._c2m_push(core, v, KIND_FREE, q[0], q[1])     # allocated first, handed back after the last pair
        P = u.desc
        if P:
            t = yield
            if t[2] != P or t[3] != (d + 4) * 4:
                raise ProgramError("attn: the tile behind the last pair is not P partial rows")
            part = core.region(t[0], t[1]).view(np.float32)[:P * (d + 4)].reshape(P, d + 4).astype(np.float64)
            M = max(m, float(part[:, d].max()))
            w_own, w = np.exp(m - M), np.exp(part[:, d] - M)
            l = l * w_own + w @ part[:, d + 1]
            o = o * w_own + w @ part[:, :d]
            m = M
            self._c2m_push(core, v, KIND_FREE, t[0], t[1])
        out = yield
        row = core.region(out[0], out[1]).view(np.float32)
        if P and not (out[2] == 1 and out[3] == d * 4):
            raise ProgramError("attn: a uop that joins partial rows writes a result row")
        if out[2] == 1 and out[3] == d * 4:
            row[:d] = (o / l).astype(np.float32)
        elif out[3] >= (d + 4) * 4:
            row[:d] = o.astype(np.float32)
            row[d:d + 4] = (np.float32(m), np.float32(l), 0.0, 0.0)
        else:
            raise ProgramError("attn: the output region is neither a result row nor a partial row")
        self._c2m_push(core, v, KIND_DATA, out[0], out[1])

    def _attn_merge(self, core, v, u):
        """`size` partial rows (o, m, l, 0, 0) of one request become its result; imm = d/4."""
        d = (u.imm & 0xFF) * 4
        t = yield
        out = yield
        if t[2] != u.size or t[3] != (d + 4) * 4:
            raise ProgramError("attn_merge: the tile is not `size` partial rows")
        part = core.region(t[0], t[1]).view(np.float32)[:u.size * (d + 4)].reshape(u.size, d + 4).astype(np.float64)
        M = part[:, d].max()
        w = np.exp(part[:, d] - M)
        res = (w @ part[:, :d]) / (w @ part[:, d + 1])
        core.region(out[0], out[1]).view(np.float32)[:d] = res.astype(np.float32)
        self._c2m_push(core, v, KIND_FREE, t[0], t[1])
        self._c2m_push(core, v, KIND_DATA, out[0], out[1])

    def _c2m_push(self, core, v, kind, slot, nslots):
        core.c2m[v].append((kind, slot, nslots))
        core.stats["c2m_push"][v] += 1

    def _vcc_enabled_and_step(self, core, v, commit):
        s = core.vccs[v]
        run = core.vcc_run[v]
        if run is None:
            if s.halted:
                return False
            u = s.fetch()
            if u.opcode in CONTROL_OPS:
                if commit:
                    s.control(u)
                return True
            handlers = {MATVEC: self._matvec, ROPE: self._rope, DROP: self._drop, COPY: self._copy, FILL: self._fill,
                        ATTN: self._attn, ATTN_MERGE: self._attn_merge}
            if u.opcode not in handlers:
                raise ProgramError("opcode %d on a compute core" % u.opcode)
            if commit:
                self.trace_vcc[core.idx][v].append((s.pc - s.begin, u.opcode, u.size, u.imm))
                g = handlers[u.opcode](core, v, u)
                try:
                    next(g)                                # runs up to the first pop_wait
                    core.vcc_run[v] = g
                except StopIteration:                      # a uop over zero regions
                    s.pc += 1
            return True
        # blocked in pop_wait: enabled when the next ticket has been delivered
        head = core.m2c_head[v]
        if head not in core.m2c[v]:
            return False
        if commit:
            msg = core.m2c[v].pop(head)
            core.m2c_head[v] += 1
            core.stats["m2c_pop"][v] += 1
            try:
                run.send(msg)
            except StopIteration:
                core.vcc_run[v] = None
                s.pc += 1
        return True

    # ---- scheduler -----------------------------------------------------------------------------
    def _agents(self):
        ag = []
        for core in self.cores:
            ag.append(lambda commit, c=core: self._cfu_enabled_and_step(c, commit))
            for q in core.ldu + core.stu:
                ag.append(lambda commit, c=core, q=q: self._unit_enabled_and_step(c, q, commit))
            for v in range(self.V):
                ag.append(lambda commit, c=core, v=v: self._drain_enabled_and_step(c, v, commit))
                ag.append(lambda commit, c=core, v=v: self._vcc_enabled_and_step(c, v, commit))
        return ag

    def finished(self):
        for c in self.cores:
            if not c.vmc.halted or any(not s.halted for s in c.vccs) or any(r is not None for r in c.vcc_run):
                return False
            if any(c.ldu) or any(c.stu) or any(c.c2m) or any(c.mailbox) or any(c.parked):
                return False
        return True

    def run(self, schedule="program", seed=0, max_steps=10**9):
        """Run to completion.  Raises DeadlockError when nothing is enabled before the end."""
        agents = self._agents()
        rng = np.random.default_rng(seed)
        n = len(agents)
        while not self.finished():
            if self.steps >= max_steps:
                raise RuntimeError("step limit")
            if schedule == "program":
                # one sweep over the agents in a fixed order; every enabled one takes a step
                progressed = 0
                for i in range(n):
                    if agents[i](True):
                        progressed += 1
                if not progressed:
                    raise DeadlockError(self.describe())
                self.steps += progressed - 1
            else:
                enabled = [i for i in range(n) if agents[i](False)]
                if not enabled:
                    raise DeadlockError(self.describe())
                agents[enabled[int(rng.integers(len(enabled)))]](True)
            self.steps += 1
        self.check_final()
        return self

    def describe(self):
        out = []
        for c in self.cores:
            if c.vmc.halted and all(s.halted for s in c.vccs):
                continue
            out.append("core %d: vmc pc %d mask %08x ldu %s stu %s m2c waiting %s" % (
                c.idx, c.vmc.pc - c.vmc.begin, c.mask, [len(q) for q in c.ldu], [len(q) for q in c.stu],
                [c.m2c_head[v] for v in range(self.V)]))
        return "no enabled action; " + "; ".join(out[:8])

    def check_final(self):
        """Invariants at termination: every slot returned, every queue drained, pushes == pops."""
        for c in self.cores:
            if c.mask != 0:
                raise ProgramError("core %d ends with slots still allocated: %08x" % (c.idx, c.mask))
            for v in range(self.V):
                if c.m2c[v]:
                    raise ProgramError("m2c not drained")
                st = c.stats
                if st["m2c_push"][v] != st["m2c_pop"][v] or st["c2m_push"][v] != st["c2m_pop"][v]:
                    raise ProgramError("queue pushes and pops differ")
