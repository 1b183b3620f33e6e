"""The lowering steps of the uop generator, on the oracle side (Section 4.2).

Test infrastructure, not product code; shares nothing with the HIP path.  The paper's generator takes the graph of
uops that the operators of a model decompose into and turns it into per-core bytecode in steps.  This module writes
those steps down for graphs whose addresses are literals, in the paper's order:

* "Dynamic Data Placement and Fusion": a store and the load that reads exactly what it wrote, neighbours on one
  compute core of one memory core with nobody else reading the data, become store.local / load.local: the data stays
  in local memory (`place_local`).
* "Dependency Graph Lowering", third paragraph: slots are allocated in program order, so the order in which one
  memory core serves its compute cores can over-commit the pool; the generator elaborates the allocation along the
  stream, and when it finds such an order it reorders independent uops (`schedule`).  Here: the stream is run on
  the interpreter without data; on DEADLOCK the memory uops of the core are merged again, one *consumption group*
  at a time (the regions one step of a compute uop holds together), round-robin over the compute cores, which never
  splits the regions a compute core needs at the same time.
* second paragraph: virtual flow assignment: the memory uops of a core fall into chains (here: per compute core and
  tensor; a load that waits for another core stalls only the chain it is on), each chain gets a virtual flow
  (`assign_flows`).
* fourth paragraph: dependencies between memory uops are embedded as depIds (one per set of producers, counted), and
  waits that in-order execution on a flow already implies are removed: a load behind another load of the same flow
  that waited for the same producers needs no wait of its own (`embed_deps`).

The graph: per (core, compute core) the memory uops in the order in which that compute core takes their regions
(this order is semantics: regions reach a compute core in the program order of the `send` uops), the compute uops,
and a list of edges (store, load) "this load reads what that store wrote".
"""
from dataclasses import dataclass, field

import numpy as np

from . import uop_asm as A
from . import uop_machine as UM


@dataclass(eq=False)
class MemOp:
    op: int                 # A.LOAD or A.STORE
    core: int
    vcc: int
    desc: tuple             # (tensor, box_rows, row_bytes, lds_pitch, gpitch)
    offset: int             # byte offset in the tensor
    rows: int
    nslots: int
    group: int = 0          # consumption group on its compute core (see `schedule`)
    nt: bool = False
    # decided by the passes
    local: bool = False
    vflow: int = -1
    dep_wait: tuple = None      # (depId, count)
    dep_signal: int = None
    device: bool = False
    seq: int = 0            # creation order (the order in which the graph's builder wrote the uops down)


@dataclass
class Graph:
    n_cores: int
    V: int
    slot_bytes: int
    mem: list                   # [core][vcc] -> list of MemOp, in the order the compute core takes the regions
    comp: list                  # [core][vcc] -> list of uop words (compute and control uops of that compute core)
    edges: list = field(default_factory=list)       # (store MemOp, load MemOp)
    temps: set = field(default_factory=set)         # tensors that nobody outside the graph reads
    order: list = None          # [core] -> list of MemOp: the memory core's stream; None: the order the builder wrote them in
    geom_tensor: int = 0        # the tensor that descriptors of local uops name (geometry only: they touch no memory)

    def stream(self, core):
        if self.order is not None:
            return self.order[core]
        return sorted((m for v in range(self.V) for m in self.mem[core][v]), key=lambda m: m.seq)

    def add(self, m):
        """Append a memory uop to its compute core's sequence."""
        self._n = getattr(self, "_n", 0) + 1
        m.seq = self._n
        self.mem[m.core][m.vcc].append(m)
        return m


def new_graph(n_cores, V, slot_bytes):
    return Graph(n_cores, V, slot_bytes, [[[] for _ in range(V)] for _ in range(n_cores)],
                 [[[] for _ in range(V)] for _ in range(n_cores)])


# ---- Section 4.2, "Dynamic Data Placement and Fusion" ----------------------------------------------------------------
def place_local(g):
    """Rewrite one-to-one store -> load pairs on one compute core into store.local / load.local.  Returns the number of
    pairs rewritten.  The pair must be neighbours in the compute core's order, move the same box of a tensor listed in
    g.temps, and be the only producer / consumer of each other."""
    n_out = {}
    n_in = {}
    for s, l in g.edges:
        n_out[id(s)] = n_out.get(id(s), 0) + 1
        n_in[id(l)] = n_in.get(id(l), 0) + 1
    kept, done = [], 0
    for s, l in g.edges:
        seq = g.mem[s.core][s.vcc]
        ok = (s.core == l.core and s.vcc == l.vcc and s.op == A.STORE and l.op == A.LOAD and s.desc[0] in g.temps
              and n_out[id(s)] == 1 and n_in[id(l)] == 1 and s.offset == l.offset and s.rows == l.rows
              and s.desc == l.desc and seq.index(l) == seq.index(s) + 1)
        if not ok:
            kept.append((s, l))
            continue
        s.local = l.local = True
        # the region keeps its slots from the store's allocation; the load allocates nothing and touches no memory
        box = (g.geom_tensor, s.desc[1], s.desc[3], s.desc[3], s.desc[4])  # the whole box, as it lies in local memory
        s.desc = l.desc = box
        s.offset = l.offset = 0
        s.rows = l.rows = s.desc[1]
        l.nslots = 0
        l.group = s.group + 1 if l.group == s.group else l.group
        done += 1
    g.edges = kept
    return done


# ---- Section 4.2, "Dependency Graph Lowering": virtual flows -----------------------------------------------------------
def assign_flows(g):
    """Chains: the loads of one compute core from one tensor form a chain (they are independent of the other chains of
    the core: a load that waits for another core stalls its own chain only); stores, and the local pair that travels with
    them, form one chain per compute core.  Flows: load chains of compute core v take 2 v and 2 v + 1 in the order in
    which the chains first appear (further chains share the second), stores take 2 V + v."""
    for core in range(g.n_cores):
        for v in range(g.V):
            chains = []
            for m in g.mem[core][v]:
                if m.op == A.STORE or m.local:
                    m.vflow = 2 * g.V + v
                    continue
                t = m.desc[0]
                if t not in chains:
                    chains.append(t)
                m.vflow = 2 * v + min(chains.index(t), 1)
    return g


# ---- Section 4.2, "Dependency Graph Lowering": embedding, and removing what flow order implies ---------------------------
def embed_deps(g, eliminate=True):
    """Every load with producers waits for one depId that all of them signal (a store signals one depId, so loads that
    share a producer must share all: checked).  With `eliminate`, a wait is dropped when an earlier load on the same
    flow of the same core already waited for the same depId.  Returns (depIds used, waits kept, waits dropped)."""
    prods = {}
    for s, l in g.edges:
        prods.setdefault(id(l), []).append(s)
    ids = {}
    by_store = {}
    kept = dropped = 0
    for core in range(g.n_cores):
        waited = {}                                 # flow -> depIds an earlier load of that flow waited for
        for m in g.stream(core):
            ps = prods.get(id(m))
            if not ps:
                continue
            key = frozenset(id(s) for s in ps)
            if key not in ids:
                ids[key] = len(ids)
                for s in ps:
                    if by_store.setdefault(id(s), ids[key]) != ids[key]:
                        raise ValueError("a store would have to signal two depIds: its consumers do not share their producers")
                    s.dep_signal = ids[key]
                    s.device = True
            dep = ids[key]
            m.device = True                         # the data was written during this run, by whoever
            if len(ps) > 255:
                raise ValueError("more producers than a dependency can count")
            seen = waited.setdefault(m.vflow, set())
            if eliminate and dep in seen:
                dropped += 1
                continue
            seen.add(dep)
            m.dep_wait = (dep, len(ps))
            kept += 1
    return len(ids), kept, dropped


# ---- to bytecode ---------------------------------------------------------------------------------------------------------------
def assemble(g):
    p = A.Program(g.n_cores, g.V)
    for core in range(g.n_cores):
        vm = p.vmc(core)
        for m in g.stream(core):
            flags = A.F_SEND | (A.F_NT if m.nt else 0)
            if m.op == A.STORE:
                flags |= A.F_RECV
            if m.local:
                flags |= A.F_LOCAL
            dep_id = dep_count = 0
            if m.dep_wait is not None:
                flags |= A.F_DEP_RECV
                dep_id, dep_count = m.dep_wait
            if m.dep_signal is not None:
                flags |= A.F_DEP_SEND
                dep_id = m.dep_signal
            if m.device and not m.local:
                flags |= A.F_DEVICE
            vm.append(A.word(m.op, flags, vflow=max(m.vflow, 0), vcc=m.vcc, nslots=m.nslots, size=m.rows, dep_id=dep_id,
                             imm=m.offset, desc=p.desc(*m.desc), dep_count=dep_count))
        for v in range(g.V):
            p.vcc(core, v).extend(g.comp[core][v])
    return p


# ---- Section 4.2, "Dependency Graph Lowering": over-allocation ---------------------------------------------------------
def completes(g, tensor_bytes, n_slots, schedule="program", seed=0):
    """Does the graph's bytecode run to its end on the interpreter (no data: tensors of zeros)?"""
    w, sb, d = assemble(g).finish()
    tensors = [np.zeros(max(4, nb) // 4, dtype=np.float32) for nb in tensor_bytes]
    try:
        UM.Machine(w, sb, d, tensors, n_cores=g.n_cores, vcc_per_core=g.V, slot_bytes=g.slot_bytes, n_slots=n_slots).run(schedule, seed)
        return True
    except UM.DeadlockError:
        return False


def schedule(g, tensor_bytes, n_slots):
    """Elaborate the slot allocation along every memory core's stream; if the stream over-commits the pool, merge the
    compute cores' memory uops again, one consumption group at a time, round-robin.  The order inside a compute core's
    own sequence never changes (it is semantics).  Returns True if the order was changed.  Raises if the merged order
    does not complete either."""
    if completes(g, tensor_bytes, n_slots):
        return False
    order = []
    for core in range(g.n_cores):
        seqs = [list(g.mem[core][v]) for v in range(g.V)]
        merged = []
        while any(seqs):
            for s in seqs:
                if not s:
                    continue
                grp = s[0].group
                while s and s[0].group == grp:
                    merged.append(s.pop(0))
        order.append(merged)
    g.order = order
    if not completes(g, tensor_bytes, n_slots):
        raise UM.DeadlockError("the graph over-commits the slots in every order this generator knows")
    return True


# ---- graphs to lower: the operators of the tests -------------------------------------------------------------------------
def matvec_rope_graph(rows, K, B, R, Kt, slot_bytes, n_cores, V=2, temp_tensor=4):
    """The running example of Section 3 before any placement decision: O = M X goes to memory (tensor `temp_tensor`,
    [B][rows]) and R = rope(O, T) reads it back.  Tensors: 0 = M, 1 = X, 2 = Y, 3 = T, temp_tensor = O."""
    assert K % Kt == 0 and rows % R == 0 and R % 2 == 0
    g = new_graph(n_cores, V, slot_bytes)
    g.temps = {temp_tensor}
    g.geom_tensor = 2
    lpr, nk = Kt // 4, K // Kt
    slots = lambda nbytes: -(-nbytes // slot_bytes)
    dm, dx = (0, R, Kt * 4, Kt * 4, K * 4), (1, B, Kt * 4, Kt * 4, K * 4)
    do, dt, dy = (temp_tensor, B, R * 4, R * 4, rows * 4), (3, B, R * 4, R * 4, rows * 4), (2, B, R * 4, R * 4, rows * 4)
    for rb in range(rows // R):
        unit = rb % (n_cores * V)
        core, v = unit // V, unit % V
        seq = g.mem[core][v]
        grp = (seq[-1].group + 1) if seq else 0
        for kt in range(nk):
            g.add(MemOp(A.LOAD, core, v, dm, (rb * R * K + kt * Kt) * 4, R, slots(R * Kt * 4), grp, nt=True))
            g.add(MemOp(A.LOAD, core, v, dx, kt * Kt * 4, B, slots(B * Kt * 4), grp))
            grp += 1
        st = g.add(MemOp(A.STORE, core, v, do, rb * R * 4, B, slots(B * R * 4), grp))
        ld = g.add(MemOp(A.LOAD, core, v, do, rb * R * 4, B, slots(B * R * 4), grp + 1))
        g.add(MemOp(A.LOAD, core, v, dt, rb * R * 4, B, slots(B * R * 4), grp + 1))
        g.add(MemOp(A.STORE, core, v, dy, rb * R * 4, B, slots(B * R * 4), grp + 2))
        g.edges.append((st, ld))
        g.comp[core][v] += [A.word(A.MATVEC, size=nk, imm=A.matvec_imm(B, R, lpr)), A.word(A.ROPE, size=1, imm=A.rope_imm(B, R))]
    return g


def chain_graph(dims, B, R, Kt, slot_bytes, n_cores, V=2):
    """A chain of matvec operators, Y_0 = M_0 X, Y_l = M_l Y_(l-1), as one graph with an edge from every store of a row
    block of layer l to every load of a vector tile of layer l + 1 that contains its rows.  Tensors as in
    uop_asm.chain_matvec_program: 0 = W, 1 = A (read), 2 = A (written)."""
    L = len(dims) - 1
    assert Kt % R == 0 and all(d % Kt == 0 for d in dims)
    g = new_graph(n_cores, V, slot_bytes)
    slots = lambda nbytes: -(-nbytes // slot_bytes)
    w_off, a_off = [0], [0]
    for l in range(L):
        w_off.append(w_off[-1] + dims[l + 1] * dims[l] * 4)
        a_off.append(a_off[-1] + B * dims[l] * 4)
    stores = {}                                     # (layer, row block) -> its STORE
    for l in range(L):
        K, rows = dims[l], dims[l + 1]
        nk = K // Kt
        dm, dx, dy = (0, R, Kt * 4, Kt * 4, K * 4), (1, B, Kt * 4, Kt * 4, K * 4), (2, B, R * 4, R * 4, rows * 4)
        for rb in range(rows // R):
            unit = rb % (n_cores * V)
            core, v = unit // V, unit % V
            seq = g.mem[core][v]
            grp = (seq[-1].group + 1) if seq else 0
            for kt in range(nk):
                g.add(MemOp(A.LOAD, core, v, dm, w_off[l] + (rb * R * K + kt * Kt) * 4, R, slots(R * Kt * 4), grp, nt=True))
                x = g.add(MemOp(A.LOAD, core, v, dx, a_off[l] + kt * Kt * 4, B, slots(B * Kt * 4), grp))
                if l > 0:
                    for prb in range(kt * Kt // R, (kt + 1) * Kt // R):
                        g.edges.append((stores[(l - 1, prb)], x))
                grp += 1
            stores[(l, rb)] = g.add(MemOp(A.STORE, core, v, dy, a_off[l + 1] + rb * R * 4, B, slots(B * R * 4), grp))
            g.comp[core][v].append(A.word(A.MATVEC, size=nk, imm=A.matvec_imm(B, R, Kt // 4)))
    # written down layer after layer, row block after row block: on every memory core a waiting load stands behind all
    # the core's uops of the layers before it
    return g
