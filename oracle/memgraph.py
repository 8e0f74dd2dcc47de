"""CPU ORACLE (test infrastructure, not the product) -- memgraph construction and checking.

Three things live here, all in plain Python over plain lists:

1. `build_memgraph_uniform`: the compile algorithm of Section 6 (Algorithms 1 and 2) for the
   case the paper presents, one slot per tensor, taking the steps in the paper's order and with
   the paper's names (execHzn, allocHzn, Evicted, simMalloc, simMallocForceReld, simMallocOffld,
   simFree).  Where the printed algorithm is silent or inconsistent the reading is stated at
   the place it is used.
2. Checkers for the three correctness requirements of Section 6, first paragraph -- data
   dependencies kept or replaced by offload/reload chains, no race conditions (the "safely
   overwrites" relation of Section 4), no cycles (every edge forward in the extended serial
   order, Section 7) -- usable on any memgraph given in the plain format below, whoever built it.
3. An address-level simulator that runs a memgraph in a given dependency-respecting order and
   reports any read of a clobbered tensor, any overlap of live tensors and the memory in use,
   plus enumerators of orders (all of them for tiny graphs, random ones otherwise).  This is the
   brute-force form of "any execution order that respects the dependencies is valid"
   (Introduction) and of the fixed-memory claim (Section 5, first paragraph).

The compile result is not unique (slot and victim choice are free; Section 4 speaks of "a
possible mapping"), so nothing here compares two memgraphs edge by edge.

Memgraph vertex kinds: "input" (tensor already in GPU memory at start), "load" (host -> GPU copy
of an input), "op" (kernel call), "offload", "reload", "drop" (eviction of a tensor whose host
copy is still valid: no bytes move), "store" (GPU -> host copy of a wanted result).

A taskgraph vertex that sums n tensors takes the form Appendix A (resources) gives a reduction: an
output that several kernels increment under a write lock.  Its memgraph vertices are "zero" (the
output is given its location and cleared; memory dependencies of the location point here),
one "increment" per operand (operands: the tensor added, then the "zero" vertex; it owns no
memory of its own) in any order, and "join" (the sum vertex itself: runs after every increment,
moves no data, and from then on stands for the finished tensor at the same location).
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass, field
from typing import Dict, Iterator, List, Optional, Sequence, Tuple

import numpy as np


class MemgraphError(Exception):
    pass


class CapTooSmall(MemgraphError):
    pass


@dataclass
class MemGraph:
    n_task: int  # vertices 0..n_task-1 are the taskgraph's, same numbering
    cap: int
    kind: List[str] = field(default_factory=list)
    src: List[int] = field(default_factory=list)  # taskgraph vertex whose tensor this vertex makes or moves
    loc: List[Optional[Tuple[int, int]]] = field(default_factory=list)  # (offset, size) in GPU memory or None
    operands: List[List[int]] = field(default_factory=list)  # memgraph vertices whose output is read
    edges: List[Tuple[int, int, str]] = field(default_factory=list)  # (from, to, "data" | "mem")
    order: List[int] = field(default_factory=list)  # extended serial order (Section 7)

    def add_vertex(self, kind, src, loc, operands) -> int:
        self.kind.append(kind)
        self.src.append(src)
        self.loc.append(loc)
        self.operands.append(list(operands))
        return len(self.kind) - 1

    def __len__(self):
        return len(self.kind)

    def preds(self) -> List[List[int]]:
        p = [[] for _ in range(len(self))]
        for a, b, _ in self.edges:
            p[b].append(a)
        return p

    def succs(self) -> List[List[int]]:
        s = [[] for _ in range(len(self))]
        for a, b, _ in self.edges:
            s[a].append(b)
        return s


# =============================================================================================
# 1. Algorithms 1 and 2, uniform slots
# =============================================================================================

def build_memgraph_uniform(preds: Sequence[Sequence[int]], V: Sequence[int], n_slots: int,
                           sums: Sequence[int] = ()) -> MemGraph:
    """BuildMemgraph (Algorithm 1) with simMalloc / simMallocForceReld / simMallocOffld
    (Algorithm 2) for tensors that take exactly one slot each.

    preds[v] = producers that taskgraph vertex v consumes; V = a serial order respecting them;
    n_slots = GPU memory locations.  Input vertices are members of V and get a slot like any
    other vertex (Section 4's example counts two input tensors among GPU 1's seven tensors).
    Returned locations are (slot, 1).  Raises CapTooSmall when some vertex's inputs and output
    cannot be co-resident.

    sums: taskgraph vertices that add up their operands by increments into a write-locked output
    (Appendix A, resources).  Such a vertex asks for no slot of its own when its turn comes: its
    output is allocated and cleared ("zero") when its first operand has been produced, every
    operand is added by an "increment" placed right after the operand's producer, and the vertex
    itself becomes the "join" that takes the slot over.  The slot cannot be evicted while
    increments are outstanding (it holds a partial sum that only they may touch).
    """
    n = len(preds)
    sums = set(sums)
    assert all(preds[s] and len(set(preds[s])) == len(preds[s]) for s in sums)
    pos = {v: i for i, v in enumerate(V)}
    assert len(pos) == n and all(pos[u] < pos[v] for v in range(n) for u in preds[v])
    mg = MemGraph(n_task=n, cap=n_slots)
    for v in range(n):
        # an input vertex materialises its tensor in the slot when it is "run"
        mg.add_vertex("load" if not preds[v] else "op", v, None, [])
    edges = set()

    # taskgraph consumer lists; `name[t]` is what tensor t is currently called (t itself or its
    # newest reload vertex): the "rename all instances" of simMallocOffld, applied only to the
    # accesses that have not been simulated yet ("future" accesses, Section 6 last paragraph).
    # (a sum consumes an operand right after the operand is produced, not at its own position)
    cons_pos = [sorted(pos[w] for w in range(n) if v in preds[w] and w not in sums) for v in range(n)]
    sums_of = [[w for w in sorted(sums, key=lambda x: pos[x]) if v in preds[w]] for v in range(n)]
    acc: Dict[int, int] = {}   # sum -> its "zero" vertex
    incs: Dict[int, List[int]] = {s: [] for s in sums}
    open_acc: set = set()      # accumulators whose join has not run
    post: List[List[int]] = [[] for _ in range(n)]  # what follows V[i] at once: clears, increments, their offloads
    name = list(range(n))
    readers: Dict[int, List[int]] = {v: [] for v in range(n)}  # per memgraph vertex with a slot: who read it so far
    owner: List[Optional[int]] = [None] * n_slots  # memgraph vertex now in the slot
    last_owner: List[Optional[int]] = [None] * n_slots  # history: previous occupant
    Evicted: Dict[int, int] = {}  # reload vertex -> its offload vertex; reload has no slot yet
    added_by_malloc: Dict[int, List[Tuple[int, int, str]]] = {}
    pre: List[List[int]] = [[] for _ in range(n)]  # offload/reload vertices placed just before V[i]
    execHzn, allocHzn = 0, 0
    sink: List[Optional[List[int]]] = [None]  # where evictions are noted instead of pre[execHzn], if set

    def add_edge(a, b, k):
        e = (a, b, k)
        if a != b and e not in edges:
            edges.add(e)
            mg.edges.append(e)
            return e
        return None

    def next_use(t: int) -> int:
        for p in cons_pos[t]:
            if p >= execHzn:
                return p
        return n + 1

    def simMalloc(v: int) -> int:
        slot = next((s for s in range(n_slots) if owner[s] is None), -1)
        if slot == -1:
            return -1
        owner[slot] = v
        mg.loc[v] = (slot, 1)
        vp = last_owner[slot]
        added = []
        if vp is not None:
            # every vertex that read the previous occupant must finish before v writes; an
            # occupant nobody read orders v after itself
            deps = readers[vp] if readers[vp] else [vp]
            for vpp in deps:
                e = add_edge(vpp, v, "mem")
                if e:
                    added.append(e)
        added_by_malloc[v] = added
        return slot

    def simFree(v: int):
        slot = mg.loc[v][0]
        assert owner[slot] == v
        owner[slot] = None
        last_owner[slot] = v

    def revoke_newest_preallocation() -> bool:
        """Undo the most recent run-ahead allocation (a slot held by a vertex that has not been
        "run" yet holds no data, so it cannot be offloaded; Algorithm 1 does not say what to do
        when only such slots are left)."""
        nonlocal allocHzn
        while True:
            if allocHzn - 1 <= execHzn:
                return False
            allocHzn -= 1
            v = V[allocHzn]
            if v not in sums:  # a sum holds no reservation of its own: look further back
                break
        owner[mg.loc[v][0]] = None
        mg.loc[v] = None
        for e in added_by_malloc.pop(v):
            edges.discard(e)
            mg.edges.remove(e)
        return True

    def simMallocOffld(v: int, pinned: set) -> int:
        while True:
            # victim: a produced, unpinned occupant; the one needed furthest in the future
            cands = [owner[s] for s in range(n_slots)
                     if owner[s] is not None and owner[s] not in pinned and produced(owner[s])]
            if cands:
                break
            if not revoke_newest_preallocation():
                raise CapTooSmall(f"vertex {V[execHzn]}: inputs and output do not fit in {n_slots} slots")
            s = simMalloc(v)
            if s != -1:
                return s
        vp = max(cands, key=lambda c: (next_use(mg.src[c]), -mg.loc[c][0]))
        t = mg.src[vp]
        off = mg.add_vertex("offload", t, None, [vp])
        rel = mg.add_vertex("reload", t, None, [off])
        readers[rel] = []
        add_edge(vp, off, "data")
        add_edge(off, rel, "data")
        readers[vp].append(off)  # the offload reads the slot; it precedes v in the order
        (sink[0] if sink[0] is not None else pre[execHzn]).append(off)
        # simMalloc on the vacated slot adds offload -> v and (earlier consumers of v') -> v
        simFree(vp)
        name[t] = rel
        Evicted[rel] = off
        s = simMalloc(v)
        assert s != -1
        return s

    def simMallocForceReld(v: int, pinned: set) -> int:
        del Evicted[v]
        pre[execHzn].append(v)
        slot = simMalloc(v)
        if slot != -1:
            return slot
        return simMallocOffld(v, pinned)

    def produced(m: int) -> bool:
        return (m >= n and m not in open_acc) or (m < n and pos[m] < execHzn)

    def increment(s: int, u: int, i_u: int):
        """u = V[i_u] has just run: add it to the sum s, clearing s's output first if u is the first."""
        sink[0] = post[i_u]
        if s not in acc:
            z = mg.add_vertex("zero", s, None, [])
            readers[z] = []
            acc[s] = z
            open_acc.add(z)
            if simMalloc(z) == -1:
                simMallocOffld(z, {name[u]})
            post[i_u].append(z)
        z = acc[s]
        i = mg.add_vertex("increment", s, None, [name[u], z])
        add_edge(name[u], i, "data")
        add_edge(z, i, "data")
        readers[name[u]].append(i)
        readers[z].append(i)
        incs[s].append(i)
        post[i_u].append(i)
        sink[0] = None

    def reserve_ahead() -> bool:
        """The allocation horizon moves on by one vertex if that takes no eviction."""
        nonlocal allocHzn
        if allocHzn >= n:
            return False
        if V[allocHzn] in sums:  # a sum's output is placed with its first increment, not here
            allocHzn += 1
            return True
        if simMalloc(V[allocHzn]) != -1:  # an open slot: the location of a result that does not exist yet
            allocHzn += 1
            return True
        return False

    def join_sum(s: int):
        """Every operand of s has been added: the cleared-and-summed slot is now s's."""
        nonlocal execHzn
        z = acc[s]
        slot = mg.loc[z][0]
        mg.kind[s] = "join"
        mg.loc[s] = mg.loc[z]
        mg.operands[s] = [z]
        for i in incs[s]:
            add_edge(i, s, "data")
        add_edge(z, s, "data")
        readers[z].append(s)
        readers[s] = readers[z]  # whoever takes the slot later waits for all of them and for s's readers
        owner[slot] = s
        open_acc.discard(z)
        execHzn += 1
        for w in sums_of[s]:
            increment(w, s, execHzn - 1)
        if sums_of[s] and next_use(s) > n:  # read by sums only, and they have taken it; a final result stays
            simFree(s)

    def run_next(v: int):
        """The execution horizon passes v, whose output already has its slot."""
        nonlocal execHzn
        deps = list(preds[v])
        # Algorithm 1 reloads, frees and adds the data edge dependency by dependency.  Freeing
        # inside that loop would let a later dependency's reload land in the slot just
        # vacated by an earlier dependency of the same vertex, which orders v before its own
        # input; Section 7 puts all reloads "just before v", so: reload all, then add the
        # data edges, then free.
        for u in deps:
            if name[u] in Evicted:
                pinned = {name[w] for w in deps if name[w] not in Evicted} | {v}
                simMallocForceReld(name[u], pinned)
        for u in deps:
            add_edge(name[u], v, "data")
            mg.operands[v].append(name[u])
            readers[name[u]].append(v)
        execHzn += 1
        for w in sums_of[v]:
            increment(w, v, execHzn - 1)
        for u in dict.fromkeys(list(deps) + ([v] if sums_of[v] else [])):
            if next_use(u) > n and name[u] not in Evicted and mg.loc[name[u]] is not None \
                    and owner[mg.loc[name[u]][0]] == name[u]:
                simFree(name[u])

    # Algorithm 1: run ahead with allocations while slots are open; otherwise the vertex at the
    # execution horizon runs -- after an eviction on its behalf if it is the very vertex that
    # could not be placed
    while execHzn < n:
        if reserve_ahead():
            continue
        v = V[execHzn]
        if v in sums:
            join_sum(v)
        elif allocHzn == execHzn:
            simMallocOffld(v, {name[u] for u in preds[v] if name[u] not in Evicted} | {v})
            allocHzn += 1
        else:
            run_next(v)
    for i, v in enumerate(V):
        offs = [m for m in pre[i] if mg.kind[m] == "offload"]
        rels = [m for m in pre[i] if mg.kind[m] == "reload"]
        mg.order.extend(offs + rels + [v] + post[i])
    # a reload that was created at eviction time but never needed afterwards (the tensor is a
    # final result that now lives in host memory) has no location and never runs: leave it out
    if Evicted:
        keep = [m for m in range(len(mg)) if m not in Evicted]
        new_id = {m: i for i, m in enumerate(keep)}
        out = MemGraph(n_task=n, cap=n_slots)
        for m in keep:
            out.add_vertex(mg.kind[m], mg.src[m], mg.loc[m], [new_id[x] for x in mg.operands[m]])
        out.edges = [(new_id[a], new_id[b], k) for a, b, k in mg.edges if a in new_id and b in new_id]
        out.order = [new_id[m] for m in mg.order]
        mg = out
    return mg


# =============================================================================================
# 2. structural checkers
# =============================================================================================

def _reach_bitsets(mg: MemGraph) -> List[int]:
    """desc[v] = bitset of the vertices reachable from v (v included).  Needs mg.order valid."""
    succ = mg.succs()
    desc = [0] * len(mg)
    for v in reversed(mg.order):
        b = 1 << v
        for w in succ[v]:
            b |= desc[w]
        desc[v] = b
    return desc


def check_forward_edges(mg: MemGraph):
    """Section 7, last paragraph: every edge points forward in the extended serial order, hence
    the memgraph is acyclic and that order is itself a valid execution."""
    if sorted(mg.order) != list(range(len(mg))):
        raise MemgraphError("extended order is not a permutation of the memgraph vertices")
    where = {v: i for i, v in enumerate(mg.order)}
    for a, b, k in mg.edges:
        if where[a] >= where[b]:
            raise MemgraphError(f"{k} edge {a}->{b} points backward in the extended order")


def check_data_deps(task_preds: Sequence[Sequence[int]], mg: MemGraph):
    """Section 6, requirement (a): each taskgraph edge u -> w is in the memgraph, or is replaced
    by u -> offload -> reload (-> offload -> reload)* -> w."""
    eset = {(a, b) for a, b, _ in mg.edges}
    incs_of: Dict[int, List[int]] = {}
    for v in range(len(mg)):
        if mg.kind[v] == "increment":
            incs_of.setdefault(mg.operands[v][1], []).append(v)
    for w in range(mg.n_task):
        ops = mg.operands[w]
        if mg.kind[w] == "join":
            # the operands of a sum arrive through its increments: zero -> increment -> join
            (z,) = ops
            if mg.kind[z] != "zero" or mg.src[z] != w or mg.loc[z] != mg.loc[w]:
                raise MemgraphError(f"join {w}: operand {z} is not its accumulator")
            incs = incs_of.get(z, [])
            for i in incs:
                if (z, i) not in eset or (i, w) not in eset or mg.src[i] != w:
                    raise MemgraphError(f"increment {i} of sum {w} lacks an edge from its accumulator or to the join")
            ops = [mg.operands[i][0] for i in incs]
            users = dict(zip(ops, incs))
        else:
            users = {x: w for x in ops}
        if sorted(mg.src[x] for x in ops) != sorted(task_preds[w]):
            raise MemgraphError(f"vertex {w}: operands {[mg.src[x] for x in ops]} differ from "
                                f"taskgraph producers {list(task_preds[w])}")
        for x in ops:
            if (x, users[x]) not in eset:
                raise MemgraphError(f"missing data edge {x}->{users[x]}")
            u, cur = mg.src[x], x
            while cur != u:  # walk the chain of copies back to the producer
                if mg.kind[cur] not in ("reload", "load") or len(mg.operands[cur]) != 1:
                    raise MemgraphError(f"vertex {cur} cannot stand for tensor {u}")
                off = mg.operands[cur][0]
                if mg.kind[off] not in ("offload", "drop") or mg.src[off] != u or (off, cur) not in eset:
                    raise MemgraphError(f"broken offload/reload chain at {cur}")
                prev = mg.operands[off][0]
                if mg.src[prev] != u or (prev, off) not in eset:
                    raise MemgraphError(f"broken offload/reload chain at {off}")
                cur = prev


def check_race_free(mg: MemGraph):
    """Section 4: whenever two outputs share memory, one must safely overwrite the other: every
    vertex that reads the earlier one (the earlier one itself if nobody reads it) has a
    dependency path to the later one."""
    desc = _reach_bitsets(mg)
    where = {v: i for i, v in enumerate(mg.order)}
    readers: List[List[int]] = [[] for _ in range(len(mg))]
    for v in range(len(mg)):
        for x in mg.operands[v]:
            if mg.loc[x] is not None:
                readers[x].append(v)
    located = sorted((v for v in range(len(mg)) if mg.loc[v] is not None and mg.loc[v][1] > 0),
                     key=lambda v: mg.loc[v][0])
    for i, x in enumerate(located):
        x0, xs = mg.loc[x]
        if x0 < 0 or x0 + xs > mg.cap:
            raise MemgraphError(f"vertex {x} placed outside [0, cap)")
        for y in located[i + 1:]:
            if mg.loc[y][0] >= x0 + xs:
                break
            a, b = (x, y) if where[x] < where[y] else (y, x)
            for r in (readers[a] or []) + [a]:
                if not (desc[r] >> b) & 1:
                    raise MemgraphError(f"race: {b} may overwrite {a} at {mg.loc[a]} before {r} has run")


# =============================================================================================
# 3. address-level simulation of one execution order
# =============================================================================================

def taskgraph_values(task_preds: Sequence[Sequence[int]], V: Sequence[int]) -> List[int]:
    """A distinct number per distinct computed value: inputs are their own id, an op's value is
    an injective function of (vertex, operand values)."""
    table: Dict[tuple, int] = {}
    val = [0] * len(task_preds)
    for v in V:
        key = (v, tuple(val[u] for u in task_preds[v]))
        val[v] = table.setdefault(key, len(table) + 1)
    return val


def simulate(mg: MemGraph, order: Sequence[int], task_preds: Sequence[Sequence[int]],
             expected: Sequence[int], operand_order_matters: bool = True) -> Dict[str, object]:
    """Execute the memgraph serially in `order` on a model of GPU memory.

    Memory is a set of written regions, each tagged with the value it holds; a write removes
    whatever it overlaps.  Every read must find exactly the value the taskgraph defines there
    (`expected`, from taskgraph_values).  A tensor is live from the moment its vertex runs until
    its last reader has run; live tensors must never overlap and their total must stay within the
    cap.  Returns the high-water mark of live bytes and of host (offloaded) bytes.
    """
    n = len(mg)
    mpreds = mg.preds()
    done = [False] * n
    regions: Dict[int, Tuple[int, int]] = {}  # offset -> (size, value)
    live: Dict[int, Tuple[int, int]] = {}  # memgraph vertex -> (offset, size), while readers remain
    remaining = [0] * n
    for v in range(n):
        for x in mg.operands[v]:
            remaining[x] += 1
    host: Dict[int, int] = {}
    host_bytes = live_bytes = hw_live = hw_host = 0
    results: Dict[int, int] = {}
    val = [None] * n

    def write(v, value):
        nonlocal live_bytes, hw_live
        off, size = mg.loc[v]
        if off < 0 or off + size > mg.cap:
            raise MemgraphError(f"vertex {v} writes outside [0, cap)")
        for u, (o, s) in live.items():
            if o < off + size and off < o + s:
                raise MemgraphError(f"vertex {v} overwrites live tensor of vertex {u}")
        for o in [o for o, (s, _) in regions.items() if o < off + size and off < o + s]:
            del regions[o]
        regions[off] = (size, value)
        val[v] = value
        # live while readers remain; a wanted result nobody reads stays live to the end
        if remaining[v] > 0 or mg.src[v] in final_needed:
            live[v] = (off, size)
            live_bytes += size
            hw_live = max(hw_live, live_bytes)

    def read(reader, x):
        nonlocal live_bytes
        off, size = mg.loc[x]
        got = regions.get(off)
        if got is None or got[0] != size or got[1] != expected[mg.src[x]]:
            raise MemgraphError(f"vertex {reader} reads {mg.loc[x]} expecting tensor {mg.src[x]}, "
                                f"found {got}")
        remaining[x] -= 1
        if remaining[x] == 0 and x in live:
            live_bytes -= live.pop(x)[1]

    # results that are read from GPU memory after the run: sinks of the taskgraph with no store
    stored = {mg.src[v] for v in range(n) if mg.kind[v] == "store"}
    consumed = {u for ps in task_preds for u in ps}
    final_needed = {t for t in range(mg.n_task) if t not in consumed and t not in stored}

    current: Dict[int, int] = {}  # tensor -> memgraph vertex holding its newest GPU copy
    # inputs that are already on the GPU are there before anything runs
    for v in range(n):
        if mg.kind[v] == "input":
            write(v, expected[mg.src[v]])
            current[mg.src[v]] = v
    for v in order:
        if done[v]:
            raise MemgraphError(f"vertex {v} executed twice")
        for p in mpreds[v]:
            if not done[p]:
                raise MemgraphError(f"order runs {v} before its dependency {p}")
        k = mg.kind[v]
        if k == "input":
            pass
        elif k == "load":  # first load, or reload of a dropped input from the caller's buffer
            write(v, expected[mg.src[v]])
            current[mg.src[v]] = v
        elif k == "op":
            for x in mg.operands[v]:
                read(v, x)
            assert sorted(mg.src[x] for x in mg.operands[v]) == sorted(task_preds[mg.src[v]])
            write(v, expected[mg.src[v]])
            current[mg.src[v]] = v
        elif k == "zero":
            write(v, ("partial sum",))
        elif k == "increment":
            x, z = mg.operands[v]
            read(v, x)
            off, size = mg.loc[z]
            got = regions.get(off)
            if got is None or got[0] != size or not isinstance(got[1], tuple) or val[z] is None:
                raise MemgraphError(f"increment {v} finds {got} where its accumulator {z} should be")
            regions[off] = (size, got[1] + (expected[mg.src[x]],))
            remaining[z] -= 1
        elif k == "join":
            (z,) = mg.operands[v]
            off, size = mg.loc[z]
            got = regions.get(off)
            want = sorted(expected[u] for u in task_preds[mg.src[v]])
            if got is None or got[0] != size or not isinstance(got[1], tuple) or sorted(got[1][1:]) != want:
                raise MemgraphError(f"join {v} finds {got}, not the sum of its operands")
            remaining[z] -= 1
            if remaining[z] != 0:
                raise MemgraphError(f"join {v} runs while increments of {z} are outstanding")
            live_bytes -= live.pop(z)[1]
            write(v, expected[mg.src[v]])
            current[mg.src[v]] = v
        elif k == "offload":
            (x,) = mg.operands[v]
            read(v, x)
            host[v] = expected[mg.src[v]]
            host_bytes += mg.loc[x][1]
            hw_host = max(hw_host, host_bytes)
            if current.get(mg.src[v]) == x:
                del current[mg.src[v]]
        elif k == "drop":
            (x,) = mg.operands[v]
            remaining[x] -= 1
            if remaining[x] == 0 and x in live:
                live_bytes -= live.pop(x)[1]
            host[v] = expected[mg.src[v]]
            if current.get(mg.src[v]) == x:
                del current[mg.src[v]]
        elif k == "reload":
            (o,) = mg.operands[v]
            if o not in host:
                raise MemgraphError(f"reload {v} before its offload {o} has run")
            write(v, host[o])
            host_bytes -= mg.loc[v][1]
            current[mg.src[v]] = v
        elif k == "store":
            (x,) = mg.operands[v]
            read(v, x)
            results[mg.src[v]] = expected[mg.src[v]]
        else:
            raise MemgraphError(f"unknown kind {k}")
        done[v] = True
    if not all(done):
        raise MemgraphError("order does not cover the memgraph")
    for t in final_needed:
        if t in current:
            x = current[t]
            got = regions.get(mg.loc[x][0])
            if got is None or got[1] != expected[t]:
                raise MemgraphError(f"result {t} was overwritten before the end of the run")
            results[t] = got[1]
        else:  # evicted and never needed again: it is in host memory
            offs = [v for v in range(n) if mg.kind[v] == "offload" and mg.src[v] == t and v in host]
            if not offs:
                raise MemgraphError(f"result {t} is nowhere at the end of the run")
            results[t] = host[offs[-1]]
    return {"hw_live": hw_live, "hw_host": hw_host, "results": results}


def all_topological_orders(mg: MemGraph, limit: Optional[int] = None) -> Iterator[List[int]]:
    """Every dependency-respecting order of the memgraph (exponential: tiny graphs only)."""
    n = len(mg)
    succ = mg.succs()
    indeg = [0] * n
    for a, b, _ in mg.edges:
        indeg[b] += 1
    order: List[int] = []
    count = 0

    def rec():
        nonlocal count
        if limit is not None and count >= limit:
            return
        if len(order) == n:
            count += 1
            yield list(order)
            return
        for v in range(n):
            if indeg[v] == 0:
                indeg[v] = -1
                for w in succ[v]:
                    indeg[w] -= 1
                order.append(v)
                yield from rec()
                order.pop()
                for w in succ[v]:
                    indeg[w] += 1
                indeg[v] = 0

    yield from rec()


def random_topological_order(mg: MemGraph, rng: np.random.Generator) -> List[int]:
    n = len(mg)
    succ = mg.succs()
    indeg = [0] * n
    for a, b, _ in mg.edges:
        indeg[b] += 1
    ready = [v for v in range(n) if indeg[v] == 0]
    out = []
    while ready:
        i = int(rng.integers(len(ready)))
        ready[i], ready[-1] = ready[-1], ready[i]
        v = ready.pop()
        out.append(v)
        for w in succ[v]:
            indeg[w] -= 1
            if indeg[w] == 0:
                ready.append(w)
    if len(out) != n:
        raise MemgraphError("memgraph has a cycle")
    return out
