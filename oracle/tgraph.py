"""TEST INFRASTRUCTURE -- oracle for the task-graph side of the method (paper Sections 3-5).

Part 1  op-level DAG of one decode step and brute-force producer sets
        (Section 4.1 "operator decomposition" and "dependency analysis": an event for a task
        pair (t1, t2) iff the output region of t1 overlaps the input region of t2).  Every output
        ELEMENT gets an owner task; every consumer task's read elements are enumerated; the
        producer set is the set of owners.  No interval arithmetic, no shortcuts.
Part 2  the graph transformations on explicit sets: pair events, successor-set fusion (Def. 4.1),
        predecessor-set fusion (Def. 4.2), normalization (Fig. 5 rewrites), linearization
        (Algorithm 1).
Part 3  a simulator of the in-kernel runtime (Section 5): workers with a JIT and an AOT queue,
        schedulers with event queues, random legal interleavings, deadlock detection and the
        "inputs produced before a task runs" check.

Shares no code with the GPU library's compiler; it only reads the exported tables in tests.
"""
from __future__ import annotations

import random
from collections import defaultdict, deque
from dataclasses import dataclass, field

import numpy as np

# fusion flags of the op list (same bit values as the library's option field; interface data)
F_NORM, F_RESID, F_SWIGLU, F_MERGE, F_ROPE = 1, 2, 4, 8, 16

# operator kinds (same numbering as the exported op table)
(K_EMBED, K_RMSNORM, K_LINEAR, K_ROPE, K_ATTN_PARTIAL, K_ATTN_MERGE, K_ADD, K_SWIGLU,
 K_GATEUP, K_ROUTER, K_EXPERT, K_DUMMY, K_COMBINE, K_ARGMAX, K_SERVE) = range(15)


def split_even(n: int, k: int):
    """Contiguous split of n units into k tiles: the first n mod k tiles get ceil(n/k) units, the
    rest floor(n/k).  Returns k+1 boundaries."""
    q, r = divmod(n, k)
    b = [0]
    for i in range(k):
        b.append(b[-1] + q + (1 if i < r else 0))
    return b


@dataclass
class OpSpec:
    name: str
    kind: int
    layer: int
    out: str                  # output tensor name
    rows: int                 # batch rows of the output
    cols: int                 # columns of the output
    unit: int                 # columns are partitioned in multiples of `unit`
    ins: list                 # input tensor names
    meta: dict = field(default_factory=dict)


def build_ops(s, fusion: int, attn_chunks: int, moe_tasks: int = 0, down_parts: int = 1,
              greedy_loop: bool = False, attn_balance: bool = False, serving: bool = False,
              sampling_tiles: int = 1):
    """Operator list of one decode step for model shape `s` (synth.gen.ModelShape) under the
    given fusion flags, in execution order.

    A mixture-of-experts block (Section 6.4: routing, expert computation, combine as chains of
    tasks in the same graph) is five operators: the router's linear operator; `route` (softmax,
    top-k, the meta-tensor: one task that needs every token's router output); the experts'
    gate/up stage and their down stage, each cut at compile time into `moe_tasks` expert tasks
    whose share of the work is refined at run time from the meta-tensor; and `combine` (weighted
    sum of a token's expert outputs plus the residual).  Which token rows an expert task touches is
    only known at run time, so an expert stage's output is modelled as one element per task and
    every consumer of the stage reads all of them (the static superset).

    down_parts > 1 (fully fused list only): the down projection is decomposed along its input as
    well.  Its output tensor is then the partial sums [B][parts x H] (part p of row r at column
    p H + r); a task reads only its part of the input rows.  Whoever reads residual-stream element
    (b, r) afterwards reads all `parts` partial sums of it (the task that adds them up is only
    known at run time; it also adds the residual, so every part task statically reads that).

    attn_balance (merge fused into the attention tasks, batch > 1): the batch x C chunk tasks of a
    KV head are dealt to the sequences in proportion to their lengths when the step runs (the
    run-time imbalance of Section 5.2), so which sequence's query and new key/value a chunk task
    reads is a run-time fact: statically it reads those columns of every row.

    serving (Section 6.1: a decoding iteration is prepared by ONE task on the start event, which
    retires and admits requests and updates the KV-cache metadata): that task comes first and
    writes one metadata element per batch slot -- the slot's token, position and page table for
    the iteration; the embedding of slot b reads element b, so everything in the iteration is
    downstream of the task."""
    B, H, d, nq, nkv = s.batch, s.hidden, s.head_dim, s.n_q_heads, s.n_kv_heads
    F, V, C = s.ffn, s.vocab, attn_chunks
    grp = nq // nkv
    QKV = (nq + 2 * nkv) * d
    ops = []
    if serving:
        ops.append(OpSpec("serve", K_SERVE, -1, "slots", B, 1, 1, []))
    ops.append(OpSpec("embed", K_EMBED, -1, "x0", B, H, H, ["slots"] if serving else []))
    x = "x0"
    x_parts = 1   # > 1: x names a tensor of partial sums
    for l in range(s.n_layers):
        p = f"L{l}."
        if fusion & F_NORM:
            ops.append(OpSpec(p + "qkv", K_LINEAR, l, p + "qkv", B, QKV, 1, [x], {"K": H, "head": d}))
        else:
            ops.append(OpSpec(p + "attn_norm", K_RMSNORM, l, p + "xn", B, H, H, [x]))
            ops.append(OpSpec(p + "qkv", K_LINEAR, l, p + "qkv", B, QKV, 1, [p + "xn"], {"K": H, "head": d}))
        if fusion & F_ROPE:
            qsrc = p + "qkv"
        else:
            ops.append(OpSpec(p + "rope", K_ROPE, l, p + "rk", B, QKV, d, [p + "qkv"]))
            qsrc = p + "rk"
        ops.append(OpSpec(p + "attn_partial", K_ATTN_PARTIAL, l, p + "part", B,
                          nkv * C * grp * (d + 2), grp * (d + 2), [qsrc],
                          {"C": C, "grp": grp, "d": d, "nq": nq, "nkv": nkv,
                           "balance": bool(attn_balance and (fusion & F_MERGE) and B > 1)}))
        if fusion & F_MERGE:
            osrc, oK = p + "part", nkv * C * grp * (d + 2)
        else:
            ops.append(OpSpec(p + "attn_merge", K_ATTN_MERGE, l, p + "o", B, nq * d, d,
                              [p + "part"], {"C": C, "grp": grp, "d": d}))
            osrc, oK = p + "o", nq * d
        if fusion & F_RESID:
            ops.append(OpSpec(p + "o_proj", K_LINEAR, l, p + "x1", B, H, 1, [osrc, x],
                              {"K": oK, "resid": x, "resid_parts": x_parts}))
        else:
            ops.append(OpSpec(p + "o_proj", K_LINEAR, l, p + "a", B, H, 1, [osrc], {"K": oK}))
            ops.append(OpSpec(p + "resid1", K_ADD, l, p + "x1", B, H, 1, [x, p + "a"]))
        x1 = p + "x1"
        if fusion & F_NORM:
            nsrc = x1
        else:
            ops.append(OpSpec(p + "mlp_norm", K_RMSNORM, l, p + "xn2", B, H, H, [x1]))
            nsrc = p + "xn2"
        xo = f"x{l + 1}"
        if s.n_experts:
            NT = moe_tasks
            ops.append(OpSpec(p + "router", K_LINEAR, l, p + "rl", B, s.n_experts, 1, [nsrc], {"K": H}))
            ops.append(OpSpec(p + "route", K_ROUTER, l, p + "meta", 1, 1, 1, [p + "rl"]))
            ops.append(OpSpec(p + "expert_gate_up", K_EXPERT, l, p + "eh", 1, NT, 1,
                              [p + "meta", nsrc]))
            ops.append(OpSpec(p + "expert_down", K_EXPERT, l, p + "ey", 1, NT, 1,
                              [p + "meta", p + "eh"]))
            ops.append(OpSpec(p + "combine", K_COMBINE, l, xo, B, H, 1, [x1, p + "ey", p + "meta"]))
            x = xo
            continue
        if fusion & F_SWIGLU:
            ops.append(OpSpec(p + "gate_up", K_GATEUP, l, p + "h", B, F, 1, [nsrc], {"K": H}))
        else:
            ops.append(OpSpec(p + "gate_up", K_LINEAR, l, p + "gu", B, 2 * F, 1, [nsrc], {"K": H}))
            ops.append(OpSpec(p + "swiglu", K_SWIGLU, l, p + "h", B, F, 1, [p + "gu"], {"F": F}))
        if down_parts > 1:
            assert (fusion & F_RESID) and (fusion & F_NORM)
            xo = p + "dpart"
            ops.append(OpSpec(p + "down", K_LINEAR, l, xo, B, down_parts * H, 1, [p + "h", x1],
                              {"K": F, "resid": x1, "parts": down_parts, "H": H}))
            x, x_parts = xo, down_parts
            continue
        if fusion & F_RESID:
            ops.append(OpSpec(p + "down", K_LINEAR, l, xo, B, H, 1, [p + "h", x1],
                              {"K": F, "resid": x1}))
        else:
            ops.append(OpSpec(p + "down", K_LINEAR, l, p + "m", B, H, 1, [p + "h"], {"K": F}))
            ops.append(OpSpec(p + "resid2", K_ADD, l, xo, B, H, 1, [x1, p + "m"]))
        x = xo
    if fusion & F_NORM:
        ops.append(OpSpec("lm_head", K_LINEAR, -1, "logits", B, V, 1, [x], {"K": H}))
    else:
        ops.append(OpSpec("final_norm", K_RMSNORM, -1, "xnf", B, H, H, [x]))
        ops.append(OpSpec("lm_head", K_LINEAR, -1, "logits", B, V, 1, ["xnf"], {"K": H}))
    if greedy_loop:
        # greedy sampling as an operator, `sampling_tiles` tasks per sequence: task j finds the
        # largest of its even share of the sequence's logits and leaves (value, index) in output
        # columns 2j, 2j+1; which of them picks the token is a run-time matter
        ops.append(OpSpec("argmax", K_ARGMAX, -1, "ntok", B, 2 * sampling_tiles, 2, ["logits"],
                          {"T": sampling_tiles, "V": V}))
    return ops


def col_bounds(op: OpSpec, tc: int, explicit=None):
    """Column boundaries (tc + 1 of them) of an operator's tiles.  One even split -- except for
    the QKV projection (params["head"]), whose tiles never straddle a head: the columns are cut
    into heads first and every head evenly into the same number of tiles.
    `explicit`: boundaries handed in (a partition is the compiler's choice, Section 4.1; the
    dependency rule is what is checked): they must cut [0, cols) into tc non-empty tiles at
    multiples of the operator's unit."""
    if explicit is not None:
        b = [int(x) for x in explicit]
        assert len(b) == tc + 1 and b[0] == 0 and b[-1] == op.cols, (op.name, len(b), tc)
        assert all(x < y for x, y in zip(b, b[1:])) and all(x % op.unit == 0 for x in b), op.name
        return b
    nu = op.cols // op.unit
    head = op.meta.get("head")
    if head and nu % head == 0 and tc % (nu // head) == 0:
        per = tc // (nu // head)
        b = []
        for h in range(nu // head):
            b += [h * head + x for x in split_even(head, per)[:-1]]
        return [u * op.unit for u in b + [nu]]
    return [u * op.unit for u in split_even(nu, tc)]


def owner_map(op: OpSpec, tb: int, tc: int, explicit=None) -> np.ndarray:
    """owner[b, col] = tile index (ib * tc + ic) of the task that writes that output element."""
    assert op.cols % op.unit == 0
    rb = split_even(op.rows, tb)
    cb = col_bounds(op, tc, explicit)
    own = np.empty((op.rows, op.cols), np.int32)
    for ib in range(tb):
        for ic in range(tc):
            own[rb[ib]:rb[ib + 1], cb[ic]:cb[ic + 1]] = ib * tc + ic
    return own


def tile_bounds(op: OpSpec, tb: int, tc: int, tile: int, explicit=None):
    ib, ic = divmod(tile, tc)
    rb = split_even(op.rows, tb)
    cb = col_bounds(op, tc, explicit)
    return rb[ib], rb[ib + 1], cb[ic], cb[ic + 1]


def read_elements(op: OpSpec, tb: int, tc: int, tile: int, shapes: dict, explicit=None):
    """Elements of each input tensor that task `tile` of `op` reads, from the operator's math.
    Returns {tensor: boolean mask [rows, cols]} (masks make unions and overlaps obvious)."""
    b0, b1, c0, c1 = tile_bounds(op, tb, tc, tile, explicit)
    out = {}

    def mask(t):
        if t not in out:
            out[t] = np.zeros(shapes[t], bool)
        return out[t]

    k = op.kind
    if k == K_SERVE:
        pass                                            # request queue and metadata are not graph tensors
    elif k == K_EMBED:
        if op.ins:                                      # serving: the slot's token comes from the serve task
            mask(op.ins[0])[b0:b1, :] = True            # (otherwise token ids are external inputs)
    elif k == K_RMSNORM:
        mask(op.ins[0])[b0:b1, :] = True                # every output needs the whole row's mean
    elif k in (K_LINEAR, K_GATEUP) and op.meta.get("parts", 1) > 1:
        P, H = op.meta["parts"], op.meta["H"]
        klen = op.meta["K"] // P
        for c in range(c0, c1):                         # partial sum (part, row): that part of the input
            part, r = divmod(c, H)
            mask(op.ins[0])[b0:b1, part * klen:(part + 1) * klen] = True
            mask(op.meta["resid"])[b0:b1, r] = True
    elif k in (K_LINEAR, K_GATEUP):
        mask(op.ins[0])[b0:b1, :] = True                # a dot product over the whole input row
        if "resid" in op.meta:
            rp = op.meta.get("resid_parts", 1)
            Hh = op.cols
            for part in range(rp):                      # epilogue: + residual at the same place
                mask(op.meta["resid"])[b0:b1, part * Hh + c0:part * Hh + c1] = True
    elif k == K_ROPE:
        m = mask(op.ins[0])
        d = op.unit
        for c in range(c0, c1):                         # element and its rotation partner
            h, i = divmod(c, d)
            m[b0:b1, c] = True
            m[b0:b1, h * d + (i + d // 2) % d] = True
    elif k == K_ATTN_PARTIAL:
        M = op.meta
        C, grp, d, nq, nkv = M["C"], M["grp"], M["d"], M["nq"], M["nkv"]
        m = mask(op.ins[0])
        per = grp * (d + 2)
        if M.get("balance"):
            b0, b1 = 0, op.rows                         # any sequence may be dealt to this task
        for u in range(c0 // per, c1 // per):
            g, c = divmod(u, C)
            m[b0:b1, g * grp * d:(g + 1) * grp * d] = True         # the group's query heads
            # this step's key and value of the KV head: which chunk holds the appended row is
            # only known at run time, so every chunk task statically depends on it
            m[b0:b1, (nq + g) * d:(nq + g + 1) * d] = True
            m[b0:b1, (nq + nkv + g) * d:(nq + nkv + g + 1) * d] = True
    elif k == K_ATTN_MERGE:
        M = op.meta
        C, grp, d = M["C"], M["grp"], M["d"]
        m = mask(op.ins[0])
        for h in range(c0 // d, c1 // d):
            g, j = divmod(h, grp)
            for c in range(C):
                base = ((g * C + c) * grp + j) * (d + 2)
                m[b0:b1, base:base + d + 2] = True
    elif k == K_ADD:
        for t in op.ins:
            mask(t)[b0:b1, c0:c1] = True
    elif k == K_SWIGLU:
        F = op.meta["F"]
        m = mask(op.ins[0])
        m[b0:b1, c0:c1] = True
        m[b0:b1, F + c0:F + c1] = True
    elif k == K_ARGMAX:
        T = op.meta.get("T", 1)
        if T == 1:
            mask(op.ins[0])[b0:b1, :] = True            # the largest of all logits of the sequence
        else:
            share = split_even(op.meta["V"], T)
            for j in range(c0 // 2, c1 // 2):           # pair j: the largest of share j
                mask(op.ins[0])[b0:b1, share[j]:share[j + 1]] = True
    elif k == K_ROUTER:
        mask(op.ins[0])[:, :] = True                    # top-k of every token, lists per expert
    elif k == K_EXPERT:
        # the meta-tensor, and whichever token rows / expert-stage results routing sends here:
        # statically, all of them
        for t in op.ins:
            mask(t)[:, :] = True
    elif k == K_COMBINE:
        mask(op.ins[0])[b0:b1, c0:c1] = True            # residual at the same place
        mask(op.ins[1])[:, :] = True                    # any expert task may hold a needed output
        mask(op.ins[2])[:, :] = True                    # combine weights
    else:
        raise ValueError(k)
    return out


def producer_sets(ops, degrees):
    """degrees: list of (tb, tc) per op, or (tb, tc, column boundaries) where the partition is not
    the even split.  Returns psets[op][tile] = sorted list of (op', tile')."""
    shapes, producer, owners = {}, {}, {}
    for i, op in enumerate(ops):
        shapes[op.out] = (op.rows, op.cols)
        producer[op.out] = i
        owners[op.out] = owner_map(op, *degrees[i])
    psets = []
    for i, op in enumerate(ops):
        tb, tc = degrees[i][:2]
        explicit = degrees[i][2] if len(degrees[i]) > 2 else None
        cache, per_op = {}, []
        for tile in range(tb * tc):
            reads = read_elements(op, tb, tc, tile, shapes, explicit)
            ps = set()
            for t, m in reads.items():
                key = (t, m.tobytes())
                if key not in cache:
                    cache[key] = [(producer[t], int(o)) for o in np.unique(owners[t][m])]
                ps.update(cache[key])
            per_op.append(sorted(ps))
        psets.append(per_op)
    return psets


def canonical_bytes(psets) -> bytes:
    """Tasks in (op, tile) order; for each: count, then the sorted producer (op, tile) pairs,
    all little-endian u32."""
    out = []
    for per_op in psets:
        for ps in per_op:
            out.append(len(ps))
            for o, t in ps:
                out += [o, t]
    return np.asarray(out, "<u4").tobytes()


# =============================================================================================
# Part 2: graph transformations on explicit sets
# =============================================================================================
@dataclass
class Event:
    ins: frozenset      # InTasks(e): tasks that trigger e
    outs: frozenset     # OutTasks(e): tasks that depend on e


def pair_events(pairs):
    """Dependency analysis output: one event per producer-consumer task pair."""
    return [Event(frozenset([a]), frozenset([b])) for a, b in sorted(set(pairs))]


def successor_set_fusion(events):
    """Def. 4.1: events with equal OutTasks merge; InTasks are united."""
    by = defaultdict(set)
    for e in events:
        by[e.outs] |= e.ins
    return [Event(frozenset(i), o) for o, i in by.items()]


def predecessor_set_fusion(events):
    """Def. 4.2: events with equal InTasks merge; OutTasks are united."""
    by = defaultdict(set)
    for e in events:
        by[e.ins] |= e.outs
    return [Event(i, frozenset(o)) for i, o in by.items()]


def normalize(events, tasks):
    """Fig. 5 rewrites.  Returns (events, tasks, dummies): afterwards every task is in the InTasks
    of at most one event and in the OutTasks of at most one event.  Tasks that trigger the same
    set of several events share one new event and one dummy per original event (the reading of
    Fig. 4(e): D1, D2 serve both A1 and A2).  New dummy tasks are named ('D', n)."""
    events = [Event(e.ins, e.outs) for e in events]
    tasks = list(tasks)
    dummies = []

    def new_dummy():
        t = ("D", len(dummies))
        dummies.append(t)
        tasks.append(t)
        return t

    # (a) fan-out of a task -> 1
    trig = defaultdict(list)
    for ei, e in enumerate(events):
        for t in e.ins:
            trig[t].append(ei)
    groups = defaultdict(list)
    for t, es in trig.items():
        if len(es) > 1:
            groups[tuple(sorted(es))].append(t)
    for es, ts in sorted(groups.items(), key=lambda kv: kv[0]):
        ds = []
        for ei in es:
            dmy = new_dummy()
            ds.append(dmy)
            events[ei] = Event((events[ei].ins - frozenset(ts)) | {dmy}, events[ei].outs)
        events.append(Event(frozenset(ts), frozenset(ds)))
    # (b) fan-in of a task -> 1
    dep = defaultdict(list)
    for ei, e in enumerate(events):
        for t in e.outs:
            dep[t].append(ei)
    groups = defaultdict(list)
    for t, es in dep.items():
        if len(es) > 1:
            groups[tuple(sorted(es))].append(t)
    for es, ts in sorted(groups.items(), key=lambda kv: kv[0]):
        ds = []
        for ei in es:
            dmy = new_dummy()
            ds.append(dmy)
            events[ei] = Event(events[ei].ins, (events[ei].outs - frozenset(ts)) | {dmy})
        events.append(Event(frozenset(ds), frozenset(ts)))
    return events, tasks, dummies


def linearize(events, tasks):
    """Algorithm 1 on a normalized graph.  A start event (no triggering tasks) is added for the
    tasks that depend on nothing.  Returns (order, ranges): `order` = the task list T, `ranges`
    = {event index: (first, last)} positions in T, last inclusive; events are indexed in the order
    they were dequeued with the start event as index 0."""
    dep_of, trig_of = {}, {}
    for ei, e in enumerate(events):
        for t in e.outs:
            assert t not in dep_of, "not normalized (fan-in)"
            dep_of[t] = ei
        for t in e.ins:
            assert t not in trig_of, "not normalized (fan-out)"
            trig_of[t] = ei
    START = -1
    sources = [t for t in tasks if t not in dep_of]
    order, placed = [], set()
    queue = deque([START])
    ranges, ev_order = {}, []
    remaining = {ei: len(e.ins) for ei, e in enumerate(events)}
    while queue:
        e = queue.popleft()
        ev_order.append(e)
        members = sources if e == START else [t for t in tasks if dep_of.get(t) == e]
        first = len(order)
        for t in members:
            order.append(t)
            placed.add(t)
            e2 = trig_of.get(t)
            if e2 is not None:
                remaining[e2] -= 1
                if remaining[e2] == 0:
                    queue.append(e2)
        ranges[e] = (first, len(order) - 1)
    return order, ranges, ev_order


# =============================================================================================
# Part 3: runtime simulator
# =============================================================================================
class Deadlock(Exception):
    pass


def simulate(tasks, events, aot_queues, n_sched, rng: random.Random, producers=None,
             start_event=0, drop_trigger=None):
    """Execute a linearized, normalized tGraph the way Section 5 describes it.

    tasks[i]  = dict(dep=event or -1, trig=event or -1, jit=bool)
    events[e] = dict(required=int, first=int, last=int)   (task index range it launches)
    aot_queues[w] = list of task indices pre-enqueued on worker w (AOT tasks only)
    JIT tasks are handed out by schedulers (event e belongs to scheduler e mod n_sched), each with
    its own round-robin cursor over workers.  One random enabled action happens per tick:
    a worker finishes/starts a task, or a scheduler dispatches an activated event.
    producers[i] (optional) = set of task indices whose outputs task i reads: checked done.
    Returns a log: list of ('run', task, worker) in start order plus per-task hop counts."""
    W = len(aot_queues)
    count = [0] * len(events)
    activated = [False] * len(events)
    evq = [deque() for _ in range(max(n_sched, 1))]
    jitq = [deque() for _ in range(W)]
    aot_pos = [0] * W
    cursor = [0] * max(n_sched, 1)
    done = [False] * len(tasks)
    hops = {}
    log = []
    n_done = 0

    def activate(e):
        activated[e] = True
        if events[e]["last"] >= events[e]["first"] and any(
                tasks[t]["jit"] for t in range(events[e]["first"], events[e]["last"] + 1)):
            evq[e % max(n_sched, 1)].append(e)

    activate(start_event)
    while n_done < len(tasks):
        actions = []
        for s in range(len(evq)):
            if evq[s]:
                actions.append(("sched", s))
        for w in range(W):
            if jitq[w]:
                actions.append(("jit", w))
            elif aot_pos[w] < len(aot_queues[w]):
                t = aot_queues[w][aot_pos[w]]
                d = tasks[t]["dep"]
                if d < 0 or activated[d]:
                    actions.append(("aot", w))
        if not actions:
            stuck = [(w, aot_queues[w][aot_pos[w]]) for w in range(W)
                     if aot_pos[w] < len(aot_queues[w])]
            raise Deadlock(f"no enabled action; {n_done}/{len(tasks)} done; waiting heads {stuck[:8]}")
        kind, who = rng.choice(actions)
        if kind == "sched":
            e = evq[who].popleft()
            for t in range(events[e]["first"], events[e]["last"] + 1):
                if tasks[t]["jit"]:
                    jitq[cursor[who] % W].append(t)
                    cursor[who] += 1
            continue
        if kind == "jit":
            t = jitq[who].popleft()
            hops[t] = 2          # worker -> scheduler, scheduler -> worker
        else:
            t = aot_queues[who][aot_pos[who]]
            aot_pos[who] += 1
            hops[t] = 1          # worker -> event counter only
        d = tasks[t]["dep"]
        assert d < 0 or activated[d], f"task {t} ran before its event"
        if producers is not None:
            missing = [p for p in producers[t] if not done[p]]
            assert not missing, f"task {t} ran before producers {missing[:4]}"
        assert not done[t], f"task {t} ran twice"
        log.append(("run", t, who))
        done[t] = True
        n_done += 1
        e = tasks[t]["trig"]
        if e >= 0 and not (drop_trigger is not None and t == drop_trigger):
            count[e] += 1
            assert count[e] <= events[e]["required"]
            if count[e] == events[e]["required"]:
                activate(e)
    return log, hops
