"""Helpers that turn an exported compiled graph into the forms the task-graph oracle checks."""
import numpy as np

from oracle import tgraph as TG

DUMMY = 0xFFFFFFFF


def in_tasks_by_event(ex):
    order = np.argsort(ex.tasks["trig_event"], kind="stable")
    trig = ex.tasks["trig_event"][order]
    out = {}
    bounds = np.flatnonzero(np.diff(trig)) + 1
    for seg in np.split(order, bounds):
        if len(seg):
            out[int(ex.tasks["trig_event"][seg[0]])] = seg
    return out


def real_in_sets(ex):
    """event -> sorted array of REAL task indices (linearized numbering) that must finish before
    the event activates, looking back through dummy tasks."""
    ins = in_tasks_by_event(ex)
    is_dummy = ex.tasks["op"] == DUMMY
    memo = {}

    def go(e):
        if e in memo:
            return memo[e]
        acc = []
        for t in ins.get(e, ()):
            if is_dummy[t]:
                acc.append(go(int(ex.tasks["dep_event"][t])))
            else:
                acc.append(np.array([t]))
        memo[e] = np.unique(np.concatenate(acc)) if acc else np.zeros(0, np.int64)
        return memo[e]
    for e in range(len(ex.events)):
        go(e)
    return memo


def compiled_producer_sets(ex):
    """psets[op][tile] = sorted list of (op, tile) producers, from the exported tables only."""
    real_in = real_in_sets(ex)
    ops, tasks = ex.ops, ex.tasks
    psets = [[None] * int(o["n_tasks"]) for o in ops]
    key = tasks["op"].astype(np.int64) * (1 << 32) + tasks["tile"]
    cache = {}
    for i in range(len(tasks)):
        if tasks["op"][i] == DUMMY:
            continue
        e = int(tasks["dep_event"][i])
        if e not in cache:
            p = real_in[e]
            k = np.sort(key[p])
            cache[e] = [(int(v >> 32), int(v & 0xFFFFFFFF)) for v in k]
        psets[int(tasks["op"][i])][int(tasks["tile"][i])] = cache[e]
    return psets


def moe_tasks_of(ex):
    """Expert tasks per expert stage of a compiled mixture-of-experts graph (0 for a dense one)."""
    for eo in ex.ops:
        if eo["kind"] == TG.K_EXPERT:
            return int(eo["cols"])
    return 0


def down_parts_of(ex, shape):
    """Input parts of the down projection (1 unless it was decomposed along its input too): the
    last linear operator of a dense layer writes hidden columns per part."""
    if shape.n_experts:
        return 1
    last = [eo for eo in ex.ops if eo["layer"] == 0 and eo["kind"] == TG.K_LINEAR][-1]
    return int(last["cols"]) // shape.hidden


def oracle_ops_and_degrees(shape, ex, fusion, attn_chunks, attn_balance=True):
    """attn_balance: the compile option's default (chunk tasks dealt to the sequences at run time
    where the merge is fused and the batch has more than one sequence); False for graphs compiled
    with no_attn_balance=1."""
    greedy = any(eo["kind"] == TG.K_ARGMAX for eo in ex.ops)
    serving = any(eo["kind"] == TG.K_SERVE for eo in ex.ops)
    sampling_tiles = max([int(eo["cols"]) // 2 for eo in ex.ops if eo["kind"] == TG.K_ARGMAX] or [1])
    ops = TG.build_ops(shape, fusion, attn_chunks, moe_tasks_of(ex), down_parts_of(ex, shape), greedy,
                       attn_balance, serving, sampling_tiles)
    assert len(ops) == len(ex.ops), (len(ops), len(ex.ops))
    for o, eo in zip(ops, ex.ops):
        assert o.kind == eo["kind"] and o.layer == eo["layer"], (o.name, o.kind, eo["kind"])
        assert (o.rows, o.cols) == (eo["rows"], eo["cols"]), o.name
    degrees = [(int(eo["tb"]), int(eo["tc"])) + ((ex.col_begin[i].tolist(),) if i in ex.col_begin else ())
               for i, eo in enumerate(ex.ops)]
    return ops, degrees


def attn_chunks_of(ex, shape):
    grp = shape.n_q_heads // shape.n_kv_heads
    for eo in ex.ops:
        if eo["kind"] == TG.K_ATTN_PARTIAL:
            return int(eo["cols"]) // (shape.n_kv_heads * grp * (shape.head_dim + 2))
    raise AssertionError("no attention operator")


def check_structure(ex):
    """Invariants of a normalized, linearized graph (Algorithm 1's guarantees and Section 3)."""
    t, ev = ex.tasks, ex.events
    n = len(t)
    # every event's required count equals the number of tasks that trigger it
    counts = np.bincount(t["trig_event"], minlength=len(ev))
    assert np.array_equal(counts, ev["required"])
    # tasks launched by one event are exactly its contiguous range
    dep = t["dep_event"]
    assert np.all(np.diff(dep.astype(np.int64)) >= 0)      # events are numbered in the order Algorithm 1 dequeues them
    for e in range(len(ev)):
        f, l = int(ev["first"][e]), int(ev["last"][e])
        assert np.all(dep[f:l] == e)
    assert int((ev["last"].astype(np.int64) - ev["first"]).sum()) == n      # each task once
    # topological: a task's triggering event launches only later tasks
    first_of_trig = ev["first"][t["trig_event"]]
    last_of_trig = ev["last"][t["trig_event"]]
    nonempty = last_of_trig > first_of_trig
    assert np.all(first_of_trig[nonempty] > np.arange(n)[nonempty])
    # AOT queues: each AOT task once, on its worker, in increasing linear order
    seen = np.zeros(n, bool)
    for w in range(len(ex.aot_off) - 1):
        q = ex.aot[ex.aot_off[w]:ex.aot_off[w + 1]]
        assert np.all(np.diff(q.astype(np.int64)) > 0)
        assert np.all(t["worker"][q] == w) and not seen[q].any()
        seen[q] = True
    assert np.array_equal(seen, t["jit"] == 0)
    assert np.all(t["worker"][t["jit"] == 1] == -1)


def sim_inputs(ex):
    tasks = [dict(dep=int(a["dep_event"]), trig=int(a["trig_event"]), jit=bool(a["jit"]))
             for a in ex.tasks]
    events = [dict(required=int(e["required"]), first=int(e["first"]), last=int(e["last"]) - 1)
              for e in ex.events]
    queues = [list(map(int, ex.aot[ex.aot_off[w]:ex.aot_off[w + 1]]))
              for w in range(len(ex.aot_off) - 1)]
    return tasks, events, queues
