"""Pins for the task-graph oracle (oracle/tgraph.py): the worked example of Fig. 4 as far as the
paper's text fixes it, Defs. 4.1/4.2 as properties, the normalization post-condition, the
guarantees stated in Algorithm 1's caption, and the runtime rules of Sections 3 and 5."""
import random

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import tgraph as TG
from synth import gen as G


# ------------------------------------------------------------------ helpers
def direct_producers(events):
    p = {}
    for e in events:
        for t in e.outs:
            p.setdefault(t, set()).update(e.ins)
    return p


def closure(prod, through=lambda t: False):
    """Transitive producer sets; tasks for which `through` holds (dummies) are looked through
    and not reported."""
    memo = {}

    def go(t):
        if t in memo:
            return memo[t]
        memo[t] = set()
        acc = set()
        for p in prod.get(t, ()):
            acc |= go(p)
            if not through(p):
                acc.add(p)
        memo[t] = acc
        return acc
    return {t: go(t) for t in list(prod)}


def real_direct(prod_norm, t, is_dummy):
    """Direct REAL producers of t in a normalized graph: walk back through dummy tasks."""
    out, stack = set(), list(prod_norm.get(t, ()))
    while stack:
        p = stack.pop()
        if is_dummy(p):
            stack += list(prod_norm.get(p, ()))
        else:
            out.add(p)
    return out


is_dummy = lambda t: isinstance(t, tuple) and t[0] == "D"


# ------------------------------------------------------------------ Fig. 4 worked example
def fig4_pairs():
    """Q, K, V -> attention A (2 tasks) -> output projection O (4 tasks) and RMSNorm R, which
    also needs an independent input X, so O and R can run in parallel after A."""
    pairs = []
    for a in ("A1", "A2"):
        pairs += [("Q", a), ("K", a), ("V", a)]
        pairs += [(a, o) for o in ("O1", "O2", "O3", "O4")]
        pairs += [(a, "R")]
    pairs += [("X", "R")]
    tasks = ["Q", "K", "V", "X", "A1", "A2", "O1", "O2", "O3", "O4", "R"]
    return tasks, pairs


def test_fig4_fusions_and_two_dummies():
    tasks, pairs = fig4_pairs()
    ev = TG.pair_events(pairs)
    assert len(ev) == 17
    s = TG.successor_set_fusion(ev)
    # the two pair events (A1,O1), (A2,O1) became one event that O1 waits on
    o1 = [e for e in s if e.outs == frozenset(["O1"])]
    assert len(o1) == 1 and o1[0].ins == frozenset(["A1", "A2"])
    assert len(s) == 7                      # one per consumer task: A1 A2 O1..O4 R
    p = TG.predecessor_set_fusion(s)
    # the four events that all depend on {A1, A2} became one, which launches four tasks
    eo = [e for e in p if e.ins == frozenset(["A1", "A2"])]
    assert len(eo) == 1 and eo[0].outs == frozenset(["O1", "O2", "O3", "O4"])
    assert len(p) == 3                      # {QKV}->{A1,A2}, {A1,A2}->{O*}, {A1,A2,X}->{R}
    # A1 and A2 each trigger two events (O's and R's) -> normalization adds exactly D1, D2
    n_ev, n_tasks, dummies = TG.normalize(p, tasks)
    assert len(dummies) == 2
    assert len(n_ev) == 4
    trig = {}
    dep = {}
    for e in n_ev:
        for t in e.ins:
            assert t not in trig
            trig[t] = e
        for t in e.outs:
            assert t not in dep
            dep[t] = e
    assert trig["A1"] is trig["A2"] and trig["A1"].outs == frozenset(dummies)
    # dependencies seen through the dummies are unchanged
    before = direct_producers(p)
    after = direct_producers(n_ev)
    for t in tasks:
        assert real_direct(after, t, is_dummy) == before.get(t, set())
    order, ranges, ev_order = TG.linearize(n_ev, n_tasks)
    assert sorted(map(str, order)) == sorted(map(str, n_tasks))
    pos = {t: i for i, t in enumerate(order)}
    # the event launching the four O tasks stores them as one contiguous range
    o_pos = sorted(pos[o] for o in ("O1", "O2", "O3", "O4"))
    assert o_pos == list(range(o_pos[0], o_pos[0] + 4))


def test_fanin_rewrite_on_handmade_graph():
    # T0 depends on two events that cannot be fused (different InTasks, and e1 has another consumer)
    ev = [TG.Event(frozenset(["a"]), frozenset(["T0", "u"])), TG.Event(frozenset(["b"]), frozenset(["T0"]))]
    n_ev, n_tasks, dummies = TG.normalize(ev, ["a", "b", "u", "T0"])
    assert len(dummies) == 2
    dep = [e for e in n_ev if "T0" in e.outs]
    assert len(dep) == 1 and dep[0].ins == frozenset(dummies)
    after = direct_producers(n_ev)
    assert real_direct(after, "T0", is_dummy) == {"a", "b"}
    assert real_direct(after, "u", is_dummy) == {"a"}


# ------------------------------------------------------------------ properties on random DAGs
@st.composite
def random_dag_pairs(draw):
    n = draw(st.integers(2, 14))
    pairs = set()
    for b in range(1, n):
        for a in draw(st.lists(st.integers(0, b - 1), max_size=4)):
            pairs.add((a, b))
    return n, sorted(pairs)


@settings(max_examples=150, deadline=None)
@given(random_dag_pairs())
def test_fusion_normalization_linearization_properties(g):
    n, pairs = g
    tasks = list(range(n))
    ev0 = TG.pair_events(pairs)
    base = direct_producers(ev0)
    s = TG.successor_set_fusion(ev0)
    assert direct_producers(s) == base                       # Def 4.1 keeps every dependency
    assert len({e.outs for e in s}) == len(s)
    p = TG.predecessor_set_fusion(s)
    assert direct_producers(p) == base                       # Def 4.2 too
    assert len({e.ins for e in p}) == len(p) and len({e.outs for e in p}) == len(p)
    # fixed point: a second round changes nothing
    again = TG.predecessor_set_fusion(TG.successor_set_fusion(p))
    assert {(e.ins, e.outs) for e in again} == {(e.ins, e.outs) for e in p}
    # after the two passes every task waits on at most one event
    for t in tasks:
        assert sum(t in e.outs for e in p) <= 1
    n_ev, n_tasks, dummies = TG.normalize(p, tasks)
    for t in n_tasks:
        assert sum(t in e.ins for e in n_ev) <= 1 and sum(t in e.outs for e in n_ev) <= 1
    forks = {t for t in tasks if sum(t in e.ins for e in p) > 1}
    assert (len(dummies) > 0) == (len(forks) > 0)             # dummies only where a fork exists
    after = direct_producers(n_ev)
    for t in tasks:
        assert real_direct(after, t, is_dummy) == base.get(t, set())
    order, ranges, ev_order = TG.linearize(n_ev, n_tasks)
    assert len(order) == len(n_tasks) and len(set(order)) == len(order)   # each task once
    assert len(set(ev_order)) == len(ev_order) == len(n_ev) + 1           # each event once
    pos = {t: i for i, t in enumerate(order)}
    for ei, e in enumerate(n_ev):                                          # contiguity
        ps = sorted(pos[t] for t in e.outs)
        assert ps == list(range(ps[0], ps[0] + len(ps)))
        assert ranges[ei] == (ps[0], ps[-1])
    for a, b in pairs:                                                     # topological
        assert pos[a] < pos[b]


# ------------------------------------------------------------------ dependency brute force
def test_split_even_rule():
    assert TG.split_even(10, 4) == [0, 3, 6, 8, 10]
    assert TG.split_even(3, 5) == [0, 1, 2, 3, 3, 3]


def test_col_bounds_hand_written_boundaries():
    """The column rule of the QKV projection (decomposition, Section 4.1; uneven splits are this
    build's reading: the first n mod k tiles are one unit longer).  Every expected list below is
    written out by hand, none is computed."""
    def qkv(cols, head):
        return TG.OpSpec("qkv", TG.K_LINEAR, 0, "qkv", 1, cols, 1, ["x"], {"K": 8, "head": head})
    # 2 heads of 8 columns in 6 tiles: 3 tiles per head of 3, 3, 2 columns
    assert TG.col_bounds(qkv(16, 8), 6) == [0, 3, 6, 8, 11, 14, 16]
    # 3 heads of 4 columns in 3 tiles: exactly the heads
    assert TG.col_bounds(qkv(12, 4), 3) == [0, 4, 8, 12]
    # 3 heads of 4 columns in 6 tiles: halves of heads
    assert TG.col_bounds(qkv(12, 4), 6) == [0, 2, 4, 6, 8, 10, 12]
    # the 70B-shaped case: heads of 128 columns, 3 tiles each -> 43, 43, 42 within every head
    b = TG.col_bounds(qkv(10 * 128, 128), 30)
    assert b[:7] == [0, 43, 86, 128, 171, 214, 256] and b[-4:] == [1152, 1195, 1238, 1280]
    assert len(b) == 31 and all(b[3 * h] == 128 * h for h in range(11))     # no tile straddles a head
    # a tile count that is not a multiple of the number of heads: one even split over all columns
    # (12 columns in 5 tiles: 3, 3, 2, 2, 2), which does straddle heads
    assert TG.col_bounds(qkv(12, 4), 5) == [0, 3, 6, 8, 10, 12]
    # an operator without the head rule splits evenly whatever the tile count
    lin = TG.OpSpec("o", TG.K_LINEAR, 0, "o", 1, 16, 1, ["x"], {"K": 8})
    assert TG.col_bounds(lin, 6) == [0, 3, 6, 9, 12, 14, 16]
    # columns that come in units (an attention head of 4 columns): boundaries are multiples of it
    rope = TG.OpSpec("rope", TG.K_ROPE, 0, "q", 1, 20, 4, ["qkv"])
    assert TG.col_bounds(rope, 3) == [0, 8, 16, 20]
    # the owner map follows the boundaries: tile index per column, for both batch rows of a 2 x 2 split
    own = TG.owner_map(TG.OpSpec("qkv", TG.K_LINEAR, 0, "qkv", 2, 16, 1, ["x"], {"K": 8, "head": 8}), 2, 6)
    assert own[0].tolist() == [0, 0, 0, 1, 1, 1, 2, 2, 3, 3, 3, 4, 4, 4, 5, 5]
    assert own[1].tolist() == [6, 6, 6, 7, 7, 7, 8, 8, 9, 9, 9, 10, 10, 10, 11, 11]


def test_explicit_column_boundaries_hand_written():
    """A partition handed in instead of the even split (tiles sized by worker speed): the oracle
    takes the boundaries as they are, refuses anything that is not a partition of the columns into
    non-empty tiles, and the brute-force producer sets follow the uneven tiles.  Expected values
    written out by hand."""
    lin = TG.OpSpec("gate_up", TG.K_LINEAR, 0, "gu", 1, 10, 1, ["x"], {"K": 4})
    assert TG.col_bounds(lin, 3, [0, 5, 7, 10]) == [0, 5, 7, 10]
    assert TG.owner_map(lin, 1, 3, [0, 5, 7, 10])[0].tolist() == [0, 0, 0, 0, 0, 1, 1, 2, 2, 2]
    assert TG.tile_bounds(lin, 1, 3, 1, [0, 5, 7, 10]) == (0, 1, 5, 7)
    for bad in ([0, 5, 7], [1, 5, 7, 10], [0, 5, 5, 10], [0, 7, 5, 10], [0, 5, 7, 9]):
        with pytest.raises(AssertionError):
            TG.col_bounds(lin, 3, bad)
    rope = TG.OpSpec("rope", TG.K_ROPE, 0, "q", 1, 12, 4, ["qkv"])
    with pytest.raises(AssertionError):
        TG.col_bounds(rope, 2, [0, 6, 12])            # not at a multiple of the unit
    # a pointwise consumer cut 0..4 | 4..10 over a producer cut 0..5 | 5..7 | 7..10:
    # its first tile overlaps producer tile 0 only, its second tile all three
    src = TG.OpSpec("src", TG.K_EMBED, -1, "x", 1, 4, 4, [])
    add = TG.OpSpec("add", TG.K_ADD, 0, "y", 1, 10, 1, ["gu", "gu"])
    ps = TG.producer_sets([src, lin, add], [(1, 1), (1, 3, [0, 5, 7, 10]), (1, 2, [0, 4, 10])])
    assert ps[2] == [[(1, 0)], [(1, 0), (1, 1), (1, 2)]]
    # the same consumer over the even split 0..4 | 4..7 | 7..10 of the producer
    ps = TG.producer_sets([src, lin, add], [(1, 1), (1, 3), (1, 2, [0, 4, 10])])
    assert ps[2] == [[(1, 0)], [(1, 1), (1, 2)]]


def test_argmax_read_set_hand_written():
    """Greedy sampling (one task per sequence) reads every logit of its own sequence and nothing
    else, so it depends on every LM-head tile that holds a column of that row (Section 4.1's
    overlap rule).  Expected sets written out by hand for 2 sequences x 10 logits."""
    lm = TG.OpSpec("lm_head", TG.K_LINEAR, -1, "logits", 2, 10, 1, ["x"], {"K": 4})
    am = TG.OpSpec("argmax", TG.K_ARGMAX, -1, "ntok", 2, 1, 1, ["logits"])
    shapes = {"logits": (2, 10), "x": (2, 4)}
    for b in range(2):
        r = TG.read_elements(am, 2, 1, b, shapes)
        assert list(r) == ["logits"]
        want = [[False] * 10, [False] * 10]
        want[b] = [True] * 10
        assert r["logits"].tolist() == want
    src = TG.OpSpec("src", TG.K_EMBED, -1, "x", 2, 4, 4, [])
    # LM head cut into 1 x 3 column tiles over both rows: each sampling task needs all three
    ps = TG.producer_sets([src, lm, am], [(2, 1), (1, 3), (2, 1)])
    assert ps[2] == [[(1, 0), (1, 1), (1, 2)], [(1, 0), (1, 1), (1, 2)]]
    # LM head cut 2 x 3 (a tile per sequence and column range): only the own row's three tiles
    ps = TG.producer_sets([src, lm, am], [(2, 1), (2, 3), (2, 1)])
    assert ps[2] == [[(1, 0), (1, 1), (1, 2)], [(1, 3), (1, 4), (1, 5)]]


def test_sampling_tasks_that_share_a_row_read_their_share_only():
    """The sampling operator cut into T tasks per sequence: task j reads the j-th even share of the
    sequence's logits, so it depends on the LM-head tiles that overlap that share and no others.
    Written out by hand for 2 sequences x 10 logits, T = 2 (shares [0, 5) and [5, 10)), LM head in
    3 column tiles [0, 4), [4, 7), [7, 10)."""
    lm = TG.OpSpec("lm_head", TG.K_LINEAR, -1, "logits", 2, 10, 1, ["x"], {"K": 4})
    am = TG.OpSpec("argmax", TG.K_ARGMAX, -1, "ntok", 2, 4, 2, ["logits"], {"T": 2, "V": 10})
    src = TG.OpSpec("src", TG.K_EMBED, -1, "x", 2, 4, 4, [])
    shapes = {"logits": (2, 10), "x": (2, 4)}
    r = TG.read_elements(am, 2, 2, 3, shapes)        # sequence 1, share 1
    assert r["logits"].tolist() == [[False] * 10, [False] * 5 + [True] * 5]
    ps = TG.producer_sets([src, lm, am], [(2, 1), (1, 3), (2, 2)])
    assert ps[2] == [[(1, 0), (1, 1)], [(1, 1), (1, 2)], [(1, 0), (1, 1)], [(1, 1), (1, 2)]]


def test_serving_task_read_sets_hand_written():
    """Serving inside the graph (Section 6.1): ONE task on the start event prepares the iteration
    and writes a metadata element per batch slot; the embedding task of slot b reads element b.
    Expected sets written out by hand for 3 slots: the serving task has no producer, every
    embedding task has exactly that task, and in the whole operator list of a small model every
    other task is downstream of it."""
    sv = TG.OpSpec("serve", TG.K_SERVE, -1, "slots", 3, 1, 1, [])
    em = TG.OpSpec("embed", TG.K_EMBED, -1, "x0", 3, 4, 4, ["slots"])
    shapes = {"slots": (3, 1), "x0": (3, 4)}
    assert TG.read_elements(sv, 1, 1, 0, shapes) == {}
    for b in range(3):
        r = TG.read_elements(em, 3, 1, b, shapes)
        assert list(r) == ["slots"]
        assert r["slots"].tolist() == [[i == b] for i in range(3)]
    ps = TG.producer_sets([sv, em], [(1, 1), (3, 1)])
    assert ps == [[[]], [[(0, 0)], [(0, 0)], [(0, 0)]]]
    s = G.small_variant("C1", batch=3, n_layers=1)
    ops = TG.build_ops(s, 31, 2, greedy_loop=True, serving=True)
    assert [o.kind for o in ops[:2]] == [TG.K_SERVE, TG.K_EMBED]
    plain = TG.build_ops(s, 31, 2, greedy_loop=True)
    assert [o.name for o in ops[2:]] == [o.name for o in plain[1:]]
    deg = tiny_degrees(ops)
    deg[0] = (1, 1)        # one task, whatever the number of slots
    psets = TG.producer_sets(ops, deg)
    reached = {(0, 0)}
    for i, per_op in enumerate(psets):
        for t, prod in enumerate(per_op):
            if (i, t) != (0, 0):
                assert prod and all(p in reached for p in prod), (ops[i].name, t)
                reached.add((i, t))


def tiny_degrees(ops, lin=4, rope=None, merge=2, pw=1):
    deg = []
    for op in ops:
        if op.kind in (TG.K_LINEAR, TG.K_GATEUP):
            deg.append((1, lin))
        elif op.kind == TG.K_ROPE:
            deg.append((op.rows, rope or op.cols // op.unit))
        elif op.kind == TG.K_ATTN_PARTIAL:
            deg.append((op.rows, op.cols // op.unit))
        elif op.kind == TG.K_ATTN_MERGE:
            deg.append((op.rows, merge))
        else:
            deg.append((op.rows, pw))
    return deg


def test_producer_sets_spot_checks_unfused():
    s = G.small_variant("C1", n_layers=1, batch=2)
    ops = TG.build_ops(s, 0, attn_chunks=3)
    names = [o.name for o in ops]
    assert names == ["embed", "L0.attn_norm", "L0.qkv", "L0.rope", "L0.attn_partial",
                     "L0.attn_merge", "L0.o_proj", "L0.resid1", "L0.mlp_norm", "L0.gate_up",
                     "L0.swiglu", "L0.down", "L0.resid2", "final_norm", "lm_head"]
    deg = tiny_degrees(ops)
    ps = TG.producer_sets(ops, deg)
    ix = {n: i for i, n in enumerate(names)}
    # norm of batch row 1 needs only embed's row-1 task
    assert ps[ix["L0.attn_norm"]][1] == [(ix["embed"], 1)]
    # every linear tile needs the norm tasks of all batch rows
    assert all(p == [(ix["L0.attn_norm"], 0), (ix["L0.attn_norm"], 1)] for p in ps[ix["L0.qkv"]])
    # rope of head slot h (512 qkv rows in 4 tiles of 128 = 2 heads each) needs qkv tile h//2
    nslots = s.n_q_heads + 2 * s.n_kv_heads
    for b in range(2):
        for h in range(nslots):
            assert ps[ix["L0.rope"]][b * nslots + h] == [(ix["L0.qkv"], h // 2)]
    # attention partial (b, g, c): q heads of group g and this step's k and v of KV head g
    C, grp = 3, s.n_q_heads // s.n_kv_heads
    for b in range(2):
        for g in range(s.n_kv_heads):
            for c in range(C):
                want = {(ix["L0.rope"], b * nslots + h) for h in range(g * grp, (g + 1) * grp)}
                want |= {(ix["L0.rope"], b * nslots + s.n_q_heads + g),
                         (ix["L0.rope"], b * nslots + s.n_q_heads + s.n_kv_heads + g)}
                assert set(ps[ix["L0.attn_partial"]][(b * s.n_kv_heads + g) * C + c]) == want
    # merge tile = 2 heads = one group -> all chunks of that (b, group)
    for b in range(2):
        for g in range(s.n_kv_heads):
            want = {(ix["L0.attn_partial"], (b * s.n_kv_heads + g) * C + c) for c in range(C)}
            assert set(ps[ix["L0.attn_merge"]][b * 2 + g]) == want
    # residual add (one tile per batch row) needs x0's row task and every o_proj tile
    assert set(ps[ix["L0.resid1"]][0]) == {(ix["embed"], 0)} | {(ix["L0.o_proj"], t) for t in range(4)}
    # swiglu reads gate and up halves: with 4 gate_up tiles over 2F rows, one h tile over all F
    assert set(ps[ix["L0.swiglu"]][0]) == {(ix["L0.gate_up"], t) for t in range(4)}


def test_producer_sets_of_attention_tasks_dealt_to_the_sequences_at_run_time():
    """With the merge fused and more than one sequence, a chunk task may be handed any sequence
    (Section 5.2's run-time imbalance, met by a length-proportional deal): it statically needs
    the query / new key / new value columns of its KV head from EVERY row.  Unfused rope makes the
    difference visible (rope tasks are per row); with one sequence, or the merge as an operator
    of its own, nothing changes."""
    s = G.small_variant("C1", n_layers=1, batch=3)
    fusion = TG.F_MERGE
    C = 2
    for balance in (False, True):
        ops = TG.build_ops(s, fusion, attn_chunks=C, attn_balance=balance)
        names = [o.name for o in ops]
        ix = {n: i for i, n in enumerate(names)}
        assert "L0.attn_merge" not in ix
        ps = TG.producer_sets(ops, tiny_degrees(ops))
        nslots = s.n_q_heads + 2 * s.n_kv_heads
        grp = s.n_q_heads // s.n_kv_heads
        for b in range(3):
            for g in range(s.n_kv_heads):
                for c in range(C):
                    rows = range(3) if balance else [b]
                    want = set()
                    for r in rows:
                        want |= {(ix["L0.rope"], r * nslots + g * grp + j) for j in range(grp)}
                        want |= {(ix["L0.rope"], r * nslots + s.n_q_heads + g),
                                 (ix["L0.rope"], r * nslots + s.n_q_heads + s.n_kv_heads + g)}
                    assert set(ps[ix["L0.attn_partial"]][(b * s.n_kv_heads + g) * C + c]) == want
    # no effect without the fused merge, or with a single sequence
    a = TG.build_ops(s, 0, attn_chunks=C, attn_balance=True)
    assert not [o for o in a if o.kind == TG.K_ATTN_PARTIAL][0].meta["balance"]
    s1 = G.small_variant("C1", n_layers=1, batch=1)
    a = TG.build_ops(s1, fusion, attn_chunks=C, attn_balance=True)
    assert not [o for o in a if o.kind == TG.K_ATTN_PARTIAL][0].meta["balance"]


def test_producer_sets_fused_residual_reads_only_its_tile():
    s = G.small_variant("C1", n_layers=2)
    fusion = TG.F_NORM | TG.F_RESID | TG.F_SWIGLU
    ops = TG.build_ops(s, fusion, attn_chunks=2)
    names = [o.name for o in ops]
    assert names[:6] == ["embed", "L0.qkv", "L0.rope", "L0.attn_partial", "L0.attn_merge", "L0.o_proj"]
    ps = TG.producer_sets(ops, tiny_degrees(ops))
    ix = {n: i for i, n in enumerate(names)}
    # layer-1 o_proj tile j: all merge tasks + layer-0 down tile j (its residual slice)
    for j in range(4):
        want = {(ix["L1.attn_merge"], t) for t in range(2)} | {(ix["L0.down"], j)}
        assert set(ps[ix["L1.o_proj"]][j]) == want


def test_producer_sets_mixture_of_experts_block():
    """Section 6.4 chain: router -> route -> expert gate/up -> expert down -> combine, with the
    static supersets spelled out by hand."""
    s = G.small_variant("C1", n_layers=1, batch=2, ffn=0, n_experts=8, top_k=2, expert_ffn=64)
    fusion = TG.F_NORM | TG.F_RESID | TG.F_SWIGLU
    NT = 5
    ops = TG.build_ops(s, fusion, attn_chunks=2, moe_tasks=NT)
    names = [o.name for o in ops]
    assert names == ["embed", "L0.qkv", "L0.rope", "L0.attn_partial", "L0.attn_merge", "L0.o_proj",
                     "L0.router", "L0.route", "L0.expert_gate_up", "L0.expert_down", "L0.combine",
                     "lm_head"]
    deg = []
    for op in ops:
        if op.kind == TG.K_EXPERT:
            deg.append((1, NT))
        elif op.kind == TG.K_ROUTER:
            deg.append((1, 1))
        elif op.kind == TG.K_COMBINE:
            deg.append((op.rows, 2))
        elif op.name == "L0.router":
            deg.append((1, 2))
        else:
            deg.append(tiny_degrees([op])[0])
    ps = TG.producer_sets(ops, deg)
    ix = {n: i for i, n in enumerate(names)}
    o_tiles = {(ix["L0.o_proj"], t) for t in range(4)}
    # the router is a linear operator over x1: every o_proj tile, for both of its row tiles
    assert all(set(p) == o_tiles for p in ps[ix["L0.router"]])
    # route: one task, every router tile (it needs every token's choice)
    assert ps[ix["L0.route"]] == [[(ix["L0.router"], 0), (ix["L0.router"], 1)]]
    # an expert gate/up task: the meta-tensor (route) + all of x1, whatever the routing
    for t in range(NT):
        assert set(ps[ix["L0.expert_gate_up"]][t]) == {(ix["L0.route"], 0)} | o_tiles
        # an expert down task: the meta-tensor + every gate/up task
        assert set(ps[ix["L0.expert_down"]][t]) == {(ix["L0.route"], 0)} | {(ix["L0.expert_gate_up"], u) for u in range(NT)}
    # combine tile (row b, column half c): every expert-down task, the meta-tensor, and the
    # o_proj tiles that hold its residual slice (4 tiles of 64 columns; half c = tiles 2c, 2c+1)
    for b in range(2):
        for c in range(2):
            want = {(ix["L0.expert_down"], u) for u in range(NT)} | {(ix["L0.route"], 0)} \
                | {(ix["L0.o_proj"], 2 * c), (ix["L0.o_proj"], 2 * c + 1)}
            assert set(ps[ix["L0.combine"]][b * 2 + c]) == want
    # the next reader of the residual stream sees combine's tiles
    assert all(set(p) == {(ix["L0.combine"], t) for t in range(4)} for p in ps[ix["lm_head"]])


def test_producer_sets_down_projection_cut_along_its_input():
    s = G.small_variant("C1", n_layers=2, batch=1, ffn=1024)
    fusion = TG.F_NORM | TG.F_RESID | TG.F_SWIGLU
    P, H = 4, s.hidden
    ops = TG.build_ops(s, fusion, attn_chunks=2, down_parts=P)
    names = [o.name for o in ops]
    ix = {n: i for i, n in enumerate(names)}
    down = ops[ix["L0.down"]]
    assert (down.rows, down.cols) == (1, P * H)
    deg = []
    for op in ops:
        if op.name.endswith(".down"):
            deg.append((1, 8))          # 2 row blocks (128 rows) x 4 parts
        elif op.name.endswith(".gate_up"):
            deg.append((1, 8))          # 8 tiles of 128 of the 1024 columns of h
        else:
            deg.append(tiny_degrees([op])[0])
    ps = TG.producer_sets(ops, deg)
    # down tile = part * 2 + row block; part p reads h[256 p, 256 (p + 1)) = gate/up tiles 2p, 2p+1,
    # and the residual x1 at its 128 rows = o_proj tiles 2 rb, 2 rb + 1 (4 tiles of 64)
    for part in range(P):
        for rb in range(2):
            want = {(ix["L0.gate_up"], 2 * part), (ix["L0.gate_up"], 2 * part + 1),
                    (ix["L0.o_proj"], 2 * rb), (ix["L0.o_proj"], 2 * rb + 1)}
            assert set(ps[ix["L0.down"]][part * 2 + rb]) == want
    # the next layer's QKV reads the whole residual stream: every (row block, part) task
    assert all(set(p) == {(ix["L0.down"], t) for t in range(8)} for p in ps[ix["L1.qkv"]])
    # the next layer's o_proj tile j (64 columns) adds residual columns [64 j, 64 j + 64): row
    # block j // 2, all four parts
    for j in range(4):
        res = {(ix["L0.down"], part * 2 + j // 2) for part in range(P)}
        assert res <= set(ps[ix["L1.o_proj"]][j])
        assert not any(o == ix["L0.down"] and (o, t) not in res for o, t in ps[ix["L1.o_proj"]][j])


# ------------------------------------------------------------------ runtime simulator
def small_linear_graph():
    """a0,a1 -> e1 -> b0,b1,b2 -> e2 -> c0 ; start event 0 launches a*."""
    tasks = [dict(dep=0, trig=1, jit=False), dict(dep=0, trig=1, jit=False),
             dict(dep=1, trig=2, jit=True), dict(dep=1, trig=2, jit=True), dict(dep=1, trig=2, jit=True),
             dict(dep=2, trig=3, jit=False)]
    events = [dict(required=0, first=0, last=1), dict(required=2, first=2, last=4),
              dict(required=3, first=5, last=5), dict(required=1, first=6, last=5)]
    producers = [set(), set(), {0, 1}, {0, 1}, {0, 1}, {2, 3, 4}]
    return tasks, events, producers


def test_simulator_random_schedules_and_hops():
    tasks, events, producers = small_linear_graph()
    for seed in range(1000):
        rng = random.Random(seed)
        log, hops = TG.simulate(tasks, events, [[0, 5], [1]], 2, rng, producers)
        assert len(log) == len(tasks)
        assert all(hops[t] == (2 if tasks[t]["jit"] else 1) for t in range(len(tasks)))


def test_simulator_detects_dropped_trigger_and_bad_aot_order():
    tasks, events, producers = small_linear_graph()
    with pytest.raises(TG.Deadlock):
        TG.simulate(tasks, events, [[0, 5], [1]], 2, random.Random(0), producers, drop_trigger=1)
    # AOT queue not a subsequence of the linearized order: worker 0 waits on c0 first while it
    # also owns a0 -> nothing can ever run
    with pytest.raises(TG.Deadlock):
        TG.simulate(tasks, events, [[5, 0], [1]], 2, random.Random(0), producers)
