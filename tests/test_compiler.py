"""Host compiler (libmpk) against the task-graph oracle: dependency sets bit-exact, structure
invariants, launch-mode labels, generic DAG passes, error handling.  No GPU needed."""
import os
import random
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import paper_2512_22219_amd as M
from oracle import tgraph as TG
from synth import gen as G
from tests import graph_util as GU

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "mpk.h")).read()
    declared = set(re.findall(r"\b(mpk_[a-z_]+)\s*\(", hdr))
    assert declared == set(M.binding.SYMBOLS), declared ^ set(M.binding.SYMBOLS)
    L = M.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_public_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 on its own."""
    import subprocess
    src = tmp_path / "t.c"
    src.write_text('#include "mpk.h"\nint main(void) { mpk_compile_options o = {0}; mpk_serve_config c = {0}; '
                   '(void)o; (void)c; return (int)MPK_OK; }\n')
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                           "-fsyntax-only", str(src)])


def host_graph(shape, **kw):
    kw.setdefault("host_only", 1)
    return M.compile_graph(shape, None, None, **kw)


CASES = [
    ("C1", {}, dict(fusion=0)),
    ("C1", {}, dict(fusion=7)),
    ("C1", dict(batch=3), dict(fusion=0, n_workers=16, attn_chunks=3)),
    ("C1", dict(batch=2), dict(fusion=7, n_workers=7, attn_chunks=5, tiles_pointwise=3)),
    ("C1", dict(batch=2), dict(fusion=3, n_workers=24, tiles_lm_head=100)),
    ("C2", dict(n_layers=2), dict(fusion=0)),
    ("C2", dict(n_layers=2), dict(fusion=7)),
    ("C3", dict(n_layers=1), dict(fusion=7)),
    ("C1", dict(batch=2), dict(fusion=31, n_workers=24, attn_chunks=3)),
    ("C1", dict(batch=2), dict(fusion=31, n_workers=24, attn_chunks=3, no_attn_balance=1)),
    ("C1", dict(batch=3), dict(fusion=15, n_workers=24, attn_chunks=2)),   # rope unfused: a dealt chunk task waits for every row's rope tasks
    ("C2", dict(n_layers=2), dict(fusion=31)),
    # mixture-of-experts blocks
    ("C1", dict(batch=2, ffn=0, n_experts=8, top_k=2, expert_ffn=64), dict(fusion=0, n_workers=12)),
    ("C1", dict(batch=3, ffn=0, n_experts=16, top_k=4, expert_ffn=32), dict(fusion=31, n_workers=24, tiles_moe=10)),
    ("C4", dict(n_layers=1), dict(fusion=31)),
    # batch > 4 with a long down-projection input: decomposed along the input as well
    ("C3", dict(n_layers=2), dict(fusion=31)),
    ("C1", dict(batch=8, ffn=8192), dict(fusion=31, n_workers=32)),
    # greedy sampling as an operator of the graph (multi-token launch)
    ("C1", dict(batch=3), dict(fusion=31, n_workers=24, greedy_loop=1)),
    ("C1", {}, dict(fusion=0, greedy_loop=1)),
    ("C1", dict(batch=2), dict(fusion=31, greedy_loop=1, tiles_sampling=5, tiles_lm_head=7)),   # sampling tasks that share a row
    # serving graphs (Section 6.1): the serving task first, every embedding task behind it
    ("C1", dict(batch=3), dict(fusion=31, greedy_loop=1, kv_page_size=16, kv_pages=40, serving=1)),
    ("C1", dict(batch=8), dict(fusion=31, greedy_loop=1, kv_page_size=32, kv_pages=64, serving=1, n_workers=40)),
    # QKV heads cut unevenly, 3 tiles of 43, 43, 42 rows per head: 80 heads (the 70B shape) and 48 heads
    # (the 8B shape with 240 tiles per linear operator)
    ("C5", dict(n_layers=1), dict(fusion=31)),
    ("C2", dict(n_layers=1), dict(fusion=31, tiles_linear=240)),
    # column tiles sized by the speed of the worker that runs them (workers by index mod 8)
    ("C1", dict(batch=2), dict(fusion=31, n_workers=24, worker_weight_permille=[1300, 700] * 4)),
    ("C1", dict(batch=3), dict(fusion=0, n_workers=16, worker_weight_permille=[1300, 700, 1000, 1000] * 2)),
    ("C2", dict(n_layers=2), dict(fusion=31, worker_weight_permille=[1047, 955] * 4)),
]


@pytest.mark.parametrize("base,variant,opts", CASES)
def test_dependency_sets_bit_exact_and_structure(base, variant, opts):
    shape = G.small_variant(base, **variant)
    g = host_graph(shape, **opts)
    ex = g.export()
    GU.check_structure(ex)
    C = GU.attn_chunks_of(ex, shape)
    ops, deg = GU.oracle_ops_and_degrees(shape, ex, opts.get("fusion", 0), C, not opts.get("no_attn_balance", 0))
    want = TG.producer_sets(ops, deg)
    got = GU.compiled_producer_sets(ex)
    assert TG.canonical_bytes(got) == TG.canonical_bytes(want)
    st_ = g.stats()
    assert st_["n_pair_deps"] == sum(len(p) for per in want for p in per)
    assert st_["n_tasks"] == len(ex.tasks) and st_["n_events"] == len(ex.events)


def closure_by_op_tile(psets):
    memo = {}

    def go(k):
        if k in memo:
            return memo[k]
        acc = set()
        for p in psets[k[0]][k[1]]:
            acc.add(p)
            acc |= go(p)
        memo[k] = acc
        return acc
    return {(o, t): go((o, t)) for o in range(len(psets)) for t in range(len(psets[o]))}


@pytest.mark.parametrize("base,variant,opts", CASES[:5] + CASES[8:12] + [c for c in CASES if c[2].get("serving")])
def test_transitive_reduction_keeps_closures(base, variant, opts):
    shape = G.small_variant(base, **variant)
    g = host_graph(shape, transitive_reduction=1, **opts)
    ex = g.export()
    GU.check_structure(ex)
    C = GU.attn_chunks_of(ex, shape)
    ops, deg = GU.oracle_ops_and_degrees(shape, ex, opts.get("fusion", 0), C, not opts.get("no_attn_balance", 0))
    want = TG.producer_sets(ops, deg)
    got = GU.compiled_producer_sets(ex)
    assert closure_by_op_tile(got) == closure_by_op_tile(want)
    # every kept pair is one of the oracle's direct pairs
    for o in range(len(want)):
        for t in range(len(want[o])):
            assert set(got[o][t]) <= set(want[o][t])
    assert g.stats()["n_dummy_tasks"] <= host_graph(shape, **opts).stats()["n_dummy_tasks"]


def test_simulated_execution_respects_oracle_producers():
    """Random legal interleavings of the compiled graph in the runtime simulator: every task's
    brute-force producers are finished before it runs, nothing deadlocks; and a dropped trigger
    or an out-of-order AOT queue is detected."""
    shape = G.small_variant("C1", batch=2)
    for opts in (dict(fusion=0), dict(fusion=7, transitive_reduction=1),
                 dict(fusion=7, n_sched_wgs=2)):
        g = host_graph(shape, n_workers=6, attn_chunks=3, **opts)
        ex = g.export()
        C = GU.attn_chunks_of(ex, shape)
        ops, deg = GU.oracle_ops_and_degrees(shape, ex, opts["fusion"], C, not opts.get("no_attn_balance", 0))
        want = TG.producer_sets(ops, deg)
        lin = {(int(t["op"]), int(t["tile"])): i for i, t in enumerate(ex.tasks)
               if t["op"] != GU.DUMMY}
        producers = [set() for _ in ex.tasks]
        for (o, tl), i in lin.items():
            producers[i] = {lin[p] for p in want[o][tl]}
        tasks, events, queues = GU.sim_inputs(ex)
        n_sched = int(ex.header["n_sched_wgs"]) * 4
        for seed in range(40):
            log, hops = TG.simulate(tasks, events, queues, n_sched, random.Random(seed), producers)
            assert len(log) == len(tasks)
        if opts.get("n_sched_wgs"):
            assert any(t["jit"] for t in tasks)
            assert all(hops[i] == (2 if tasks[i]["jit"] else 1) for i in range(len(tasks)))
        victim = next(i for i, t in enumerate(tasks) if t["trig"] != int(ex.header["terminal_event"]))
        with pytest.raises(TG.Deadlock):
            TG.simulate(tasks, events, queues, n_sched, random.Random(0), producers, drop_trigger=victim)
        bad = [list(q) for q in queues]
        w = next(w for w, q in enumerate(bad) if len(q) >= 2)
        bad[w][0], bad[w][-1] = bad[w][-1], bad[w][0]
        with pytest.raises((TG.Deadlock, AssertionError)):
            for seed in range(5):
                TG.simulate(tasks, events, bad, n_sched, random.Random(seed), producers)


def test_launch_mode_labels_follow_the_barrier_rule():
    """Attention is JIT; an operator downstream of a JIT operator stays JIT unless each of its
    tasks waits for all tasks of that operator (Section 5.2).  Recomputed from the oracle sets."""
    shape = G.small_variant("C1", batch=2)
    for fusion in (0, 7):
        g = host_graph(shape, n_workers=8, attn_chunks=3, n_sched_wgs=1, fusion=fusion)
        ex = g.export()
        ops, deg = GU.oracle_ops_and_degrees(shape, ex, fusion, 3)
        want = TG.producer_sets(ops, deg)
        jit = []
        for oi, op in enumerate(ops):
            if op.kind == TG.K_ATTN_PARTIAL:
                jit.append(1)
                continue
            j = 0
            for ps in want[oi]:
                per = {}
                for (po, pt) in ps:
                    per[po] = per.get(po, 0) + 1
                for po, n in per.items():
                    if jit[po] and n != deg[po][0] * deg[po][1]:
                        j = 1
            jit.append(j)
        assert list(ex.ops["jit"]) == jit
        names = [o.name for o in ops]
        assert jit[names.index("L0.attn_merge")] == 1 and jit[names.index("L0.o_proj")] == 0
        # with no scheduler every task is pre-enqueued
        ex0 = host_graph(shape, n_workers=8, attn_chunks=3, fusion=fusion).export()
        assert not ex0.tasks["jit"].any()


def test_fully_fused_8b_graph_has_no_fork_join_and_five_events_per_layer():
    """With every fusion, head-aligned QKV tiles and transitive reduction the compiled graph of
    the 8B shape is purely sequential: no dummy tasks (Section 6.5 reports none for its LLM
    graphs) and one event per operator."""
    shape = G.small_variant("C2", n_layers=3)
    g = host_graph(shape, fusion=31, transitive_reduction=1)
    s = g.stats()
    assert s["n_dummy_tasks"] == 0
    assert s["n_ops"] == 1 + 5 * 3 + 1
    ex = g.export()
    qkv = [o for o in ex.ops if o["kind"] == M.binding.OP_LINEAR and o["cols"] == 6144][0]
    # every one of the 48 heads is cut into the same number of tiles, so none straddles a head;
    # 4 per head here: the projection is small, and 64 workers stay free for the attention tasks
    assert int(qkv["tc"]) == 48 * 4
    # start and terminal events, the LM head's event, and per layer one event each for qkv, the
    # 8 attention groups, o_proj, gate_up and down
    assert s["n_events"] == 2 + 1 + 3 * (1 + 8 + 1 + 1 + 1)


def test_no_dummies_when_nothing_forks_and_paper_style_stats():
    """A purely sequential fused graph needs no normalization (Section 6.5: no fork/join groups in
    the compiled LLM graphs); event storage after linearization is 8 bytes per event."""
    shape = G.small_variant("C1", n_kv_heads=4)      # one query head per KV head
    g = host_graph(shape, fusion=7, transitive_reduction=1, attn_chunks=1, n_workers=8,
                   tiles_linear=4)
    s = g.stats()
    assert s["successor_bytes_linearized"] == 8 * s["n_events"]
    assert s["successor_bytes_unlinearized"] >= 4 * (s["n_tasks"] - 1)
    assert s["n_events_fused"] < s["n_pair_deps"]


# ------------------------------------------------------------------ generic DAG entry point
def export_as_sets(ex):
    real_in = GU.real_in_sets(ex)
    prod = {}
    for i, t in enumerate(ex.tasks):
        if t["op"] == GU.DUMMY:
            continue
        prod[int(t["tile"])] = {int(ex.tasks["tile"][p]) for p in real_in[int(t["dep_event"])]}
    return prod


def test_compile_dag_fig4_example():
    names = ["Q", "K", "V", "X", "A1", "A2", "O1", "O2", "O3", "O4", "R"]
    ix = {n: i for i, n in enumerate(names)}
    pairs = []
    for a in ("A1", "A2"):
        pairs += [(ix[s], ix[a]) for s in ("Q", "K", "V")]
        pairs += [(ix[a], ix[o]) for o in ("O1", "O2", "O3", "O4")] + [(ix[a], ix["R"])]
    pairs += [(ix["X"], ix["R"])]
    g = M.compile_dag(len(names), pairs, n_workers=4)
    s, ex = g.stats(), g.export()
    assert s["n_pair_deps"] == 17 and s["n_events_fused"] == 3 and s["n_dummy_tasks"] == 2
    GU.check_structure(ex)
    # the event that launches O1..O4 stores them as one range of four
    o_pos = sorted(i for i, t in enumerate(ex.tasks) if t["op"] != GU.DUMMY and names[t["tile"]].startswith("O"))
    assert o_pos == list(range(o_pos[0], o_pos[0] + 4))
    e = int(ex.tasks["dep_event"][o_pos[0]])
    assert (int(ex.events["first"][e]), int(ex.events["last"][e])) == (o_pos[0], o_pos[0] + 4)
    prod = export_as_sets(ex)
    assert prod[ix["R"]] == {ix["A1"], ix["A2"], ix["X"]} and prod[ix["O3"]] == {ix["A1"], ix["A2"]}


@st.composite
def random_dag(draw):
    n = draw(st.integers(2, 16))
    pairs = set()
    for b in range(1, n):
        for a in draw(st.lists(st.integers(0, b - 1), max_size=4)):
            pairs.add((a, b))
    return n, sorted(pairs)


@settings(max_examples=100, deadline=None)
@given(random_dag())
def test_compile_dag_matches_oracle_passes(gr):
    n, pairs = gr
    if not pairs:
        return
    g = M.compile_dag(n, pairs, n_workers=3)
    ex, s = g.export(), g.stats()
    GU.check_structure(ex)
    ev = TG.predecessor_set_fusion(TG.successor_set_fusion(TG.pair_events(pairs)))
    n_ev, n_tasks, dummies = TG.normalize(ev, list(range(n)))
    assert s["n_events_fused"] == len(ev)
    assert s["n_dummy_tasks"] == len(dummies)
    assert s["n_events"] == len(n_ev) + 2            # + start and terminal events
    want = {}
    for a, b in pairs:
        want.setdefault(b, set()).add(a)
    got = export_as_sets(ex)
    for t in range(n):
        assert got.get(t, set()) == want.get(t, set())


# ------------------------------------------------------------------ error handling
def test_error_paths():
    s = G.CONFIGS["C1"]
    with pytest.raises(M.MpkError) as e:
        host_graph(G.small_variant("C1", head_dim=48))
    assert e.value.status == M.binding.MPK_ERR_UNSUPPORTED
    with pytest.raises(M.MpkError) as e:
        host_graph(G.small_variant("C1", hidden=0))
    assert e.value.status == M.binding.MPK_ERR_INVALID_ARG
    with pytest.raises(M.MpkError) as e:
        host_graph(s, fusion=1 << 9)
    assert e.value.status == M.binding.MPK_ERR_INVALID_ARG
    with pytest.raises(M.MpkError) as e:
        host_graph(G.small_variant("C1", n_q_heads=3))
    assert e.value.status == M.binding.MPK_ERR_UNSUPPORTED
    cfg = M.binding.model_config(s)
    cfg.struct_size = 4
    import ctypes as C
    h = C.c_void_p()
    o = M.binding.compile_options(host_only=1)
    assert M.lib().mpk_compile(C.byref(cfg), None, None, C.byref(o), C.byref(h)) == M.binding.MPK_ERR_INVALID_ARG
    assert b"struct_size" in M.lib().mpk_last_error()
    # a host-only graph refuses to run
    g = host_graph(s)
    assert M.lib().mpk_decode_step(g._h, 1, 1, 1, None) == M.binding.MPK_ERR_INVALID_ARG
    with pytest.raises(M.MpkError):
        M.compile_dag(3, [(0, 5)])


def test_kv_batch_option_is_validated_and_leaves_the_graph_alone():
    """kv_batch only changes where a layer's cache starts: same task graph; below batch = error."""
    s = G.small_variant("C1", batch=2)
    a = host_graph(s, fusion=31).export()
    b = host_graph(s, fusion=31, kv_batch=8).export()
    assert np.array_equal(a.tasks, b.tasks) and np.array_equal(a.events, b.events)
    with pytest.raises(M.MpkError) as e:
        host_graph(s, kv_batch=1)
    assert e.value.status == M.binding.MPK_ERR_INVALID_ARG


def test_moe_error_paths_and_graph_shape():
    moe = dict(ffn=0, n_experts=8, top_k=2, expert_ffn=64)
    for bad, status in ((dict(top_k=9), M.binding.MPK_ERR_INVALID_ARG),
                        (dict(top_k=0), M.binding.MPK_ERR_INVALID_ARG),
                        (dict(expert_ffn=60), M.binding.MPK_ERR_UNSUPPORTED),
                        (dict(expert_ffn=24), M.binding.MPK_ERR_UNSUPPORTED),
                        (dict(n_experts=1024, top_k=8), M.binding.MPK_ERR_UNSUPPORTED),
                        (dict(n_experts=64, top_k=32), M.binding.MPK_ERR_UNSUPPORTED),
                        (dict(batch=16, n_experts=64, top_k=16, hidden=264), M.binding.MPK_ERR_UNSUPPORTED)):
        with pytest.raises(M.MpkError) as e:
            host_graph(G.small_variant("C1", **{**moe, **bad}))
        assert e.value.status == status, bad
    with pytest.raises(M.MpkError) as e:      # dense model with stray MoE fields
        host_graph(G.small_variant("C1", top_k=2))
    assert e.value.status == M.binding.MPK_ERR_INVALID_ARG
    g = host_graph(G.small_variant("C1", batch=2, **moe), fusion=31, n_workers=12, tiles_moe=7)
    ex = g.export()
    kinds = [int(o["kind"]) for o in ex.ops if o["layer"] == 0]
    assert kinds == [M.binding.OP_LINEAR, M.binding.OP_ATTN_PARTIAL, M.binding.OP_LINEAR, M.binding.OP_LINEAR,
                     M.binding.OP_ROUTER, M.binding.OP_EXPERT, M.binding.OP_EXPERT, M.binding.OP_COMBINE]
    per_op = {int(o["kind"]): int(o["n_tasks"]) for o in ex.ops if o["layer"] == 0}
    assert per_op[M.binding.OP_ROUTER] == 1 and per_op[M.binding.OP_EXPERT] == 7
    st_ = g.stats()
    s = G.small_variant("C1", batch=2, **moe)
    assert st_["expert_bytes"] == 3 * s.expert_ffn * s.hidden * 2
    # the selection read-back needs a device graph
    with pytest.raises(M.MpkError) as e:
        g.moe_active()
    assert e.value.status == M.binding.MPK_ERR_INVALID_ARG
    # hybrid launch labels the expert stages just-in-time and combine ahead-of-time again
    gj = host_graph(G.small_variant("C1", batch=2, **moe), fusion=31, n_workers=12, n_sched_wgs=1)
    jit = {int(o["kind"]): int(o["jit"]) for o in gj.export().ops if o["layer"] == 0}
    assert jit[M.binding.OP_EXPERT] == 1 and jit[M.binding.OP_COMBINE] == 0 and jit[M.binding.OP_ROUTER] == 0


def test_weighted_column_tiles_follow_the_worker_speeds():
    """worker_weight_permille: a linear operator's column tiles are proportional to the speed of
    the worker (index mod 8) that runs each of them; operators that are not eligible (the head-
    aligned QKV projection) keep the even split; the weights [1000] * 8 change nothing."""
    shape = G.small_variant("C2", n_layers=2)
    even = host_graph(shape, fusion=31).export()
    same = host_graph(shape, fusion=31, worker_weight_permille=[1000] * 8).export()
    assert not even.col_begin and not same.col_begin
    ex = host_graph(shape, fusion=31, worker_weight_permille=[1047, 955] * 4).export()
    assert ex.header["version"] == 2 and ex.col_begin
    worker_of = {(int(t["op"]), int(t["tile"])): int(t["worker"]) for t in ex.tasks if t["op"] != M.binding.TASK_DUMMY_OP}
    seen_kinds = set()
    for oi, op in enumerate(ex.ops):
        if oi not in ex.col_begin:
            continue
        b = ex.col_begin[oi].astype(np.int64)
        assert b[0] == 0 and b[-1] == op["cols"] and len(b) == op["tc"] + 1 and (np.diff(b) > 0).all()
        size = np.diff(b)
        fast = np.array([worker_of[(oi, i)] % 2 == 0 for i in range(int(op["tc"]))])
        # sizes follow 1047 : 955 to within the rounding of a boundary (one column either way)
        ideal = op["cols"] / op["tc"]
        assert np.all(np.abs(size[fast] - ideal * 1.047 / 1.001) <= 1.01) and np.all(np.abs(size[~fast] - ideal * 0.955 / 1.001) <= 1.01)
        seen_kinds.add(int(op["kind"]))
    assert seen_kinds == {TG.K_LINEAR, TG.K_GATEUP}     # O, down, LM head; the fused gate/up projection
    qkv = [oi for oi, op in enumerate(ex.ops) if op["kind"] == TG.K_LINEAR and op["cols"] == (shape.n_q_heads + 2 * shape.n_kv_heads) * shape.head_dim]
    assert qkv and all(oi not in ex.col_begin for oi in qkv)
    # batch > 4 runs the matrix-core body, whose tiles are made of 16-row blocks: left alone
    big = host_graph(G.small_variant("C3", n_layers=1), fusion=31, worker_weight_permille=[1047, 955] * 4).export()
    assert not big.col_begin


def test_lds_page_preload_makes_the_preloaded_tiles_larger():
    """Batch 1, all ahead-of-time: a worker that runs a QKV task and then waits through the
    attention phase pre-loads the first 16 weight rows per compute unit of its gate/up task into
    LDS pages; the gate/up tiles of those workers are 8 columns (16 rows) larger than the tiles of
    the workers that ran attention, so that all have the same amount left to stream.  8B shape:
    192 tiles of 50 columns and 64 of 42; switched off, the split is even again.  (Pages need the worker's tasks back to back, i.e. the graph
    without fork/join dummies that transitive reduction gives; its closures are compared with the
    oracle's, over these uneven tiles, in test_transitive_reduction_keeps_closures.)"""
    shape = G.small_variant("C2", n_layers=2)
    g = host_graph(shape, fusion=31, transitive_reduction=1)
    ex = g.export()
    gateup = [oi for oi, op in enumerate(ex.ops) if op["kind"] == TG.K_GATEUP]
    assert gateup and all(oi in ex.col_begin for oi in gateup) and len(ex.col_begin) == len(gateup)
    worker_of = {(int(t["op"]), int(t["tile"])): int(t["worker"]) for t in ex.tasks if t["op"] != M.binding.TASK_DUMMY_OP}
    attn_workers = {worker_of[(oi, i)] for oi, op in enumerate(ex.ops) if op["kind"] == TG.K_ATTN_PARTIAL
                    for i in range(int(op["n_tasks"]))}
    assert len(attn_workers) == 64
    for oi in gateup:
        size = np.diff(ex.col_begin[oi].astype(np.int64))
        ran_attention = np.array([worker_of[(oi, i)] in attn_workers for i in range(len(size))])
        assert set(size[~ran_attention]) == {50} and set(size[ran_attention]) == {42}
        assert size.sum() == shape.ffn
    assert g.stats()["lds_bytes"] == 160 * 1024
    off = host_graph(shape, fusion=31, transitive_reduction=1, no_lds_pages=1)
    assert not off.export().col_begin and off.stats()["lds_bytes"] < 160 * 1024
    # nothing of it with scheduler workgroups, per-operator launches, batch > 1 or pre-loading off
    for kw in (dict(n_sched_wgs=1), dict(launch_mode=1), dict(no_preload=1)):
        assert not host_graph(shape, fusion=31, transitive_reduction=1, **kw).export().col_begin
    assert not host_graph(G.small_variant("C2", n_layers=2, batch=2), fusion=31, transitive_reduction=1).export().col_begin


@pytest.mark.parametrize("tiles_per_expert,n_tasks", [(96, 256), (128, 256), (96, 37), (2, 9), (5, 1), (40, 512)])
def test_expert_tasks_share_the_active_tiles_disjointly_in_order_and_completely(tiles_per_expert, n_tasks):
    """Section 6.4, tasks re-balanced at run time: for every number of active experts the shares
    of the expert tasks are consecutive ranges that start at tile 0, end at the last tile and
    leave no gap; an expert boundary inside a share costs the task tiles (it is charged like 8),
    so shares differ by no more than that charge plus rounding, and a share that crosses no
    boundary is never smaller than one that does."""
    from paper_2512_22219_amd.binding import moe_task_share
    for n_active in [0, 1, 2, 3, 7, 82, 128]:
        total = n_active * tiles_per_expert
        at = 0
        sizes, crossing = [], []
        for task in range(n_tasks):
            first, last = moe_task_share(n_active, tiles_per_expert, n_tasks, task)
            assert first == at and last >= first, (n_active, task, first, last, at)
            at = last
            sizes.append(last - first)
            # expert boundaries strictly inside the share (a tile on each side of them)
            crossing.append(0 if last == first else (last - 1) // tiles_per_expert - first // tiles_per_expert)
        assert at == total
        if n_active:
            cost = [s + 8 * c for s, c in zip(sizes, crossing)]
            assert max(cost) - min(cost) <= 8 + 2, (n_active, max(cost), min(cost))
    with pytest.raises(M.MpkError):
        moe_task_share(3, tiles_per_expert, n_tasks, n_tasks)
    with pytest.raises(M.MpkError):
        moe_task_share(3, 0, n_tasks, 0)
