"""Pins for the serving oracle (oracle/serving.py; paper Section 6.1, "supporting runtime
dynamism"): the paged decoder against the contiguous one, the start-event task against iterations
worked by hand and against its invariants, whole serving runs against requests decoded alone.
CPU only."""
import os

import numpy as np
import pytest

from oracle import decoder as D
from oracle import serving as S
from synth import gen as G

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "serving_trace.txt")


def _small(**kw):
    return G.small_variant("C1", **kw)


# ------------------------------------------------------------------ paged decoder
@pytest.mark.parametrize("page_size,table_seed", [(16, 1), (16, 2), (64, 3)])
def test_paged_decoder_is_bit_identical_to_the_contiguous_one(page_size, table_seed):
    """Paging is indirection only: same logits to the bit, for several steps, whatever pages the
    blocks live in; the rows appended on the way land where the table says."""
    s = _small(batch=3, n_layers=2, max_seq=192)
    pos0 = np.array([37, 5, 130])
    steps = 3
    n_pages = 3 * (192 // page_size) + 5
    table = G.page_table(table_seed, s, page_size, n_pages, pos0 + steps)
    ref = D.DecoderOracle(s, G.SynthWeights(s, 7), "f32")
    pag = S.PagedDecoderOracle(s, G.PagedWeights(s, 7, table, page_size, n_pages), page_size, "f32")
    pag.page_table = table
    tok = np.array([3, 100, 77])
    for k in range(steps):
        a = ref.step(tok, pos0 + k)
        b = pag.step(tok, pos0 + k)
        assert np.isfinite(b).all()            # pages nobody owns hold NaN: none was read
        assert np.array_equal(a, b)
        tok = np.array([ref.ops.argmax(a[i]) for i in range(3)])
    for l in range(s.n_layers):
        for b in range(3):
            for t in range(pos0[b] + steps):
                pg = table[b][t // page_size]
                assert np.array_equal(pag.pool[l][0][pg, :, t % page_size], ref.kv[l][0][b, :, t])
                assert np.array_equal(pag.pool[l][1][pg, :, t % page_size], ref.kv[l][1][b, :, t])


def test_paged_decoder_follows_the_table():
    """Two sequences' first pages exchanged in the table: each now reads the other's rows, and
    both results change (the comparison above is not blind to the table)."""
    s = _small(batch=2, n_layers=1, max_seq=64)
    pos = np.array([20, 20])
    table = G.page_table(5, s, 16, 12, pos + 1)
    prov = G.PagedWeights(s, 7, table, 16, 12)
    good = S.PagedDecoderOracle(s, prov, 16, "f32")
    good.page_table = table
    swapped = table.copy()
    swapped[0, 0], swapped[1, 0] = table[1, 0], table[0, 0]
    bad = S.PagedDecoderOracle(s, prov, 16, "f32")
    bad.page_table = swapped
    a, b = good.step([1, 2], pos), bad.step([1, 2], pos)
    assert not np.array_equal(a[0], b[0]) and not np.array_equal(a[1], b[1])


# ------------------------------------------------------------------ start-event task
def _parse_golden():
    scen, cur = [], None
    ints = lambda t: [int(x) for x in t.split()]
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, body = line.split(":", 1)
        kind = head.split()[0]
        if kind == "scenario":
            cur = {"name": head.split()[1], "cfg": ints(body), "submit": [], "iter": [], "out": {}}
            scen.append(cur)
        elif kind == "submit":
            p, m = body.split("|")
            cur["submit"].append((int(head.split()[1]), ints(p), int(m)))
        elif kind == "iter":
            f = [x.strip() for x in body.split("|")]
            cur["iter"].append({"sampled": ints(f[0]), "tokens": ints(f[1]), "pos": ints(f[2]),
                                "slot_req": ints(f[3]), "table": [ints(r) for r in f[4].split(";")],
                                "free": ints(f[5]), "promised": int(f[6])})
        elif kind == "out":
            cur["out"][int(head.split()[1])] = ints(body)
    return scen


@pytest.mark.parametrize("sc", _parse_golden(), ids=lambda sc: sc["name"])
def test_start_event_task_reproduces_the_hand_worked_iterations(sc):
    B, ps, n_pages, max_seq, eos = sc["cfg"]
    st = S.ServeState(B, ps, n_pages, max_seq, eos)
    for k, it in enumerate(sc["iter"]):
        for when, prompt, max_new in sc["submit"]:
            if when == k:
                st.submit(prompt, max_new)
        tokens, positions = st.begin_iteration(it["sampled"])
        assert tokens == it["tokens"], k
        assert positions == it["pos"], k
        assert st.slot_req == it["slot_req"], k
        assert [row[:2] for row in st.table] == it["table"], k
        assert st.free == it["free"], k
        assert st.promised == it["promised"], k
    for r, want in sc["out"].items():
        assert st.requests[r].out == want
        assert st.requests[r].state == S.DONE


@pytest.mark.parametrize("seed", range(6))
def test_start_event_task_invariants_under_random_arrivals(seed):
    """Whatever arrives and whatever is sampled: no page has two owners, no page is lost, a pop
    never finds the stack empty, requests start in arrival order, the running requests fill the
    lowest slots in arrival order, every request is fed its prompt
    and then its own outputs at positions 0, 1, 2, ..., and ends on the end-of-sequence token or
    with max_new tokens."""
    rng = np.random.default_rng(seed)
    B, ps, max_seq, eos = int(rng.integers(1, 9)), int(rng.choice([2, 4, 8])), 32, 3
    n_pages = B + int(rng.integers(max_seq // ps, 3 * max_seq // ps))
    st = S.ServeState(B, ps, n_pages, max_seq, eos)
    fed = {}
    started = []
    sampled = [0] * B
    n_req = 0
    for k in range(4000):
        if n_req < 40 and rng.random() < 0.4:
            for _ in range(int(rng.integers(1, 4))):
                plen = int(rng.integers(1, 12))
                st.submit(rng.integers(4, 50, plen).tolist(), int(rng.integers(1, max_seq - plen + 2)))
                n_req += 1
        tokens, positions = st.begin_iteration(sampled)
        n_run = st.n_running()
        assert all(r >= 0 for r in st.slot_req[:n_run]) and all(r < 0 for r in st.slot_req[n_run:])
        assert st.slot_req[:n_run] == sorted(st.slot_req[:n_run])      # ranks closed, order kept
        owned = [pg for b in range(B) if st.slot_req[b] >= 0 for pg in st.table[b][:st.slot_held[b]]]
        assert len(set(owned)) == len(owned)
        assert sorted(owned + st.free) == list(range(B, n_pages))
        assert 0 <= st.promised <= len(st.free)
        for b in range(B):
            r = st.slot_req[b]
            if r < 0:
                assert (tokens[b], positions[b], st.table[b][0]) == (0, 0, b)
                continue
            if r not in fed:
                started.append(r)
            assert st.slot_held[b] == positions[b] // ps + 1
            assert all(pg >= B for pg in st.table[b][:st.slot_held[b]])
            fed.setdefault(r, []).append((positions[b], tokens[b]))
        sampled = rng.integers(0, 50, B).tolist()      # token 3 = end of sequence, now and then
        if n_req >= 40 and st.q_head == n_req and st.n_running() == 0:
            break
    assert started == list(range(n_req))
    for r, q in enumerate(st.requests):
        assert q.state == S.DONE
        assert 1 <= len(q.out) <= q.max_new
        assert (q.out[-1] == eos or len(q.out) == q.max_new) and eos not in q.out[:-1]
        want = q.prompt + q.out[:-1]
        assert fed[r] == list(enumerate(want))


def test_a_request_that_can_never_fit_is_refused_at_submission():
    st = S.ServeState(2, 4, 2 + 3, 32, 0)
    with pytest.raises(AssertionError):
        st.submit([1] * 10, 8)       # 17 rows = 5 pages > 3
    with pytest.raises(AssertionError):
        st.submit([1] * 30, 4)       # 33 rows > max_seq


# ------------------------------------------------------------------ whole iterations
def test_served_requests_produce_what_they_produce_alone():
    """Continuous batching changes WHEN a request runs and WHERE its rows live, never what it
    computes: every request's tokens equal those of the same request decoded alone on the
    contiguous oracle (prompt fed token by token, then greedy)."""
    s = _small(batch=3, n_layers=2, max_seq=32)
    s1 = _small(batch=1, n_layers=2, max_seq=32)
    rng = np.random.default_rng(3)
    reqs = [(rng.integers(0, s.vocab, int(rng.integers(1, 6))).tolist(), int(rng.integers(1, 7)))
            for _ in range(7)]

    def alone(prompt, max_new, eos):
        ref = D.DecoderOracle(s1, G.SynthWeights(s1, 9), "f32")
        out = []
        tok = prompt[0]
        for pos in range(len(prompt) + max_new - 1):
            lg = ref.step([tok], [pos])
            if pos + 1 < len(prompt):
                tok = prompt[pos + 1]
                continue
            tok = ref.ops.argmax(lg[0])
            out.append(tok)
            if tok == eos or len(out) == max_new:
                break
        return out

    # an end-of-sequence token that really occurs: the second token request 1 produces alone
    eos = alone(reqs[1][0], 6, -1)[1]
    reqs[1] = (reqs[1][0], 6)
    ps, n_pages = 4, 3 + 7
    table0 = np.full((3, 32 // ps), -1)
    srv = S.ServingOracle(s, G.PagedWeights(s, 9, table0, ps, n_pages), ps, n_pages, eos, "f32")
    ids = [srv.submit(*reqs[i]) for i in range(4)]
    for k in range(60):
        if k == 5:
            ids += [srv.submit(*reqs[i]) for i in range(4, 7)]
        srv.iteration()
        assert np.isfinite(srv.last_logits).all()
    for r, (prompt, max_new) in zip(ids, reqs):
        out, state = srv.outputs(r)
        assert state == S.DONE
        assert out == alone(prompt, max_new, eos), r
    assert len(srv.outputs(ids[1])[0]) == 2     # the end-of-sequence path was taken
