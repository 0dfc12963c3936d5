"""GPU parity of the paged KV cache and of serving inside the task graph (paper Section 6.1,
"supporting runtime dynamism") against oracle/serving.py, through the C-ABI.

Integer work (slot table, page tables, free stack, queue, tokens fed, positions) is compared bit
for bit; logits to the tolerance of the other parity tests, with the appended K/V rows held (see
tests/gpu_util.py)."""
import numpy as np
import pytest
import torch

import paper_2512_22219_amd as M
from oracle import decoder as D
from oracle import serving as S
from synth import gen as G
from synth.device import DeviceModel
from tests.gpu_util import check_rows_are_valid_roundings, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-2
FUSED = dict(fusion=31, transitive_reduction=1)


def _nan_pool(s, n_pages, ps, dev):
    pool = torch.full((s.n_layers, n_pages, s.n_kv_heads, ps, s.head_dim), G.BF16_NAN_BITS,
                      dtype=torch.int16, device=dev)
    return pool.view(torch.bfloat16)


def _rows(pool, table, positions, ps):
    """Rows the step appended: uint16 [L][B][n_kv][d], gathered through the table."""
    out = []
    for b, p in enumerate(positions):
        pg = int(table[b][int(p) // ps])
        out.append(pool[:, pg, :, int(p) % ps, :])
    r = torch.stack(out, 1).contiguous()
    return r.view(torch.int16).cpu().numpy().view(np.uint16)


class PagedGpu:
    """Device model whose seeded contiguous cache is re-filed into pages under `table`."""

    def __init__(self, s, seed, table, ps, n_pages, **opts):
        self.s, self.ps, self.n_pages = s, ps, n_pages
        self.model = DeviceModel(s, seed)
        dev = self.model.device
        self.pool_k, self.pool_v = _nan_pool(s, n_pages, ps, dev), _nan_pool(s, n_pages, ps, dev)
        if table is not None:
            for b in range(s.batch):
                for i, pg in enumerate(table[b]):
                    if pg >= 0:
                        self.pool_k[:, pg] = self.model.k[:, b, :, i * ps:(i + 1) * ps, :]
                        self.pool_v[:, pg] = self.model.v[:, b, :, i * ps:(i + 1) * ps, :]
        self.graph = M.compile_graph(s, self.model.weight_ptrs(), (self.pool_k.data_ptr(), self.pool_v.data_ptr()),
                                     kv_page_size=ps, kv_pages=n_pages, **opts)
        self.tok = torch.zeros(s.batch, dtype=torch.int32, device=dev)
        self.pos = torch.zeros(s.batch, dtype=torch.int32, device=dev)
        self.logits = torch.empty((s.batch, s.vocab), dtype=torch.float32, device=dev)

    def close(self):
        self.graph.destroy()


@pytest.mark.parametrize("variant,ps,opts", [
    (dict(batch=3, n_layers=2), 16, FUSED),
    (dict(batch=1, n_layers=2), 64, FUSED),
    (dict(batch=8, n_layers=2, head_dim=128, n_q_heads=4, n_kv_heads=2), 32, FUSED),
    (dict(batch=8, n_layers=2, head_dim=128, n_q_heads=8, n_kv_heads=2), 32, FUSED),      # the kernels compiled for 4 heads per KV head
    (dict(batch=2, n_q_heads=8, n_kv_heads=1), 16, dict(fusion=23)),                      # merge operator of its own
    (dict(batch=4, ffn=0, n_experts=8, top_k=2, expert_ffn=64), 16, FUSED),
    (dict(batch=3, n_layers=2), 8, dict(fusion=31, launch_mode=1)),                       # kernel per operator
])
def test_paged_cache_matches_oracle_for_a_shuffled_page_table(variant, ps, opts):
    """One decode step after another on a cache whose pages are scattered over the pool: logits
    within tolerance of the paged oracle, appended rows are valid roundings and sit in the page
    the table names, and no page outside the table is touched."""
    s = G.small_variant("C1", max_seq=192, **variant)
    rng = np.random.default_rng(5)
    pos0 = rng.integers(1, 180, s.batch)
    pos0[0] = 2 * ps - 1                      # the next row opens a page
    steps = 3
    n_pages = s.batch * (192 // ps) + 7
    table = G.page_table(11, s, ps, n_pages, pos0 + steps)
    gpu = PagedGpu(s, 4, table, ps, n_pages, **opts)
    dev = gpu.model.device
    d_table = torch.as_tensor(table, dtype=torch.int32, device=dev).contiguous()
    stream = torch.cuda.current_stream().cuda_stream
    with pytest.raises(M.MpkError):           # no table yet
        gpu.graph.decode_step(gpu.tok.data_ptr(), gpu.pos.data_ptr(), gpu.logits.data_ptr(), stream)
    gpu.graph.set_page_table(d_table.data_ptr())
    ref = S.PagedDecoderOracle(s, G.PagedWeights(s, 4, table, ps, n_pages), ps, "f32")
    ref.page_table = table
    tok = rng.integers(0, s.vocab, s.batch)
    for k in range(steps):
        pos = pos0 + k
        gpu.tok.copy_(torch.as_tensor(tok.astype(np.int32)))
        gpu.pos.copy_(torch.as_tensor(pos.astype(np.int32)))
        gpu.logits.fill_(float("nan"))
        gpu.graph.decode_step(gpu.tok.data_ptr(), gpu.pos.data_ptr(), gpu.logits.data_ptr(), stream)
        torch.cuda.synchronize()
        gpu.graph.status()
        got = gpu.logits.cpu().numpy()
        k_rows, v_rows = _rows(gpu.pool_k, table, pos, ps), _rows(gpu.pool_v, table, pos, ps)
        experts = None
        if s.n_experts:
            ex, _ = gpu.graph.moe_selection()
            experts = ex.reshape(s.n_layers, s.batch, s.top_k).astype(np.int32)
        want = ref.step(tok, pos, held=D.Held(k_rows, v_rows, experts))
        check_rows_are_valid_roundings(k_rows, ref.last_k_exact)
        check_rows_are_valid_roundings(v_rows, ref.last_v_exact)
        assert rel_err(got, want) < TOL, (k, rel_err(got, want))
        tok = got.argmax(-1)
    owned = np.unique(table[table >= 0])
    others = np.setdiff1d(np.arange(n_pages), owned)
    for pool in (gpu.pool_k, gpu.pool_v):
        raw = pool.view(torch.int16)[:, torch.as_tensor(others, device=dev)]
        assert bool((raw == G.BF16_NAN_BITS).all())
    gpu.close()


def test_a_page_outside_the_pool_is_reported_and_never_dereferenced():
    s = G.small_variant("C1", max_seq=64, batch=2)
    ps, n_pages = 16, 12
    table = G.page_table(3, s, ps, n_pages, [40, 40])
    gpu = PagedGpu(s, 4, table, ps, n_pages, **FUSED)
    bad = table.copy()
    bad[1, 1] = n_pages + 1000
    d_table = torch.as_tensor(bad, dtype=torch.int32, device=gpu.model.device).contiguous()
    gpu.graph.set_page_table(d_table.data_ptr())
    gpu.pos.fill_(38)
    gpu.graph.decode_step(gpu.tok.data_ptr(), gpu.pos.data_ptr(), gpu.logits.data_ptr(),
                          torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    with pytest.raises(M.MpkError) as e:
        gpu.graph.status()
    assert e.value.status == M.binding.MPK_ERR_DEVICE and "page" in str(e.value)
    gpu.close()


# ------------------------------------------------------------------ serving
def _requests(rng, vocab, n, max_prompt, max_new):
    return [(rng.integers(0, vocab, int(rng.integers(1, max_prompt + 1))).tolist(), int(rng.integers(1, max_new + 1)))
            for _ in range(n)]


def _same_state(gs, st, k):
    snap = st.snapshot()
    assert gs["slot_req"] == snap["slot_req"], k
    assert gs["slot_pos"] == snap["slot_pos"], k
    assert gs["slot_held"] == snap["slot_held"], k
    assert gs["table"] == snap["table"], k
    assert gs["free"] == snap["free"], k
    assert (gs["promised"], gs["q_head"]) == (snap["promised"], snap["q_head"]), k


@pytest.mark.parametrize("variant,ps,n_pages,opts", [
    (dict(batch=3, n_layers=2), 8, 3 + 4, FUSED),
    (dict(batch=8, n_layers=1, head_dim=128, n_q_heads=4, n_kv_heads=2), 16, 8 + 5, FUSED),
    (dict(batch=2, n_layers=1), 8, 2 + 3, dict(fusion=31, launch_mode=1)),
])
def test_serving_iterations_match_the_oracle_one_by_one(variant, ps, n_pages, opts):
    """One iteration per launch, the state read back after each: the start-event task's decisions
    (who leaves, who enters, which page, which token at which position) equal the oracle's bit for
    bit when it is given the tokens the GPU sampled; every iteration's logits are within
    tolerance of the paged oracle on the same metadata.  The pool is too small for the queue, so
    requests wait for pages and for slots."""
    s = G.small_variant("C1", max_seq=48, **variant)
    rng = np.random.default_rng(21)
    reqs = _requests(rng, s.vocab, 4 * s.batch, 6, 9)
    gpu = PagedGpu(s, 4, None, ps, n_pages, greedy_loop=1, serving=1, **opts)
    dev = gpu.model.device
    stream = torch.cuda.current_stream().cuda_stream
    # an end-of-sequence token that occurs: whatever the second iteration samples for slot 0
    probe = gpu.graph.serve(8, 8, 8, -1)
    probe.submit(reqs[0][0], 8, stream)
    probe.run(len(reqs[0][0]) + 1, stream)
    torch.cuda.synchronize()
    eos = probe.result(0)[0][-1]
    probe.destroy()
    gpu.pool_k.view(torch.int16).fill_(G.BF16_NAN_BITS)
    gpu.pool_v.view(torch.int16).fill_(G.BF16_NAN_BITS)

    srv = gpu.graph.serve(64, 8, 16, eos)
    st = S.ServeState(s.batch, ps, n_pages, s.max_seq, eos)
    table0 = np.full((s.batch, s.max_seq // ps), -1)
    ref = S.PagedDecoderOracle(s, G.PagedWeights(s, 4, table0, ps, n_pages), ps, "f32")
    sampled = [0] * s.batch
    submitted = 0
    saw_wait = False
    for k in range(200):
        if k in (0, 9, 10, 30) and submitted < len(reqs):
            for r in reqs[submitted:submitted + s.batch]:
                assert srv.submit(r[0], r[1], stream) == st.submit(r[0], r[1])
            submitted += s.batch
        tokens, positions = st.begin_iteration(sampled)
        srv.run(1, stream)
        torch.cuda.synchronize()
        gpu.graph.status()
        gs = srv.state()
        _same_state(gs, st, k)
        assert gs["positions"] == positions, k
        assert gs["q_tail"] == submitted and gs["iterations"] == k + 1
        saw_wait = saw_wait or (st.q_head < submitted and st.n_running() < s.batch)
        got = _server_logits(srv, s, dev)
        k_rows, v_rows = _rows(gpu.pool_k, st.table, positions, ps), _rows(gpu.pool_v, st.table, positions, ps)
        ref.page_table = st.table
        want = ref.step(tokens, positions, held=D.Held(k_rows, v_rows))
        check_rows_are_valid_roundings(k_rows, ref.last_k_exact)
        check_rows_are_valid_roundings(v_rows, ref.last_v_exact)
        assert rel_err(got, want) < TOL, (k, rel_err(got, want))
        sampled = got.argmax(-1).tolist()
        assert gs["tokens"] == sampled, k       # (after the launch the token array holds what it sampled;
                                                #  that the right tokens were FED shows in the logits)
        if submitted == len(reqs) and st.q_head == submitted and st.n_running() == 0:
            break
    assert saw_wait                                   # a request did wait for pages with a slot idle
    assert all(q.state == S.DONE for q in st.requests)
    assert any(q.out[-1] == eos and len(q.out) < q.max_new for q in st.requests)   # the end-of-sequence path
    for r, q in enumerate(st.requests):
        assert srv.result(r) == (q.out, S.DONE)
    assert gs["tokens_produced"] == sum(len(q.out) for q in st.requests)
    srv.destroy()
    gpu.close()


class _DeviceWords:
    """A raw device address as something torch.as_tensor understands."""

    def __init__(self, ptr, n):
        self.__cuda_array_interface__ = {"shape": (n,), "typestr": "<f4", "data": (ptr, False), "version": 2}


def _server_logits(srv, s, dev):
    """Copy of the server's logits buffer [batch][vocab] as numpy."""
    t = torch.as_tensor(_DeviceWords(srv.logits_ptr(), s.batch * s.vocab), device=dev)
    return t.clone().cpu().numpy().reshape(s.batch, s.vocab)


@pytest.mark.parametrize("variant,ps,n_pages,n_iter,extra", [
    (dict(batch=3, n_layers=2), 8, 3 + 12, 7, {}),
    (dict(batch=8, n_layers=2, head_dim=128, n_q_heads=4, n_kv_heads=2), 16, 8 + 14, 25, {}),
    (dict(batch=4, ffn=0, n_experts=8, top_k=2, expert_ffn=64), 8, 4 + 10, 11, {}),
    # every task starts after a pseudo-random delay, buffers that cross tasks are poisoned before
    # each launch: a task that read metadata or activations too early would show
    (dict(batch=3, n_layers=2), 8, 3 + 12, 5, dict(debug_flags=M.binding.DEBUG_POISON | M.binding.DEBUG_JITTER)),
    (dict(batch=1, n_layers=2), 16, 1 + 3, 9, {}),
    (dict(batch=3, n_layers=2), 8, 3 + 12, 6, dict(tiles_sampling=4)),
    # batch <= 4, one launch of the loop kernel for all iterations (the default is a launch per iteration)
    (dict(batch=3, n_layers=2), 8, 3 + 12, 7, dict(greedy_loop=2)),
    (dict(batch=1, n_layers=2), 16, 1 + 3, 9, dict(greedy_loop=2, debug_flags=M.binding.DEBUG_JITTER)),
    # batch 8: serving calls are a launch per iteration by default as well; the one launch of the loop kernel
    (dict(batch=8, n_layers=2, head_dim=128, n_q_heads=4, n_kv_heads=2), 16, 8 + 14, 25, dict(greedy_loop=2)),
    # the kernels compiled for head dimension 128 and 4 query heads per KV head (dense, batch 5..16): both launch forms
    (dict(batch=8, n_layers=2, head_dim=128, n_q_heads=8, n_kv_heads=2), 16, 8 + 14, 25, {}),
    (dict(batch=8, n_layers=2, head_dim=128, n_q_heads=8, n_kv_heads=2), 16, 8 + 14, 25, dict(greedy_loop=2)),
    (dict(batch=8, n_layers=1, head_dim=128, n_q_heads=8, n_kv_heads=1, ffn=0, n_experts=8, top_k=2, expert_ffn=64), 8, 8 + 20, 9, {}),
    (dict(batch=8, n_layers=1, head_dim=128, n_q_heads=8, n_kv_heads=1, ffn=0, n_experts=8, top_k=2, expert_ffn=64), 8, 8 + 20, 9,
     dict(greedy_loop=2, debug_flags=M.binding.DEBUG_JITTER)),
])
def test_many_iterations_per_launch_serve_every_request_as_if_alone(variant, ps, n_pages, n_iter, extra):
    """The kernel keeps running through n_iter iterations per launch (no host round trip between
    tokens, none for retiring or admitting): every request ends with the tokens the whole-iteration
    oracle produces -- which are the tokens of the request decoded alone -- the final state equals
    the oracle's, and all pages are back on the stack."""
    s = G.small_variant("C1", max_seq=48, **variant)
    rng = np.random.default_rng(8)
    reqs = _requests(rng, s.vocab, 3 * s.batch + 1, 5, 8)
    table0 = np.full((s.batch, s.max_seq // ps), -1)
    ora = S.ServingOracle(s, G.PagedWeights(s, 4, table0, ps, n_pages), ps, n_pages, -1, "f32")
    # end of sequence: the second token request 0 produces when nothing ends early
    for r in reqs:
        ora.submit(*r)
    while not all(q.state == S.DONE for q in ora.state.requests):
        ora.iteration()
    eos = ora.state.requests[0].out[min(1, len(ora.state.requests[0].out) - 1)]
    ora = S.ServingOracle(s, G.PagedWeights(s, 4, table0, ps, n_pages), ps, n_pages, eos, "f32")
    gpu = PagedGpu(s, 4, None, ps, n_pages, **{"greedy_loop": 1, "serving": 1, **FUSED, **extra})
    stream = torch.cuda.current_stream().cuda_stream
    srv = gpu.graph.serve(64, 8, 8, eos)
    half = len(reqs) // 2
    for r in reqs[:half]:
        assert srv.submit(r[0], r[1], stream) == ora.submit(*r)
    launches = ran = 0
    while launches < 40:
        if launches == 1:
            for r in reqs[half:]:
                assert srv.submit(r[0], r[1], stream) == ora.submit(*r)
        srv.run(n_iter, stream)
        ran += ora.launch(n_iter)
        launches += 1
        torch.cuda.synchronize()
        gpu.graph.status()
        gs = srv.state()
        assert gs["iterations"] == ran, launches      # (a launch ends with the iteration that finds the server drained)
        if launches > 1 and gs["q_head"] == len(reqs) and all(r < 0 for r in gs["slot_req"]):
            break
    # a launch with nothing to do is over after one iteration, and the events are where a launch
    # that ran all its steps would have left them: the next launch serves a new request
    srv.run(9, stream)
    assert ora.launch(9) == 1
    torch.cuda.synchronize()
    gpu.graph.status()
    assert srv.state()["iterations"] == ran + 1
    assert srv.submit(reqs[0][0], reqs[0][1], stream) == ora.submit(*reqs[0])
    srv.run(40, stream)
    more = ora.launch(40)
    torch.cuda.synchronize()
    gpu.graph.status()
    gs = srv.state()
    assert gs["iterations"] == ran + 1 + more and more < 40
    assert srv.result(len(reqs)) == ora.outputs(len(reqs))
    _same_state(gs, ora.state, launches)
    assert sorted(gs["free"]) == list(range(s.batch, n_pages)) and gs["promised"] == 0
    for r in range(len(reqs)):
        assert srv.result(r) == ora.outputs(r), r
    srv.destroy()
    gpu.close()


def test_serving_entry_points_refuse_what_they_cannot_run():
    s = G.small_variant("C1", max_seq=48, batch=2)
    model = DeviceModel(s, 4)
    kv = model.kv_ptrs()
    with pytest.raises(M.MpkError):      # serving without a paged cache
        M.compile_graph(s, model.weight_ptrs(), kv, fusion=31, greedy_loop=1, serving=1)
    with pytest.raises(M.MpkError):      # paged cache with the rotation as an operator of its own
        M.compile_graph(s, model.weight_ptrs(), kv, fusion=15, kv_page_size=16, kv_pages=8)
    with pytest.raises(M.MpkError):      # page size not a power of two
        M.compile_graph(s, model.weight_ptrs(), kv, fusion=31, kv_page_size=24, kv_pages=8)
    gpu = PagedGpu(s, 4, None, 8, 2 + 4, greedy_loop=1, serving=1, **FUSED)
    stream = torch.cuda.current_stream().cuda_stream
    with pytest.raises(M.MpkError):      # a serving graph runs through its server
        gpu.graph.decode_steps(1, gpu.tok.data_ptr(), gpu.pos.data_ptr(), 0, gpu.logits.data_ptr(), 0, stream)
    srv = gpu.graph.serve(4, 8, 48, -1)
    with pytest.raises(M.MpkError):      # one server per graph
        gpu.graph.serve(4, 8, 8, -1)
    with pytest.raises(M.MpkError):      # 8 + 42 - 1 = 49 rows, max_seq is 48
        srv.submit([1] * 8, 42, stream)
    with pytest.raises(M.MpkError):      # 33 rows = 5 pages, only 4 can ever be free
        srv.submit([1] * 8, 26, stream)
    with pytest.raises(M.MpkError):      # token outside the vocabulary
        srv.submit([s.vocab], 1, stream)
    for _ in range(4):
        srv.submit([1, 2], 2, stream)
    with pytest.raises(M.MpkError):      # max_requests taken
        srv.submit([1, 2], 2, stream)
    srv.run(12, stream)
    torch.cuda.synchronize()
    gpu.graph.status()
    assert [srv.result(r)[1] for r in range(4)] == [S.DONE] * 4
    srv.destroy()
    gpu.close()


def test_a_served_graph_set_runs_the_smallest_graph_that_holds_the_open_requests():
    """A graph per power-of-two batch size over ONE server state (Section 6.1: the graph that fits
    the current batch is selected at run time; here by the host, per launch).  The running
    requests always fill the lowest slots, so whichever graph runs sees all of them: the outputs of
    every request and the final state equal the full-batch oracle's, and the batch size of the
    graph launched follows the number of open requests."""
    s = G.small_variant("C1", max_seq=48, batch=8, n_layers=2)
    ps, n_pages = 8, 8 + 16
    model = DeviceModel(s, 4)
    dev = model.device
    pool_k, pool_v = _nan_pool(s, n_pages, ps, dev), _nan_pool(s, n_pages, ps, dev)
    gset = M.compile_set(s, model.weight_ptrs(), (pool_k.data_ptr(), pool_v.data_ptr()), greedy_loop=1, serving=1,
                         kv_page_size=ps, kv_pages=n_pages, **FUSED)
    assert len(gset) == 4
    stream = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(17)
    reqs = _requests(rng, s.vocab, 12, 4, 6)
    table0 = np.full((s.batch, s.max_seq // ps), -1)
    ora = S.ServingOracle(s, G.PagedWeights(s, 4, table0, ps, n_pages), ps, n_pages, -1, "f32")
    srv = gset.serve(32, 8, 8, -1)
    # (requests submitted before the launch, iterations, batch size of the graph that must run)
    plan = [(1, 3, 1), (1, 2, 2), (5, 4, 8), (0, 30, 2), (2, 3, 2), (0, 20, 2), (3, 2, 4), (0, 25, 2)]
    nxt = 0
    for n_new, n_iter, want_batch in plan:
        for r in reqs[nxt:nxt + n_new]:
            assert srv.submit(r[0], r[1], stream) == ora.submit(*r)
        nxt += n_new
        srv.run(n_iter, stream)
        ora.launch(n_iter)
        torch.cuda.synchronize()
        srv.status()
        assert srv.last_batch() == want_batch, (nxt, srv.last_batch(), want_batch)
        _same_state(srv.state(), ora.state, nxt)          # (also tells the host how many have finished)
    assert nxt == len(reqs)
    for r in range(len(reqs)):
        assert srv.result(r) == ora.outputs(r), r
        assert srv.result(r)[1] == S.DONE
    srv.destroy()
    gset.destroy()


def test_a_graph_set_over_a_paged_cache_needs_no_batch_extent():
    """mpk_compile_set over a paged pool (no serving): every graph reads the same pool through
    the table it was given, so the graph for 2 sequences runs the first two rows of a table laid
    out for 4."""
    s = G.small_variant("C1", max_seq=64, batch=4)
    ps, n_pages = 16, 4 * 4 + 3
    pos = np.array([20, 33, 5, 47])
    table = G.page_table(9, s, ps, n_pages, pos + 1)
    model = DeviceModel(s, 4)
    dev = model.device
    pool_k, pool_v = _nan_pool(s, n_pages, ps, dev), _nan_pool(s, n_pages, ps, dev)
    for b in range(s.batch):
        for i, pg in enumerate(table[b]):
            if pg >= 0:
                pool_k[:, pg] = model.k[:, b, :, i * ps:(i + 1) * ps, :]
                pool_v[:, pg] = model.v[:, b, :, i * ps:(i + 1) * ps, :]
    gset = M.compile_set(s, model.weight_ptrs(), (pool_k.data_ptr(), pool_v.data_ptr()), kv_page_size=ps, kv_pages=n_pages, **FUSED)
    d_table = torch.as_tensor(table, dtype=torch.int32, device=dev).contiguous()
    for i in range(len(gset)):
        gset.graph(i).set_page_table(d_table.data_ptr())
    ref = S.PagedDecoderOracle(s, G.PagedWeights(s, 4, table, ps, n_pages), ps, "f32")
    ref.page_table = table
    tok = np.array([7, 8, 9, 10])
    d_tok = torch.as_tensor(tok.astype(np.int32), device=dev)
    d_pos = torch.as_tensor(pos.astype(np.int32), device=dev)
    logits = torch.full((s.batch, s.vocab), float("nan"), dtype=torch.float32, device=dev)
    gset.decode_step(2, d_tok.data_ptr(), d_pos.data_ptr(), logits.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    gset.graph(1).status()
    got = logits.cpu().numpy()
    k_rows, v_rows = _rows(pool_k, table, pos, ps), _rows(pool_v, table, pos, ps)
    want = ref.step(tok, pos)     # (all four on the oracle; the first two are compared)
    assert rel_err(got[:2], want[:2]) < TOL
    assert np.isnan(got[2:]).all()
    gset.destroy()


@pytest.mark.parametrize("variant,ps,n_pages,n_req,extra,seed", [
    (dict(batch=8, n_layers=2, head_dim=128, n_q_heads=4, n_kv_heads=2), 8, 8 + 14, 60, {}, 1),
    (dict(batch=3, n_layers=2), 8, 3 + 7, 40, dict(debug_flags=M.binding.DEBUG_JITTER), 3),
    (dict(batch=16, n_layers=1, head_dim=128, n_q_heads=8, n_kv_heads=1), 8, 16 + 30, 80, {}, 6),
    (dict(batch=8, n_layers=2, head_dim=128, n_q_heads=4, n_kv_heads=2), 8, 8 + 14, 40, dict(greedy_loop=2), 7),
])
def test_random_arrivals_and_call_lengths_against_the_oracle(variant, ps, n_pages, n_req, extra, seed):
    """A long randomized run: requests of random prompt and output lengths arrive in bursts of
    random size between calls of random length, pages are scarce, an end-of-sequence token occurs
    now and then.  After every call the whole serving state equals the oracle's; at the end so do
    the outputs of every request."""
    s = G.small_variant("C1", max_seq=64, **variant)
    rng = np.random.default_rng(seed)
    reqs = _requests(rng, s.vocab, n_req, 9, 20)
    table0 = np.full((s.batch, s.max_seq // ps), -1)
    ora = S.ServingOracle(s, G.PagedWeights(s, 4, table0, ps, n_pages), ps, n_pages, 7, "f32")
    gpu = PagedGpu(s, 4, None, ps, n_pages, **{"greedy_loop": 1, "serving": 1, **FUSED, **extra})
    stream = torch.cuda.current_stream().cuda_stream
    srv = gpu.graph.serve(n_req, 16, 32, 7)
    nxt = calls = 0
    while not (nxt == len(reqs) and ora.state.drained()):
        k = int(rng.integers(0, 6))
        for r in reqs[nxt:nxt + k]:
            assert srv.submit(r[0], r[1], stream) == ora.submit(*r)
        nxt = min(len(reqs), nxt + k)
        n = int(rng.integers(1, 30))
        srv.run(n, stream)
        ora.launch(n)
        calls += 1
        torch.cuda.synchronize()
        gpu.graph.status()
        gs = srv.state()
        _same_state(gs, ora.state, calls)
        assert calls < 400
    assert [r for r in range(len(reqs)) if srv.result(r) != ora.outputs(r)] == []
    srv.destroy()
    gpu.close()
