"""mpk_decode_step_static -- the decode step whose scratch memory (activations, partial results,
event and arrival counters) is one static device array of the library instead of buffers allocated
per graph -- against mpk_decode_step, through the C ABI: two calls in a row, the second on a smaller
graph, each compared bit for bit (same kernels, same task order per worker, same summation order)."""
import numpy as np
import pytest
import torch

import paper_2512_22219_amd as M
from synth import gen as G
from synth.device import DeviceModel

pytestmark = pytest.mark.gpu


def _both(shape, seed, opts, steps=2):
    """Logits of `steps` steps through both entry points, on one graph and one model (the K/V row
    a step appends is the same either way, so the second entry point re-appends identical rows)."""
    model = DeviceModel(shape, seed)
    graph = M.compile_graph(shape, model.weight_ptrs(), model.kv_ptrs(), **opts)
    dev = model.device
    tok = torch.as_tensor(G.tokens(seed, shape), device=dev)
    pos = torch.as_tensor(G.kv_lengths(seed, shape), device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    out = []
    for step in range(steps):
        a = torch.full((shape.batch, shape.vocab), float("nan"), dtype=torch.float32, device=dev)
        b = torch.full_like(a, float("nan"))
        graph.decode_step(tok.data_ptr(), pos.data_ptr(), a.data_ptr(), stream)
        graph.decode_step_static(tok.data_ptr(), pos.data_ptr(), b.data_ptr(), stream)
        torch.cuda.synchronize()
        graph.status()
        out.append((a.cpu().numpy(), b.cpu().numpy()))
        tok = a.argmax(-1).to(torch.int32)
        pos = pos + 1
    need = graph.static_scratch_need()
    graph.destroy()
    return out, need


@pytest.mark.parametrize("opts", [dict(fusion=31, transitive_reduction=1),
                                  dict(fusion=31, transitive_reduction=1, launch_mode=1)])
def test_static_scratch_step_equals_the_allocating_step_twice_in_a_row(opts):
    big = G.small_variant("C1", batch=8, n_layers=3, max_seq=192)       # matrix-core bodies, split-KV merge counters
    small = G.CONFIGS["C1"]                                             # batch 1, fewer events, a smaller arena
    first, need_big = _both(big, 5, opts)
    second, need_small = _both(small, 6, opts)
    assert 0 < need_small < need_big <= 32 << 20
    for got in (first, second):
        for a, b in got:
            assert np.isfinite(a).all() and np.isfinite(b).all()
            assert np.array_equal(a, b)


def test_static_scratch_step_refuses_what_does_not_fit_or_cannot_share():
    s = G.small_variant("C1", batch=2)
    model = DeviceModel(s, 0)
    tok = torch.as_tensor(G.tokens(0, s), device=model.device)
    pos = torch.as_tensor(G.kv_lengths(0, s), device=model.device)
    lg = torch.empty((s.batch, s.vocab), dtype=torch.float32, device=model.device)
    for opts in (dict(fusion=7, n_sched_wgs=2), dict(fusion=31, greedy_loop=1), dict(fusion=31, debug_flags=1)):
        g = M.compile_graph(s, model.weight_ptrs(), model.kv_ptrs(), **opts)
        with pytest.raises(M.binding.MpkError) as e:
            g.decode_step_static(tok.data_ptr(), pos.data_ptr(), lg.data_ptr(), 0)
        assert e.value.status == M.binding.MPK_ERR_UNSUPPORTED
        g.destroy()
    deep = G.small_variant("C1", batch=16, n_layers=260, max_seq=192)   # 35 MiB of activations: more than the array holds
    model = DeviceModel(deep, 0)
    g = M.compile_graph(deep, model.weight_ptrs(), model.kv_ptrs(), fusion=31, transitive_reduction=1)
    assert g.static_scratch_need() > 32 << 20
    tok = torch.as_tensor(G.tokens(0, deep), device=model.device)
    pos = torch.as_tensor(G.kv_lengths(0, deep), device=model.device)
    lg = torch.empty((deep.batch, deep.vocab), dtype=torch.float32, device=model.device)
    with pytest.raises(M.binding.MpkError) as e:
        g.decode_step_static(tok.data_ptr(), pos.data_ptr(), lg.data_ptr(), 0)
    assert e.value.status == M.binding.MPK_ERR_UNSUPPORTED and "more scratch" in str(e.value)
    g.decode_step(tok.data_ptr(), pos.data_ptr(), lg.data_ptr(), 0)     # the allocating entry point still runs it
    torch.cuda.synchronize()
    g.status()
    assert torch.isfinite(lg).all()
    g.destroy()
