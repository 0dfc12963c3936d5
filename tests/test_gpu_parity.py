"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

import paper_2512_22219_amd as M
from oracle import decoder as D
from synth import gen as G
from synth.device import DeviceModel
from tests.gpu_util import GpuDecoder, held_step, rel_err

pytestmark = pytest.mark.gpu
TOL = 2e-2   # the target's bound on logits (bf16 weights, fp32 accumulation)


def strict_steps(s, seed, opts, tok, pos, n_steps):
    """n_steps greedy steps, every one compared element by element with the fp64 build of the
    oracle while both sides hold the same discrete decisions (the GPU's appended bf16 K/V rows and
    expert sets, each checked to be a valid one: tests/gpu_util.held_step).  With the decisions
    held, what is left is rounding order: the bound of the target on every element at every step,
    and 2e-5 of the largest logit (activations are fp32 end to end)."""
    ref = D.DecoderOracle(s, G.SynthWeights(s, seed), "f64")
    gpu = GpuDecoder(s, seed, **opts)
    flips = 0
    for step in range(n_steps):
        got, want, f, _ = held_step(ref, gpu, tok, pos)
        flips += f
        assert np.isfinite(got).all(), step
        assert rel_err(got, want) < TOL, step
        assert np.abs(got - want).max() / np.abs(want).max() < 2e-5, step
        assert got.argmax(-1).tolist() == want.argmax(-1).tolist(), step
        tok, pos = want.argmax(-1).astype(np.int32), pos + 1
    gpu.close()
    return flips


def test_device_generator_matches_host_bit_exact():
    from synth.device import DeviceModel
    s = G.CONFIGS["C1"]
    m = DeviceModel(s, seed=3)
    host = G.SynthWeights(s, 3)
    w0 = host.layer(1)
    assert np.array_equal(m.layers[1]["wqkv"].view(torch.int16).cpu().numpy().view(np.uint16), w0[G.L_WQKV])
    assert np.array_equal(m.layers[1]["attn_norm"].view(torch.int16).cpu().numpy().view(np.uint16), w0[G.L_ATTN_NORM])
    assert np.array_equal(m.lm_head.view(torch.int16).cpu().numpy().view(np.uint16), host.lm_head())
    k, v = host.kv_layer(0)
    assert np.array_equal(m.k[0].view(torch.int16).cpu().numpy().view(np.uint16), k)
    assert np.array_equal(m.v[0].view(torch.int16).cpu().numpy().view(np.uint16), v)


MODES = [
    dict(fusion=0),
    dict(fusion=0, launch_mode=1),
    dict(fusion=7),
    dict(fusion=7, transitive_reduction=1),
    dict(fusion=7, transitive_reduction=1, launch_mode=1),
    dict(fusion=3, transitive_reduction=1, n_workers=37, attn_chunks=5, tiles_pointwise=3),
    dict(fusion=31, transitive_reduction=1),
    dict(fusion=31, transitive_reduction=1, launch_mode=1),
    dict(fusion=16 + 7),
    dict(fusion=8 + 7, attn_chunks=1),
    dict(fusion=31, transitive_reduction=1, n_workers=37, attn_chunks=5),
    # hybrid launch: scheduler wavefronts hand the attention tasks out just-in-time
    dict(fusion=0, n_sched_wgs=1, n_workers=16),
    dict(fusion=7, transitive_reduction=1, n_sched_wgs=2),
    dict(fusion=31, transitive_reduction=1, n_sched_wgs=2, attn_chunks=5),
    dict(fusion=31, transitive_reduction=1, n_sched_wgs=1, n_workers=37, attn_chunks=3),
]


@pytest.mark.parametrize("opts", MODES)
def test_c1_one_step_matches_oracle(opts):
    s = G.CONFIGS["C1"]
    tok, pos = G.tokens(0, s), G.kv_lengths(0, s)
    ref = D.DecoderOracle(s, G.SynthWeights(s, 0), "f32")
    want = ref.step(tok, pos)
    gpu = GpuDecoder(s, 0, **opts)
    got = gpu.step(tok, pos)
    assert np.isfinite(got).all()
    assert rel_err(got, want) < TOL
    assert np.abs(got - want).max() / np.abs(want).max() < 1e-4     # fp32 activations end to end
    assert got.argmax(-1).tolist() == want.argmax(-1).tolist()
    # the appended K/V rows: bf16 patterns equal to the oracle's (value within one bf16 ulp where
    # the fp32 value before rounding differed in its last bits)
    p = int(pos[0])
    for l in range(s.n_layers):
        for dev_c, host_c in ((gpu.model.k, ref.kv[l][0]), (gpu.model.v, ref.kv[l][1])):
            g_rows = dev_c[l, :, :, p].view(torch.int16).cpu().numpy().view(np.uint16)
            h_rows = host_c[:, :, p]
            diff = np.abs(g_rows.astype(np.int32) - h_rows.astype(np.int32))
            assert diff.max() <= 1 and (diff != 0).mean() < 0.02
            # nothing else in the cache changed
            before = G.host_kv_layer(0, s, l)[0 if dev_c is gpu.model.k else 1]
            g_all = dev_c[l].view(torch.int16).cpu().numpy().view(np.uint16)
            mask = np.ones(s.max_seq, bool)
            mask[p] = False
            assert np.array_equal(g_all[:, :, mask], before[:, :, mask])
    gpu.close()


@pytest.mark.parametrize("opts", [dict(fusion=0), dict(fusion=7, transitive_reduction=1),
                                  dict(fusion=31, transitive_reduction=1),
                                  dict(fusion=31, transitive_reduction=1, n_sched_wgs=2)])
def test_small_batch_and_ragged_positions(opts):
    """Batch 3 with different KV lengths (one of them tiny), ragged tiles (n_workers = 37)."""
    s = G.small_variant("C1", batch=3, n_layers=2)
    tok = G.tokens(1, s)
    pos = np.array([0, 77, 150], np.int32)
    ref = D.DecoderOracle(s, G.SynthWeights(s, 1), "f32")
    want = ref.step(tok, pos)
    gpu = GpuDecoder(s, 1, n_workers=37, **opts)
    if opts.get("n_sched_wgs"):
        assert gpu.graph.stats()["n_jit_tasks"] > 0
    got = gpu.step(tok, pos)
    assert rel_err(got, want) < TOL
    assert np.abs(got - want).max() / np.abs(want).max() < 1e-4
    gpu.close()


@pytest.mark.parametrize("batch,pos,opts", [
    # one long sequence takes most of the chunk tasks, two sequences of length 1 keep one each
    (4, [0, 180, 0, 7], dict(attn_chunks=4)),
    (4, [0, 180, 0, 7], dict(attn_chunks=4, no_attn_balance=1)),
    # 16 sequences, lengths 1 .. 189, three chunks each: the deal runs its left-over loop
    (16, [(37 * i) % 189 for i in range(16)], dict(attn_chunks=3)),
    (8, [188, 3, 188, 3, 188, 3, 188, 3], dict(attn_chunks=2, n_sched_wgs=2)),
    (5, [11, 150, 60, 0, 99], dict(attn_chunks=5, launch_mode=1)),
])
def test_attention_chunk_tasks_dealt_to_the_sequences_by_length(batch, pos, opts):
    """Merge fused, several sequences of very different lengths: which sequence a chunk task
    works on is decided when the step runs; three steps, so that the deal changes under way."""
    s = G.small_variant("C1", batch=batch, n_layers=2)
    gpu = GpuDecoder(s, 5, fusion=31, transitive_reduction=1, n_workers=29, **opts)
    ref = D.DecoderOracle(s, G.SynthWeights(s, 5), "f64")
    tok = G.tokens(5, s)
    p = np.array(pos, np.int32)
    for _ in range(3):
        got, want, _, _ = held_step(ref, gpu, tok, p)
        assert rel_err(got, want) < TOL
        assert np.array_equal(got.argmax(-1), want.argmax(-1))
        tok = want.argmax(-1).astype(np.int32)
        p = p + 1
    gpu.close()


@pytest.mark.parametrize("variant,opts", [
    # ffn 4360: the down projection's input is one full 4096-element segment plus a short one
    (dict(hidden=1000, ffn=4360, batch=1), dict(fusion=31, transitive_reduction=1, n_workers=13)),
    (dict(hidden=1000, ffn=4360, batch=3), dict(fusion=31, transitive_reduction=1, n_workers=13)),
    # hidden 8200: every projection from the residual stream walks three segments, the last 8 long
    (dict(hidden=8200, ffn=696, batch=2, vocab=520), dict(fusion=31, transitive_reduction=1, n_workers=29)),
    (dict(hidden=4104, ffn=696, batch=4, vocab=520), dict(fusion=0, n_workers=29, launch_mode=1)),
    # one weight row per wavefront and fewer rows than wavefronts (vocab 40 over 7 workers)
    (dict(hidden=264, ffn=72, batch=1, vocab=40), dict(fusion=31, transitive_reduction=1, n_workers=7)),
])
def test_linear_stream_odd_shapes(variant, opts):
    """The two-buffer weight stream of the batch <= 4 linear body on shapes that exercise its
    corners: odd numbers of rows per wavefront (a pair with one row), inputs of several segments
    with a short last one, tasks with fewer rows than wavefronts, more half blocks than buffers."""
    s = G.small_variant("C1", n_layers=2, **variant)
    rng = np.random.default_rng(11)
    tok = rng.integers(0, s.vocab, s.batch).astype(np.int32)
    pos = rng.integers(5, 150, s.batch).astype(np.int32)
    strict_steps(s, 2, opts, tok, pos, 2)


@pytest.mark.parametrize("shape,pos,opts", [
    # 4 query heads per KV head, batch 8: lengths 1 and 2 leave chunks empty, chunks that hold
    # only the row appended this step, and chunks with a single row of an earlier step
    (dict(batch=8, n_q_heads=8, n_kv_heads=2), [0, 1, 2, 3, 40, 95, 150, 0], dict(attn_chunks=4)),
    (dict(batch=8, n_q_heads=8, n_kv_heads=2), [0, 1, 2, 3, 40, 95, 150, 0], dict(attn_chunks=4, no_attn_balance=1)),
    (dict(batch=8, n_q_heads=8, n_kv_heads=2), [150, 149, 33, 32, 31, 64, 65, 97], dict(attn_chunks=1)),
    (dict(batch=16, n_q_heads=4, n_kv_heads=1), [(37 * i) % 150 for i in range(16)], dict(attn_chunks=3)),
    (dict(batch=5, n_q_heads=4, n_kv_heads=1), [0, 150, 0, 7, 99], dict(attn_chunks=2, launch_mode=1)),
    # 8 query heads per KV head, mixture of experts, batch 16
    (dict(batch=16, n_q_heads=8, n_kv_heads=1, ffn=0, n_experts=16, top_k=4, expert_ffn=96),
     [(53 * i) % 150 for i in range(16)], dict(attn_chunks=2)),
    (dict(batch=8, n_q_heads=8, n_kv_heads=1, ffn=0, n_experts=16, top_k=4, expert_ffn=96),
     [0, 1, 2, 3, 150, 95, 31, 32], dict(attn_chunks=4)),
])
def test_kernels_specialised_for_batch_5_to_16_on_short_and_ragged_chunks(shape, pos, opts):
    """Head dimension 128 with 4 (dense) or 8 (mixture of experts) query heads per KV head selects
    the kernels compiled for those shapes, whose attention body requests cache rows a fixed number
    of rounds ahead with no branch around a request: chunks shorter than that, empty chunks,
    chunks that are nothing but the appended row, and the deal changing from step to step."""
    s = G.small_variant("C1", n_layers=2, hidden=512, head_dim=128, max_seq=192, **shape)
    ref = D.DecoderOracle(s, G.SynthWeights(s, 4), "f64")
    gpu = GpuDecoder(s, 4, fusion=31, transitive_reduction=1, **opts)
    tok = G.tokens(4, s)
    p = np.array(pos, np.int32)
    for step in range(3):
        # (the oracle holds the GPU's appended bf16 rows and expert sets, each checked to be a
        # valid outcome: at positions 0..3 one rounding decision is most of the attention output)
        got, want, _, _ = held_step(ref, gpu, tok, p)
        assert np.isfinite(got).all()
        assert rel_err(got, want) < TOL, step
        assert np.array_equal(got.argmax(-1), want.argmax(-1))
        tok = want.argmax(-1).astype(np.int32)
        p = p + 1
    gpu.close()


@pytest.mark.parametrize("batch,opts", [
    (8, dict(fusion=31, transitive_reduction=1)),
    (8, dict(fusion=0)),
    (8, dict(fusion=31, transitive_reduction=1, launch_mode=1)),
    (8, dict(fusion=7, transitive_reduction=1, n_workers=37)),
    (8, dict(fusion=31, transitive_reduction=1, n_sched_wgs=2)),
    (5, dict(fusion=31, transitive_reduction=1)),
    (16, dict(fusion=31, transitive_reduction=1, tiles_lm_head=64)),
])
def test_matrix_core_linear_body_batch_5_to_16(batch, opts):
    """Batch 5..16 runs the linear operators on the matrix cores (activations split into three
    bf16 planes): ragged KV lengths, K that is not a multiple of 32 (ffn 688), K-sliced and
    row-tiled tasks (LM head), several steps so that appended rows are read back."""
    s = G.small_variant("C1", batch=batch, n_layers=2, max_seq=192)
    tok = G.tokens(2, s)
    pos = np.array([(37 * b + 5) % 150 for b in range(batch)], np.int32)
    strict_steps(s, 2, opts, tok, pos, 3)


@pytest.mark.parametrize("variant,opts", [
    (dict(hidden=2056, ffn=3000, batch=5), dict(fusion=31, transitive_reduction=1, n_workers=24)),
    (dict(hidden=4096, ffn=2304, batch=8, vocab=520), dict(fusion=31, transitive_reduction=1, n_workers=32)),
    (dict(hidden=2056, ffn=3000, batch=7, vocab=520), dict(fusion=0, n_workers=16, launch_mode=1)),
    # batch 9..16: tiles of 512 inputs; 1032 is two tiles and 8 inputs, 2048 four tiles
    (dict(hidden=2048, ffn=1032, batch=12), dict(fusion=31, transitive_reduction=1, n_workers=24)),
    # inputs of at most two tiles are staged whole: 1000 at batch 16, 2040 at batch 6
    (dict(hidden=1000, ffn=520, batch=16, vocab=520), dict(fusion=31, transitive_reduction=1, n_workers=24)),
    (dict(hidden=2040, ffn=1016, batch=6, vocab=520), dict(fusion=31, transitive_reduction=1, n_workers=24)),
    # one or two 16-row weight tiles per task: the K slices of several input tiles share a round
    # of weight requests (hidden 4096 over 128 workers: O projection 32 rows, QKV 8 and 16)
    (dict(hidden=4096, ffn=2048, batch=8, vocab=2048), dict(fusion=31, transitive_reduction=1, n_workers=128)),
    (dict(hidden=2560, ffn=1536, batch=16, vocab=1024), dict(fusion=31, transitive_reduction=1, n_workers=160)),
])
def test_matrix_core_body_inputs_of_one_to_two_staging_tiles(variant, opts):
    """Batch 5..16 with inputs from under one to several staging tiles long (tiles of 1024 inputs
    up to batch 8, 512 above; at most two tiles are staged whole), the last pass ragged or full,
    tasks of one, two and more 16-row weight tiles.  Two steps each."""
    s = G.small_variant("C1", n_layers=2, max_seq=192, **variant)
    rng = np.random.default_rng(13)
    tok = rng.integers(0, s.vocab, s.batch).astype(np.int32)
    pos = rng.integers(5, 150, s.batch).astype(np.int32)
    strict_steps(s, 4, opts, tok, pos, 2)


@pytest.mark.parametrize("batch,ffn,opts", [
    (8, 8192, dict(fusion=31, transitive_reduction=1, n_workers=32)),            # 4 parts of 2048
    (8, 6272, dict(fusion=31, transitive_reduction=1, n_workers=32)),            # 2 parts of 3136: ragged second tile
    (16, 4096, dict(fusion=31, transitive_reduction=1, n_workers=64)),           # 1024-input tiles, 4 parts
    (8, 8192, dict(fusion=31, transitive_reduction=1, n_workers=32, launch_mode=1)),
    (8, 8192, dict(fusion=31, n_workers=32, n_sched_wgs=2)),
])
def test_down_projection_decomposed_along_its_input(batch, ffn, opts):
    """Batch > 4 with a long down-projection input: (row block, input part) tasks write partial
    sums and the last task of a row block to arrive adds them and the residual.  The compiled
    graph must really contain such tasks, and logits must match over steps (the arrival counters
    only ever grow)."""
    s = G.small_variant("C1", batch=batch, ffn=ffn, n_layers=2, max_seq=192)
    tok = G.tokens(3, s)
    pos = np.array([(29 * b + 11) % 150 for b in range(batch)], np.int32)
    ref = D.DecoderOracle(s, G.SynthWeights(s, 3), "f32")
    gpu = GpuDecoder(s, 3, **opts)
    ex = gpu.graph.export()
    down = [o for o in ex.ops if o["layer"] == 0 and o["kind"] == M.binding.OP_LINEAR][-1]
    assert down["cols"] >= 2 * s.hidden, "the down projection of this graph is not decomposed"
    for step in range(3):
        want = ref.step(tok, pos)
        got = gpu.step(tok, pos)
        assert np.isfinite(got).all()
        assert rel_err(got, want) < TOL, step
        assert np.abs(got - want).max() / np.abs(want).max() < 1e-4, step
        assert got.argmax(-1).tolist() == want.argmax(-1).tolist(), step
        tok, pos = want.argmax(-1).astype(np.int32), pos + 1
    gpu.close()


def test_captured_per_operator_launches_replay_correctly_and_persistent_capture_is_refused():
    """Kernel-per-operator launches of a graph with (row block, input part) tasks, captured once
    into a HIP graph: every replay must give what an eager launch gives (the arrival counters of
    the row blocks must not depend on the step number, which a replay carries frozen).  Replays
    alternate with eager work and synchronisations.  Capturing a persistent-kernel launch is an
    error: its events are compared with the step number."""
    s = G.small_variant("C1", batch=8, ffn=8192, n_layers=2, max_seq=192)
    tok = G.tokens(3, s)
    pos = np.array([(29 * b + 11) % 150 for b in range(8)], np.int32)
    ref = D.DecoderOracle(s, G.SynthWeights(s, 3), "f32")
    gpu = GpuDecoder(s, 3, fusion=31, transitive_reduction=1, n_workers=32, launch_mode=1)
    side = torch.cuda.Stream()
    gpu.tok.copy_(torch.as_tensor(tok)); gpu.pos.copy_(torch.as_tensor(pos))
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            gpu.graph.decode_step(gpu.tok.data_ptr(), gpu.pos.data_ptr(), gpu.logits.data_ptr(), side.cuda_stream)
    for step in range(4):
        want = ref.step(tok, pos)
        gpu.tok.copy_(torch.as_tensor(tok)); gpu.pos.copy_(torch.as_tensor(pos))
        gpu.logits.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        gpu.graph.status()
        got = gpu.logits.cpu().numpy()
        assert np.isfinite(got).all(), step
        assert rel_err(got, want) < TOL, step
        assert got.argmax(-1).tolist() == want.argmax(-1).tolist(), step
        tok, pos = want.argmax(-1).astype(np.int32), pos + 1
    gpu.close()
    mega = GpuDecoder(s, 3, fusion=31, transitive_reduction=1, n_workers=32)
    g2 = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g2, stream=side):
            with pytest.raises(M.MpkError, match="captured"):
                mega.graph.decode_step(mega.tok.data_ptr(), mega.pos.data_ptr(), mega.logits.data_ptr(), side.cuda_stream)
    want = D.DecoderOracle(s, G.SynthWeights(s, 3), "f32").step(G.tokens(3, s), np.array([(29 * b + 11) % 150 for b in range(8)], np.int32))
    got = mega.step(G.tokens(3, s), np.array([(29 * b + 11) % 150 for b in range(8)], np.int32))
    assert rel_err(got, want) < TOL   # the graph is still usable after the refused launch
    mega.close()


def test_greedy_32_steps_free_running_and_teacher_forced():
    s = G.small_variant("C1", max_seq=192)
    tok, pos = G.tokens(0, s), G.kv_lengths(0, s)
    ref = D.DecoderOracle(s, G.SynthWeights(s, 0), "f32")
    want_t, want_l = ref.greedy(tok, pos, 32)
    for opts in (dict(fusion=0), dict(fusion=7, transitive_reduction=1),
                 dict(fusion=31, transitive_reduction=1),
                 dict(fusion=31, transitive_reduction=1, n_sched_wgs=2)):
        gpu = GpuDecoder(s, 0, **opts)
        t, p, toks = np.array(tok), np.array(pos), []
        for i in range(32):
            lg = gpu.step(t, p)
            assert rel_err(lg, want_l[i]) < TOL, i
            t = lg.argmax(-1).astype(np.int32)
            p = p + 1
            toks.append(t.copy())
        assert np.array_equal(np.stack(toks), want_t)
        gpu.model.reset_kv()
        gpu.graph.reset()
        t, p = np.array(tok), np.array(pos)
        for i in range(32):              # teacher forced: fed the oracle's tokens
            lg = gpu.step(t, p)
            assert lg.argmax(-1).tolist() == want_t[i].tolist(), i
            t, p = want_t[i].astype(np.int32), p + 1
        gpu.close()


def test_full_width_two_layers_of_the_8b_shape():
    """Two layers of the Qwen3-8B-shaped config at full width and vocabulary: every tile shape
    the benchmark launches (24/16/96-row tiles, the ragged 593/594-row LM-head tiles)."""
    s = G.small_variant("C2", n_layers=2)
    tok, pos = G.tokens(0, s), G.kv_lengths(0, s)
    ref = D.DecoderOracle(s, G.SynthWeights(s, 0), "f32")
    want = ref.step(tok, pos)
    from synth.device import DeviceModel
    model = DeviceModel(s, 0)
    for opts in (dict(fusion=0), dict(fusion=7, transitive_reduction=1),
                 dict(fusion=7, transitive_reduction=1, launch_mode=1),
                 dict(fusion=31, transitive_reduction=1),
                 dict(fusion=31, transitive_reduction=1, launch_mode=1)):
        model.reset_kv()
        gpu = GpuDecoder(s, 0, model=model, **opts)
        got = gpu.step(tok, pos)
        assert rel_err(got, want) < TOL
        assert np.abs(got - want).max() / np.abs(want).max() < 1e-4
        assert got.argmax(-1).tolist() == want.argmax(-1).tolist()
        gpu.close()


def test_device_errors_are_reported_not_fatal():
    s = G.CONFIGS["C1"]
    gpu = GpuDecoder(s, 0, fusion=0)
    tok = G.tokens(0, s)
    with pytest.raises(M.MpkError) as e:
        gpu.step(tok, np.array([s.max_seq], np.int32))
    assert e.value.status == M.binding.MPK_ERR_DEVICE
    gpu.graph.reset()
    with pytest.raises(M.MpkError) as e:
        gpu.step(np.array([s.vocab + 5], np.int32), G.kv_lengths(0, s))
    assert e.value.status == M.binding.MPK_ERR_DEVICE
    gpu.graph.reset()
    gpu.model.reset_kv()
    want = D.DecoderOracle(s, G.SynthWeights(s, 0), "f32").step(tok, G.kv_lengths(0, s))
    assert rel_err(gpu.step(tok, G.kv_lengths(0, s)), want) < TOL
    gpu.close()


# ------------------------------------------------------------------ mixture of experts
def _check_routing(gpu, ref, s):
    """Selected expert sets and combine weights of the last step, layer by layer.  Where the
    oracle's top_k-th and next router outputs are closer than 1e-5 either set is accepted (top-k
    is discontinuous); returns the number of such decisions."""
    ex, wt = gpu.graph.moe_selection()
    ex = ex.reshape(s.n_layers, s.batch, s.top_k).astype(np.int64)
    ambiguous = 0
    for l in range(s.n_layers):
        for b in range(s.batch):
            want = ref.last_moe_sel[l, b].tolist()
            got = ex[l, b].tolist()
            assert got == sorted(got) and len(set(got)) == s.top_k
            if got != want:
                r = np.sort(ref.last_moe_logits[l, b].astype(np.float64))[::-1]
                assert r[s.top_k - 1] - r[s.top_k] < 1e-5, (l, b, got, want)
                ambiguous += 1
    wt = wt.reshape(s.n_layers, s.batch, s.top_k)
    assert np.allclose(wt.sum(-1), 1.0, atol=1e-5)
    return ambiguous


MOE_CASES = [
    (dict(batch=1, n_experts=8, top_k=2, expert_ffn=64), dict(fusion=0)),
    (dict(batch=2, n_experts=8, top_k=2, expert_ffn=64), dict(fusion=0, launch_mode=1)),
    (dict(batch=3, n_experts=16, top_k=4, expert_ffn=96), dict(fusion=31, transitive_reduction=1)),
    (dict(batch=16, n_experts=32, top_k=8, expert_ffn=160), dict(fusion=31, transitive_reduction=1)),
    (dict(batch=16, n_experts=128, top_k=8, expert_ffn=768, hidden=512, n_q_heads=8, n_kv_heads=1,
          head_dim=64), dict(fusion=31, transitive_reduction=1)),
    (dict(batch=5, n_experts=12, top_k=3, expert_ffn=40), dict(fusion=7, n_workers=37, tiles_moe=9)),
    (dict(batch=16, n_experts=32, top_k=8, expert_ffn=160),
     dict(fusion=31, transitive_reduction=1, launch_mode=1)),
    (dict(batch=4, n_experts=16, top_k=4, expert_ffn=96),
     dict(fusion=31, transitive_reduction=1, n_sched_wgs=2)),
]


@pytest.mark.parametrize("variant,opts", MOE_CASES)
def test_moe_three_steps_match_oracle(variant, opts):
    """Router, top-k routing, expert stages sized at run time from the meta-tensor, combine
    (Section 6.4), on small mixture-of-experts models: logits and routing decisions of three
    teacher-forced steps with ragged positions."""
    s = G.small_variant("C1", ffn=0, **variant)
    rng = np.random.default_rng(7)
    pos = rng.integers(60, 128, s.batch)
    tok = rng.integers(0, s.vocab, s.batch)
    ref = D.DecoderOracle(s, G.SynthWeights(s, 1), "f32")
    gpu = GpuDecoder(s, 1, **opts)
    for step in range(3):
        want = ref.step(tok, pos)
        got = gpu.step(tok, pos)
        assert np.isfinite(got).all()
        ambiguous = _check_routing(gpu, ref, s)
        if ambiguous == 0:
            assert rel_err(got, want) < TOL, step
            assert np.abs(got - want).max() / np.abs(want).max() < 1e-4
        active = gpu.graph.moe_active()
        sel = ref.last_moe_sel
        assert ambiguous or active.tolist() == [len(np.unique(sel[l])) for l in range(s.n_layers)]
        tok = want.argmax(-1)
        pos = pos + 1
    gpu.close()


@pytest.mark.parametrize("batch", [1, 8])
def test_moe_routing_ties_take_the_lower_expert_index(batch):
    """Exact ties among router outputs (duplicated router rows): both sides must keep the lower
    expert indices, in the GEMV path (batch 1) and the matrix-core path (batch 8)."""
    from synth.device import DeviceModel
    s = G.small_variant("C1", ffn=0, batch=batch, n_experts=8, top_k=2, expert_ffn=64)
    prov = G.SynthWeights(s, 5)
    model = DeviceModel(s, 5)
    for l in range(s.n_layers):
        host_r = prov.layer(l)[G.L_ROUTER]
        dev_r = model.layers[l]["router"]
        if l == 0:      # every expert ties with every other
            host_r[1:] = host_r[0]
            dev_r[1:] = dev_r[0:1].clone()
        else:           # two groups of four identical rows
            host_r[1:4] = host_r[0]
            host_r[5:8] = host_r[4]
            dev_r[1:4] = dev_r[0:1].clone()
            dev_r[5:8] = dev_r[4:5].clone()
    torch.cuda.synchronize()
    ref = D.DecoderOracle(s, prov, "f32")
    gpu = GpuDecoder(s, 5, model=model, fusion=31, transitive_reduction=1)
    rng = np.random.default_rng(3)
    tok, pos = rng.integers(0, s.vocab, batch), rng.integers(10, 120, batch)
    want = ref.step(tok, pos)
    got = gpu.step(tok, pos)
    ex, wt = gpu.graph.moe_selection()
    ex = ex.reshape(s.n_layers, batch, s.top_k)
    wt = wt.reshape(s.n_layers, batch, s.top_k)
    assert np.array_equal(ex[0], np.tile([0, 1], (batch, 1)))
    assert np.allclose(wt[0], 0.5, atol=1e-6)
    assert np.array_equal(ex, ref.last_moe_sel)
    assert set(map(tuple, ex[1].tolist())) <= {(0, 1), (4, 5)}
    assert rel_err(got, want) < TOL
    gpu.close()


# ------------------------------------------------------------------ several tokens per launch
@pytest.mark.parametrize("variant,opts,n_steps", [
    (dict(), dict(fusion=31, transitive_reduction=1), 32),
    (dict(), dict(fusion=0), 8),
    (dict(batch=3, n_layers=2), dict(fusion=31, transitive_reduction=1, n_workers=37), 12),
    (dict(batch=8, n_layers=2), dict(fusion=31, transitive_reduction=1), 6),
    (dict(batch=2), dict(fusion=31, transitive_reduction=1, launch_mode=1), 5),
    (dict(batch=4, ffn=0, n_experts=16, top_k=4, expert_ffn=96), dict(fusion=31, transitive_reduction=1), 6),
    # several sampling tasks per sequence: each scans a share of the logits, the last to arrive picks
    (dict(batch=3, n_layers=2), dict(fusion=31, transitive_reduction=1, tiles_sampling=5), 8),
    (dict(batch=2), dict(fusion=31, transitive_reduction=1, launch_mode=1, tiles_sampling=32), 5),
    (dict(), dict(fusion=0, tiles_sampling=3, debug_flags=6), 6),
    # batch <= 4 issues a launch per step by default; greedy_loop = 2: the one launch of the loop kernel
    (dict(), dict(fusion=31, transitive_reduction=1, greedy_loop=2), 16),
    (dict(batch=3, n_layers=2), dict(fusion=31, transitive_reduction=1, greedy_loop=2, tiles_sampling=2), 7),
    # the kernels compiled for head dimension 128 at batch 5..16: a launch per step, and the loop kernel
    (dict(batch=8, n_layers=2, head_dim=128, n_q_heads=8, n_kv_heads=2), dict(fusion=31, transitive_reduction=1), 6),
    (dict(batch=8, n_layers=2, head_dim=128, n_q_heads=8, n_kv_heads=2), dict(fusion=31, transitive_reduction=1, greedy_loop=2), 6),
    (dict(batch=16, head_dim=128, n_q_heads=8, n_kv_heads=1, ffn=0, n_experts=16, top_k=4, expert_ffn=96), dict(fusion=31, transitive_reduction=1), 5),
])
def test_greedy_loop_decodes_several_tokens_in_one_launch(variant, opts, n_steps):
    """Graph with the sampling operator: n_steps tokens from ONE launch of the persistent kernel
    (the epoch advances inside the kernel) must be the oracle's greedy tokens, with every step's
    logits within tolerance; tokens and positions come back advanced; a second launch continues."""
    s = G.small_variant("C1", max_seq=192, **variant)
    rng = np.random.default_rng(11)
    tok0 = rng.integers(0, s.vocab, s.batch)
    pos0 = rng.integers(20, 100, s.batch)
    ref = D.DecoderOracle(s, G.SynthWeights(s, 4), "f32")
    want_t, want_l = ref.greedy(tok0, pos0, 2 * n_steps)
    gpu = GpuDecoder(s, 4, **{"greedy_loop": 1, **opts})
    dev = gpu.model.device
    tok = torch.as_tensor(tok0.astype(np.int32), device=dev)
    pos = torch.as_tensor(pos0.astype(np.int32), device=dev)
    toks = torch.full((n_steps, s.batch), -1, dtype=torch.int32, device=dev)
    all_l = torch.full((n_steps, s.batch, s.vocab), float("nan"), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    for launch in range(2):
        gpu.graph.decode_steps(n_steps, tok.data_ptr(), pos.data_ptr(), toks.data_ptr(),
                               gpu.logits.data_ptr(), all_l.data_ptr(), stream)
        torch.cuda.synchronize()
        gpu.graph.status()
        lo = launch * n_steps
        got_l = all_l.cpu().numpy()
        for i in range(n_steps):
            if lo + i == 0:
                assert rel_err(got_l[i], want_l[0]) < TOL
            # later steps read K/V rows each side appended itself (a bf16 rounding boundary may
            # fall either way): bound relative to the largest logit
            assert np.abs(got_l[i] - want_l[lo + i]).max() / np.abs(want_l[lo + i]).max() < 2e-3, (launch, i)
        assert np.array_equal(toks.cpu().numpy(), want_t[lo:lo + n_steps])
        assert np.array_equal(tok.cpu().numpy(), want_t[lo + n_steps - 1])
        assert np.array_equal(pos.cpu().numpy(), pos0 + lo + n_steps)
        assert np.array_equal(gpu.logits.cpu().numpy(), got_l[-1])
    # the single-step entry point refuses such a graph (it would not advance tokens itself)
    with pytest.raises(M.MpkError):
        gpu.graph.decode_step(tok.data_ptr(), pos.data_ptr(), gpu.logits.data_ptr(), stream)
    gpu.close()


@pytest.mark.parametrize("variant,opts", [
    (dict(), dict(fusion=0)),                                                     # rope operator
    (dict(), dict(fusion=31, transitive_reduction=1)),                            # fused, register-resident body
    (dict(batch=3), dict(fusion=31, transitive_reduction=1, launch_mode=1)),
    (dict(n_q_heads=8, n_kv_heads=1, batch=2), dict(fusion=31, transitive_reduction=1)),   # 8 heads per KV head: online body
    (dict(head_dim=128, n_q_heads=4, n_kv_heads=2, batch=8), dict(fusion=31, transitive_reduction=1)),
    (dict(head_dim=128, n_q_heads=2, n_kv_heads=1), dict(fusion=7)),
    (dict(ffn=0, n_experts=8, top_k=2, expert_ffn=64, batch=4), dict(fusion=31, transitive_reduction=1)),   # Qwen3-MoE-like
])
def test_qk_norm_models_match_oracle(variant, opts):
    """Per-head RMSNorm of q and k before RoPE (MPK_MODEL_QK_NORM): rope operator, both fused
    attention bodies, head_dim 64 and 128, three steps so that normalised keys are read back."""
    s = G.small_variant("C1", qk_norm=True, max_seq=192, **variant)
    rng = np.random.default_rng(5)
    tok, pos = rng.integers(0, s.vocab, s.batch), rng.integers(30, 120, s.batch)
    ref = D.DecoderOracle(s, G.SynthWeights(s, 6), "f32")
    gpu = GpuDecoder(s, 6, **opts)
    for step in range(3):
        want = ref.step(tok, pos)
        got = gpu.step(tok, pos)
        assert np.isfinite(got).all()
        assert rel_err(got, want) < TOL, step
        assert np.abs(got - want).max() / np.abs(want).max() < 1e-4, step
        assert got.argmax(-1).tolist() == want.argmax(-1).tolist(), step
        tok, pos = want.argmax(-1), pos + 1
    # the same weights without the flag give different logits: the norm is really applied
    plain = GpuDecoder(G.small_variant("C1", max_seq=192, **variant), 6, model=gpu.model, **opts)
    assert np.abs(plain.step(tok, pos) - ref.step(tok, pos)).max() > 1e-2
    plain.close()
    gpu.close()


@pytest.mark.parametrize("variant,opts", [
    (dict(batch=6, max_seq=192), dict(fusion=31, transitive_reduction=1)),
    (dict(batch=8, max_seq=192, ffn=0, n_experts=8, top_k=2, expert_ffn=64), dict(fusion=31, transitive_reduction=1, n_workers=24)),
    (dict(batch=5, max_seq=192), dict(fusion=0, launch_mode=1)),
])
def test_graph_set_runs_the_smallest_graph_that_holds_the_active_sequences(variant, opts):
    """One graph per power-of-two batch size over ONE KV cache laid out for the maximum batch:
    n_active sequences run on the smallest graph that holds them, and their logits must be what
    the oracle computes for those sequences alone (sequences are independent; the synthetic cache
    of sequence b does not depend on the batch size).  The number of active sequences changes
    from step to step, so rows appended by one graph are read by another."""
    s = G.small_variant("C1", n_layers=2, **variant)
    B = s.batch
    model = DeviceModel(s, 5)
    gs = M.compile_set(s, model.weight_ptrs(), model.kv_ptrs(), **opts)
    want_sizes = [b for b in (1, 2, 4, 8, 16) if b < B] + [B]
    assert len(gs) == len(want_sizes)
    assert all(gs.graph(i).stats()["n_workers"] > 0 for i in range(len(gs)))
    assert gs.batch_for(0) == 0 and gs.batch_for(B + 1) == 0 and gs.batch_for(B) == B and gs.batch_for(3) == 4
    # the oracle keeps ONE model of the maximum batch; a step on the first n sequences is a step
    # of a batch-n oracle that shares its cache rows: run the full batch and compare n rows
    ref = D.DecoderOracle(s, G.SynthWeights(s, 5), "f32")
    tok = G.tokens(5, s)
    pos = np.array([(31 * b + 7) % 120 for b in range(B)], np.int32)
    dev = model.device
    d_tok = torch.zeros(B, dtype=torch.int32, device=dev)
    d_pos = torch.zeros(B, dtype=torch.int32, device=dev)
    logits = torch.empty((B, s.vocab), dtype=torch.float32, device=dev)
    st = torch.cuda.current_stream().cuda_stream
    for step, n in enumerate([B, 1, 3, 2, B - 1, B]):
        b_run = gs.batch_for(n)
        # padding slots n .. b_run-1 are computed too (and append their rows): the reference does
        # the same for exactly those slots, so both caches stay identical
        want = ref.step(tok, pos)
        d_tok.copy_(torch.as_tensor(tok)); d_pos.copy_(torch.as_tensor(pos))
        logits.fill_(float("nan"))
        gs.decode_step(n, d_tok.data_ptr(), d_pos.data_ptr(), logits.data_ptr(), st)
        torch.cuda.synchronize()
        for i in range(len(gs)):
            gs.graph(i).status()
        got = logits.cpu().numpy().reshape(-1)[: b_run * s.vocab].reshape(b_run, s.vocab)
        assert np.isfinite(got[:n]).all(), (step, n)
        ambiguous = False
        if s.n_experts:   # top-k is discontinuous: a decision may differ where the margin is below fp32 resolution
            ex, _ = gs.graph(want_sizes.index(b_run)).moe_selection()
            ex = ex.reshape(s.n_layers, b_run, s.top_k)
            for l in range(s.n_layers):
                for b in range(b_run):
                    if ex[l, b].tolist() != ref.last_moe_sel[l, b].tolist():
                        r = np.sort(ref.last_moe_logits[l, b].astype(np.float64))[::-1]
                        assert r[s.top_k - 1] - r[s.top_k] < 1e-5, (step, l, b)
                        ambiguous = True
        if not ambiguous:
            if step == 0:
                assert rel_err(got[:n], want[:n]) < TOL, (step, n)
            # later steps read K/V rows each side appended itself: a value on a bf16 rounding
            # boundary may have gone the other way, so the bound is on the largest logit
            assert np.abs(got[:n] - want[:n]).max() / np.abs(want[:n]).max() < 2e-3, (step, n)
            assert got[:n].argmax(-1).tolist() == want[:n].argmax(-1).tolist(), (step, n)
        # advance only the slots that ran (active and padding); the others keep token and position
        nxt = want.argmax(-1).astype(np.int32)
        ran = np.arange(B) < b_run
        # the reference appended rows for ALL slots; slots that did not run on the GPU must not
        # move on, so their next reference step rewrites the same row with the same token
        tok = np.where(ran, nxt, tok).astype(np.int32)
        pos = np.where(ran, pos + 1, pos).astype(np.int32)
    with pytest.raises(M.MpkError):
        gs.decode_step(0, d_tok.data_ptr(), d_pos.data_ptr(), logits.data_ptr(), st)
    with pytest.raises(M.MpkError):
        gs.decode_step(B + 1, d_tok.data_ptr(), d_pos.data_ptr(), logits.data_ptr(), st)
    gs.destroy()


# ------------------------------------------------------------------ debug modes, pre-load ablation
POISON, JITTER = M.binding.DEBUG_POISON, M.binding.DEBUG_JITTER


@pytest.mark.parametrize("variant,opts", [
    (("C1", {}), dict(fusion=31, transitive_reduction=1)),
    (("C1", {}), dict(fusion=0)),
    (("C1", dict(batch=3)), dict(fusion=7, transitive_reduction=1, n_sched_wgs=2)),
    (("C1", dict(batch=8, max_seq=192)), dict(fusion=31, transitive_reduction=1)),
    (("C1", dict(batch=4, ffn=0, n_experts=16, top_k=4, expert_ffn=96)), dict(fusion=31, transitive_reduction=1)),
    (("C2", dict(n_layers=2)), dict(fusion=31, transitive_reduction=1)),
    # inputs that end inside a k-group of the matrix-core body (2056 = 32 x 64 + 8): what lies
    # between the end of a staged row, or of the gains, and the end of the k-group is multiplied too
    (("C1", dict(n_layers=2, hidden=2056, ffn=3000, batch=5, max_seq=192)), dict(fusion=31, transitive_reduction=1, n_workers=24)),
    # the kernels compiled for head dimension 128 at batch 5..16, dense (1000 inputs: under one staging tile) and experts
    (("C1", dict(n_layers=2, hidden=1000, ffn=520, batch=16, vocab=520, head_dim=128, n_q_heads=8, n_kv_heads=2, max_seq=192)),
     dict(fusion=31, transitive_reduction=1, n_workers=24)),
    (("C1", dict(n_layers=2, hidden=528, batch=16, head_dim=128, n_q_heads=8, n_kv_heads=1, ffn=0, n_experts=16, top_k=4, expert_ffn=104, max_seq=192)),
     dict(fusion=31, transitive_reduction=1)),
])
@pytest.mark.parametrize("debug", [POISON, JITTER, POISON | JITTER])
def test_poisoned_buffers_and_jittered_task_starts_change_nothing(variant, opts, debug):
    """The event protocol under stress: every buffer that carries data between tasks is filled
    with NaN before each launch (a task that reads what this step has not produced yet, or relies
    on what the previous step left, turns the logits into NaN) and every task starts after a
    pseudo-random delay of up to 20 us that differs from step to step (a consumer that does not
    really wait for its producers reads the poison).  Three steps each, compared as strictly as
    without the modes; all waits stay bounded, nothing is made to hang."""
    base, kw = variant
    s = G.small_variant(base, **kw)
    tok, pos = G.tokens(1, s), G.kv_lengths(1, s)
    if base == "C1":
        pos = np.array([(41 * b + 7) % 120 for b in range(s.batch)], np.int32)
    strict_steps(s, 1, dict(debug_flags=debug, **opts), tok, pos, 3)


@pytest.mark.parametrize("variant,opts", [
    (("C1", {}), dict(fusion=31, transitive_reduction=1)),
    (("C1", dict(batch=8, max_seq=192)), dict(fusion=31, transitive_reduction=1)),
    (("C1", dict(batch=2)), dict(fusion=7, n_sched_wgs=2)),
    (("C1", dict(batch=4, ffn=0, n_experts=16, top_k=4, expert_ffn=96)), dict(fusion=31, transitive_reduction=1)),
])
def test_cross_task_preloading_switched_off(variant, opts):
    """no_preload = 1 (the ablation of Section 6.5): no weight or cache-row request before a
    task's event; same results."""
    base, kw = variant
    s = G.small_variant(base, **kw)
    tok = G.tokens(1, s)
    pos = np.array([(41 * b + 7) % 120 for b in range(s.batch)], np.int32)
    strict_steps(s, 1, dict(no_preload=1, **opts), tok, pos, 2)


def test_watchdog_ends_a_step_whose_event_never_activates_and_reset_recovers():
    """MPK_DEBUG_LOSE_NOTIFY: the first launch loses worker 0's notifications, so the events they
    belong to never activate.  Every wait is bounded by the watchdog (20 ms here): all workgroups
    exit by themselves, the status is MPK_ERR_TIMEOUT (not a hang, not a fault), mpk_graph_reset
    clears counters and queues, and the next steps are correct again."""
    s = G.small_variant("C1", batch=2)
    tok, pos = G.tokens(0, s), G.kv_lengths(0, s)
    ref = D.DecoderOracle(s, G.SynthWeights(s, 0), "f64")
    for opts in (dict(fusion=31, transitive_reduction=1), dict(fusion=7, n_sched_wgs=2)):
        gpu = GpuDecoder(s, 0, spin_timeout_ms=20, debug_flags=M.binding.DEBUG_LOSE_NOTIFY, **opts)
        stream = torch.cuda.current_stream().cuda_stream
        gpu.tok.copy_(torch.as_tensor(tok))
        gpu.pos.copy_(torch.as_tensor(pos))
        gpu.graph.decode_step(gpu.tok.data_ptr(), gpu.pos.data_ptr(), gpu.logits.data_ptr(), stream)
        torch.cuda.synchronize()
        with pytest.raises(M.binding.MpkError) as e:
            gpu.graph.status()
        assert e.value.status == M.binding.MPK_ERR_TIMEOUT and "watchdog" in str(e.value)
        gpu.graph.reset()
        gpu.graph.status()                     # clean again
        gpu.model.reset_kv()
        fresh = D.DecoderOracle(s, G.SynthWeights(s, 0), "f64")
        t, p = tok.copy(), pos.copy()
        for step in range(2):
            got, want, _, _ = held_step(fresh, gpu, t, p)
            assert rel_err(got, want) < TOL, step
            t, p = want.argmax(-1).astype(np.int32), p + 1
        gpu.close()
    del ref
