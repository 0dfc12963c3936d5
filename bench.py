#!/usr/bin/env python3
"""Decode benchmark on one MI355X.  Default workload: the Qwen3-8B-shaped config, batch 1, KV
1024, greedy steps (--config C3: Llama-3-8B-shaped, batch 8, ragged KV; --config C4: Qwen3-30B-A3B-
shaped mixture of experts, batch 16; --config C5: 70B-shaped).

A "step" is one decode step through the persistent mega-kernel (mpk_decode_step) followed by the
greedy token feedback (arg max on the device, no host sync).  Prints ONE JSON line.
The default run also attaches `batch8` (the batch-8 shape timed the same way) and `serving` (the
batch-1 workload served from inside the kernel: paged KV cache, serving task, 32 iterations per
call) and `offline` (one request of the paper's end-to-end workload -- 64-token prompt, 1024
generated tokens -- served in one call until the queue has drained).
Also measured and attached: the same task bodies launched one kernel per operator (eager and as
a replayed HIP graph), and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def cpu_baseline(shape, seed, n_layers_sample=4, reps=3):
    """The oracle as it stands, on the host cores: one decode step restricted to the first
    `n_layers_sample` layers (weights generated beforehand, not timed) plus the LM head, scaled to
    the full depth."""
    import numpy as np
    from oracle import decoder as D
    from synth import gen as G
    prov = G.SynthWeights(shape, seed, cache=True)
    for l in range(n_layers_sample):
        prov.layer(l)
    prov.lm_head()
    prov.final_norm()
    o = D.DecoderOracle(shape, prov, "f32", n_layers=n_layers_sample)
    for l in range(n_layers_sample):
        o._kv(l)
    tok, pos = G.tokens(seed, shape), G.kv_lengths(seed, shape)
    t_layers, t_head = [], []
    for _ in range(reps):
        t0 = time.perf_counter()
        hid = o.step(tok, pos, return_hidden=True)
        t1 = time.perf_counter()
        g, W = prov.final_norm(), prov.lm_head()
        for b in range(shape.batch):
            o.ops.linear(W, o.ops.rmsnorm(hid[b], g, shape.rms_eps))
        t2 = time.perf_counter()
        t_layers.append(t1 - t0)
        t_head.append(t2 - t1)
    per_layer = min(t_layers) / n_layers_sample
    step_s = per_layer * shape.n_layers + min(t_head)
    return {"value": step_s * 1e3 / shape.batch, "unit": "ms/token",
            "cores": int(D.lib("f32").orc_threads()), "kind": "oracle",
            "sample": f"one decode step over the first {n_layers_sample} of {shape.n_layers} "
                      f"layers + LM head, best of {reps}, layer time scaled to full depth"}


def measured_traffic(config):
    """HBM bytes per launch of the persistent kernel from the committed counter summary of this
    workload (two rocprofv3 --pmc runs, scaled by a copy kernel of known size), or None."""
    import glob
    import re
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", f"mpk_mega_kernel_{config}_*.md"))):
        m = re.search(r"traffic_bytes_per_launch:\s*(\d+)", open(path).read())
        if m:
            return int(m.group(1))
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--config", default="C2")
    ap.add_argument("--fusion", type=int, default=31)
    ap.add_argument("--no-baselines", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain copy kernel of this many MiB (synth_copy_kernel): "
                         "a launch of known HBM traffic to scale profiler byte counters by")
    ap.add_argument("--tokens-per-launch", type=int, default=1,
                    help="N > 1: compile the graph with the sampling operator and decode N tokens per "
                         "launch of the persistent kernel (no arg max / copy kernels between tokens); "
                         "--steps must be a multiple of N")
    ap.add_argument("--opt", action="append", default=[], metavar="NAME=INT",
                    help="extra mpk_compile_options field, e.g. --opt attn_chunks=32")
    ap.add_argument("--serving", type=int, default=0, metavar="PAGE_SIZE",
                    help="also time the same workload served from inside the kernel (paged KV cache of this "
                         "page size, serving task on the start event, --steps iterations in one launch) and "
                         "attach it as the 'serving' sub-record; prompts are fed through the decode path "
                         "first, off the clock, until every slot stands at the workload's KV length")
    ap.add_argument("--offline", type=int, default=0, metavar="N_REQUESTS",
                    help="also run the paper's end-to-end workload on this config (offline batched inference: N "
                         "requests of a 64-token prompt and 1024 generated tokens, served from inside the kernel "
                         "until the queue has drained) and attach it as the 'offline' sub-record")
    ap.add_argument("--no-serving", action="store_true",
                    help="default run (C2) only: skip the serving and offline sub-records")
    ap.add_argument("--no-batch8", action="store_true",
                    help="default run (C2, batch 1) only: skip the batch-8 half of the metric (C3)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    b8 = None
    if args.config == "C2" and not args.no_batch8 and args.tokens_per_launch == 1:
        # the metric is ms/token at batch 1 AND 8: the batch-8 shape (C3) timed the same way, as a
        # sub-record of the same line.  In a process of its own, started before this one touches
        # the GPU: measured after the batch-1 workload in one process the batch-8 step came out
        # 3 to 4 % slower (5.53-5.57 against 5.37 ms, three runs each) -- where the allocator
        # places 20 GB after 16 GB were freed is not part of either workload.
        import subprocess
        cmd = [sys.executable, os.path.abspath(__file__), "--config", "C3", "--no-cpu", "--steps", str(args.steps),
               "--warmup", str(args.warmup), "--fusion", str(args.fusion)] + (["--no-baselines"] if args.no_baselines else [])
        for o in args.opt:
            cmd += ["--opt", o]
        child = subprocess.run(cmd, capture_output=True, text=True)
        if child.returncode != 0:
            sys.stderr.write(child.stderr)
            sys.exit(child.returncode)
        b8 = json.loads(child.stdout.strip().splitlines()[-1])
    out = measure(args, args.config, baselines=not args.no_baselines, cpu=not args.no_cpu)
    if args.serving or (args.config == "C2" and not args.no_serving and args.tokens_per_launch == 1):
        # (the default run: the batch-1 workload also served from inside the kernel, pages of 64 rows)
        out["serving"] = measure_serving(args, args.config, args.serving or 64)
    if args.offline or (args.config == "C2" and not args.no_serving and args.tokens_per_launch == 1):
        # (the default run: one request of the paper's offline workload on the batch-1 shape)
        out["offline"] = measure_offline(args, args.config, args.offline or 1)
    if b8 is not None:
        out["batch8"] = {k: b8[k] for k in ("metric", "value", "unit", "ms_per_step", "tokens_per_s", "steps", "warmup",
                                            "achieved_hbm_GBps", "bytes_per_step", "roofline", "config", "final_tokens")
                         if k in b8}
        for k in ("per_op_eager_ms_per_step", "per_op_graph_ms_per_step", "per_op_tokens_match"):
            if k in b8:
                out["batch8"][k] = b8[k]
    print(json.dumps(out))


def measure_serving(args, config, page_size):
    """The workload of `config` served from inside the persistent kernel (paper Section 6.1):
    one request per batch slot, its prompt as long as the slot's KV length in the workload, fed
    through the decode path off the clock (requests are submitted longest first, so that all
    slots reach their lengths in the same iteration); then args.steps iterations -- serving
    task, decode step through the page tables, greedy sampling -- timed as ONE mpk_serve_run call
    (one launch of the persistent kernel at batch > 4, a launch per iteration back to back with
    no host synchronisation at batch <= 4: the library's choice)."""
    import numpy as np
    import torch
    import paper_2512_22219_amd as M
    from synth import gen as G
    from synth.device import DeviceModel

    shape = G.CONFIGS[config]
    seed = 0
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    model = DeviceModel(shape, seed, dev)
    model.k = model.v = None          # the contiguous cache is not used here
    torch.cuda.empty_cache()
    n_pages = shape.batch + shape.batch * (shape.max_seq // page_size)
    pools = []
    for which in (G.L_KCACHE, G.L_VCACHE):
        pool = torch.empty((shape.n_layers, n_pages, shape.n_kv_heads, page_size, shape.head_dim),
                           dtype=torch.bfloat16, device=dev)
        for l in range(shape.n_layers):
            G.fill_device(pool[l], seed, G.layer_tid(l, which), 0, "kv")
        pools.append(pool)
    common = dict(fusion=args.fusion, transitive_reduction=1)
    common.update({k: int(v) for k, v in (o.split("=", 1) for o in args.opt)})
    graph = M.compile_graph(shape, model.weight_ptrs(), (pools[0].data_ptr(), pools[1].data_ptr()), launch_mode=0,
                            **{"greedy_loop": 1, "serving": 1, "kv_page_size": page_size, "kv_pages": n_pages, **common})
    stats = graph.stats()
    lens = sorted((int(x) for x in G.kv_lengths(seed, shape)), reverse=True)
    max_new = args.steps + args.warmup + 1          # nobody finishes on the clock
    assert lens[0] + max_new - 1 <= shape.max_seq
    srv = graph.serve(shape.batch, lens[0], max_new, -1)
    stream = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(seed)

    def run(n):
        while n > 0:
            k = min(n, 4096)
            srv.run(k, stream)
            n -= k

    for i, L in enumerate(lens):
        srv.submit(rng.integers(0, shape.vocab, L), max_new, stream)
        run((L - lens[i + 1]) if i + 1 < len(lens) else L + args.warmup)
    torch.cuda.synchronize()
    graph.status()
    st = srv.state()
    assert sorted(st["positions"], reverse=True) == [L + args.warmup - 1 for L in lens], st["positions"]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    srv.run(args.steps, stream)
    e1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    graph.status()
    st = srv.state()
    assert all(r >= 0 for r in st["slot_req"]) and st["iterations"] == lens[0] + args.warmup + args.steps
    ms = dt * 1e3 / args.steps
    pos_avg = float(sum(lens)) + shape.batch * (args.warmup + (args.steps - 1) / 2 + 1)
    bytes_step = stats["weight_bytes"] + stats["kv_row_bytes"] * pos_avg
    kern_ms = e0.elapsed_time(e1) / args.steps
    out = {"ms_per_iteration": ms, "tokens_per_s": shape.batch * 1e3 / ms, "kernel_ms_per_iteration": kern_ms,
           "iterations_per_call": args.steps, "page_size": page_size, "kv_pages": n_pages,
           "achieved_hbm_GBps": bytes_step / (kern_ms * 1e-3) / 1e9,
           "prompt_iterations_off_the_clock": lens[0] + args.warmup,
           "tokens_produced": st["tokens_produced"]}
    srv.destroy()
    graph.destroy()
    del model, pools
    torch.cuda.empty_cache()
    return out


def measure_offline(args, config, n_requests, prompt_len=64, new_tokens=1024, page_size=64):
    """The paper's end-to-end workload (Section 6.2: offline batched inference, every request a
    64-token prompt and 1024 generated tokens, paged attention and continuous batching on, the
    maximum batch size = the config's batch): n_requests seeded requests are queued up front and
    served from inside the persistent kernel until the server has drained -- mpk_serve_run calls of
    up to 512 iterations, each ending by itself when nothing is left.  Prompts go through the
    decode path."""
    import numpy as np
    import torch
    import paper_2512_22219_amd as M
    from synth import gen as G
    from synth.device import DeviceModel

    shape = G.CONFIGS[config]
    seed = 0
    assert prompt_len + new_tokens - 1 <= shape.max_seq
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    model = DeviceModel(shape, seed, dev)
    model.k = model.v = None
    torch.cuda.empty_cache()
    per_req = -(-(prompt_len + new_tokens - 1) // page_size)
    n_pages = shape.batch + shape.batch * per_req
    pools = [torch.zeros((shape.n_layers, n_pages, shape.n_kv_heads, page_size, shape.head_dim),
                         dtype=torch.bfloat16, device=dev) for _ in range(2)]
    common = dict(fusion=args.fusion, transitive_reduction=1)
    common.update({k: int(v) for k, v in (o.split("=", 1) for o in args.opt)})
    graph = M.compile_graph(shape, model.weight_ptrs(), (pools[0].data_ptr(), pools[1].data_ptr()), launch_mode=0,
                            **{"greedy_loop": 1, "serving": 1, "kv_page_size": page_size, "kv_pages": n_pages, **common})
    srv = graph.serve(n_requests, prompt_len, new_tokens, -1)
    stream = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(seed)
    for _ in range(n_requests):
        srv.submit(rng.integers(0, shape.vocab, prompt_len), new_tokens, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    launches = 0
    while True:
        srv.run(512, stream)      # (a call per 512 iterations: the host looks at the queue in between)
        launches += 1
        torch.cuda.synchronize()
        st = srv.state()
        if st["q_head"] == n_requests and all(r < 0 for r in st["slot_req"]):
            break
        assert launches < 64
    dt = time.perf_counter() - t0
    graph.status()
    assert st["tokens_produced"] == n_requests * new_tokens
    assert all(srv.result(r)[1] == 2 for r in range(n_requests))
    out = {"workload": f"{n_requests} requests, prompt {prompt_len}, {new_tokens} generated tokens each, max batch {shape.batch}, "
                       f"pages of {page_size} rows",
           "seconds": dt, "iterations": st["iterations"], "calls": launches,
           "ms_per_iteration": dt * 1e3 / st["iterations"],
           "generated_tokens_per_s": n_requests * new_tokens / dt,
           "ms_per_generated_token_per_request": dt * 1e3 * min(shape.batch, n_requests) / (n_requests * new_tokens)}
    srv.destroy()
    graph.destroy()
    del model, pools
    torch.cuda.empty_cache()
    return out


def measure(args, config, baselines=True, cpu=True):
    """One workload: the persistent kernel timed over args.steps greedy steps, then (optionally)
    the kernel-per-operator launches of the same graph and the CPU oracle.  Returns the record."""
    import numpy as np
    import torch
    import paper_2512_22219_amd as M
    from synth import gen as G
    from synth.device import DeviceModel

    shape = G.CONFIGS[config]
    seed = 0
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    model = DeviceModel(shape, seed, dev)
    tok0 = torch.as_tensor(G.tokens(seed, shape), device=dev)
    pos0 = torch.as_tensor(G.kv_lengths(seed, shape), device=dev)
    tok, pos = tok0.clone(), pos0.clone()
    logits = torch.empty((shape.batch, shape.vocab), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    n_total = args.steps + args.warmup
    assert int(pos0.max()) + n_total <= shape.max_seq

    tpl = args.tokens_per_launch
    assert tpl >= 1 and args.steps % tpl == 0 and args.warmup % tpl == 0, "--steps and --warmup must be multiples of --tokens-per-launch"

    def run(graph, n, events=None):
        if tpl > 1 and getattr(graph, "multi", False):
            for i in range(0, n, tpl):
                if events is not None:
                    events[i][0].record()
                graph.decode_steps(tpl, tok.data_ptr(), pos.data_ptr(), 0, logits.data_ptr(), 0, stream)
                if events is not None:
                    events[i][1].record()
            return
        for i in range(n):
            if events is not None:
                events[i][0].record()
            graph.decode_step(tok.data_ptr(), pos.data_ptr(), logits.data_ptr(), stream)
            if events is not None:
                events[i][1].record()
            torch.argmax(logits, dim=-1, out=tok64)
            tok.copy_(tok64)
            pos.add_(1)

    tok64 = torch.empty(shape.batch, dtype=torch.int64, device=dev)

    def timed(graph):
        tok.copy_(tok0)
        pos.copy_(pos0)
        model.reset_kv()
        run(graph, args.warmup)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(graph, args.steps, ev)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        graph.status()
        step = tpl if getattr(graph, "multi", False) else 1
        kern_ms = [ev[i][0].elapsed_time(ev[i][1]) / step for i in range(0, args.steps, step)]
        return dt, kern_ms

    common = dict(fusion=args.fusion, transitive_reduction=1)
    common.update({k: int(v) for k, v in (o.split("=", 1) for o in args.opt)})
    mega = M.compile_graph(shape, model.weight_ptrs(), model.kv_ptrs(), launch_mode=0,
                           **{**({"greedy_loop": 1} if tpl > 1 else {}), **common})
    mega.multi = tpl > 1
    stats = mega.stats()
    dt, kern_ms = timed(mega)
    final_tokens = tok.cpu().numpy().tolist()
    ms_per_step = dt * 1e3 / args.steps
    # algorithmic bytes of one launch: weights streamed once + K/V rows read (grows by one row a
    # step; averaged over the timed steps)
    pos_avg = float(pos0.float().sum()) + shape.batch * (args.warmup + (args.steps - 1) / 2 + 1)
    bytes_step = stats["weight_bytes"] + stats["kv_row_bytes"] * pos_avg
    moe_active_avg = None
    assert not (stats["expert_bytes"] and tpl > 1), "--tokens-per-launch > 1 is not wired up for the MoE byte count"
    if stats["expert_bytes"]:
        # mixture of experts: a step streams only the experts it selected.  Replay the same greedy
        # trajectory off the clock and read the number of distinct experts per layer after
        # every step.
        tok.copy_(tok0)
        pos.copy_(pos0)
        model.reset_kv()
        counts = []
        for i in range(args.warmup + args.steps):
            run(mega, 1)
            torch.cuda.synchronize()
            if i >= args.warmup:
                counts.append(int(mega.moe_active().sum()))
        moe_active_avg = sum(counts) / len(counts)
        bytes_step += stats["expert_bytes"] * moe_active_avg
    kern_avg_ms = sum(kern_ms) / len(kern_ms)
    achieved = bytes_step / (kern_avg_ms * 1e-3) / 1e9
    out = {
        "metric": f"decode_ms_per_token_batch{shape.batch}", "value": ms_per_step / shape.batch,
        "unit": "ms/token", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 weights, fp32 activations/accumulation",
        "data": "synthetic",
        "config": {"workload": f"{shape.name}: {shape.n_layers} layers, hidden {shape.hidden}, "
                               f"{shape.n_q_heads}q/{shape.n_kv_heads}kv heads, ffn {shape.ffn}, "
                               f"vocab {shape.vocab}, batch {shape.batch}, KV "
                               f"{shape.kv_len_lo}" + (f"..{shape.kv_len_hi}" if shape.kv_len_hi != shape.kv_len_lo else "")
                               + " prior positions, greedy decode",
                   "launch": "persistent mega-kernel" + (f", {tpl} tokens per mpk_decode_steps call" if tpl > 1 else ""),
                   "fusion": args.fusion,
                   "n_workers": stats["n_workers"], "tasks": stats["n_tasks"],
                   "events": stats["n_events"],
                   **({"distinct_experts_per_step": moe_active_avg} if moe_active_avg is not None else {})},
        "tokens_per_s": shape.batch * 1e3 / ms_per_step,
        "achieved_hbm_GBps": bytes_step / (ms_per_step * 1e-3) / 1e9,
        "bytes_per_step": bytes_step,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": 8000.0, "unit": "GB/s",
                     "frac": achieved / 8000.0, "traffic": measured_traffic(config),
                     "kernel": "mpk_mega_kernel", "kernel_avg_ms": kern_avg_ms},
        "final_tokens": final_tokens,
    }
    mega.destroy()
    if args.calib_copy_mib:
        a = torch.zeros(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        G.copy_device(b, a)
        torch.cuda.synchronize()
        del a, b
    if baselines:
        per_op = M.compile_graph(shape, model.weight_ptrs(), model.kv_ptrs(), launch_mode=1, **common)
        dt_e, _ = timed(per_op)
        out["per_op_eager_ms_per_step"] = dt_e * 1e3 / args.steps
        out["per_op_tokens_match"] = tok.cpu().numpy().tolist() == final_tokens
        # the same launches captured once and replayed as a HIP graph
        tok.copy_(tok0); pos.copy_(pos0); model.reset_kv()
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            per_op.decode_step(tok.data_ptr(), pos.data_ptr(), logits.data_ptr(), side.cuda_stream)
            side.synchronize()
            tok.copy_(tok0); pos.copy_(pos0); model.reset_kv()
            with torch.cuda.graph(g, stream=side):
                per_op.decode_step(tok.data_ptr(), pos.data_ptr(), logits.data_ptr(), side.cuda_stream)
                torch.argmax(logits, dim=-1, out=tok64)
                tok.copy_(tok64)
                pos.add_(1)
        tok.copy_(tok0); pos.copy_(pos0); model.reset_kv()
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        out["per_op_graph_ms_per_step"] = (time.perf_counter() - t0) * 1e3 / args.steps
        out["per_op_graph_tokens_match"] = tok.cpu().numpy().tolist() == final_tokens
        per_op.status()
        per_op.destroy()
    if cpu:
        out["cpu_baseline"] = cpu_baseline(shape, seed)
    del model
    torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
