"""Thin ctypes binding over include/mpk.h: argument marshalling only.

Every step of the decode path runs inside libmpk.so; nothing here computes.  If the library is
missing the import fails loudly (there is no fallback path)."""
from __future__ import annotations

import ctypes as C
import os
import weakref

import numpy as np

from . import build as _build

_HERE = os.path.dirname(os.path.abspath(__file__))

(MPK_OK, MPK_ERR_INVALID_ARG, MPK_ERR_UNSUPPORTED, MPK_ERR_OOM, MPK_ERR_RESIDENCY, MPK_ERR_HIP,
 MPK_ERR_TIMEOUT, MPK_ERR_INTERNAL, MPK_ERR_DEVICE) = range(9)
FUSE_NORM, FUSE_RESID, FUSE_SWIGLU, FUSE_MERGE, FUSE_ROPE = 1, 2, 4, 8, 16
LAUNCH_MEGA, LAUNCH_PER_OP = 0, 1
TASK_DUMMY_OP = 0xFFFFFFFF
(OP_EMBED, OP_RMSNORM, OP_LINEAR, OP_ROPE, OP_ATTN_PARTIAL, OP_ATTN_MERGE, OP_ADD, OP_SWIGLU,
 OP_GATEUP, OP_ROUTER, OP_EXPERT) = range(11)
OP_COMBINE = 12
OP_ARGMAX = 13
OP_SERVE = 14


class ModelConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_layers", C.c_uint32), ("hidden", C.c_uint32),
                ("n_q_heads", C.c_uint32), ("n_kv_heads", C.c_uint32), ("head_dim", C.c_uint32),
                ("ffn", C.c_uint32), ("vocab", C.c_uint32), ("rms_eps", C.c_float),
                ("rope_theta", C.c_float), ("batch", C.c_uint32), ("max_seq", C.c_uint32),
                ("n_experts", C.c_uint32), ("top_k", C.c_uint32), ("expert_ffn", C.c_uint32),
                ("flags", C.c_uint32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wqkv", "wo", "mlp_norm", "wgu", "wd",
                                          "router", "expert_wgu", "expert_wd", "q_norm", "k_norm")]


class WeightPtrs(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(LayerWeights))]


class KvPtrs(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p)]


class CompileOptions(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in
                ("struct_size", "n_workers", "n_sched_wgs", "fusion", "transitive_reduction",
                 "attn_chunks", "tiles_linear", "tiles_lm_head", "tiles_pointwise", "launch_mode",
                 "force_aot", "no_preload", "host_only", "spin_timeout_ms", "debug_flags",
                 "tiles_moe", "greedy_loop", "kv_batch")] + [("worker_weight_permille", C.c_uint32 * 8),
                                                             ("no_lds_pages", C.c_uint32),
                                                             ("xcd_balance", C.c_uint32),
                                                             ("no_attn_balance", C.c_uint32),
                                                             ("kv_page_size", C.c_uint32),
                                                             ("kv_pages", C.c_uint32),
                                                             ("serving", C.c_uint32),
                                                             ("tiles_sampling", C.c_uint32)]


class ServeConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("max_requests", C.c_uint32), ("max_prompt", C.c_uint32),
                ("max_new", C.c_uint32), ("eos_token", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_ops", C.c_uint32), ("n_tasks", C.c_uint32),
                ("n_dummy_tasks", C.c_uint32), ("n_events", C.c_uint32),
                ("n_events_fused", C.c_uint32), ("n_pair_deps", C.c_uint64),
                ("n_pairs_removed", C.c_uint64), ("n_jit_tasks", C.c_uint32),
                ("n_aot_tasks", C.c_uint32), ("n_workers", C.c_uint32),
                ("n_sched_wgs", C.c_uint32), ("lds_bytes", C.c_uint32),
                ("task_desc_bytes", C.c_uint32), ("successor_bytes_unlinearized", C.c_uint64),
                ("successor_bytes_linearized", C.c_uint64), ("weight_bytes", C.c_uint64),
                ("kv_row_bytes", C.c_uint64), ("act_bytes", C.c_uint64),
                ("expert_bytes", C.c_uint64)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


EXPORT_HEADER = np.dtype([(n, "<u4") for n in
                          ("magic", "version", "n_ops", "n_tasks", "n_events", "n_workers",
                           "n_sched_wgs", "start_event", "terminal_event", "n_real_tasks",
                           "fusion", "reserved")])
EXPORT_OP = np.dtype([("kind", "<u4"), ("layer", "<i4"), ("tb", "<u4"), ("tc", "<u4"),
                      ("n_tasks", "<u4"), ("jit", "<u4"), ("rows", "<u4"), ("cols", "<u4")])
EXPORT_TASK = np.dtype([("op", "<u4"), ("tile", "<u4"), ("dep_event", "<i4"),
                        ("trig_event", "<i4"), ("worker", "<i4"), ("jit", "<u4")])
EXPORT_EVENT = np.dtype([("required", "<u4"), ("first", "<u4"), ("last", "<u4"),
                         ("flags", "<u4")])

SYMBOLS = ("mpk_compile", "mpk_compile_dag", "mpk_decode_step", "mpk_decode_steps", "mpk_graph_status",
           "mpk_graph_reset", "mpk_graph_stats", "mpk_graph_export", "mpk_graph_trace",
           "mpk_graph_moe_active", "mpk_graph_moe_selection", "mpk_moe_task_share", "mpk_compile_set",
           "mpk_set_decode_step", "mpk_decode_step_static", "mpk_set_size", "mpk_set_batch_for", "mpk_set_graph",
           "mpk_set_destroy", "mpk_last_error", "mpk_graph_destroy", "mpk_static_scratch_need",
           "mpk_graph_set_page_table", "mpk_serve_create", "mpk_serve_submit", "mpk_serve_run",
           "mpk_serve_result", "mpk_serve_state", "mpk_serve_logits", "mpk_serve_destroy",
           "mpk_serve_create_set", "mpk_serve_last_batch", "mpk_serve_status")
DEBUG_TRACE, DEBUG_POISON, DEBUG_JITTER, DEBUG_LOSE_NOTIFY = 1, 2, 4, 8

_lib = None


def lib():
    """Load libmpk.so (building it only if nothing has been built yet)."""
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build(force=True)
        L = C.CDLL(path)
        vp = C.c_void_p
        L.mpk_compile.argtypes = [C.POINTER(ModelConfig), C.POINTER(WeightPtrs), C.POINTER(KvPtrs),
                                  C.POINTER(CompileOptions), C.POINTER(vp)]
        L.mpk_compile_dag.argtypes = [C.c_uint32, vp, C.c_size_t, C.POINTER(CompileOptions),
                                      C.POINTER(vp)]
        L.mpk_decode_step.argtypes = [vp, vp, vp, vp, vp]
        L.mpk_decode_step_static.argtypes = [vp, vp, vp, vp, vp]
        L.mpk_static_scratch_need.argtypes = [vp]
        L.mpk_static_scratch_need.restype = C.c_size_t
        L.mpk_decode_steps.argtypes = [vp, C.c_uint32, vp, vp, vp, vp, vp, vp]
        L.mpk_graph_status.argtypes = [vp]
        L.mpk_graph_reset.argtypes = [vp]
        L.mpk_graph_stats.argtypes = [vp, C.POINTER(Stats)]
        L.mpk_graph_export.argtypes = [vp, vp, C.c_size_t, C.POINTER(C.c_size_t)]
        L.mpk_graph_trace.argtypes = [vp, vp, C.c_size_t, C.POINTER(C.c_size_t)]
        L.mpk_graph_moe_active.argtypes = [vp, vp, C.c_size_t, C.POINTER(C.c_size_t)]
        L.mpk_moe_task_share.argtypes = [C.c_uint32] * 4 + [C.POINTER(C.c_uint32)] * 2
        L.mpk_graph_moe_selection.argtypes = [vp, vp, vp, C.c_size_t, C.POINTER(C.c_size_t)]
        L.mpk_last_error.restype = C.c_char_p
        L.mpk_graph_destroy.argtypes = [vp]
        L.mpk_graph_destroy.restype = None
        L.mpk_compile_set.argtypes = L.mpk_compile.argtypes
        L.mpk_set_decode_step.argtypes = [vp, C.c_uint32, vp, vp, vp, vp]
        L.mpk_set_size.argtypes = [vp]
        L.mpk_set_size.restype = C.c_uint32
        L.mpk_set_batch_for.argtypes = [vp, C.c_uint32]
        L.mpk_set_batch_for.restype = C.c_uint32
        L.mpk_set_graph.argtypes = [vp, C.c_uint32]
        L.mpk_set_graph.restype = vp
        L.mpk_set_destroy.argtypes = [vp]
        L.mpk_set_destroy.restype = None
        L.mpk_graph_set_page_table.argtypes = [vp, vp]
        L.mpk_serve_create.argtypes = [vp, C.POINTER(ServeConfig), C.POINTER(vp)]
        L.mpk_serve_submit.argtypes = [vp, vp, C.c_uint32, C.c_uint32, vp, C.POINTER(C.c_uint32)]
        L.mpk_serve_run.argtypes = [vp, C.c_uint32, vp]
        L.mpk_serve_result.argtypes = [vp, C.c_uint32, vp, C.c_size_t, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        L.mpk_serve_state.argtypes = [vp, vp, C.c_size_t, C.POINTER(C.c_size_t)]
        L.mpk_serve_logits.argtypes = [vp]
        L.mpk_serve_logits.restype = vp
        L.mpk_serve_destroy.argtypes = [vp]
        L.mpk_serve_destroy.restype = None
        L.mpk_serve_create_set.argtypes = [vp, C.POINTER(ServeConfig), C.POINTER(vp)]
        L.mpk_serve_create_set.restype = C.c_int
        L.mpk_serve_last_batch.argtypes = [vp]
        L.mpk_serve_last_batch.restype = C.c_uint32
        L.mpk_serve_status.argtypes = [vp]
        L.mpk_serve_status.restype = C.c_int
        for n in SYMBOLS[:14] + ("mpk_graph_set_page_table", "mpk_serve_create", "mpk_serve_submit",
                                 "mpk_serve_run", "mpk_serve_result", "mpk_serve_state"):
            getattr(L, n).restype = C.c_int
        _lib = L
    return _lib


class MpkError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"mpk status {status}: {msg}")
        self.status = status


def _check(st):
    if st != MPK_OK:
        raise MpkError(st, lib().mpk_last_error().decode())


def model_config(shape) -> ModelConfig:
    """shape: any object with the ModelShape fields (synth.gen.ModelShape)."""
    return ModelConfig(C.sizeof(ModelConfig), shape.n_layers, shape.hidden, shape.n_q_heads,
                       shape.n_kv_heads, shape.head_dim, shape.ffn, shape.vocab, shape.rms_eps,
                       shape.rope_theta, shape.batch, shape.max_seq, shape.n_experts, shape.top_k,
                       shape.expert_ffn, 1 if getattr(shape, "qk_norm", False) else 0)


def compile_options(**kw) -> CompileOptions:
    o = CompileOptions()
    o.struct_size = C.sizeof(CompileOptions)
    for k, v in kw.items():
        if not hasattr(o, k):
            raise TypeError(k)
        if k == "worker_weight_permille":
            for i, x in enumerate(v):
                o.worker_weight_permille[i] = int(x)
        else:
            setattr(o, k, int(v))
    return o


class Export:
    """Parsed mpk_graph_export blob."""

    def __init__(self, blob: bytes):
        off = 0
        self.header = np.frombuffer(blob, EXPORT_HEADER, 1, off)[0]
        off += EXPORT_HEADER.itemsize
        h = self.header
        assert h["magic"] == 0x4B504D54
        self.ops = np.frombuffer(blob, EXPORT_OP, int(h["n_ops"]), off)
        off += EXPORT_OP.itemsize * int(h["n_ops"])
        self.tasks = np.frombuffer(blob, EXPORT_TASK, int(h["n_tasks"]), off)
        off += EXPORT_TASK.itemsize * int(h["n_tasks"])
        self.events = np.frombuffer(blob, EXPORT_EVENT, int(h["n_events"]), off)
        off += EXPORT_EVENT.itemsize * int(h["n_events"])
        nw = int(h["n_workers"])
        self.aot_off = np.frombuffer(blob, "<u4", nw + 1, off)
        off += 4 * (nw + 1)
        self.aot = np.frombuffer(blob, "<u4", int(self.aot_off[-1]), off)
        off += 4 * int(self.aot_off[-1])
        self.col_begin = {}          # operator index -> explicit column boundaries (tc + 1 of them)
        n_explicit = int(np.frombuffer(blob, "<u4", 1, off)[0])
        off += 4
        for _ in range(n_explicit):
            op, n = (int(x) for x in np.frombuffer(blob, "<u4", 2, off))
            off += 8
            self.col_begin[op] = np.frombuffer(blob, "<u4", n, off)
            off += 4 * n
        assert off == len(blob)


class Graph:
    """Owner of one mpk_graph handle."""

    def __init__(self, handle, keepalive=None):
        self._h = handle
        self._keep = keepalive

    def decode_step(self, token_ids_ptr: int, positions_ptr: int, logits_ptr: int, stream: int = 0):
        _check(lib().mpk_decode_step(self._h, token_ids_ptr, positions_ptr, logits_ptr, stream))

    def decode_step_static(self, token_ids_ptr: int, positions_ptr: int, logits_ptr: int, stream: int = 0):
        _check(lib().mpk_decode_step_static(self._h, token_ids_ptr, positions_ptr, logits_ptr, stream))

    def static_scratch_need(self) -> int:
        return int(lib().mpk_static_scratch_need(self._h))

    def decode_steps(self, n_steps: int, token_ids_ptr: int, positions_ptr: int, tokens_out_ptr: int,
                     logits_ptr: int, logits_all_ptr: int = 0, stream: int = 0):
        _check(lib().mpk_decode_steps(self._h, n_steps, token_ids_ptr, positions_ptr, tokens_out_ptr or None,
                                      logits_ptr, logits_all_ptr or None, stream))

    def set_page_table(self, page_table_ptr: int):
        _check(lib().mpk_graph_set_page_table(self._h, page_table_ptr))

    def serve(self, max_requests: int, max_prompt: int, max_new: int, eos_token: int = -1) -> "Server":
        cfg = ServeConfig(C.sizeof(ServeConfig), max_requests, max_prompt, max_new, eos_token)
        h = C.c_void_p()
        _check(lib().mpk_serve_create(self._h, C.byref(cfg), C.byref(h)))
        srv = Server(h, self)
        self._server = weakref.ref(srv)
        return srv

    def status(self):
        _check(lib().mpk_graph_status(self._h))

    def reset(self):
        _check(lib().mpk_graph_reset(self._h))

    def stats(self) -> dict:
        s = Stats()
        _check(lib().mpk_graph_stats(self._h, C.byref(s)))
        return s.as_dict()

    def export(self) -> Export:
        need = C.c_size_t(0)
        _check(lib().mpk_graph_export(self._h, None, 0, C.byref(need)))
        buf = C.create_string_buffer(need.value)
        _check(lib().mpk_graph_export(self._h, buf, need.value, C.byref(need)))
        return Export(buf.raw)

    def trace(self) -> np.ndarray:
        need = C.c_size_t(0)
        _check(lib().mpk_graph_trace(self._h, None, 0, C.byref(need)))
        buf = np.zeros(need.value, np.uint64)
        _check(lib().mpk_graph_trace(self._h, buf.ctypes.data, need.value, C.byref(need)))
        return buf.reshape(-1, 12)

    def moe_active(self) -> np.ndarray:
        need = C.c_size_t(0)
        _check(lib().mpk_graph_moe_active(self._h, None, 0, C.byref(need)))
        buf = np.zeros(need.value, np.uint32)
        _check(lib().mpk_graph_moe_active(self._h, buf.ctypes.data, need.value, C.byref(need)))
        return buf

    def moe_selection(self):
        """(experts u32 [layers][batch*top_k], weights f32 same shape) of the last step."""
        need = C.c_size_t(0)
        _check(lib().mpk_graph_moe_selection(self._h, None, None, 0, C.byref(need)))
        ex = np.zeros(need.value, np.uint32)
        wt = np.zeros(need.value, np.float32)
        _check(lib().mpk_graph_moe_selection(self._h, ex.ctypes.data, wt.ctypes.data, need.value,
                                             C.byref(need)))
        return ex, wt

    def destroy(self):
        srv = getattr(self, "_server", None)
        if srv is not None and srv() is not None:
            srv().destroy()          # (the library would destroy it with the graph: drop our handle first)
        if self._h:
            lib().mpk_graph_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class Server:
    """Owner of one mpk_server handle (destroyed before its graph)."""

    def __init__(self, handle, graph):
        self._h = handle
        self._graph = graph

    def submit(self, prompt, max_new_tokens: int, stream: int = 0) -> int:
        p = np.ascontiguousarray(np.asarray(prompt, dtype=np.int32).reshape(-1))
        rid = C.c_uint32(0)
        _check(lib().mpk_serve_submit(self._h, p.ctypes.data, len(p), max_new_tokens, stream, C.byref(rid)))
        return rid.value

    def run(self, n_iterations: int, stream: int = 0):
        _check(lib().mpk_serve_run(self._h, n_iterations, stream))

    def result(self, request_id: int):
        """(tokens produced so far, state: 0 queued / 1 running / 2 done)."""
        n, st = C.c_uint32(0), C.c_uint32(0)
        _check(lib().mpk_serve_result(self._h, request_id, None, 0, C.byref(n), C.byref(st)))
        buf = np.zeros(max(n.value, 1), np.int32)
        _check(lib().mpk_serve_result(self._h, request_id, buf.ctypes.data, len(buf), C.byref(n), C.byref(st)))
        return buf[:n.value].tolist(), st.value

    def state(self) -> dict:
        need = C.c_size_t(0)
        _check(lib().mpk_serve_state(self._h, None, 0, C.byref(need)))
        w = np.zeros(need.value, np.int32)
        _check(lib().mpk_serve_state(self._h, w.ctypes.data, need.value, C.byref(need)))
        B, M, n_free = int(w[0]), int(w[1]), int(w[2])
        o = 8
        out = {"n_free": n_free, "promised": int(w[3]), "q_head": int(w[4]), "q_tail": int(w[5]),
               "iterations": int(w[6]), "tokens_produced": int(w[7])}
        for name in ("slot_req", "slot_pos", "slot_held", "tokens", "positions"):
            out[name] = w[o:o + B].tolist()
            o += B
        out["table"] = w[o:o + B * M].reshape(B, M).tolist()
        o += B * M
        out["free"] = w[o:o + n_free].tolist()
        return out

    def logits_ptr(self) -> int:
        return int(lib().mpk_serve_logits(self._h) or 0)

    def last_batch(self) -> int:
        return int(lib().mpk_serve_last_batch(self._h))

    def status(self):
        _check(lib().mpk_serve_status(self._h))

    def destroy(self):
        if self._h:
            lib().mpk_serve_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class GraphSet:
    """Owner of one mpk_graph_set handle: a graph per power-of-two batch size up to shape.batch."""

    def __init__(self, handle, keepalive=None):
        self._h = handle
        self._keep = keepalive

    def __len__(self):
        return lib().mpk_set_size(self._h)

    def batch_for(self, n_active: int) -> int:
        return lib().mpk_set_batch_for(self._h, n_active)

    def graph(self, i: int) -> Graph:
        """Graph i of the set, borrowed: valid while the set lives, never destroyed through it."""
        h = lib().mpk_set_graph(self._h, i)
        if not h:
            raise IndexError(i)
        g = Graph(None, self)
        g._h = C.c_void_p(h)
        g.destroy = lambda: None
        return g

    def serve(self, max_requests: int, max_prompt: int, max_new: int, eos_token: int = -1) -> "Server":
        cfg = ServeConfig(C.sizeof(ServeConfig), max_requests, max_prompt, max_new, eos_token)
        h = C.c_void_p()
        _check(lib().mpk_serve_create_set(self._h, C.byref(cfg), C.byref(h)))
        srv = Server(h, self)
        self._server = weakref.ref(srv)
        return srv

    def decode_step(self, n_active: int, token_ids_ptr: int, positions_ptr: int, logits_ptr: int, stream: int = 0):
        _check(lib().mpk_set_decode_step(self._h, n_active, token_ids_ptr, positions_ptr, logits_ptr, stream))

    def destroy(self):
        srv = getattr(self, "_server", None)
        if srv is not None and srv() is not None:
            srv().destroy()
        if self._h:
            lib().mpk_set_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _marshal_model(shape, weights, kv):
    arr = (LayerWeights * shape.n_layers)()
    for l, lw in enumerate(weights["layers"]):
        for k, v in lw.items():
            setattr(arr[l], k, v)
    wp = WeightPtrs(weights["embed"], weights["final_norm"], weights["lm_head"], arr)
    kp = KvPtrs(kv[0], kv[1])
    return arr, wp, kp


def compile_set(shape, weights: dict, kv: tuple, **opts) -> GraphSet:
    """Graphs for batch 1, 2, 4, ... and shape.batch over one KV cache laid out for shape.batch."""
    cfg = model_config(shape)
    o = compile_options(**opts)
    h = C.c_void_p()
    arr, wp, kp = _marshal_model(shape, weights, kv)
    _check(lib().mpk_compile_set(C.byref(cfg), C.byref(wp), C.byref(kp), C.byref(o), C.byref(h)))
    return GraphSet(h, [arr, wp, kp])


def moe_task_share(n_active: int, tiles_per_expert: int, n_tasks: int, task: int) -> tuple:
    """Tiles [first, last) of the active experts' tiles that expert task `task` works on."""
    a, b = C.c_uint32(0), C.c_uint32(0)
    _check(lib().mpk_moe_task_share(n_active, tiles_per_expert, n_tasks, task, C.byref(a), C.byref(b)))
    return a.value, b.value


def compile_graph(shape, weights: dict | None, kv: tuple | None, **opts) -> Graph:
    """weights: {'embed': ptr, 'final_norm': ptr, 'lm_head': ptr, 'layers': [dict per layer with
    attn_norm, wqkv, wo, mlp_norm, wgu, wd]} of integer device addresses; kv: (k_ptr, v_ptr).
    Both may be None with host_only=1."""
    cfg = model_config(shape)
    o = compile_options(**opts)
    h = C.c_void_p()
    keep = []
    if weights is None:
        st = lib().mpk_compile(C.byref(cfg), None, None, C.byref(o), C.byref(h))
    else:
        arr = (LayerWeights * shape.n_layers)()
        for l, lw in enumerate(weights["layers"]):
            for k, v in lw.items():
                setattr(arr[l], k, v)
        wp = WeightPtrs(weights["embed"], weights["final_norm"], weights["lm_head"], arr)
        kp = KvPtrs(kv[0], kv[1])
        keep = [arr, wp, kp]
        st = lib().mpk_compile(C.byref(cfg), C.byref(wp), C.byref(kp), C.byref(o), C.byref(h))
    _check(st)
    return Graph(h, keep)


def compile_dag(n_tasks: int, pairs, **opts) -> Graph:
    p = np.ascontiguousarray(np.asarray(pairs, dtype=np.uint32).reshape(-1, 2))
    o = compile_options(**opts)
    h = C.c_void_p()
    _check(lib().mpk_compile_dag(n_tasks, p.ctypes.data, len(p), C.byref(o), C.byref(h)))
    return Graph(h)
