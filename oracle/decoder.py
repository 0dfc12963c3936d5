"""TEST INFRASTRUCTURE -- Python driver of the CPU decoder oracle (oracle/decoder_oracle.c).

Runs the operator sequence of one decode step exactly as listed in the target description:
embedding, then per layer RMSNorm, QKV projection, RoPE, decode attention over the KV cache,
O projection, residual, RMSNorm, SwiGLU MLP (or top-k MoE), residual; then final RMSNorm and the
LM head; greedy next token = arg max (lowest index on ties).  The paper (Section 6.2) only says
the models are the public bf16 decoder architectures; the numeric definition of each operator is
the textbook one and lives in the C file.

Nothing here is imported by the GPU library; only tests, smoke() and bench.py's cpu_baseline leg
use it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))


def build(force: bool = False):
    """Compile the C oracle in both precisions.  Returns {'f32': path, 'f64': path}."""
    src = os.path.join(_HERE, "decoder_oracle.c")
    outs = {}
    for prec, flag in (("f32", []), ("f64", ["-DORC_F64"])):
        out = os.path.join(_HERE, f"liboracle_{prec}.so")
        if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
            subprocess.check_call(["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-shared",
                                   "-fPIC", *flag, "-o", out, src, "-lm"])
        outs[prec] = out
    return outs


class _LayerCfg(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int), ("n_q", ctypes.c_int), ("n_kv", ctypes.c_int),
                ("d", ctypes.c_int), ("ffn", ctypes.c_int), ("max_seq", ctypes.c_int),
                ("eps", ctypes.c_float), ("theta", ctypes.c_double),
                ("n_experts", ctypes.c_int), ("top_k", ctypes.c_int),
                ("expert_ffn", ctypes.c_int), ("qk_norm", ctypes.c_int)]


class _LayerW(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("attn_norm", "wqkv", "wo", "mlp_norm", "wgu", "wd", "router", "exp_wgu",
                 "exp_wd", "q_norm", "k_norm")]


class _Held(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("k_rows", "v_rows", "experts", "k_exact", "v_exact")]


class Held:
    """Discrete decisions of one decode step held fixed for the oracle (see orc_held in the C
    file): the bf16 K/V rows appended by every (layer, sequence) and, for mixture-of-experts
    layers, the selected expert sets.  Shapes: k_rows, v_rows uint16 [L][B][n_kv][d]; experts
    int32 [L][B][top_k] ascending.  Either may be None."""

    def __init__(self, k_rows=None, v_rows=None, experts=None):
        self.k_rows = None if k_rows is None else np.ascontiguousarray(k_rows, dtype=np.uint16)
        self.v_rows = None if v_rows is None else np.ascontiguousarray(v_rows, dtype=np.uint16)
        self.experts = None if experts is None else np.ascontiguousarray(experts, dtype=np.int32)


_libs = {}


def lib(prec: str = "f32"):
    if prec not in _libs:
        L = ctypes.CDLL(build()[prec])
        vp, ci = ctypes.c_void_p, ctypes.c_int
        L.orc_real_bytes.restype = ci
        L.orc_threads.restype = ci
        L.orc_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.orc_bf16_to_f32.restype = ctypes.c_float
        L.orc_f32_to_bf16.argtypes = [ctypes.c_float]
        L.orc_f32_to_bf16.restype = ctypes.c_uint16
        L.orc_embed.argtypes = [vp, ci, ci, vp]
        L.orc_rmsnorm.argtypes = [vp, vp, ci, ctypes.c_float, vp]
        L.orc_linear.argtypes = [vp, ci, ci, vp, vp]
        L.orc_rope.argtypes = [vp, ci, ci, ctypes.c_double]
        L.orc_kv_store.argtypes = [vp, vp, ci]
        L.orc_attention_head.argtypes = [vp, vp, vp, ci, ci, vp, vp]
        L.orc_swiglu.argtypes = [vp, ci, vp]
        L.orc_add.argtypes = [vp, vp, ci, vp]
        L.orc_argmax.argtypes = [vp, ci]
        L.orc_argmax.restype = ci
        L.orc_router_topk.argtypes = [vp, ci, ci, vp, vp]
        L.orc_layer.argtypes = [ctypes.POINTER(_LayerCfg), ctypes.POINTER(_LayerW), vp, vp, ci,
                                vp, vp, vp, vp, ctypes.POINTER(_Held)]
        for f in ("orc_embed", "orc_rmsnorm", "orc_linear", "orc_rope", "orc_kv_store",
                  "orc_attention_head", "orc_swiglu", "orc_add", "orc_router_topk", "orc_layer"):
            getattr(L, f).restype = None
        _libs[prec] = L
    return _libs[prec]


def _p(a: np.ndarray):
    assert a.flags.c_contiguous
    return a.ctypes.data


class Ops:
    """Thin numpy front end over the C functions (one precision)."""

    def __init__(self, prec: str = "f32"):
        self.L = lib(prec)
        self.dt = np.float32 if prec == "f32" else np.float64
        assert self.L.orc_real_bytes() == np.dtype(self.dt).itemsize

    def _r(self, a):
        return np.ascontiguousarray(a, dtype=self.dt)

    def embed(self, E, token):
        E = np.ascontiguousarray(E, dtype=np.uint16)
        x = np.empty(E.shape[1], self.dt)
        self.L.orc_embed(_p(E), E.shape[1], int(token), _p(x))
        return x

    def rmsnorm(self, x, g, eps):
        x = self._r(x)
        g = np.ascontiguousarray(g, dtype=np.uint16).reshape(-1)
        y = np.empty_like(x)
        self.L.orc_rmsnorm(_p(x), _p(g), x.size, eps, _p(y))
        return y

    def linear(self, W, x):
        W = np.ascontiguousarray(W, dtype=np.uint16)
        x = self._r(x)
        assert W.shape[1] == x.size
        y = np.empty(W.shape[0], self.dt)
        self.L.orc_linear(_p(W), W.shape[0], W.shape[1], _p(x), _p(y))
        return y

    def rope(self, u, pos, theta):
        u = self._r(u).copy()
        self.L.orc_rope(_p(u), u.size, int(pos), float(theta))
        return u

    def kv_store(self, u):
        u = self._r(u)
        row = np.empty(u.size, np.uint16)
        self.L.orc_kv_store(_p(row), _p(u), u.size)
        return row

    def attention_head(self, q, K, V, n_pos):
        q = self._r(q)
        K = np.ascontiguousarray(K, dtype=np.uint16)
        V = np.ascontiguousarray(V, dtype=np.uint16)
        d = q.size
        assert K.shape[1] == d and V.shape[1] == d and K.shape[0] >= n_pos
        scr = np.empty(n_pos, self.dt)
        o = np.empty(d, self.dt)
        self.L.orc_attention_head(_p(q), _p(K), _p(V), int(n_pos), d, _p(scr), _p(o))
        return o

    def swiglu(self, gu):
        gu = self._r(gu)
        F = gu.size // 2
        h = np.empty(F, self.dt)
        self.L.orc_swiglu(_p(gu), F, _p(h))
        return h

    def add(self, a, b):
        a, b = self._r(a), self._r(b)
        y = np.empty_like(a)
        self.L.orc_add(_p(a), _p(b), a.size, _p(y))
        return y

    def argmax(self, x):
        x = self._r(x)
        return int(self.L.orc_argmax(_p(x), x.size))

    def router_topk(self, logits, k):
        logits = self._r(logits)
        sel = np.empty(k, np.int32)
        w = np.empty(k, self.dt)
        self.L.orc_router_topk(_p(logits), logits.size, k, _p(sel), _p(w))
        return sel, w


class DecoderOracle:
    """One model instance: weights from a provider, host KV cache, greedy stepping.

    provider interface (all arrays uint16 bf16 bit patterns):
      embed_row(token) -> [hidden];  layer(l) -> dict {which: [rows, cols]} keyed as in
      synth.gen (L_ATTN_NORM ...);  final_norm() -> [hidden];  lm_head() -> [vocab, hidden];
      kv_layer(l) -> (K, V) each [B][n_kv][max_seq][d] (prior cache; copied, then owned here).
    """

    def __init__(self, shape, provider, prec: str = "f32", n_layers: int | None = None):
        self.s = shape
        self.p = provider
        self.ops = Ops(prec)
        self.dt = self.ops.dt
        self.n_layers = shape.n_layers if n_layers is None else n_layers
        self.kv = {}
        self.last_moe_sel = None      # [layers, B, top_k] selected experts of the last step
        self.last_moe_logits = None   # [layers, B, n_experts] router outputs of the last step

    def _kv(self, l):
        if l not in self.kv:
            k, v = self.p.kv_layer(l)
            self.kv[l] = (np.ascontiguousarray(k).copy(), np.ascontiguousarray(v).copy())
        return self.kv[l]

    def _rows_in(self, l, b, K, V, pos):
        """The cache of sequence b in layer l as the layer function wants it: [n_kv][max_seq][d]
        with rows 0..pos-1 valid; it writes row pos.  Here the cache is stored that way."""
        return K[b], V[b]

    def _rows_out(self, l, b, Kb, Vb, pos):
        """Called after the layer function appended row pos to (Kb, Vb): nothing to put back."""

    def step(self, tokens, positions, return_hidden=False, held: "Held | None" = None):
        """tokens[B], positions[B] (= rows already cached).  Returns logits [B, vocab].
        held: decisions to hold fixed (class Held).  After the call last_k_exact / last_v_exact
        hold the oracle's own K/V rows of this step before rounding, [L][B][n_kv][d]."""
        s, L = self.s, self.ops.L
        B = len(tokens)
        ffn_like = max(s.ffn, s.expert_ffn)
        qkv_rows = (s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim
        work = np.empty(6 * s.hidden + 2 * qkv_rows + 4 * ffn_like + s.max_seq
                        + max(s.n_experts, 1) + 64, self.dt)
        cfg = _LayerCfg(s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn, s.max_seq,
                        s.rms_eps, s.rope_theta, s.n_experts, s.top_k, s.expert_ffn,
                        int(getattr(s, "qk_norm", False)))
        xs = [self.ops.embed(self.p.embed_row(int(t)).reshape(1, -1), 0) for t in tokens]
        moe_sel = np.zeros((self.n_layers, B, max(s.top_k, 1)), np.int32)
        moe_logits = np.zeros((self.n_layers, B, max(s.n_experts, 1)), self.dt)
        k_exact = np.zeros((self.n_layers, B, s.n_kv_heads, s.head_dim), self.dt)
        v_exact = np.zeros_like(k_exact)
        from synth import gen as G
        for l in range(self.n_layers):
            wl = self.p.layer(l)
            keep = [np.ascontiguousarray(a) for a in wl.values()]  # keep alive during the call

            def ptr(which):
                a = wl.get(which)
                return None if a is None else np.ascontiguousarray(a).ctypes.data
            w = _LayerW(ptr(G.L_ATTN_NORM), ptr(G.L_WQKV), ptr(G.L_WO), ptr(G.L_MLP_NORM),
                        ptr(G.L_WGU), ptr(G.L_WD), ptr(G.L_ROUTER), ptr(G.L_EXP_WGU),
                        ptr(G.L_EXP_WD), ptr(G.L_QNORM), ptr(G.L_KNORM))
            K, V = self._kv(l)
            for b in range(B):
                assert 0 <= positions[b] < s.max_seq
                Kb, Vb = self._rows_in(l, b, K, V, int(positions[b]))
                h = _Held(None, None, None, k_exact[l, b].ctypes.data, v_exact[l, b].ctypes.data)
                if held is not None and held.k_rows is not None:
                    h.k_rows = held.k_rows[l, b].ctypes.data
                if held is not None and held.v_rows is not None:
                    h.v_rows = held.v_rows[l, b].ctypes.data
                if held is not None and held.experts is not None:
                    h.experts = held.experts[l, b].ctypes.data
                L.orc_layer(ctypes.byref(cfg), ctypes.byref(w), Kb.ctypes.data,
                            Vb.ctypes.data, int(positions[b]), _p(xs[b]), _p(work),
                            moe_sel[l, b].ctypes.data, moe_logits[l, b].ctypes.data, ctypes.byref(h))
                self._rows_out(l, b, Kb, Vb, int(positions[b]))
            del keep
        self.last_moe_sel = moe_sel
        self.last_moe_logits = moe_logits
        self.last_k_exact, self.last_v_exact = k_exact, v_exact
        if return_hidden:
            return np.stack(xs)
        g = self.p.final_norm()
        Wlm = self.p.lm_head()
        logits = np.stack([self.ops.linear(Wlm, self.ops.rmsnorm(x, g, s.rms_eps)) for x in xs])
        return logits

    def greedy(self, tokens, positions, n_steps):
        """Free-running greedy decode.  Returns (tokens[n_steps, B], logits list)."""
        toks = np.array(tokens, np.int64)
        pos = np.array(positions, np.int64)
        out_t, out_l = [], []
        for _ in range(n_steps):
            lg = self.step(toks, pos)
            toks = np.array([self.ops.argmax(lg[b]) for b in range(len(toks))], np.int64)
            pos = pos + 1
            out_t.append(toks.copy())
            out_l.append(lg)
        return np.stack(out_t), out_l
