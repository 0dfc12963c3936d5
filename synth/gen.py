"""Seeded synthetic inputs shared by the CPU oracle and the GPU harness.

Only input data lives here (shapes of the benchmark configurations, tensor ids, the counter-based
value generator).  No decoder arithmetic, no task-graph logic.

Value recipe: element i of tensor `tid` under `seed` = table[mix64(seed, tid, i) >> 48], where
`table` holds the 65,536 quantiles  q_j = F^-1((j + 1/2) / 65536)  of the wanted distribution
rounded to bf16 (round-to-nearest-even).  Three tables are used:
  normal(0.02)  : linear weights and the embedding table
  normal(1.0)   : prior KV-cache rows
  gain(0.02)    : RMSNorm gains, 1 + 0.02 z
"""
from __future__ import annotations

import ctypes
import functools
import hashlib
import os
import subprocess
from dataclasses import dataclass, asdict

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
M64 = (1 << 64) - 1


# ----------------------------------------------------------------------------- configurations
@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float
    rope_theta: float
    batch: int
    max_seq: int
    n_experts: int = 0
    top_k: int = 0
    expert_ffn: int = 0
    qk_norm: bool = False    # per-head RMSNorm of q and k before RoPE (Qwen3)
    # workload
    kv_len_lo: int = 0       # prior cached positions per sequence: uniform integer in [lo, hi]
    kv_len_hi: int = 0
    steps: int = 1

    def as_dict(self):
        return asdict(self)


CONFIGS = {
    # tiny decoder, one step
    "C1": ModelShape("C1-tiny", 2, 256, 4, 2, 64, 688, 1024, 1e-6, 1e4, 1, 192,
                     kv_len_lo=128, kv_len_hi=128, steps=1),
    # Qwen3-8B-shaped, batch 1
    "C2": ModelShape("C2-qwen3-8b-shaped", 36, 4096, 32, 8, 128, 12288, 151936, 1e-6, 1e6, 1,
                     1088, kv_len_lo=1024, kv_len_hi=1024, steps=32),
    # Llama-3-8B-shaped, batch 8, ragged KV lengths
    "C3": ModelShape("C3-llama3-8b-shaped", 32, 4096, 32, 8, 128, 14336, 128256, 1e-6, 5e5, 8,
                     4160, kv_len_lo=512, kv_len_hi=4096, steps=32),
    # Qwen3-30B-A3B-shaped MoE, batch 16
    "C4": ModelShape("C4-qwen3-30b-a3b-shaped", 48, 2048, 32, 4, 128, 0, 151936, 1e-6, 1e6, 16,
                     2112, n_experts=128, top_k=8, expert_ffn=768,
                     kv_len_lo=2048, kv_len_hi=2048, steps=8),
    # Llama-3-70B-shaped, batch 1
    "C5": ModelShape("C5-llama3-70b-shaped", 80, 8192, 64, 8, 128, 28672, 128256, 1e-6, 5e5, 1,
                     2112, kv_len_lo=2048, kv_len_hi=2048, steps=16),
}


def small_variant(base: str, **kw) -> ModelShape:
    """A config with some fields replaced (used for reduced-size parity cases)."""
    d = CONFIGS[base].as_dict()
    d.update(kw)
    return ModelShape(**d)


# ----------------------------------------------------------------------------- tensor ids
TID_EMBED, TID_FINAL_NORM, TID_LM_HEAD, TID_TOKENS, TID_KVLEN = 1, 2, 3, 4, 5
(L_ATTN_NORM, L_WQKV, L_WO, L_MLP_NORM, L_WGU, L_WD, L_ROUTER, L_EXP_WGU, L_EXP_WD,
 L_KCACHE, L_VCACHE, L_QNORM, L_KNORM) = range(13)


def layer_tid(layer: int, which: int) -> int:
    return 1000 + layer * 16 + which


def layer_tensor_shapes(s: ModelShape):
    """(which, rows, cols, table) for every per-layer weight tensor, row-major [rows, cols]."""
    qkv_rows = (s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim
    out = [(L_ATTN_NORM, 1, s.hidden, "gain"),
           (L_WQKV, qkv_rows, s.hidden, "w"),
           (L_WO, s.hidden, s.n_q_heads * s.head_dim, "w"),
           (L_MLP_NORM, 1, s.hidden, "gain")]
    if s.qk_norm:
        out += [(L_QNORM, 1, s.head_dim, "gain"), (L_KNORM, 1, s.head_dim, "gain")]
    if s.n_experts == 0:
        out += [(L_WGU, 2 * s.ffn, s.hidden, "w"), (L_WD, s.hidden, s.ffn, "w")]
    else:
        out += [(L_ROUTER, s.n_experts, s.hidden, "w"),
                (L_EXP_WGU, s.n_experts * 2 * s.expert_ffn, s.hidden, "w"),
                (L_EXP_WD, s.n_experts * s.hidden, s.expert_ffn, "w")]
    return out


# ----------------------------------------------------------------------------- the hash
def mix64(seed: int, tid: int, i):
    """splitmix64 output function on seed*C1 + tid*C2 + i (all mod 2^64).  i: int or ndarray."""
    base = (seed * 0x9E3779B97F4A7C15 + tid * 0xD1B54A32D192ED03) & M64
    with np.errstate(over="ignore"):
        z = np.asarray(i, dtype=np.uint64) + np.uint64(base)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


@functools.lru_cache(maxsize=None)
def table(kind: str) -> np.ndarray:
    """65,536 bf16 bit patterns.  kind: 'w' N(0,0.02), 'kv' N(0,1), 'gain' 1+N(0,0.02),
    'gain_literal' N(0,0.02) (the literal reading of 'weights ~N(0,0.02)' for norm gains)."""
    from scipy.special import ndtri
    z = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
    if kind in ("w", "gain_literal"):
        v = 0.02 * z
    elif kind == "kv":
        v = z
    elif kind == "gain":
        v = 1.0 + 0.02 * z
    else:
        raise ValueError(kind)
    # fp64 -> fp32 -> bf16 (double rounding is irrelevant here: the table *defines* the values)
    t = f32_to_bf16_bits(v.astype(np.float32))
    t.setflags(write=False)
    return t


def table_digest(kind: str) -> str:
    return hashlib.sha256(table(kind).tobytes()).hexdigest()[:16]


def fill_numpy(seed: int, tid: int, i0: int, n: int, kind: str) -> np.ndarray:
    """Reference (slow) generator: bf16 bit patterns of elements [i0, i0+n)."""
    idx = (mix64(seed, tid, np.arange(i0, i0 + n, dtype=np.uint64)) >> np.uint64(48))
    return table(kind)[idx.astype(np.int64)]


# ----------------------------------------------------------------------------- C fast path
def _build(src, out, cmd):
    if (not os.path.exists(out)) or os.path.getmtime(out) < os.path.getmtime(src):
        subprocess.check_call(cmd)
    return out


def build_cpu(force=False) -> str:
    src = os.path.join(_HERE, "synth_cpu.c")
    out = os.path.join(_HERE, "libsynth_cpu.so")
    if force and os.path.exists(out):
        os.remove(out)
    return _build(src, out, ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", out, src])


def build_hip(force=False) -> str:
    src = os.path.join(_HERE, "synth_hip.hip")
    out = os.path.join(_HERE, "libsynth_hip.so")
    if force and os.path.exists(out):
        os.remove(out)
    return _build(src, out, ["hipcc", "--offload-arch=gfx950", "-O3", "-shared", "-fPIC",
                             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                             "-o", out, src])


@functools.lru_cache(maxsize=None)
def _cpu_lib():
    lib = ctypes.CDLL(build_cpu())
    lib.synth_fill_bf16.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64,
                                    ctypes.c_uint64, ctypes.c_uint64, ctypes.c_void_p]
    lib.synth_fill_bf16.restype = None
    lib.synth_hash.argtypes = [ctypes.c_uint64] * 3
    lib.synth_hash.restype = ctypes.c_uint64
    return lib


def fill_host(seed: int, tid: int, i0: int, n: int, kind: str, out: np.ndarray | None = None):
    """Fast host generator (C, OpenMP).  Returns uint16 bf16 bit patterns."""
    if out is None:
        out = np.empty(n, dtype=np.uint16)
    assert out.dtype == np.uint16 and out.size >= n and out.flags.c_contiguous
    t = table(kind)
    _cpu_lib().synth_fill_bf16(out.ctypes.data, seed, tid, i0, n, t.ctypes.data)
    return out


@functools.lru_cache(maxsize=None)
def _hip_lib():
    lib = ctypes.CDLL(build_hip())
    lib.synth_fill_bf16_device.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64,
                                           ctypes.c_uint64, ctypes.c_uint64, ctypes.c_void_p,
                                           ctypes.c_void_p]
    lib.synth_fill_bf16_device.restype = ctypes.c_int
    lib.synth_copy_device.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64,
                                      ctypes.c_void_p]
    lib.synth_copy_device.restype = ctypes.c_int
    return lib


_dev_tables = {}


def fill_device(t, seed: int, tid: int, i0: int = 0, kind: str = "w"):
    """Fill a contiguous torch bf16 (or int16) CUDA tensor in place on the current stream."""
    import torch
    assert t.is_cuda and t.is_contiguous() and t.element_size() == 2
    key = (kind, t.device.index)
    if key not in _dev_tables:
        _dev_tables[key] = torch.from_numpy(table(kind).view(np.int16).copy()).to(t.device)
    rc = _hip_lib().synth_fill_bf16_device(t.data_ptr(), seed, tid, i0, t.numel(),
                                           _dev_tables[key].data_ptr(),
                                           torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError(f"synth_fill_bf16_device: hip error {rc}")
    return t


def copy_device(dst, src):
    """Plain device copy kernel of known traffic (reads and writes dst.nbytes once each)."""
    import torch
    assert dst.is_cuda and src.is_cuda and dst.is_contiguous() and src.is_contiguous()
    n = dst.numel() * dst.element_size()
    assert n == src.numel() * src.element_size()
    rc = _hip_lib().synth_copy_device(dst.data_ptr(), src.data_ptr(), n,
                                      torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError(f"synth_copy_device: error {rc}")


# ----------------------------------------------------------------------------- workload pieces
def tokens(seed: int, s: ModelShape) -> np.ndarray:
    return (mix64(seed, TID_TOKENS, np.arange(s.batch, dtype=np.uint64))
            % np.uint64(s.vocab)).astype(np.int32)


def kv_lengths(seed: int, s: ModelShape) -> np.ndarray:
    span = s.kv_len_hi - s.kv_len_lo + 1
    return (s.kv_len_lo + (mix64(seed, TID_KVLEN, np.arange(s.batch, dtype=np.uint64))
                           % np.uint64(span))).astype(np.int32)


def kv_layer_numel(s: ModelShape) -> int:
    return s.batch * s.n_kv_heads * s.max_seq * s.head_dim


def host_layer_weights(seed: int, s: ModelShape, layer: int, gain_kind="gain") -> dict:
    """All weight tensors of one layer as uint16 arrays shaped [rows, cols]."""
    out = {}
    for which, rows, cols, kind in layer_tensor_shapes(s):
        k = gain_kind if kind == "gain" else kind
        out[which] = fill_host(seed, layer_tid(layer, which), 0, rows * cols, k).reshape(rows, cols)
    return out


def host_kv_layer(seed: int, s: ModelShape, layer: int):
    """Prior K and V cache of one layer, physical layout [B][n_kv][max_seq][d] (all rows filled;
    rows at or beyond a sequence's length are overwritten before they are ever read)."""
    n = kv_layer_numel(s)
    shp = (s.batch, s.n_kv_heads, s.max_seq, s.head_dim)
    k = fill_host(seed, layer_tid(layer, L_KCACHE), 0, n, "kv").reshape(shp)
    v = fill_host(seed, layer_tid(layer, L_VCACHE), 0, n, "kv").reshape(shp)
    return k, v


class SynthWeights:
    """Host-side provider of the seeded tensors of one model (bf16 bit patterns as uint16).

    cache=True keeps every generated tensor (fine up to the 8B shapes on a 64 GB host);
    cache=False regenerates a layer each time it is asked for (70B shape)."""

    def __init__(self, shape: ModelShape, seed: int = 0, cache: bool = True,
                 gain_kind: str = "gain"):
        self.s, self.seed, self.cache, self.gain_kind = shape, seed, cache, gain_kind
        self._layers, self._misc = {}, {}

    def embed_row(self, token: int) -> np.ndarray:
        h = self.s.hidden
        return fill_host(self.seed, TID_EMBED, int(token) * h, h, "w")

    def layer(self, l: int) -> dict:
        if l in self._layers:
            return self._layers[l]
        w = host_layer_weights(self.seed, self.s, l, self.gain_kind)
        if self.cache:
            self._layers[l] = w
        return w

    def final_norm(self) -> np.ndarray:
        if "fn" not in self._misc:
            self._misc["fn"] = fill_host(self.seed, TID_FINAL_NORM, 0, self.s.hidden,
                                         self.gain_kind)
        return self._misc["fn"]

    def lm_head(self) -> np.ndarray:
        if "lm" in self._misc:
            return self._misc["lm"]
        w = fill_host(self.seed, TID_LM_HEAD, 0, self.s.vocab * self.s.hidden, "w").reshape(
            self.s.vocab, self.s.hidden)
        if self.cache:
            self._misc["lm"] = w
        return w

    def kv_layer(self, l: int):
        return host_kv_layer(self.seed, self.s, l)


# ----------------------------------------------------------------------------- paged KV cache
# Input provisioning for the paged layout: which page every (sequence, block of page_size rows)
# lives in, and the seeded contiguous cache re-filed into pages.  No arithmetic of the method.
BF16_NAN_BITS = 0x7FC0


def page_table(seed: int, s: ModelShape, page_size: int, n_pages: int, rows) -> np.ndarray:
    """int32 [B][max_seq // page_size]: sequence b gets a page of its own, drawn from a seeded
    shuffle of all pages, for every block that holds one of its first rows[b] rows; the other
    entries are -1."""
    nb = s.max_seq // page_size
    need = [-(-int(r) // page_size) for r in rows]
    assert sum(need) <= n_pages and max(need) <= nb
    perm = np.random.default_rng(seed).permutation(n_pages)
    t = np.full((s.batch, nb), -1, np.int32)
    k = 0
    for b in range(s.batch):
        for i in range(need[b]):
            t[b, i] = perm[k]
            k += 1
    return t


def paginate(cache: np.ndarray, table: np.ndarray, page_size: int, n_pages: int) -> np.ndarray:
    """cache uint16 [B][n_kv][max_seq][d] -> pool uint16 [n_pages][n_kv][page_size][d]; pages no
    table entry names hold NaN patterns."""
    B, nkv, _, d = cache.shape
    pool = np.full((n_pages, nkv, page_size, d), BF16_NAN_BITS, np.uint16)
    for b in range(B):
        for i, pg in enumerate(table[b]):
            if pg >= 0:
                pool[pg] = cache[b, :, i * page_size:(i + 1) * page_size, :]
    return pool


class PagedWeights(SynthWeights):
    """SynthWeights whose prior cache is handed out in pages (kv_pool) under a given table."""

    def __init__(self, shape, seed, table, page_size, n_pages, **kw):
        super().__init__(shape, seed, **kw)
        self.table, self.page_size, self.n_pages = np.asarray(table), page_size, n_pages

    def kv_pool(self, l: int):
        k, v = host_kv_layer(self.seed, self.s, l)
        return (paginate(k, self.table, self.page_size, self.n_pages),
                paginate(v, self.table, self.page_size, self.n_pages))
