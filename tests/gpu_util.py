"""GPU-side helpers for the parity tests: device model + compiled graph + stepping."""
import numpy as np
import torch

import paper_2512_22219_amd as M
from synth import gen as G
from synth.device import DeviceModel


def rel_err(gpu: np.ndarray, ref: np.ndarray) -> float:
    """max_i |gpu_i - ref_i| / max(|ref_i|, 1e-3 * max|ref|): the tolerance metric of the target
    ("max relative error 2e-2"), with a floor so near-zero logits do not blow it up."""
    ref = ref.astype(np.float64)
    denom = np.maximum(np.abs(ref), 1e-3 * np.abs(ref).max())
    return float((np.abs(gpu.astype(np.float64) - ref) / denom).max())


class GpuDecoder:
    def __init__(self, shape, seed=0, model=None, **opts):
        self.s = shape
        self.model = model if model is not None else DeviceModel(shape, seed)
        self.graph = M.compile_graph(shape, self.model.weight_ptrs(), self.model.kv_ptrs(), **opts)
        dev = self.model.device
        self.tok = torch.zeros(shape.batch, dtype=torch.int32, device=dev)
        self.pos = torch.zeros(shape.batch, dtype=torch.int32, device=dev)
        self.logits = torch.empty((shape.batch, shape.vocab), dtype=torch.float32, device=dev)

    def step(self, tokens, positions) -> np.ndarray:
        self.tok.copy_(torch.as_tensor(np.asarray(tokens, np.int32)))
        self.pos.copy_(torch.as_tensor(np.asarray(positions, np.int32)))
        self.logits.fill_(float("nan"))
        stream = torch.cuda.current_stream().cuda_stream
        self.graph.decode_step(self.tok.data_ptr(), self.pos.data_ptr(), self.logits.data_ptr(), stream)
        torch.cuda.synchronize()
        self.graph.status()
        return self.logits.cpu().numpy()

    def close(self):
        self.graph.destroy()


# ---------------------------------------------------------------- held decisions
# Two places of a decode step turn floating point into something discrete: the bf16 rounding of
# the appended K/V rows and the top-k expert sets.  Implementations that sum in different orders
# may take such a decision either way when the value sits on the boundary, and everything after
# it then differs legitimately.  The strict comparisons below hand the GPU's decisions to the
# oracle (oracle.decoder.Held), check each of them against what the oracle computed itself, and
# compare the logits element by element with both sides on the same decisions.

def bf16_bits_to_f64(u16: np.ndarray) -> np.ndarray:
    return (u16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def appended_rows(model, positions):
    """The K and V rows a step wrote at positions[b]: uint16 [L][B][n_kv][d] each."""
    B = len(positions)
    idx = torch.as_tensor(np.asarray(positions, np.int64), device=model.device)
    bb = torch.arange(B, device=model.device)
    out = []
    for cache in (model.k, model.v):
        rows = cache[:, bb, :, idx, :]                 # advanced indices first: [B][L][n_kv][d]
        rows = rows.permute(1, 0, 2, 3).contiguous()
        out.append(rows.view(torch.int16).cpu().numpy().view(np.uint16))
    return out


def check_rows_are_valid_roundings(rows_u16, exact, tol_rel=3e-5):
    """Every appended element must be the bf16 rounding (to nearest) of a value within tol_rel x
    the head vector's largest magnitude of the oracle's unrounded value.  Returns the number of
    elements that differ from the oracle's own rounding (boundary cases taken the other way)."""
    r = bf16_bits_to_f64(rows_u16)
    e = np.asarray(exact, np.float64)
    scale = np.abs(e).max(axis=-1, keepdims=True)
    mag = np.maximum(np.abs(r), np.finfo(np.float32).tiny)
    half_ulp = 2.0 ** (np.floor(np.log2(mag)) - 8)     # bf16 keeps 8 significand bits
    bad = np.abs(r - e) > half_ulp + tol_rel * scale
    assert not bad.any(), (int(bad.sum()), float(np.abs(r - e)[bad].max()))
    own = (np.asarray(exact, np.float32).view(np.uint32).astype(np.uint64))
    own = ((own + 0x7FFF + ((own >> 16) & 1)) >> 16).astype(np.uint16)   # round to nearest even
    return int((own != rows_u16).sum())


def check_experts_are_valid(experts, router_out, margin_rel=1e-4):
    """A held expert set is valid when none of its members scores below the oracle's top_k-th
    router output by more than margin_rel x the spread of that token's router outputs.  Returns
    the number of (layer, token) sets that differ from the oracle's own choice."""
    ro = np.asarray(router_out, np.float64)                       # [L][B][E]
    k = experts.shape[-1]
    kth = np.sort(ro, axis=-1)[..., -k]                           # the k-th largest
    spread = ro.max(-1) - ro.min(-1)
    chosen = np.take_along_axis(ro, experts.astype(np.int64), axis=-1)
    assert (chosen.min(-1) >= kth - margin_rel * spread).all()
    assert (np.diff(experts, axis=-1) > 0).all()
    own = np.sort(np.argsort(-ro, axis=-1, kind="stable")[..., :k], axis=-1)
    return int((own != experts).any(-1).sum())


def held_step(ref, gpu, tokens, positions):
    """One step on the GPU, then the same step on the oracle `ref` with the GPU's discrete
    decisions held.  Returns (gpu logits, oracle logits, flipped K/V elements, differing sets)."""
    from oracle.decoder import Held
    got = gpu.step(tokens, positions)
    k_rows, v_rows = appended_rows(gpu.model, positions)
    experts = None
    if gpu.s.n_experts:
        ex, _ = gpu.graph.moe_selection()
        experts = ex.reshape(gpu.s.n_layers, gpu.s.batch, gpu.s.top_k).astype(np.int32)
    want = ref.step(tokens, positions, held=Held(k_rows, v_rows, experts))
    flips = check_rows_are_valid_roundings(k_rows, ref.last_k_exact)
    flips += check_rows_are_valid_roundings(v_rows, ref.last_v_exact)
    sets = check_experts_are_valid(experts, ref.last_moe_logits) if experts is not None else 0
    return got, want, flips, sets
