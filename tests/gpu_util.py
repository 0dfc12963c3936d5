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
