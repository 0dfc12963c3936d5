"""Device-side seeded inputs: allocates torch tensors in HBM and fills them with the same
counter-based generator as the host side (synth/synth_hip.hip).  Input provisioning only."""
from __future__ import annotations

import numpy as np
import torch

from . import gen as G


class DeviceModel:
    """All weights and the KV cache of one synthetic model, resident on one GPU."""

    def __init__(self, shape: G.ModelShape, seed: int = 0, device="cuda:0", gain_kind="gain"):
        s = self.s = shape
        self.seed = seed
        dev = self.device = torch.device(device)
        bf = torch.bfloat16

        def new(tid, rows, cols, kind):
            t = torch.empty((rows, cols), dtype=bf, device=dev)
            G.fill_device(t, seed, tid, 0, gain_kind if kind == "gain" else kind)
            return t

        self.embed = new(G.TID_EMBED, s.vocab, s.hidden, "w")
        self.final_norm = new(G.TID_FINAL_NORM, 1, s.hidden, "gain")
        self.lm_head = new(G.TID_LM_HEAD, s.vocab, s.hidden, "w")
        names = {G.L_ATTN_NORM: "attn_norm", G.L_WQKV: "wqkv", G.L_WO: "wo",
                 G.L_MLP_NORM: "mlp_norm", G.L_WGU: "wgu", G.L_WD: "wd", G.L_ROUTER: "router",
                 G.L_EXP_WGU: "expert_wgu", G.L_EXP_WD: "expert_wd", G.L_QNORM: "q_norm",
                 G.L_KNORM: "k_norm"}
        self.layers = []
        for l in range(s.n_layers):
            d = {}
            for which, rows, cols, kind in G.layer_tensor_shapes(s):
                d[names[which]] = new(G.layer_tid(l, which), rows, cols, kind)
            self.layers.append(d)
        n = G.kv_layer_numel(s)
        self.k = torch.empty((s.n_layers, s.batch, s.n_kv_heads, s.max_seq, s.head_dim), dtype=bf, device=dev)
        self.v = torch.empty_like(self.k)
        for l in range(s.n_layers):
            G.fill_device(self.k[l], seed, G.layer_tid(l, G.L_KCACHE), 0, "kv")
            G.fill_device(self.v[l], seed, G.layer_tid(l, G.L_VCACHE), 0, "kv")
        torch.cuda.synchronize(dev)

    def reset_kv(self):
        for l in range(self.s.n_layers):
            G.fill_device(self.k[l], self.seed, G.layer_tid(l, G.L_KCACHE), 0, "kv")
            G.fill_device(self.v[l], self.seed, G.layer_tid(l, G.L_VCACHE), 0, "kv")
        torch.cuda.synchronize(self.device)

    def weight_ptrs(self) -> dict:
        return {"embed": self.embed.data_ptr(), "final_norm": self.final_norm.data_ptr(),
                "lm_head": self.lm_head.data_ptr(),
                "layers": [{k: v.data_ptr() for k, v in d.items()} for d in self.layers]}

    def kv_ptrs(self):
        return (self.k.data_ptr(), self.v.data_ptr())
