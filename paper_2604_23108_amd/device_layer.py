"""A synthetic workload placed on the GPU: moves seeded inputs to the device (bit exact), builds
the layer object, runs a forward pass and brings the results back as numpy arrays.  Used by the
benchmark, the smoke entry and the GPU tests.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as M


def to_dev(t, bf16: bool) -> torch.Tensor:
    """synth.Tensor -> device tensor of the workload's storage type (bit exact)."""
    if bf16:
        return torch.from_numpy(t.bits.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(t.f32).cuda()


def from_dev(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()


class DeviceLayer:
    def __init__(self, w, inp, training=None, backward=False, **cfg_kw):
        bf = w.dtype == "bf16"
        self.w, self.bf = w, bf
        self.cfg = M.Config.from_workload(w, **cfg_kw)
        self.x = to_dev(inp.x, bf)
        self.w_group = torch.from_numpy(inp.w_group).cuda()
        self.w_expert = torch.from_numpy(inp.w_expert).cuda()
        self.bias = None if inp.expert_logit_bias is None else torch.from_numpy(inp.expert_logit_bias).cuda()
        self.w13 = [M.pack_w13(to_dev(g, bf), to_dev(u, bf)) for g, u in zip(inp.w_gate, inp.w_up)]
        self.w2 = [to_dev(t, bf) for t in inp.w_down]
        self.layer = M.MoHGELayer(self.cfg, self.w_group, self.w_expert, self.w13, self.w2, self.bias,
                                  training=(w.training if training is None else training) or backward,
                                  backward=backward)

    def run(self):
        L = self.layer
        y = L.forward(self.x)
        torch.cuda.synchronize()
        out = dict(group_idx=L.group_idx.cpu().numpy(), expert_idx=L.expert_idx.cpu().numpy(),
                   gates=L.gates.cpu().numpy(), counts=L.counts.cpu().numpy(),
                   offsets=L.offsets.cpu().numpy(), perm=L.perm.cpu().numpy()[:self.cfg.n_pairs],
                   inv_perm=L.inv_perm.cpu().numpy()[:self.cfg.n_pairs], y=from_dev(y),
                   y_perm=L.y_perm)
        if L.training:
            out.update(gs=L.gs.cpu().numpy(), es1=L.es1.cpu().numpy(), losses=L.losses.cpu().numpy(),
                       stats=L.stats.cpu().numpy())
        return out
