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


class GuardBands:
    """Out-of-bounds canaries: re-homes tensors inside larger buffers filled with a sentinel byte,
    256 bytes before and at least 256 after, and checks later that the sentinels are intact."""
    SENTINEL, PAD = 0xA5, 256

    def __init__(self):
        self.items = []

    def wrap(self, t: torch.Tensor, name: str) -> torch.Tensor:
        nbytes = t.numel() * t.element_size()
        body = (nbytes + 255) // 256 * 256
        buf = torch.full((self.PAD + body + self.PAD,), self.SENTINEL, dtype=torch.uint8, device=t.device)
        self.items.append((name, buf, nbytes))
        return buf[self.PAD:self.PAD + nbytes].view(t.dtype).view(t.shape)

    def check(self):
        for name, buf, nbytes in self.items:
            assert bool((buf[:self.PAD] == self.SENTINEL).all()), f"write in front of {name}"
            assert bool((buf[self.PAD + nbytes:] == self.SENTINEL).all()), f"write behind {name}"


# every tensor a layer call writes (inputs, weights and workspaces are not re-homed)
_OUTPUTS = ("group_idx", "expert_idx", "gates", "gs", "es1", "counts", "offsets", "perm", "inv_perm", "y_perm", "y",
            "losses", "stats", "dgates", "dy_perm", "dx_perm", "dx", "dw_group", "dw_expert", "dz")


class DeviceLayer:
    def __init__(self, w, inp, training=None, backward=False, guard=False, **cfg_kw):
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
        self.guards = None
        if guard:
            # guard bands around everything the calls write; checked by run() and check_guards()
            self.guards, L = GuardBands(), self.layer
            for name in _OUTPUTS:
                t = getattr(L, name, None)
                if isinstance(t, torch.Tensor):
                    setattr(L, name, self.guards.wrap(t, name))
            for name in ("dw13", "dw2"):
                if getattr(L, name, None) is not None:
                    setattr(L, name, [self.guards.wrap(t, f"{name}[{g}]") for g, t in enumerate(getattr(L, name))])

    def check_guards(self):
        if self.guards is not None:
            torch.cuda.synchronize()
            self.guards.check()

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
        self.check_guards()
        return out
