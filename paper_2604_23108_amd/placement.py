"""All-size Group-decoupling Allocation (paper section 3.4.1) as a host-side rule.

An all-size expert set is the i-th expert of every group; every GPU is given the same
number of such sets, so every GPU holds the same number of expert parameters whatever
the group widths are.  This module only decides WHICH experts live on which GPU (and
therefore which weights are handed to the layer of one GPU as an `N_g x N_local` layer);
it moves no data and involves no communication.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np


def local_expert_indices(experts_per_group: int, n_gpus: int, rank: int, mode: str = "contiguous") -> List[int]:
    """Indices i (inside every group) of the all-size sets held by GPU `rank`.

    mode "contiguous": GPU r holds i in [r*N/R, (r+1)*N/R); mode "strided": i with i % R == r
    (the paper's experiment places the i-th expert of each group on the i-th GPU, which both
    modes reproduce when N == R).
    """
    N, R = experts_per_group, n_gpus
    if R < 1 or N % R != 0:
        raise ValueError("experts_per_group must be a multiple of the number of GPUs")
    if not 0 <= rank < R:
        raise ValueError("rank out of range")
    per = N // R
    if mode == "contiguous":
        return list(range(rank * per, (rank + 1) * per))
    if mode == "strided":
        return list(range(rank, N, R))
    raise ValueError("mode must be 'contiguous' or 'strided'")


def owner_of(expert_in_group: int, experts_per_group: int, n_gpus: int, mode: str = "contiguous") -> int:
    per = experts_per_group // n_gpus
    return expert_in_group // per if mode == "contiguous" else expert_in_group % n_gpus


def local_global_ids(n_groups: int, experts_per_group: int, n_gpus: int, rank: int,
                     mode: str = "contiguous") -> np.ndarray:
    """Global expert ids e = g*N + i held by `rank`, as an [N_g, N_local] array: the local
    layer's expert (g, j) is the global expert ids[g, j]."""
    idx = local_expert_indices(experts_per_group, n_gpus, rank, mode)
    return np.asarray([[g * experts_per_group + i for i in idx] for g in range(n_groups)], dtype=np.int64)


def parameter_bytes_per_gpu(d: int, d_ff: Sequence[int], experts_per_group: int, n_gpus: int,
                            bytes_per_elem: int = 2) -> List[int]:
    """Expert parameter bytes on every GPU (three d x F matrices per expert): equal by construction."""
    per = experts_per_group // n_gpus
    one = sum(3 * d * f * bytes_per_elem for f in d_ff) * per
    return [one] * n_gpus


def load_report(expert_idx: np.ndarray, n_groups: int, experts_per_group: int, n_gpus: int,
                d_ff: Sequence[int], mode: str = "contiguous") -> Dict[str, np.ndarray]:
    """Replays a routing result through `n_gpus` virtual GPUs.

    Returns, per GPU: the share of routed (token, expert) pairs inside every group
    (`share_by_group[g, r]`, each column of the paper's per-GPU load table sums to 1 over r)
    and the share of expert FLOPs (`flop_share[r]`, pairs weighted by the group width).
    """
    e = np.asarray(expert_idx).reshape(-1)
    g, i = e // experts_per_group, e % experts_per_group
    per = experts_per_group // n_gpus
    owner = i // per if mode == "contiguous" else i % n_gpus
    share = np.zeros((n_groups, n_gpus))
    np.add.at(share, (g, owner), 1.0)
    tot = share.sum(axis=1, keepdims=True)
    share_by_group = np.divide(share, tot, out=np.zeros_like(share), where=tot > 0)
    w = np.asarray(d_ff, dtype=np.float64)[g]
    flops = np.zeros(n_gpus)
    np.add.at(flops, owner, w)
    return dict(share_by_group=share_by_group, flop_share=flops / flops.sum())


def format_report(report: Dict[str, np.ndarray], title: str = "") -> str:
    """The load report as a text table in the shape of the paper's per-GPU load table: one row per
    virtual GPU, one column per group (share of that group's routed pairs, in percent), then the
    GPU's share of the expert FLOPs."""
    share, flops = report["share_by_group"], report["flop_share"]
    n_groups, n_gpus = share.shape
    lines = [title] if title else []
    lines.append("GPU   " + " ".join(f"grp{g:<3d}" for g in range(n_groups)) + "   FLOPs")
    for r in range(n_gpus):
        lines.append(f"{r:<5d} " + " ".join(f"{100 * share[g, r]:6.2f}" for g in range(n_groups)) +
                     f"  {100 * flops[r]:6.2f}")
    dev = 100 * np.abs(share - 1.0 / n_gpus).max()
    lines.append(f"ideal {100.0 / n_gpus:.2f} % per GPU; largest deviation {dev:.2f} points")
    return "\n".join(lines)
