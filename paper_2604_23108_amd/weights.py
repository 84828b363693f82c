"""Offline preparation of quantised expert weights for the decode calls mohge_expert_ffn_w8 /
mohge_expert_ffn_w4 (plain torch, run once when weights are loaded; not on the layer's path and
not part of the binding).  The formats are the ones `include/mohge.h` documents."""
from __future__ import annotations

import torch


def quantize_rows_e4m3(w: torch.Tensor):
    """Per-row FP8 E4M3 quantisation of a weight tensor [..., rows, cols]: scale[row] = max|row| / 448 (1 for an all-zero row), codes = the row divided
    by its scale, rounded to nearest even.  Returns (codes uint8 of w's shape, scales f32 of
    w's shape without the last axis)."""
    wf = w.float()
    amax = wf.abs().amax(dim=-1)
    scale = torch.where(amax > 0, amax / 448.0, torch.ones_like(amax))
    codes = (wf / scale.unsqueeze(-1)).to(torch.float8_e4m3fn).view(torch.uint8)
    return codes.contiguous(), scale.contiguous()


def quantize_mxfp4(w: torch.Tensor):
    """MXFP4 quantisation of a weight tensor [..., rows, cols], cols a multiple of 32: per block of 32 elements of a row the shared scale is
    2^(floor(log2 max|block|) - 2) (the largest E2M1 magnitude is 6 = 1.5 * 2^2), kept within scale
    codes 1..254; elements are divided by it, rounded to the nearest E2M1 value (ties to the even
    code) and clamped to +-6.  Returns (packed uint8 [..., rows, cols/2], two codes per byte, even
    element in the low four bits; scale codes uint8 [..., rows, cols/32])."""
    K = w.shape[-1]
    if K % 32:
        raise ValueError(f"quantize_mxfp4: last dimension {K} is not a multiple of 32")
    blk = w.float().reshape(*w.shape[:-1], K // 32, 32)
    amax = blk.abs().amax(dim=-1, keepdim=True)
    _, ex = torch.frexp(amax)                      # amax = m * 2^ex, m in [0.5, 1): floor(log2) = ex - 1
    e = torch.where(amax > 0, ex - 1 - 2, torch.zeros_like(ex)).clamp(-126, 127)
    v = torch.ldexp(blk, -e)
    m = v.abs()
    code = torch.zeros_like(m, dtype=torch.int32)
    for j, mid in enumerate((0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0)):
        # from an even code to the odd one above it only when strictly past the midpoint
        code += ((m > mid) if j % 2 == 0 else (m >= mid)).to(torch.int32)
    code |= (v < 0).to(torch.int32) << 3
    code = code.reshape(*w.shape[:-1], K // 2, 2)
    packed = (code[..., 0] | (code[..., 1] << 4)).to(torch.uint8)
    scales = (e.squeeze(-1) + 127).to(torch.uint8)
    return packed.contiguous(), scales.contiguous()


