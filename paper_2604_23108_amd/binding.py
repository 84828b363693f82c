"""ctypes binding of libmohge.so: argument marshalling only.

Function names and argument order are those of `include/mohge.h`.  Tensors must live on
the GPU; pointers are taken with `data_ptr()` and the current torch stream is passed as
the HIP stream.  PyTorch is used for device memory and streams only.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmohge.so")

SELECT_GLOBAL, SELECT_PER_GROUP = 0, 1
F32, BF16 = 0, 1
CALL_PERMUTE, CALL_EXPERT_FFN, CALL_AUX_LOSS = 0, 1, 2
CALL_FFN_SAVED, CALL_EXPERT_FFN_BWD, CALL_ROUTE_BWD, CALL_ROUTE, CALL_DECODE_LAYER = 3, 4, 5, 6, 7

EXPORTS = ["mohge_route", "mohge_permute", "mohge_permute_static", "mohge_expert_ffn", "mohge_combine",
           "mohge_aux_loss", "mohge_expert_ffn_up", "mohge_expert_ffn_down", "mohge_fused_status",
           "mohge_expert_ffn_train", "mohge_expert_ffn_w8", "mohge_fp8_decode", "mohge_expert_ffn_w4",
           "mohge_mxfp4_decode", "mohge_combine_bwd",
           "mohge_expert_ffn_bwd", "mohge_route_bwd", "mohge_shared_routing", "mohge_combine_add",
           "mohge_decode_layer", "mohge_decode_layer_ctl_bytes",
           "mohge_workspace_size", "mohge_last_error"]

_SIZE_RETURNS = ("mohge_workspace_size", "mohge_decode_layer_ctl_bytes")


class MohgeError(RuntimeError):
    pass


class _CConfig(C.Structure):
    _fields_ = [("T", C.c_int32), ("d", C.c_int32), ("n_groups", C.c_int32),
                ("experts_per_group", C.c_int32), ("d_ff", C.POINTER(C.c_int32)),
                ("k_groups", C.c_int32), ("k_experts", C.c_int32), ("select_mode", C.c_int32),
                ("dtype", C.c_int32), ("alpha_g", C.c_float), ("alpha_e", C.c_float),
                ("eps", C.c_float), ("aux_freq_norm", C.c_int32)]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise MohgeError(f"{_LIB_PATH} is missing: build it with "
                             "`python -m paper_2604_23108_amd.build` (there is no fallback path)")
        l = C.CDLL(_LIB_PATH)
        for n in EXPORTS[:-1]:
            getattr(l, n).restype = C.c_size_t if n in _SIZE_RETURNS else C.c_int
        l.mohge_last_error.restype = C.c_char_p
        _lib = l
    return _lib


class Config:
    """Python mirror of `mohge_config`."""

    def __init__(self, T: int, d: int, n_groups: int, experts_per_group: int, d_ff: Sequence[int],
                 k_groups: int, k_experts: int, select_mode: int = SELECT_PER_GROUP,
                 dtype: int = BF16, alpha_g: float = 1e-4, alpha_e: float = 2.5e-3,
                 eps: float = 1e-9, aux_freq_norm: int = 1):
        self.T, self.d, self.n_groups, self.experts_per_group = T, d, n_groups, experts_per_group
        self.d_ff = tuple(int(f) for f in d_ff)
        self.k_groups, self.k_experts, self.select_mode, self.dtype = k_groups, k_experts, select_mode, dtype
        self.alpha_g, self.alpha_e, self.eps, self.aux_freq_norm = alpha_g, alpha_e, eps, aux_freq_norm
        self._dff = (C.c_int32 * max(1, len(self.d_ff)))(*self.d_ff)
        self._c = _CConfig(T, d, n_groups, experts_per_group, self._dff, k_groups, k_experts,
                           select_mode, dtype, alpha_g, alpha_e, eps, aux_freq_norm)

    @classmethod
    def from_workload(cls, w, **kw) -> "Config":
        args = dict(T=w.T, d=w.d, n_groups=w.n_groups, experts_per_group=w.experts_per_group,
                    d_ff=w.d_ff, k_groups=w.k_groups, k_experts=w.k_experts,
                    select_mode=w.select_mode, dtype=BF16 if w.dtype == "bf16" else F32,
                    alpha_g=w.alpha_g, alpha_e=w.alpha_e, eps=w.eps)
        args.update(kw)
        return cls(**args)

    @property
    def n_experts(self) -> int:
        return self.n_groups * self.experts_per_group

    @property
    def n_pairs(self) -> int:
        return self.T * self.k_experts

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == BF16 else torch.float32

    def ref(self):
        return C.byref(self._c)


def mohge_last_error() -> str:
    return lib().mohge_last_error().decode()


def _check(rc: int, what: str):
    if rc != 0:
        raise MohgeError(f"{what} failed with code {rc}: {mohge_last_error()}")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return C.c_void_p(0)
    if not t.is_cuda:
        raise MohgeError("tensors handed to the library must be on the GPU")
    if not t.is_contiguous():
        raise MohgeError("tensors handed to the library must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def mohge_workspace_size(cfg: Config, which_call: int) -> int:
    return int(lib().mohge_workspace_size(cfg.ref(), C.c_int(which_call)))


def mohge_route(cfg, x, w_group, w_expert, expert_logit_bias, group_idx, expert_idx, gates,
                gs_out=None, es1_out=None, workspace=None):
    _check(lib().mohge_route(cfg.ref(), _ptr(x), _ptr(w_group), _ptr(w_expert),
                             _ptr(expert_logit_bias), _ptr(group_idx), _ptr(expert_idx),
                             _ptr(gates), _ptr(gs_out), _ptr(es1_out), _ptr(workspace),
                             _nbytes(workspace) if workspace is not None else C.c_size_t(0), _stream()),
           "mohge_route")


def mohge_permute(cfg, expert_idx, counts, offsets, perm, inv_perm, x, x_perm, workspace):
    _check(lib().mohge_permute(cfg.ref(), _ptr(expert_idx), _ptr(counts), _ptr(offsets), _ptr(perm),
                               _ptr(inv_perm), _ptr(x), _ptr(x_perm), _ptr(workspace),
                               C.c_size_t(workspace.numel() * workspace.element_size()), _stream()),
           "mohge_permute")


def mohge_permute_static(cfg, expert_idx, counts, offsets, perm, inv_perm, x, x_perm):
    _check(lib().mohge_permute_static(cfg.ref(), _ptr(expert_idx), _ptr(counts), _ptr(offsets), _ptr(perm),
                                      _ptr(inv_perm), _ptr(x), _ptr(x_perm), _stream()),
           "mohge_permute_static")


def _ptr_table(ts: Sequence[torch.Tensor]):
    return (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])


def mohge_expert_ffn(cfg, x, perm, offsets, w13: Sequence[torch.Tensor], w2: Sequence[torch.Tensor],
                     y_perm, workspace):
    for t in list(w13) + list(w2):
        _ptr(t)
    _check(lib().mohge_expert_ffn(cfg.ref(), _ptr(x), _ptr(perm), _ptr(offsets), _ptr_table(w13),
                                  _ptr_table(w2), _ptr(y_perm), _ptr(workspace),
                                  C.c_size_t(workspace.numel() * workspace.element_size()),
                                  _stream()), "mohge_expert_ffn")


def mohge_fused_status(cfg, which_call: int, workspace) -> int:
    """Synchronises; 0, or MOHGE_ETIMEOUT (-6) when a tile of the last fused launch gave up waiting
    (CALL_DECODE_LAYER: also MOHGE_EINVAL (-1) when the workspace counters were not zero)."""
    rc = lib().mohge_fused_status(cfg.ref(), C.c_int(which_call), _ptr(workspace), _nbytes(workspace), _stream())
    if rc not in (0, -6) and not (rc == -1 and which_call == CALL_DECODE_LAYER):
        _check(rc, "mohge_fused_status")
    return rc


def mohge_decode_layer(cfg, x, w_group, w_expert, expert_logit_bias, w13, w2, group_idx, expert_idx, gates, y,
                       workspace):
    for t in list(w13) + list(w2):
        _ptr(t)
    _check(lib().mohge_decode_layer(cfg.ref(), _ptr(x), _ptr(w_group), _ptr(w_expert), _ptr(expert_logit_bias),
                                    _ptr_table(w13), _ptr_table(w2), _ptr(group_idx), _ptr(expert_idx),
                                    _ptr(gates), _ptr(y), _ptr(workspace), _nbytes(workspace), _stream()),
           "mohge_decode_layer")


def mohge_decode_layer_ctl_bytes(cfg: Config) -> int:
    return int(lib().mohge_decode_layer_ctl_bytes(cfg.ref()))


def mohge_expert_ffn_w8(cfg, x, perm, offsets, w13q, w13_scale, w2q, w2_scale, y_perm, workspace):
    for t in list(w13q) + list(w13_scale) + list(w2q) + list(w2_scale):
        _ptr(t)
    _check(lib().mohge_expert_ffn_w8(cfg.ref(), _ptr(x), _ptr(perm), _ptr(offsets), _ptr_table(w13q),
                                     _ptr_table(w13_scale), _ptr_table(w2q), _ptr_table(w2_scale),
                                     _ptr(y_perm), _ptr(workspace), _nbytes(workspace), _stream()),
           "mohge_expert_ffn_w8")


def mohge_fp8_decode(codes: torch.Tensor, out: torch.Tensor):
    _check(lib().mohge_fp8_decode(_ptr(codes), _ptr(out), C.c_size_t(codes.numel()), _stream()),
           "mohge_fp8_decode")


def mohge_expert_ffn_w4(cfg, x, perm, offsets, w13q, w13_scale, w2q, w2_scale, y_perm, workspace):
    for t in list(w13q) + list(w13_scale) + list(w2q) + list(w2_scale):
        _ptr(t)
    _check(lib().mohge_expert_ffn_w4(cfg.ref(), _ptr(x), _ptr(perm), _ptr(offsets), _ptr_table(w13q),
                                     _ptr_table(w13_scale), _ptr_table(w2q), _ptr_table(w2_scale),
                                     _ptr(y_perm), _ptr(workspace), _nbytes(workspace), _stream()),
           "mohge_expert_ffn_w4")


def mohge_mxfp4_decode(packed: torch.Tensor, scales: torch.Tensor, out: torch.Tensor):
    _check(lib().mohge_mxfp4_decode(_ptr(packed), _ptr(scales), _ptr(out), C.c_size_t(out.numel()), _stream()),
           "mohge_mxfp4_decode")


def mohge_expert_ffn_up(cfg, x, perm, offsets, w13: Sequence[torch.Tensor], h):
    for t in w13:
        _ptr(t)
    _check(lib().mohge_expert_ffn_up(cfg.ref(), _ptr(x), _ptr(perm), _ptr(offsets), _ptr_table(w13),
                                     _ptr(h), C.c_size_t(h.numel() * h.element_size()), _stream()),
           "mohge_expert_ffn_up")


def mohge_expert_ffn_down(cfg, h, offsets, w2: Sequence[torch.Tensor], y_perm):
    for t in w2:
        _ptr(t)
    _check(lib().mohge_expert_ffn_down(cfg.ref(), _ptr(h), _nbytes(h), _ptr(offsets), _ptr_table(w2),
                                       _ptr(y_perm), _stream()), "mohge_expert_ffn_down")


def mohge_combine(cfg, y_perm, inv_perm, gates, y):
    _check(lib().mohge_combine(cfg.ref(), _ptr(y_perm), _ptr(inv_perm), _ptr(gates), _ptr(y),
                               _stream()), "mohge_combine")


def mohge_combine_add(cfg, y_perm, inv_perm, gates, y_add, y):
    _check(lib().mohge_combine_add(cfg.ref(), _ptr(y_perm), _ptr(inv_perm), _ptr(gates), _ptr(y_add),
                                   _ptr(y), _stream()), "mohge_combine_add")


def mohge_shared_routing(cfg, expert_idx, gates, counts, offsets, perm, inv_perm):
    _check(lib().mohge_shared_routing(cfg.ref(), _ptr(expert_idx), _ptr(gates), _ptr(counts),
                                      _ptr(offsets), _ptr(perm), _ptr(inv_perm), _stream()),
           "mohge_shared_routing")


def mohge_aux_loss(cfg, gs, es1, group_idx, expert_idx, losses, stats, workspace):
    _check(lib().mohge_aux_loss(cfg.ref(), _ptr(gs), _ptr(es1), _ptr(group_idx), _ptr(expert_idx),
                                _ptr(losses), _ptr(stats), _ptr(workspace),
                                C.c_size_t(workspace.numel() * workspace.element_size()),
                                _stream()), "mohge_aux_loss")


def _nbytes(t: torch.Tensor):
    return C.c_size_t(t.numel() * t.element_size())


def mohge_expert_ffn_train(cfg, x, perm, offsets, w13, w2, y_perm, saved):
    for t in list(w13) + list(w2):
        _ptr(t)
    _check(lib().mohge_expert_ffn_train(cfg.ref(), _ptr(x), _ptr(perm), _ptr(offsets), _ptr_table(w13),
                                        _ptr_table(w2), _ptr(y_perm), _ptr(saved), _nbytes(saved),
                                        _stream()), "mohge_expert_ffn_train")


def mohge_combine_bwd(cfg, dy, y_perm, inv_perm, gates, dgates, dy_perm):
    _check(lib().mohge_combine_bwd(cfg.ref(), _ptr(dy), _ptr(y_perm), _ptr(inv_perm), _ptr(gates),
                                   _ptr(dgates), _ptr(dy_perm), _stream()), "mohge_combine_bwd")


def mohge_expert_ffn_bwd(cfg, x, perm, offsets, w13, w2, saved, dy_perm, dx_perm, dw13, dw2,
                         workspace):
    for t in list(w13) + list(w2) + list(dw13) + list(dw2):
        _ptr(t)
    _check(lib().mohge_expert_ffn_bwd(cfg.ref(), _ptr(x), _ptr(perm), _ptr(offsets), _ptr_table(w13),
                                      _ptr_table(w2), _ptr(saved), _ptr(dy_perm), _ptr(dx_perm),
                                      _ptr_table(dw13), _ptr_table(dw2), _ptr(workspace),
                                      _nbytes(workspace), _stream()), "mohge_expert_ffn_bwd")


def mohge_route_bwd(cfg, x, w_group, w_expert, gs, es1, group_idx, expert_idx, gates, dgates, stats,
                    dx_perm, inv_perm, dx, dw_group, dw_expert, dz_out, workspace):
    _check(lib().mohge_route_bwd(cfg.ref(), _ptr(x), _ptr(w_group), _ptr(w_expert), _ptr(gs), _ptr(es1),
                                 _ptr(group_idx), _ptr(expert_idx), _ptr(gates), _ptr(dgates),
                                 _ptr(stats), _ptr(dx_perm), _ptr(inv_perm), _ptr(dx), _ptr(dw_group),
                                 _ptr(dw_expert), _ptr(dz_out), _ptr(workspace), _nbytes(workspace),
                                 _stream()), "mohge_route_bwd")


def pack_w13(w_gate: torch.Tensor, w_up: torch.Tensor) -> torch.Tensor:
    """Layout helper: [N,F,d] gate and up matrices -> the [N,2F,d] block the library reads
    (gate rows first).  Pure data movement."""
    return torch.cat([w_gate, w_up], dim=1).contiguous()


class SharedExperts:
    """N_s always-on experts of one width: buffers and the constant routing, made once."""

    def __init__(self, T: int, d: int, w13: torch.Tensor, w2: torch.Tensor, dtype: int = BF16,
                 device="cuda", backward: bool = False):
        n_s, f_s = w2.shape[0], w2.shape[2]
        self.cfg = Config(T=T, d=d, n_groups=1, experts_per_group=n_s, d_ff=(f_s,), k_groups=1,
                          k_experts=n_s, select_mode=SELECT_PER_GROUP, dtype=dtype)
        self.w13, self.w2 = [w13], [w2]
        P = T * n_s
        i32 = dict(dtype=torch.int32, device=device)
        self.expert_idx = torch.empty((T, n_s), **i32)
        self.gates = torch.empty((T, n_s), dtype=torch.float32, device=device)
        self.counts, self.offsets = torch.empty(n_s, **i32), torch.empty(n_s + 1, **i32)
        self.perm, self.inv_perm = torch.empty(max(P, 1), **i32), torch.empty(max(P, 1), **i32)
        self.y_perm = torch.empty((max(P, 1), d), dtype=self.cfg.torch_dtype, device=device)
        self.y = torch.empty((T, d), dtype=self.cfg.torch_dtype, device=device)
        self.ws = torch.empty(max(16, mohge_workspace_size(self.cfg, CALL_EXPERT_FFN)), dtype=torch.uint8,
                              device=device)
        mohge_shared_routing(self.cfg, self.expert_idx, self.gates, self.counts, self.offsets, self.perm,
                             self.inv_perm)
        self.has_backward = backward
        if backward:
            if dtype != BF16:
                raise MohgeError("backward needs bf16 shared experts")
            u8 = dict(dtype=torch.uint8, device=device)
            bf = dict(dtype=torch.bfloat16, device=device)
            self.saved = torch.empty(max(16, mohge_workspace_size(self.cfg, CALL_FFN_SAVED)), **u8)
            self.ws_bwd = torch.empty(max(16, mohge_workspace_size(self.cfg, CALL_EXPERT_FFN_BWD)), **u8)
            self.dgates = torch.empty((T, n_s), dtype=torch.float32, device=device)
            self.dy_perm = torch.empty((max(P, 1), d), **bf)
            self.dx_perm = torch.empty((max(P, 1), d), **bf)
            self.dw13, self.dw2 = [torch.empty_like(w13)], [torch.empty_like(w2)]
            self.dx = torch.empty((T, d), **bf)

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        c = self.cfg
        if self.has_backward:
            mohge_expert_ffn_train(c, x, self.perm, self.offsets, self.w13, self.w2, self.y_perm, self.saved)
        else:
            mohge_expert_ffn(c, x, self.perm, self.offsets, self.w13, self.w2, self.y_perm, self.ws)
        mohge_combine(c, self.y_perm, self.inv_perm, self.gates, self.y)
        return self.y

    def backward(self, x: torch.Tensor, dy: torch.Tensor, dx_add: torch.Tensor) -> torch.Tensor:
        """After `forward(x)`: weight gradients into dw13 / dw2, and dx = dx_add + the shared
        experts' input gradient.  Every token hands dy[t] to each expert with weight 1, so the
        layer's own calls do it: the combine backward with the constant gates, the expert
        backward, and a gated combine of the K rows of dx_perm per token on top of dx_add."""
        if not self.has_backward:
            raise MohgeError("SharedExperts was created without backward=True")
        c = self.cfg
        mohge_combine_bwd(c, dy, self.y_perm, self.inv_perm, self.gates, self.dgates, self.dy_perm)
        mohge_expert_ffn_bwd(c, x, self.perm, self.offsets, self.w13, self.w2, self.saved, self.dy_perm,
                             self.dx_perm, self.dw13, self.dw2, self.ws_bwd)
        mohge_combine_add(c, self.dx_perm, self.inv_perm, self.gates, dx_add, self.dx)
        return self.dx


class MoHGELayer:
    """Holds the device buffers of one layer call and runs the five C calls in order.

    All buffers are allocated once here (by torch); `forward()` allocates nothing and only
    enqueues kernels on the current stream.
    """

    def __init__(self, cfg: Config, w_group, w_expert, w13: List[torch.Tensor],
                 w2: List[torch.Tensor], expert_logit_bias=None, training: bool = False,
                 backward: bool = False, shared: Optional["SharedExperts"] = None, device="cuda"):
        self.cfg = cfg
        self.w_group, self.w_expert, self.w13, self.w2 = w_group, w_expert, list(w13), list(w2)
        self.bias = expert_logit_bias
        self.training = training
        self.shared = shared
        self.ffn_options = None   # bench_binding.FfnOptions: the expert calls then go through the
                                  # benchmark library with these launch options (tests, benchmarks)
        self.w8 = None          # (codes13, scales13, codes2, scales2) once use_fp8_weights() was called
        self.w4 = None          # the same for MXFP4 weights, once use_mxfp4_weights() was called
        T, P, Ne, Ng = cfg.T, cfg.n_pairs, cfg.n_experts, cfg.n_groups
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        self.group_idx = torch.empty((T, cfg.k_groups), **i32)
        self.expert_idx = torch.empty((T, cfg.k_experts), **i32)
        self.gates = torch.empty((T, cfg.k_experts), **f32)
        self.gs = torch.empty((T, Ng), **f32) if training else None
        self.es1 = torch.empty((T, Ne), **f32) if training else None
        self.counts = torch.empty(Ne, **i32)
        self.offsets = torch.empty(Ne + 1, **i32)
        self.perm = torch.empty(max(P, 1), **i32)
        self.inv_perm = torch.empty(max(P, 1), **i32)
        self.y_perm = torch.empty((max(P, 1), cfg.d), dtype=cfg.torch_dtype, device=device)
        self.y = torch.empty((T, cfg.d), dtype=cfg.torch_dtype, device=device)
        u8 = dict(dtype=torch.uint8, device=device)
        self.ws_permute = torch.empty(max(16, mohge_workspace_size(cfg, CALL_PERMUTE)), **u8)
        self.ws_ffn = torch.empty(max(16, mohge_workspace_size(cfg, CALL_EXPERT_FFN)), **u8)
        n_route = mohge_workspace_size(cfg, CALL_ROUTE)
        self.ws_route = torch.empty(n_route, **u8) if n_route else None
        self.losses = torch.empty(2, **f32) if training else None
        self.stats = torch.empty(2 * Ng + 2 * Ne, **f32) if training else None
        self.ws_aux = torch.empty(max(16, mohge_workspace_size(cfg, CALL_AUX_LOSS)), **u8) if training else None
        # backward pass (bf16 layers): everything it writes is allocated here, once
        if backward and shared is not None and not shared.has_backward:
            raise MohgeError("backward with shared experts needs SharedExperts(..., backward=True)")
        if backward and not (training and cfg.dtype == BF16):
            raise MohgeError("backward needs a bf16 layer created with training=True")
        self.has_backward = backward
        if self.has_backward:
            bf = dict(dtype=torch.bfloat16, device=device)
            self.saved = torch.empty(max(16, mohge_workspace_size(cfg, CALL_FFN_SAVED)), **u8)
            self.ws_ffn_bwd = torch.empty(max(16, mohge_workspace_size(cfg, CALL_EXPERT_FFN_BWD)), **u8)
            self.ws_route_bwd = torch.empty(max(16, mohge_workspace_size(cfg, CALL_ROUTE_BWD)), **u8)
            self.dw13 = [torch.empty_like(w) for w in self.w13]
            self.dw2 = [torch.empty_like(w) for w in self.w2]
            self.dgates = torch.empty((T, cfg.k_experts), **f32)
            self.dy_perm = torch.empty((max(P, 1), cfg.d), **bf)
            self.dx_perm = torch.empty((max(P, 1), cfg.d), **bf)
            self.dx = torch.empty((T, cfg.d), **bf)
            self.dw_group = torch.empty((Ng, cfg.d), **f32)
            self.dw_expert = torch.empty((Ne, cfg.d), **f32)
            self.dz = torch.empty((T, Ng + Ne), **f32)

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        c = self.cfg
        mohge_route(c, x, self.w_group, self.w_expert, self.bias, self.group_idx, self.expert_idx,
                    self.gates, self.gs, self.es1, self.ws_route)
        mohge_permute(c, self.expert_idx, self.counts, self.offsets, self.perm, self.inv_perm,
                      None, None, self.ws_permute)
        if self.ffn_options is not None:
            from . import bench_binding as BB
            if self.has_backward:
                BB.mohge_bench_expert_ffn_train(c, x, self.perm, self.offsets, self.w13, self.w2, self.y_perm,
                                                self.saved, self.ffn_options)
            else:
                BB.mohge_bench_expert_ffn(c, x, self.perm, self.offsets, self.w13, self.w2, self.y_perm,
                                          self.ws_ffn, self.ffn_options)
        elif self.has_backward:
            mohge_expert_ffn_train(c, x, self.perm, self.offsets, self.w13, self.w2, self.y_perm,
                                   self.saved)
        elif self.w8 is not None:
            mohge_expert_ffn_w8(c, x, self.perm, self.offsets, *self.w8, self.y_perm, self.ws_ffn)
        elif self.w4 is not None:
            mohge_expert_ffn_w4(c, x, self.perm, self.offsets, *self.w4, self.y_perm, self.ws_ffn)
        else:
            mohge_expert_ffn(c, x, self.perm, self.offsets, self.w13, self.w2, self.y_perm, self.ws_ffn)
        if self.shared is not None:
            mohge_combine_add(c, self.y_perm, self.inv_perm, self.gates, self.shared.forward(x), self.y)
        else:
            mohge_combine(c, self.y_perm, self.inv_perm, self.gates, self.y)
        if self.training:
            mohge_aux_loss(c, self.gs, self.es1, self.group_idx, self.expert_idx, self.losses,
                           self.stats, self.ws_aux)
        return self.y

    def forward_decode(self, x: torch.Tensor) -> torch.Tensor:
        """The forward pass of a decode-sized bf16 call as one launch (mohge_decode_layer): fills
        group_idx, expert_idx, gates and y like forward().  The workspace is allocated and cleared
        on first use."""
        if getattr(self, "ws_decode", None) is None:
            n = mohge_workspace_size(self.cfg, CALL_DECODE_LAYER)
            if n == 0:
                raise MohgeError("mohge_decode_layer serves bf16 calls of at most 32 tokens")
            self.ws_decode = torch.zeros(n, dtype=torch.uint8, device=x.device)
        mohge_decode_layer(self.cfg, x, self.w_group, self.w_expert, self.bias, self.w13, self.w2,
                           self.group_idx, self.expert_idx, self.gates, self.y, self.ws_decode)
        return self.y

    def use_fp8_weights(self):
        """Decode only (T <= 32): quantises the expert weights per row to FP8 E4M3 once and makes
        forward() stream those instead of the bf16 weights."""
        if self.cfg.T > 32 or self.cfg.dtype != BF16 or self.has_backward:
            raise MohgeError("FP8 expert weights are served by the bf16 decode path only (T <= 32)")
        from .weights import quantize_rows_e4m3
        q = [quantize_rows_e4m3(w) for w in self.w13], [quantize_rows_e4m3(w) for w in self.w2]
        self.w8 = ([c for c, _ in q[0]], [s for _, s in q[0]], [c for c, _ in q[1]], [s for _, s in q[1]])
        self.w4 = None

    def use_mxfp4_weights(self):
        """Decode only (T <= 32): quantises the expert weights to MXFP4 once and makes forward()
        stream those instead of the bf16 weights."""
        if self.cfg.T > 32 or self.cfg.dtype != BF16 or self.has_backward:
            raise MohgeError("MXFP4 expert weights are served by the bf16 decode path only (T <= 32)")
        from .weights import quantize_mxfp4
        q = [quantize_mxfp4(w) for w in self.w13], [quantize_mxfp4(w) for w in self.w2]
        self.w8 = None
        self.w4 = ([c for c, _ in q[0]], [s for _, s in q[0]], [c for c, _ in q[1]], [s for _, s in q[1]])

    def capture(self, x: torch.Tensor, dy: Optional[torch.Tensor] = None):
        """Records one step (forward, or forward + backward when `dy` is
        given) into a HIP graph; `replay()` then launches the whole step with one call.  The step
        allocates nothing and never synchronises with the host, so the recorded launches are
        exactly the eager ones; `x` / `dy` are read from the same buffers on every replay."""
        def step():
            self.forward(x)
            if dy is not None:
                self.backward(x, dy)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()                      # first launches set kernel attributes: keep them out of the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        self._graph = graph
        return graph

    def replay(self):
        self._graph.replay()

    def backward(self, x: torch.Tensor, dy: torch.Tensor) -> torch.Tensor:
        """Gradients of  sum(dy*y) + L_G + L_E  after `forward(x)`; returns dx, leaves the weight
        gradients in dw13 / dw2 / dw_group / dw_expert."""
        if not self.has_backward:
            raise MohgeError("backward needs a layer created with training=True, backward=True")
        c = self.cfg
        mohge_combine_bwd(c, dy, self.y_perm, self.inv_perm, self.gates, self.dgates, self.dy_perm)
        if self.ffn_options is not None:
            from . import bench_binding as BB
            BB.mohge_bench_expert_ffn_bwd(c, x, self.perm, self.offsets, self.w13, self.w2, self.saved,
                                          self.dy_perm, self.dx_perm, self.dw13, self.dw2, self.ws_ffn_bwd,
                                          self.ffn_options)
        else:
            mohge_expert_ffn_bwd(c, x, self.perm, self.offsets, self.w13, self.w2, self.saved,
                                 self.dy_perm, self.dx_perm, self.dw13, self.dw2, self.ws_ffn_bwd)
        mohge_route_bwd(c, x, self.w_group, self.w_expert, self.gs, self.es1, self.group_idx,
                        self.expert_idx, self.gates, self.dgates, self.stats, self.dx_perm,
                        self.inv_perm, self.dx, self.dw_group, self.dw_expert, self.dz,
                        self.ws_route_bwd)
        if self.shared is not None:
            return self.shared.backward(x, dy, self.dx)
        return self.dx
