"""ctypes binding of libmohge_bench.so (`include/mohge_bench.h`): the expert-network calls with
their launch options, and the two ceiling probes.  Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

from . import binding as B
from .binding import MohgeError, _check, _nbytes, _ptr, _ptr_table, _stream

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmohge_bench.so")

EXPORTS = ["mohge_ffn_default_options", "mohge_bench_cycles_bytes", "mohge_bench_expert_ffn",
           "mohge_bench_expert_ffn_train", "mohge_bench_expert_ffn_bwd", "mohge_probe_read", "mohge_probe_mfma",
           "mohge_bench_decode_layer", "mohge_bench_decode_trace_bytes"]


class _COptions(C.Structure):
    _fields_ = [("tile_rows_up", C.c_int32), ("tile_rows_down", C.c_int32), ("fused", C.c_int32),
                ("spin_limit", C.c_int32), ("band_rows", C.c_int32), ("group_major", C.c_int32),
                ("steal", C.c_int32), ("short_last", C.c_int32), ("defer_signal", C.c_int32), ("cycles_launch", C.c_int32), ("cycles", C.c_void_p),
                ("cycles_bytes", C.c_size_t)]


_lib = None


def lib():
    """The loaded benchmark library (loads the layer library first); raises if it has not been built."""
    global _lib
    if _lib is None:
        B.lib()
        if not os.path.exists(_LIB_PATH):
            raise MohgeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2604_23108_amd.build`")
        l = C.CDLL(_LIB_PATH)
        for n in EXPORTS[2:]:
            getattr(l, n).restype = C.c_size_t if n == "mohge_bench_decode_trace_bytes" else C.c_int
        l.mohge_bench_cycles_bytes.restype = C.c_size_t
        l.mohge_ffn_default_options.restype = None
        _lib = l
    return _lib


class FfnOptions:
    """Python mirror of `mohge_ffn_options`, starting from the library's defaults."""

    def __init__(self, cycles: Optional[torch.Tensor] = None, **kw):
        self._c = _COptions()
        lib().mohge_ffn_default_options(C.byref(self._c))
        for k, v in kw.items():
            if k not in dict(_COptions._fields_) or k in ("cycles", "cycles_bytes"):
                raise MohgeError(f"unknown option {k}")
            setattr(self._c, k, int(v))
        self.cycles = cycles
        if cycles is not None:
            self._c.cycles = _ptr(cycles).value
            self._c.cycles_bytes = cycles.numel() * cycles.element_size()

    def ref(self):
        return C.byref(self._c)


def _opt(o: Optional[FfnOptions]):
    return o.ref() if o is not None else None


def cycles_buffer() -> torch.Tensor:
    """A zeroed counter buffer of the size the library asks for, as int64 [2, workgroups, 8]."""
    n = int(lib().mohge_bench_cycles_bytes()) // 8
    return torch.zeros((2, n // 16, 8), dtype=torch.int64, device="cuda")


def mohge_bench_expert_ffn(cfg, x, perm, offsets, w13, w2, y_perm, workspace, options=None, parts: int = 3):
    for t in list(w13) + list(w2):
        _ptr(t)
    _check(lib().mohge_bench_expert_ffn(cfg.ref(), _ptr(x), _ptr(perm), _ptr(offsets), _ptr_table(w13),
                                        _ptr_table(w2), _ptr(y_perm), _ptr(workspace), _nbytes(workspace),
                                        _opt(options), C.c_int(parts), _stream()), "mohge_bench_expert_ffn")


def mohge_bench_expert_ffn_train(cfg, x, perm, offsets, w13, w2, y_perm, saved, options=None):
    for t in list(w13) + list(w2):
        _ptr(t)
    _check(lib().mohge_bench_expert_ffn_train(cfg.ref(), _ptr(x), _ptr(perm), _ptr(offsets), _ptr_table(w13),
                                              _ptr_table(w2), _ptr(y_perm), _ptr(saved), _nbytes(saved),
                                              _opt(options), _stream()), "mohge_bench_expert_ffn_train")


def mohge_bench_expert_ffn_bwd(cfg, x, perm, offsets, w13, w2, saved, dy_perm, dx_perm, dw13, dw2, workspace,
                               options=None):
    for t in list(w13) + list(w2) + list(dw13) + list(dw2):
        _ptr(t)
    _check(lib().mohge_bench_expert_ffn_bwd(cfg.ref(), _ptr(x), _ptr(perm), _ptr(offsets), _ptr_table(w13),
                                            _ptr_table(w2), _ptr(saved), _ptr(dy_perm), _ptr(dx_perm),
                                            _ptr_table(dw13), _ptr_table(dw2), _ptr(workspace), _nbytes(workspace),
                                            _opt(options), _stream()), "mohge_bench_expert_ffn_bwd")


def mohge_bench_decode_layer(cfg, x, w_group, w_expert, expert_logit_bias, w13, w2, group_idx, expert_idx, gates, y,
                             workspace, spin_limit: int = 0, trace=None):
    for t in list(w13) + list(w2):
        _ptr(t)
    _check(lib().mohge_bench_decode_layer(cfg.ref(), _ptr(x), _ptr(w_group), _ptr(w_expert), _ptr(expert_logit_bias),
                                          _ptr_table(w13), _ptr_table(w2), _ptr(group_idx), _ptr(expert_idx),
                                          _ptr(gates), _ptr(y), _ptr(workspace), _nbytes(workspace),
                                          C.c_int(spin_limit), _ptr(trace),
                                          _nbytes(trace) if trace is not None else C.c_size_t(0), _stream()), "mohge_bench_decode_layer")


def decode_trace_buffer(cfg) -> torch.Tensor:
    """A zeroed trace buffer for mohge_bench_decode_layer: int64 [pieces, 4]."""
    n = int(lib().mohge_bench_decode_trace_bytes(cfg.ref())) // 32
    return torch.zeros((n, 4), dtype=torch.int64, device="cuda")


def mohge_probe_read(buf: torch.Tensor, row_bytes: int, staggered: bool, out: torch.Tensor) -> int:
    """Enqueues the read probe on buf; returns the bytes the kernel reads."""
    n = C.c_size_t(0)
    _check(lib().mohge_probe_read(_ptr(buf), _nbytes(buf), C.c_int(row_bytes), C.c_int(int(staggered)), _ptr(out),
                                  C.byref(n), _stream()), "mohge_probe_read")
    return n.value


def mohge_probe_mfma(out: torch.Tensor, iters: int) -> float:
    """Enqueues the MFMA probe; returns the FLOPs of the launch."""
    f = C.c_double(0.0)
    _check(lib().mohge_probe_mfma(_ptr(out), _nbytes(out), C.c_int(iters), C.byref(f), _stream()), "mohge_probe_mfma")
    return f.value
