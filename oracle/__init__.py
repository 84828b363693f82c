"""Python face of the CPU oracle (`mohge_oracle.c`).

TEST INFRASTRUCTURE ONLY: imported by `tests/`, by the smoke check and by the
benchmark's cpu_baseline leg.  Nothing here touches the HIP library, and the HIP
library never touches this.  All results are float64 numpy arrays computed by the
plain C loops; this file only marshals arguments.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mohge_oracle.c")
_SRC_BWD = os.path.join(_HERE, "mohge_oracle_bwd.c")
_LIB = os.path.join(_HERE, "libmohge_oracle.so")


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (OpenMP over independent tokens / pairs)."""
    stale = not os.path.exists(_LIB) or any(
        os.path.getmtime(f) > os.path.getmtime(_LIB) for f in (_SRC, _SRC_BWD))
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared",
               "-fPIC", "-o", _LIB, _SRC, _SRC_BWD, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_LIB_SAN = os.path.join(_HERE, "libmohge_oracle_san.so")


def build_sanitized() -> str:
    """The oracle under AddressSanitizer + UndefinedBehaviorSanitizer (gcc), as a separate file.
    A process that loads it needs gcc's libasan first in its library list (LD_PRELOAD); the
    environment variable MOHGE_ORACLE_SANITIZED=1 makes this module load it instead of the
    plain build."""
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-shared", "-fPIC", "-o", _LIB_SAN,
           _SRC, _SRC_BWD, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB_SAN


def gcc_asan_runtime() -> str:
    p = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True)
    path = p.stdout.strip()
    return path if p.returncode == 0 and os.path.isabs(path) and os.path.exists(path) else ""


class _Cfg(C.Structure):
    _fields_ = [("T", C.c_int32), ("d", C.c_int32), ("n_groups", C.c_int32),
                ("n_per_group", C.c_int32), ("d_ff", C.POINTER(C.c_int32)),
                ("k_groups", C.c_int32), ("k_experts", C.c_int32),
                ("select_mode", C.c_int32), ("aux_freq_norm", C.c_int32),
                ("alpha_g", C.c_double), ("alpha_e", C.c_double), ("eps", C.c_double)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        if os.environ.get("MOHGE_ORACLE_SANITIZED") == "1":
            _lib = C.CDLL(_LIB_SAN)
        else:
            build(force=False)
            _lib = C.CDLL(_LIB)
        _lib.oracle_num_threads.restype = C.c_int
        for name in ("oracle_route", "oracle_permute", "oracle_expert_ffn", "oracle_combine",
                     "oracle_aux_loss", "oracle_combine_bwd", "oracle_expert_ffn_bwd",
                     "oracle_route_bwd"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _cfg(w, aux_freq_norm: int = 1, alpha_g=None, alpha_e=None):
    dff = (C.c_int32 * w.n_groups)(*w.d_ff)
    c = _Cfg(w.T, w.d, w.n_groups, w.experts_per_group, dff, w.k_groups, w.k_experts,
             w.select_mode, aux_freq_norm,
             float(w.alpha_g if alpha_g is None else alpha_g),
             float(w.alpha_e if alpha_e is None else alpha_e), float(w.eps))
    c._keep = dff
    return c


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"{what}: oracle rejected the configuration (code {rc})")


def route(w, x, w_group, w_expert, bias=None):
    """Section 3.2.  Returns dict(group_idx, expert_idx, gates, gs, es1, margin)."""
    lib = _load()
    c = _cfg(w)
    x, w_group, w_expert = _f32(x), _f32(w_group), _f32(w_expert)
    assert x.shape == (w.T, w.d) and w_group.shape == (w.n_groups, w.d)
    assert w_expert.shape == (w.n_experts, w.d)
    bias = None if bias is None else _f32(bias)
    out = dict(
        group_idx=np.empty((w.T, w.k_groups), np.int32),
        expert_idx=np.empty((w.T, w.k_experts), np.int32),
        gates=np.empty((w.T, w.k_experts), np.float64),
        gs=np.empty((w.T, w.n_groups), np.float64),
        es1=np.empty((w.T, w.n_experts), np.float64),
        margin=np.empty((w.T,), np.float64),
    )
    _check(lib.oracle_route(C.byref(c), _p(x), _p(w_group), _p(w_expert), _p(bias),
                            _p(out["group_idx"]), _p(out["expert_idx"]), _p(out["gates"]),
                            _p(out["gs"]), _p(out["es1"]), _p(out["margin"])), "route")
    return out


def permute(w, expert_idx):
    """Stable bucketing of the (token, slot) pairs by expert."""
    lib = _load()
    c = _cfg(w)
    expert_idx = np.ascontiguousarray(expert_idx, dtype=np.int32)
    assert expert_idx.shape == (w.T, w.k_experts)
    P, Ne = w.n_pairs, w.n_experts
    out = dict(counts=np.empty(Ne, np.int32), offsets=np.empty(Ne + 1, np.int32),
               perm=np.empty(P, np.int32), inv_perm=np.empty(P, np.int32))
    _check(lib.oracle_permute(C.byref(c), _p(expert_idx), _p(out["counts"]), _p(out["offsets"]),
                              _p(out["perm"]), _p(out["inv_perm"])), "permute")
    return out


def _ptr_array(arrs: Sequence[np.ndarray]):
    keep = [_f32(a) for a in arrs]
    arr = (C.c_void_p * len(keep))(*[a.ctypes.data for a in keep])
    return arr, keep


def expert_ffn(w, x, w_gate: List[np.ndarray], w_up: List[np.ndarray], w_down: List[np.ndarray],
               pair_token, pair_expert, want_h: bool = False):
    """E_e(x_t) for the listed pairs.  Returns y_pairs [n, d] (and h [n, max F] if asked)."""
    lib = _load()
    c = _cfg(w)
    x = _f32(x)
    pg, kg = _ptr_array(w_gate)
    pu, ku = _ptr_array(w_up)
    pd, kd = _ptr_array(w_down)
    for g in range(w.n_groups):
        assert kg[g].shape == (w.experts_per_group, w.d_ff[g], w.d)
        assert ku[g].shape == (w.experts_per_group, w.d_ff[g], w.d)
        assert kd[g].shape == (w.experts_per_group, w.d, w.d_ff[g])
    pair_token = np.ascontiguousarray(pair_token, dtype=np.int32)
    pair_expert = np.ascontiguousarray(pair_expert, dtype=np.int32)
    n = pair_token.shape[0]
    assert pair_expert.shape == (n,)
    assert n == 0 or (0 <= pair_token.min() and pair_token.max() < w.T)
    assert n == 0 or (0 <= pair_expert.min() and pair_expert.max() < w.n_experts)
    y = np.empty((n, w.d), np.float64)
    fmax = max(w.d_ff)
    h = np.zeros((n, fmax), np.float64) if want_h else None
    _check(lib.oracle_expert_ffn(C.byref(c), _p(x), pg, pu, pd, C.c_int64(n), _p(pair_token),
                                 _p(pair_expert), _p(y), _p(h), C.c_int64(fmax)), "expert_ffn")
    return (y, h) if want_h else y


def combine(w, y_pairs, gates):
    """y[q] = sum_slot gates[q, slot] * y_pairs[q*K_e + slot] for the n_tok rows given."""
    lib = _load()
    c = _cfg(w)
    gates = np.ascontiguousarray(gates, dtype=np.float64)
    n_tok = gates.shape[0]
    y_pairs = np.ascontiguousarray(y_pairs, dtype=np.float64)
    assert y_pairs.shape == (n_tok * w.k_experts, w.d)
    y = np.empty((n_tok, w.d), np.float64)
    _check(lib.oracle_combine(C.byref(c), C.c_int64(n_tok), _p(y_pairs), _p(gates), _p(y)),
           "combine")
    return y


def aux_loss(w, gs, es1, group_idx, expert_idx, aux_freq_norm: int = 1, alpha_g=None,
             alpha_e=None):
    """Sections 3.3 and 3.4.2.  Returns dict(L_G, L_E, f_G, p_G, f_E, p_E)."""
    lib = _load()
    c = _cfg(w, aux_freq_norm, alpha_g, alpha_e)
    gs = np.ascontiguousarray(gs, dtype=np.float64)
    es1 = np.ascontiguousarray(es1, dtype=np.float64)
    group_idx = np.ascontiguousarray(group_idx, dtype=np.int32)
    expert_idx = np.ascontiguousarray(expert_idx, dtype=np.int32)
    assert gs.shape == (w.T, w.n_groups) and es1.shape == (w.T, w.n_experts)
    losses = np.empty(2, np.float64)
    Ng, Ne = w.n_groups, w.n_experts
    stats = np.empty(2 * Ng + 2 * Ne, np.float64)
    _check(lib.oracle_aux_loss(C.byref(c), _p(gs), _p(es1), _p(group_idx), _p(expert_idx),
                               _p(losses), _p(stats)), "aux_loss")
    return dict(L_G=float(losses[0]), L_E=float(losses[1]), f_G=stats[:Ng].copy(),
                p_G=stats[Ng:2 * Ng].copy(), f_E=stats[2 * Ng:2 * Ng + Ne].copy(),
                p_E=stats[2 * Ng + Ne:].copy())


def shared_experts(w, x, w_gate_s, w_up_s, w_down_s, tokens=None):
    """Always-on experts (architecture table of the appendix; the reading is that every token
    goes through all N_s of them with weight 1): returns sum_s E_s(x_t) [len(tokens), d].
    w_gate_s / w_up_s are [N_s, F_s, d], w_down_s is [N_s, d, F_s]."""
    n_s, f_s = w_down_s.shape[0], w_down_s.shape[2]
    tok = np.arange(x.shape[0], dtype=np.int32) if tokens is None else np.asarray(tokens, np.int32)
    ws = w.replace(T=x.shape[0], d=x.shape[1], n_groups=1, experts_per_group=n_s, d_ff=(f_s,), k_groups=1, k_experts=n_s)
    y_pairs = expert_ffn(ws, x, [w_gate_s], [w_up_s], [w_down_s], np.repeat(tok, n_s),
                         np.tile(np.arange(n_s, dtype=np.int32), len(tok)))
    return combine(ws, y_pairs, np.ones((len(tok), n_s)))


def decode_e4m3(codes):
    """FP8 E4M3 (the OCP 8-bit format without infinities: 1 sign, 4 exponent bits with bias 7, 3
    mantissa bits; exponent field 0 is subnormal, S.1111.111 is NaN, largest finite value 448)
    -> float64.  `codes` is any uint8 array."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    ex = (c >> 3) & 0xF
    man = (c & 0x7).astype(np.float64)
    normal = (1.0 + man / 8.0) * np.exp2((ex - 7).astype(np.float64))
    subnormal = (man / 8.0) * 2.0 ** -6
    val = sign * np.where(ex == 0, subnormal, normal)
    return np.where((ex == 15) & ((c & 0x7) == 7), np.nan, val)


def dequantize_rows(codes, scale):
    """Weights stored as E4M3 codes with one fp32 scale per row (last axis = the row's elements):
    value = scale[row] * decode(code), as float32 (exact: 4 significant bits times an fp32 scale
    rounds once, like the multiplication the kernel's epilogue does on the accumulated sum would
    not; the oracle therefore multiplies the weights, in float64, and rounds nothing)."""
    return decode_e4m3(codes) * np.asarray(scale, np.float64)[..., None]


def decode_e2m1(nibbles):
    """FP4 E2M1 (the OCP microscaling element format: 1 sign, 2 exponent bits with bias 1, 1
    mantissa bit, no infinities or NaN; exponent field 0 is subnormal) -> float64.  `nibbles` is
    any integer array with values 0..15."""
    c = np.asarray(nibbles).astype(np.int64)
    sign = np.where(c & 0x8, -1.0, 1.0)
    ex = (c >> 1) & 0x3
    man = (c & 0x1).astype(np.float64)
    normal = (1.0 + man / 2.0) * np.exp2((ex - 1).astype(np.float64))
    subnormal = man / 2.0
    return sign * np.where(ex == 0, subnormal, normal)


def decode_e8m0(codes):
    """E8M0 block scale of the microscaling formats: 2^(code - 127), code 255 is NaN."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.float64)
    return np.where(c == 255, np.nan, np.exp2(c - 127.0))


def dequantize_mxfp4(packed, scales):
    """Weights stored in the MXFP4 microscaling format: along the last axis, blocks of 32 elements
    share one E8M0 scale; elements are E2M1 codes packed two to a byte, the element with the even
    index in the low four bits.  packed [..., K/2] uint8, scales [..., K/32] uint8 ->
    [..., K] float64 = scale(block) * decode(code), exact."""
    p = np.asarray(packed, dtype=np.uint8)
    lo, hi = p & 0xF, p >> 4
    codes = np.stack([lo, hi], axis=-1).reshape(*p.shape[:-1], p.shape[-1] * 2)
    sc = np.repeat(decode_e8m0(scales), 32, axis=-1)
    assert sc.shape == codes.shape
    return decode_e2m1(codes) * sc


def layer(w, inp, tokens=None):
    """Forward pass of the layer for all tokens, or for the listed token ids.

    Returns dict with the routing of ALL tokens (`route`), the permutation, and
    `y` [len(tokens), d] float64 for the requested tokens, plus `y_pairs`.
    """
    r = route(w, inp.x.f32, inp.w_group, inp.w_expert, inp.expert_logit_bias)
    perm = permute(w, r["expert_idx"])
    tok = np.arange(w.T, dtype=np.int32) if tokens is None else np.asarray(tokens, np.int32)
    pair_token = np.repeat(tok, w.k_experts)
    pair_expert = r["expert_idx"][tok].reshape(-1)
    y_pairs = expert_ffn(w, inp.x.f32, [t.f32 for t in inp.w_gate], [t.f32 for t in inp.w_up],
                         [t.f32 for t in inp.w_down], pair_token, pair_expert)
    y = combine(w, y_pairs, r["gates"][tok])
    return dict(route=r, permute=perm, tokens=tok, y_pairs=y_pairs, y=y)


# ---------------------------------------------------------------------------------------
# Backward pass (chain rule over the forward definitions; see mohge_oracle_bwd.c)
# ---------------------------------------------------------------------------------------

def combine_bwd(w, y_pairs, gates, dy):
    """dgates[q, slot] and dy_pairs[q*K_e+slot] for the n_tok rows given."""
    lib = _load()
    c = _cfg(w)
    gates = np.ascontiguousarray(gates, dtype=np.float64)
    y_pairs = np.ascontiguousarray(y_pairs, dtype=np.float64)
    dy = _f32(dy)
    n_tok = gates.shape[0]
    assert y_pairs.shape == (n_tok * w.k_experts, w.d) and dy.shape == (n_tok, w.d)
    dgates = np.empty((n_tok, w.k_experts), np.float64)
    dy_pairs = np.empty((n_tok * w.k_experts, w.d), np.float64)
    _check(lib.oracle_combine_bwd(C.byref(c), C.c_int64(n_tok), _p(y_pairs), _p(gates), _p(dy),
                                  _p(dgates), _p(dy_pairs)), "combine_bwd")
    return dgates, dy_pairs


def expert_ffn_bwd(w, x, w_gate, w_up, w_down, pair_token, pair_expert, dy_pairs,
                   want_weight_grads: bool = True):
    """Returns dict(dx_pairs [n,d], dw_gate, dw_up, dw_down (lists per group, or None))."""
    lib = _load()
    c = _cfg(w)
    x = _f32(x)
    pg, kg = _ptr_array(w_gate)
    pu, ku = _ptr_array(w_up)
    pd, kd = _ptr_array(w_down)
    for g in range(w.n_groups):
        assert kg[g].shape == (w.experts_per_group, w.d_ff[g], w.d)
        assert ku[g].shape == (w.experts_per_group, w.d_ff[g], w.d)
        assert kd[g].shape == (w.experts_per_group, w.d, w.d_ff[g])
    pair_token = np.ascontiguousarray(pair_token, dtype=np.int32)
    pair_expert = np.ascontiguousarray(pair_expert, dtype=np.int32)
    dy_pairs = np.ascontiguousarray(dy_pairs, dtype=np.float64)
    n = pair_token.shape[0]
    assert pair_expert.shape == (n,) and dy_pairs.shape == (n, w.d)
    assert n == 0 or (0 <= pair_token.min() and pair_token.max() < x.shape[0])
    assert n == 0 or (0 <= pair_expert.min() and pair_expert.max() < w.n_experts)
    dx_pairs = np.zeros((n, w.d), np.float64)
    out = dict(dx_pairs=dx_pairs, dw_gate=None, dw_up=None, dw_down=None)
    tabs = [None, None, None]
    if want_weight_grads:
        out["dw_gate"] = [np.zeros(a.shape, np.float64) for a in kg]
        out["dw_up"] = [np.zeros(a.shape, np.float64) for a in ku]
        out["dw_down"] = [np.zeros(a.shape, np.float64) for a in kd]
        tabs = [(C.c_void_p * w.n_groups)(*[a.ctypes.data for a in out[k]])
                for k in ("dw_gate", "dw_up", "dw_down")]
    _check(lib.oracle_expert_ffn_bwd(C.byref(c), _p(x), pg, pu, pd, C.c_int64(n), _p(pair_token),
                                     _p(pair_expert), _p(dy_pairs), _p(dx_pairs), tabs[0],
                                     tabs[1], tabs[2]), "expert_ffn_bwd")
    return out


def route_bwd(w, x, w_group, w_expert, bias, group_idx, expert_idx, dgates, f_G, f_E,
              alpha_g=None, alpha_e=None):
    """Router backward including both auxiliary losses.  Returns dict(dx, dw_group, dw_expert, dz)."""
    lib = _load()
    c = _cfg(w, 1, alpha_g, alpha_e)
    x, w_group, w_expert = _f32(x), _f32(w_group), _f32(w_expert)
    bias = None if bias is None else _f32(bias)
    group_idx = np.ascontiguousarray(group_idx, dtype=np.int32)
    expert_idx = np.ascontiguousarray(expert_idx, dtype=np.int32)
    dgates = np.ascontiguousarray(dgates, dtype=np.float64)
    f_G = np.ascontiguousarray(f_G, dtype=np.float64)
    f_E = np.ascontiguousarray(f_E, dtype=np.float64)
    assert x.shape == (w.T, w.d) and dgates.shape == (w.T, w.k_experts)
    assert group_idx.shape == (w.T, w.k_groups) and expert_idx.shape == (w.T, w.k_experts)
    assert f_G.shape == (w.n_groups,) and f_E.shape == (w.n_experts,)
    out = dict(dx=np.empty((w.T, w.d), np.float64), dw_group=np.empty((w.n_groups, w.d), np.float64),
               dw_expert=np.empty((w.n_experts, w.d), np.float64),
               dz=np.empty((w.T, w.n_groups + w.n_experts), np.float64))
    _check(lib.oracle_route_bwd(C.byref(c), _p(x), _p(w_group), _p(w_expert), _p(bias),
                                _p(group_idx), _p(expert_idx), _p(dgates), _p(f_G), _p(f_E),
                                _p(out["dx"]), _p(out["dw_group"]), _p(out["dw_expert"]),
                                _p(out["dz"])), "route_bwd")
    return out


def shared_experts_bwd(w, x, dy, w_gate_s, w_up_s, w_down_s):
    """Backward of `shared_experts` for all tokens: every token passes dy[t] (weight 1) to each of
    the N_s experts.  Returns dict(dx [T,d], dw_gate, dw_up [N_s,F_s,d], dw_down [N_s,d,F_s])."""
    n_s, f_s = w_down_s.shape[0], w_down_s.shape[2]
    T = x.shape[0]
    ws = w.replace(T=T, d=x.shape[1], n_groups=1, experts_per_group=n_s, d_ff=(f_s,), k_groups=1, k_experts=n_s)
    pair_token = np.repeat(np.arange(T, dtype=np.int32), n_s)
    pair_expert = np.tile(np.arange(n_s, dtype=np.int32), T)
    dy_pairs = np.repeat(np.asarray(dy, np.float64), n_s, axis=0)
    f = expert_ffn_bwd(ws, x, [w_gate_s], [w_up_s], [w_down_s], pair_token, pair_expert, dy_pairs)
    return dict(dx=f["dx_pairs"].reshape(T, n_s, x.shape[1]).sum(axis=1), dw_gate=f["dw_gate"][0],
                dw_up=f["dw_up"][0], dw_down=f["dw_down"][0])


def layer_bwd(w, inp, dy, fwd=None, alpha_g=None, alpha_e=None):
    """Gradient of  sum(dy*y) + L_G + L_E  for the whole layer (all tokens).

    Returns dict(dx, dw_group, dw_expert, dw_gate, dw_up, dw_down, dgates, dy_pairs, dx_pairs).
    """
    fwd = layer(w, inp) if fwd is None else fwd
    r = fwd["route"]
    aux = aux_loss(w, r["gs"], r["es1"], r["group_idx"], r["expert_idx"], 1, alpha_g, alpha_e)
    dgates, dy_pairs = combine_bwd(w, fwd["y_pairs"], r["gates"], dy)
    pair_token = np.repeat(np.arange(w.T, dtype=np.int32), w.k_experts)
    pair_expert = r["expert_idx"].reshape(-1)
    f = expert_ffn_bwd(w, inp.x.f32, [t.f32 for t in inp.w_gate], [t.f32 for t in inp.w_up],
                       [t.f32 for t in inp.w_down], pair_token, pair_expert, dy_pairs)
    rb = route_bwd(w, inp.x.f32, inp.w_group, inp.w_expert, inp.expert_logit_bias,
                   r["group_idx"], r["expert_idx"], dgates, aux["f_G"], aux["f_E"], alpha_g, alpha_e)
    dx = rb["dx"] + f["dx_pairs"].reshape(w.T, w.k_experts, w.d).sum(axis=1)
    return dict(dx=dx, dw_group=rb["dw_group"], dw_expert=rb["dw_expert"], dw_gate=f["dw_gate"],
                dw_up=f["dw_up"], dw_down=f["dw_down"], dgates=dgates, dy_pairs=dy_pairs,
                dx_pairs=f["dx_pairs"], dz=rb["dz"], dx_route=rb["dx"], aux=aux)
