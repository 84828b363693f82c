"""Independent numpy / brute-force references used ONLY to pin the CPU oracle.

They are written in a different style from the oracle (whole-array operations,
stable sorts, subset enumeration, library matmuls) so that a slip in one is not
repeated in the other.  Nothing here is used by the HIP library or its tests.
"""
from __future__ import annotations

import itertools

import numpy as np


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def topk_mask_sorted(key: np.ndarray, k: int) -> np.ndarray:
    """Boolean mask of the k largest entries along the last axis; a stable sort
    of the negated key puts the lowest index first among equals."""
    order = np.argsort(-key, axis=-1, kind="stable")
    mask = np.zeros(key.shape, dtype=bool)
    np.put_along_axis(mask, order[..., :k], True, axis=-1)
    return mask


def dense_routing(x, w_group, w_expert, bias, n_groups, n_per, k_groups, k_experts, mode):
    """Dense ES[T, N_e] (zeros off the kept experts), GS[T,N_g], ES'[T,N_e] and the
    group mask, from whole-array float64 operations (section 3.2)."""
    x = np.asarray(x, np.float64)
    zG = x @ np.asarray(w_group, np.float64).T
    GS = sigmoid(zG)
    gmask = topk_mask_sorted(zG, k_groups)                       # [T, N_g]
    zE = x @ np.asarray(w_expert, np.float64).T
    if bias is not None:
        zE = zE + np.asarray(bias, np.float64)[None, :]
    T = x.shape[0]
    zE3 = zE.reshape(T, n_groups, n_per)
    sm = np.exp(zE3 - zE3.max(axis=2, keepdims=True))
    sm = sm / sm.sum(axis=2, keepdims=True)
    es1 = np.where(gmask[:, :, None], sm, 0.0)
    es2 = es1 * GS[:, :, None]
    if mode == 0:
        key = np.where(gmask[:, :, None], es2, -np.inf).reshape(T, -1)
        emask = topk_mask_sorted(key, k_experts)
    else:
        k = k_experts // k_groups
        key = np.where(gmask[:, :, None], zE3, -np.inf)
        emask = (topk_mask_sorted(key, k) & gmask[:, :, None]).reshape(T, -1)
    es3 = np.where(emask, es2.reshape(T, -1), 0.0)
    ES = es3 / es3.sum(axis=1, keepdims=True)
    return dict(ES=ES, GS=GS, es1=es1.reshape(T, -1), gmask=gmask, emask=emask, zG=zG, zE=zE,
                es2=es2.reshape(T, -1))


def best_subset(key: np.ndarray, cand, k: int):
    """Brute force: the k-subset of `cand` with the largest key sum; among equal
    sums the lexicographically smallest index tuple."""
    best, best_sum = None, None
    for sub in itertools.combinations(sorted(cand), k):
        s = sum(key[j] for j in sub)
        if best is None or s > best_sum:
            best, best_sum = sub, s
    return best


def dense_layer(x, ES, w_gate, w_up, w_down, n_per):
    """Apply EVERY expert to every token with library matmuls, weight by the dense
    gate matrix ES and add up (appendix, background: y = sum_i G_i(x) E_i(x))."""
    x = np.asarray(x, np.float64)
    y = np.zeros_like(x)
    for g in range(len(w_gate)):
        for i in range(n_per):
            a = x @ np.asarray(w_gate[g][i], np.float64).T
            b = x @ np.asarray(w_up[g][i], np.float64).T
            h = a * sigmoid(a) * b
            y += ES[:, g * n_per + i][:, None] * (h @ np.asarray(w_down[g][i], np.float64).T)
    return y
