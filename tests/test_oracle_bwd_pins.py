"""Pins for the backward oracle (oracle/mohge_oracle_bwd.c), none of which re-uses it.

1. Automatic differentiation: the forward definitions of section 3.2 and of the two
   auxiliary losses (3.3, 3.4.2) are written once more in torch float64 tensor algebra
   (dense over all experts, masks from the forward's decisions) and torch.autograd gives
   every gradient of  sum(dy*y) + L_G + L_E.
2. Central finite differences of the oracle's own FORWARD functions.
3. Invariants the chain rule fixes: softmax logit gradients sum to zero inside a group,
   gate normalisation kills the radial direction, linearity in dy, zero-gate experts.
"""
import numpy as np
import pytest
import torch

import oracle
from synth import SELECT_GLOBAL, SELECT_PER_GROUP, WORKLOADS, generate

ALPHA_G, ALPHA_E = 0.7, 0.9   # large on purpose, so that a wrong aux term is visible


def _small(select_mode, seed=21, bias=False, T=24, d=16):
    w = WORKLOADS["tiny_f32"].replace(T=T, d=d, d_ff=(8, 12, 20), select_mode=select_mode,
                                      k_groups=2, k_experts=4, seed=seed, training=True,
                                      skew_beta=1.0 if bias else 0.0)
    inp = generate(w)
    # router weights of the generator are small (0.02): scale them so that sigmoid / softmax
    # are away from their flat regions and the gradients have structure
    inp.w_group = (inp.w_group * 20).astype(np.float32)
    inp.w_expert = (inp.w_expert * 20).astype(np.float32)
    for lst in (inp.w_gate, inp.w_up, inp.w_down):
        for t in lst:
            t.f32 *= np.float32(10.0)
    return w, inp


def _torch_reference(w, inp, fwd):
    """Forward in torch float64, dense over experts, then autograd."""
    T, d, Ng, N = w.T, w.d, w.n_groups, w.experts_per_group
    Ne = Ng * N
    r = fwd["route"]
    dt = torch.float64
    leaf = lambda a: torch.tensor(np.asarray(a, np.float64), dtype=dt, requires_grad=True)
    x, WG, WE = leaf(inp.x.f32), leaf(inp.w_group), leaf(inp.w_expert)
    Wg = [leaf(t.f32) for t in inp.w_gate]
    Wu = [leaf(t.f32) for t in inp.w_up]
    Wd = [leaf(t.f32) for t in inp.w_down]
    bias = torch.zeros(Ne, dtype=dt) if inp.expert_logit_bias is None else torch.tensor(
        inp.expert_logit_bias.astype(np.float64))
    dy = torch.tensor(inp.dy.f32.astype(np.float64))
    gmask = torch.zeros(T, Ng, dtype=dt)
    gmask.scatter_(1, torch.tensor(r["group_idx"].astype(np.int64)), 1.0)
    emask = torch.zeros(T, Ne, dtype=dt)
    emask.scatter_(1, torch.tensor(r["expert_idx"].astype(np.int64)), 1.0)

    GS = torch.sigmoid(x @ WG.T)                                   # group scores
    zE = (x @ WE.T + bias).reshape(T, Ng, N)
    ES1 = torch.softmax(zE, dim=-1) * gmask[:, :, None]            # step 1
    ES2 = (ES1 * GS[:, :, None]).reshape(T, Ne)                    # step 2
    kept = ES2 * emask
    gates = kept / kept.sum(dim=1, keepdim=True)                   # step 3
    y = torch.zeros(T, d, dtype=dt)
    for g in range(Ng):
        for i in range(N):
            a = x @ Wg[g][i].T
            b = x @ Wu[g][i].T
            h = a * torch.sigmoid(a) * b
            y = y + gates[:, g * N + i, None] * (h @ Wd[g][i].T)
    # auxiliary losses, frequencies are constants
    fG = torch.tensor(np.bincount(r["group_idx"].reshape(-1), minlength=Ng) * (Ng / w.k_groups) / T, dtype=dt)
    fE = torch.tensor(np.bincount(r["expert_idx"].reshape(-1), minlength=Ne) * (N / w.k_experts) / T, dtype=dt)
    ratio = torch.tensor(np.asarray(w.d_ff, np.float64) / max(w.d_ff))
    pG = (GS / GS.sum(dim=1, keepdim=True)).mean(dim=0)
    LG = ALPHA_G * (ratio * fG * pG).sum()
    SE = ES1 / (ES1.sum(dim=-1, keepdim=True) + w.eps)
    pE = SE.reshape(T, Ne).mean(dim=0)
    LE = ALPHA_E * (fE * pE).sum()
    L = (dy * y).sum() + LG + LE
    L.backward()
    n = lambda t: t.grad.numpy()
    return dict(dx=n(x), dw_group=n(WG), dw_expert=n(WE), dw_gate=[n(t) for t in Wg],
                dw_up=[n(t) for t in Wu], dw_down=[n(t) for t in Wd], y=y.detach().numpy(),
                LG=float(LG.detach()), LE=float(LE.detach()))


def _close(a, b, rel=1e-9, what=""):
    scale = max(np.abs(b).max(), 1e-300)
    err = np.abs(np.asarray(a) - np.asarray(b)).max()
    assert err <= rel * scale, f"{what}: max err {err:.3e} vs scale {scale:.3e}"


@pytest.mark.parametrize("mode,bias", [(SELECT_GLOBAL, False), (SELECT_PER_GROUP, False),
                                       (SELECT_GLOBAL, True)])
def test_backward_matches_autograd(mode, bias):
    w, inp = _small(mode, bias=bias)
    fwd = oracle.layer(w, inp)
    ref = _torch_reference(w, inp, fwd)
    _close(fwd["y"], ref["y"], 1e-10, "forward y")          # same function on both sides
    got = oracle.layer_bwd(w, inp, inp.dy.f32, fwd, ALPHA_G, ALPHA_E)
    _close(got["aux"]["L_G"], ref["LG"], 1e-10, "L_G")
    _close(got["aux"]["L_E"], ref["LE"], 1e-10, "L_E")
    for k in ("dx", "dw_group", "dw_expert"):
        _close(got[k], ref[k], 1e-9, k)
    for k in ("dw_gate", "dw_up", "dw_down"):
        for g in range(w.n_groups):
            _close(got[k][g], ref[k][g], 1e-9, f"{k}[{g}]")
    # every tensor has a non-trivial gradient, so the comparison above is not vacuous
    assert min(np.abs(got[k]).max() for k in ("dx", "dw_group", "dw_expert")) > 1e-6


def test_aux_only_gradient_matches_autograd():
    # dy = 0 leaves only the two auxiliary losses: their router gradients alone
    w, inp = _small(SELECT_GLOBAL, seed=22)
    inp.dy.f32[:] = 0
    fwd = oracle.layer(w, inp)
    ref = _torch_reference(w, inp, fwd)
    got = oracle.layer_bwd(w, inp, inp.dy.f32, fwd, ALPHA_G, ALPHA_E)
    for k in ("dx", "dw_group", "dw_expert"):
        assert np.abs(ref[k]).max() > 1e-8
        _close(got[k], ref[k], 1e-9, k)
    for g in range(w.n_groups):
        assert np.abs(got["dw_gate"][g]).max() == 0.0


def _objective(w, inp):
    f = oracle.layer(w, inp)
    r = f["route"]
    a = oracle.aux_loss(w, r["gs"], r["es1"], r["group_idx"], r["expert_idx"], 1, ALPHA_G, ALPHA_E)
    return float((inp.dy.f32.astype(np.float64) * f["y"]).sum() + a["L_G"] + a["L_E"]), r


def test_backward_matches_finite_differences_of_the_forward_oracle():
    w, inp = _small(SELECT_PER_GROUP, seed=23, T=10, d=8)
    fwd = oracle.layer(w, inp)
    assert fwd["route"]["margin"].min() > 0.01           # decisions stay put under the probes
    got = oracle.layer_bwd(w, inp, inp.dy.f32, fwd, ALPHA_G, ALPHA_E)
    rng = np.random.default_rng(5)
    h = 2.0 ** -9
    targets = [("dx", inp.x.f32), ("dw_group", inp.w_group), ("dw_expert", inp.w_expert)]
    for g in range(w.n_groups):
        targets += [(("dw_gate", g), inp.w_gate[g].f32), (("dw_up", g), inp.w_up[g].f32),
                    (("dw_down", g), inp.w_down[g].f32)]
    for key, arr in targets:
        grad = got[key] if isinstance(key, str) else got[key[0]][key[1]]
        flat = arr.reshape(-1)
        scale = np.abs(grad).max()
        for idx in rng.choice(flat.size, size=6, replace=False):
            old = flat[idx]
            flat[idx] = old + np.float32(h)
            up, r1 = _objective(w, inp)
            flat[idx] = old - np.float32(h)
            dn, r2 = _objective(w, inp)
            step = float(np.float32(old + np.float32(h)) - np.float32(old - np.float32(h)))
            flat[idx] = old
            assert (r1["expert_idx"] == fwd["route"]["expert_idx"]).all()
            assert (r2["expert_idx"] == fwd["route"]["expert_idx"]).all()
            fd = (up - dn) / step
            assert abs(fd - grad.reshape(-1)[idx]) <= 2e-4 * scale + 1e-9, (key, idx, fd, grad.reshape(-1)[idx])


def test_chain_rule_invariants():
    w, inp = _small(SELECT_GLOBAL, seed=24)
    fwd = oracle.layer(w, inp)
    r = fwd["route"]
    Ng, N = w.n_groups, w.experts_per_group
    got = oracle.layer_bwd(w, inp, inp.dy.f32, fwd, 0.0, 0.0)
    # softmax: the expert-logit gradients of one group sum to zero; unselected groups get none
    dzE = got["dz"][:, Ng:].reshape(w.T, Ng, N)
    assert np.abs(dzE.sum(axis=2)).max() < 1e-12 * max(1.0, np.abs(dzE).max())
    sel = np.zeros((w.T, Ng), bool)
    np.put_along_axis(sel, r["group_idx"], True, axis=1)
    assert (dzE[~sel] == 0).all() and np.abs(dzE[sel]).max() > 0
    # without auxiliary losses an unselected group's score has no influence at all
    assert (got["dz"][:, :Ng][~sel] == 0).all()
    # gates sum to one: adding a constant to every dgate of a token changes nothing
    rb0 = oracle.route_bwd(w, inp.x.f32, inp.w_group, inp.w_expert, None, r["group_idx"],
                           r["expert_idx"], got["dgates"], np.zeros(Ng), np.zeros(Ng * N), 0.0, 0.0)
    rb1 = oracle.route_bwd(w, inp.x.f32, inp.w_group, inp.w_expert, None, r["group_idx"],
                           r["expert_idx"], got["dgates"] + 3.25, np.zeros(Ng), np.zeros(Ng * N), 0.0, 0.0)
    _close(rb1["dx"], rb0["dx"], 1e-9, "gate shift")
    # linear in dy when the auxiliary losses are off
    got2 = oracle.layer_bwd(w, inp, 2.0 * inp.dy.f32, fwd, 0.0, 0.0)
    for k in ("dx", "dw_group", "dw_expert"):
        _close(got2[k], 2.0 * got[k], 1e-12, k)
    _close(got2["dw_down"][1], 2.0 * got["dw_down"][1], 1e-12, "dw_down")
    # an expert no token chose has zero weight gradients
    counts = np.bincount(r["expert_idx"].reshape(-1), minlength=Ng * N)
    for e in np.nonzero(counts == 0)[0]:
        assert np.abs(got["dw_gate"][e // N][e % N]).max() == 0.0
    # the layer gradient is the router part plus the sum of the token's pairs
    _close(got["dx"], got["dx_route"] + got["dx_pairs"].reshape(w.T, w.k_experts, w.d).sum(1), 1e-15, "dx split")


def test_single_expert_reduces_to_a_dense_swiglu_mlp():
    # N_g = 1, N = 1, K = 1: gate == 1 whatever the router says, so the layer is one dense
    # SwiGLU block whose gradients have a closed matrix form
    w = WORKLOADS["tiny_f32"].replace(T=9, d=8, n_groups=1, experts_per_group=1, d_ff=(12,),
                                      k_groups=1, k_experts=1, seed=25, training=True)
    inp = generate(w)
    for t in (inp.w_gate[0], inp.w_up[0], inp.w_down[0]):
        t.f32 *= np.float32(10.0)
    got = oracle.layer_bwd(w, inp, inp.dy.f32, None, 0.0, 0.0)
    X = inp.x.f32.astype(np.float64)
    G, U, Dn = (t.f32[0].astype(np.float64) for t in (inp.w_gate[0], inp.w_up[0], inp.w_down[0]))
    dY = inp.dy.f32.astype(np.float64)
    A, B = X @ G.T, X @ U.T
    S = 1 / (1 + np.exp(-A))
    H = A * S * B
    dH = dY @ Dn
    dA = dH * B * (S + A * S * (1 - S))
    dB = dH * A * S
    _close(got["dw_down"][0][0], dY.T @ H, 1e-12, "dW_down")
    _close(got["dw_gate"][0][0], dA.T @ X, 1e-12, "dW_gate")
    _close(got["dw_up"][0][0], dB.T @ X, 1e-12, "dW_up")
    _close(got["dx"], dA @ G + dB @ U, 1e-12, "dx")
    assert np.abs(got["dw_expert"]).max() < 1e-18 and np.abs(got["dgates"]).max() > 0


def test_shared_experts_backward_matches_autograd():
    """Always-on experts: y[t] = sum_s W_down_s (SiLU(W_gate_s x_t) * (W_up_s x_t)), written in torch
    float64; autograd of sum(dy*y) against the oracle's composition."""
    rng = np.random.default_rng(5)
    T, d, n_s, f_s = 13, 10, 3, 7
    x = rng.standard_normal((T, d)).astype(np.float32)
    dy = rng.standard_normal((T, d)).astype(np.float32)
    g_s = rng.standard_normal((n_s, f_s, d)).astype(np.float32) * 0.5
    u_s = rng.standard_normal((n_s, f_s, d)).astype(np.float32) * 0.5
    d_s = rng.standard_normal((n_s, d, f_s)).astype(np.float32) * 0.5
    w = WORKLOADS["tiny_f32"]
    got = oracle.shared_experts_bwd(w, x, dy, g_s, u_s, d_s)
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tg, tu, td = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (g_s, u_s, d_s))
    y = torch.zeros((T, d), dtype=torch.float64)
    for s in range(n_s):
        a, b = tx @ tg[s].T, tx @ tu[s].T
        y = y + (torch.nn.functional.silu(a) * b) @ td[s].T
    # the forward agrees with the oracle's forward first
    assert np.allclose(y.detach().numpy(), oracle.shared_experts(w, x, g_s, u_s, d_s), rtol=1e-10, atol=1e-12)
    (y * torch.tensor(dy, dtype=torch.float64)).sum().backward()
    for name, ref in (("dx", tx.grad), ("dw_gate", tg.grad), ("dw_up", tu.grad), ("dw_down", td.grad)):
        assert np.allclose(got[name], ref.numpy(), rtol=1e-9, atol=1e-11), name
