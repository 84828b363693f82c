"""Pins for the CPU oracle: it is checked against things other than itself.

 - numbers worked by hand from the paper's equations (tests/golden);
 - brute-force subset enumeration for both top-k levels;
 - invariants the definitions fix (gates sum to 1, exactly K_e experts inside the
   kept groups, counts sum to T*K_e, the permutation is a stable bijection);
 - special cases that reduce to textbook / library routines (softmax over top-k
   logits, normalised sigmoid top-k, a dense SwiGLU MLP);
 - a dense reference (every expert applied, masked by gates) built from numpy
   matmuls and sort-based selection;
 - closed forms of both auxiliary losses.
All run on the CPU.
"""
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle
from synth import SELECT_GLOBAL, SELECT_PER_GROUP, Workload, WORKLOADS, generate

from np_reference import best_subset, dense_layer, dense_routing, sigmoid


def small(name="s", **kw):
    base = dict(T=48, d=32, n_groups=3, experts_per_group=4, d_ff=(16, 24, 40), k_groups=2,
                k_experts=2, dtype="f32", seed=5)
    base.update(kw)
    return Workload(name, **base)


# --------------------------------------------------------------------------
# hand-worked numbers
# --------------------------------------------------------------------------
def _hand_case(golden_dir):
    with open(os.path.join(golden_dir, "handworked_routing.json")) as f:
        return json.load(f)


def test_handworked_routing_and_losses(golden_dir):
    G = _hand_case(golden_dir)
    d, Ng, N = G["d"], G["n_groups"], G["experts_per_group"]
    x = np.asarray([G["x"]], np.float32)
    wG = np.zeros((Ng, d), np.float32)
    wE = np.zeros((Ng * N, d), np.float32)
    wG[:, 0] = np.log(np.asarray(G["w_group_col0_ln"], np.float64))
    wE[:, 0] = np.log(np.asarray(G["w_expert_col0_ln"], np.float64))
    for case in G["cases"]:
        w = Workload("hand", T=1, d=d, n_groups=Ng, experts_per_group=N, d_ff=tuple(G["d_ff"]),
                     k_groups=case["k_groups"], k_experts=case["k_experts"],
                     select_mode=case["select_mode"], dtype="f32", alpha_g=1.0, alpha_e=1.0)
        r = oracle.route(w, x, wG, wE)
        assert r["group_idx"][0].tolist() == case["group_idx"]
        assert r["expert_idx"][0].tolist() == case["expert_idx"]
        np.testing.assert_allclose(r["gates"][0], case["gates"], atol=2e-7)
        np.testing.assert_allclose(r["gs"][0], G["gs"], atol=2e-7)
        np.testing.assert_allclose(r["es1"][0], case["es1"], atol=2e-7)
        assert abs(r["margin"][0] - case["margin"]) < 2e-7
        a = oracle.aux_loss(w, r["gs"], r["es1"], r["group_idx"], r["expert_idx"])
        assert abs(a["L_G"] - case["L_G"]) < 1e-6
        assert abs(a["L_E"] - case["L_E"] / (1.0 + w.eps)) < 1e-6


def test_handworked_permutation(golden_dir):
    ex = _hand_case(golden_dir)["permute_example"]
    w = Workload("p", T=4, d=4, n_groups=2, experts_per_group=2, d_ff=(8, 8), k_groups=2,
                 k_experts=2, dtype="f32")
    p = oracle.permute(w, np.asarray(ex["expert_idx"], np.int32))
    for k in ("counts", "offsets", "perm", "inv_perm"):
        assert p[k].tolist() == ex[k], k


# --------------------------------------------------------------------------
# brute force and invariants
# --------------------------------------------------------------------------
@pytest.mark.parametrize("mode", [SELECT_GLOBAL, SELECT_PER_GROUP])
@pytest.mark.parametrize("shape", [(3, 4, 2, 2), (4, 3, 3, 6), (2, 5, 1, 1), (4, 4, 2, 4), (3, 2, 3, 3)])
def test_selection_matches_brute_force(mode, shape):
    Ng, N, Kg, Ke = shape
    w = small(n_groups=Ng, experts_per_group=N, d_ff=tuple([16] * Ng), k_groups=Kg, k_experts=Ke,
              select_mode=mode, T=40, seed=17 + Ng * 7 + N)
    inp = generate(w)
    wG, wE = inp.w_group * 20, inp.w_expert * 20          # spread the scores out
    r = oracle.route(w, inp.x.f32, wG, wE)
    ref = dense_routing(inp.x.f32, wG, wE, None, Ng, N, Kg, Ke, mode)
    for t in range(w.T):
        groups = best_subset(ref["zG"][t], range(Ng), Kg)
        assert tuple(r["group_idx"][t]) == groups
        GS = sigmoid(ref["zG"][t])
        # ES'' recomputed here for the brute-force groups
        es2 = np.full(Ng * N, -np.inf)
        for g in groups:
            z = ref["zE"][t, g * N:(g + 1) * N]
            p = np.exp(z - z.max())
            es2[g * N:(g + 1) * N] = p / p.sum() * GS[g]
        if mode == SELECT_GLOBAL:
            cand = [g * N + i for g in groups for i in range(N)]
            experts = best_subset(es2, cand, Ke)
        else:
            experts = ()
            for g in groups:
                experts += best_subset(ref["zE"][t], range(g * N, (g + 1) * N), Ke // Kg)
        assert tuple(r["expert_idx"][t]) == tuple(sorted(experts))
        kept = np.asarray([es2[e] for e in sorted(experts)])
        np.testing.assert_allclose(r["gates"][t], kept / kept.sum(), rtol=1e-12)


def test_ties_go_to_lowest_index():
    # an all-zero router makes every score equal
    w = small(T=5, k_groups=2, k_experts=4, select_mode=SELECT_PER_GROUP)
    inp = generate(w)
    for mode in (SELECT_GLOBAL, SELECT_PER_GROUP):
        w2 = w.replace(select_mode=mode)
        r = oracle.route(w2, inp.x.f32, np.zeros_like(inp.w_group), np.zeros_like(inp.w_expert))
        assert (r["group_idx"] == np.asarray([0, 1])).all()
        expect = [0, 1, 2, 3] if mode == SELECT_GLOBAL else [0, 1, 4, 5]
        assert (r["expert_idx"] == np.asarray(expect)).all()
        np.testing.assert_allclose(r["gates"], 0.25, rtol=1e-12)
        assert (r["margin"] == 0).all()


@pytest.mark.parametrize("mode", [SELECT_GLOBAL, SELECT_PER_GROUP])
@pytest.mark.parametrize("name", ["tiny_f32", "paper_1b"])
def test_routing_invariants(mode, name):
    w = WORKLOADS[name].replace(select_mode=mode, T=96, d=64)
    if mode == SELECT_PER_GROUP and w.k_experts % w.k_groups:
        pytest.skip("not divisible")
    inp = generate(w)
    r = oracle.route(w, inp.x.f32, inp.w_group * 8, inp.w_expert * 8)
    N = w.experts_per_group
    np.testing.assert_allclose(r["gates"].sum(axis=1), 1.0, atol=1e-12)
    assert (r["gates"] > 0).all()
    for t in range(w.T):
        e = r["expert_idx"][t]
        g = r["group_idx"][t]
        assert len(set(e.tolist())) == w.k_experts and (np.diff(e) > 0).all()
        assert len(set(g.tolist())) == w.k_groups and (np.diff(g) > 0).all()
        assert set((e // N).tolist()) <= set(g.tolist())
        if mode == SELECT_PER_GROUP:
            assert np.bincount(e // N, minlength=w.n_groups)[g].tolist() == \
                [w.k_experts // w.k_groups] * w.k_groups
        rows = r["es1"][t].reshape(w.n_groups, N).sum(axis=1)
        sel = np.zeros(w.n_groups, bool)
        sel[g] = True
        np.testing.assert_allclose(rows[sel], 1.0, atol=1e-12)
        assert (rows[~sel] == 0).all()
    p = oracle.permute(w, r["expert_idx"])
    P = w.n_pairs
    assert p["counts"].sum() == P
    assert p["offsets"][0] == 0 and (np.diff(p["offsets"]) == p["counts"]).all()
    assert sorted(p["perm"].tolist()) == list(range(P))
    assert (p["inv_perm"][p["perm"]] == np.arange(P)).all()
    e_sorted = r["expert_idx"].reshape(-1)[p["perm"]]
    assert (np.diff(e_sorted) >= 0).all()
    same = np.diff(e_sorted) == 0
    assert (np.diff(p["perm"])[same] > 0).all()      # stable inside a bucket
    assert (np.bincount(r["expert_idx"].reshape(-1), minlength=w.n_experts) == p["counts"]).all()


# --------------------------------------------------------------------------
# special cases that reduce to textbook routines
# --------------------------------------------------------------------------
def test_single_group_is_softmax_over_topk_logits():
    # N_g = 1: GS cancels in the normalisation, leaving the standard MoE gate of
    # the appendix: softmax over the top-k logits.
    w = small(n_groups=1, experts_per_group=8, d_ff=(16,), k_groups=1, k_experts=3,
              select_mode=SELECT_GLOBAL)
    inp = generate(w)
    wE = inp.w_expert * 10
    r = oracle.route(w, inp.x.f32, inp.w_group, wE)
    logits = torch.from_numpy(inp.x.f32.astype(np.float64) @ wE.astype(np.float64).T)
    top = torch.topk(logits, 3, dim=1)
    gate = torch.softmax(top.values, dim=1)
    order = torch.argsort(top.indices, dim=1)
    assert (r["expert_idx"] == torch.gather(top.indices, 1, order).numpy()).all()
    np.testing.assert_allclose(r["gates"], torch.gather(gate, 1, order).numpy(), rtol=1e-12)


def test_one_expert_per_group_is_normalised_sigmoid_topk():
    w = small(n_groups=6, experts_per_group=1, d_ff=tuple([16] * 6), k_groups=3, k_experts=3,
              select_mode=SELECT_GLOBAL)
    inp = generate(w)
    wG = inp.w_group * 10
    for mode in (SELECT_GLOBAL, SELECT_PER_GROUP):
        r = oracle.route(w.replace(select_mode=mode), inp.x.f32, wG, inp.w_expert)
        z = torch.from_numpy(inp.x.f32.astype(np.float64) @ wG.astype(np.float64).T)
        top = torch.topk(z, 3, dim=1)
        idx, _ = torch.sort(top.indices, dim=1)
        s = torch.sigmoid(torch.gather(z, 1, idx))
        assert (r["expert_idx"] == idx.numpy()).all() and (r["group_idx"] == idx.numpy()).all()
        np.testing.assert_allclose(r["gates"], (s / s.sum(1, keepdim=True)).numpy(), rtol=1e-12)


def test_keep_all_experts_of_kept_groups():
    # K_e = K_g*N: gate = ES' * GS / sum of kept GS
    w = small(k_groups=2, k_experts=8, select_mode=SELECT_GLOBAL)
    inp = generate(w)
    r = oracle.route(w, inp.x.f32, inp.w_group * 10, inp.w_expert * 10)
    N = w.experts_per_group
    for t in range(w.T):
        g = r["group_idx"][t]
        expect = [r["es1"][t, e] * r["gs"][t, e // N] / r["gs"][t, g].sum() for e in r["expert_idx"][t]]
        np.testing.assert_allclose(r["gates"][t], expect, rtol=1e-12)
    assert np.isinf(r["margin"]).sum() == 0      # group level still rejects one group


def test_group_weight_as_mean_of_expert_embeddings():
    # the other reading of "centroid": W_G[g] = mean_i W_E[g,i]; same interface
    w = small()
    inp = generate(w)
    wE = inp.w_expert * 10
    wG = wE.reshape(w.n_groups, w.experts_per_group, w.d).mean(axis=1)
    r = oracle.route(w, inp.x.f32, wG, wE)
    zE = inp.x.f32.astype(np.float64) @ wE.astype(np.float64).T
    zG = zE.reshape(w.T, w.n_groups, -1).mean(axis=2)
    np.testing.assert_allclose(r["gs"], sigmoid(zG), rtol=1e-6)


# --------------------------------------------------------------------------
# expert network and the whole layer
# --------------------------------------------------------------------------
def test_single_expert_is_dense_swiglu_mlp():
    w = small(n_groups=1, experts_per_group=1, d_ff=(24,), k_groups=1, k_experts=1)
    inp = generate(w)
    tok = np.arange(w.T, dtype=np.int32)
    y, h = oracle.expert_ffn(w, inp.x.f32, [inp.w_gate[0].f32], [inp.w_up[0].f32],
                             [inp.w_down[0].f32], tok, np.zeros(w.T, np.int32), want_h=True)
    X = torch.from_numpy(inp.x.f32).double()
    Wg, Wu, Wd = (torch.from_numpy(a[0].f32[0]).double() for a in (inp.w_gate, inp.w_up, inp.w_down))
    H = torch.nn.functional.silu(X @ Wg.T) * (X @ Wu.T)
    np.testing.assert_allclose(h, H.numpy(), rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(y, (H @ Wd.T).numpy(), rtol=1e-10, atol=1e-14)
    # linear in W_down
    y3 = oracle.expert_ffn(w, inp.x.f32, [inp.w_gate[0].f32], [inp.w_up[0].f32],
                           [inp.w_down[0].f32 * 4.0], tok, np.zeros(w.T, np.int32))
    np.testing.assert_allclose(y3, 4.0 * y, rtol=1e-12)


@pytest.mark.parametrize("mode", [SELECT_GLOBAL, SELECT_PER_GROUP])
@pytest.mark.parametrize("skew", [0.0, 2.0])
def test_layer_matches_dense_masked_reference(mode, skew):
    w = small(select_mode=mode, skew_beta=skew, k_experts=4, T=40)
    inp = generate(w)
    inp.w_group *= 10
    inp.w_expert *= 10
    out = oracle.layer(w, inp)
    ref = dense_routing(inp.x.f32, inp.w_group, inp.w_expert, inp.expert_logit_bias, w.n_groups,
                        w.experts_per_group, w.k_groups, w.k_experts, mode)
    # routing agrees with the sort-based whole-array implementation
    ES = np.zeros((w.T, w.n_experts))
    np.put_along_axis(ES, out["route"]["expert_idx"].astype(np.int64), out["route"]["gates"], axis=1)
    np.testing.assert_allclose(ES, ref["ES"], rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(out["route"]["gs"], ref["GS"], rtol=1e-12)
    np.testing.assert_allclose(out["route"]["es1"], ref["es1"], rtol=1e-11, atol=1e-15)
    y_dense = dense_layer(inp.x.f32, ref["ES"], [t.f32 for t in inp.w_gate],
                          [t.f32 for t in inp.w_up], [t.f32 for t in inp.w_down],
                          w.experts_per_group)
    np.testing.assert_allclose(out["y"], y_dense, rtol=1e-9, atol=1e-12 * np.abs(y_dense).max())
    assert np.abs(y_dense).max() > 0


def test_layer_on_token_subset_equals_full():
    w = small(k_experts=4)
    inp = generate(w)
    full = oracle.layer(w, inp)
    sub = oracle.layer(w, inp, tokens=[3, 17, 40])
    np.testing.assert_array_equal(sub["y"], full["y"][[3, 17, 40]])


def test_equal_widths_single_group_is_standard_topk_moe():
    # N_g = 1 and one width: the layer is the standard MoE layer of the appendix
    w = small(n_groups=1, experts_per_group=6, d_ff=(24,), k_groups=1, k_experts=2,
              select_mode=SELECT_GLOBAL)
    inp = generate(w)
    inp.w_expert *= 10
    out = oracle.layer(w, inp)
    X = torch.from_numpy(inp.x.f32).double()
    logits = X @ torch.from_numpy(inp.w_expert).double().T
    top = torch.topk(logits, 2, dim=1)
    gate = torch.softmax(top.values, dim=1)
    y = torch.zeros_like(X)
    for t in range(w.T):
        for s in range(2):
            i = int(top.indices[t, s])
            Wg, Wu, Wd = (torch.from_numpy(a[0].f32[i]).double() for a in (inp.w_gate, inp.w_up, inp.w_down))
            y[t] += gate[t, s] * (Wd @ (torch.nn.functional.silu(Wg @ X[t]) * (Wu @ X[t])))
    np.testing.assert_allclose(out["y"], y.numpy(), rtol=1e-10, atol=1e-14)


# --------------------------------------------------------------------------
# auxiliary losses
# --------------------------------------------------------------------------
@pytest.mark.parametrize("mode", [SELECT_GLOBAL, SELECT_PER_GROUP])
def test_aux_losses_closed_form_for_zero_router(mode):
    # All scores tie: groups 0..K_g-1 and the lowest experts are always taken,
    # s' = 1/N_g, ES' = 1/N inside kept groups.
    w = small(select_mode=mode, k_groups=2, k_experts=4, alpha_g=0.3, alpha_e=0.7, T=20)
    inp = generate(w)
    r = oracle.route(w, inp.x.f32, np.zeros_like(inp.w_group), np.zeros_like(inp.w_expert))
    a = oracle.aux_loss(w, r["gs"], r["es1"], r["group_idx"], r["expert_idx"])
    ratios = np.asarray(w.d_ff) / max(w.d_ff)
    # f^G = N_g/K_g on kept groups, p^G = 1/N_g
    LG = w.alpha_g * sum(ratios[g] * (w.n_groups / w.k_groups) * (1 / w.n_groups) for g in range(w.k_groups))
    assert abs(a["L_G"] - LG) < 1e-12
    # sum f^E = N, and p^E = 1/N/(1+eps) on every expert of a kept group
    LE = w.alpha_e / (1 + w.eps)
    assert abs(a["L_E"] - LE) < 1e-12
    lit = oracle.aux_loss(w, r["gs"], r["es1"], r["group_idx"], r["expert_idx"], aux_freq_norm=0)
    assert abs(lit["L_G"] - w.T * a["L_G"]) < 1e-9 and abs(lit["L_E"] - w.T * a["L_E"]) < 1e-9


@pytest.mark.parametrize("mode", [SELECT_GLOBAL, SELECT_PER_GROUP])
def test_aux_loss_invariants_and_whole_array_form(mode):
    w = small(select_mode=mode, k_groups=2, k_experts=4, alpha_g=1.0, alpha_e=1.0, T=64)
    inp = generate(w)
    r = oracle.route(w, inp.x.f32, inp.w_group * 10, inp.w_expert * 10)
    a = oracle.aux_loss(w, r["gs"], r["es1"], r["group_idx"], r["expert_idx"])
    Ng, N, T = w.n_groups, w.experts_per_group, w.T
    assert abs(a["f_G"].sum() - Ng) < 1e-12
    assert abs(a["p_G"].sum() - 1.0) < 1e-12
    assert abs(a["f_E"].sum() - N) < 1e-12
    np.testing.assert_allclose(a["p_E"].reshape(Ng, N).sum(1),
                               (w.k_groups / Ng) * a["f_G"] / (1 + w.eps), rtol=1e-12)
    # whole-array restatement from the dense reference's masks
    ref = dense_routing(inp.x.f32, inp.w_group * 10, inp.w_expert * 10, None, Ng, N, w.k_groups,
                        w.k_experts, mode)
    fG = Ng / w.k_groups * ref["gmask"].mean(0)
    pG = (ref["GS"] / ref["GS"].sum(1, keepdims=True)).mean(0)
    LG = (np.asarray(w.d_ff) / max(w.d_ff) * fG * pG).sum()
    fE = N / w.k_experts * ref["emask"].mean(0)
    es1 = ref["es1"].reshape(T, Ng, N)
    pE = (es1 / (es1.sum(2, keepdims=True) + w.eps)).mean(0).reshape(-1)
    assert abs(a["L_G"] - LG) < 1e-12 and abs(a["L_E"] - (fE * pE).sum()) < 1e-12


def test_intra_group_loss_single_group_is_expert_level_balance_loss():
    # N_g = 1: L_E is the expert-level balance loss it was adapted from:
    # alpha * sum_i f_i P_i, f_i = N/(K T) * #(i kept), P_i = mean softmax prob.
    w = small(n_groups=1, experts_per_group=8, d_ff=(16,), k_groups=1, k_experts=2,
              select_mode=SELECT_GLOBAL, alpha_e=1.0, T=64)
    inp = generate(w)
    wE = inp.w_expert * 10
    r = oracle.route(w, inp.x.f32, inp.w_group, wE)
    a = oracle.aux_loss(w, r["gs"], r["es1"], r["group_idx"], r["expert_idx"])
    logits = torch.from_numpy(inp.x.f32.astype(np.float64) @ wE.astype(np.float64).T)
    prob = torch.softmax(logits, dim=1)
    kept = torch.zeros_like(prob).scatter_(1, torch.topk(prob, 2, dim=1).indices, 1.0)
    f = 8 / (2 * w.T) * kept.sum(0)
    P = prob.mean(0)
    assert abs(a["L_E"] - float((f * P).sum()) / (1 + w.eps)) < 1e-9
    # and L_G with one group: f = 1, p = 1, ratio 1
    assert abs(a["L_G"] - w.alpha_g) < 1e-15


def test_oracle_rejects_bad_configs():
    w = small()
    inp = generate(w)
    for bad in (w.replace(k_groups=4), w.replace(k_experts=9), w.replace(k_experts=3, select_mode=SELECT_PER_GROUP)):
        with pytest.raises(ValueError):
            oracle.route(bad, inp.x.f32, inp.w_group, inp.w_expert)


def test_synth_bf16_rounding_is_nearest_even():
    from synth import bf16_bits_to_f32, f32_to_bf16_bits
    a = np.asarray([1.0, 1.00390625, 1.01171875, -2.5, 3.140625, 1e-3], np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: even mantissa (1.0) wins;
    # 1 + 3*2^-8 ties between 1+2^-7 (odd) and 1+2^-6 (even): goes up.
    got = bf16_bits_to_f32(f32_to_bf16_bits(a))
    ref = torch.from_numpy(a).to(torch.bfloat16).float().numpy()
    np.testing.assert_array_equal(got, ref)
    assert got[1] == 1.0 and got[2] == 1.015625
    big = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    np.testing.assert_array_equal(bf16_bits_to_f32(f32_to_bf16_bits(big)),
                                  torch.from_numpy(big).to(torch.bfloat16).float().numpy())


def test_skewed_workload_counts_range_over_ten_x():
    # routing only (cheap) at the full skewed shape's expert layout, fewer tokens and d
    w = WORKLOADS["large_prefill_skewed"].replace(T=8192, d=256)
    inp = generate(w)
    # keep the logit scale of the full shape: std 0.02*sqrt(4096)
    s = math.sqrt(4096 / w.d)
    r = oracle.route(w, inp.x.f32, inp.w_group * s, inp.w_expert * s, inp.expert_logit_bias)
    counts = np.bincount(r["expert_idx"].reshape(-1), minlength=w.n_experts)
    assert counts.sum() == w.n_pairs
    assert counts.max() / max(1, counts.min()) > 10


def test_shared_experts_are_a_sum_of_dense_swiglu_blocks():
    # the always-on experts of the architecture table: every token, weight 1
    rng = np.random.default_rng(3)
    T, d, n_s, f_s = 7, 16, 2, 24
    x = rng.standard_normal((T, d)).astype(np.float32)
    g, u = (rng.standard_normal((n_s, f_s, d)).astype(np.float32) * 0.3 for _ in range(2))
    dn = rng.standard_normal((n_s, d, f_s)).astype(np.float32) * 0.3
    w = WORKLOADS["tiny_f32"]
    got = oracle.shared_experts(w, x, g, u, dn)
    want = np.zeros((T, d))
    X = x.astype(np.float64)
    for s_ in range(n_s):
        a, b = X @ g[s_].astype(np.float64).T, X @ u[s_].astype(np.float64).T
        want += (a / (1 + np.exp(-a)) * b) @ dn[s_].astype(np.float64).T
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.shared_experts(w, x, g, u, dn, tokens=[5, 1]), want[[5, 1]], rtol=1e-12)


def test_e4m3_decoder_against_the_format_definition_and_a_library():
    """FP8 E4M3 (OCP 8-bit floating point, the variant with NaN but no infinities): values the
    format definition fixes, and all 256 codes against torch's float8_e4m3fn."""
    import torch
    d = oracle.decode_e4m3
    fixed = {0x00: 0.0, 0x38: 1.0, 0x40: 2.0, 0x30: 0.5, 0x3C: 1.5, 0x08: 2.0 ** -6, 0x01: 2.0 ** -9,
             0x07: 7 * 2.0 ** -9, 0x7E: 448.0, 0x77: 240.0, 0xB8: -1.0, 0xFE: -448.0, 0x3F: 1.875}
    for code, val in fixed.items():
        assert d(np.uint8(code)) == val, hex(code)
    assert np.isnan(d(np.uint8(0x7F))) and np.isnan(d(np.uint8(0xFF)))
    assert np.signbit(d(np.uint8(0x80))) and d(np.uint8(0x80)) == 0.0
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    got = d(codes)
    assert np.array_equal(np.isnan(got), np.isnan(lib))
    ok = ~np.isnan(got)
    assert np.array_equal(got[ok], lib[ok])
    # monotone in the code within a sign, 4 significant bits
    assert (np.diff(got[:0x7F]) > 0).all()
    q = oracle.dequantize_rows(np.array([[0x38, 0x40], [0xB8, 0x30]], np.uint8), np.array([2.0, 0.5], np.float32))
    assert np.array_equal(q, np.array([[2.0, 4.0], [-0.5, 0.25]]))


def test_mxfp4_decoders_against_the_format_tables_and_a_library():
    """MXFP4 (OCP microscaling): the eight E2M1 magnitudes the format lists, the E8M0 scale as a
    power of two (checked against torch's float8_e8m0fnu for all codes), and a hand-packed block."""
    import torch
    mags = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    got = oracle.decode_e2m1(np.arange(16))
    assert np.array_equal(got[:8], np.array(mags))
    assert np.array_equal(got[8:], -np.array(mags)) and np.signbit(got[8])
    codes = np.arange(256, dtype=np.uint8)
    sc = oracle.decode_e8m0(codes)
    assert sc[127] == 1.0 and sc[128] == 2.0 and sc[0] == 2.0 ** -127 and sc[254] == 2.0 ** 127 and np.isnan(sc[255])
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e8m0fnu).to(torch.float32).numpy()
    assert np.array_equal(sc[:255], lib[:255].astype(np.float64)) and np.isnan(lib[255])
    # one row of 64 elements = two blocks; element 2j in the low nibble of byte j
    packed = np.zeros((1, 32), np.uint8)
    packed[0, 0] = 0x72          # elements 0, 1 = codes 2 (1.0), 7 (6.0)
    packed[0, 15] = 0xF1         # elements 30, 31 = codes 1 (0.5), 15 (-6.0)
    packed[0, 16] = 0x0C         # elements 32, 33 = codes 12 (-2.0), 0
    scales = np.array([[128, 125]], np.uint8)       # 2, 1/4
    w = oracle.dequantize_mxfp4(packed, scales)
    assert w.shape == (1, 64)
    expect = np.zeros(64)
    expect[0], expect[1], expect[30], expect[31], expect[32] = 2.0, 12.0, 1.0, -12.0, -0.5
    assert np.array_equal(w[0], expect)
