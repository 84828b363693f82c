"""GPU parity of the backward pass (combine, expert networks, router with both auxiliary
losses) against the fp64 oracle, through the C ABI.

Tolerances: tensors the GPU stores in bf16 and everything computed from them (dgates come
from the bf16 y_perm) are held to 2e-2 * max|reference| per tensor; the router chain fed with
the same fp32 dgates on both sides is held to 1e-4 * max|reference|.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_23108_amd as M
from gpu_harness import DeviceLayer, from_dev, to_dev
from synth import SELECT_GLOBAL, SELECT_PER_GROUP, WORKLOADS, generate

pytestmark = pytest.mark.gpu

BF16_TOL, F32_TOL = 2e-2, 1e-4


def _close(got, ref, tol, what, atol=1e-30):
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    scale = np.abs(ref).max()
    err = np.abs(got - ref).max() if ref.size else 0.0
    assert np.isfinite(got).all(), what
    assert err <= tol * scale + atol, f"{what}: max err {err:.3e}, allowed {tol * scale + atol:.3e}"


def _run_backward(w, inp):
    """Forward + backward on the GPU; returns the device layer and host copies."""
    print(f"[backward] workload {w.name} T={w.T} d={w.d} d_ff={w.d_ff} mode={w.select_mode}", flush=True)
    dl = DeviceLayer(w, inp, backward=True)
    L = dl.layer
    fwd = dl.run()
    dy = to_dev(inp.dy, True)
    L.backward(dl.x, dy)
    torch.cuda.synchronize()
    dl.check_guards()            # nothing was written outside dx, dx_perm, dy_perm, dgates, the weight gradients
    return dl, fwd, dy


def _upload_routing(L, r, aux):
    """Overwrites the layer's forward routing results with the oracle's (fp32 roundings), so
    that a router-backward comparison starts from identical inputs."""
    L.gs.copy_(torch.from_numpy(r["gs"].astype(np.float32)))
    L.es1.copy_(torch.from_numpy(r["es1"].astype(np.float32)))
    L.gates.copy_(torch.from_numpy(r["gates"].astype(np.float32)))
    L.group_idx.copy_(torch.from_numpy(r["group_idx"]))
    L.expert_idx.copy_(torch.from_numpy(r["expert_idx"]))
    stats = np.concatenate([aux["f_G"], aux["p_G"], aux["f_E"], aux["p_E"]]).astype(np.float32)
    L.stats.copy_(torch.from_numpy(stats))


def _w13_split(t, F):
    a = from_dev(t)
    return a[:, :F, :], a[:, F:, :]


def _medium(select_mode, seed, T=600, skew=0.0, d_ff=(128, 192, 320), N=4):
    return WORKLOADS["training"].replace(name="bwd_medium", T=T, d=256, n_groups=3, experts_per_group=N,
                                         d_ff=d_ff, k_groups=2, k_experts=4, select_mode=select_mode,
                                         seed=seed, skew_beta=skew)


@pytest.mark.parametrize("mode,seed,T,skew", [(SELECT_PER_GROUP, 31, 600, 0.0),
                                              (SELECT_GLOBAL, 32, 333, 0.0),
                                              (SELECT_PER_GROUP, 33, 70, 3.0)])
def test_backward_matches_oracle(mode, seed, T, skew):
    w = _medium(mode, seed, T, skew)
    inp = generate(w)
    dl, fwd, dy = _run_backward(w, inp)
    L = dl.layer
    ref_fwd = oracle.layer(w, inp)
    r = ref_fwd["route"]
    ok = r["margin"] > 1e-6
    assert (fwd["expert_idx"][ok] == r["expert_idx"][ok]).all()
    if not ok.all():
        pytest.skip("a routing decision inside the exclusion margin changes the permutation")
    ref = oracle.layer_bwd(w, inp, inp.dy.f32, ref_fwd)
    perm = fwd["perm"]
    P = w.n_pairs
    # combine backward
    _close(L.dgates.cpu().numpy(), ref["dgates"], BF16_TOL, "dgates")
    _close(from_dev(L.dy_perm)[:P], ref["dy_pairs"][perm], BF16_TOL, "dy_perm")
    # expert networks
    _close(from_dev(L.dx_perm)[:P], ref["dx_pairs"][perm], BF16_TOL, "dx_perm")
    for g in range(w.n_groups):
        dg, du = _w13_split(L.dw13[g], w.d_ff[g])
        _close(dg, ref["dw_gate"][g], BF16_TOL, f"dw_gate[{g}]")
        _close(du, ref["dw_up"][g], BF16_TOL, f"dw_up[{g}]")
        _close(from_dev(L.dw2[g]), ref["dw_down"][g], BF16_TOL, f"dw_down[{g}]")
    # an expert without tokens has exactly zero gradients
    counts = np.bincount(r["expert_idx"].reshape(-1), minlength=w.n_experts)
    for e in np.nonzero(counts == 0)[0]:
        g, i = divmod(int(e), w.experts_per_group)
        assert (from_dev(L.dw13[g])[i] == 0).all() and (from_dev(L.dw2[g])[i] == 0).all()
    if skew > 0:
        assert (counts == 0).any(), "this case is meant to contain an expert without tokens"
    # router and the assembled input gradient
    _close(L.dw_group.cpu().numpy(), ref["dw_group"], BF16_TOL, "dw_group")
    _close(L.dw_expert.cpu().numpy(), ref["dw_expert"], BF16_TOL, "dw_expert")
    _close(from_dev(L.dx), ref["dx"], BF16_TOL, "dx")


def _compare_all_gradients(w, inp, dl, fwd, ref_fwd):
    L = dl.layer
    ref = oracle.layer_bwd(w, inp, inp.dy.f32, ref_fwd)
    P = w.n_pairs
    _close(from_dev(L.dx_perm)[:P], ref["dx_pairs"][fwd["perm"]], BF16_TOL, "dx_perm")
    for g in range(w.n_groups):
        dg, du = _w13_split(L.dw13[g], w.d_ff[g])
        _close(dg, ref["dw_gate"][g], BF16_TOL, f"dw_gate[{g}]")
        _close(du, ref["dw_up"][g], BF16_TOL, f"dw_up[{g}]")
        _close(from_dev(L.dw2[g]), ref["dw_down"][g], BF16_TOL, f"dw_down[{g}]")
    # (with one group, or when every expert of the kept groups is kept, a router gradient is
    # mathematically zero and the reference holds rounding noise: absolute floor)
    _close(L.dw_group.cpu().numpy(), ref["dw_group"], BF16_TOL, "dw_group", atol=1e-7)
    _close(L.dw_expert.cpu().numpy(), ref["dw_expert"], BF16_TOL, "dw_expert", atol=1e-7)
    _close(from_dev(L.dx), ref["dx"], BF16_TOL, "dx")


def test_backward_random_configurations():
    # 10 seeded random layer shapes through forward + backward, every gradient against the oracle
    rng = np.random.default_rng(4242)
    done = 0
    for case in range(14):
        Ng = int(rng.integers(1, 6))
        N = int(rng.integers(1, 7))
        Kg = int(rng.integers(1, Ng + 1))
        mode = int(rng.integers(0, 2))
        Ke = Kg * int(rng.integers(1, N + 1)) if mode == SELECT_PER_GROUP else int(rng.integers(1, Kg * N + 1))
        d = 64 * int(rng.integers(1, 4))
        widths = tuple(64 * int(v) for v in rng.integers(1, 5, Ng))
        T = int(rng.choice([3, 40, 130, 300, 700]))
        w = WORKLOADS["training"].replace(name=f"bwd_random{case}", T=T, d=d, n_groups=Ng, experts_per_group=N,
                                          d_ff=widths, k_groups=Kg, k_experts=Ke, select_mode=mode,
                                          seed=2000 + case, skew_beta=float(rng.choice([0.0, 2.0])))
        inp = generate(w)
        inp.w_group = (inp.w_group * 10).astype(np.float32)
        inp.w_expert = (inp.w_expert * 10).astype(np.float32)
        dl, fwd, dy = _run_backward(w, inp)
        ref_fwd = oracle.layer(w, inp)
        if not (ref_fwd["route"]["margin"] > 1e-6).all():
            continue                                   # a decision inside the exclusion margin
        assert (fwd["expert_idx"] == ref_fwd["route"]["expert_idx"]).all()
        _compare_all_gradients(w, inp, dl, fwd, ref_fwd)
        done += 1
    assert done >= 10


def test_backward_many_experts_wide_model():
    """More than 32 router rows (two passes of the router weight-gradient kernel), a model width
    that is not a multiple of its 512-column blocks, several token splits."""
    w = WORKLOADS["training"].replace(name="bwd_many", T=900, d=576, n_groups=4, experts_per_group=12,
                                      d_ff=(64, 128, 64, 192), k_groups=3, k_experts=6,
                                      select_mode=SELECT_PER_GROUP, seed=77)
    inp = generate(w)
    inp.w_group = (inp.w_group * 10).astype(np.float32)
    inp.w_expert = (inp.w_expert * 10).astype(np.float32)
    dl, fwd, dy = _run_backward(w, inp)
    ref_fwd = oracle.layer(w, inp)
    keep = ref_fwd["route"]["margin"] > 1e-6
    assert keep.all(), "pick another seed: a routing decision falls inside the exclusion margin"
    assert (fwd["expert_idx"] == ref_fwd["route"]["expert_idx"]).all()
    _compare_all_gradients(w, inp, dl, fwd, ref_fwd)


def test_route_backward_fp32_chain_and_aux_terms():
    # the router chain alone, same fp32 dgates on both sides; large loss coefficients so that
    # a wrong auxiliary term cannot hide below the tolerance
    w = _medium(SELECT_GLOBAL, 34, T=500).replace(alpha_g=0.7, alpha_e=0.9)
    inp = generate(w)
    inp.w_group = (inp.w_group * 20).astype(np.float32)
    inp.w_expert = (inp.w_expert * 20).astype(np.float32)
    dl, fwd, dy = _run_backward(w, inp)
    L, c = dl.layer, dl.cfg
    r = oracle.route(w, inp.x.f32, inp.w_group, inp.w_expert)
    aux = oracle.aux_loss(w, r["gs"], r["es1"], r["group_idx"], r["expert_idx"])
    # both sides start from the same forward values: the oracle's, rounded to fp32
    _upload_routing(L, r, aux)
    rng = np.random.default_rng(7)
    for case, dg in (("random dgates", rng.standard_normal((w.T, w.k_experts)).astype(np.float32)),
                     ("aux only", np.zeros((w.T, w.k_experts), np.float32))):
        print(f"[route_bwd] {case}", flush=True)
        dgd = torch.from_numpy(dg).cuda()
        M.mohge_route_bwd(c, dl.x, L.w_group, L.w_expert, L.gs, L.es1, L.group_idx, L.expert_idx,
                          L.gates, dgd, L.stats, None, None, L.dx, L.dw_group, L.dw_expert, L.dz,
                          L.ws_route_bwd)
        torch.cuda.synchronize()
        ref = oracle.route_bwd(w, inp.x.f32, inp.w_group, inp.w_expert, None, r["group_idx"],
                               r["expert_idx"], dg, aux["f_G"], aux["f_E"])
        assert np.abs(ref["dz"]).max() > 1e-6
        _close(L.dz.cpu().numpy(), ref["dz"], F32_TOL, case + " dz")
        _close(L.dw_group.cpu().numpy(), ref["dw_group"], F32_TOL, case + " dw_group")
        _close(L.dw_expert.cpu().numpy(), ref["dw_expert"], F32_TOL, case + " dw_expert")
        _close(from_dev(L.dx), ref["dx"], BF16_TOL, case + " dx (router part)")
    # stats == NULL leaves the auxiliary losses out: zero dgates then give zero gradients
    M.mohge_route_bwd(c, dl.x, L.w_group, L.w_expert, L.gs, L.es1, L.group_idx, L.expert_idx,
                      L.gates, dgd, None, None, None, L.dx, L.dw_group, L.dw_expert, L.dz,
                      L.ws_route_bwd)
    torch.cuda.synchronize()
    assert (L.dz == 0).all() and (L.dw_expert == 0).all() and (L.dx == 0).all()


def test_training_forward_and_backward_determinism():
    w = _medium(SELECT_PER_GROUP, 35, T=200)
    inp = generate(w)
    dl, fwd, dy = _run_backward(w, inp)
    L = dl.layer
    # the training forward gives the same y as the inference forward, bit for bit
    dl2 = DeviceLayer(w, inp, training=False)
    out2 = dl2.run()
    assert np.array_equal(out2["y"], fwd["y"])
    # determinism of the backward pass
    keep = [L.dx.clone(), L.dw_group.clone()] + [t.clone() for t in L.dw13 + L.dw2]
    L.backward(dl.x, dy)
    torch.cuda.synchronize()
    for a, b in zip(keep, [L.dx, L.dw_group] + L.dw13 + L.dw2):
        assert torch.equal(a, b)


def test_expert_backward_with_rows_already_in_sorted_order():
    """perm == NULL: x holds one row per (token, slot) pair in sorted order; same gradients."""
    w = _medium(SELECT_GLOBAL, 36, T=333)
    inp = generate(w)
    dl, fwd, dy = _run_backward(w, inp)
    L = dl.layer
    keep = [t.clone() for t in L.dw13 + L.dw2] + [L.dx_perm.clone()]
    xs = dl.x[(L.perm[:dl.cfg.n_pairs] // dl.cfg.k_experts).long()].contiguous()
    for t in L.dw13 + L.dw2 + [L.dx_perm]:
        t.fill_(float("nan"))
    M.mohge_expert_ffn_bwd(dl.cfg, xs, None, L.offsets, L.w13, L.w2, L.saved, L.dy_perm, L.dx_perm,
                           L.dw13, L.dw2, L.ws_ffn_bwd)
    torch.cuda.synchronize()
    for a, b in zip(keep, L.dw13 + L.dw2 + [L.dx_perm]):
        assert torch.equal(a, b)


def test_backward_rejects_fp32_layers():
    w = WORKLOADS["tiny_f32"]
    cfg = M.Config.from_workload(w)
    t = torch.zeros(64, device="cuda")
    with pytest.raises(M.MohgeError, match="MOHGE_BF16"):
        M.mohge_combine_bwd(cfg, t, t, t, t, t, t)


def _check_backward_sampled(w, n_tok, experts, n_units=16):
    """Full-size run, oracle on samples: gradients of sampled tokens, the router chain at full
    size, and the weight gradients of sampled hidden units of the listed experts."""
    inp = generate(w)
    dl, fwd, dy = _run_backward(w, inp)
    L, c = dl.layer, dl.cfg
    r = oracle.route(w, inp.x.f32, inp.w_group, inp.w_expert)
    ok = r["margin"] > 1e-6
    assert (fwd["expert_idx"][ok] == r["expert_idx"][ok]).all()
    assert ok.mean() > 0.999
    same = (fwd["expert_idx"] == r["expert_idx"]).all(axis=1)
    rng = np.random.default_rng(11)
    Ke, d = w.k_experts, w.d
    wg = [t.f32 for t in inp.w_gate]
    wu = [t.f32 for t in inp.w_up]
    wd = [t.f32 for t in inp.w_down]

    # (1) sampled tokens: dgates, dy_perm, dx_perm and dx of those tokens
    tok = np.sort(rng.choice(np.nonzero(same)[0], size=n_tok, replace=False)).astype(np.int32)
    f = oracle.layer(w, inp, tokens=tok)
    dgates_ref, dy_pairs_ref = oracle.combine_bwd(w, f["y_pairs"], r["gates"][tok], inp.dy.f32[tok])
    pair_token = np.repeat(tok, Ke)
    pair_expert = r["expert_idx"][tok].reshape(-1)
    fb = oracle.expert_ffn_bwd(w, inp.x.f32, wg, wu, wd, pair_token, pair_expert, dy_pairs_ref,
                               want_weight_grads=False)
    rows = fwd["inv_perm"].reshape(w.T, Ke)[tok].reshape(-1)
    rows_t = torch.from_numpy(rows.astype(np.int64)).cuda()
    _close(L.dgates.cpu().numpy()[tok], dgates_ref, BF16_TOL, "dgates (sampled tokens)")
    _close(from_dev(L.dy_perm[rows_t]), dy_pairs_ref, BF16_TOL, "dy_perm (sampled)")
    _close(from_dev(L.dx_perm[rows_t]), fb["dx_pairs"], BF16_TOL, "dx_perm (sampled)")

    # (2) the router chain at full size on the device's own dgates, then dx of the sampled tokens
    dg_dev = L.dgates.cpu().numpy()
    aux = oracle.aux_loss(w, r["gs"], r["es1"], r["group_idx"], r["expert_idx"])
    rb = oracle.route_bwd(w, inp.x.f32, inp.w_group, inp.w_expert, None, r["group_idx"],
                          r["expert_idx"], dg_dev, aux["f_G"], aux["f_E"])
    dx_ref = rb["dx"][tok] + fb["dx_pairs"].reshape(len(tok), Ke, d).sum(axis=1)
    _close(from_dev(L.dx)[tok], dx_ref, BF16_TOL, "dx (sampled tokens)")
    dz_dev = L.dz.cpu().numpy()
    _close(dz_dev[same], rb["dz"][same], 1e-3, "dz (tokens with identical decisions)")
    # same call again from the oracle's forward values: every token comparable, fp32 bar
    _upload_routing(L, r, aux)
    M.mohge_route_bwd(c, dl.x, L.w_group, L.w_expert, L.gs, L.es1, L.group_idx, L.expert_idx,
                      L.gates, L.dgates, L.stats, None, None, L.dx, L.dw_group, L.dw_expert, L.dz,
                      L.ws_route_bwd)
    torch.cuda.synchronize()
    _close(L.dz.cpu().numpy(), rb["dz"], F32_TOL, "dz (full size)")
    _close(L.dw_group.cpu().numpy(), rb["dw_group"], F32_TOL, "dw_group (full size)")
    _close(L.dw_expert.cpu().numpy(), rb["dw_expert"], F32_TOL, "dw_expert (full size)")

    # (3) weight gradients of sampled (expert, hidden unit) sets: a hidden unit's gradient rows
    # depend on no other unit, so the oracle runs on the expert cut down to those units
    N = w.experts_per_group
    for e in experts:
        g, i = divmod(e, N)
        F = w.d_ff[g]
        J = np.sort(rng.choice(F, size=n_units, replace=False))
        pairs = np.nonzero(r["expert_idx"].reshape(-1) == e)[0]
        if not same[pairs // Ke].all():
            continue
        ptok = (pairs // Ke).astype(np.int32)
        gate = r["gates"].reshape(-1)[pairs]
        dyp = gate[:, None] * inp.dy.f32[ptok].astype(np.float64)
        w1 = w.replace(n_groups=1, experts_per_group=1, d_ff=(len(J),), k_groups=1, k_experts=1)
        sub = oracle.expert_ffn_bwd(w1, inp.x.f32, [wg[g][i:i + 1, J, :]], [wu[g][i:i + 1, J, :]],
                                    [wd[g][i:i + 1][:, :, J]], ptok, np.zeros(len(pairs), np.int32), dyp)
        Jt = torch.from_numpy(J).cuda()
        _close(from_dev(L.dw13[g][i][Jt]), sub["dw_gate"][0][0], BF16_TOL, f"dw_gate expert {e}")
        _close(from_dev(L.dw13[g][i][Jt + F]), sub["dw_up"][0][0], BF16_TOL, f"dw_up expert {e}")
        _close(from_dev(L.dw2[g][i][:, Jt]), sub["dw_down"][0][0], BF16_TOL, f"dw_down expert {e}")


def test_backward_full_size_training_config_sampled():
    # sampled tokens for the row gradients, the full-size router chain, and the weight gradients
    # of EVERY expert on 16 sampled hidden units each
    w = WORKLOADS["training"]
    _check_backward_sampled(w, 24, tuple(range(w.n_experts)), n_units=16)


def test_backward_element_offsets_beyond_2_31():
    # P*d and P*2*max F exceed 2^31 elements
    w = WORKLOADS["training"].replace(name="big_offsets_bwd", T=135168, d=4096, n_groups=2,
                                      experts_per_group=2, d_ff=(256, 4096), k_groups=2, k_experts=4, seed=62)
    assert w.n_pairs * w.d > 2 ** 31
    _check_backward_sampled(w, 10, (3,), n_units=2)


def test_backward_with_shared_experts():
    """A training layer with always-on experts: dx and the shared experts' weight gradients
    against the oracle (routed part + shared part)."""
    from synth import bf16_bits_to_f32, f32_to_bf16_bits
    w = _medium(SELECT_PER_GROUP, 41, T=450)
    inp = generate(w)
    rng = np.random.default_rng(17)
    n_s, f_s = 2, 192
    rb = lambda a: bf16_bits_to_f32(f32_to_bf16_bits(a))
    g_s = rb(rng.standard_normal((n_s, f_s, w.d)).astype(np.float32) * 0.05)
    u_s = rb(rng.standard_normal((n_s, f_s, w.d)).astype(np.float32) * 0.05)
    d_s = rb(rng.standard_normal((n_s, w.d, f_s)).astype(np.float32) * 0.05)
    dev = lambda a: torch.from_numpy(a).cuda().to(torch.bfloat16)       # exact: values are bf16 already
    print(f"[backward, shared] T={w.T} d={w.d} N_s={n_s} F_s={f_s}", flush=True)
    shared = M.SharedExperts(w.T, w.d, M.pack_w13(dev(g_s), dev(u_s)), dev(d_s), backward=True)
    cfg = M.Config.from_workload(w)
    w13 = [M.pack_w13(to_dev(g, True), to_dev(u, True)) for g, u in zip(inp.w_gate, inp.w_up)]
    w2 = [to_dev(t, True) for t in inp.w_down]
    L = M.MoHGELayer(cfg, torch.from_numpy(inp.w_group).cuda(), torch.from_numpy(inp.w_expert).cuda(), w13, w2,
                     training=True, backward=True, shared=shared)
    x, dy = to_dev(inp.x, True), to_dev(inp.dy, True)
    y = L.forward(x)
    dx = L.backward(x, dy)
    torch.cuda.synchronize()
    ref_fwd = oracle.layer(w, inp)
    assert (ref_fwd["route"]["margin"] > 1e-6).all(), "pick another seed"
    assert (L.expert_idx.cpu().numpy() == ref_fwd["route"]["expert_idx"]).all()
    y_sh = oracle.shared_experts(w, inp.x.f32, g_s, u_s, d_s)
    _close(from_dev(y), ref_fwd["y"] + y_sh, BF16_TOL, "y with shared experts")
    g = oracle.layer_bwd(w, inp, inp.dy.f32, ref_fwd)
    gs = oracle.shared_experts_bwd(w, inp.x.f32, inp.dy.f32, g_s, u_s, d_s)
    assert np.abs(gs["dx"]).max() > 0.1 * np.abs(g["dx"]).max()          # the shared part is not negligible
    _close(from_dev(dx), g["dx"] + gs["dx"], BF16_TOL, "dx with shared experts")
    dw13 = from_dev(shared.dw13[0])
    _close(dw13[:, :f_s], gs["dw_gate"], BF16_TOL, "shared dw_gate")
    _close(dw13[:, f_s:], gs["dw_up"], BF16_TOL, "shared dw_up")
    _close(from_dev(shared.dw2[0]), gs["dw_down"], BF16_TOL, "shared dw_down")
    # the routed experts' gradients are untouched by the shared term
    _close(from_dev(L.dw2[0]), g["dw_down"][0], BF16_TOL, "routed dw_down[0]")


def test_fused_backward_launches_equal_separate_launches():
    """The backward products as two fused launches (dH -> dX with row-block counters, the two
    weight gradients back to back) against the four-launch form, bit for bit, with inputs that
    change from call to call."""
    w = _medium(SELECT_PER_GROUP, 52, T=900, d_ff=(128, 448, 640))
    dl = DeviceLayer(w, generate(w), backward=True)
    L = dl.layer
    from paper_2604_23108_amd import bench_binding as BB
    if True:
        for it in range(4):
            wi = w.replace(seed=500 + it, skew_beta=float(it % 2) * 2.0)
            inp = generate(wi)
            x, dy = to_dev(inp.x, True), to_dev(inp.dy, True)
            print(f"[fused backward] call {it} seed={wi.seed}", flush=True)
            res = []
            for knob in (1, 0):
                L.ffn_options = BB.FfnOptions(fused=knob)
                L.forward(x)
                for t in L.dw13 + L.dw2 + [L.dx_perm, L.dx]:
                    t.fill_(float("nan"))
                L.backward(x, dy)
                torch.cuda.synchronize()
                res.append([t.clone() for t in L.dw13 + L.dw2 + [L.dx_perm[:dl.cfg.n_pairs], L.dx, L.dw_expert]])
            for a, b in zip(*res):
                assert torch.equal(a, b), f"call {it}"
                assert torch.isfinite(a.float()).all()


def test_fused_status_reports_a_tile_that_gave_up_waiting():
    """mohge_fused_status: MOHGE_OK after ordinary fused launches (inference forward, training
    forward, backward); with the test hook that makes every dependent tile give up without
    looking (the host forces the condition, the kernels run to their normal end) it reports
    MOHGE_ETIMEOUT for each of them and the outputs hold NaN instead of numbers; afterwards
    everything is back to normal and bit-identical."""
    import paper_2604_23108_amd as M
    from paper_2604_23108_amd import bench_binding as BB
    w = WORKLOADS["training"].replace(T=1500, d=512, d_ff=(128, 256, 384), seed=97)
    inp = generate(w)
    dl = DeviceLayer(w, inp, training=True, backward=True)
    L = dl.layer
    dy = to_dev(inp.dy, True)
    calls = ((M.CALL_FFN_SAVED, lambda: L.saved), (M.CALL_EXPERT_FFN_BWD, lambda: L.ws_ffn_bwd))

    def step():
        L.forward(dl.x)
        L.backward(dl.x, dy)
        # the inference form on its own workspace
        BB.mohge_bench_expert_ffn(dl.cfg, dl.x, L.perm, L.offsets, L.w13, L.w2, y_inf, ws_inf, L.ffn_options)
        torch.cuda.synchronize()

    ws_inf = torch.empty(M.mohge_workspace_size(dl.cfg, M.CALL_EXPERT_FFN), dtype=torch.uint8, device="cuda")
    y_inf = torch.empty_like(L.y_perm)
    step()
    ref = (L.y.clone(), L.dx.clone(), [t.clone() for t in L.dw13])
    for call, ws in calls + ((M.CALL_EXPERT_FFN, lambda: ws_inf),):
        assert M.mohge_fused_status(dl.cfg, call, ws()) == 0, call
    print("[fused status] forcing every dependent tile to give up", flush=True)
    L.ffn_options = BB.FfnOptions(spin_limit=-1)
    step()
    for call, ws in calls + ((M.CALL_EXPERT_FFN, lambda: ws_inf),):
        assert M.mohge_fused_status(dl.cfg, call, ws()) == -6, call
    assert "gave up" in M.mohge_last_error()
    # a tile that gave up wrote NaN, not numbers: the failure cannot go unnoticed downstream
    n = dl.cfg.n_pairs
    assert torch.isnan(y_inf[:n].float()).all() and torch.isnan(L.y.float()).all()
    assert torch.isnan(L.dx_perm[:n].float()).all()
    L.ffn_options = None
    step()
    for call, ws in calls + ((M.CALL_EXPERT_FFN, lambda: ws_inf),):
        assert M.mohge_fused_status(dl.cfg, call, ws()) == 0, call
    assert torch.equal(L.y, ref[0]) and torch.equal(L.dx, ref[1])
    for a, b in zip(L.dw13, ref[2]):
        assert torch.equal(a, b)
    # calls without such a launch answer at once
    wd = WORKLOADS["decode"].replace(T=8, d=512, d_ff=(128, 256, 384, 512), seed=98)
    cd = M.Config.from_workload(wd)
    assert M.lib().mohge_fused_status(cd.ref(), M.CALL_EXPERT_FFN, None, 0, None) == 0
    assert M.lib().mohge_fused_status(dl.cfg.ref(), M.CALL_PERMUTE, None, 0, None) == -1
