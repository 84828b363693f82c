"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by
element, on the same seeded inputs.

Bars: routing indices and the permutation bit-exact (tokens whose top-k margin in the
oracle is below 1e-6 are excluded from index / output comparison and counted); gates
within 1e-6; layer output max|err| <= 2e-2 * max|ref| in bf16 and <= 1e-4 in fp32;
auxiliary losses within 1e-4 relative.
"""
import numpy as np
import pytest
import torch

import oracle
from synth import SELECT_GLOBAL, SELECT_PER_GROUP, WORKLOADS, Workload, generate

pytestmark = pytest.mark.gpu

MARGIN = 1e-6


def _dev():
    from gpu_harness import DeviceLayer
    return DeviceLayer


def check_routing(w, out, ref, what=""):
    keep = ref["margin"] >= MARGIN
    n_excl = int((~keep).sum())
    assert n_excl <= max(2, w.T // 500), f"{what}: {n_excl} tokens inside the margin"
    assert (out["group_idx"][keep] == ref["group_idx"][keep]).all(), f"{what}: group ids differ"
    assert (out["expert_idx"][keep] == ref["expert_idx"][keep]).all(), f"{what}: expert ids differ"
    err = np.abs(out["gates"][keep] - ref["gates"][keep]).max() if keep.any() else 0.0
    assert err <= 1e-6, f"{what}: gate error {err}"
    return keep, n_excl


def check_permutation(w, out):
    # the permutation of whatever expert ids the GPU produced must be the stable bucket sort
    p = oracle.permute(w, out["expert_idx"])
    for k in ("counts", "offsets", "perm", "inv_perm"):
        assert (out[k] == p[k]).all(), f"{k} differs"


def check_output(w, inp, out, ref_route, keep, tokens, tol_rel=2e-2, tol_abs_f32=1e-4):
    tokens = np.asarray([t for t in tokens if keep[t]], np.int32)
    pair_token = np.repeat(tokens, w.k_experts)
    pair_expert = ref_route["expert_idx"][tokens].reshape(-1)
    y_pairs = oracle.expert_ffn(w, inp.x.f32, [t.f32 for t in inp.w_gate], [t.f32 for t in inp.w_up],
                                [t.f32 for t in inp.w_down], pair_token, pair_expert)
    y_ref = oracle.combine(w, y_pairs, ref_route["gates"][tokens])
    # expert outputs, looked up through the GPU's own inverse permutation
    pair_ids = (tokens[:, None] * w.k_experts + np.arange(w.k_experts)[None, :]).reshape(-1)
    rows = torch.from_numpy(out["inv_perm"][pair_ids].astype(np.int64)).cuda()
    y_perm_rows = out["y_perm"][rows].float().cpu().numpy()
    if w.dtype == "bf16":
        assert np.abs(y_perm_rows - y_pairs).max() <= tol_rel * np.abs(y_pairs).max()
        err = np.abs(out["y"][tokens] - y_ref).max()
        assert err <= tol_rel * np.abs(y_ref).max(), f"y error {err} vs max|ref| {np.abs(y_ref).max()}"
    else:
        assert np.abs(y_perm_rows - y_pairs).max() <= tol_abs_f32
        assert np.abs(out["y"][tokens] - y_ref).max() <= tol_abs_f32
    return float(np.abs(out["y"][tokens] - y_ref).max()), float(np.abs(y_ref).max())


def full_check(w, tokens=None, scale_router=1.0, inp=None):
    inp = generate(w) if inp is None else inp
    if scale_router != 1.0:
        inp.w_group *= np.float32(scale_router)
        inp.w_expert *= np.float32(scale_router)
    dl = _dev()(w, inp, training=True)
    out = dl.run()
    ref = oracle.route(w, inp.x.f32, inp.w_group, inp.w_expert, inp.expert_logit_bias)
    keep, n_excl = check_routing(w, out, ref, w.name)
    check_permutation(w, out)
    toks = np.arange(w.T) if tokens is None else tokens
    check_output(w, inp, out, ref, keep, toks)
    # properties that hold at any size
    assert np.isfinite(out["y"]).all() and np.abs(out["gates"].sum(axis=1) - 1.0).max() <= 2e-6
    assert out["counts"].sum() == w.n_pairs and (out["gates"] > 0).all()
    # scores and auxiliary losses
    np.testing.assert_allclose(out["gs"], ref["gs"], atol=1e-6)
    # ES' = exp(z - max) / sum in fp32: the difference z - max carries an absolute error of about
    # an ulp of |z|, which becomes a relative error of the score (2e-6 at |z| ~ 30)
    np.testing.assert_allclose(out["es1"][keep], ref["es1"][keep], atol=1e-6, rtol=2e-6)
    if n_excl == 0:
        a = oracle.aux_loss(w, ref["gs"], ref["es1"], ref["group_idx"], ref["expert_idx"])
        assert abs(out["losses"][0] - a["L_G"]) <= 1e-4 * abs(a["L_G"])
        assert abs(out["losses"][1] - a["L_E"]) <= 1e-4 * abs(a["L_E"])
        Ng, Ne = w.n_groups, w.n_experts
        np.testing.assert_allclose(out["stats"][:Ng], a["f_G"], rtol=1e-5)
        np.testing.assert_allclose(out["stats"][Ng:2 * Ng], a["p_G"], rtol=1e-5)
        np.testing.assert_allclose(out["stats"][2 * Ng:2 * Ng + Ne], a["f_E"], rtol=1e-5, atol=1e-7)
        np.testing.assert_allclose(out["stats"][2 * Ng + Ne:], a["p_E"], rtol=1e-5, atol=1e-7)
    return out, ref


# ---- configuration 1 in full ------------------------------------------------------------
def test_tiny_f32_layer_all_tokens():
    full_check(WORKLOADS["tiny_f32"])


@pytest.mark.parametrize("mode", [SELECT_GLOBAL, SELECT_PER_GROUP])
def test_tiny_f32_both_selection_modes_spread_router(mode):
    full_check(WORKLOADS["tiny_f32"].replace(select_mode=mode, k_experts=4, T=77), scale_router=10.0)


# ---- bf16, several row tiles with ragged tails, ragged column tiles ----------------------
MID = Workload("mid_bf16", T=1500, d=256, n_groups=3, experts_per_group=4, d_ff=(64, 192, 320),
               k_groups=2, k_experts=4, seed=21)


@pytest.mark.parametrize("mode", [SELECT_GLOBAL, SELECT_PER_GROUP])
def test_mid_bf16_tiled_path(mode):
    full_check(MID.replace(select_mode=mode), scale_router=5.0)


def test_mid_bf16_skewed_counts():
    w = MID.replace(skew_beta=2.0, experts_per_group=8, seed=22, T=2100)
    out, _ = full_check(w, scale_router=5.0)
    c = out["counts"]
    assert c.max() / max(1, c.min()) > 10


def test_paper_shape_global_selection_eight_widths():
    w = WORKLOADS["paper_1b"].replace(T=900, d=256)
    full_check(w, tokens=np.arange(0, 900, 3), scale_router=8.0)


def test_random_configurations():
    # 24 seeded random layer shapes: group count, experts per group, widths (multiples of 64),
    # hidden size, K_g, K_e, selection mode, token count (ragged tails, tiles of every height,
    # the single-workgroup permutation and the tiled one, the weight-streaming path for T <= 32)
    rng = np.random.default_rng(2024)
    for case in range(24):
        Ng = int(rng.integers(1, 7))
        N = int(rng.integers(1, 9))
        Kg = int(rng.integers(1, Ng + 1))
        mode = int(rng.integers(0, 2))
        if mode == SELECT_PER_GROUP:
            Ke = Kg * int(rng.integers(1, N + 1))
        else:
            Ke = int(rng.integers(1, Kg * N + 1))
        d = 64 * int(rng.integers(1, 5))
        widths = tuple(64 * int(v) for v in rng.integers(1, 7, Ng))
        T = int(rng.choice([1, 5, 31, 33, 64, 200, 517, 1100]))
        w = Workload(f"random{case}", T=T, d=d, n_groups=Ng, experts_per_group=N, d_ff=widths,
                     k_groups=Kg, k_experts=Ke, select_mode=mode, seed=1000 + case, training=True,
                     skew_beta=float(rng.choice([0.0, 1.5])))
        print(f"[random] case {case}: T={T} d={d} {Ng}x{N} d_ff={widths} Kg={Kg} Ke={Ke} mode={mode}", flush=True)
        full_check(w, scale_router=10.0)


def test_largest_supported_expert_grid():
    # N_g = 16 groups of 16 experts (N_e = 256, the documented maximum), 16 distinct widths,
    # 16 experts per token, both selection modes
    widths = tuple(64 * (1 + (5 * g) % 16) for g in range(16))
    for mode in (SELECT_GLOBAL, SELECT_PER_GROUP):
        w = Workload("max_grid", T=700, d=128, n_groups=16, experts_per_group=16, d_ff=widths,
                     k_groups=4, k_experts=16, select_mode=mode, seed=41 + mode, training=True)
        full_check(w, tokens=np.arange(0, 700, 5), scale_router=12.0)


# ---- decode-shaped: the weight-streaming path --------------------------------------------
@pytest.mark.parametrize("T", [1, 7, 32])
def test_decode_shaped_small(T):
    w = Workload("dec", T=T, d=512, n_groups=4, experts_per_group=4, d_ff=(64, 128, 192, 256),
                 k_groups=2, k_experts=4, seed=30 + T)
    full_check(w, scale_router=4.0)


def test_all_tokens_to_one_expert_decode_and_tiled():
    # degenerate routing: a huge bias on one expert per group
    for T in (32, 700):
        w = Workload("one", T=T, d=128, n_groups=2, experts_per_group=4, d_ff=(64, 128), k_groups=2,
                     k_experts=2, seed=40)
        inp = generate(w)
        bias = np.zeros(w.n_experts, np.float32)
        bias[1] = 50.0
        bias[6] = 50.0
        inp.expert_logit_bias = bias
        dl = _dev()(w, inp, training=False)
        out = dl.run()
        ref = oracle.route(w, inp.x.f32, inp.w_group, inp.w_expert, bias)
        keep, _ = check_routing(w, out, ref)
        assert out["counts"].tolist() == [0, T, 0, 0, 0, 0, T, 0]
        check_permutation(w, out)
        check_output(w, inp, out, ref, keep, np.arange(T))


def test_empty_call_and_error_paths():
    import paper_2604_23108_amd as M
    w = MID.replace(T=0)
    cfg = M.Config.from_workload(w)
    i32 = dict(dtype=torch.int32, device="cuda")
    eidx = torch.empty((0, w.k_experts), **i32)
    counts = torch.full((w.n_experts,), -1, **i32)
    offsets = torch.full((w.n_experts + 1,), -1, **i32)
    perm = torch.empty(4, **i32)
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda")
    M.mohge_permute(cfg, eidx.reshape(-1).new_empty(4), counts, offsets, perm, perm.clone(), None, None, ws)
    torch.cuda.synchronize()
    assert (counts == 0).all() and (offsets == 0).all()
    # workspace too small, misaligned pointer
    w2 = MID
    cfg2 = M.Config.from_workload(w2)
    with pytest.raises(M.MohgeError, match="workspace"):
        M.mohge_permute(cfg2, torch.zeros(w2.n_pairs, **i32), counts, offsets,
                        torch.empty(w2.n_pairs, **i32), torch.empty(w2.n_pairs, **i32), None, None,
                        torch.empty(16, dtype=torch.uint8, device="cuda"))
    g = torch.empty(w2.T * w2.k_experts + 1, dtype=torch.float32, device="cuda")
    with pytest.raises(M.MohgeError, match="aligned"):
        M.mohge_combine(cfg2, torch.empty((w2.n_pairs, w2.d), dtype=torch.bfloat16, device="cuda"),
                        torch.zeros(w2.n_pairs, **i32), g[1:],
                        torch.empty((w2.T, w2.d), dtype=torch.bfloat16, device="cuda"))


def test_x_perm_materialisation_and_prepermuted_ffn_input():
    import paper_2604_23108_amd as M
    w = MID.replace(T=600)
    inp = generate(w)
    dl = _dev()(w, inp, training=False)
    out = dl.run()
    L = dl.layer
    x_perm = torch.empty((w.n_pairs, w.d), dtype=torch.bfloat16, device="cuda")
    M.mohge_permute(dl.cfg, L.expert_idx, L.counts, L.offsets, L.perm, L.inv_perm, dl.x, x_perm, L.ws_permute)
    torch.cuda.synchronize()
    src = torch.from_numpy((out["perm"] // w.k_experts).astype(np.int64)).cuda()
    assert torch.equal(x_perm, dl.x[src])
    y_perm2 = torch.empty_like(L.y_perm)
    M.mohge_expert_ffn(dl.cfg, x_perm, None, L.offsets, dl.w13, dl.w2, y_perm2, L.ws_ffn)
    torch.cuda.synchronize()
    assert torch.equal(y_perm2[:w.n_pairs], L.y_perm[:w.n_pairs])


def test_route_and_permute_many_pairs_three_kernel_path():
    # more than 256 wave segments (P > 131072): the permutation takes its separate scan kernel
    import paper_2604_23108_amd as M
    from gpu_harness import to_dev
    w = Workload("many", T=41000, d=64, n_groups=4, experts_per_group=8, d_ff=(64, 64, 64, 64),
                 k_groups=2, k_experts=4, seed=55, skew_beta=1.0)
    inp = generate(w)
    inp.w_group *= np.float32(20)
    inp.w_expert *= np.float32(20)
    cfg = M.Config.from_workload(w)
    x = to_dev(inp.x, True)
    wg, we = torch.from_numpy(inp.w_group).cuda(), torch.from_numpy(inp.w_expert).cuda()
    bias = torch.from_numpy(inp.expert_logit_bias).cuda()
    i32 = dict(dtype=torch.int32, device="cuda")
    gidx = torch.empty((w.T, w.k_groups), **i32)
    eidx = torch.empty((w.T, w.k_experts), **i32)
    gates = torch.empty((w.T, w.k_experts), dtype=torch.float32, device="cuda")
    M.mohge_route(cfg, x, wg, we, bias, gidx, eidx, gates)
    counts = torch.empty(w.n_experts, **i32)
    offsets = torch.empty(w.n_experts + 1, **i32)
    perm = torch.empty(w.n_pairs, **i32)
    inv = torch.empty(w.n_pairs, **i32)
    ws = torch.empty(M.mohge_workspace_size(cfg, M.CALL_PERMUTE), dtype=torch.uint8, device="cuda")
    M.mohge_permute(cfg, eidx, counts, offsets, perm, inv, None, None, ws)
    torch.cuda.synchronize()
    out = dict(group_idx=gidx.cpu().numpy(), expert_idx=eidx.cpu().numpy(), gates=gates.cpu().numpy(),
               counts=counts.cpu().numpy(), offsets=offsets.cpu().numpy(), perm=perm.cpu().numpy(),
               inv_perm=inv.cpu().numpy())
    ref = oracle.route(w, inp.x.f32, inp.w_group, inp.w_expert, inp.expert_logit_bias)
    check_routing(w, out, ref, "many pairs")
    check_permutation(w, out)


@pytest.mark.parametrize("T,Ng,N", [(25, 3, 4), (512, 3, 8), (513, 16, 16), (4096, 16, 16), (8192, 3, 8), (8193, 3, 8),
                                    (17500, 16, 16), (32768, 3, 8), (32769, 3, 8), (41000, 8, 8)])
def test_permute_every_launch_path(T, Ng, N):
    # K_e = 4: P = 100 and 2048 (one workgroup), 2052 ... 131076 (histogram launch + scatter
    # launch with the scan folded in, while segments x experts <= 8192: 24 experts up to the
    # largest P here, 256 experts only for the small ones), else histogram, scan, scatter;
    # expert ids drawn directly, skewed
    import paper_2604_23108_amd as M
    w = Workload("perm", T=T, d=64, n_groups=Ng, experts_per_group=N, d_ff=(64,) * Ng, k_groups=2,
                 k_experts=4, seed=0)
    rng = np.random.default_rng(T)
    pmf = 1.0 / (1.0 + np.arange(w.n_experts)) ** 1.1
    eidx_h = rng.choice(w.n_experts, size=(T, 4), p=pmf / pmf.sum()).astype(np.int32)
    print(f"[permute] P={w.n_pairs} Ne={w.n_experts}", flush=True)
    cfg = M.Config.from_workload(w)
    i32 = dict(dtype=torch.int32, device="cuda")
    eidx = torch.from_numpy(eidx_h).cuda()
    counts, offsets = torch.empty(w.n_experts, **i32), torch.empty(w.n_experts + 1, **i32)
    perm, inv = torch.full((w.n_pairs,), -1, **i32), torch.full((w.n_pairs,), -1, **i32)
    ws = torch.empty(M.mohge_workspace_size(cfg, M.CALL_PERMUTE), dtype=torch.uint8, device="cuda")
    M.mohge_permute(cfg, eidx, counts, offsets, perm, inv, None, None, ws)
    torch.cuda.synchronize()
    check_permutation(w, dict(expert_idx=eidx_h, counts=counts.cpu().numpy(), offsets=offsets.cpu().numpy(),
                              perm=perm.cpu().numpy(), inv_perm=inv.cpu().numpy()))


def test_shared_experts_added_to_the_routed_output():
    import paper_2604_23108_amd as M
    from gpu_harness import to_dev
    w = WORKLOADS["paper_1b"].replace(T=800, d=256)
    inp = generate(w)
    inp.w_group *= np.float32(8)
    inp.w_expert *= np.float32(8)
    rng = np.random.default_rng(9)
    n_s, f_s = 2, 192
    from synth import bf16_bits_to_f32, f32_to_bf16_bits
    rb = lambda a: bf16_bits_to_f32(f32_to_bf16_bits(a))
    g_s = rb(rng.standard_normal((n_s, f_s, w.d)).astype(np.float32) * 0.02)
    u_s = rb(rng.standard_normal((n_s, f_s, w.d)).astype(np.float32) * 0.02)
    d_s = rb(rng.standard_normal((n_s, w.d, f_s)).astype(np.float32) * 0.02)
    dev = lambda a: torch.from_numpy(a).cuda().to(torch.bfloat16)       # exact: values are bf16 already
    print(f"[shared] T={w.T} d={w.d} N_s={n_s} F_s={f_s}", flush=True)
    shared = M.SharedExperts(w.T, w.d, M.pack_w13(dev(g_s), dev(u_s)), dev(d_s))
    cfg = M.Config.from_workload(w)
    w13 = [M.pack_w13(to_dev(g, True), to_dev(u, True)) for g, u in zip(inp.w_gate, inp.w_up)]
    w2 = [to_dev(t, True) for t in inp.w_down]
    L = M.MoHGELayer(cfg, torch.from_numpy(inp.w_group).cuda(), torch.from_numpy(inp.w_expert).cuda(), w13, w2,
                     shared=shared)
    y = L.forward(to_dev(inp.x, True)).float().cpu().numpy()
    torch.cuda.synchronize()
    # constant routing of the shared configuration
    assert (shared.expert_idx.cpu().numpy() == np.arange(n_s)[None, :]).all()
    p = oracle.permute(w.replace(n_groups=1, experts_per_group=n_s, k_groups=1, k_experts=n_s, d_ff=(f_s,)),
                       shared.expert_idx.cpu().numpy())
    assert (shared.perm.cpu().numpy() == p["perm"]).all() and (shared.inv_perm.cpu().numpy() == p["inv_perm"]).all()
    assert (shared.offsets.cpu().numpy() == p["offsets"]).all() and (shared.counts.cpu().numpy() == p["counts"]).all()
    tok = np.arange(0, w.T, 4)
    ref = oracle.layer(w, inp, tokens=tok)
    keep = ref["route"]["margin"][tok] >= MARGIN
    assert (L.expert_idx.cpu().numpy()[tok][keep] == ref["route"]["expert_idx"][tok][keep]).all()
    y_sh = oracle.shared_experts(w, inp.x.f32, g_s, u_s, d_s, tokens=tok)
    want = ref["y"] + y_sh
    assert np.abs(y_sh).max() > 0.2 * np.abs(ref["y"]).max()           # the shared term is not negligible
    err = np.abs(y[tok][keep] - want[keep]).max()
    assert err <= 2e-2 * np.abs(want).max(), f"error {err}"
    sh_err = np.abs(shared.y.float().cpu().numpy()[tok] - y_sh).max()
    assert sh_err <= 2e-2 * np.abs(y_sh).max()


def test_runs_are_bit_identical():
    w = MID.replace(T=1111)
    inp = generate(w)
    dl = _dev()(w, inp, training=True)
    a = dl.run()
    ya, la = a["y"].copy(), a["losses"].copy()
    pa = a["perm"].copy()
    b = dl.run()
    assert (ya == b["y"]).all() and (la == b["losses"]).all() and (pa == b["perm"]).all()


# ---- the named configurations at full size, in the launch configuration bench.py times -----
_GEN = {}


def _generated(name):
    """Seeded inputs of a named workload, drawn once per test session (the selection mode does
    not enter the draws)."""
    if name not in _GEN:
        _GEN.clear()                      # one large workload in host memory at a time
        _GEN[name] = generate(WORKLOADS[name])
    return _GEN[name]


def full_check_generated(w, inp, tokens=None):
    """full_check on inputs that are already drawn (`w` may differ from the inputs' workload in
    the selection mode only)."""
    return full_check(w, tokens=tokens, inp=inp)


@pytest.mark.parametrize("mode", [SELECT_PER_GROUP, SELECT_GLOBAL])
@pytest.mark.parametrize("name", ["mid_prefill", "decode", "training"])
def test_full_size_configs_every_token(name, mode):
    # routing, permutation, scores, losses, y_perm and y of EVERY token against the oracle, in the
    # mode the configuration names (per group) and in the paper's own (global top-K_e)
    w = WORKLOADS[name].replace(select_mode=mode)
    print(f"[full size] {name} mode={mode} T={w.T}", flush=True)
    full_check_generated(w, _generated(name))


def check_row_blocks(w, inp, out, ref, keep, rows_per_block=128, rng=None):
    """y_perm against the oracle at the first row, the last row and one seeded row of every
    `rows_per_block` sorted positions of every expert (so every row tile of every expert, whatever
    tile height the schedule chose, has a row compared in every column tile)."""
    rng = rng or np.random.default_rng(5)
    offs, perm = out["offsets"], out["perm"]
    rows = []
    for e in range(w.n_experts):
        lo, hi = int(offs[e]), int(offs[e + 1])
        if hi == lo:
            continue
        rows += [lo, hi - 1]
        for b in range(lo, hi, rows_per_block):
            rows.append(int(rng.integers(b, min(b + rows_per_block, hi))))
    rows = np.unique(np.asarray(rows, np.int64))
    pairs = perm[rows]
    tok = (pairs // w.k_experts).astype(np.int32)
    ok = keep[tok]
    rows, pairs, tok = rows[ok], pairs[ok], tok[ok]
    exp = out["expert_idx"].reshape(-1)[pairs].astype(np.int32)
    assert (exp == ref["expert_idx"].reshape(-1)[pairs]).all()
    y_ref = oracle.expert_ffn(w, inp.x.f32, [t.f32 for t in inp.w_gate], [t.f32 for t in inp.w_up],
                              [t.f32 for t in inp.w_down], tok, exp)
    got = out["y_perm"][torch.from_numpy(rows).cuda()].float().cpu().numpy()
    err = np.abs(got - y_ref).max()
    assert err <= 2e-2 * np.abs(y_ref).max(), f"y_perm rows: error {err} vs max|ref| {np.abs(y_ref).max()}"
    return len(rows)


@pytest.mark.parametrize("mode", [SELECT_PER_GROUP, SELECT_GLOBAL])
def test_full_size_large_prefill_skewed(mode):
    # the largest configuration: routing, permutation, scores and losses of every token; y and
    # y_perm of 256 whole tokens; y_perm rows in every row tile of every expert
    name = "large_prefill_skewed"
    w = WORKLOADS[name].replace(select_mode=mode)
    inp = _generated(name)
    rng = np.random.default_rng(321)
    toks = np.sort(rng.choice(w.T, size=256, replace=False))
    print(f"[full size] {name} mode={mode} T={w.T}", flush=True)
    out, ref = full_check_generated(w, inp, tokens=toks)
    c = out["counts"]
    assert c.sum() == w.n_pairs and c.max() / max(1, c.min()) > 10
    keep = ref["margin"] >= MARGIN
    n = check_row_blocks(w, inp, out, ref, keep)
    print(f"[full size] {name}: {n} y_perm rows compared", flush=True)


@pytest.mark.parametrize("name", ["mid_prefill", "large_prefill_skewed"])
def test_fused_forward_equals_separate_launches_at_full_size(name):
    """The one-launch expert networks against the two-launch form, bit for bit, where many rounds
    of tiles cross the XCD ranges and workgroups steal from other ranges; also with a tile order of
    whole-expert columns, another visiting order and no stealing."""
    import paper_2604_23108_amd as M
    from paper_2604_23108_amd import bench_binding as BB
    w = WORKLOADS[name]
    dl = _dev()(w, _generated(name), training=False)
    L = dl.layer
    L.forward(dl.x)
    torch.cuda.synchronize()
    ref = L.y_perm.clone()
    assert M.mohge_fused_status(dl.cfg, M.CALL_EXPERT_FFN, L.ws_ffn) == 0
    for kw in (dict(fused=0), dict(fused=1, band_rows=1000, group_major=1, steal=0), dict(fused=1, band_rows=1),
               dict(fused=1, tile_rows_up=128)):
        print(f"[fused, full size] {name} {kw}", flush=True)
        y = torch.full_like(L.y_perm, float("nan"))
        BB.mohge_bench_expert_ffn(dl.cfg, dl.x, L.perm, L.offsets, L.w13, L.w2, y, L.ws_ffn, BB.FfnOptions(**kw))
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), ref.view(torch.int16)), kw


@pytest.mark.parametrize("name", ["paper_1b", "paper_3b", "paper_14b"])
def test_full_size_paper_layer_shapes_sampled(name):
    # the paper's own layer shapes (appendix, architecture table): d = 1024, eight widths,
    # K_g = 3, K_e = 6 chosen globally, 32 / 64 / 128 experts, a 4096-token sequence
    w = WORKLOADS[name].replace(training=True)
    rng = np.random.default_rng(17)
    toks = np.sort(rng.choice(w.T, size=24, replace=False))
    full_check(w, tokens=toks, scale_router=8.0)


def test_element_offsets_beyond_2_31():
    # P*d and P*max F both exceed 2^31 elements (P = 540672 rows of 4096): every row offset must
    # be computed in 64 bits.  Two groups of two experts, every token goes to all four.
    w = Workload("big_offsets", T=135168, d=4096, n_groups=2, experts_per_group=2, d_ff=(256, 4096),
                 k_groups=2, k_experts=4, seed=61)
    assert w.n_pairs * w.d > 2 ** 31 and w.n_pairs * max(w.d_ff) > 2 ** 31
    rng = np.random.default_rng(7)
    toks = np.sort(np.concatenate([rng.choice(w.T, size=12, replace=False), [0, w.T - 1]]))
    print(f"[big offsets] T={w.T} P={w.n_pairs} d={w.d}", flush=True)
    inp = generate(w)
    out, ref = full_check_generated(w, inp, tokens=toks)
    assert (out["counts"] == w.T).all()
    n = check_row_blocks(w, inp, out, ref, ref["margin"] >= MARGIN, rows_per_block=2048)
    print(f"[big offsets] {n} y_perm rows compared", flush=True)


def test_graph_replay_matches_eager():
    # a captured step replayed several times, with eager work and synchronisations in between,
    # must reproduce the eager result bit for bit on every replay
    w = WORKLOADS["mid_prefill"].replace(T=1500, d=512, d_ff=(128, 256, 384))
    inp = generate(w)
    DeviceLayer = _dev()
    dl = DeviceLayer(w, inp, training=False)
    L = dl.layer
    print(f"[graph] workload {w.name} T={w.T}", flush=True)
    y_eager = L.forward(dl.x).clone()
    idx_eager = L.expert_idx.clone()
    torch.cuda.synchronize()
    L.capture(dl.x)
    other = DeviceLayer(w.replace(seed=77), generate(w.replace(seed=77)), training=False)
    for i in range(4):
        L.y.zero_(); L.expert_idx.zero_(); L.y_perm.zero_()
        L.replay()
        torch.cuda.synchronize()
        assert torch.equal(L.y, y_eager), f"replay {i}"
        assert torch.equal(L.expert_idx, idx_eager)
        other.layer.forward(other.x)            # unrelated eager work between the replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("training", [False, True])
def test_fused_forward_equals_separate_launches(training):
    """The one-launch forward (up and down tiles share the persistent workgroups, down tiles wait
    for the row-block counters) against the two-launch forward, bit for bit, on one layer object
    whose input changes from call to call: a down tile that read hidden activations of an earlier
    call (a missing wait, a stale cache line) would show."""
    from paper_2604_23108_amd import bench_binding as BB
    from gpu_harness import to_dev
    w = WORKLOADS["mid_prefill"].replace(T=2300, d=768, d_ff=(128, 448, 640), seed=91)
    DeviceLayer = _dev()
    dl = DeviceLayer(w, generate(w), training=training, backward=training)
    L = dl.layer
    if True:
        for it in range(6):
            wi = w.replace(seed=100 + it, skew_beta=float(it % 3))
            x = to_dev(generate(wi).x, True)
            print(f"[fused] training={training} call {it} seed={wi.seed}", flush=True)
            L.ffn_options = BB.FfnOptions(fused=1)
            y_fused = L.forward(x).clone()
            saved_fused = L.saved.clone() if training else None
            counts = L.counts.clone()
            L.ffn_options = BB.FfnOptions(fused=0)
            y_two = L.forward(x).clone()
            torch.cuda.synchronize()
            assert torch.equal(L.counts, counts)
            assert torch.equal(y_fused, y_two), f"call {it}"
            if training:
                # the saved hidden activations and backward factors (behind the schedule area,
                # whose records differ between the two launch forms)
                tail = L.saved.numel() - 3 * max(dl.cfg.n_pairs, 1) * max(w.d_ff) * 2
                assert torch.equal(saved_fused[tail:], L.saved[tail:]), f"call {it}: saved activations"


@pytest.mark.parametrize("T,d,Ng,N", [(1, 4096, 4, 16), (7, 4096, 4, 16), (32, 4096, 4, 16), (200, 1024, 8, 16),
                                      (256, 320, 3, 5), (40, 64, 2, 2)])
def test_router_with_and_without_workspace(T, d, Ng, N):
    """Few tokens: with its optional workspace the router spreads the reduction over many
    workgroups (two kernels).  Both forms against the oracle, and against each other."""
    import paper_2604_23108_amd as M
    from gpu_harness import to_dev
    w = Workload("route_ws", T=T, d=d, n_groups=Ng, experts_per_group=N, d_ff=tuple([64] * Ng),
                 k_groups=min(2, Ng), k_experts=min(2, Ng) * min(2, N), seed=300 + T, training=True)
    inp = generate(w)
    cfg = M.Config.from_workload(w)
    x = to_dev(inp.x, True)
    wg, we = torch.from_numpy(inp.w_group).cuda(), torch.from_numpy(inp.w_expert).cuda()
    bias = None if inp.expert_logit_bias is None else torch.from_numpy(inp.expert_logit_bias).cuda()
    n_ws = M.mohge_workspace_size(cfg, M.CALL_ROUTE)
    assert n_ws >= 16 * T * (Ng + Ng * N) * 8
    ref = oracle.route(w, inp.x.f32, inp.w_group, inp.w_expert, inp.expert_logit_bias)
    outs = []
    for ws in (None, torch.empty(n_ws, dtype=torch.uint8, device="cuda")):
        print(f"[route] T={T} d={d} workspace={'yes' if ws is not None else 'no'}", flush=True)
        i32 = dict(dtype=torch.int32, device="cuda")
        f32 = dict(dtype=torch.float32, device="cuda")
        gidx = torch.full((T, w.k_groups), -1, **i32)
        eidx = torch.full((T, w.k_experts), -1, **i32)
        gates = torch.full((T, w.k_experts), float("nan"), **f32)
        gs = torch.full((T, Ng), float("nan"), **f32)
        es1 = torch.full((T, Ng * N), float("nan"), **f32)
        M.mohge_route(cfg, x, wg, we, bias, gidx, eidx, gates, gs, es1, ws)
        torch.cuda.synchronize()
        out = dict(group_idx=gidx.cpu().numpy(), expert_idx=eidx.cpu().numpy(), gates=gates.cpu().numpy())
        keep, _ = check_routing(w, out, ref, f"workspace={ws is not None}")
        assert np.abs(gs.cpu().numpy() - ref["gs"]).max() <= 1e-6
        assert np.allclose(es1.cpu().numpy(), ref["es1"], rtol=2e-6, atol=1e-6)
        outs.append((out, keep))
    (a, keep), (b, _) = outs
    assert (a["expert_idx"][keep] == b["expert_idx"][keep]).all()
    assert np.abs(a["gates"][keep] - b["gates"][keep]).max() <= 1e-6


def test_fp8_code_conversion_matches_the_format():
    """All 256 E4M3 codes through the hardware conversion the quantised-weight kernel uses."""
    import paper_2604_23108_amd as M
    codes = torch.arange(256, dtype=torch.uint8).repeat(5)[:1277].cuda()      # ragged length
    out = torch.full((codes.numel(),), 123.0, dtype=torch.float32, device="cuda")
    M.mohge_fp8_decode(codes, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    ref = oracle.decode_e4m3(codes.cpu().numpy())
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(got[ok], ref[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(ref[ok]))


@pytest.mark.parametrize("T", [1, 9, 32])
def test_decode_with_fp8_weights(T):
    """Decode with quantised expert weights against the oracle run on the dequantised weights
    (scale * value(code), decoded by the oracle's own decoder)."""
    import paper_2604_23108_amd as M
    from gpu_harness import to_dev
    w = WORKLOADS["decode"].replace(T=T, d=1024, d_ff=(192, 256, 384, 512), seed=600 + T)
    inp = generate(w)
    DeviceLayer = _dev()
    dl = DeviceLayer(w, inp, training=False)
    L = dl.layer
    print(f"[fp8 weights] T={T} d={w.d}", flush=True)
    L.forward(dl.x)                                   # routing, permutation (and the bf16 result)
    q13, s13, q2, s2 = [], [], [], []
    for g in range(w.n_groups):
        c, s = M.quantize_rows_e4m3(L.w13[g]); q13.append(c); s13.append(s)
        c, s = M.quantize_rows_e4m3(L.w2[g]); q2.append(c); s2.append(s)
    y_perm = torch.full_like(L.y_perm, float("nan"))
    M.mohge_expert_ffn_w8(dl.cfg, dl.x, L.perm, L.offsets, q13, s13, q2, s2, y_perm, L.ws_ffn)
    y = torch.empty_like(L.y)
    M.mohge_combine(dl.cfg, y_perm, L.inv_perm, L.gates, y)
    torch.cuda.synchronize()
    # oracle on the dequantised weights
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    wg, wu, wd = [], [], []
    for g in range(w.n_groups):
        F = w.d_ff[g]
        w13 = oracle.dequantize_rows(q13[g].cpu().numpy(), s13[g].cpu().numpy())     # [N, 2F, d]
        wg.append(f32(w13[:, :F])); wu.append(f32(w13[:, F:]))
        wd.append(f32(oracle.dequantize_rows(q2[g].cpu().numpy(), s2[g].cpu().numpy())))
    # (fp32 holds scale * code exactly enough: 4 significant bits times an fp32 scale)
    r = oracle.route(w, inp.x.f32, inp.w_group, inp.w_expert, inp.expert_logit_bias)
    keep = r["margin"] >= MARGIN
    assert (L.expert_idx.cpu().numpy()[keep] == r["expert_idx"][keep]).all()
    tok = np.arange(w.T, dtype=np.int32)
    y_pairs = oracle.expert_ffn(w, inp.x.f32, wg, wu, wd, np.repeat(tok, w.k_experts), r["expert_idx"].reshape(-1))
    want = oracle.combine(w, y_pairs, r["gates"])
    got = y.float().cpu().numpy()
    assert np.isfinite(got).all()
    err = np.abs(got[keep] - want[keep]).max()
    assert err <= 2e-2 * np.abs(want).max(), f"error {err} vs {np.abs(want).max()}"
    # quantisation really happened: the result differs from the bf16-weight result, by little
    ref16 = L.y.float().cpu().numpy()
    dq = np.abs(got - ref16).max()
    assert 0 < dq <= 0.15 * np.abs(ref16).max()
    # prefill sizes are refused
    cfg_big = M.Config.from_workload(w.replace(T=64))
    with pytest.raises(M.MohgeError, match="decode"):
        M.mohge_expert_ffn_w8(cfg_big, dl.x, L.perm, L.offsets, q13, s13, q2, s2, y_perm, L.ws_ffn)


def test_mxfp4_conversion_matches_the_format():
    """Every (byte, scale) combination of interest through the hardware conversion the MXFP4
    kernel uses: all 256 byte values (both codes of a byte, so the order inside a byte is
    checked), scale codes 1..254."""
    import paper_2604_23108_amd as M
    rng = np.random.default_rng(5)
    nblk = 254 * 4
    packed = rng.integers(0, 256, size=(nblk, 16), dtype=np.uint8)
    packed[:16] = np.arange(256, dtype=np.uint8).reshape(16, 16)
    scales = (np.arange(nblk) % 254 + 1).astype(np.uint8)
    out = torch.full((nblk * 32,), 123.0, dtype=torch.float32, device="cuda")
    M.mohge_mxfp4_decode(torch.from_numpy(packed).cuda(), torch.from_numpy(scales).cuda(), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64).reshape(nblk, 32)
    ref = oracle.dequantize_mxfp4(packed, scales[:, None])
    # bf16 holds 2 significant bits times 2^(code-127) exactly unless the product is outside its
    # normal range (scale code 1 with the element 0.5, codes 253 and 254 with large elements):
    # those are excluded
    ok = (ref == 0) | ((np.abs(ref) >= 2.0 ** -126) & (np.abs(ref) < 2.0 ** 128))
    assert ok.mean() > 0.98
    bad = ok & (got != ref)
    assert not bad.any(), (int(bad.sum()), got[bad][:8], ref[bad][:8], np.argwhere(bad)[:8])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(ref[ok]))
    with pytest.raises(M.MohgeError, match="multiple"):
        M.mohge_mxfp4_decode(torch.from_numpy(packed).cuda(), torch.from_numpy(scales).cuda(), out[:40])


@pytest.mark.parametrize("T,d", [(1, 1024), (9, 1088), (32, 1024)])
def test_decode_with_mxfp4_weights(T, d):
    """Decode with MXFP4 expert weights against the oracle run on the dequantised weights
    (block scale * value(code), decoded by the oracle's own decoders).  Widths and d cover
    reduction lengths that end in a full, a half and no partial unit of 128."""
    import paper_2604_23108_amd as M
    w = WORKLOADS["decode"].replace(T=T, d=d, d_ff=(192, 256, 384, 512), seed=700 + T)
    inp = generate(w)
    DeviceLayer = _dev()
    dl = DeviceLayer(w, inp, training=False)
    L = dl.layer
    print(f"[mxfp4 weights] T={T} d={w.d}", flush=True)
    L.forward(dl.x)                                   # routing, permutation (and the bf16 result)
    q13, s13, q2, s2 = [], [], [], []
    for g in range(w.n_groups):
        c, s = M.quantize_mxfp4(L.w13[g]); q13.append(c); s13.append(s)
        c, s = M.quantize_mxfp4(L.w2[g]); q2.append(c); s2.append(s)
    y_perm = torch.full_like(L.y_perm, float("nan"))
    M.mohge_expert_ffn_w4(dl.cfg, dl.x, L.perm, L.offsets, q13, s13, q2, s2, y_perm, L.ws_ffn)
    y = torch.empty_like(L.y)
    M.mohge_combine(dl.cfg, y_perm, L.inv_perm, L.gates, y)
    torch.cuda.synchronize()
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    wg, wu, wd = [], [], []
    for g in range(w.n_groups):
        F = w.d_ff[g]
        w13 = oracle.dequantize_mxfp4(q13[g].cpu().numpy(), s13[g].cpu().numpy())     # [N, 2F, d]
        assert w13.shape == (w.experts_per_group, 2 * F, w.d)
        wg.append(f32(w13[:, :F])); wu.append(f32(w13[:, F:]))
        wd.append(f32(oracle.dequantize_mxfp4(q2[g].cpu().numpy(), s2[g].cpu().numpy())))
    r = oracle.route(w, inp.x.f32, inp.w_group, inp.w_expert, inp.expert_logit_bias)
    keep = r["margin"] >= MARGIN
    assert (L.expert_idx.cpu().numpy()[keep] == r["expert_idx"][keep]).all()
    tok = np.arange(w.T, dtype=np.int32)
    y_pairs = oracle.expert_ffn(w, inp.x.f32, wg, wu, wd, np.repeat(tok, w.k_experts), r["expert_idx"].reshape(-1))
    want = oracle.combine(w, y_pairs, r["gates"])
    got = y.float().cpu().numpy()
    assert np.isfinite(got).all()
    err = np.abs(got[keep] - want[keep]).max()
    assert err <= 2e-2 * np.abs(want).max(), f"error {err} vs {np.abs(want).max()}"
    assert np.abs(got - L.y.float().cpu().numpy()).max() > 0          # quantisation really happened
    cfg_big = M.Config.from_workload(w.replace(T=64))
    with pytest.raises(M.MohgeError, match="decode"):
        M.mohge_expert_ffn_w4(cfg_big, dl.x, L.perm, L.offsets, q13, s13, q2, s2, y_perm, L.ws_ffn)


def test_decode_kernels_with_many_tokens_on_one_expert():
    """The MXFP4 kernel stages an expert's tokens in LDS 16 at a time, in chunks of the reduction
    dimension that shrink as the token count grows: a hand-made, heavily skewed assignment
    (experts with 23, 17, 16, 5, 3 tokens, most with none) against the oracle."""
    import paper_2604_23108_amd as M
    w = WORKLOADS["decode"].replace(T=32, d=2048, d_ff=(192, 320, 512, 1024), seed=741)
    inp = generate(w)
    DeviceLayer = _dev()
    dl = DeviceLayer(w, inp, training=False)
    L = dl.layer
    rng = np.random.default_rng(3)
    Ne = w.n_groups * w.experts_per_group
    eidx = np.zeros((w.T, w.k_experts), np.int32)
    heavy = [(0, 23), (Ne - 1, 17), (17, 16), (34, 5), (50, 3)]       # (expert, tokens), slot s of token t
    free = [[s for s in range(w.k_experts)] for _ in range(w.T)]
    eidx[:] = -1
    for e, n in heavy:
        for t in rng.permutation(w.T)[:n]:
            if free[t]:
                eidx[t, free[t].pop(0)] = e
    others = [e for e in range(Ne) if e not in dict(heavy)]
    for t in range(w.T):
        for s in free[t]:
            eidx[t, s] = others[rng.integers(len(others))]
    ed = torch.from_numpy(eidx).cuda()
    M.mohge_permute(dl.cfg, ed, L.counts, L.offsets, L.perm, L.inv_perm, None, None, L.ws_permute)
    q13, s13, q2, s2 = [], [], [], []
    for g in range(w.n_groups):
        c, s = M.quantize_mxfp4(L.w13[g]); q13.append(c); s13.append(s)
        c, s = M.quantize_mxfp4(L.w2[g]); q2.append(c); s2.append(s)
    y_perm = torch.full_like(L.y_perm, float("nan"))
    print("[mxfp4 skewed] counts", np.bincount(eidx.reshape(-1), minlength=Ne).max(), flush=True)
    M.mohge_expert_ffn_w4(dl.cfg, dl.x, L.perm, L.offsets, q13, s13, q2, s2, y_perm, L.ws_ffn)
    torch.cuda.synchronize()
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    wg, wu, wd = [], [], []
    for g in range(w.n_groups):
        F = w.d_ff[g]
        w13 = oracle.dequantize_mxfp4(q13[g].cpu().numpy(), s13[g].cpu().numpy())
        wg.append(f32(w13[:, :F])); wu.append(f32(w13[:, F:]))
        wd.append(f32(oracle.dequantize_mxfp4(q2[g].cpu().numpy(), s2[g].cpu().numpy())))
    tok = np.arange(w.T, dtype=np.int32)
    y_pairs = oracle.expert_ffn(w, inp.x.f32, wg, wu, wd, np.repeat(tok, w.k_experts), eidx.reshape(-1))
    perm = L.perm.cpu().numpy()
    got = y_perm.float().cpu().numpy()
    want = y_pairs[perm]                               # sorted position p holds pair perm[p]
    assert np.isfinite(got).all()
    err = np.abs(got - want).max()
    assert err <= 2e-2 * np.abs(want).max(), f"error {err} vs {np.abs(want).max()}"
    # and the bf16 and FP8 kernels on the same skewed assignment
    y16 = torch.full_like(L.y_perm, float("nan"))
    M.mohge_expert_ffn(dl.cfg, dl.x, L.perm, L.offsets, L.w13, L.w2, y16, L.ws_ffn)
    torch.cuda.synchronize()
    y_pairs16 = oracle.expert_ffn(w, inp.x.f32, [t.f32 for t in inp.w_gate], [t.f32 for t in inp.w_up],
                                  [t.f32 for t in inp.w_down], np.repeat(tok, w.k_experts), eidx.reshape(-1))
    err16 = np.abs(y16.float().cpu().numpy() - y_pairs16[perm]).max()
    assert err16 <= 2e-2 * np.abs(y_pairs16).max()
    q13, s13, q2, s2 = [], [], [], []
    for g in range(w.n_groups):
        c, s = M.quantize_rows_e4m3(L.w13[g]); q13.append(c); s13.append(s)
        c, s = M.quantize_rows_e4m3(L.w2[g]); q2.append(c); s2.append(s)
    y8 = torch.full_like(L.y_perm, float("nan"))
    M.mohge_expert_ffn_w8(dl.cfg, dl.x, L.perm, L.offsets, q13, s13, q2, s2, y8, L.ws_ffn)
    torch.cuda.synchronize()
    wg, wu, wd = [], [], []
    for g in range(w.n_groups):
        F = w.d_ff[g]
        w13 = oracle.dequantize_rows(q13[g].cpu().numpy(), s13[g].cpu().numpy())
        wg.append(f32(w13[:, :F])); wu.append(f32(w13[:, F:]))
        wd.append(f32(oracle.dequantize_rows(q2[g].cpu().numpy(), s2[g].cpu().numpy())))
    y_pairs8 = oracle.expert_ffn(w, inp.x.f32, wg, wu, wd, np.repeat(tok, w.k_experts), eidx.reshape(-1))
    err8 = np.abs(y8.float().cpu().numpy() - y_pairs8[perm]).max()
    assert err8 <= 2e-2 * np.abs(y_pairs8).max()


def test_ffn_schedule_and_product_launch_issued_separately():
    """mohge_bench_expert_ffn: schedule (parts 1) then product launch (2) gives the bits of the one-call
    form, twice in a row; the decode path, where there is one launch only, refuses parts 1 and 2."""
    import paper_2604_23108_amd as M
    from paper_2604_23108_amd import bench_binding as BB
    w = WORKLOADS["mid_prefill"].replace(T=700, d=512, d_ff=(128, 256, 384), seed=811)
    inp = generate(w)
    DeviceLayer = _dev()
    dl = DeviceLayer(w, inp, training=False)
    L = dl.layer
    L.forward(dl.x)
    torch.cuda.synchronize()
    ref = L.y_perm.clone()
    for rep in range(2):
        y_perm = torch.full_like(L.y_perm, float("nan"))
        BB.mohge_bench_expert_ffn(dl.cfg, dl.x, L.perm, L.offsets, L.w13, L.w2, y_perm, L.ws_ffn, None, 1)
        BB.mohge_bench_expert_ffn(dl.cfg, dl.x, L.perm, L.offsets, L.w13, L.w2, y_perm, L.ws_ffn, None, 2)
        torch.cuda.synchronize()
        assert torch.equal(y_perm.view(torch.int16), ref.view(torch.int16)), rep
    y3 = torch.full_like(L.y_perm, float("nan"))
    BB.mohge_bench_expert_ffn(dl.cfg, dl.x, L.perm, L.offsets, L.w13, L.w2, y3, L.ws_ffn, None, 3)
    torch.cuda.synchronize()
    assert torch.equal(y3.view(torch.int16), ref.view(torch.int16))
    with pytest.raises(M.MohgeError, match="parts"):
        BB.mohge_bench_expert_ffn(dl.cfg, dl.x, L.perm, L.offsets, L.w13, L.w2, y3, L.ws_ffn, None, 4)
    wd = WORKLOADS["decode"].replace(T=8, d=512, d_ff=(128, 256, 384, 512), seed=812)
    dd = DeviceLayer(wd, generate(wd), training=False)
    dd.layer.forward(dd.x)
    with pytest.raises(M.MohgeError, match="separate launches"):
        BB.mohge_bench_expert_ffn(dd.cfg, dd.x, dd.layer.perm, dd.layer.offsets, dd.layer.w13, dd.layer.w2,
                                  dd.layer.y_perm, dd.layer.ws_ffn, None, 2)


def test_box_probes_run_and_report_their_work():
    """The measurement aids: every pattern of the read probe on a buffer that is not a whole number
    of its units, and the MFMA probe; argument errors."""
    import paper_2604_23108_amd as M
    from paper_2604_23108_amd import bench_binding as BB
    buf = torch.ones(3 * (1 << 20) + 4096, dtype=torch.uint8, device="cuda")
    out = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    n = BB.mohge_probe_read(buf, 0, False, out)
    assert 0 < n <= buf.numel() and n % (256 * 8 * 16) == 0
    for row in (512, 2048, 8192):
        for stag in (False, True):
            n = BB.mohge_probe_read(buf, row, stag, out)
            assert n == (buf.numel() // row // 128) * 128 * row, (row, stag)
    assert BB.mohge_probe_read(buf[:4096], 8192, False, out) == 0          # less than one unit: nothing launched
    flops = BB.mohge_probe_mfma(out, 100)
    assert flops == 1024 * 4 * 4 * 100 * 2.0 * 32 * 32 * 16
    torch.cuda.synchronize()
    with pytest.raises(M.MohgeError, match="row_bytes"):
        BB.mohge_probe_read(buf, 1000, False, out)
    with pytest.raises(M.MohgeError, match="needed"):
        BB.mohge_probe_mfma(out[:4096], 10)


@pytest.mark.parametrize("seed", range(10))
def test_quantised_decode_random_shapes(seed):
    """Seeded random decode shapes (hidden sizes and widths that are odd multiples of 64, one to
    four groups, 1 to 32 tokens) through both quantised-weight kernels against the oracle on the
    dequantised weights: reduction lengths that end in partial units, chunked token staging."""
    import paper_2604_23108_amd as M
    from synth import SELECT_GLOBAL, SELECT_PER_GROUP
    rng = np.random.default_rng(5000 + seed)
    Ng = int(rng.integers(1, 5))
    N = int(rng.integers(1, 7))
    d = int(rng.choice([64, 128, 192, 320, 448, 1024, 2112]))
    d_ff = tuple(int(64 * rng.integers(1, 9)) for _ in range(Ng))
    kg = int(rng.integers(1, Ng + 1))
    per = int(rng.integers(1, N + 1))
    mode = SELECT_PER_GROUP if rng.integers(2) else SELECT_GLOBAL
    ke = kg * per if mode == SELECT_PER_GROUP else int(rng.integers(1, kg * N + 1))
    T = int(rng.integers(1, 33))
    w = WORKLOADS["decode"].replace(T=T, d=d, n_groups=Ng, experts_per_group=N, d_ff=d_ff, k_groups=kg,
                                    k_experts=ke, select_mode=mode, seed=5100 + seed)
    inp = generate(w)
    DeviceLayer = _dev()
    dl = DeviceLayer(w, inp, training=False)
    L = dl.layer
    print(f"[quantised decode] seed={seed} T={T} d={d} d_ff={d_ff} {Ng}x{N} kg={kg} ke={ke} mode={mode}", flush=True)
    L.forward(dl.x)
    r = oracle.route(w, inp.x.f32, inp.w_group, inp.w_expert, inp.expert_logit_bias)
    keep = r["margin"] >= MARGIN
    tok = np.arange(w.T, dtype=np.int32)
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    for name, quant, deq, call in (("fp8", M.quantize_rows_e4m3, oracle.dequantize_rows, M.mohge_expert_ffn_w8),
                                   ("mxfp4", M.quantize_mxfp4, oracle.dequantize_mxfp4, M.mohge_expert_ffn_w4)):
        q13, s13, q2, s2 = [], [], [], []
        for g in range(w.n_groups):
            c, s = quant(L.w13[g]); q13.append(c); s13.append(s)
            c, s = quant(L.w2[g]); q2.append(c); s2.append(s)
        y_perm = torch.full_like(L.y_perm, float("nan"))
        call(dl.cfg, dl.x, L.perm, L.offsets, q13, s13, q2, s2, y_perm, L.ws_ffn)
        y = torch.empty_like(L.y)
        M.mohge_combine(dl.cfg, y_perm, L.inv_perm, L.gates, y)
        torch.cuda.synchronize()
        wg, wu, wd = [], [], []
        for g in range(w.n_groups):
            F = w.d_ff[g]
            w13 = deq(q13[g].cpu().numpy(), s13[g].cpu().numpy())
            wg.append(f32(w13[:, :F])); wu.append(f32(w13[:, F:]))
            wd.append(f32(deq(q2[g].cpu().numpy(), s2[g].cpu().numpy())))
        y_pairs = oracle.expert_ffn(w, inp.x.f32, wg, wu, wd, np.repeat(tok, w.k_experts), r["expert_idx"].reshape(-1))
        want = oracle.combine(w, y_pairs, r["gates"])
        got = y.float().cpu().numpy()
        assert np.isfinite(got).all(), name
        if keep.any():
            err = np.abs(got[keep] - want[keep]).max()
            assert err <= 2e-2 * max(np.abs(want).max(), 1e-6), f"{name}: error {err} vs {np.abs(want).max()}"


def test_shared_routing_with_the_largest_expert_count():
    # N_s = 256 always-on experts: offsets has 257 entries, one more than the filling kernel's block
    import paper_2604_23108_amd as M
    T, n_s = 5, 256
    cfg = M.Config(T=T, d=64, n_groups=1, experts_per_group=n_s, d_ff=(64,), k_groups=1, k_experts=n_s)
    i32 = dict(dtype=torch.int32, device="cuda")
    eidx, gates = torch.full((T, n_s), -1, **i32), torch.zeros((T, n_s), dtype=torch.float32, device="cuda")
    counts, offsets = torch.full((n_s,), -1, **i32), torch.full((n_s + 1,), -1, **i32)
    perm, inv = torch.full((T * n_s,), -1, **i32), torch.full((T * n_s,), -1, **i32)
    M.mohge_shared_routing(cfg, eidx, gates, counts, offsets, perm, inv)
    torch.cuda.synchronize()
    assert (offsets.cpu().numpy() == np.arange(n_s + 1) * T).all() and (counts == T).all()
    p = oracle.permute(WORKLOADS["tiny_f32"].replace(T=T, n_groups=1, experts_per_group=n_s, k_groups=1,
                                                     k_experts=n_s, d_ff=(64,)), eidx.cpu().numpy())
    assert (perm.cpu().numpy() == p["perm"]).all() and (inv.cpu().numpy() == p["inv_perm"]).all()
    assert (gates == 1).all()


@pytest.mark.parametrize("Ng,N,mode", [(3, 3, SELECT_PER_GROUP), (4, 16, SELECT_PER_GROUP), (4, 16, SELECT_GLOBAL),
                                       (8, 16, SELECT_GLOBAL), (16, 16, SELECT_PER_GROUP)])
def test_router_matrix_core_form_many_tokens(Ng, N, mode):
    # from 8192 bf16 tokens on the logits come from the bf16 matrix cores (router rows split into
    # three bf16 parts): 12 router rows (one column tile), 68 (one pass of five), 136 and 272
    # (several passes), a token count that is not a multiple of the 32 / 64 a workgroup takes
    import paper_2604_23108_amd as M
    from gpu_harness import to_dev
    w = Workload("route_mfma", T=8192 + 37, d=256, n_groups=Ng, experts_per_group=N, d_ff=(64,) * Ng,
                 k_groups=2, k_experts=4, select_mode=mode, seed=300 + Ng * N, skew_beta=1.0)
    inp = generate(w)
    inp.w_group *= np.float32(12)
    inp.w_expert *= np.float32(12)
    cfg = M.Config.from_workload(w)
    assert M.mohge_workspace_size(cfg, M.CALL_ROUTE) >= 3 * (Ng + Ng * N) * w.d * 2
    x = to_dev(inp.x, True)
    wg, we = torch.from_numpy(inp.w_group).cuda(), torch.from_numpy(inp.w_expert).cuda()
    bias = torch.from_numpy(inp.expert_logit_bias).cuda()
    i32 = dict(dtype=torch.int32, device="cuda")
    f32 = dict(dtype=torch.float32, device="cuda")
    outs = []
    for use_ws in (True, False):            # without the workspace: the fp32 matrix-core form
        gidx, eidx = torch.full((w.T, w.k_groups), -1, **i32), torch.full((w.T, w.k_experts), -1, **i32)
        gates, gs, es1 = torch.zeros((w.T, w.k_experts), **f32), torch.zeros((w.T, Ng), **f32), torch.zeros((w.T, Ng * N), **f32)
        ws = torch.empty(M.mohge_workspace_size(cfg, M.CALL_ROUTE), dtype=torch.uint8, device="cuda") if use_ws else None
        print(f"[router] Ng={Ng} N={N} mode={mode} workspace={use_ws}", flush=True)
        M.mohge_route(cfg, x, wg, we, bias, gidx, eidx, gates, gs, es1, ws)
        torch.cuda.synchronize()
        outs.append(dict(group_idx=gidx.cpu().numpy(), expert_idx=eidx.cpu().numpy(), gates=gates.cpu().numpy(),
                         gs=gs.cpu().numpy(), es1=es1.cpu().numpy()))
    ref = oracle.route(w, inp.x.f32, inp.w_group, inp.w_expert, inp.expert_logit_bias)
    for out in outs:
        keep, _ = check_routing(w, out, ref, "router, many tokens")
        np.testing.assert_allclose(out["gs"], ref["gs"], atol=1e-6)
        np.testing.assert_allclose(out["es1"][keep], ref["es1"][keep], atol=1e-6, rtol=2e-6)


def test_guard_bands_notice_a_write_outside_a_tensor():
    # the canaries the harness puts around every output tensor do report a stray write (made here
    # by the host, next to the tensor: no kernel is asked to misbehave)
    from gpu_harness import GuardBands
    g = GuardBands()
    t = g.wrap(torch.zeros((5, 3), dtype=torch.float32, device="cuda"), "t")
    t.fill_(1.0)
    g.check()
    buf = g.items[0][1]
    buf[GuardBands.PAD + 5 * 3 * 4] = 0          # first byte behind the tensor
    with pytest.raises(AssertionError, match="behind t"):
        g.check()
