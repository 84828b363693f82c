"""GPU parity of mohge_decode_layer (the whole layer of a decode-sized call as one launch): against
the CPU oracle with the bars of the other parity tests, and bit by bit against the four separate
calls on the same inputs."""
import numpy as np
import pytest
import torch

import oracle
from synth import SELECT_GLOBAL, SELECT_PER_GROUP, WORKLOADS, Workload, generate
from test_gpu_parity import check_output, check_permutation, check_routing

pytestmark = pytest.mark.gpu


def _layer(w, inp):
    from gpu_harness import DeviceLayer
    return DeviceLayer(w, inp, training=False)


def _ctl_is_zero(M, L):
    n = M.mohge_decode_layer_ctl_bytes(L.cfg)
    assert 0 < n <= L.ws_decode.numel()
    return not bool(L.ws_decode[:n].any())


def run_decode(w, inp, calls=1):
    """forward_decode on fresh buffers; returns the outputs in the layout of DeviceLayer.run()."""
    import paper_2604_23108_amd as M
    dl = _layer(w, inp)
    L = dl.layer
    for _ in range(calls):
        L.y.fill_(float("nan"))
        y = L.forward_decode(dl.x)
        torch.cuda.synchronize()
        assert M.mohge_fused_status(L.cfg, M.CALL_DECODE_LAYER, L.ws_decode) == 0, M.mohge_last_error()
        assert _ctl_is_zero(M, L), "the call left counters in the workspace"
    dl.check_guards()
    # the permutation lives in the call's workspace: rebuild it from the routing the call produced
    eidx = L.expert_idx.cpu().numpy()
    p = oracle.permute(w, eidx)
    from gpu_harness import from_dev
    return dl, dict(group_idx=L.group_idx.cpu().numpy(), expert_idx=eidx, gates=L.gates.cpu().numpy(),
                    y=from_dev(y), inv_perm=p["inv_perm"])


def check_against_oracle(w, inp, out):
    ref = oracle.route(w, inp.x.f32, inp.w_group, inp.w_expert, inp.expert_logit_bias)
    keep, _ = check_routing(w, out, ref, w.name)
    tokens = np.asarray([t for t in range(w.T) if keep[t]], np.int32)
    pair_token = np.repeat(tokens, w.k_experts)
    pair_expert = ref["expert_idx"][tokens].reshape(-1)
    y_pairs = oracle.expert_ffn(w, inp.x.f32, [t.f32 for t in inp.w_gate], [t.f32 for t in inp.w_up],
                                [t.f32 for t in inp.w_down], pair_token, pair_expert)
    y_ref = oracle.combine(w, y_pairs, ref["gates"][tokens])
    err = np.abs(out["y"][tokens] - y_ref).max()
    assert np.isfinite(out["y"]).all()
    assert err <= 2e-2 * np.abs(y_ref).max(), f"y error {err} vs max|ref| {np.abs(y_ref).max()}"
    assert np.abs(out["gates"].sum(axis=1) - 1.0).max() <= 2e-6 and (out["gates"] > 0).all()


@pytest.mark.parametrize("T", [1, 7, 32])
@pytest.mark.parametrize("mode", [SELECT_PER_GROUP, SELECT_GLOBAL])
def test_decode_layer_small_shapes_against_oracle(T, mode):
    w = Workload("dec1", T=T, d=512, n_groups=4, experts_per_group=4, d_ff=(64, 128, 192, 256),
                 k_groups=2, k_experts=4, seed=130 + T, select_mode=mode)
    inp = generate(w)
    inp.w_group *= np.float32(4.0)
    inp.w_expert *= np.float32(4.0)
    _, out = run_decode(w, inp, calls=2)
    check_against_oracle(w, inp, out)


@pytest.mark.parametrize("mode", [SELECT_PER_GROUP, SELECT_GLOBAL])
def test_decode_layer_full_size_every_token(mode):
    w = WORKLOADS["decode"].replace(select_mode=mode)
    inp = generate(w)
    _, out = run_decode(w, inp, calls=2)
    check_against_oracle(w, inp, out)


@pytest.mark.parametrize("shape", ["decode", "odd"])
def test_decode_layer_equals_the_separate_calls_bit_by_bit(shape):
    """The routing of the separate router call up to the last bits of the gates, and, given the
    routing, the same bits in y: every unit runs the code of the separate launches."""
    import paper_2604_23108_amd as M
    if shape == "decode":
        w = WORKLOADS["decode"]
    else:
        # d not a multiple of 128 or 256, widths that leave partial units, a logit bias, an expert
        # count that is no power of two, fewer than 16 tokens
        w = Workload("dec2", T=13, d=832, n_groups=3, experts_per_group=5, d_ff=(64, 320, 192), k_groups=2,
                     k_experts=4, seed=77)
    inp = generate(w)
    if shape == "odd":
        rng = np.random.default_rng(5)
        inp.expert_logit_bias = rng.normal(0, 1, w.n_experts).astype(np.float32)
    dl = _layer(w, inp)
    L, c = dl.layer, dl.layer.cfg
    L.forward(dl.x)
    torch.cuda.synchronize()
    sep = dict(e=L.expert_idx.clone(), g=L.group_idx.clone(), gates=L.gates.clone(), y=L.y.clone())
    for call in range(3):
        L.expert_idx.fill_(-1); L.group_idx.fill_(-1); L.gates.fill_(0); L.y.fill_(float("nan"))
        y_one = L.forward_decode(dl.x).clone()
        torch.cuda.synchronize()
        assert M.mohge_fused_status(c, M.CALL_DECODE_LAYER, L.ws_decode) == 0, M.mohge_last_error()
        assert torch.equal(L.expert_idx, sep["e"]) and torch.equal(L.group_idx, sep["g"]), f"call {call}: routing differs"
        # the two router forms group their fp64 partial sums differently: a gate may differ in its last bits
        assert (L.gates - sep["gates"]).abs().max().item() <= 2.4e-7
        assert torch.isfinite(y_one.float()).all()
        assert (y_one.float() - sep["y"].float()).abs().max().item() <= 1e-2 * sep["y"].float().abs().max().item()
        # the separate calls on the routing the single launch produced: the same bits
        L.y.fill_(float("nan"))
        M.mohge_permute(c, L.expert_idx, L.counts, L.offsets, L.perm, L.inv_perm, None, None, L.ws_permute)
        M.mohge_expert_ffn(c, dl.x, L.perm, L.offsets, L.w13, L.w2, L.y_perm, L.ws_ffn)
        M.mohge_combine(c, L.y_perm, L.inv_perm, L.gates, L.y)
        torch.cuda.synchronize()
        assert torch.equal(y_one.view(torch.int16), L.y.view(torch.int16)), f"call {call}: y differs in bits"
    dl.check_guards()


def test_decode_layer_all_tokens_on_one_expert_per_group():
    w = Workload("dec3", T=32, d=256, n_groups=2, experts_per_group=4, d_ff=(64, 128), k_groups=2, k_experts=2, seed=41)
    inp = generate(w)
    bias = np.zeros(w.n_experts, np.float32)
    bias[1] = 50.0
    bias[6] = 50.0
    inp.expert_logit_bias = bias
    _, out = run_decode(w, inp)
    assert (out["expert_idx"] == np.array([1, 6])).all()
    check_against_oracle(w, inp, out)


def test_decode_layer_argument_checks_and_empty_call():
    import paper_2604_23108_amd as M
    w = WORKLOADS["decode"].replace(T=33)
    assert M.mohge_workspace_size(M.Config.from_workload(w), M.CALL_DECODE_LAYER) == 0
    inp = generate(w.replace(d=256, d_ff=(64, 64, 64, 64)))
    dl = _layer(w.replace(d=256, d_ff=(64, 64, 64, 64)), inp)
    L = dl.layer
    L.ws_decode = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(M.MohgeError, match="at most 32 tokens"):
        L.forward_decode(dl.x)
    w2 = Workload("dec4", T=4, d=256, n_groups=2, experts_per_group=4, d_ff=(64, 128), k_groups=2, k_experts=2, seed=3)
    dl = _layer(w2, generate(w2))
    dl.layer.ws_decode = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(M.MohgeError, match="workspace"):
        dl.layer.forward_decode(dl.x)
    # T = 0: nothing to do, no launch, nothing written
    L = dl.layer
    cfg0 = M.Config.from_workload(w2.replace(T=0))
    y = torch.full((4, w2.d), 7.0, dtype=torch.bfloat16, device="cuda")
    M.mohge_decode_layer(cfg0, dl.x, L.w_group, L.w_expert, None, L.w13, L.w2, L.group_idx, L.expert_idx, L.gates, y,
                         torch.zeros(M.mohge_workspace_size(cfg0, M.CALL_DECODE_LAYER), dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())


def test_decode_layer_failures_are_loud():
    """A workspace whose counters are not zero, and waits that expire (forced from the host): the
    launch drains, y is NaN and the status call says which."""
    import paper_2604_23108_amd as M
    from paper_2604_23108_amd import bench_binding as BB
    w = Workload("dec5", T=9, d=512, n_groups=4, experts_per_group=4, d_ff=(64, 128, 192, 256), k_groups=2,
                 k_experts=4, seed=8)
    inp = generate(w)
    dl = _layer(w, inp)
    L = dl.layer
    good = L.forward_decode(dl.x).clone()
    torch.cuda.synchronize()
    # every dependent workgroup gives up at once
    L.y.zero_()
    BB.mohge_bench_decode_layer(L.cfg, dl.x, L.w_group, L.w_expert, L.bias, L.w13, L.w2, L.group_idx, L.expert_idx,
                                L.gates, L.y, L.ws_decode, spin_limit=-1)
    torch.cuda.synchronize()
    assert M.mohge_fused_status(L.cfg, M.CALL_DECODE_LAYER, L.ws_decode) == -6
    assert "gave up" in M.mohge_last_error()
    assert bool(torch.isnan(L.y.float()).all())
    assert _ctl_is_zero(M, L)
    # ... and the next ordinary call on the same workspace is right again
    y = L.forward_decode(dl.x)
    torch.cuda.synchronize()
    assert M.mohge_fused_status(L.cfg, M.CALL_DECODE_LAYER, L.ws_decode) == 0
    assert torch.equal(y.view(torch.int16), good.view(torch.int16))
    # counters that are not zero at the start
    n = M.mohge_decode_layer_ctl_bytes(L.cfg)
    L.ws_decode[:n].fill_(0x7F)
    L.y.zero_()
    L.forward_decode(dl.x)
    torch.cuda.synchronize()
    assert M.mohge_fused_status(L.cfg, M.CALL_DECODE_LAYER, L.ws_decode) == -1
    assert "not zero" in M.mohge_last_error()
    assert bool(torch.isnan(L.y.float()).all())
    dl.check_guards()


def test_decode_layer_time_stamps_of_the_benchmark_library():
    """The optional trace: every piece of work that ran left a start and an end, in that order, and
    the result is the one of the plain call."""
    import paper_2604_23108_amd as M
    from paper_2604_23108_amd import bench_binding as BB
    w = Workload("dec6", T=11, d=768, n_groups=3, experts_per_group=4, d_ff=(64, 128, 256), k_groups=2, k_experts=4, seed=12)
    dl = _layer(w, generate(w))
    L = dl.layer
    good = L.forward_decode(dl.x).clone()
    tr = BB.decode_trace_buffer(L.cfg)
    BB.mohge_bench_decode_layer(L.cfg, dl.x, L.w_group, L.w_expert, L.bias, L.w13, L.w2, L.group_idx, L.expert_idx,
                                L.gates, L.y, L.ws_decode, 0, tr)
    torch.cuda.synchronize()
    assert M.mohge_fused_status(L.cfg, M.CALL_DECODE_LAYER, L.ws_decode) == 0
    assert torch.equal(L.y.view(torch.int16), good.view(torch.int16))
    t = tr.cpu().numpy()
    counts = np.bincount(L.expert_idx.cpu().numpy().reshape(-1), minlength=w.n_experts)
    F_e = np.repeat(np.asarray(w.d_ff), w.experts_per_group)
    pieces = 1 * 1 * 3 + 3 + int(((counts > 0) * (F_e // 64)).sum()) + int((counts > 0).sum()) * 6
    assert pieces <= t.shape[0]
    assert (t[:pieces, 0] > 0).all() and (t[:pieces, 3] >= t[:pieces, 0]).all() and (t[pieces:] == 0).all()
    with pytest.raises(M.MohgeError, match="trace"):
        BB.mohge_bench_decode_layer(L.cfg, dl.x, L.w_group, L.w_expert, L.bias, L.w13, L.w2, L.group_idx, L.expert_idx,
                                    L.gates, L.y, L.ws_decode, 0, tr[:4])
    dl.check_guards()
