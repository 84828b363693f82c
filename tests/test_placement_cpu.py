"""The All-size Group-decoupling Allocation rule (paper section 3.4.1) as a host function."""
import numpy as np
import pytest

import oracle
from paper_2604_23108_amd import placement
from synth import WORKLOADS, generate


def test_every_gpu_gets_the_same_indices_of_every_group_and_equal_bytes():
    Ng, N, R = 8, 16, 8
    seen = set()
    for r in range(R):
        for mode in ("contiguous", "strided"):
            ids = placement.local_global_ids(Ng, N, R, r, mode)
            assert ids.shape == (Ng, N // R)
            # same in-group indices in every group: an all-size set per column
            assert (ids % N == ids[0] % N).all() and (ids // N == np.arange(Ng)[:, None]).all()
        seen.update(placement.local_expert_indices(N, R, r))
    assert seen == set(range(N))
    b = placement.parameter_bytes_per_gpu(1024, (640, 768, 896, 1024, 1152, 1280, 1408, 1536), N, R)
    assert len(set(b)) == 1
    # the paper's experiment: the i-th expert of each group on the i-th GPU
    assert [placement.owner_of(i, 8, 8, "strided") for i in range(8)] == list(range(8))
    with pytest.raises(ValueError):
        placement.local_expert_indices(10, 4, 0)


def test_balanced_intra_group_routing_gives_balanced_gpus():
    # synthetic stand-in for the per-GPU load table: with (near) uniform routing inside the
    # groups every GPU receives about 1/R of every group's tokens and of the FLOPs
    w = WORKLOADS["paper_14b"].replace(T=8192, d=64)
    inp = generate(w)
    r = oracle.route(w, inp.x.f32, inp.w_group, inp.w_expert)
    rep = placement.load_report(r["expert_idx"], w.n_groups, w.experts_per_group, 8, w.d_ff)
    np.testing.assert_allclose(rep["share_by_group"].sum(axis=1), 1.0)
    assert np.abs(rep["share_by_group"] - 0.125).max() < 0.08
    assert np.abs(rep["flop_share"] - 0.125).max() < 0.02


def test_a_local_share_is_itself_a_layer():
    # the experts a GPU holds form an N_g x N_local layer: routing restricted to them uses
    # exactly the router rows of those experts
    w = WORKLOADS["tiny_f32"]
    inp = generate(w)
    ids = placement.local_global_ids(w.n_groups, w.experts_per_group, 2, 1)
    local = w.replace(experts_per_group=2)
    r = oracle.route(local, inp.x.f32, inp.w_group, inp.w_expert[ids.reshape(-1)])
    assert r["expert_idx"].max() < local.n_experts


def test_load_report_table_prints_the_shares_it_was_given():
    # hand-made routing: 2 groups x 4 experts on 2 virtual GPUs (contiguous: experts 0,1 | 2,3)
    eidx = np.array([[0, 4], [1, 5], [2, 6], [0, 7], [1, 4], [0, 5]])      # group 0: 0,1,2,0,1,0  group 1: 0,1,2,3,0,1
    rep = placement.load_report(eidx, 2, 4, 2, (64, 128))
    np.testing.assert_allclose(rep["share_by_group"], [[5 / 6, 1 / 6], [4 / 6, 2 / 6]])
    np.testing.assert_allclose(rep["flop_share"], [(5 * 64 + 4 * 128) / (6 * 192), (64 + 2 * 128) / (6 * 192)])
    text = placement.format_report(rep, "title")
    rows = text.splitlines()
    assert rows[0] == "title" and rows[1].split() == ["GPU", "grp0", "grp1", "FLOPs"]
    assert rows[2].split() == ["0", "83.33", "66.67", "72.22"]
    assert rows[3].split() == ["1", "16.67", "33.33", "27.78"]
    assert "ideal 50.00 %" in rows[4] and "33.33 points" in rows[4]
    # strided sets: experts 0,2 | 1,3
    rep2 = placement.load_report(eidx, 2, 4, 2, (64, 128), "strided")
    np.testing.assert_allclose(rep2["share_by_group"], [[4 / 6, 2 / 6], [3 / 6, 3 / 6]])
