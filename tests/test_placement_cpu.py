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
