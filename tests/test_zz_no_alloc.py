"""mohge_permute_static (the entry point that allocates nothing: its scratch is a static device
array inside the library) against mohge_permute, through the C ABI, on consecutive calls that
share the array: a large input, then a smaller one, then the three-kernel path."""
import numpy as np
import pytest
import torch

from synth import Workload

pytestmark = pytest.mark.gpu


def _both(M, T, Ng, N, seed, with_x):
    w = Workload("perm", T=T, d=64, n_groups=Ng, experts_per_group=N, d_ff=(64,) * Ng, k_groups=2,
                 k_experts=4, seed=0)
    rng = np.random.default_rng(seed)
    pmf = 1.0 / (1.0 + np.arange(w.n_experts)) ** 1.1
    eidx_h = rng.choice(w.n_experts, size=(T, 4), p=pmf / pmf.sum()).astype(np.int32)
    cfg = M.Config.from_workload(w)
    i32 = dict(dtype=torch.int32, device="cuda")
    eidx = torch.from_numpy(eidx_h).cuda()
    x = torch.randn((T, 64), device="cuda").to(torch.bfloat16) if with_x else None
    res = []
    for static in (False, True):
        counts, offsets = torch.full((w.n_experts,), -1, **i32), torch.full((w.n_experts + 1,), -1, **i32)
        perm, inv = torch.full((w.n_pairs,), -1, **i32), torch.full((w.n_pairs,), -1, **i32)
        x_perm = torch.zeros((w.n_pairs, 64), dtype=torch.bfloat16, device="cuda") if with_x else None
        if static:
            M.mohge_permute_static(cfg, eidx, counts, offsets, perm, inv, x, x_perm)
        else:
            ws = torch.empty(M.mohge_workspace_size(cfg, M.CALL_PERMUTE), dtype=torch.uint8, device="cuda")
            M.mohge_permute(cfg, eidx, counts, offsets, perm, inv, x, x_perm, ws)
        torch.cuda.synchronize()
        res.append((counts, offsets, perm, inv, x_perm))
    for a, b in zip(*res):
        if a is not None:
            assert torch.equal(a, b)
    # and the result is a permutation at all (the two calls share kernels)
    perm = res[1][2].cpu().numpy()
    assert (np.sort(perm) == np.arange(w.n_pairs)).all()
    assert int(res[1][1][-1]) == w.n_pairs


def test_permute_static_matches_permute_on_consecutive_calls():
    import paper_2604_23108_amd as M
    print("[no-alloc] T=16384 (two-launch path)", flush=True)
    _both(M, 16384, 4, 16, 1, False)
    print("[no-alloc] T=1500 (smaller input, same array)", flush=True)
    _both(M, 1500, 4, 16, 2, True)
    print("[no-alloc] T=41000, 64 experts (three-launch path)", flush=True)
    _both(M, 41000, 8, 8, 3, False)
    print("[no-alloc] T=300 (single workgroup, no scratch)", flush=True)
    _both(M, 300, 3, 4, 4, False)


def test_permute_static_rejects_sizes_beyond_its_array():
    import paper_2604_23108_amd as M
    # 256 experts x (P / 512) segments x 4 bytes > 1 MiB  <=>  P > 2^19
    cfg = M.Config(T=200000, d=64, n_groups=16, experts_per_group=16, d_ff=(64,) * 16, k_groups=2, k_experts=4)
    assert M.mohge_workspace_size(cfg, M.CALL_PERMUTE) > (1 << 20)
    t = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(M.MohgeError, match="static buffer"):
        M.mohge_permute_static(cfg, t, t, t, t, t, None, None)
