"""Host-side checks of the C boundary that need no GPU: the library loads, exports every
symbol the header declares, validates configurations and reports workspace sizes."""
import ctypes as C
import os
import re

import pytest

import paper_2604_23108_amd as M
from paper_2604_23108_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    from paper_2604_23108_amd import bench_binding
    for hdr, exports, lib in (("mohge.h", binding.EXPORTS, M.lib()),
                              ("mohge_bench.h", bench_binding.EXPORTS, bench_binding.lib())):
        header = open(os.path.join(ROOT, "include", hdr)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)          # declarations only
        declared = set(re.findall(r"\b(mohge_[a-z_0-9]+)\s*\(", header))
        assert declared == set(exports), hdr
        for name in declared:
            assert hasattr(lib, name), name
    # the layer header carries no measurement or tuning hooks
    layer = open(os.path.join(ROOT, "include", "mohge.h")).read()
    assert "probe" not in layer and "mohge_tune" not in layer


def test_struct_layout_matches_header():
    # 4 int32, pointer, 4 int32, 3 float, int32 -> 4*4 + 8 + 4*4 + 3*4 + 4 = 56 bytes on LP64
    assert C.sizeof(binding._CConfig) == 56
    assert binding._CConfig.d_ff.offset == 16 and binding._CConfig.k_groups.offset == 24


@pytest.mark.parametrize("kw,msg", [
    (dict(d=100), "multiple of 64"),
    (dict(n_groups=17, d_ff=(64,) * 17), "n_groups"),
    (dict(experts_per_group=100), "outside 1.."),
    (dict(k_groups=4), "k_groups"),
    (dict(k_experts=9), "k_experts"),
    (dict(k_experts=3), "per-group"),
    (dict(select_mode=7), "select_mode"),
    (dict(dtype=5), "dtype"),
    (dict(d_ff=(64, 100, 128)), "d_ff[1]"),
    (dict(T=-1), "negative"),
])
def test_invalid_configs_are_rejected_with_a_message(kw, msg):
    base = dict(T=64, d=128, n_groups=3, experts_per_group=4, d_ff=(64, 128, 256), k_groups=2, k_experts=2)
    base.update(kw)
    cfg = M.Config(**base)
    assert M.mohge_workspace_size(cfg, M.CALL_PERMUTE) == 0
    assert msg in M.mohge_last_error()
    # every entry point refuses it before touching any pointer
    rc = M.lib().mohge_combine(cfg.ref(), None, None, None, None, None)
    assert rc == -1


def test_null_pointers_and_workspace_sizes():
    cfg = M.Config(T=4096, d=2048, n_groups=3, experts_per_group=8, d_ff=(512, 1024, 1536), k_groups=2, k_experts=4)
    assert M.lib().mohge_combine(cfg.ref(), None, None, None, None, None) == -2
    assert "NULL" in M.mohge_last_error()
    assert M.lib().mohge_route(None, None, None, None, None, None, None, None, None, None, None, 0, None) == -2
    P = 4096 * 4
    # hidden activations plus the tile schedules of the matrix-core path
    assert P * 1536 * 2 <= M.mohge_workspace_size(cfg, M.CALL_EXPERT_FFN) <= P * 1536 * 2 + (1 << 20)
    assert M.mohge_workspace_size(cfg, M.CALL_PERMUTE) >= (P // 512) * 24 * 4
    assert M.mohge_workspace_size(cfg, M.CALL_AUX_LOSS) > 0
    assert M.mohge_workspace_size(cfg, 99) == 0
    f32 = M.Config(T=64, d=128, n_groups=3, experts_per_group=4, d_ff=(64, 128, 256), k_groups=2, k_experts=2, dtype=M.F32)
    assert M.mohge_workspace_size(f32, M.CALL_EXPERT_FFN) == 128 * 256 * 4


def test_binding_refuses_cpu_tensors():
    import torch
    cfg = M.Config(T=64, d=128, n_groups=3, experts_per_group=4, d_ff=(64, 128, 256), k_groups=2, k_experts=2)
    t = torch.zeros(4)
    with pytest.raises(M.MohgeError, match="GPU"):
        M.mohge_combine(cfg, t, t, t, t)


def test_training_entry_points_check_their_arguments():
    cfg = M.Config(T=8192, d=2048, n_groups=3, experts_per_group=8, d_ff=(512, 1024, 1536), k_groups=2, k_experts=4)
    P, Fmax, d = 8192 * 4, 1536, 2048
    # saved = schedules + h [P, Fmax] + pre-activations [P, 2 Fmax]
    saved = M.mohge_workspace_size(cfg, M.CALL_FFN_SAVED)
    assert 3 * P * Fmax * 2 <= saved <= 3 * P * Fmax * 2 + (1 << 20)
    # backward workspace holds [dA|dB] and the rows of x in sorted order
    bwd = M.mohge_workspace_size(cfg, M.CALL_EXPERT_FFN_BWD)
    need = P * 2 * Fmax * 2 + P * d * 2
    assert need <= bwd <= need + (1 << 20)
    assert M.mohge_workspace_size(cfg, M.CALL_ROUTE_BWD) >= 8192 * 27 * 4
    lib = M.lib()
    assert lib.mohge_combine_bwd(cfg.ref(), None, None, None, None, None, None, None) == -2
    assert "NULL" in M.mohge_last_error()
    assert lib.mohge_expert_ffn_bwd(cfg.ref(), *([None] * 13)) == -2
    assert lib.mohge_route_bwd(cfg.ref(), *([None] * 19)) == -2
    assert lib.mohge_expert_ffn_train(cfg.ref(), *([None] * 9)) == -2
    # fp32 layers have no backward pass
    f32 = M.Config(T=64, d=128, n_groups=3, experts_per_group=4, d_ff=(64, 128, 256), k_groups=2, k_experts=2, dtype=M.F32)
    assert lib.mohge_combine_bwd(f32.ref(), None, None, None, None, None, None, None) == -1
    assert "MOHGE_BF16" in M.mohge_last_error()
    # shared routing only for the one-group, all-experts configuration
    assert lib.mohge_shared_routing(cfg.ref(), None, None, None, None, None, None, None) == -1
    assert "shared routing" in M.mohge_last_error()


def test_mxfp4_quantiser_against_the_oracle_decoder():
    """The package's offline MXFP4 weight preparation (torch, CPU here): decoding its output with the
    oracle gives the nearest representable value of every element, values that are representable
    come back exactly, and scale codes stay within 1..254."""
    import numpy as np
    import torch
    import oracle
    from paper_2604_23108_amd.weights import quantize_mxfp4
    rng = np.random.default_rng(11)
    w = (rng.standard_normal((3, 8, 96)) * np.exp(rng.uniform(-6, 6, size=(3, 8, 1)))).astype(np.float32)
    w[0, 0, :32] = 0.0                                     # an all-zero block
    w[0, 1, :8] = [0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0, -6.0]   # block maximum 6: scale 1, exact
    w[0, 1, 8:32] = 0.25                                   # ties: 0.25 -> 0 (even code)
    packed, scales = quantize_mxfp4(torch.from_numpy(w))
    assert packed.shape == (3, 8, 48) and scales.shape == (3, 8, 3)
    s = scales.numpy()
    assert s.min() >= 1 and s.max() <= 254
    deq = oracle.dequantize_mxfp4(packed.numpy(), s)
    assert np.array_equal(deq[0, 0, :32], np.zeros(32))
    assert np.array_equal(deq[0, 1, :8], w[0, 1, :8].astype(np.float64))
    assert np.array_equal(deq[0, 1, 8:32], np.zeros(24))
    # nearest representable: error at most half the gap to the neighbouring values at that scale
    sc = np.repeat(oracle.decode_e8m0(s), 32, axis=-1)
    v = np.abs(w.astype(np.float64)) / sc
    assert v.max() < 8.0
    grid = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6.0])
    nearest = grid[np.abs(v[..., None] - grid).argmin(-1)]         # values above 6 clamp to 6
    assert (np.abs(np.abs(deq) / sc - v) <= np.abs(nearest - v)).all()
    assert (np.sign(deq) * np.sign(w) >= 0).all()
    # quantising the decoded values again changes nothing
    p2, s2 = quantize_mxfp4(torch.from_numpy(deq.astype(np.float32)))
    assert np.array_equal(oracle.dequantize_mxfp4(p2.numpy(), s2.numpy()), deq)


def test_quantised_and_split_entry_points_check_their_arguments():
    """Argument checks of the decode-only quantised-weight calls and of the two-step form of
    mohge_expert_ffn return before anything touches a GPU."""
    lib = M.lib()
    prefill = M.Config(T=4096, d=2048, n_groups=3, experts_per_group=8, d_ff=(512, 1024, 1536), k_groups=2, k_experts=4)
    decode = M.Config(T=32, d=4096, n_groups=4, experts_per_group=16, d_ff=(768, 1024, 1536, 2048), k_groups=2, k_experts=4)
    f32 = M.Config(T=16, d=128, n_groups=3, experts_per_group=4, d_ff=(64, 128, 256), k_groups=2, k_experts=2, dtype=M.F32)
    for fn in (lib.mohge_expert_ffn_w8, lib.mohge_expert_ffn_w4):
        assert fn(prefill.ref(), *([None] * 9), 0, None) == -1          # prefill sizes: refused
        assert "decode" in M.mohge_last_error()
        assert fn(f32.ref(), *([None] * 9), 0, None) == -1              # fp32 activations: refused
        assert "MOHGE_BF16" in M.mohge_last_error()
        assert fn(decode.ref(), *([None] * 9), 0, None) == -2           # NULL arguments
        assert "NULL" in M.mohge_last_error()
    assert lib.mohge_fp8_decode(None, None, 0, None) == 0                # nothing to do
    assert lib.mohge_fp8_decode(None, None, 8, None) == -2
    assert lib.mohge_mxfp4_decode(None, None, None, 0, None) == 0
    assert lib.mohge_mxfp4_decode(None, None, None, 48, None) == -1      # not whole blocks of 32
    assert "multiple" in M.mohge_last_error()
    assert lib.mohge_mxfp4_decode(None, None, None, 64, None) == -2
    # the two-step form (benchmark library) exists on the fused matrix-core path only
    import ctypes as C
    from paper_2604_23108_amd import bench_binding as BB
    bl = BB.lib()
    assert bl.mohge_bench_expert_ffn(decode.ref(), *([None] * 7), 0, None, C.c_int(1), None) == -1
    assert "separate launches" in M.mohge_last_error()
    assert bl.mohge_bench_expert_ffn(prefill.ref(), *([None] * 7), 0, None, C.c_int(5), None) == -1
    assert "parts" in M.mohge_last_error()
    assert bl.mohge_bench_expert_ffn(prefill.ref(), *([None] * 7), 0, None, C.c_int(2), None) == -2
    assert bl.mohge_bench_expert_ffn(prefill.ref(), *([None] * 7), 0, None, C.c_int(3), None) == -2
    two = BB.FfnOptions(fused=0)
    assert bl.mohge_bench_expert_ffn(prefill.ref(), *([None] * 7), 0, two.ref(), C.c_int(1), None) == -1
    bad = BB.FfnOptions(tile_rows_up=100)
    assert bl.mohge_bench_expert_ffn(prefill.ref(), *([None] * 7), 0, bad.ref(), C.c_int(3), None) == -1
    assert "tile rows" in M.mohge_last_error()
    # the down projection checks the size of the hidden-activation buffer it is handed
    assert lib.mohge_expert_ffn_down(prefill.ref(), C.c_void_p(256), C.c_size_t(1024), C.c_void_p(256),
                                     (C.c_void_p * 3)(256, 256, 256), C.c_void_p(256), None) == -4


def test_shared_routing_accepts_the_largest_expert_count():
    """N_s = 256 (the block size of the kernel that fills offsets) is a valid configuration."""
    cfg = M.Config(T=0, d=64, n_groups=1, experts_per_group=256, d_ff=(64,), k_groups=1, k_experts=256)
    import ctypes as C
    p = C.c_void_p(256)
    assert M.lib().mohge_shared_routing(cfg.ref(), p, p, p, p, p, p, None) == 0     # T = 0: nothing enqueued


def test_bench_refuses_more_than_one_gpu_and_graft_entry_has_both_functions():
    """bench.py --gpus N > 1 exits with a message (one GPU only, by design); the entry file has
    build() and smoke()."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "one GPU" in (p.stderr + p.stdout)
    src = open(os.path.join(root, "__graft_entry__.py")).read()
    assert "def build(" in src and "def smoke(" in src


def test_decode_layer_entry_point_checks_its_arguments():
    """mohge_decode_layer: sizes and refusals that need no GPU."""
    dec = M.Config(T=32, d=4096, n_groups=4, experts_per_group=16, d_ff=(768, 1024, 1536, 2048), k_groups=2, k_experts=4)
    P = 32 * 4
    ws = M.mohge_workspace_size(dec, M.CALL_DECODE_LAYER)
    ctl = M.mohge_decode_layer_ctl_bytes(dec)
    # hidden activations, y_perm, the fp64 partial logits, the index arrays; counters first
    assert P * 2048 * 2 + P * 4096 * 2 <= ws <= P * 2048 * 2 + P * 4096 * 2 + (1 << 20)
    assert 0 < ctl <= 64 * 1024 and ctl % 256 == 0 and ctl < ws
    lib = M.lib()
    assert lib.mohge_decode_layer(dec.ref(), *([None] * 13)) == -2
    assert "NULL" in M.mohge_last_error()
    # more than 32 tokens, fp32 layers, too many pairs: no workspace size, and the call refuses
    for bad in (M.Config(T=33, d=4096, n_groups=4, experts_per_group=16, d_ff=(768, 1024, 1536, 2048), k_groups=2, k_experts=4),
                M.Config(T=16, d=128, n_groups=3, experts_per_group=4, d_ff=(64, 128, 256), k_groups=2, k_experts=2, dtype=M.F32),
                M.Config(T=32, d=128, n_groups=16, experts_per_group=16, d_ff=(64,) * 16, k_groups=16, k_experts=128,
                         select_mode=M.SELECT_GLOBAL)):
        assert M.mohge_workspace_size(bad, M.CALL_DECODE_LAYER) == 0
        assert M.mohge_decode_layer_ctl_bytes(bad) == 0
        assert lib.mohge_decode_layer(bad.ref(), *([None] * 13)) == -1
        assert "mohge_decode_layer serves" in M.mohge_last_error()
    # an empty call is sized like a call of one token (nothing is launched)
    empty = M.Config(T=0, d=4096, n_groups=4, experts_per_group=16, d_ff=(768, 1024, 1536, 2048), k_groups=2, k_experts=4)
    assert M.mohge_workspace_size(empty, M.CALL_DECODE_LAYER) > 0
