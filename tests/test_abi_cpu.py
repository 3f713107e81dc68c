"""The C-ABI library loads, exports what include/blstm_mi355.h declares, and its host-side
logic (validation, layouts, the ring schedule) behaves; no kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import blstm_oracle as orc
from paper_1904_04956_amd import binding as bl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "blstm_mi355.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", " ".join(l for l in text.splitlines() if not l.startswith("#")))))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"blstm_forward", "blstm_backward", "softmax_xent_fwd_bwd", "sgd_step", "adpsgd_mix"} <= set(names)
    L = bl.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(bl.EXPORTS) == names


def test_param_count_and_offsets_match_the_closed_form():
    # the paper's own model: 43 130 368 parameters (165 MB in float)
    ctx = bl.blstm_create(21, 256, 260, 512, 6, 256, 32000, 1)
    try:
        assert bl.blstm_param_count(ctx) == 43_130_368
        assert bl.blstm_workspace_bytes(ctx) > 0
    finally:
        bl.blstm_destroy(ctx)
    for shape in (dict(T=3, B=2, D=5, H=4, L=2, P=3, V=7), dict(T=21, B=8, D=40, H=32, L=1, P=0, V=100),
                  dict(T=21, B=256, D=260, H=512, L=4, P=256, V=32000)):
        ctx = bl.blstm_create(mode=0, **shape)
        try:
            dm = orc.Dims(**shape)
            assert bl.blstm_param_count(ctx) == orc.param_count(dm)
            lay = {n: (o, int(np.prod(s))) for n, o, s in orc.layout(dm)}
            for l in range(dm.L):
                for d in range(2):
                    assert bl.blstm_param_offset(ctx, l, d, bl.BLSTM_WX) == lay[f"Wx{l}.{d}"]
                    assert bl.blstm_param_offset(ctx, l, d, bl.BLSTM_UH) == lay[f"Uh{l}.{d}"]
                    assert bl.blstm_param_offset(ctx, l, d, bl.BLSTM_B) == lay[f"b{l}.{d}"]
            if dm.P > 0:
                assert bl.blstm_param_offset(ctx, 0, 0, bl.BLSTM_WP) == lay["Wp"]
                assert bl.blstm_param_offset(ctx, 0, 0, bl.BLSTM_BP) == lay["bp"]
            else:
                assert bl.blstm_param_offset(ctx, 0, 0, bl.BLSTM_WP)[1] == 0
            assert bl.blstm_param_offset(ctx, 0, 0, bl.BLSTM_WS) == lay["Ws"]
            assert bl.blstm_param_offset(ctx, 0, 0, bl.BLSTM_BS) == lay["bs"]
        finally:
            bl.blstm_destroy(ctx)


def test_create_rejects_bad_dimensions():
    for bad in (dict(T=0), dict(B=0), dict(H=-1), dict(V=0), dict(P=-1), dict(mode=2), dict(L=0)):
        kw = dict(T=2, B=2, D=2, H=2, L=1, P=0, V=2, mode=0)
        kw.update(bad)
        with pytest.raises(bl.BlstmError) as e:
            bl.blstm_create(**kw)
        assert e.value.code == -2
    L = bl.lib()
    assert L.blstm_create(None, None) == -1
    assert L.blstm_param_count(None) == 0
    L.blstm_destroy(None)


def test_options_take_their_values_only():
    ctx = bl.blstm_create(2, 2, 2, 2, 1, 0, 2, 0)
    L = bl.lib()
    try:
        for opt in (bl.BLSTM_OPT_RECURRENT_PATH, bl.BLSTM_OPT_RECURRENT_SYNC, bl.BLSTM_OPT_KEEP_WEIGHT_COPIES,
                    bl.BLSTM_OPT_TEST_ABORT, bl.BLSTM_OPT_DEFER_SOFTMAX_WGRAD):
            assert L.blstm_set_option(ctx, opt, 1) == 0
            assert L.blstm_set_option(ctx, opt, 0) == 0
            assert L.blstm_set_option(ctx, opt, 2) == -2
        assert L.blstm_set_option(ctx, 99, 0) == -2
        assert L.blstm_set_option(None, bl.BLSTM_OPT_DEFER_SOFTMAX_WGRAD, 1) == -1
    finally:
        bl.blstm_destroy(ctx)


def test_calls_validate_before_launching():
    ctx = bl.blstm_create(2, 2, 2, 2, 1, 0, 2, 0)
    L = bl.lib()
    try:
        assert L.blstm_forward(ctx, None, None, None, None) == -1
        # valid-looking (never dereferenced) addresses, but no workspace bound
        assert L.blstm_forward(ctx, 4096, 4096, 4096, None) == -3
        assert "workspace" in bl.blstm_last_error()
        assert L.blstm_backward(ctx, 4096, 4096, 4096, 4096, None) == -3
        assert L.softmax_xent_fwd_bwd(ctx, 4096, 4096, 4096, 4096, 4096, 4096, None) == -3
        assert L.blstm_bind(ctx, 4096, 1) == -3
        assert L.blstm_bind(ctx, 4100, 1 << 30) == -4
        assert L.blstm_bind(ctx, 4096, 1 << 30) == 0
        assert L.blstm_forward(ctx, 4100, 4096, 4096, None) == -4
        assert L.blstm_backward(ctx, 4096, 4096, 4096, 4096, None) == -3      # no forward pass held
        assert L.sgd_step(None, None, None, 0, 0.1, 0.0, None, None) == -1
        assert L.sgd_step(4096, None, 4096, 8, 0.1, 0.9, None, None) == -1    # momentum without velocity
        assert L.sgd_step(4100, None, 4096, 8, 0.1, 0.0, None, None) == -4
        assert L.blstm_shadow_refresh(None, None, 0, None) == -1
        with pytest.raises(bl.BlstmError):
            bl.blstm_param_offset(ctx, 5, 0, bl.BLSTM_WX)
        with pytest.raises(bl.BlstmError):
            bl.blstm_param_offset(ctx, 0, 0, 99)
    finally:
        bl.blstm_destroy(ctx)


def test_noalloc_entry_validates_and_rejects_oversized_shapes():
    L = bl.lib()
    small = bl.blstm_create(2, 2, 2, 2, 1, 0, 2, 0)
    big = bl.blstm_create(21, 256, 260, 512, 4, 256, 32000, 1)          # 344 MB of logits: beyond the resident array
    try:
        assert L.softmax_xent_fwd_bwd_noalloc(small, None, None, None, None, None, None, None) == -1
        assert L.softmax_xent_fwd_bwd_noalloc(small, 4100, 4096, 4096, 4096, 4096, 4096, None) == -4
        assert L.softmax_xent_fwd_bwd_noalloc(big, 4096, 4096, 4096, 4096, 4096, 4096, None) == -3
        assert "scratch" in bl.blstm_last_error()
    finally:
        bl.blstm_destroy(small); bl.blstm_destroy(big)


def test_mix_validation():
    L = bl.lib()
    ptrs = (ctypes.c_void_p * 4)(4096, 8192, 12288, 16384)
    ok = (ctypes.c_int32 * 4)(1, 0, 3, 2)
    bad = (ctypes.c_int32 * 4)(1, 2, 3, 0)
    assert L.adpsgd_mix(None, None, 16, 4, ok, None) == -1
    assert L.adpsgd_mix(ptrs, None, 16, 0, ok, None) == -2
    assert L.adpsgd_mix(ptrs, None, 16, 65, ok, None) == -2
    assert L.adpsgd_mix(ptrs, None, 16, 4, bad, None) == -2
    assert "involution" in bl.blstm_last_error()
    same = (ctypes.c_void_p * 4)(4096, 8192, 4096, 16384)
    assert L.adpsgd_mix(same, None, 16, 4, ok, None) == -2
    odd = (ctypes.c_void_p * 4)(4096, 8196, 12288, 16384)
    assert L.adpsgd_mix(odd, None, 16, 4, ok, None) == -4
    # nothing to do: n == 0 launches nothing and succeeds
    assert L.adpsgd_mix(ptrs, None, 0, 4, ok, None) == 0


def test_ring_partner_matches_the_oracle_schedule():
    for R in (2, 4, 16, 64):
        for step in range(5):
            assert bl.adpsgd_ring_partner(R, step) == orc.adpsgd_ring_partner(R, step)
    for R, step in ((0, 0), (5, 0), (4, -1)):
        with pytest.raises(bl.BlstmError):
            bl.adpsgd_ring_partner(R, step)


def test_profile_names():
    L = bl.lib()
    k = L.blstm_profile_classes()
    names = [L.blstm_profile_name(i).decode() for i in range(k)]
    assert len(set(names)) == k and all(names)
    assert L.blstm_profile_name(k) == b""


def test_lr_schedule_matches_the_oracle():
    # section 3.1's recipe, evaluated by the library on the host, against the oracle's closed form
    for base, peak in ((0.1, 1.0), (0.1, 0.1), (0.05, 0.8)):
        for epoch in range(1, 21):
            assert bl.blstm_lr_schedule(epoch, base, peak) == pytest.approx(orc.lr_schedule(epoch, base, peak), rel=1e-12)
    assert bl.blstm_lr_schedule(3, 0.1, 1.0, warmup_epochs=1, anneal_from=2) == pytest.approx(orc.lr_schedule(3, 0.1, 1.0, 1, 2), rel=1e-12)


def test_pair_and_average_validation():
    # rejected on the host before anything is launched (no GPU needed)
    L = bl.lib()
    a, b, ga, gb = 4096, 8192, 12288, 16384
    assert L.sgd_mix_pair(None, b, None, None, ga, gb, 16, 0.1, 0.0, None, None, None) == -1
    assert L.sgd_mix_pair(a, b, None, None, ga, gb, 16, 0.1, 0.9, None, None, None) == -1       # momentum without velocities
    assert L.sgd_mix_pair(a, b, 20480, None, ga, gb, 16, 0.1, 0.0, None, None, None) == -1       # one bf16 copy only
    assert L.sgd_mix_pair(a, a, None, None, ga, gb, 16, 0.1, 0.0, None, None, None) == -2
    assert L.sgd_mix_pair(a, b + 4, None, None, ga, gb, 16, 0.1, 0.0, None, None, None) == -4
    assert L.sgd_mix_pair(a, b, None, None, ga, gb, 0, 0.1, 0.0, None, None, None) == 0         # n == 0: nothing to do
    assert L.sgd_mix_pair(a, b, None, None, ga, None, 0, 0.1, 0.0, None, None, None) == 0       # no gradient for replica j: allowed
    assert L.sgd_mix_pair(a, b, None, None, ga, None, 0, 0.1, 0.9, 24576, None, None) == 0      # ... and then no velocity for it either
    assert L.sgd_mix_pair(a, b, None, None, None, gb, 16, 0.1, 0.0, None, None, None) == -1     # replica i always has one
    ptrs = (ctypes.c_void_p * 4)(4096, 8192, 12288, 16384)
    assert L.sync_average(None, None, 16, 4, None) == -1
    assert L.sync_average(ptrs, None, 16, 0, None) == -2
    assert L.sync_average(ptrs, None, 16, 65, None) == -2
    same = (ctypes.c_void_p * 4)(4096, 8192, 4096, 16384)
    assert L.sync_average(same, None, 16, 4, None) == -2
    odd = (ctypes.c_void_p * 4)(4096, 8196, 12288, 16384)
    assert L.sync_average(odd, None, 16, 4, None) == -4
    assert L.sync_average(ptrs, None, 0, 4, None) == 0


def test_bench_flop_counts_match_the_closed_forms():
    # forward + backward FLOP per frame = 2 (3 MACs - layer 1's input-gradient product): 180.8 M for the 4x512 model,
    # 256.3 M for the paper's 6x512 model, 866.1 M for 6x1024; the per-class split adds up to the same total
    import bench
    assert round(bench.flop_per_frame(260, 512, 4, 256, 32000) / 1e6, 1) == 180.8
    assert round(bench.flop_per_frame(260, 512, 6, 256, 32000) / 1e6, 1) == 256.3
    assert round(bench.flop_per_frame(260, 1024, 6, 256, 32000) / 1e6, 1) == 866.1
    T, B = 21, 256
    f = bench.flops_by_class(T, B, 260, 512, 4, 256, 32000)
    total = sum(f[k] for k in ("gemm_input_projection", "gemm_bottleneck", "gemm_logits", "gemm_softmax_bwd", "gemm_wgrad", "gemm_dgrad"))
    # the recurrent products count T - 1 frames per sequence (the first visited frame has no previous h), forward,
    # backward and in the weight gradient (which is in gemm_wgrad with T - 1 already)
    total += f["recurrent_fwd_persistent"] + f["recurrent_bwd_persistent"]
    per_frame = bench.flop_per_frame(260, 512, 4, 256, 32000)
    missing = 2 * 3 * (2 * 4 * 512 * 512) * 4 * B          # the frame the recurrent products skip, all three passes, four layers
    assert total == per_frame * T * B - missing
    # with the softmax layer's weight gradient in the backward pass's grouped launch one product changes class
    fd = bench.flops_by_class(T, B, 260, 512, 4, 256, 32000, softmax_wgrad_deferred=True)
    moved = 2 * T * B * 32000 * 256
    assert fd["gemm_softmax_bwd"] == f["gemm_softmax_bwd"] - moved and fd["gemm_wgrad"] == f["gemm_wgrad"] + moved
    assert all(fd[k] == f[k] for k in f if k not in ("gemm_softmax_bwd", "gemm_wgrad"))


def test_bench_traffic_file_is_keyed_to_the_kernel_sources(tmp_path, monkeypatch):
    import bench
    prof = tmp_path / "profiles"
    prof.mkdir()
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    assert bench.measured_traffic("paper4x512", 256) == {}                       # no file
    (tmp_path / "paper_1904_04956_amd" / "csrc").mkdir(parents=True)
    (tmp_path / "paper_1904_04956_amd" / "csrc" / "k.hip").write_text("kernel v1")
    h = bench.source_hash()
    (prof / "hbm_traffic_paper4x512.txt").write_text(f"# prose\nsources {h}\nbatch 256\nbytes_per_launch gemm_wgrad 123.0  # note\n")
    assert bench.measured_traffic("paper4x512", 256) == {"gemm_wgrad": 123.0}
    assert bench.measured_traffic("paper4x512", 128) == {}                       # another batch size
    (tmp_path / "paper_1904_04956_amd" / "csrc" / "k.hip").write_text("kernel v2")
    assert bench.measured_traffic("paper4x512", 256) == {}                       # the sources have changed since
