"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs, element by element.  Tolerance: 1e-4 * sum|x*w| per output (tests/parity.py)."""
import ctypes

import numpy as np
import pytest

from oracle import conv as oc

from paper_2008_04567_amd import binding as B
from paper_2008_04567_amd import workloads as W
from tests import parity as PT

pytestmark = pytest.mark.gpu

# several tiles in both dimensions with ragged tails against every tile size:
# M = 2*19*23 = 874 pixels, K = 72 channels, reduction 20*9 = 180
RAGGED = W.layer("ragged", 2, 20, (19, 23), 72, 3, 1, 1, x_dist="u11", w_dist="u11", seed=77)


def test_extension_is_loaded_and_sees_the_gpu():
    name, cus = B.device_info()
    print("device", name, cus, flush=True)
    assert "gfx950" in name and cus >= 1


def test_reference_kernel_configs_1_and_2():
    for l in W.config1() + W.config2():
        print(l["name"], flush=True)
        PT.check_layer(l, mode="ref")


def test_default_path_configs_1_and_2():
    for l in W.config1() + W.config2():
        print(l["name"], flush=True)
        PT.check_layer(l)


def test_every_tile_variant_on_a_ragged_shape():
    desc = B.make_desc(RAGGED)
    x, w = W.make_inputs(RAGGED)
    y_ref, d_ref = PT.oracle_full(RAGGED, x, w)
    cfgs = B.legal_configs(desc, split_k=[1], xcd_remap=1, persist=[0])
    assert len(cfgs) >= 120          # every tile combination at every prefetch depth
    for c in cfgs:
        print(c, flush=True)
        y = PT.run_gpu(RAGGED, x, w, cfg=c)
        PT.assert_close(y, y_ref, d_ref, repr(c))


def test_persistent_schedule():
    """Persistent workgroups: whole rounds of tiles stored plainly, the tiles of the last partial
    round cut into equal runs of reduction steps and summed through the fix-up workspace -- on a
    shape with more tiles than workgroups (several rounds plus a remainder) and on one with fewer
    (everything split).  Each configuration runs twice: the second launch finds the arrival
    counters as the first left them."""
    many = W.layer("many_tiles", 6, 12, (60, 64), 40, 3, 1, 1, x_dist="u11", w_dist="u11", seed=78)
    for l in (RAGGED, many):
        desc = B.make_desc(l)
        x, w = W.make_inputs(l)
        y_ref, d_ref = PT.oracle_full(l, x, w)
        for (bm, bn, bk, wm, wn) in [(64, 32, 16, 2, 1), (128, 64, 32, 4, 2), (64, 64, 8, 2, 1)]:
            for persist in (1, 2, 3, 4):
                c = B.make_config(bm, bn, bk, wm, wn, persist=persist, stages=1 + persist % 3,
                                  reduce=persist % 2)     # both ways of summing shared tiles
                assert B.config_legal(desc, c)
                print(l["name"], c, flush=True)
                for again in range(2):
                    y = PT.run_gpu(l, x, w, cfg=c)
                    PT.assert_close(y, y_ref, d_ref, repr(c) + " launch %d" % again)


def test_persistent_runs_beside_and_before_whole_tiles():
    """More tiles than one round of persistent workgroups, with a remainder: the remainder's
    reduction steps are dealt out in runs.  Small tiles leave room on a compute unit, so the runs
    go to workgroups appended to the grid and proceed beside the whole tiles; four workgroups of
    four waves per compute unit leave no room (and the largest tile may not either), so there the
    first workgroups do a run before their tiles.  Both gather forms
    ([N][C][H][W] with C = 8: row by row; C = 32: one filter tap per step), both ways of summing."""
    for c_in, seed in ((8, 91), (32, 92)):
        l = W.layer("rounds_and_rest_c%d" % c_in, 19, c_in, (64, 64), 128, 3, 1, 1, x_dist="u11", w_dist="u11", seed=seed)
        desc = B.make_desc(l)
        x, w = W.make_inputs(l)
        y_ref, d_ref = PT.oracle_full(l, x, w)
        cfgs = [B.make_config(256, 128, 16, 4, 2, persist=1, stages=1),                 # 304 tiles on 256 workgroups
                B.make_config(256, 128, 16, 4, 2, persist=1, stages=1, reduce=1)]
        for persist in (1, 2, 3, 4):                                                    # 2432 tiles
            cfgs.append(B.make_config(64, 64, 16, 2, 2, persist=persist, xcd_remap=1, stages=2, reduce=persist % 2))
        cfgs.append(B.make_config(64, 32, 16, 2, 1, persist=3, xcd_remap=1))            # 4864 tiles on 768 + runners
        for c in cfgs:
            assert B.config_legal(desc, c), c
            print(l["name"], c, flush=True)
            for again in range(2):
                y = PT.run_gpu(l, x, w, cfg=c)
                PT.assert_close(y, y_ref, d_ref, repr(c) + " launch %d" % again)


def test_tiles_numbered_along_the_pixels_first():
    """Weights larger than the activations: the tiles are numbered along the pixels first (neighbours in
    the order share weights).  Plain, split and persistent schedules -- 288 tiles on 256 persistent
    workgroups, so a whole round plus a remainder that is a range of channels --, both ways of summing
    (with atomics the whole output is zeroed first), plain and with the fused epilogue."""
    l = W.layer("heavy_w", 2, 256, (24, 24), 512, 3, 1, 1, x_dist="u11", w_dist="u11", seed=93)
    desc = B.make_desc(l)
    x, w = W.make_inputs(l)
    assert w.size > x.size
    y_ref, d_ref = PT.oracle_full(l, x, w)
    bias, res = _fused_operands(l, 16)
    f_ref, fd_ref = oc.conv2d_fused(oc.shape_from_layer(l), x, w, bias=bias, residual=res, relu=True)
    cfgs = [B.make_config(64, 32, 16, 2, 1), B.make_config(64, 32, 16, 2, 1, 5, 1), B.make_config(64, 32, 16, 2, 1, 3, 0, reduce=1)]
    for persist in (1, 2):
        for reduce in (0, 1):
            cfgs.append(B.make_config(64, 32, 16, 2, 1, persist=persist, reduce=reduce))
    cfgs.append(B.make_config(128, 64, 32, 4, 2, persist=1))
    for c in cfgs:
        assert B.config_legal(desc, c), c
        print(l["name"], c, flush=True)
        for again in range(2):
            PT.assert_close(PT.run_gpu(l, x, w, cfg=c), y_ref, d_ref, repr(c) + " launch %d" % again)
        PT.assert_close(PT.run_gpu_fused(l, x, w, bias=bias, residual=res, relu=True, cfg=c), f_ref, fd_ref,
                        repr(c) + " fused")


def test_wave_split_members_every_variant_and_way_of_meeting():
    """The members whose waves cut the reduction between them (bm = 32): every built combination of
    channels per tile, waves and fetch depth, alone and with the reduction cut between workgroups as
    well (partial tiles through the workspace and through atomics, slices that do not divide the
    octets, more waves than octets), on ragged pixels with a channel count that is no multiple of 32,
    on a pointwise layer and on a strided one; every case twice, so the second launch finds the
    arrival counters as the first left them.  Then all four layout codes, plain and with bias,
    residual and rectifier fused."""
    la = W.layer("ws.ragged", 2, 32, (13, 11), 40, 3, 1, 1, x_dist="u11", seed=111)
    lb = W.layer("ws.pointwise", 3, 64, (9, 10), 96, 1, 1, 0, x_dist="u11", seed=112)
    lc = W.layer("ws.strided", 2, 32, (15, 14), 64, 3, 2, 1, x_dist="u11", seed=113)
    ld = W.layer("ws.dilated", 1, 32, (12, 12), 33, 3, 1, 2, dil=2, x_dist="u11", seed=114)
    le = W.layer("ws.49taps", 1, 32, (20, 17), 32, 7, 2, 3, x_dist="u11", seed=115)     # more taps than table padding
    seen = set()
    for l in (la, lb, lc, ld, le):
        desc = B.make_desc(l)
        x, w = W.make_inputs(l)
        y_ref, d_ref = PT.oracle_full(l, x, w)
        for bn in (32, 64):
            for wm, wn in ((1, 1), (2, 1), (4, 1), (4, 2)):
                for stages in (1, 2, 3):
                    for split, reduce in ((1, 0), (2, 0), (3, 1), (5, 0), (7, 1)):
                        c = B.ConvConfig(32, bn, 8, wm, wn, split, 1 if split in (2, 7) else 0, 0, stages, reduce)
                        if not B.config_legal(desc, c):
                            assert split > l["c"] * l["r"] * l["s"] // 8, c   # only: more slices than octets
                            continue
                        seen.add((bn, wm, wn, stages))
                        print(l["name"], c, flush=True)
                        for again in range(2 if split > 1 else 1):
                            y = PT.run_gpu(l, x, w, cfg=c)
                            PT.assert_close(y, y_ref, d_ref, "%s %r launch %d" % (l["name"], c, again))
    assert len(seen) == 24
    assert not B.config_legal(B.make_desc(RAGGED), B.ConvConfig(32, 32, 8, 4, 1, 1, 0, 0, 1, 0))   # C = 20
    assert not B.config_legal(B.make_desc(la), B.ConvConfig(32, 32, 8, 4, 1, 1, 1, 1, 1, 0))       # persistent
    assert not B.config_legal(B.make_desc(la), B.ConvConfig(32, 32, 16, 4, 1, 1, 0, 0, 1, 0))      # not in octets
    rng = np.random.default_rng(3)
    for l in (la, lb):
        P, Q = B.conv_out_shape(B.make_desc(l))
        bias = rng.uniform(-0.5, 0.5, l["k"]).astype(np.float32)
        res = rng.uniform(-1, 1, (l["n"], l["k"], P, Q)).astype(np.float32)
        for layout in (0, 1, 2, 3):
            for c in (B.ConvConfig(32, 32, 8, 4, 1, 1, 0, 0, 2, 0), B.ConvConfig(32, 64, 8, 2, 1, 3, 1, 0, 1, 0),
                      B.ConvConfig(32, 64, 8, 4, 2, 2, 0, 0, 3, 1)):
                print(l["name"], "layout", layout, c, flush=True)
                PT.check_layout(l, layout, cfg=c)
                PT.check_layout(l, layout, cfg=c, bias=bias, residual=res, relu=True)


def test_split_k_and_remap_settings():
    desc = B.make_desc(RAGGED)
    x, w = W.make_inputs(RAGGED)
    y_ref, d_ref = PT.oracle_full(RAGGED, x, w)
    for (bm, bn, bk, wm, wn) in [(128, 64, 16, 2, 2), (64, 64, 8, 2, 2), (256, 128, 32, 4, 2)]:
        for split in (2, 3, 5, 7, 8, 11, 16, 20, 24):
            for remap in (0, 1):
                c = B.make_config(bm, bn, bk, wm, wn, split, remap, stages=1 + split % 3,
                                  reduce=(split // 2) % 2)   # both ways of summing the slices
                if not B.config_legal(desc, c):
                    continue
                print(c, flush=True)
                y = PT.run_gpu(RAGGED, x, w, cfg=c)
                PT.assert_close(y, y_ref, d_ref, repr(c))


SWEEP = [
    # name, n, c, hw, k, rs, stride, pad, dil
    ("s2", 2, 5, (17, 15), 9, 3, 2, 1, 1),
    ("s3_pad0", 1, 7, (20, 22), 33, 3, 3, 0, 1),
    ("dil2", 2, 6, (16, 18), 10, 3, 1, 2, 2),
    ("dil_mixed", 1, 4, (15, 21), 6, (3, 2), (1, 2), (2, 1), (2, 3)),
    ("rect_filter", 1, 3, (12, 30), 17, (5, 3), 1, (2, 1), 1),
    ("seven", 2, 3, (30, 30), 16, 7, 2, 3, 1),
    ("one_by_one", 3, 37, (9, 11), 70, 1, 1, 0, 1),
    ("one_by_one_s2", 2, 40, (13, 13), 20, 1, 2, 0, 1),
    ("pad_gt_half", 1, 3, (6, 6), 4, 3, 1, 3, 1),          # outer ring of outputs has no in-image tap
    ("full_window", 4, 8, (5, 6), 12, (5, 6), 1, 0, 1),   # one output pixel per image
    ("single", 1, 1, (1, 1), 1, 1, 1, 0, 1),
    ("k1_c1", 1, 1, (40, 40), 1, 3, 1, 1, 1),
    ("wide_k", 1, 8, (6, 6), 300, 3, 1, 1, 1),
    ("long_reduction", 1, 520, (5, 5), 8, 3, 1, 1, 1),
    ("table1_like", 1, 3, (28, 24), 16, 3, 1, 0, 1),
]


@pytest.mark.parametrize("row", SWEEP, ids=[r[0] for r in SWEEP])
def test_shape_sweep_default_and_fixed_configs(row):
    name, n, c, hw, k, rs, st, pd, dl = row
    l = W.layer(name, n, c, hw, k, rs, st, pd, dl, x_dist="u11", w_dist="u11", seed=hash(name) % 1000)
    desc = B.make_desc(l)
    x, w = W.make_inputs(l)
    y_ref, d_ref = PT.oracle_full(l, x, w)
    print(name, "ref", flush=True)
    PT.assert_close(PT.run_gpu(l, x, w, mode="ref"), y_ref, d_ref, name + " ref")
    print(name, "default", B.config_default(desc), flush=True)
    PT.assert_close(PT.run_gpu(l, x, w), y_ref, d_ref, name + " default")
    for c_ in [B.make_config(64, 32, 8, 2, 1), B.make_config(128, 128, 16, 2, 2),
               B.make_config(256, 64, 32, 4, 1, stages=3), B.make_config(128, 64, 16, 4, 2, 2, 0, stages=1),
               B.make_config(64, 64, 32, 2, 2, persist=2, stages=3)]:
        if B.config_legal(desc, c_):
            print(name, c_, flush=True)
            PT.assert_close(PT.run_gpu(l, x, w, cfg=c_), y_ref, d_ref, name + repr(c_))


@pytest.mark.parametrize("layer", W.table1_convs() + W.unique_layers(W.resnet18_stack(1)),
                         ids=lambda l: l["name"])
def test_section3_workloads(layer):
    """The shapes the paper's Section 3 measures: Table 1's non-square, unpadded production
    layers and the distinct layers of ResNet-18 at batch 1 -- default configuration, then one
    split and one persistent member of the family where legal."""
    x, w = W.make_inputs(layer)
    y_ref, d_ref = PT.oracle_full(layer, x, w)
    desc = B.make_desc(layer)
    PT.assert_close(PT.run_gpu(layer, x, w), y_ref, d_ref, layer["name"] + " default")
    for c in [B.make_config(64, 64, 16, 2, 2, 4), B.make_config(128, 32, 32, 4, 1, persist=2)]:
        if B.config_legal(desc, c):
            print(layer["name"], c, flush=True)
            PT.assert_close(PT.run_gpu(layer, x, w, cfg=c), y_ref, d_ref, layer["name"] + repr(c))


def _fused_operands(l, seed):
    rng = np.random.default_rng(seed)
    P, Q = B.conv_out_shape(B.make_desc(l))
    bias = rng.uniform(-1, 1, l["k"]).astype(np.float32)
    res = rng.uniform(-2, 2, (l["n"], l["k"], P, Q)).astype(np.float32)
    return bias, res


def test_fused_epilogue_every_schedule():
    """Bias, residual and rectifier applied inside the launch: plain tiles, split reduction and
    persistent schedules (both meet through the workspace), in every combination of the three
    terms; then the default entry point and the direct kernel's two-launch form."""
    import itertools
    l = RAGGED
    desc = B.make_desc(l)
    x, w = W.make_inputs(l)
    bias, res = _fused_operands(l, 5)
    sh = oc.shape_from_layer(l)
    cfgs = [B.make_config(64, 32, 16, 2, 1), B.make_config(128, 64, 16, 2, 2, 5),
            B.make_config(64, 64, 8, 2, 1, persist=2), B.make_config(128, 128, 32, 2, 2, persist=1)]
    for use_b, use_r, relu in itertools.product((False, True), repeat=3):
        b_, r_ = (bias if use_b else None), (res if use_r else None)
        y_ref, d_ref = oc.conv2d_fused(sh, x, w, bias=b_, residual=r_, relu=relu)
        for c in cfgs + [None]:
            assert c is None or B.config_legal(desc, c)
            what = "bias %d residual %d relu %d %r" % (use_b, use_r, relu, c)
            print(what, flush=True)
            y = PT.run_gpu_fused(l, x, w, bias=b_, residual=r_, relu=relu, cfg=c)
            PT.assert_close(y, y_ref, d_ref, what)
    big = W.layer("big_filter", 1, 2, (20, 20), 3, (17, 2), 1, 2, 1, x_dist="u11", w_dist="u11", seed=5)
    x, w = W.make_inputs(big)
    bias, res = _fused_operands(big, 6)
    y_ref, d_ref = oc.conv2d_fused(oc.shape_from_layer(big), x, w, bias=bias, residual=res, relu=True)
    PT.assert_close(PT.run_gpu_fused(big, x, w, bias=bias, residual=res, relu=True), y_ref, d_ref,
                    "direct kernel + epilogue")


def test_without_workspace_shared_tiles_use_atomics():
    """With the workspace turned off, split and persistent launches zero y and accumulate with
    fp32 atomics, and a fused epilogue follows as a launch of its own."""
    l = RAGGED
    desc = B.make_desc(l)
    x, w = W.make_inputs(l)
    bias, res = _fused_operands(l, 15)
    sh = oc.shape_from_layer(l)
    y_ref, d_ref = PT.oracle_full(l, x, w)
    f_ref, fd_ref = oc.conv2d_fused(sh, x, w, bias=bias, residual=res, relu=True)
    B.set_workspace_limit(0)
    try:
        for c in [B.make_config(128, 64, 16, 2, 2, 5), B.make_config(64, 64, 8, 2, 1, 11, 0),
                  B.make_config(64, 64, 8, 2, 1, persist=2), B.make_config(64, 32, 16, 2, 1, persist=4)]:
            assert B.config_legal(desc, c)
            print(c, flush=True)
            PT.assert_close(PT.run_gpu(l, x, w, cfg=c), y_ref, d_ref, repr(c) + " atomics")
            PT.assert_close(PT.run_gpu_fused(l, x, w, bias=bias, residual=res, relu=True, cfg=c),
                            f_ref, fd_ref, repr(c) + " atomics, fused")
    finally:
        B.set_workspace_limit(1 << 30)


def test_fused_epilogue_rectifier_bites_and_full_size():
    """A config-3 layer at full size with all three terms, sampled against the oracle; the bias is
    chosen so that about half of the outputs are cut off by the rectifier."""
    l = W.config3()[2]
    desc = B.make_desc(l)
    x, w = W.make_inputs(l)
    bias, res = _fused_operands(l, 9)
    bias -= 1.0
    c = B.make_config(64, 64, 16, 2, 2, 5)
    y = PT.run_gpu_fused(l, x, w, bias=bias, residual=res, relu=True, cfg=c)
    frac = float((y == 0).mean())
    assert 0.1 < frac < 0.9, frac
    rng = np.random.default_rng(3)
    idx = np.unique(rng.integers(0, y.size, 4096))
    yc, dc = oc.conv2d_sampled(oc.shape_from_layer(l), x, w, idx)
    kk = (idx // (y.shape[2] * y.shape[3])) % l["k"]
    z = yc + bias.astype(np.float64)[kk] + res.reshape(-1).astype(np.float64)[idx]
    d = dc + np.abs(bias.astype(np.float64))[kk] + np.abs(res.reshape(-1).astype(np.float64))[idx]
    PT.assert_close(y.reshape(-1)[idx], np.maximum(z, 0.0), d, "config 3 layer fused")


# channels-last: C = 32 so that every K-step of the family divides it; same ragged pixel and channel
# tails as RAGGED
RAGGED_CL = W.layer("ragged_cl", 2, 32, (19, 23), 72, 3, 1, 1, x_dist="u11", w_dist="u11", seed=79)


def test_channels_last_every_tile_combination():
    desc = B.make_desc(RAGGED_CL, layout=B.NHWC)
    cfgs = B.legal_configs(desc, split_k=[1], xcd_remap=1, persist=[0])
    assert len(cfgs) >= 120
    for c in cfgs:
        print(c, flush=True)
        PT.check_layout(RAGGED_CL, B.NHWC, cfg=c)


def test_channels_last_layouts_schedules_and_epilogue():
    """All four layout codes (the mixed ones transform the layout in the same launch), through
    plain, split and persistent schedules with both ways of summing shared tiles, with and
    without the fused epilogue; then the default entry point."""
    l = RAGGED_CL
    P, Q = B.conv_out_shape(B.make_desc(l))
    rng = np.random.default_rng(21)
    bias = rng.uniform(-1, 1, l["k"]).astype(np.float32)
    res = rng.uniform(-2, 2, (l["n"], l["k"], P, Q)).astype(np.float32)
    cfgs = [B.make_config(64, 32, 16, 2, 1), B.make_config(128, 64, 16, 2, 2, 5),
            B.make_config(128, 64, 32, 4, 2, 3, reduce=1), B.make_config(64, 64, 8, 2, 1, persist=2),
            B.make_config(128, 128, 32, 2, 2, persist=1, reduce=1), None]
    for layout in (B.NHWC, B.X_NHWC, B.Y_NHWC):
        desc = B.make_desc(l, layout=layout)
        for c in cfgs:
            assert c is None or B.config_legal(desc, c), c
            print(layout, c, flush=True)
            PT.check_layout(l, layout, cfg=c)
            PT.check_layout(l, layout, cfg=c, bias=bias, residual=res, relu=True)


CL_SWEEP = [
    # name, n, c, hw, k, rs, stride, pad, dil
    ("cl_s2", 2, 16, (17, 15), 9, 3, 2, 1, 1),
    ("cl_1x1", 2, 40, (9, 11), 36, 1, 1, 0, 1),
    ("cl_1x1_s2", 2, 64, (14, 14), 48, 1, 2, 0, 1),
    ("cl_5x3_dil", 1, 8, (21, 19), 10, (5, 3), (1, 2), (4, 2), (2, 2)),
    ("cl_stem_like", 1, 8, (40, 40), 16, 7, 2, 3, 1),
    ("cl_c24", 1, 24, (12, 12), 20, 3, 1, 1, 1),
    ("cl_tiny", 1, 8, (5, 5), 3, 3, 1, 1, 1),
]


@pytest.mark.parametrize("case", CL_SWEEP, ids=lambda c: c[0])
def test_channels_last_shape_sweep(case):
    name, n, c, hw, k, rs, stride, pad, dil = case
    l = W.layer(name, n, c, hw, k, rs, stride, pad, dil, x_dist="u11", w_dist="u11", seed=31)
    desc = B.make_desc(l, layout=B.NHWC)
    PT.check_layout(l, B.NHWC)
    for c_ in [B.make_config(64, 32, 8, 2, 1), B.make_config(128, 128, 16, 2, 2),
               B.make_config(256, 64, 32, 4, 1, stages=3), B.make_config(128, 64, 8, 2, 2, 2, 0, stages=1),
               B.make_config(64, 64, 32, 2, 2, persist=2, stages=3)]:
        if B.config_legal(desc, c_):
            print(name, c_, flush=True)
            PT.check_layout(l, B.NHWC, cfg=c_)


def test_channels_last_output_not_16_byte_aligned():
    """A channels-last y that starts 4 bytes past a 16-byte boundary takes the scalar stores."""
    torch, dev = PT.torch_dev()
    l = RAGGED_CL
    desc = B.make_desc(l, layout=B.NHWC)
    x, w = W.make_inputs(l)
    x_cl = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
    y_ref, d_ref = oc.conv2d_layout(oc.shape_from_layer(l), x_cl, w, "NHWC", "NHWC")
    buf = torch.full((y_ref.size + 9,), 12345.0, device=dev, dtype=torch.float32)
    yd = buf[1:1 + y_ref.size]
    assert yd.data_ptr() % 16 == 4
    B.conv2d_fwd_fused(desc, PT.to_dev(x_cl), PT.to_dev(w), yd, relu=False,
                       cfg=B.make_config(128, 64, 16, 2, 2, 3))
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert host[0] == 12345.0 and np.all(host[1 + y_ref.size:] == 12345.0)
    PT.assert_close(host[1:1 + y_ref.size], y_ref, d_ref, "unaligned channels-last y")


def test_channels_last_any_channel_count():
    """C a multiple of 32 is gathered in 16-byte channel quads; any other C (here an RGB stem and
    C = 20) row by row through the same kernels; K not a multiple of 4 or an unaligned y takes
    the scalar stores."""
    rgb = W.layer("cl_rgb", 1, 3, (30, 28), 16, 7, 2, 3, 1, x_dist="u11", w_dist="u11", seed=33)
    c20 = W.layer("cl_c20", 2, 20, (13, 11), 18, 3, 1, 1, 1, x_dist="u11", w_dist="u11", seed=34)
    for l in (rgb, c20):
        for layout in (B.NHWC, B.X_NHWC, B.Y_NHWC):
            desc = B.make_desc(l, layout=layout)
            assert B.legal_configs(desc) != []
            PT.check_layout(l, layout)
            for c in (B.make_config(64, 32, 32, 2, 1), B.make_config(128, 64, 16, 2, 2, 3),
                      B.make_config(64, 64, 8, 2, 1, persist=2)):
                if B.config_legal(desc, c):
                    PT.check_layout(l, layout, cfg=c)


def test_oversized_filter_uses_the_direct_kernel():
    # the tiled family tracks at most 16 filter rows and 15 filter columns per pixel
    for rs in [(17, 2), (2, 16)]:
        l = W.layer("big_filter", 1, 2, (20, 20), 3, rs, 1, 2, 1, x_dist="u11", w_dist="u11", seed=5)
        assert B.legal_configs(B.make_desc(l)) == []
        PT.check_layer(l)
    l = W.layer("filter_16x15", 1, 2, (20, 19), 3, (16, 15), 1, 3, 1, x_dist="u11", w_dist="u11", seed=6)
    assert B.legal_configs(B.make_desc(l)) != []
    PT.check_layer(l)


def test_illegal_config_is_refused_before_launch():
    torch, dev = PT.torch_dev()
    desc = B.make_desc(RAGGED)
    t = torch.zeros(16, device=dev)
    rc = B.lib().wpk_conv2d_fwd_config(ctypes.byref(desc), ctypes.byref(B.make_config(128, 64, 16, 1, 1)),
                                       ctypes.c_void_p(t.data_ptr()), ctypes.c_void_p(t.data_ptr()),
                                       ctypes.c_void_p(t.data_ptr()), None)
    assert rc == B.E_NO_CONFIG


@pytest.mark.parametrize("layer", W.config3() + W.config4(), ids=lambda l: l["name"])
def test_full_size_configs_3_and_4(layer):
    """The full sizes of the batched 3x3 workload (N=16), whole output tensor against the oracle."""
    print(layer["name"], B.config_default(B.make_desc(layer)), flush=True)
    PT.check_layer(layer)


def test_non_default_stream():
    torch, dev = PT.torch_dev()
    l = W.config2()[0]
    desc = B.make_desc(l)
    x, w = W.make_inputs(l)
    y_ref, d_ref = PT.oracle_full(l, x, w)
    xd, wd = PT.to_dev(x), PT.to_dev(w)
    yd = torch.empty(y_ref.shape, device=dev, dtype=torch.float32)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        B.conv2d_fwd(desc, xd, wd, yd, stream=s)
    s.synchronize()
    PT.assert_close(yd.cpu().numpy(), y_ref, d_ref, "side stream")
