"""GPU parity of the tap-major gather: activations [N][C][H][W] with C a multiple of 32, reduction
ordered (r, s, c), one filter tap per K-step, the masked lane offset formed once per step.  A
pointwise layer is its single-tap case.  Same bar as everywhere: 1e-4 * sum|x*w| per output
against the CPU oracle, element by element."""
import numpy as np
import pytest

from paper_2008_04567_amd import binding as B
from paper_2008_04567_amd import workloads as W
from tests import parity as PT

pytestmark = pytest.mark.gpu

# M = 2*19*23 = 874 pixels (ragged against 64, 128, 256), K = 72 (ragged against 32, 64, 128),
# C = 32: every K-step divides it; reduction 288 = 9 taps of 32 channels
RAGGED32 = W.layer("ragged32", 2, 32, (19, 23), 72, 3, 1, 1, x_dist="u11", w_dist="u11", seed=177)


def test_every_tile_variant_tap_major():
    desc = B.make_desc(RAGGED32)
    x, w = W.make_inputs(RAGGED32)
    y_ref, d_ref = PT.oracle_full(RAGGED32, x, w)
    cfgs = B.legal_configs(desc, split_k=[1], xcd_remap=1, persist=[0])
    assert len(cfgs) >= 120
    for c in cfgs:
        print(c, flush=True)
        PT.assert_close(PT.run_gpu(RAGGED32, x, w, cfg=c), y_ref, d_ref, repr(c))


def test_tap_major_split_and_persistent_schedules():
    """Slices that start in the middle of a tap's channel range, slice counts that do not divide the
    step count, persistent schedules (XCD-contiguous rounds and runs), both ways of summing."""
    l = W.layer("tm_sched", 3, 64, (21, 18), 96, 3, 1, 1, x_dist="u11", w_dist="u11", seed=178)
    desc = B.make_desc(l)
    x, w = W.make_inputs(l)
    y_ref, d_ref = PT.oracle_full(l, x, w)
    cfgs = []
    for (bm, bn, bk, wm, wn) in [(64, 64, 16, 2, 2), (128, 64, 32, 4, 2), (64, 32, 8, 2, 1)]:
        for split in (2, 3, 5, 7, 11, 16):
            cfgs.append(B.make_config(bm, bn, bk, wm, wn, split, split % 2, stages=1 + split % 3,
                                      reduce=(split // 2) % 2))
        for persist in (1, 2, 3, 4):
            for reduce in (0, 1):
                cfgs.append(B.ConvConfig(bm, bn, bk, wm, wn, 1, 1, persist, 1 + persist % 3, reduce))
    ran = 0
    for c in cfgs:
        if not B.config_legal(desc, c):
            continue
        print(c, flush=True)
        for again in range(2):
            PT.assert_close(PT.run_gpu(l, x, w, cfg=c), y_ref, d_ref, repr(c) + " launch %d" % again)
        ran += 1
    assert ran >= 30


SWEEP32 = [
    # name, n, c, hw, k, rs, stride, pad, dil
    ("tm_s2", 2, 32, (17, 15), 40, 3, 2, 1, 1),
    ("tm_s3_pad0", 1, 64, (20, 22), 33, 3, 3, 0, 1),
    ("tm_dil2", 2, 32, (16, 18), 10, 3, 1, 2, 2),
    ("tm_dil_mixed", 1, 96, (15, 21), 6, (3, 2), (1, 2), (2, 1), (2, 3)),
    ("tm_rect_filter", 1, 32, (12, 30), 17, (5, 3), 1, (2, 1), 1),
    ("tm_seven", 2, 32, (30, 30), 16, 7, 2, 3, 1),
    ("tm_1x1", 3, 64, (9, 11), 70, 1, 1, 0, 1),
    ("tm_1x1_s2", 2, 160, (13, 13), 20, 1, 2, 0, 1),
    ("tm_1x1_pad1", 1, 32, (7, 9), 12, 1, 1, 1, 1),        # a ring of outputs with no in-image tap
    ("tm_pad_gt_half", 1, 32, (6, 6), 4, 3, 1, 3, 1),
    ("tm_full_window", 4, 32, (5, 6), 12, (5, 6), 1, 0, 1),
    ("tm_one_pixel", 1, 32, (1, 1), 1, 1, 1, 0, 1),
    ("tm_wide_k", 1, 32, (6, 6), 300, 3, 1, 1, 1),
    ("tm_long_reduction", 1, 544, (5, 5), 8, 3, 1, 1, 1),
    ("tm_big_filter", 1, 32, (20, 19), 8, (16, 15), 1, (8, 7), 1),   # the largest filter the tiled family takes
]


@pytest.mark.parametrize("row", SWEEP32, ids=[r[0] for r in SWEEP32])
def test_tap_major_shape_sweep(row):
    name, n, c, hw, k, rs, st, pd, dl = row
    l = W.layer(name, n, c, hw, k, rs, st, pd, dl, x_dist="u11", w_dist="u11", seed=200 + hash(name) % 500)
    desc = B.make_desc(l)
    x, w = W.make_inputs(l)
    y_ref, d_ref = PT.oracle_full(l, x, w)
    print(name, "default", B.config_default(desc), flush=True)
    PT.assert_close(PT.run_gpu(l, x, w), y_ref, d_ref, name + " default")
    for c_ in [B.make_config(64, 32, 8, 2, 1), B.make_config(128, 128, 16, 2, 2),
               B.make_config(256, 64, 32, 4, 1, stages=3), B.make_config(128, 64, 16, 4, 2, 2, 0, stages=1),
               B.make_config(64, 64, 32, 2, 2, 3, reduce=1),
               B.ConvConfig(64, 64, 32, 2, 2, 1, 1, 2, 3, 0)]:
        if B.config_legal(desc, c_):
            print(name, c_, flush=True)
            PT.assert_close(PT.run_gpu(l, x, w, cfg=c_), y_ref, d_ref, name + repr(c_))


def test_tap_major_fused_and_mixed_layout_output():
    """The epilogue is shared with the other gather forms: bias + residual + rectifier on a tap-major
    layer, stored [N][K][P][Q] and channels-last."""
    l = W.layer("tm_fused", 2, 64, (14, 13), 48, 3, 1, 1, x_dist="u11", seed=179)
    rng = np.random.default_rng(7)
    P, Q = B.conv_out_shape(B.make_desc(l))
    bias = rng.uniform(-1, 1, l["k"]).astype(np.float32)
    res = rng.uniform(-2, 2, (l["n"], l["k"], P, Q)).astype(np.float32)
    for layout in (B.NCHW, B.Y_NHWC):
        for cfg in (None, B.make_config(64, 64, 16, 2, 2, 3), B.ConvConfig(64, 32, 32, 2, 1, 1, 1, 2, 2, 0)):
            PT.check_layout(l, layout, cfg=cfg, bias=bias, residual=res, relu=True)
