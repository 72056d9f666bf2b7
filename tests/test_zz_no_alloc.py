"""GPU test of the entry point that allocates nothing (wpk_conv2d_fwd_noalloc): its output against
wpk_conv2d_fwd_config's on the same inputs, two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

from oracle import conv as oc
from paper_2008_04567_amd import binding as B
from paper_2008_04567_amd import workloads as W
from tests import parity as PT

pytestmark = pytest.mark.gpu


def _both(layer, cfg):
    """(output of the entry point that does not allocate, output of the existing one, oracle y, D)."""
    torch, dev = PT.torch_dev()
    desc = B.make_desc(layer)
    P, Q = B.conv_out_shape(desc)
    x, w = W.make_inputs(layer)
    xd, wd = PT.to_dev(x), PT.to_dev(w)
    n_out = layer["n"] * layer["k"] * P * Q
    guard = 256
    outs = []
    for fn in (B.conv2d_fwd_noalloc, None):
        buf = torch.full((n_out + 2 * guard,), 12345.0, device=dev, dtype=torch.float32)
        yd = buf[guard:guard + n_out]
        if fn is not None:
            fn(desc, xd, wd, yd, cfg=cfg)
        elif cfg is not None:
            B.conv2d_fwd_config(desc, cfg, xd, wd, yd)
        else:
            B.conv2d_fwd(desc, xd, wd, yd)
        torch.cuda.synchronize()
        host = buf.cpu().numpy()
        assert np.all(host[:guard] == 12345.0) and np.all(host[guard + n_out:] == 12345.0), \
            "write outside the output tensor"
        outs.append(host[guard:guard + n_out].reshape(layer["n"], layer["k"], P, Q).astype(np.float64))
    y_ref, d_ref, _ = oc.conv2d(oc.shape_from_layer(layer), x, w)
    return outs[0], outs[1], y_ref, d_ref


def test_no_alloc_entry_point_matches_the_allocating_one():
    # first call: a reduction split three ways, the partial tiles meeting in the static workspace
    big = W.layer("na.big", 2, 40, (23, 19), 72, 3, 1, 1, x_dist="u11", seed=401)
    cfg = B.make_config(64, 64, 16, 2, 2, split_k=3)
    assert B.config_legal(B.make_desc(big), cfg)
    assert B.config_workspace(B.make_desc(big), cfg)[0] > 0
    # second call, right after it: a smaller input of another shape, the library's own choice of
    # configuration; whatever the first call left in the array must not show
    small = W.layer("na.small", 1, 12, (9, 11), 20, (3, 2), (2, 1), (1, 0), x_dist="u11", seed=402)
    # third: a persistent launch whose left-over tiles meet in the workspace, then atomics
    third = W.layer("na.third", 3, 16, (20, 20), 32, 3, 1, 1, x_dist="u11", seed=403)
    # fifth: a wave-split member (tap-major input), slices meeting in the workspace, then the default, which
    # for so small a problem is a wave-split member too
    fifth = W.layer("na.fifth", 1, 32, (14, 13), 48, 3, 1, 1, x_dist="u11", seed=404)
    cases = [(big, cfg), (small, None), (third, B.make_config(64, 32, 16, 2, 1, persist=1)),
             (big, B.make_config(64, 64, 16, 2, 2, split_k=4, reduce=1)),
             (fifth, B.make_config(32, 32, 8, 4, 1, split_k=3, stages=1)), (fifth, None)]
    assert B.config_default(B.make_desc(fifth)).bm == 32
    for layer, c in cases:
        mine, theirs, y_ref, d_ref = _both(layer, c)
        # the two entry points run the same kernels; split sums come in arrival order, so they are
        # compared within the tolerance of the path (1e-4 * D), and each against the oracle
        err = np.abs(mine - theirs) / np.where(d_ref == 0, 1.0, d_ref)
        assert err.max() <= PT.TOL, "%s: entry points differ by %.3g" % (layer["name"], err.max())
        PT.assert_close(mine, y_ref, d_ref, layer["name"] + " no-alloc")
        PT.assert_close(theirs, y_ref, d_ref, layer["name"] + " allocating")
        print(layer["name"], c, "max difference between the entry points %.3g" % err.max(), flush=True)


def test_no_alloc_entry_point_rejects_what_does_not_fit():
    torch, dev = PT.torch_dev()
    layer = W.layer("na.huge", 1, 2048, (7, 7), 2048, 3, 1, 1)
    t = torch.zeros(16, device=dev)
    with pytest.raises(B.WpkError) as e:
        B.conv2d_fwd_noalloc(B.make_desc(layer), t, t, t)     # rejected before anything is touched
    assert e.value.status == B.E_TOO_LARGE
    assert "static scratch" in str(e.value)
