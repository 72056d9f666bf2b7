"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI on seeded
inputs and compare with the CPU oracle element by element.

Tolerance (fp32 arithmetic): |y_gpu - y_oracle| <= 1e-4 * D per output, D = sum |x*w| over the
output's taps (fp64, from the oracle); where D == 0 the GPU value must be exactly 0."""
import numpy as np

from oracle import conv as oc
from paper_2008_04567_amd import binding as B
from paper_2008_04567_amd import workloads as W

TOL = 1e-4
# Regression guard beside the pass bar.  An honest fp32 kernel lands far inside TOL: the largest
# normalised error ever recorded over this suite is 3e-6 (a 4608-term reduction summed in slices).
# A mistake worth a single dropped or doubled term is about 1/L of D on the outputs it touches,
# 2e-4 for the longest reduction here but diluted below TOL on outputs where that term is small,
# so a tenfold margin over the recorded worst is asserted as well.
RECORDED_WORST = 3e-6
GUARD = 10 * RECORDED_WORST


def torch_dev():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch, torch.device("cuda:0")


def to_dev(a):
    torch, dev = torch_dev()
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def oracle_full(layer, x, w):
    sh = oc.shape_from_layer(layer)
    y, d, _ = oc.conv2d(sh, x, w)
    return y, d


def assert_close(y_gpu, y_ref, d_ref, what=""):
    y_gpu = np.asarray(y_gpu, dtype=np.float64).reshape(y_ref.shape)
    assert np.all(np.isfinite(y_gpu)), what + ": non-finite output"
    zero = d_ref == 0
    assert np.all(y_gpu[zero] == 0.0), what + ": nonzero output where no tap contributes"
    err = np.abs(y_gpu - y_ref) / np.where(zero, 1.0, d_ref)
    worst = float(err.max()) if err.size else 0.0
    assert worst <= TOL, "%s: max normalised error %.3g > %g" % (what, worst, TOL)
    assert worst <= GUARD, ("%s: max normalised error %.3g is inside the tolerance but above %g, ten times "
                            "the worst this suite has recorded" % (what, worst, GUARD))
    return worst


def run_gpu(layer, x, w, cfg=None, mode="fwd"):
    """One convolution through the C ABI; returns the output as a NumPy array."""
    torch, dev = torch_dev()
    desc = B.make_desc(layer)
    P, Q = B.conv_out_shape(desc)
    xd, wd = to_dev(x), to_dev(w)
    # canary-filled output with guard bands to catch stray writes
    n_out = layer["n"] * layer["k"] * P * Q
    guard = 256
    buf = torch.full((n_out + 2 * guard,), 12345.0, device=dev, dtype=torch.float32)
    yd = buf[guard:guard + n_out]
    if mode == "ref":
        B.conv2d_ref(desc, xd, wd, yd)
    elif cfg is not None:
        B.conv2d_fwd_config(desc, cfg, xd, wd, yd)
    else:
        B.conv2d_fwd(desc, xd, wd, yd)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert np.all(host[:guard] == 12345.0) and np.all(host[guard + n_out:] == 12345.0), \
        "write outside the output tensor"
    return host[guard:guard + n_out].reshape(layer["n"], layer["k"], P, Q)


def run_gpu_fused(layer, x, w, bias=None, residual=None, relu=False, cfg=None):
    """The fused operator through the C ABI; returns the output as a NumPy array."""
    torch, dev = torch_dev()
    desc = B.make_desc(layer)
    P, Q = B.conv_out_shape(desc)
    n_out = layer["n"] * layer["k"] * P * Q
    guard = 256
    buf = torch.full((n_out + 2 * guard,), 12345.0, device=dev, dtype=torch.float32)
    yd = buf[guard:guard + n_out]
    B.conv2d_fwd_fused(desc, to_dev(x), to_dev(w), yd, bias=None if bias is None else to_dev(bias),
                       residual=None if residual is None else to_dev(residual), relu=relu, cfg=cfg)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert np.all(host[:guard] == 12345.0) and np.all(host[guard + n_out:] == 12345.0), \
        "write outside the output tensor"
    return host[guard:guard + n_out].reshape(layer["n"], layer["k"], P, Q)


def check_layer(layer, cfg=None, mode="fwd", what=None):
    x, w = W.make_inputs(layer)
    y_ref, d_ref = oracle_full(layer, x, w)
    y = run_gpu(layer, x, w, cfg=cfg, mode=mode)
    return assert_close(y, y_ref, d_ref, what or layer["name"])


LAYOUT_NAMES = {0: ("NCHW", "NCHW"), 1: ("NHWC", "NCHW"), 2: ("NCHW", "NHWC"), 3: ("NHWC", "NHWC")}


def check_layout(layer, layout, cfg=None, bias=None, residual=None, relu=False, what=None):
    """One convolution with activations in the given layout code (bit 0: x channels-last, bit 1:
    y and the residual channels-last) against the oracle in the same layouts.  ``layer`` and the
    seeded inputs are the usual NCHW ones; the host permutes them."""
    torch, dev = torch_dev()
    xl, yl = LAYOUT_NAMES[layout]
    x, w = W.make_inputs(layer)
    desc = B.make_desc(layer, layout=layout)
    P, Q = B.conv_out_shape(desc)
    x_host = np.ascontiguousarray(x.transpose(0, 2, 3, 1)) if xl == "NHWC" else x
    res_host = None
    if residual is not None:    # given as [N][K][P][Q]
        res_host = np.ascontiguousarray(residual.transpose(0, 2, 3, 1)) if yl == "NHWC" else residual
    sh = oc.shape_from_layer(layer)
    y_ref, d_ref = oc.conv2d_fused(sh, x_host, w, bias=bias, residual=res_host, relu=relu,
                                   x_layout=xl, y_layout=yl)
    n_out = y_ref.size
    guard = 256
    buf = torch.full((n_out + 2 * guard,), 12345.0, device=dev, dtype=torch.float32)
    yd = buf[guard:guard + n_out]
    B.conv2d_fwd_fused(desc, to_dev(x_host), to_dev(w), yd, bias=None if bias is None else to_dev(bias),
                       residual=None if res_host is None else to_dev(res_host), relu=relu, cfg=cfg)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert np.all(host[:guard] == 12345.0) and np.all(host[guard + n_out:] == 12345.0), \
        "write outside the output tensor"
    return assert_close(host[guard:guard + n_out], y_ref, d_ref,
                        what or "%s layout %d %r" % (layer["name"], layout, cfg))
