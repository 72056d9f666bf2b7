"""Pins for the convolution oracle (CPU only).

Each test fixes the oracle to something other than itself: a hand-worked example, a
differently structured brute-force evaluator written here, a closed form, an identity,
or a library routine for a special case.  A dropped term, a flipped filter, a swapped
h/w index, a wrong pad/stride/dilation factor or a transposed operand fails one of them.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import conv as oc

pytestmark = pytest.mark.filterwarnings("ignore")


def rand(shape, seed):
    return np.random.default_rng(seed).uniform(-1, 1, size=shape).astype(np.float32)


# --------------------------------------------------------------------------------------
# independent evaluators (scatter form and im2col form), pure Python / NumPy fp64
# --------------------------------------------------------------------------------------
def scatter_conv(sh, x, w):
    """Loop over INPUT taps and add each product into every output that uses it.  The
    output coordinate is solved from the input coordinate, so the index algebra runs in
    the opposite direction from the oracle's gather."""
    P = (sh.h + 2 * sh.pad_h - sh.dil_h * (sh.r - 1) - 1) // sh.stride_h + 1
    Q = (sh.w + 2 * sh.pad_w - sh.dil_w * (sh.s - 1) - 1) // sh.stride_w + 1
    y = np.zeros((sh.n, sh.k, P, Q))
    d = np.zeros_like(y)
    x = x.astype(np.float64)
    w = w.astype(np.float64)
    for n, c, ih, iw in itertools.product(range(sh.n), range(sh.c), range(sh.h), range(sh.w)):
        for r, s in itertools.product(range(sh.r), range(sh.s)):
            ph = ih + sh.pad_h - r * sh.dil_h
            qw = iw + sh.pad_w - s * sh.dil_w
            if ph % sh.stride_h or qw % sh.stride_w:
                continue
            p, q = ph // sh.stride_h, qw // sh.stride_w
            if 0 <= p < P and 0 <= q < Q:
                for k in range(sh.k):
                    t = x[n, c, ih, iw] * w[k, c, r, s]
                    y[n, k, p, q] += t
                    d[n, k, p, q] += abs(t)
    return y, d


def im2col_conv(sh, x, w):
    """Materialise the (C*R*S) x (P*Q) patch matrix of a zero-padded copy of x, then one
    fp64 matrix product per image."""
    P = (sh.h + 2 * sh.pad_h - sh.dil_h * (sh.r - 1) - 1) // sh.stride_h + 1
    Q = (sh.w + 2 * sh.pad_w - sh.dil_w * (sh.s - 1) - 1) // sh.stride_w + 1
    xp = np.zeros((sh.n, sh.c, sh.h + 2 * sh.pad_h, sh.w + 2 * sh.pad_w))
    xp[:, :, sh.pad_h:sh.pad_h + sh.h, sh.pad_w:sh.pad_w + sh.w] = x
    cols = np.empty((sh.n, sh.c, sh.r, sh.s, P, Q))
    for r, s in itertools.product(range(sh.r), range(sh.s)):
        h0, w0 = r * sh.dil_h, s * sh.dil_w
        cols[:, :, r, s] = xp[:, :, h0:h0 + (P - 1) * sh.stride_h + 1:sh.stride_h,
                              w0:w0 + (Q - 1) * sh.stride_w + 1:sh.stride_w]
    wm = w.astype(np.float64).reshape(sh.k, -1)
    return np.einsum("kj,njm->nkm", wm, cols.reshape(sh.n, sh.c * sh.r * sh.s, P * Q)
                     ).reshape(sh.n, sh.k, P, Q)


TINY = [
    # n c h w k r s stride pad dil
    (1, 1, 3, 3, 1, 3, 3, (1, 1), (1, 1), (1, 1)),
    (2, 3, 6, 5, 3, 3, 3, (1, 1), (1, 1), (1, 1)),
    (1, 2, 6, 6, 2, 3, 2, (2, 1), (0, 1), (1, 1)),
    (2, 3, 5, 6, 2, 2, 3, (1, 2), (2, 0), (1, 1)),
    (1, 2, 6, 6, 3, 3, 3, (3, 3), (2, 2), (1, 1)),
    (1, 3, 6, 6, 2, 3, 3, (1, 1), (2, 2), (2, 2)),
    (1, 2, 6, 5, 2, 2, 3, (2, 1), (1, 2), (2, 1)),
    (2, 1, 4, 6, 3, 1, 1, (1, 1), (0, 0), (1, 1)),
    (1, 3, 5, 5, 2, 1, 1, (2, 2), (0, 0), (1, 1)),
    (1, 2, 4, 4, 2, 3, 3, (1, 1), (3, 3), (1, 1)),   # pad larger than R/2
    (1, 2, 6, 6, 2, 1, 3, (1, 2), (0, 1), (1, 2)),
]


@pytest.mark.parametrize("cfg", TINY)
def test_brute_force_scatter_and_im2col(cfg):
    n, c, h, w_, k, r, s, st, pd, dl = cfg
    sh = oc.make_shape(n, c, h, w_, k, r, s, st, pd, dl)
    x, w = rand((n, c, h, w_), 11), rand((k, c, r, s), 12)
    y, d, _ = oc.conv2d(sh, x, w)
    ys, ds = scatter_conv(sh, x, w)
    yi = im2col_conv(sh, x, w)
    assert y.shape == ys.shape == yi.shape
    tol = 1e-12 * np.maximum(d, 1e-30)
    assert np.all(np.abs(y - ys) <= tol)
    assert np.all(np.abs(y - yi) <= tol)
    assert np.all(np.abs(d - ds) <= 1e-12 * np.maximum(ds, 1e-30))


# --------------------------------------------------------------------------------------
# hand-worked example and a library routine for the single-channel case
# --------------------------------------------------------------------------------------
def read_blocks(path):
    blocks, cur = {}, None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line[0].isalpha():
            cur = line
            blocks[cur] = []
        else:
            blocks[cur].append([float(v) for v in line.split()])
    return {k: np.array(v) for k, v in blocks.items()}


def test_hand_worked_sample(golden_dir):
    b = read_blocks(os.path.join(golden_dir, "sample_3x3_worked.txt"))
    sh = oc.make_shape(1, 1, 3, 3, 1, 3, 3, (1, 1), (1, 1))
    y, d, _ = oc.conv2d(sh, b["in"].reshape(1, 1, 3, 3), b["filter"].reshape(1, 1, 3, 3))
    assert np.array_equal(y[0, 0], b["out"])
    # the same fixture against SciPy's 2-D cross-correlation (a second, unrelated code)
    from scipy.signal import correlate2d
    assert np.array_equal(correlate2d(b["in"], b["filter"], mode="same"), b["out"])


def test_single_channel_matches_scipy_correlate2d():
    from scipy.signal import correlate2d
    x, w = rand((1, 1, 9, 7), 5), rand((1, 1, 3, 5), 6)
    sh = oc.make_shape(1, 1, 9, 7, 1, 3, 5, (1, 1), (1, 2))
    y, _, _ = oc.conv2d(sh, x, w)
    ref = correlate2d(x[0, 0].astype(np.float64), w[0, 0].astype(np.float64), mode="same")
    assert np.allclose(y[0, 0], ref, rtol=0, atol=1e-13)
    sh = oc.make_shape(1, 1, 9, 7, 1, 3, 5)                      # VALID
    y, _, _ = oc.conv2d(sh, x, w)
    ref = correlate2d(x[0, 0].astype(np.float64), w[0, 0].astype(np.float64), mode="valid")
    assert np.allclose(y[0, 0], ref, rtol=0, atol=1e-13)


# --------------------------------------------------------------------------------------
# identities and closed forms
# --------------------------------------------------------------------------------------
def test_delta_1x1_is_identity():
    x = rand((2, 5, 6, 7), 1)
    w = np.eye(5, dtype=np.float32).reshape(5, 5, 1, 1)
    y, _, _ = oc.conv2d(oc.make_shape(2, 5, 6, 7, 5, 1, 1), x, w)
    assert np.array_equal(y.astype(np.float32), x)


@pytest.mark.parametrize("r,s,dil", [(3, 3, 1), (5, 3, 1), (3, 3, 2), (3, 5, 2)])
def test_centred_delta_is_identity(r, s, dil):
    x = rand((1, 3, 8, 9), 2)
    w = np.zeros((3, 3, r, s), np.float32)
    for c in range(3):
        w[c, c, (r - 1) // 2, (s - 1) // 2] = 1
    sh = oc.make_shape(1, 3, 8, 9, 3, r, s, (1, 1), (dil * (r - 1) // 2, dil * (s - 1) // 2),
                       (dil, dil))
    y, _, _ = oc.conv2d(sh, x, w)
    assert np.array_equal(y.astype(np.float32), x)


def test_off_centre_delta_shifts_with_zero_fill():
    x = rand((1, 1, 6, 7), 3)
    w = np.zeros((1, 1, 3, 3), np.float32)
    w[0, 0, 0, 2] = 1           # tap (r=0, s=2): y[p,q] = x[p-1, q+1]
    y, _, _ = oc.conv2d(oc.make_shape(1, 1, 6, 7, 1, 3, 3, (1, 1), (1, 1)), x, w)
    ref = np.zeros((6, 7))
    ref[1:, :-1] = x[0, 0, :-1, 1:]
    assert np.array_equal(y[0, 0], ref)


def test_strided_delta_subsamples():
    x = rand((2, 2, 9, 8), 4)
    w = np.eye(2, dtype=np.float32).reshape(2, 2, 1, 1)
    y, _, _ = oc.conv2d(oc.make_shape(2, 2, 9, 8, 2, 1, 1, (2, 3)), x, w)
    assert np.array_equal(y.astype(np.float32), x[:, :, ::2, ::3])


def taps_in_bounds(out, size, win, stride, pad, dil):
    return np.array([sum(0 <= p * stride - pad + r * dil < size for r in range(win))
                     for p in range(out)])


@pytest.mark.parametrize("h,w_,r,s,st,pd,dl", [(7, 7, 3, 3, 1, 1, 1), (8, 6, 3, 5, 2, 2, 1),
                                              (9, 9, 3, 3, 1, 2, 2), (14, 14, 7, 7, 2, 3, 1),
                                              (5, 5, 3, 3, 1, 3, 1)])
def test_all_ones_counts_taps(h, w_, r, s, st, pd, dl):
    C, K = 5, 2
    sh = oc.make_shape(1, C, h, w_, K, r, s, (st, st), (pd, pd), (dl, dl))
    P, Q = oc.out_shape(sh)
    y, d, _ = oc.conv2d(sh, np.ones((1, C, h, w_), np.float32), np.ones((K, C, r, s), np.float32))
    ref = C * np.outer(taps_in_bounds(P, h, r, st, pd, dl), taps_in_bounds(Q, w_, s, st, pd, dl))
    assert np.array_equal(y[0, 0], ref) and np.array_equal(y[0, 1], ref)
    assert np.array_equal(d, y)
    if (r, s, st, pd, dl) == (3, 3, 1, 1, 1):
        assert y[0, 0, 0, 0] == 4 * C and y[0, 0, 0, 3] == 6 * C and y[0, 0, 3, 3] == 9 * C


def test_linearity_in_x_and_w():
    """conv(a*x1 + b*x2, w) = a*conv(x1, w) + b*conv(x2, w), and alike in w.  Inputs are
    multiples of 1/8 and the factors powers of two, so the combined inputs are exact in
    fp32 and the identity has to hold to fp64 round-off of the sums."""
    sh = oc.make_shape(2, 3, 7, 6, 4, 3, 3, (2, 1), (1, 1))
    q8 = lambda a: (np.round(8 * a) / 8).astype(np.float32)
    x1, x2 = q8(rand((2, 3, 7, 6), 7)), q8(rand((2, 3, 7, 6), 8))
    w1, w2 = q8(rand((4, 3, 3, 3), 9)), q8(rand((4, 3, 3, 3), 10))
    a, b = 0.5, -2.0
    y11, d11, _ = oc.conv2d(sh, x1, w1)
    y21, d21, _ = oc.conv2d(sh, x2, w1)
    y12, d12, _ = oc.conv2d(sh, x1, w2)
    yx, _, _ = oc.conv2d(sh, a * x1 + b * x2, w1)
    assert np.all(np.abs(yx - (a * y11 + b * y21)) <= 1e-13 * (abs(a) * d11 + abs(b) * d21))
    yw, _, _ = oc.conv2d(sh, x1, a * w1 + b * w2)
    assert np.all(np.abs(yw - (a * y11 + b * y12)) <= 1e-13 * (abs(a) * d11 + abs(b) * d12))
    assert np.abs(yx).max() > 0.1 and np.abs(yw).max() > 0.1


def test_1x1_is_a_matrix_product():
    n, c, h, w_, k = 2, 7, 5, 6, 4
    x, w = rand((n, c, h, w_), 21), rand((k, c, 1, 1), 22)
    y, _, _ = oc.conv2d(oc.make_shape(n, c, h, w_, k, 1, 1), x, w)
    ref = np.matmul(w.reshape(k, c).astype(np.float64),
                    x.reshape(n, c, h * w_).astype(np.float64)).reshape(n, k, h, w_)
    assert np.allclose(y, ref, rtol=0, atol=1e-13)


def test_full_window_is_a_dot_product():
    n, c, h, w_, k = 3, 4, 5, 3, 2
    x, w = rand((n, c, h, w_), 23), rand((k, c, h, w_), 24)
    sh = oc.make_shape(n, c, h, w_, k, h, w_)
    assert oc.out_shape(sh) == (1, 1)
    y, _, _ = oc.conv2d(sh, x, w)
    ref = x.reshape(n, -1).astype(np.float64) @ w.reshape(k, -1).astype(np.float64).T
    assert np.allclose(y.reshape(n, k), ref, rtol=0, atol=1e-13)


def test_translation_equivariance_interior():
    x = np.zeros((1, 2, 12, 12), np.float32)
    x[:, :, 3:8, 3:8] = rand((1, 2, 5, 5), 25)
    w = rand((3, 2, 3, 3), 26)
    sh = oc.make_shape(1, 2, 12, 12, 3, 3, 3, (1, 1), (1, 1))
    y0, _, _ = oc.conv2d(sh, x, w)
    y1, _, _ = oc.conv2d(sh, np.roll(x, (2, 1), axis=(2, 3)), w)
    assert np.array_equal(np.roll(y0, (2, 1), axis=(2, 3)), y1)


def test_channels_and_filters_are_not_transposed():
    # K != C, R != S, H != W with a one-hot weight: exactly one (k,c,r,s) tap is live
    n, c, h, w_, k, r, s = 1, 3, 6, 8, 4, 2, 3
    x = rand((n, c, h, w_), 27)
    w = np.zeros((k, c, r, s), np.float32)
    w[3, 1, 1, 2] = 2.0
    y, _, _ = oc.conv2d(oc.make_shape(n, c, h, w_, k, r, s), x, w)
    assert y.shape == (1, 4, 5, 6)
    assert np.array_equal(y[0, 3], 2.0 * x[0, 1, 1:6, 2:8].astype(np.float64))
    assert not y[0, :3].any()


# --------------------------------------------------------------------------------------
# normaliser, sampled entry point, threads, shapes, errors
# --------------------------------------------------------------------------------------
def test_normaliser_is_conv_of_absolute_values():
    sh = oc.make_shape(2, 3, 6, 6, 3, 3, 3, (1, 1), (1, 1))
    x, w = rand((2, 3, 6, 6), 31), rand((3, 3, 3, 3), 32)
    y, d, _ = oc.conv2d(sh, x, w)
    yabs, _, _ = oc.conv2d(sh, np.abs(x), np.abs(w))
    assert np.allclose(d, yabs, rtol=1e-14, atol=0)
    assert np.all(np.abs(y) <= d * (1 + 1e-15))


def test_sampled_equals_full_and_threads_change_nothing():
    sh = oc.make_shape(2, 4, 9, 8, 5, 3, 3, (2, 1), (1, 1))
    x, w = rand((2, 4, 9, 8), 33), rand((5, 4, 3, 3), 34)
    y1, d1, u1 = oc.conv2d(sh, x, w, threads=1)
    y4, d4, u4 = oc.conv2d(sh, x, w, threads=4)
    assert u1 == 1 and u4 == 4
    assert np.array_equal(y1, y4) and np.array_equal(d1, d4)
    idx = np.random.default_rng(0).integers(0, y1.size, size=50)
    ys, ds = oc.conv2d_sampled(sh, x, w, idx)
    assert np.array_equal(ys, y1.reshape(-1)[idx]) and np.array_equal(ds, d1.reshape(-1)[idx])
    with pytest.raises(ValueError):
        oc.conv2d_sampled(sh, x, w, [y1.size])


@pytest.mark.parametrize("h,r,st,pd,dl,p", [(224, 7, 2, 3, 1, 112), (56, 3, 1, 1, 1, 56),
                                           (56, 3, 2, 1, 1, 28), (56, 1, 2, 0, 1, 28),
                                           (14, 1, 2, 0, 1, 7), (7, 3, 1, 1, 1, 7),
                                           (112, 3, 1, 0, 1, 110), (110, 3, 2, 0, 1, 54),
                                           (54, 3, 2, 0, 1, 26), (26, 3, 2, 0, 1, 12),
                                           (10, 3, 1, 0, 3, 4), (5, 3, 1, 0, 3, None)])
def test_output_extent_values(h, r, st, pd, dl, p):
    # ResNet extents named by the workload text, Table 1's row-to-row sizes, dilation
    sh = oc.make_shape(1, 1, h, h, 1, r, r, (st, st), (pd, pd), (dl, dl))
    assert oc.out_shape(sh) == (None if p is None else (p, p))


def test_illegal_shapes_are_rejected():
    assert oc.out_shape(oc.make_shape(0, 1, 4, 4, 1, 3, 3)) is None
    assert oc.out_shape(oc.make_shape(1, 1, 4, 4, 1, 3, 3, (0, 1))) is None
    assert oc.out_shape(oc.make_shape(1, 1, 4, 4, 1, 3, 3, (1, 1), (-1, 0))) is None
    assert oc.out_shape(oc.make_shape(1, 1, 2, 2, 1, 3, 3)) is None
    assert oc.out_shape(oc.make_shape(1, 1, 4, 4, 1, 3, 3, (1, 1), (0, 0), (0, 1))) is None


def test_planted_mistakes_are_caught():
    """The evaluators above disagree with plausible wrong variants: a flipped filter and a
    swapped pad -- shows the pins have teeth (mistakes planted here, on the CPU)."""
    sh = oc.make_shape(1, 2, 6, 5, 2, 3, 3, (1, 1), (1, 1))
    x, w = rand((1, 2, 6, 5), 41), rand((2, 2, 3, 3), 42)
    y, d, _ = oc.conv2d(sh, x, w)
    y_flip, _, _ = oc.conv2d(sh, x, w[:, :, ::-1, ::-1])
    assert np.max(np.abs(y - y_flip) / d) > 1e-3
    sh2 = oc.make_shape(1, 2, 6, 5, 2, 3, 3, (1, 1), (0, 2))
    if oc.out_shape(sh2) == oc.out_shape(sh):
        y_pad, _, _ = oc.conv2d(sh2, x, w)
        assert np.max(np.abs(y - y_pad)) > 1e-3


# ---- fused operator (Section 2.1, operator fusion) ---------------------------------------------
def _read_blocks(path):
    blocks, cur = {}, None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line[0].isalpha():
            cur = line
            blocks[cur] = []
        else:
            blocks[cur].append([float(v) for v in line.split()])
    return {k: np.array(v) for k, v in blocks.items()}


def test_fused_hand_worked_sample(golden_dir):
    conv_fix = _read_blocks(os.path.join(golden_dir, "sample_3x3_worked.txt"))
    fix = _read_blocks(os.path.join(golden_dir, "fused_worked.txt"))
    assert np.array_equal(fix["conv"], conv_fix["out"])
    sh = oc.make_shape(1, 1, 3, 3, 1, 3, 3, pad=(1, 1))
    x, w = conv_fix["in"].reshape(1, 1, 3, 3), conv_fix["filter"].reshape(1, 1, 3, 3)
    bias = fix["bias"].reshape(1)
    y, d = oc.conv2d_fused(sh, x, w, bias=bias, residual=fix["residual"], relu=True)
    assert np.array_equal(y.reshape(3, 3), fix["out"])
    z, _ = oc.conv2d_fused(sh, x, w, bias=bias, residual=fix["residual"], relu=False)
    assert np.array_equal(z.reshape(3, 3), fix["z"])


def test_fused_special_cases():
    rng = np.random.default_rng(11)
    sh = oc.make_shape(2, 3, 6, 5, 4, 3, 2, stride=(1, 2), pad=(1, 0))
    P, Q = oc.out_shape(sh)
    x = rng.uniform(-1, 1, (2, 3, 6, 5)).astype(np.float32)
    w = rng.uniform(-1, 1, (4, 3, 3, 2)).astype(np.float32)
    b = rng.uniform(-1, 1, 4).astype(np.float32)
    r = rng.uniform(-1, 1, (2, 4, P, Q)).astype(np.float32)
    y0, d0, _ = oc.conv2d(sh, x, w)
    # nothing fused: the plain convolution and its normaliser
    y, d = oc.conv2d_fused(sh, x, w)
    assert np.array_equal(y, y0) and np.array_equal(d, d0)
    # zero weights: what remains is the rectified sum of bias and residual, channel by channel
    y, d = oc.conv2d_fused(sh, x, np.zeros_like(w), bias=b, residual=r, relu=True)
    for k in range(4):
        assert np.array_equal(y[:, k], np.maximum(r[:, k].astype(np.float64) + np.float64(b[k]), 0.0))
        assert np.array_equal(d[:, k], np.abs(r[:, k].astype(np.float64)) + abs(np.float64(b[k])))
    # the bias lands on the channel axis, not on a spatial one: a one-hot bias changes one channel
    onehot = np.zeros(4, np.float32)
    onehot[2] = 5.0
    y, _ = oc.conv2d_fused(sh, x, w, bias=onehot)
    diff = y - y0
    assert np.allclose(diff[:, 2], 5.0, rtol=0, atol=1e-12) and np.all(np.delete(diff, 2, axis=1) == 0.0)
    # rectifier: max(z,0) = (z + |z|)/2, and the negative part is removed, not mirrored
    z, _ = oc.conv2d_fused(sh, x, w, bias=b, residual=r)
    y, _ = oc.conv2d_fused(sh, x, w, bias=b, residual=r, relu=True)
    assert np.allclose(y, 0.5 * (z + np.abs(z)), rtol=0, atol=1e-15)
    assert y.min() == 0.0 and (z < 0).any() and np.array_equal(y[z > 0], z[z > 0])
    # residual addition commutes with the convolution's linearity: conv(x,w)+r == fused(r)
    assert np.array_equal(z, y0 + b.astype(np.float64)[None, :, None, None] + r.astype(np.float64))


# ---- channels-last activations (Section 2.1, data layout transformation) ------------------------
def _brute_nhwc(n_, c_, h_, w_, k_, r_, s_, st, pd, dl, x, w):
    """Second evaluator, written on flat channels-last buffers with its own index arithmetic:
    scatter form (every input element is pushed to the outputs it feeds)."""
    p_ = (h_ + 2 * pd[0] - dl[0] * (r_ - 1) - 1) // st[0] + 1
    q_ = (w_ + 2 * pd[1] - dl[1] * (s_ - 1) - 1) // st[1] + 1
    xf, wf = np.asarray(x, np.float64).ravel(), np.asarray(w, np.float64).ravel()
    y = np.zeros(n_ * p_ * q_ * k_)
    for n in range(n_):
        for hi in range(h_):
            for wi in range(w_):
                for c in range(c_):
                    xv = xf[((n * h_ + hi) * w_ + wi) * c_ + c]
                    for r in range(r_):
                        ph = hi + pd[0] - r * dl[0]
                        if ph % st[0] or not 0 <= ph // st[0] < p_:
                            continue
                        for s in range(s_):
                            qw = wi + pd[1] - s * dl[1]
                            if qw % st[1] or not 0 <= qw // st[1] < q_:
                                continue
                            base = ((n * p_ + ph // st[0]) * q_ + qw // st[1]) * k_
                            for k in range(k_):
                                y[base + k] += xv * wf[((k * c_ + c) * r_ + r) * s_ + s]
    return y.reshape(n_, p_, q_, k_)


@pytest.mark.parametrize("cfg", [
    (2, 3, 5, 4, 2, 3, 2, (1, 1), (1, 0), (1, 1)),
    (1, 4, 6, 5, 3, 2, 3, (2, 1), (0, 2), (1, 2)),
    (2, 2, 7, 6, 3, 3, 3, (2, 3), (2, 1), (2, 1)),
])
def test_channels_last_against_flat_scatter_evaluator(cfg):
    n_, c_, h_, w_, k_, r_, s_, st, pd, dl = cfg
    rng = np.random.default_rng(hash(cfg) % 1000)
    x = rng.uniform(-1, 1, (n_, h_, w_, c_)).astype(np.float32)          # channels last
    w = rng.uniform(-1, 1, (k_, c_, r_, s_)).astype(np.float32)
    sh = oc.make_shape(n_, c_, h_, w_, k_, r_, s_, st, pd, dl)
    y, d = oc.conv2d_layout(sh, x, w, "NHWC", "NHWC")
    ref = _brute_nhwc(n_, c_, h_, w_, k_, r_, s_, st, pd, dl, x, w)
    assert y.shape == ref.shape
    assert np.max(np.abs(y - ref)) <= 1e-12 * max(1.0, d.max())
    # mixed layouts are the same values, permuted
    y2, d2 = oc.conv2d_layout(sh, x, w, "NHWC", "NCHW")
    assert np.array_equal(y2, y.transpose(0, 3, 1, 2)) and np.array_equal(d2, d.transpose(0, 3, 1, 2))
    y3, _ = oc.conv2d_layout(sh, x.transpose(0, 3, 1, 2), w, "NCHW", "NHWC")
    assert np.array_equal(y3, y)


def test_channels_last_delta_and_channel_order():
    # 1x1 identity weights: y == x in the same layout; a channel permutation in w permutes the
    # last axis (the channel axis of a channels-last tensor), not a spatial one
    rng = np.random.default_rng(8)
    x = rng.uniform(-1, 1, (2, 5, 4, 6)).astype(np.float32)              # N H W C
    sh = oc.make_shape(2, 6, 5, 4, 6, 1, 1)
    eye = np.eye(6, dtype=np.float32).reshape(6, 6, 1, 1)
    y, _ = oc.conv2d_layout(sh, x, eye, "NHWC", "NHWC")
    assert np.array_equal(y, x.astype(np.float64))
    perm = np.array([3, 0, 5, 1, 4, 2])
    y, _ = oc.conv2d_layout(sh, x, eye[perm], "NHWC", "NHWC")
    assert np.array_equal(y, x[..., perm].astype(np.float64))


@pytest.mark.parametrize("cfg", [
    (2, 3, 5, 4, 2, 3, 2, (1, 1), (1, 0), (1, 1)),
    (1, 4, 6, 5, 3, 2, 3, (2, 1), (0, 2), (1, 2)),
])
def test_fused_channels_last_against_flat_evaluator(cfg):
    """The fused operator with channels-last tensors, against an evaluator that works on flat
    buffers: output element i of [N][P][Q][K] gets bias[i mod K] and the residual's element i."""
    n_, c_, h_, w_, k_, r_, s_, st, pd, dl = cfg
    rng = np.random.default_rng(77 + c_)
    x = rng.uniform(-1, 1, (n_, h_, w_, c_)).astype(np.float32)
    w = rng.uniform(-1, 1, (k_, c_, r_, s_)).astype(np.float32)
    b = rng.uniform(-1, 1, k_).astype(np.float32)
    conv = _brute_nhwc(n_, c_, h_, w_, k_, r_, s_, st, pd, dl, x, w)
    res = rng.uniform(-1, 1, conv.shape).astype(np.float32)
    flat = conv.ravel().copy()
    for i in range(flat.size):
        flat[i] += float(b[i % k_]) + float(res.ravel()[i])
        flat[i] = flat[i] if flat[i] > 0.0 else 0.0
    sh = oc.make_shape(n_, c_, h_, w_, k_, r_, s_, st, pd, dl)
    y, d = oc.conv2d_fused(sh, x, w, bias=b, residual=res, relu=True, x_layout="NHWC", y_layout="NHWC")
    assert y.shape == conv.shape and (y == 0).any() and (y > 0).any()
    assert np.max(np.abs(y.ravel() - flat)) <= 1e-12 * max(1.0, d.max())
    # the normaliser: the convolution's, plus |bias| along the LAST axis, plus |residual|
    _, d0 = oc.conv2d_layout(sh, x, w, "NHWC", "NHWC")
    assert np.array_equal(d, d0 + np.abs(b.astype(np.float64)) + np.abs(res.astype(np.float64)))
    # mixed layouts: x in one layout, y and the residual in the other -- same values, permuted
    y2, d2 = oc.conv2d_fused(sh, x, w, bias=b, residual=res.transpose(0, 3, 1, 2), relu=True,
                             x_layout="NHWC", y_layout="NCHW")
    assert np.array_equal(y2, y.transpose(0, 3, 1, 2)) and np.array_equal(d2, d.transpose(0, 3, 1, 2))
    y3, _ = oc.conv2d_fused(sh, x.transpose(0, 3, 1, 2), w, bias=b, residual=res, relu=True,
                            x_layout="NCHW", y_layout="NHWC")
    assert np.array_equal(y3, y)
    # a one-hot bias changes one index of the last axis only
    onehot = np.zeros(k_, np.float32)
    onehot[1] = 3.0
    y4, _ = oc.conv2d_fused(sh, x, w, bias=onehot, x_layout="NHWC", y_layout="NHWC")
    y5, _ = oc.conv2d_layout(sh, x, w, "NHWC", "NHWC")
    diff = y4 - y5
    assert np.allclose(diff[..., 1], 3.0, rtol=0, atol=1e-12) and np.all(np.delete(diff, 1, axis=3) == 0.0)
