"""GPU parity on seeded random problems: shape, stride, padding, dilation, layout, configuration and
epilogue drawn together, each case against the oracle element by element (bound of tests/parity.py).
The draws are fixed by the seed, so a failure names its case."""
import numpy as np
import pytest

from paper_2008_04567_amd import binding as B
from paper_2008_04567_amd import workloads as W
from tests import parity as PT

pytestmark = pytest.mark.gpu


def _draw(rng, idx):
    r = int(rng.choice([1, 1, 2, 3, 3, 5, 7]))
    s = int(rng.choice([1, 2, 3, 3, 4])) if r != 1 else int(rng.choice([1, 1, 3]))
    dil = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
    stride = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
    pad = (int(rng.integers(0, dil[0] * (r - 1) + 1)), int(rng.integers(0, dil[1] * (s - 1) + 1)))
    h = int(rng.integers(dil[0] * (r - 1) + 1, 34))
    w = int(rng.integers(dil[1] * (s - 1) + 1, 34))
    c = int(rng.choice([1, 3, 5, 8, 16, 20, 32, 33, 64, 96]))
    k = int(rng.choice([1, 4, 7, 16, 31, 64, 65, 130]))
    n = int(rng.integers(1, 5))
    return W.layer("rand%d" % idx, n, c, (h, w), k, (r, s), stride, pad, dil, x_dist="u11", w_dist="u11",
                   seed=9000 + idx)


@pytest.mark.parametrize("chunk", range(6))
def test_random_problems(chunk):
    rng = np.random.default_rng(1234 + chunk)
    lo, hi = B.config_gene_ranges()
    for i in range(30):
        l = _draw(rng, 100 * chunk + i)
        layout = int(rng.integers(0, 4))
        desc = B.make_desc(l, layout=layout)
        P, Q = B.conv_out_shape(desc)
        cfg = None
        for _ in range(200):                       # a random legal member of the family, if any
            c = B.config_from_genes([int(rng.integers(a, b + 1)) for a, b in zip(lo, hi)])
            if B.config_legal(desc, c):
                cfg = c
                break
        fused = bool(rng.integers(0, 2))
        bias = rng.uniform(-1, 1, l["k"]).astype(np.float32) if fused and rng.integers(0, 2) else None
        res = (rng.uniform(-1, 1, (l["n"], l["k"], P, Q)).astype(np.float32)
               if fused and rng.integers(0, 2) else None)
        relu = fused and bool(rng.integers(0, 2))
        print(l["name"], {k_: l[k_] for k_ in ("n", "c", "h", "w", "k", "r", "s", "stride_h", "stride_w",
                                                "pad_h", "pad_w", "dil_h", "dil_w")},
              "layout", layout, cfg, "bias", bias is not None, "residual", res is not None, "relu", relu,
              flush=True)
        PT.check_layout(l, layout, cfg=cfg, bias=bias, residual=res, relu=relu)
