"""Host-side tests of the layout optimiser (wpk_choose_layouts): exact against brute force over all
assignments on small random graphs shaped like networks -- chains with shortcut branches, residual
ties, tensors the caller fixes.  (The expected value is an enumeration of every assignment, not a
second copy of the elimination.)"""
import itertools

import numpy as np
import pytest

from paper_2008_04567_amd import binding as B


def brute(x_t, y_t, r_t, fixed, cost):
    nt = len(fixed)
    best, arg = None, None
    for lay in itertools.product((0, 1), repeat=nt):
        if any(f >= 0 and f != v for f, v in zip(fixed, lay)):
            continue
        if r_t is not None and any(r >= 0 and lay[r] != lay[y] for r, y in zip(r_t, y_t)):
            continue
        tot = sum(cost[i][lay[x]][lay[y]] for i, (x, y) in enumerate(zip(x_t, y_t)))
        if best is None or tot < best:
            best, arg = tot, lay
    return best, arg


def random_network(rng, blocks):
    """A residual network's tensor graph: per block a chain of 2-3 layers from tensor `cur`, the last
    adding a shortcut: either `cur` itself or a projection layer's output."""
    x_t, y_t, r_t = [], [], []
    nt, cur = 1, 0
    for _ in range(blocks):
        depth = int(rng.integers(2, 4))
        src = cur
        if rng.random() < 0.5:                      # projection shortcut: a layer of its own
            x_t.append(cur); y_t.append(nt); r_t.append(-1)
            short, nt = nt, nt + 1
        else:
            short = cur
        for k in range(depth):
            x_t.append(src); y_t.append(nt)
            r_t.append(short if k == depth - 1 else -1)
            src, nt = nt, nt + 1
        cur = src
    return x_t, y_t, r_t, nt


@pytest.mark.parametrize("seed", range(40))
def test_exact_against_enumeration(seed):
    rng = np.random.default_rng(seed)
    x_t, y_t, r_t, nt = random_network(rng, int(rng.integers(1, 4)))
    if nt > 12:
        x_t, y_t, r_t = x_t[:8], y_t[:8], r_t[:8]
        nt = max(max(x_t), max(y_t), max(r_t)) + 1
    fixed = [-1] * nt
    fixed[0] = int(rng.integers(0, 2))
    if rng.random() < 0.7:
        fixed[y_t[-1]] = int(rng.integers(0, 2))
    cost = rng.uniform(1.0, 2.0, (len(x_t), 2, 2)).round(3).tolist()
    want, _ = brute(x_t, y_t, r_t, fixed, cost)
    if want is None:                                # ties force two fixed tensors to differ
        with pytest.raises(B.WpkError):
            B.choose_layouts(x_t, y_t, r_t, fixed, cost)
        return
    lay, tot = B.choose_layouts(x_t, y_t, r_t, fixed, cost)
    assert abs(tot - want) <= 1e-9
    assert all(f < 0 or f == v for f, v in zip(fixed, lay))
    assert all(r < 0 or lay[r] == lay[y] for r, y in zip(r_t, y_t))
    assert abs(sum(cost[i][lay[x]][lay[y]] for i, (x, y) in enumerate(zip(x_t, y_t))) - want) <= 1e-9


def test_plain_chain_and_special_cases():
    # the optimum needs BOTH inner tensors flipped together (either flip alone loses)
    cost = [[[10, 12], [99, 99]], [[10, 99], [99, 5]], [[10, 99], [12, 99]]]
    lay, tot = B.choose_layouts([0, 1, 2], [1, 2, 3], None, [0, -1, -1, 0], cost)
    assert lay == [0, 1, 1, 0] and tot == 12 + 5 + 12
    # everything fixed: nothing to choose, the total is the fixed assignment's
    lay, tot = B.choose_layouts([0, 1], [1, 2], None, [1, 0, 1], [[[1, 2], [3, 4]], [[5, 6], [7, 8]]])
    assert lay == [1, 0, 1] and tot == 3 + 6
    # a layer that reads and writes the same group (residual = its own input): cost[l][l] only
    lay, tot = B.choose_layouts([0], [1], [0], [-1, -1], [[[4, 0], [0, 3]]])
    assert lay == [1, 1] and tot == 3
    # tensors no layer touches take their fixed layout, else 0
    lay, _ = B.choose_layouts([0], [1], None, [0, 0, 1, -1], [[[1, 1], [1, 1]]])
    assert lay == [0, 0, 1, 0]
    # errors: tensor number out of range; tied tensors fixed to different layouts
    with pytest.raises(B.WpkError):
        B.choose_layouts([0], [5], None, [0, 0], [[[1, 1], [1, 1]]])
    with pytest.raises(B.WpkError):
        B.choose_layouts([0], [1], [2], [0, 0, 1], [[[1, 1], [1, 1]]])


def test_a_deep_chain_is_fast_and_exact():
    """200 layers in a chain with shortcuts every third layer: the frontier stays small, so the
    elimination is instant; checked against a chain dynamic programme written out here."""
    rng = np.random.default_rng(5)
    n = 200
    cost = rng.uniform(1.0, 2.0, (n, 2, 2))
    x_t, y_t = list(range(n)), list(range(1, n + 1))
    fixed = [0] + [-1] * (n - 1) + [0]
    lay, tot = B.choose_layouts(x_t, y_t, None, fixed, cost.tolist())
    best = np.array([0.0, np.inf])                  # tensor 0 is fixed to 0
    for i in range(n):
        best = np.array([min(best[a] + cost[i, a, b] for a in range(2)) for b in range(2)])
    assert abs(tot - best[0]) <= 1e-9 and lay[0] == 0 and lay[-1] == 0
