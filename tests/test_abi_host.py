"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and its host logic (descriptor validation, output-size rule, configuration encoding and
constraint check, cache, search engine) behaves as the header says.  No compute call."""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

from oracle import conv as oc
from oracle import ga as oga
from paper_2008_04567_amd import binding as B
from paper_2008_04567_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "wpk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(wpk_[a-z0-9_]+)\s*\(", text)
    return sorted(set(n for n in names if not n.endswith("_fn")))


def test_library_loads_and_exports_every_declared_symbol():
    L = B.lib()
    names = header_functions()
    assert len(names) >= 35
    for n in names:
        assert hasattr(L, n), "missing export " + n
    assert set(L._signatures) == set(names), "binding and header disagree"
    assert "gfx950" in B.version()


def test_struct_layouts_match_the_header(tmp_path):
    """Sizes and field offsets as a C compiler sees the header, against the ctypes mirrors."""
    import subprocess
    src = tmp_path / "sizes.c"
    src.write_text("""#include <stdio.h>
#include <stddef.h>
#include "wpk.h"
int main(void) {
  printf("%zu %zu %zu %zu %zu %zu %zu %zu\\n", sizeof(wpk_conv_desc), sizeof(wpk_conv_config),
         sizeof(wpk_tune_options), sizeof(wpk_tune_report), offsetof(wpk_tune_options, seed),
         offsetof(wpk_tune_options, min_group_us), offsetof(wpk_tune_report, best_us),
         offsetof(wpk_tune_report, seconds));
  return 0; }
""")
    exe = tmp_path / "sizes"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    got = [int(v) for v in subprocess.run([str(exe)], check=True, capture_output=True,
                                          text=True).stdout.split()]
    assert got == [ctypes.sizeof(B.ConvDesc), ctypes.sizeof(B.ConvConfig),
                   ctypes.sizeof(B.TuneOptions), ctypes.sizeof(B.TuneReport),
                   B.TuneOptions.seed.offset, B.TuneOptions.min_group_us.offset,
                   B.TuneReport.best_us.offset, B.TuneReport.seconds.offset]
    assert got[0] == 60 and got[1] == 40


def d13(n, c, h, w, k, r, s, st=(1, 1), pd=(0, 0), dl=(1, 1)):
    return B.make_desc(dict(n=n, c=c, h=h, w=w, k=k, r=r, s=s, stride_h=st[0], stride_w=st[1],
                            pad_h=pd[0], pad_w=pd[1], dil_h=dl[0], dil_w=dl[1]))


def test_out_shape_agrees_with_the_oracle_rule_over_a_sweep():
    import itertools
    for h, w, r, s, sh, sw, ph, pw, dh, dw in itertools.product(
            [1, 5, 8, 13], [3, 9], [1, 3, 4], [1, 2, 5], [1, 2, 3], [1, 2], [0, 1, 3], [0, 2],
            [1, 2], [1, 3]):
        ref = oc.out_shape(oc.make_shape(1, 1, h, w, 1, r, s, (sh, sw), (ph, pw), (dh, dw)))
        d = d13(1, 1, h, w, 1, r, s, (sh, sw), (ph, pw), (dh, dw))
        if ref is None:
            assert B.lib().wpk_conv_out_shape(ctypes.byref(d), None, None) == B.E_BAD_DESC
        else:
            assert B.conv_out_shape(d) == ref


def test_workload_shapes_and_flops():
    want = {"stem": 112, "s1b0.c2": 56, "s2b0.c2": 28, "s3b0.c2": 14, "s4b0.c2": 7,
            "s2b0.proj": 28, "s4b2.c3": 7}
    total = 0.0
    for l in W.resnet50_stack(1):
        d = B.make_desc(l)
        p, q = B.conv_out_shape(d)
        if l["name"] in want:
            assert (p, q) == (want[l["name"]],) * 2
        total += B.conv_flops(d)
    assert abs(total / 1e9 - 8.174) < 0.01
    for l in W.config3():
        assert abs(B.conv_flops(B.make_desc(l)) / 1e9 - 3.699) < 0.001


def test_error_codes():
    L = B.lib()
    good = d13(1, 4, 8, 8, 4, 3, 3, pd=(1, 1))
    assert L.wpk_conv_out_shape(None, None, None) == B.E_NULL_PTR
    for field, val in [("n", 0), ("c", -1), ("stride_h", 0), ("dil_w", 0), ("pad_h", -1), ("k", 0)]:
        bad = d13(1, 4, 8, 8, 4, 3, 3, pd=(1, 1))
        setattr(bad, field, val)
        assert L.wpk_conv_out_shape(ctypes.byref(bad), None, None) == B.E_BAD_DESC
    assert L.wpk_conv_out_shape(ctypes.byref(d13(1, 1, 2, 2, 1, 3, 3)), None, None) == B.E_BAD_DESC
    bad = d13(1, 4, 8, 8, 4, 3, 3)
    bad.dtype = 1
    assert L.wpk_conv_out_shape(ctypes.byref(bad), None, None) == B.E_UNSUPPORTED
    bad = d13(1, 4, 8, 8, 4, 3, 3)
    bad.layout = 4
    assert L.wpk_conv_out_shape(ctypes.byref(bad), None, None) == B.E_UNSUPPORTED
    for layout in (B.NCHW, B.X_NHWC, B.Y_NHWC, B.NHWC):
        ok = d13(1, 4, 8, 8, 4, 3, 3)
        ok.layout = layout
        assert L.wpk_conv_out_shape(ctypes.byref(ok), None, None) == 0
    # null tensors are rejected before anything touches the GPU
    assert L.wpk_conv2d_fwd(ctypes.byref(good), None, None, None, None) == B.E_NULL_PTR
    assert L.wpk_conv2d_ref(ctypes.byref(good), None, None, None, None) == B.E_NULL_PTR
    assert L.wpk_conv2d_fwd(None, None, None, None, None) == B.E_NULL_PTR
    assert B.conv_flops(bad) == 0.0
    for s in range(-8, 1):
        assert B.status_string(s) and "unknown" not in B.status_string(s)
    assert "unknown" in B.status_string(-99)


def test_config_encoding_roundtrip_and_constraint_check():
    lo, hi = B.config_gene_ranges()
    assert lo == [0] * 10 and hi == [3, 2, 2, 2, 2, 17, 1, 4, 2, 1]
    d = B.make_desc(W.config3()[1])
    legal = B.legal_configs(d)
    assert 3000 < len(legal) < 20000
    assert any(c.bm == 32 for c in legal)
    ids = set()
    for c in legal:
        cid = B.config_id(c)
        assert B.config_from_id(cid).astuple() == c.astuple()
        assert B.config_from_genes(B.config_to_genes(c)).astuple() == c.astuple()
        assert B.config_kernel_name(c) == "wpk_igemm_%dx%dx%d_%dx%d_p%d" % (c.bm, c.bn, c.bk, c.wm, c.wn, c.stages)
        # the constraints the header states
        assert 64 * c.wm * c.wn <= 1024
        if c.bm == 32:      # wave-split members: the waves cut the reduction, every wave holds the whole tile
            assert c.bk == 8 and c.persist == 0 and c.bn in (32, 64) and c.wm * c.wn in (1, 2, 4, 8)
            assert (c.wm * c.wn - 1) * 32 * c.bn * 4 <= 80 * 1024
        else:
            assert 2 * (c.bk + 4) * (c.bm + c.bn) * 4 <= 80 * 1024
            assert (c.bm // c.wm) % 32 == 0 and (c.bn // c.wn) % 32 == 0
        ids.add(cid)
    assert len(ids) == len(legal)
    assert not B.config_legal(d, B.make_config(128, 64, 16, 1, 1))          # not built
    assert not B.config_legal(d, B.make_config(100, 64, 16, 2, 2))          # not in the list
    tiny = d13(1, 1, 4, 4, 8, 1, 1)                                            # 1 reduction step
    assert not B.config_legal(tiny, B.make_config(128, 64, 16, 2, 2, split_k=2))
    assert B.config_legal(tiny, B.make_config(128, 64, 16, 2, 2, split_k=1))
    assert B.config_legal(d, B.make_config(128, 64, 16, 2, 2, persist=2))
    assert not B.config_legal(d, B.ConvConfig(128, 64, 16, 2, 2, 2, 0, 2, 2))   # persistent + split
    assert B.config_legal(d, B.ConvConfig(128, 64, 16, 2, 2, 1, 1, 2, 2))       # persistent: XCD-contiguous
    assert not B.config_legal(d, B.ConvConfig(128, 64, 16, 2, 2, 1, 0, 2, 2))   # ... and only so
    assert not B.config_legal(d, B.ConvConfig(128, 64, 16, 2, 2, 1, 1, 0, 4))   # stages not in list
    assert B.config_legal(d, B.make_config(128, 64, 16, 2, 2, split_k=3, reduce=1))
    assert B.config_legal(d, B.make_config(128, 64, 16, 2, 2, persist=2, reduce=1))
    assert not B.config_legal(d, B.make_config(128, 64, 16, 2, 2, reduce=1))   # nothing shared
    assert not B.config_legal(d, B.make_config(128, 64, 16, 2, 2, split_k=3, reduce=2))
    assert B.legal_configs(d13(1, 1, 20, 20, 8, 17, 2)) == []                  # > 16 filter rows
    assert B.legal_configs(d13(1, 1, 20, 20, 8, 2, 16)) == []                  # > 15 filter columns
    assert B.legal_configs(d13(1, 1, 20, 20, 8, 16, 15)) != []
    # channels-last x takes every K-step whatever C is (quads when C % 32 == 0, rows otherwise)
    for c_in in (3, 20, 24, 64):
        cl = B.make_desc(W.layer("cl", 1, c_in, 12, 20, 3, 1, 1), layout=B.NHWC)
        assert {c.bk for c in B.legal_configs(cl, split_k=[1], persist=[0])} == {8, 16, 32}
    with pytest.raises(B.WpkError):
        B.config_from_id(10 ** 9)
    with pytest.raises(B.WpkError):
        B.config_id(B.make_config(100, 64, 16, 2, 2))


def test_default_config_is_legal_for_every_workload_layer():
    layers = (W.config1() + W.config2() + W.config3() + W.config4() + W.resnet50_stack(1)
              + W.resnet50_stack(16) + W.table1_convs())
    for l in layers:
        d = B.make_desc(l)
        assert B.config_legal(d, B.config_default(d)), l["name"]


def test_default_config_schedules_by_tile_count():
    """The untuned rule: just over whole rounds of three workgroups per compute unit (784 tiles on 256
    compute units) -> three persistent workgroups; between one and two tiles per compute unit (392) ->
    one; fewer tiles than compute units -> the reduction split (host rule, no device needed: 256
    compute units assumed)."""
    c64, c128, c256, c512 = (B.config_default(B.make_desc(l)) for l in W.config3())
    assert (c64.persist, c64.split_k, c64.xcd_remap) == (3, 1, 1)
    assert (c128.persist, c128.split_k, c128.xcd_remap, c128.reduce) == (1, 1, 1, 0)
    assert c256.persist == 0 and c256.split_k > 1
    assert c512.persist == 0 and c512.split_k > 1


def test_cache_roundtrip_and_identity_criterion(tmp_path):
    B.cache_clear()
    a, b = W.config3()[0], W.config3()[1]
    da, db = B.make_desc(a), B.make_desc(b)
    assert B.cache_lookup(da) is None
    ca = B.make_config(128, 64, 16, 2, 2, 1, 0, 2)
    B.cache_store(da, ca, 12.5)
    assert B.cache_lookup(da).astuple() == ca.astuple()
    assert B.cache_lookup(db) is None
    # any differing field is a different operator
    for f in ("n", "pad_h", "dil_w", "stride_w", "k"):
        other = B.make_desc(a)
        setattr(other, f, getattr(other, f) + 1)
        if B.lib().wpk_conv_out_shape(ctypes.byref(other), None, None) == 0:
            assert B.cache_lookup(other) is None
    with pytest.raises(B.WpkError):
        B.cache_store(da, B.make_config(128, 64, 16, 1, 1))
    path = str(tmp_path / "cache.txt")
    B.cache_save(path)
    B.cache_clear()
    assert B.cache_size() == 0
    assert B.cache_load(path) == 1
    assert B.cache_lookup(da).astuple() == ca.astuple()
    with pytest.raises(B.WpkError):
        B.cache_load(str(tmp_path / "missing.txt"))
    B.cache_clear()


# ---- the search engine against the step-by-step oracle ------------------------------------------
LO, HI = [0, 0, 0, 0], [7, 5, 9, 3]


def fit_sep(ch):
    return 1.0 / (1.0 + sum((a - b) ** 2 for a, b in zip(ch, (5, 2, 7, 1))))


def fit_rugged(ch):
    a, b, c, d = ch
    return 1.0 / (10.0 + abs(a * b - 12) + 0.5 * abs(c - 2 * d) + ((a + c) % 3) * 0.7)


@pytest.mark.parametrize("seed", [0, 1, 7, 2008])
@pytest.mark.parametrize("fit,cons", [(fit_sep, None), (fit_rugged, lambda ch: sum(ch) % 2 == 0),
                                      (fit_rugged, lambda ch: ch[0] != ch[1])])
def test_engine_matches_oracle_generation_by_generation(seed, fit, cons):
    kw = dict(pop=16, elites=3, next_pop=12, participants=10, pm=0.2, eps=0.01, patience=4,
              max_gen=9)
    ref = oga.genetic_search(LO, HI, cons or (lambda ch: True), fit, seed=seed, retries=8, **kw)
    opt = B.tune_default_options(population=16, elites=3, next_population=12, participants=10,
                                 mutation=0.2, eps=0.01, patience=4, max_generations=9, seed=seed)
    got = B.ga_search(LO, HI, cons, fit, opt, history_capacity=9)
    assert got["generations"] == len(ref["history"])
    assert got["history"] == ref["history"]            # same chromosomes, same fitness, bit for bit
    assert got["best"] == ref["best"]
    assert got["best_fitness"] == ref["best_fitness"]
    assert got["evaluations"] == ref["evaluations"]


def test_engine_default_sizes_and_flat_fitness():
    opt = B.tune_default_options(seed=3)
    ref = oga.genetic_search(LO, HI, lambda ch: True, fit_sep, seed=3, pop=64, elites=8, pm=0.15,
                             eps=0.03, patience=5, max_gen=16)
    got = B.ga_search(LO, HI, None, fit_sep, opt, history_capacity=16)
    assert got["history"] == ref["history"]
    flat = B.ga_search(LO, HI, None, lambda ch: 2.0, opt, history_capacity=16)
    assert flat["generations"] == 1


def test_engine_random_mode_and_bad_arguments():
    opt = B.tune_default_options(seed=5, mode=1, max_generations=5, patience=0, eps=0.0)
    got = B.ga_search(LO, HI, None, fit_sep, opt, history_capacity=5)
    assert got["generations"] == 5
    assert all(len(p) == 64 for p, _ in got["history"])
    with pytest.raises(B.WpkError):
        B.ga_search([0, 3], [1, 2], None, fit_sep)       # empty gene range
    with pytest.raises(B.WpkError):
        B.ga_search([0], [3], lambda ch: False, lambda ch: 1.0)   # nothing is legal


def test_workspace_limit_argument_check():
    L = B.lib()
    assert L.wpk_set_workspace_limit(-1) == B.E_BAD_ARG
    assert L.wpk_set_workspace_limit(1 << 30) == 0


def test_workspace_slots_cover_every_sharer_of_a_tile():
    """The kernel indexes a shared tile's slots by the position of a workgroup among the tile's
    sharers.  Re-derive the sharers from the schedule's definition (persistent: the steps of the
    tiles beyond the last whole round, laid end to end and cut into runs of q or q+1, one for each
    of the first min(G, units / max(1, 64 / BK)) workgroups; split:
    the non-empty slices) and check that the slot count the host reserves is never too small."""
    rng = np.random.default_rng(5)
    checked = 0
    for _ in range(300):
        n, c, hw, k = int(rng.integers(1, 9)), int(rng.integers(1, 200)), int(rng.integers(3, 40)), int(rng.integers(1, 300))
        rs = int(rng.choice([1, 3, 5]))
        d = B.make_desc(W.layer("w", n, c, hw, k, rs, 1, rs // 2))
        P, Q = B.conv_out_shape(d)
        cus = int(rng.choice([8, 64, 256, 304]))
        for cfg in (B.make_config(64, 32, 8, 2, 1, persist=int(rng.integers(1, 5))),
                    B.make_config(128, 64, 16, 2, 2, persist=int(rng.integers(1, 5))),
                    B.make_config(64, 64, 32, 2, 2, split_k=int(rng.choice([2, 3, 5, 7, 11, 16, 24])))):
            if not B.config_legal(d, cfg):
                continue
            nbytes, shared, slots = B.config_workspace(d, cfg, cus)
            tiles = -(-n * P * Q // cfg.bm) * -(-k // cfg.bn)
            nsteps = -(-c * rs * rs // cfg.bk)
            if cfg.persist == 0:
                per = -(-nsteps // cfg.split_k)
                want_shared, want_slots = tiles, -(-nsteps // per)
                if want_slots <= 1:
                    want_shared = want_slots = 0
            else:
                G = cfg.persist * cus
                rest = tiles - tiles // G * G
                units = rest * nsteps
                groups = min(G, max(1, units // max(1, 64 // cfg.bk))) if units else 0   # runs of >= 64 rows
                q, rem = divmod(units, groups) if groups else (0, 0)
                start = lambda g: g * q + min(g, rem)
                owners = [0] * rest
                for g in range(groups):       # every run marks the tiles it touches
                    u0, u1 = start(g), start(g + 1)
                    if u1 > u0:
                        for j in range(u0 // nsteps, (u1 - 1) // nsteps + 1):
                            owners[j] += 1
                want_shared = rest if rest and nsteps > 1 else 0
                want_slots = max(owners) if want_shared else 0
            if nbytes == 0:
                assert want_shared == 0 or want_slots <= 1 or shared == 0
                continue
            assert shared == want_shared
            assert slots >= want_slots, (cfg, cus, tiles, nsteps, slots, want_slots)
            assert nbytes == (1 << 20) + shared * slots * cfg.bm * cfg.bn * 4
            checked += 1
    assert checked > 100


def test_fast_division_by_launch_constants(tmp_path):
    """The kernels divide by launch constants with a host-computed multiplier, an add and a shift;
    the quotient must be exact for every dividend below 2^31 and every divisor from 1 up.  Compiled from the library's own
    header and checked against the plain quotient: every small pair, then edge and random ones."""
    src = tmp_path / "fdiv.cpp"
    src.write_text(r'''
#include <cstdio>
#include <cstdint>
#include <string>
#include <vector>
#include "wpk_internal.h"
static uint32_t q(uint32_t n, const wpk::FastDiv &f)
{
    return ((uint32_t)(((uint64_t)n * f.mul) >> 32) + n) >> f.sh;
}
int main()
{
    uint64_t state = 12345, bad = 0, checked = 0;
    auto rnd = [&]() { state = state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(state >> 33); };
    for (uint32_t d = 1; d <= 3000; ++d) {
        wpk::FastDiv f = wpk::make_fastdiv(d);
        for (uint32_t n = 0; n <= 6000; ++n, ++checked) bad += q(n, f) != n / d;
        for (uint32_t n : {0x7fffffffu, 0x7ffffffeu, 0x40000000u, d * 715827u, d * 715827u - 1})
            if (n < 0x80000000u) { bad += q(n, f) != n / d; ++checked; }
    }
    for (int i = 0; i < 2000000; ++i, ++checked) {
        uint32_t d = rnd() % 0x7fffffffu + 1, n = rnd() & 0x7fffffffu;
        if (i & 1) d = d % 100000 + 1;
        bad += q(n, wpk::make_fastdiv(d)) != n / d;
    }
    printf("%llu %llu\n", (unsigned long long)checked, (unsigned long long)bad);
    return 0;
}
''')
    exe = tmp_path / "fdiv"
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    subprocess.run(["g++", "-O1", "-std=c++17", "-I", os.path.join(root, "include"),
                    "-I", os.path.join(root, "paper_2008_04567_amd", "csrc"), str(src), "-o", str(exe)], check=True)
    checked, bad = [int(v) for v in subprocess.run([str(exe)], check=True, capture_output=True,
                                                   text=True).stdout.split()]
    assert checked > 10 ** 7 and bad == 0
