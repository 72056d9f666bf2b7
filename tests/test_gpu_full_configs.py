"""GPU parity at the full sizes of the benchmark configurations, in the launch configurations the
benchmark times: the ResNet-50 stack at N=16 (every layer, sampled outputs), a plan that tunes its
own layers, a full-size layer under a searched (cached) configuration, and a pipelined pass on
buffers that tensors of different sizes reuse in turns."""
import numpy as np
import pytest

from oracle import conv as oc
from paper_2008_04567_amd import binding as B
from paper_2008_04567_amd import workloads as W
from tests import parity as PT

pytestmark = pytest.mark.gpu


def sampled(layer, x, w, y_gpu, count, seed):
    """Oracle values of `count` outputs drawn uniformly, plus the first and the last and the corners
    of the first and last image's last channel, computed one by one."""
    sh = oc.shape_from_layer(layer)
    total = int(np.prod(y_gpu.shape))
    pq = y_gpu.shape[2] * y_gpu.shape[3]
    fixed = [0, total - 1, pq - 1, total - pq, total // 2]
    idx = np.random.default_rng(seed).integers(0, total, size=min(count, total))
    idx = np.unique(np.concatenate([idx, fixed]))
    y_ref, d_ref = oc.conv2d_sampled(sh, x, w, idx)
    return PT.assert_close(y_gpu.reshape(-1)[idx], y_ref, d_ref, layer["name"])


def test_resnet50_stack_n16_every_layer_sampled():
    """Config 5 at N=16 through a plan: all 53 layers (23 distinct shapes), 4096 sampled outputs
    each, full batch, in the configurations a plan built without a search uses."""
    torch, dev = PT.torch_dev()
    layers = W.resnet50_stack(16)
    descs = [B.make_desc(l) for l in layers]
    plan = B.Plan(descs, tune=False)
    assert plan.num_layers() == 53 and plan.num_unique() == 23
    # distinct shapes share one set of operands: 23 input tensors instead of 53 (0.4 GB, not 0.8)
    by_shape, xs, ys = {}, [], []
    for i, l in enumerate(layers):
        key = W.shape_key(l)
        if key not in by_shape:
            x, w = W.make_inputs(l)
            by_shape[key] = (x, w, PT.to_dev(x), PT.to_dev(w))
        x, w, xd, wd = by_shape[key]
        P, Q = B.conv_out_shape(descs[i])
        xs.append(xd)
        ys.append(torch.full((l["n"], l["k"], P, Q), 777.0, device=dev, dtype=torch.float32))
        plan.set_weights(i, wd)
    xa, ya = plan.pointer_arrays(xs, ys)
    plan.run(xa, ya)
    torch.cuda.synchronize()
    worst = 0.0
    for i, l in enumerate(layers):
        x, w = by_shape[W.shape_key(l)][:2]
        worst = max(worst, sampled(l, x, w, ys[i].cpu().numpy(), 4096, seed=i))
    print("ResNet-50 N=16: worst normalised error over 53 layers %.3g" % worst, flush=True)
    plan.destroy()


def test_plan_that_tunes_its_own_layers():
    """wpk_conv_plan with tune = 1: every distinct descriptor is searched when the plan is built, the
    winners land in the cache, and the plan's outputs under those winners equal the oracle."""
    torch, dev = PT.torch_dev()
    B.cache_clear()
    layers = [W.layer("pt.a", 2, 24, (30, 26), 48, 3, 1, 1, x_dist="u11", seed=301),
              W.layer("pt.b", 2, 48, (30, 26), 24, 1, 1, 0, x_dist="u11", seed=302),
              W.layer("pt.c", 2, 24, (30, 26), 48, 3, 1, 1, x_dist="u11", seed=303)]
    descs = [B.make_desc(l) for l in layers]
    plan = B.Plan(descs, tune=True)
    assert plan.num_layers() == 3 and plan.num_unique() == 2
    assert B.cache_size() == 2
    for i, d in enumerate(descs):
        cached = B.cache_lookup(d)
        assert cached is not None and B.config_legal(d, cached)
        assert plan.layer_config(i).astuple() == cached.astuple()
        print(layers[i]["name"], cached, flush=True)
    x0, _ = W.make_inputs(layers[0])
    ws = [W.make_inputs(l)[1] for l in layers]
    for i, w in enumerate(ws):
        plan.set_weights(i, PT.to_dev(w))
    xd = PT.to_dev(x0)
    ys = [torch.full((2, l["k"], 30, 26), 777.0, device=dev) for l in layers]
    xa, ya = plan.pointer_arrays([xd, ys[0], ys[1]], ys)
    plan.run(xa, ya)
    torch.cuda.synchronize()
    h = [y.cpu().numpy() for y in ys]
    ins = [x0, h[0], h[1]]          # later layers are held to the oracle on the device's own inputs
    for i, l in enumerate(layers):
        r, d, _ = oc.conv2d(oc.shape_from_layer(l), ins[i], ws[i])
        PT.assert_close(h[i], r, d, "tuned plan layer %d" % i)
    plan.destroy()
    B.cache_clear()


@pytest.mark.parametrize("which", [1, 3])
def test_full_size_config3_layer_under_a_searched_configuration(which):
    """The benchmark times searched configurations, not defaults: search one config-3 layer (the
    genetic search with the additions the benchmark leaves on, smaller budget), then hold the whole
    output tensor under the cached winner to the oracle."""
    B.cache_clear()
    l = W.config3()[which]
    desc = B.make_desc(l)
    opt = B.tune_default_options(population=24, elites=4, next_population=24, participants=24,
                                 max_generations=4, reps=3, zero_ahead=1, seed=5)
    cid, rep = B.conv_tune_ex(desc, opt, force=True)
    cfg = B.config_from_id(cid)
    print(l["name"], "searched:", cfg, "%.1f us (default %.1f us), stage %s, search alone %.1f us"
          % (rep.best_us, rep.default_us, rep.stage_name, rep.search_us), flush=True)
    assert rep.rejected == 0 and rep.search_us > 0 and rep.best_us <= rep.search_us * 1.10
    assert B.cache_lookup(desc).astuple() == cfg.astuple()
    x, w = W.make_inputs(l)
    y_ref, d_ref = PT.oracle_full(l, x, w)
    PT.assert_close(PT.run_gpu(l, x, w, cfg=cfg), y_ref, d_ref, l["name"] + " searched config, one-shot")
    # and through a plan, which picks the cached configuration up by itself
    torch, dev = PT.torch_dev()
    plan = B.Plan([desc], tune=False)
    assert plan.layer_config(0).astuple() == cfg.astuple()
    plan.set_weights(0, PT.to_dev(w))
    yd = torch.full(y_ref.shape, 777.0, device=dev, dtype=torch.float32)
    plan.run_layer(0, PT.to_dev(x), yd)
    torch.cuda.synchronize()
    PT.assert_close(yd.cpu().numpy(), y_ref, d_ref, l["name"] + " searched config, plan")
    plan.destroy()
    B.cache_clear()


def test_pipelined_pass_on_reused_buffers_of_different_sizes():
    """Two-way pipelining with ResNet-style ping-pong buffers: P holds a wide tensor (N x 48 x HW),
    later a narrow one (N x 16 x HW).  The second half of the narrow tensor starts inside the first
    half of the wide one, so the two half-batch chains cannot run unordered; the pass must notice
    and still give the unsplit result.  On separate buffers the same plan does split."""
    torch, dev = PT.torch_dev()
    n, hw = 4, (12, 10)
    layers = [W.layer("pp.a", n, 16, hw, 48, 1, 1, 0, x_dist="u11", seed=311),   # X -> P (wide)
              W.layer("pp.b", n, 48, hw, 16, 3, 1, 1, x_dist="u11", seed=312),   # P -> Q (narrow)
              W.layer("pp.c", n, 16, hw, 16, 3, 1, 1, x_dist="u11", seed=313),   # Q -> P (narrow, reuses P)
              W.layer("pp.d", n, 16, hw, 48, 1, 1, 0, x_dist="u11", seed=314)]   # P -> Q (wide, reuses Q)
    descs = [B.make_desc(l) for l in layers]
    plan = B.Plan(descs, tune=False)
    x0, _ = W.make_inputs(layers[0])
    ws = [W.make_inputs(l)[1] for l in layers]
    for i, w in enumerate(ws):
        plan.set_weights(i, PT.to_dev(w))
    wide = n * 48 * hw[0] * hw[1]
    xd = PT.to_dev(x0)
    p_ = torch.full((wide,), 555.0, device=dev)
    q_ = torch.full((wide,), 555.0, device=dev)
    xa, ya = plan.pointer_arrays([xd, p_, q_, p_], [p_, q_, p_, q_])

    def run_and_collect(ways):
        plan.set_pipeline(ways)
        p_.fill_(555.0)
        q_.fill_(555.0)
        for _ in range(3):
            plan.run(xa, ya)
        torch.cuda.synchronize()
        return q_.cpu().numpy()[:wide].reshape(n, 48, hw[0], hw[1]).copy()

    one = run_and_collect(1)
    two = run_and_collect(2)
    # The same chain layer by layer: each layer is held to the oracle on the device's own input, and
    # the input of the last layer is kept for the expected value of the whole passes above.
    plan.set_pipeline(1)
    bufs = [(xd, p_), (p_, q_), (q_, p_), (p_, q_)]
    inter = [x0]
    for i, l in enumerate(layers):
        plan.run_layer(i, bufs[i][0], bufs[i][1])
        torch.cuda.synchronize()
        P, Q = B.conv_out_shape(descs[i])
        got = bufs[i][1].cpu().numpy()[:n * l["k"] * P * Q].reshape(n, l["k"], P, Q).copy()
        r, d, _ = oc.conv2d(oc.shape_from_layer(l), inter[i], ws[i])
        PT.assert_close(got, r, d, "layer by layer %d" % i)
        inter.append(got)
    # (the 3x3 layers split their reduction, so sums come in arrival order: the oracle bound, not
    # bit equality, is what the whole passes are held to, on the last layer's device input)
    r, d, _ = oc.conv2d(oc.shape_from_layer(layers[3]), inter[3], ws[3])
    PT.assert_close(one, r, d, "one chain, reused buffers")
    PT.assert_close(two, r, d, "two chains asked for, reused buffers")
    # separate buffers: the split pass is taken and agrees as well
    sep = [torch.full((wide,), 555.0, device=dev) for _ in range(4)]
    xs = [xd, sep[0], sep[1], sep[2]]
    xa2, ya2 = plan.pointer_arrays(xs, sep)
    plan.set_pipeline(2)
    plan.run(xa2, ya2)
    torch.cuda.synchronize()
    a = x0
    for i, l in enumerate(layers):
        P, Q = B.conv_out_shape(descs[i])
        got = sep[i].cpu().numpy()[:n * l["k"] * P * Q].reshape(n, l["k"], P, Q)
        r, d, _ = oc.conv2d(oc.shape_from_layer(l), a, ws[i])
        PT.assert_close(got, r, d, "two chains, separate buffers, layer %d" % i)
        a = got.copy()
    plan.destroy()


def _run_graph_plan(layers, x_t, y_t, r_t, fixed, tune=False):
    """Build a plan that chooses its tensors' layouts, run the chain, return (plan facts, outputs in
    [N][K][P][Q] order) -- and hold every layer to the oracle on the device's own input tensor."""
    torch, dev = PT.torch_dev()
    descs = [B.make_desc(l) for l in layers]
    plan = B.Plan(descs, tune=tune, graph=(x_t, y_t, r_t, fixed))
    nt = len(fixed)
    lay = [plan.tensor_layout(t) for t in range(nt)]
    for i in range(len(layers)):
        assert plan.layer_layout(i) == lay[x_t[i]] | (lay[y_t[i]] << 1)
    assert all(f < 0 or f == v for f, v in zip(fixed, lay))
    x0, _ = W.make_inputs(layers[0])
    ws = [W.make_inputs(l)[1] for l in layers]
    for i, w in enumerate(ws):
        plan.set_weights(i, PT.to_dev(w))
        plan.set_epilogue(i, None, relu=True)
    # tensor t as the device holds it (in its chosen layout) and as [N][C][H][W] on the host
    shape = {x_t[0]: x0.shape}
    for i, l in enumerate(layers):
        P, Q = B.conv_out_shape(descs[i])
        shape[y_t[i]] = (l["n"], l["k"], P, Q)
    to_layout = lambda a, cl: np.ascontiguousarray(a.transpose(0, 2, 3, 1)) if cl else a
    dev_t = {t: torch.full((int(np.prod(s)),), 777.0, device=dev) for t, s in shape.items()}
    dev_t[x_t[0]].copy_(torch.from_numpy(to_layout(x0, lay[x_t[0]]).reshape(-1)))
    xs = [dev_t[x_t[i]] for i in range(len(layers))]
    ys = [dev_t[y_t[i]] for i in range(len(layers))]
    rs = [dev_t[r_t[i]] if r_t is not None and r_t[i] >= 0 else None for i in range(len(layers))]
    xa, ya = plan.pointer_arrays(xs, ys)
    plan.run_fused(xa, plan.residual_array(rs), ya)
    torch.cuda.synchronize()
    host = {t: dev_t[t].cpu().numpy() for t in dev_t}     # flat, in the chosen layouts
    names = ("NCHW", "NHWC")
    for i, l in enumerate(layers):
        n, k, P, Q = shape[y_t[i]]
        res = host[r_t[i]] if r_t is not None and r_t[i] >= 0 else None
        y_ref, d_ref = oc.conv2d_fused(oc.shape_from_layer(l), host[x_t[i]], ws[i], residual=res, relu=True,
                                       x_layout=names[lay[x_t[i]]], y_layout=names[lay[y_t[i]]])
        PT.assert_close(host[y_t[i]], y_ref, d_ref, "graph plan layer %d (layout code %d)" % (i, plan.layer_layout(i)))
    plan.destroy()
    return lay


def test_plan_chooses_the_layouts_of_inner_tensors():
    """wpk_conv_plan_graph on a three-layer chain whose ends are fixed [N][C][H][W].  (a) With stored
    runtimes that make the channels-last forms cheaper, both inner tensors move to channels-last: the
    first layer transforms on its way out, the last on its way in, and every layer still equals the
    oracle in the layouts chosen.  (b) A residual that ties the first inner tensor to the fixed
    output keeps that tensor [N][C][H][W].  (c) Without stored runtimes the plan times the defaults
    itself; whatever it picks must be consistent and correct."""
    layers = [W.layer("lg.a", 2, 32, (14, 12), 32, 3, 1, 1, x_dist="u11", seed=321),
              W.layer("lg.b", 2, 32, (14, 12), 32, 1, 1, 0, x_dist="u11", seed=322),
              W.layer("lg.c", 2, 32, (14, 12), 32, 3, 1, 1, x_dist="u11", seed=323)]
    x_t, y_t, fixed = [0, 1, 2], [1, 2, 3], [0, -1, -1, 0]
    B.device_info()                    # cache keys carry the device's name: look at the device first
    B.cache_clear()
    for l in layers:                   # stored runtimes: every channels-last side takes 3 us off
        for code in range(4):
            d = B.make_desc(l, layout=code)
            B.cache_store(d, B.config_default(d), us=20.0 - 3.0 * bin(code).count("1"))
    assert _run_graph_plan(layers, x_t, y_t, None, fixed) == [0, 1, 1, 0]
    assert _run_graph_plan(layers, x_t, y_t, [-1, -1, 1], fixed) == [0, 0, 1, 0]
    B.cache_clear()
    lay = _run_graph_plan(layers, x_t, y_t, None, fixed)
    print("layouts chosen from timed defaults:", lay, flush=True)
    assert B.cache_size() == 0         # timing the defaults stores nothing
    B.cache_clear()
