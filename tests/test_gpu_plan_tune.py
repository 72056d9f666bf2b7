"""GPU tests of plans and of the on-device tuner."""
import numpy as np
import pytest

from oracle import conv as oc
from paper_2008_04567_amd import binding as B
from paper_2008_04567_amd import workloads as W
from tests import parity as PT

pytestmark = pytest.mark.gpu


def sampled_check(layer, x, w, y_gpu, count=400, seed=0):
    """Oracle values for a sample of outputs, computed one by one."""
    sh = oc.shape_from_layer(layer)
    total = int(np.prod(y_gpu.shape))
    idx = np.random.default_rng(seed).integers(0, total, size=min(count, total))
    idx = np.unique(np.concatenate([idx, [0, total - 1]]))
    y_ref, d_ref = oc.conv2d_sampled(sh, x, w, idx)
    return PT.assert_close(y_gpu.reshape(-1)[idx], y_ref, d_ref, layer["name"])


@pytest.mark.parametrize("n", [1, 2])
def test_plan_resnet50_stack(n):
    torch, dev = PT.torch_dev()
    layers = W.resnet50_stack(n)
    descs = [B.make_desc(l) for l in layers]
    plan = B.Plan(descs, tune=False)
    assert plan.num_layers() == 53 and plan.num_unique() == 23
    xs, ws, ys, host = [], [], [], []
    for i, l in enumerate(layers):
        x, w = W.make_inputs(l)
        host.append((x, w))
        P, Q = B.conv_out_shape(descs[i])
        xs.append(PT.to_dev(x))
        ws.append(PT.to_dev(w))
        ys.append(torch.full((l["n"], l["k"], P, Q), 777.0, device=dev, dtype=torch.float32))
        plan.set_weights(i, ws[-1])
    xa, ya = plan.pointer_arrays(xs, ys)
    plan.run(xa, ya)
    torch.cuda.synchronize()
    for i, l in enumerate(layers):
        print(l["name"], plan.layer_config(i), flush=True)
        sampled_check(l, host[i][0], host[i][1], ys[i].cpu().numpy(), seed=i)
    # a second run after changing one layer's weights picks the new weights up
    w_new = (2.0 * host[5][1]).astype(np.float32)
    plan.set_weights(5, PT.to_dev(w_new))
    plan.run(xa, ya)
    torch.cuda.synchronize()
    sampled_check(layers[5], host[5][0], w_new, ys[5].cpu().numpy())
    plan.destroy()


def test_plan_requires_weights():
    torch, dev = PT.torch_dev()
    l = W.config1()[0]
    plan = B.Plan([B.make_desc(l)])
    t = torch.zeros(16 * 14 * 14, device=dev)
    with pytest.raises(B.WpkError):
        plan.run_layer(0, t, t)
    plan.destroy()


def test_tuner_small_budget_result_is_legal_cached_and_correct():
    B.cache_clear()
    l = W.config2()[0]
    desc = B.make_desc(l)
    opt = B.tune_default_options(population=10, elites=2, next_population=10, participants=10,
                                 max_generations=3, reps=3, min_group_us=100.0, seed=1)
    cid, rep = B.conv_tune_ex(desc, opt, force=True)
    cfg = B.config_from_id(cid)
    print("tuned", cfg, rep.best_us, rep.default_us, rep.evaluations, rep.generations,
          rep.rejected, rep.seconds, flush=True)
    assert B.config_legal(desc, cfg)
    assert rep.rejected == 0
    assert 0 < rep.best_us <= rep.default_us * 1.0001
    assert rep.evaluations >= 10 and 1 <= rep.generations <= 3
    assert B.cache_lookup(desc).astuple() == cfg.astuple()
    assert B.conv_tune(desc) == cid                      # cache hit returns at once
    PT.check_layer(l)                                    # one-shot path now runs the tuned config
    B.cache_clear()
