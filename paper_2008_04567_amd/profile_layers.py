"""Launch the layers of a workload one after another, a fixed number of times each, for a profiler.

    rocprofv3 --kernel-trace --stats -- python3 -m paper_2008_04567_amd.profile_layers \
        --workload config3 --cache tuned.cache --reps 20 --manifest order.json

``--config LAYER=...`` pins a layer's configuration.  With ``--cache`` the layers run under the
configurations a search stored there (``--tune`` searches
the missing ones first and saves them: do that in a run of its own, outside the profiler); without
it under the library's defaults.  The manifest lists the convolution launches in order -- layer,
configuration, kernel name, grid size, algorithmic bytes and FLOPs -- so that a per-dispatch
counter file can be read layer by layer: the n-th dispatch of a convolution kernel (``igemm_kernel``,
``wsplit_kernel`` or the direct kernel) belongs to the n-th manifest entry.  ``--calibrate-copy`` appends three device copies of 256 MiB, whose
byte counters give the scale of FETCH_SIZE / WRITE_SIZE.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def workload(W, name):
    table = {"config1": W.config1, "config2": W.config2, "config3": W.config3, "config4": W.config4,
             "resnet50_n1": lambda: W.resnet50_stack(1), "resnet50_n16": lambda: W.resnet50_stack(16),
             "resnet18_n1": lambda: W.resnet18_stack(1), "table1": W.table1_convs}
    if name not in table:
        raise SystemExit("unknown workload " + name)
    return table[name]()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="config3")
    ap.add_argument("--cache", default=None)
    ap.add_argument("--tune", action="store_true", help="search layers the cache does not hold, then save it")
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--warm", type=int, default=2, help="launches per layer before the counted ones (also listed)")
    ap.add_argument("--unique", action="store_true", help="each distinct shape once")
    ap.add_argument("--layout", default="nchw", choices=["nchw", "nhwc"])
    ap.add_argument("--config", action="append", default=[], metavar="LAYER=bm,bn,bk,wm,wn,split,remap,persist,stages,reduce",
                    help="run the named layer under this configuration instead (may be repeated)")
    ap.add_argument("--sweep", default=None, metavar="FILE",
                    help="text file of lines 'LAYER bm,bn,bk,wm,wn,split,remap,persist,stages,reduce': run exactly "
                         "these (layer, configuration) pairs, in the file's order, instead of every layer once")
    ap.add_argument("--manifest", default=None)
    ap.add_argument("--calibrate-copy", action="store_true")
    args = ap.parse_args()

    import torch
    from paper_2008_04567_amd import binding as B
    from paper_2008_04567_amd import workloads as W

    assert torch.cuda.is_available(), "needs a GPU"
    dev = torch.device("cuda:0")
    layout = B.NHWC if args.layout == "nhwc" else B.NCHW
    layers = workload(W, args.workload)
    if args.unique:
        layers = W.unique_layers(layers)
    descs = [B.make_desc(l, layout=layout) for l in layers]
    if args.cache and os.path.exists(args.cache):
        B.cache_load(args.cache)
    if args.tune:
        opt = B.tune_default_options(zero_ahead=1)
        for d in descs:
            try:
                B.conv_tune_ex(d, opt, force=False)
            except B.WpkError as e:
                if e.status != B.E_UNSUPPORTED:
                    raise
        if args.cache:
            B.cache_save(args.cache)
    plan = B.Plan(descs, tune=False)
    forced = dict(c.split("=", 1) for c in args.config)
    for i, l in enumerate(layers):
        if l["name"] in forced:
            plan.set_layer_config(i, B.ConvConfig(*[int(v) for v in forced[l["name"]].split(",")]))
    stream = torch.cuda.current_stream()
    order = []
    runs = [(i, None) for i in range(len(layers))]
    if args.sweep:
        index = {l["name"]: i for i, l in enumerate(layers)}
        runs = []
        for line in open(args.sweep):
            t = line.split()
            if len(t) == 2 and not line.startswith("#"):
                cfg = B.ConvConfig(*[int(v) for v in t[1].split(",")])
                if B.config_legal(descs[index[t[0]]], cfg):
                    runs.append((index[t[0]], cfg))
    operands = {}
    for i, pinned in runs:
        l, d = layers[i], descs[i]
        if i not in operands:
            operands.clear()                 # one layer's tensors at a time
            x, w = W.make_inputs(l)
            if layout & 1:
                x = x.transpose(0, 2, 3, 1).copy()
            P, Q = B.conv_out_shape(d)
            operands[i] = (torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev),
                           torch.empty(l["n"] * l["k"] * P * Q, device=dev, dtype=torch.float32), x.size, w.size)
            plan.set_weights(i, operands[i][1])
        xd, wd, yd, nx, nw = operands[i]
        if pinned is not None:
            plan.set_layer_config(i, pinned)
        torch.cuda.synchronize()
        cfg = plan.layer_config(i)
        for rep in range(args.warm + args.reps):
            plan.run_layer(i, xd, yd, stream)
            order.append({"layer": l["name"], "counted": rep >= args.warm, "config_id": B.config_id(cfg),
                          "config": cfg.asdict(), "kernel": B.config_kernel_name(cfg),
                          "flops": B.conv_flops(d),
                          "bytes_read": 4 * (nx + nw), "bytes_written": 4 * yd.numel()})
        torch.cuda.synchronize()
    operands.clear()
    if args.calibrate_copy:
        src = torch.zeros(64 << 20, device=dev, dtype=torch.float32)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    plan.destroy()
    if args.manifest:
        with open(args.manifest, "w") as f:
            json.dump({"workload": args.workload, "launches": order}, f)
    print("launched %d convolutions of %d layers" % (len(order), len(layers)))


if __name__ == "__main__":
    main()
