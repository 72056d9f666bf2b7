"""Genetic search next to random search and to exhaustive enumeration, per layer shape
(Section 3.2 compares the searches by the speed of the operator they find; Section 3.3 reports
the search time).

For every distinct layer of a workload: one exhaustive pass over the legal points of the
kernel family gives the fastest member; then, for several seeds, the genetic search (Section 2.3,
Steps 1-4) and a random search that draws a fresh legal generation each time run the same number
of generations of the same size, both without the refinement stage and without early stopping.
Printed per layer: points enumerated, the fastest time, and per search the mean and worst ratio
"found / fastest", how often the search came within 3 % of the fastest, candidates timed and
wall seconds.  Timing noise between two measurements of one candidate is about 1-2 %.

    python -m paper_2008_04567_amd.search_report --workload config3 --seeds 5
"""
import argparse
import sys

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="config3",
                    help="config2|config3|config4|table1|resnet18_n1|resnet50_n1|resnet50_n16")
    ap.add_argument("--seeds", type=int, default=5)
    ap.add_argument("--generations", type=int, default=12)
    ap.add_argument("--population", type=int, default=64)
    ap.add_argument("--max-layers", type=int, default=0, help="only the first so many distinct layers")
    args = ap.parse_args()

    import torch
    from . import binding as B
    from . import workloads as W

    assert torch.cuda.is_available(), "the search report times kernels: it needs a GPU"
    sets = {"config2": W.config2, "config3": W.config3, "config4": W.config4,
            "table1": W.table1_convs, "resnet18_n1": lambda: W.resnet18_stack(1),
            "resnet50_n1": lambda: W.resnet50_stack(1), "resnet50_n16": lambda: W.resnet50_stack(16)}
    layers = W.unique_layers(sets[args.workload]())
    if args.max_layers:
        layers = layers[:args.max_layers]
    name, cus = B.device_info()
    print("# search comparison: workload %s on %s (%d CUs); %d generations of %d, %d seeds"
          % (args.workload, name, cus, args.generations, args.population, args.seeds))
    print()
    print("| layer | legal points | fastest us | exhaustive s | search | found/fastest mean | worst "
          "| within 3 % | candidates timed | seconds |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    summary = {"genetic": [], "random": []}
    for l in layers:
        d = B.make_desc(l)
        _, ex = B.conv_tune_ex(d, B.tune_default_options(mode=2, refine=0), force=True)
        for label, mode in (("genetic", 0), ("random", 1)):
            ratios, evals, secs = [], [], []
            for s in range(args.seeds):
                opt = B.tune_default_options(mode=mode, refine=0, seed=1000 + s, patience=0, eps=0.0,
                                             max_generations=args.generations,
                                             elites=max(1, args.population // 8),
                                             population=args.population,
                                             next_population=args.population,
                                             participants=args.population)
                _, rep = B.conv_tune_ex(d, opt, force=True)
                ratios.append(rep.best_us / ex.best_us)
                evals.append(rep.evaluations)
                secs.append(rep.seconds)
            summary[label] += ratios
            print("| %s | %d | %.2f | %.1f | %s | %.3f | %.3f | %d/%d | %.0f | %.2f |"
                  % (l["name"], ex.evaluations, ex.best_us, ex.seconds, label, np.mean(ratios),
                     np.max(ratios), sum(r <= 1.03 for r in ratios), len(ratios), np.mean(evals),
                     np.mean(secs)))
            sys.stdout.flush()
    print()
    for label in ("genetic", "random"):
        r = np.array(summary[label])
        print("%s search over all layers and seeds: found/fastest mean %.3f, median %.3f, worst %.3f, "
              "within 3 %% in %d of %d" % (label, r.mean(), np.median(r), r.max(), (r <= 1.03).sum(), r.size))


if __name__ == "__main__":
    main()
