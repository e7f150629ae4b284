"""Point discovery through libnova from the command line: the evolution strategy of Sec. "Evolution
Strategy" with the paper's hyper-parameters (population 50, 100 generations, 3 restarts), then
snap-to-rational with the neighbourhood search, for a number of seeds; and the exhaustive symmetric
search beside it.  Prints what each run found, and per tile the mean / std / min / max of kappa(V)
in the layout of Table "ES reproducibility across 5 random seeds".

    python -m paper_2512_18453_amd.discover [--m 4 6 8] [--r 3] [--seeds 5] [--d-max 10]

The standard normal draws the strategy consumes come from numpy's default_rng(seed) and are
passed to the library as an argument; all arithmetic is the library's.
"""
import argparse
import time

import numpy as np

from . import nova


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--m", type=int, nargs="+", default=[4, 6, 8])
    ap.add_argument("--r", type=int, default=3)
    ap.add_argument("--seeds", type=int, default=5)
    ap.add_argument("--d-max", type=int, default=10)
    ap.add_argument("--generations", type=int, default=100)
    ap.add_argument("--population", type=int, default=50)
    ap.add_argument("--restarts", type=int, default=3)
    args = ap.parse_args()
    for m in args.m:
        print(f"F({m},{args.r}): evolution strategy, population {args.population}, {args.generations} generations, "
              f"{args.restarts} restarts, snapped with d_max = {args.d_max}")
        kappas = []
        for seed in range(args.seeds):
            count = nova.nova_es_normals_needed(m, args.r, args.generations, args.population, args.restarts)
            z = np.random.default_rng(seed).standard_normal(count)
            tic = time.perf_counter()
            x, f = nova.nova_evolution_strategy(m, args.r, z, args.generations, args.population, args.restarts)
            points, kappa = nova.nova_snap_points(m, args.r, x, args.d_max)
            took = time.perf_counter() - tic
            parts = nova.nova_es_fitness(m, args.r, x)
            kappas.append(kappa)
            print(f"  seed {seed}: fitness {f:.6g} (tensor error {parts[1]:.1e}, |p|^2/(n-1) {parts[2]:.4f}, kappa {parts[3]:.1f}); "
                  f"snapped {{{', '.join(str(p) for p in sorted(points))}}} kappa(V) {kappa:.1f}  [{took:.2f} s]")
        k = np.array(kappas)
        print(f"  kappa(V) over {args.seeds} seeds: mean {k.mean():.1f} std {k.std():.1f} CV {100 * k.std() / k.mean():.1f} % "
              f"min {k.min():.1f} max {k.max():.1f}")
        tic = time.perf_counter()
        pts, kappa = nova.nova_symmetric_search(m, args.r, 6)
        print(f"  symmetric search (d_max = 6): {{{', '.join(str(p) for p in sorted(pts))}}} kappa(V) {kappa:.1f}  "
              f"[{time.perf_counter() - tic:.2f} s]")


if __name__ == "__main__":
    main()
