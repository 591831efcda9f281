#!/usr/bin/env python3
"""Regenerates tests/golden/tile_counts.txt from the CPU oracle alone.

For every benchmark shape the oracle's per-query-tile routine (brute force over the
element mask of Sec. 3.1 / 3.3, block cover of Fig. 4) is summed over all query tiles
for the spatial and the temporal pattern.  Nothing of the HIP library is imported or
called.  Takes several minutes on 8 cores (the 120k-token shapes dominate).

    python tests/golden/make_tile_counts.py            # rewrite the file
    python tests/golden/make_tile_counts.py --check    # recompute and compare with the file
"""
from __future__ import annotations

import argparse
import os
import sys
from concurrent.futures import ProcessPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)

from oracle import svg_oracle as O          # noqa: E402
from workloads import get_config            # noqa: E402  (shapes only: no method arithmetic lives there)

PATH = os.path.join(HERE, "tile_counts.txt")
SHAPES = ["cogvideox_v1", "wan21_14b", "cogvideox_v15", "hunyuan", "hunyuan_skip85", "hunyuan_keep31"]

HEADER = """\
# Kept 128x64 tiles per pattern for the benchmark shapes (block semantics: a tile is kept iff
# one of its elements is kept by the spatial mask |f_i - f_j| <= w_s resp. the temporal mask
# |p_i - p_j| <= w_t of Sec. 3.1 / 3.3, text keys always kept, text queries dense; temporal
# counts in the token-major order of Sec. 4.2).
# Written by tests/golden/make_tile_counts.py, which sums the CPU oracle's brute-force per-tile
# routine over all query tiles and calls nothing of the HIP library.  The same six rows were
# first derived, independently of this repository's code, when the benchmark workloads were
# specified (the workload table of the benchmark description); the two derivations agree.
# workload        spatial   temporal  all_tiles
"""


def _count(job):
    name, pattern, a0, a1 = job
    g = O.Geometry.from_config(get_config(name))
    return name, pattern, sum(len(O.kept_tiles_of_row(g, pattern, a)) for a in range(a0, a1))


def compute(workers: int):
    jobs = []
    for name in SHAPES:
        g = O.Geometry.from_config(get_config(name))
        nq, _ = O.n_tiles(g)
        step = 16
        for pattern in (O.SPATIAL, O.TEMPORAL):
            jobs += [(name, pattern, a, min(nq, a + step)) for a in range(0, nq, step)]
    totals = {(n, p): 0 for n in SHAPES for p in (O.SPATIAL, O.TEMPORAL)}
    with ProcessPoolExecutor(max_workers=workers) as pool:
        for i, (name, pattern, c) in enumerate(pool.map(_count, jobs, chunksize=4)):
            totals[(name, pattern)] += c
            if i % 200 == 0:
                print(f"  {i}/{len(jobs)} chunks", file=sys.stderr, flush=True)
    rows = []
    for name in SHAPES:
        g = O.Geometry.from_config(get_config(name))
        nq, nk = O.n_tiles(g)
        rows.append((name, totals[(name, O.SPATIAL)], totals[(name, O.TEMPORAL)], nq * nk))
    return rows


def render(rows) -> str:
    return HEADER + "".join(f"{n:<17} {s:<9} {t:<9} {a}\n" for n, s, t, a in rows)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--check", action="store_true")
    ap.add_argument("--workers", type=int, default=min(8, os.cpu_count() or 1))
    args = ap.parse_args()
    rows = compute(args.workers)
    if args.check:
        stored = [tuple(l.split()) for l in open(PATH) if l.strip() and not l.startswith("#")]
        got = [(n, str(s), str(t), str(a)) for n, s, t, a in rows]
        if stored != got:
            print("MISMATCH\nstored:", stored, "\ncomputed:", got)
            sys.exit(1)
        print("tile_counts.txt agrees with the oracle for all", len(rows), "shapes")
    else:
        with open(PATH, "w") as f:
            f.write(render(rows))
        print("wrote", PATH)


if __name__ == "__main__":
    main()
