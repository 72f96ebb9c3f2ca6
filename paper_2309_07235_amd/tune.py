"""Search over the tile / block parameters the library exposes.

The paper tunes its kernels with an iterative loop (Section "Proposed Autotuning Framework", steps 1-5):
a search method proposes a parameter configuration, the kernel is built and run with it, the measured
runtime goes back to the search and into a performance database, until a budget of n evaluations is
spent; the best entry of the database is the result.  Its search method (Section "Backgrounds", ytopt)
is Bayesian optimisation with a Random-Forest surrogate and the lower-confidence-bound acquisition
function; its baseline is random enumeration.

Here the "code mold" is the library's pre-instantiated schedule menu, so an evaluation is one timed call:
  - `SearchSpace`     ordinal parameters (each a list of allowed values, as in the paper's ConfigSpace
                      definition of P0..P5), with a legality filter;
  - `random_search`   uniform sampling without repetition;
  - `surrogate_search` Random-Forest surrogate on the parameter values, refitted after every evaluation,
                      next point = argmin over a candidate pool of  mean - kappa * std  (LCB);
  - `PerformanceDatabase`  every (configuration, runtime) pair, optionally mirrored to a CSV file;
  - `mm3_problem`, `factor_problem`  the search spaces and timed objectives of the three kernels.

Nothing here is on the hot path; it only drives the C ABI through the Python binding.

  python -m paper_2309_07235_amd.tune --kernel mm3 --evals 100 --strategy rf --db mm3.csv
"""
from __future__ import annotations

import argparse
import csv
import json
import math
import random
import sys
import time
from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence, Tuple

Config = Tuple[int, ...]  # one index per parameter into that parameter's value list


def _plain(x):
    return tuple(x) if isinstance(x, (list, tuple)) else x


@dataclass
class SearchSpace:
    """Ordinal parameters: names[i] takes one of values[i]; a configuration is a tuple of indices."""
    names: List[str]
    values: List[Sequence]
    legal: Optional[Callable[[Dict[str, object]], bool]] = None

    def size(self) -> int:
        return math.prod(len(v) for v in self.values)

    def decode(self, cfg: Config) -> Dict[str, object]:
        return {n: v[i] for n, v, i in zip(self.names, self.values, cfg)}

    def encode(self, point: Dict[str, object]) -> Config:
        """Inverse of decode; raises ValueError when a value is not in its parameter's list."""
        return tuple(list(map(_plain, v)).index(_plain(point[n])) for n, v in zip(self.names, self.values))

    def features(self, cfg: Config) -> List[float]:
        """What the surrogate sees: numeric values as they are, tuples of numbers (a schedule of the menu:
        tile, slab depth, unroll, wave split) field by field, anything else by its index."""
        out: List[float] = []
        for v, i in zip(self.values, cfg):
            x = v[i]
            if isinstance(x, (int, float)):
                out.append(float(x))
            elif isinstance(x, (tuple, list)) and all(isinstance(e, (int, float)) for e in x):
                out.extend(float(e) for e in x)
            else:
                out.append(float(i))
        return out

    def is_legal(self, cfg: Config) -> bool:
        return self.legal is None or bool(self.legal(self.decode(cfg)))

    def sample(self, rng: random.Random, exclude=(), tries: int = 10000) -> Optional[Config]:
        for _ in range(tries):
            cfg = tuple(rng.randrange(len(v)) for v in self.values)
            if cfg not in exclude and self.is_legal(cfg):
                return cfg
        return None


@dataclass
class PerformanceDatabase:
    """Every evaluated configuration with its runtime (ms); mirrors rows to a CSV file when a path is given."""
    space: SearchSpace
    path: Optional[str] = None
    rows: List[Tuple[Config, float]] = field(default_factory=list)

    def __post_init__(self):
        if self.path:
            with open(self.path, "w", newline="") as f:
                csv.writer(f).writerow(["eval", *self.space.names, "runtime_ms", "elapsed_s"])
        self._t0 = time.perf_counter()

    def record(self, cfg: Config, ms: float) -> None:
        self.rows.append((cfg, ms))
        if self.path:
            with open(self.path, "a", newline="") as f:
                d = self.space.decode(cfg)
                csv.writer(f).writerow([len(self.rows), *[json.dumps(d[n]) for n in self.space.names],
                                        f"{ms:.6f}", f"{time.perf_counter() - self._t0:.3f}"])

    def seen(self):
        return {c for c, _ in self.rows}

    def best(self) -> Tuple[Dict[str, object], float]:
        cfg, ms = min(self.rows, key=lambda r: r[1])
        return self.space.decode(cfg), ms


def random_search(space: SearchSpace, objective: Callable[[Dict[str, object]], float], evals: int, seed: int = 0,
                  db: Optional[PerformanceDatabase] = None) -> PerformanceDatabase:
    """The random-enumeration baseline: `evals` distinct legal configurations, uniformly at random."""
    rng = random.Random(seed)
    db = db or PerformanceDatabase(space)
    while len(db.rows) < evals:
        cfg = space.sample(rng, db.seen())
        if cfg is None:
            break  # space exhausted
        db.record(cfg, float(objective(space.decode(cfg))))
    return db


def lcb(mean, std, kappa: float):
    """Lower confidence bound of a predicted runtime: small mean (exploitation) or large spread (exploration)."""
    return mean - kappa * std


def surrogate_search(space: SearchSpace, objective: Callable[[Dict[str, object]], float], evals: int, seed: int = 0,
                     n_init: int = 10, pool: int = 512, kappa: float = 1.96, trees: int = 64,
                     db: Optional[PerformanceDatabase] = None) -> PerformanceDatabase:
    """Bayesian optimisation with a Random-Forest surrogate and the LCB acquisition function.

    n_init random configurations seed the model; then, per evaluation: fit the forest on
    (parameter values -> log runtime), draw `pool` unevaluated legal candidates, predict each with
    every tree, and evaluate the candidate whose  mean - kappa * std  over the trees is smallest.
    """
    import numpy as np
    from sklearn.ensemble import RandomForestRegressor

    rng = random.Random(seed)
    db = db or PerformanceDatabase(space)
    while len(db.rows) < min(n_init, evals):
        cfg = space.sample(rng, db.seen())
        if cfg is None:
            return db
        db.record(cfg, float(objective(space.decode(cfg))))
    while len(db.rows) < evals:
        X = np.array([space.features(c) for c, _ in db.rows], dtype=float)
        y = np.log(np.array([max(ms, 1e-9) for _, ms in db.rows]))
        forest = RandomForestRegressor(n_estimators=trees, min_samples_leaf=1, random_state=seed + len(db.rows))
        forest.fit(X, y)
        seen = db.seen()
        cands = []
        for _ in range(pool):
            c = space.sample(rng, seen)
            if c is None:
                break
            cands.append(c)
        cands = list(dict.fromkeys(cands))
        if not cands:
            break
        C = np.array([space.features(c) for c in cands], dtype=float)
        per_tree = np.stack([t.predict(C) for t in forest.estimators_])
        score = lcb(per_tree.mean(axis=0), per_tree.std(axis=0), kappa)
        cfg = cands[int(np.argmin(score))]
        db.record(cfg, float(objective(space.decode(cfg))))
    return db


# ------------------------------------------------------------------ the three kernels as tuning problems
def _time_ms(fn, reps: int) -> float:
    """Median device time of fn() in ms (events on the current stream), after one untimed call."""
    import torch
    fn()
    torch.cuda.synchronize()
    times = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        e1.synchronize()
        times.append(e0.elapsed_time(e1))
    times.sort()
    return times[len(times) // 2]


def mm3_problem(dims: Dict[str, int], seed: int = 4, reps: int = 5, dtype: str = "f64"):
    """Search space and objective of 3mm: one schedule of the menu per product (the paper's P0..P5 are the
    macro-tiles of E, F and G; the native k-slab / unroll / wave-split knobs ride along in the same entry)."""
    import torch
    from . import binding as B
    from . import inputs

    dt = B.DLA_F64 if dtype == "f64" else B.DLA_F32
    tdt = torch.float64 if dtype == "f64" else torch.float32
    menu = [t.as_tuple() for t in B.enumerate_tiles(dt)]
    space = SearchSpace(["e", "f", "g"], [menu, menu, menu])
    ops = [torch.from_numpy(x).to("cuda").to(tdt) for x in inputs.mm3_operands(seed, **dims)]
    g = torch.empty((dims["ni"], dims["nl"]), dtype=tdt, device="cuda")
    ws = torch.empty(B.mm3_workspace_bytes(dims["ni"], dims["nj"], dims["nl"], dt), dtype=torch.uint8, device="cuda")

    def objective(cfg):
        p = B.Mm3Params(B.GemmParams(*cfg["e"]), B.GemmParams(*cfg["f"]), B.GemmParams(*cfg["g"]))
        return _time_ms(lambda: B.mm3(*ops, g, p, workspace=ws), reps)

    d = B.default_params(B.DLA_KERNEL_MM3, dims["nk"], dt)
    return space, objective, {"e": d.e.as_tuple(), "f": d.f.as_tuple(), "g": d.g.as_tuple()}


def factor_problem(kind: str, n: int, seed: int = 5, reps: int = 3, dtype: str = "f64"):
    """Search space and objective of lu_factor / cholesky_factor: block size (one level up to 128, two sub-panels
    above), look-ahead, the trailing-update schedule (entry 0 = the library's own update kernel, the others = tiled
    GEMM schedules of the menu), and the size from which bulk updates run two panels deep."""
    import torch
    from . import binding as B
    from . import inputs

    dt = B.DLA_F64 if dtype == "f64" else B.DLA_F32
    tdt = torch.float64 if dtype == "f64" else torch.float32
    host = inputs.diag_dominant_matrix(n, seed) if kind == "lu" else inputs.spd_matrix(n, seed)
    src = torch.from_numpy(host).to("cuda").to(tdt)
    work = torch.empty_like(src)
    fn = B.lu_factor if kind == "lu" else B.cholesky_factor
    updates = [(0, 0, 0, 0, 0, 0)] + [t.as_tuple() for t in B.enumerate_tiles(dt)]
    def legal(c):
        if c["nb"] > 128 and (c["lookahead"] == 0 or any(c["update"])):
            return False  # two sub-panels per panel need the pipeline and the library's own update kernel
        if c["defer_min_rows"] != 0 and (c["nb"] != 128 or any(c["update"])):
            return False  # the threshold only exists for block size 128 (keeps the space free of duplicates)
        return kind == "lu" or c["update"][0] == c["update"][1]  # Cholesky: square tiles

    space = SearchSpace(["nb", "lookahead", "update", "defer_min_rows"],
                        [list(range(16, 129, 16)) + [160, 192, 224, 256], [0, 1], updates, [0, -1, 1, 1024, 2048]],
                        legal=legal)
    ws = torch.empty(B.factor_workspace_bytes(n, dt, None), dtype=torch.uint8, device="cuda")
    info = torch.zeros(1, dtype=torch.int32, device="cuda")  # look-ahead 1 hands over inside kernels only with an info pointer

    def objective(cfg):
        p = B.FactorParams(cfg["nb"], cfg["lookahead"], B.GemmParams(*cfg["update"]), cfg["defer_min_rows"])

        def call():
            work.copy_(src)  # in place: restore the input (a device copy, part of every evaluation alike)
            fn(work, p, workspace=ws, info=info)

        return _time_ms(call, reps)

    d = B.default_params(B.DLA_KERNEL_LU if kind == "lu" else B.DLA_KERNEL_CHOLESKY, n, dt)
    return space, objective, {"nb": d.nb, "lookahead": d.lookahead, "update": d.update.as_tuple(),
                              "defer_min_rows": d.defer_min_rows}


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description="search the exposed tile / block parameters of one kernel")
    ap.add_argument("--kernel", choices=["mm3", "lu", "cholesky"], default="mm3")
    ap.add_argument("--n", type=int, default=4000, help="matrix size of the factorisations")
    ap.add_argument("--dataset", choices=["small", "extralarge"], default="extralarge", help="3mm shape")
    ap.add_argument("--evals", type=int, default=100, help="evaluation budget (the paper uses 100)")
    ap.add_argument("--strategy", choices=["rf", "random"], default="rf")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--db", default=None, help="CSV file for the performance database")
    ap.add_argument("--from-default", action="store_true",
                    help="spend the first evaluation on the library's default configuration, so that the result is "
                         "never worse than it (the paper's searches start from random points)")
    args = ap.parse_args(argv)

    from . import inputs
    t0 = time.perf_counter()
    if args.kernel == "mm3":
        dims = inputs.MM3_EXTRALARGE if args.dataset == "extralarge" else inputs.MM3_SMALL
        space, objective, default = mm3_problem(dims)
    else:
        space, objective, default = factor_problem("lu" if args.kernel == "lu" else "chol", args.n)
    db = PerformanceDatabase(space, args.db)
    if args.from_default and args.evals > 0:
        db.record(space.encode(default), float(objective(default)))
    search = surrogate_search if args.strategy == "rf" else random_search
    search(space, objective, args.evals, seed=args.seed, db=db)
    cfg, ms = db.best()
    print(json.dumps({"kernel": args.kernel, "strategy": args.strategy, "space_size": space.size(),
                      "evaluations": len(db.rows), "best_runtime_ms": round(ms, 4), "best": cfg,
                      "process_time_s": round(time.perf_counter() - t0, 2)}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
