"""The search driver against the real kernels: a few evaluations on small problems."""
import pytest

from paper_2309_07235_amd import inputs, tune
from tests.gpu_util import announce

pytestmark = pytest.mark.gpu


def test_tune_mm3_small_budget():
    announce("tune mm3 128^3, 14 evaluations")
    space, objective, default = tune.mm3_problem(inputs.MM3_SMALL, reps=3)
    assert space.decode(space.encode(default)) == default  # the library default is a point of the space
    assert space.size() == len(space.values[0]) ** 3 and len(space.values[0]) > 50
    db = tune.surrogate_search(space, objective, 14, seed=0, n_init=8, pool=128, trees=16)
    cfg, ms = db.best()
    assert len(db.rows) == 14 and 0.0 < ms < 50.0
    assert ms == min(r[1] for r in db.rows)
    assert all(len(cfg[k]) == 6 for k in ("e", "f", "g"))


@pytest.mark.parametrize("kind", ["lu", "chol"])
def test_tune_factor_small_budget(kind):
    announce(f"tune {kind} n=700, 8 evaluations")
    space, objective, default = tune.factor_problem(kind, 700, reps=2)
    assert space.decode(space.encode(default)) == default and default["nb"] == 128
    db = tune.random_search(space, objective, 8, seed=1)
    cfg, ms = db.best()
    assert len(db.rows) == 8 and 0.0 < ms < 200.0
    assert cfg["nb"] % 16 == 0 and cfg["lookahead"] in (0, 1)
    if kind == "chol":
        assert all(space.decode(c)["update"][0] == space.decode(c)["update"][1] for c, _ in db.rows)


def test_search_that_starts_from_the_default_never_ends_worse_than_it(tmp_path, capsys):
    import json
    announce("tune mm3 small from the default, 6 evaluations")
    db = tmp_path / "perf.csv"
    assert tune.main(["--kernel", "mm3", "--dataset", "small", "--evals", "6", "--strategy", "random", "--seed", "3",
                      "--from-default", "--db", str(db)]) == 0
    out = json.loads(capsys.readouterr().out.strip().splitlines()[-1])
    rows = db.read_text().strip().splitlines()
    assert len(rows) == 7 and out["evaluations"] == 6
    first_ms = float(rows[1].split(",")[-2])
    assert out["best_runtime_ms"] <= first_ms + 1e-3
