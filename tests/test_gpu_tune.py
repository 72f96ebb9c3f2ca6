"""The search driver against the real kernels: a few evaluations on small problems."""
import pytest

from paper_2309_07235_amd import inputs, tune
from tests.gpu_util import announce

pytestmark = pytest.mark.gpu


def test_tune_mm3_small_budget():
    announce("tune mm3 128^3, 14 evaluations")
    space, objective = tune.mm3_problem(inputs.MM3_SMALL, reps=3)
    assert space.size() == len(space.values[0]) ** 3 and len(space.values[0]) > 50
    db = tune.surrogate_search(space, objective, 14, seed=0, n_init=8, pool=128, trees=16)
    cfg, ms = db.best()
    assert len(db.rows) == 14 and 0.0 < ms < 50.0
    assert ms == min(r[1] for r in db.rows)
    assert all(len(cfg[k]) == 6 for k in ("e", "f", "g"))


@pytest.mark.parametrize("kind", ["lu", "chol"])
def test_tune_factor_small_budget(kind):
    announce(f"tune {kind} n=700, 8 evaluations")
    space, objective = tune.factor_problem(kind, 700, reps=2)
    db = tune.random_search(space, objective, 8, seed=1)
    cfg, ms = db.best()
    assert len(db.rows) == 8 and 0.0 < ms < 200.0
    assert cfg["nb"] % 16 == 0 and cfg["lookahead"] in (0, 1)
    if kind == "chol":
        assert all(space.decode(c)["update"][0] == space.decode(c)["update"][1] for c, _ in db.rows)
