"""Host-only tests of the parameter search driver (no GPU: synthetic objectives)."""
import csv
import random

import numpy as np
import pytest

from paper_2309_07235_amd import tune


def _bowl_space():
    vals = list(range(12))
    return tune.SearchSpace(["i", "j", "k"], [vals, vals, vals])


def _bowl(cfg):
    return 1.0 + (cfg["i"] - 7) ** 2 + 2.0 * (cfg["j"] - 3) ** 2 + (cfg["k"] - 9) ** 2


def test_space_decode_size_and_legality():
    sp = tune.SearchSpace(["a", "b"], [[16, 32, 64], ["x", "y"]], legal=lambda c: not (c["a"] == 64 and c["b"] == "y"))
    assert sp.size() == 6
    assert sp.decode((2, 0)) == {"a": 64, "b": "x"}
    assert not sp.is_legal((2, 1)) and sp.is_legal((1, 1))
    rng = random.Random(0)
    seen = set()
    for _ in range(5):  # exactly five legal configurations exist
        c = sp.sample(rng, seen)
        assert c is not None and sp.is_legal(c) and c not in seen
        seen.add(c)
    assert sp.sample(rng, seen, tries=200) is None


def test_encode_is_the_inverse_of_decode():
    space = tune.SearchSpace(["a", "t"], [[16, 32, 48], [(0, 0), (64, 64), (128, 64)]])
    for cfg in [(0, 0), (2, 1), (1, 2)]:
        assert space.encode(space.decode(cfg)) == cfg
    assert space.encode({"a": 32, "t": [128, 64]}) == (1, 2)  # lists and tuples name the same value
    with pytest.raises(ValueError):
        space.encode({"a": 20, "t": (0, 0)})


def test_random_search_is_seeded_distinct_and_stops_when_exhausted():
    sp = _bowl_space()
    a = tune.random_search(sp, _bowl, 40, seed=3)
    b = tune.random_search(sp, _bowl, 40, seed=3)
    assert a.rows == b.rows and len(a.rows) == 40
    assert len({c for c, _ in a.rows}) == 40
    tiny = tune.SearchSpace(["a"], [[1, 2, 3]])
    db = tune.random_search(tiny, lambda c: float(c["a"]), 10, seed=0)
    assert len(db.rows) == 3 and db.best() == ({"a": 1}, 1.0)


def test_lcb_prefers_low_mean_and_high_spread():
    mean, std = np.array([5.0, 5.0, 4.0]), np.array([0.0, 1.0, 0.0])
    assert list(np.argsort(tune.lcb(mean, std, 1.96))) == [1, 2, 0]
    assert list(np.argsort(tune.lcb(mean, std, 0.0)))[0] == 2


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_surrogate_search_finds_the_bowl(seed):
    """60 evaluations in a space of 1728: the forest + LCB search must get close to the minimum (value 1 at
    (7, 3, 9)); 19 of the 1728 points have a value <= 4, so uniform sampling gets there about every second time."""
    sp = _bowl_space()
    db = tune.surrogate_search(sp, _bowl, 60, seed=seed, n_init=10, pool=256, trees=32)
    assert len(db.rows) == 60 and len(db.seen()) == 60
    cfg, val = db.best()
    assert val <= 4.0, (cfg, val)
    again = tune.surrogate_search(sp, _bowl, 60, seed=seed, n_init=10, pool=256, trees=32)
    assert again.rows == db.rows  # reproducible for a fixed seed


def test_database_csv(tmp_path):
    sp = _bowl_space()
    path = tmp_path / "db.csv"
    db = tune.PerformanceDatabase(sp, str(path))
    tune.random_search(sp, _bowl, 7, seed=1, db=db)
    rows = list(csv.reader(open(path)))
    assert rows[0] == ["eval", "i", "j", "k", "runtime_ms", "elapsed_s"]
    assert len(rows) == 8 and [r[0] for r in rows[1:]] == [str(i) for i in range(1, 8)]
    best_cfg, best_ms = db.best()
    assert best_ms == min(float(r[4]) for r in rows[1:])
