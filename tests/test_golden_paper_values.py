"""Pins of the oracle and of the input recipe to values the paper itself prints (fixtures under tests/golden/,
each with its citation).  CPU only."""
import os

import numpy as np

import dipaco_inputs as gen
from oracle import dipaco_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_module_sharing_of_the_three_level_toy_example():
    """Section 2.6: the order in which the module choices collapse into one path number.  With level 1 as the most
    significant digit the oracle reproduces every sharing set of the illustration; the other order would give
    {1, 3} for the first module of level 2."""
    rows = _lines("module_sharing_toy_example.txt")
    assert rows[0][0] == "modules_per_level"
    K = tuple(int(v) for v in rows[0][1:])
    for r in rows[1:]:
        level, module, paths = int(r[0]), int(r[1]), [int(v) for v in r[2:]]
        got = [j + 1 for j in orc.paths_through_module(level - 1, module - 1, K)]
        assert got == paths, (level, module, got, paths)
        assert len(got) == int(np.prod(K)) // K[level - 1]            # P_{l,e} = P / K_l of Algorithm 1
    # and the paths of one module differ in the other levels only
    assert orc.modules_of_path(1, K) == (0, 0, 1) and orc.path_index((0, 1, 0), K) == 2


def test_path_counts_of_the_papers_grids():
    for r in _lines("path_count_example.txt"):
        K = tuple(int(v) for v in r[:r.index("->")])
        P = int(r[-1])
        js = {orc.path_index(m, K) for m in np.ndindex(*K)}
        assert js == set(range(P))
        assert sorted(sum((orc.paths_through_module(0, e, K) for e in range(K[0])), [])) == list(range(P))


def test_architecture_and_recipe_follow_the_papers_table():
    """The benchmark configurations take the paper's sizes and constants; and the oracle's parameter layout, given the
    paper's own 16 heads and one shared embedding / output matrix, lands on the path size the paper names."""
    g = {k: float(v) for k, v in _lines("hyperparameters_150m.txt")}
    for c in (2, 5):
        cfg = gen.CONFIGS[c]
        assert sum(cfg["layers_per_level"]) == g["layers"] and cfg["d_model"] == g["hidden"]
        assert cfg["d_head"] == g["key_value_size"] and cfg["vocab"] == g["vocab"]
        assert cfg["wd"] == g["weight_decay"] and cfg["lr"] == g["max_learning_rate"]
    assert gen.CONFIGS[2]["seq"] == g["train_sequence_length"] and gen.CONFIGS[5]["seq"] == g["eval_sequence_length"]
    for c in (1, 3, 5):
        assert gen.CONFIGS[c]["outer_lr"] == g["outer_learning_rate"]
        assert gen.CONFIGS[c]["outer_momentum"] == g["outer_momentum"]
    paper = orc.Arch((6, 6), int(g["hidden"]), int(g["heads_paper"]), int(g["key_value_size"]), 4 * int(g["hidden"]),
                     int(g["vocab"]), int(g["train_sequence_length"]))
    tied = orc.param_count(paper) - int(g["vocab"]) * int(g["hidden"])       # one matrix for embedding and output
    assert abs(tied - g["path_parameters_nominal"]) / g["path_parameters_nominal"] < 0.01
    # the benchmark architecture (14 heads, untied) is the same family: only the attention width and the head differ
    bench = orc.Arch((6, 6), 896, 14, 64, 3584, 32000, 1024)
    assert orc.param_count(bench) == 174_008_576
    lay_p, lay_b = orc.param_layout(paper), orc.param_layout(bench)
    assert lay_p.keys() == lay_b.keys()
