"""Pins for the oracle's Sharded-LRTF scheduler (paper Section 2.4)."""
import itertools
import os

import numpy as np
import pytest

import synth_inputs as SI
from oracle import spilled as SP

GOLD = os.path.join(os.path.dirname(__file__), "golden", "sched_lrtf_example.txt")


def _cases():
    cases, cur = [], None
    for line in open(GOLD):
        line = line.strip()
        if line.startswith("n_tasks:"):
            cur = [[1] * int(x) for x in line.split()[1:]]
        elif line.startswith("costs:"):
            cur = [[int(c) for c in grp.split(",")] for grp in line.split()[1:]]
        elif line.startswith("order:"):
            cases.append((cur, line.split()[1:]))
    return cases


@pytest.mark.parametrize("costs,expect", _cases())
def test_hand_worked_examples(costs, expect):
    chains = [list(range(len(c))) for c in costs]
    order = SP.sharded_lrtf(chains, costs)
    assert ["ABC"[m] for m, _ in order] == expect


def _independent_lrtf(costs):
    """Written separately from the oracle: simulate with explicit task lists."""
    todo = [list(c) for c in costs]
    done = [0] * len(costs)
    out = []
    while any(todo):
        rem = [sum(t) if t else -1 for t in todo]
        m = rem.index(max(rem))          # index() returns the lowest index on ties
        todo[m].pop(0)
        out.append((m, done[m]))
        done[m] += 1
    return out


def test_bruteforce_small_cost_tables():
    vals = (1, 2, 5)
    for n_models in (1, 2, 3):
        for lens in itertools.product((1, 2, 3), repeat=n_models):
            rng = np.random.default_rng(sum(lens) * 7 + n_models)
            for _ in range(6):
                costs = [[int(rng.choice(vals)) for _ in range(n)] for n in lens]
                chains = [list(range(n)) for n in lens]
                assert SP.sharded_lrtf(chains, costs) == _independent_lrtf(costs)


def test_equal_models_degenerate_to_round_robin_and_chain_order():
    cfg = SI.small_cfg(L=4, k=2)
    n_models, nmb = 3, 2
    chains = [SP.model_task_chain(cfg, nmb) for _ in range(n_models)]
    fc, bc = SI.task_costs(cfg)
    costs = [[(fc if ph == SP.FWD else bc)[s] for s, ph in ch] for ch in chains]
    order = SP.sharded_lrtf(chains, costs)
    assert [m for m, _ in order] == [0, 1, 2] * len(chains[0])
    S = cfg["L"] // cfg["k"]
    one = [(s, SP.FWD) for s in range(S + 2)] + [(s, SP.BWD) for s in range(S + 1, -1, -1)]
    for m in range(n_models):
        mine = [chains[m][i] for mm, i in order if mm == m]
        assert mine == one * nmb
        assert len(mine) == 2 * (S + 2) * nmb      # every shard visited exactly twice per minibatch
    # finish times differ by at most one task per model when costs are equal
    last = {m: max(i for i, (mm, _) in enumerate(order) if mm == m) for m in range(n_models)}
    assert max(last.values()) - min(last.values()) <= n_models - 1
