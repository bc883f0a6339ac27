"""Pins for the oracle partitioner (paper Section 2.2, Algorithm 1) and the
library's host-side partitioner against it.  No GPU."""
import itertools

import numpy as np
import pytest

import synth_inputs as SI
from oracle import partition as OP
from paper_2110_08633_amd import hydra as H


def _brute_force(sizes, overhead, bound):
    """All ways to cut a chain; feasible = every shard's summed size + overhead <= bound.  Returns the feasible
    partitions with the fewest shards."""
    n = len(sizes)
    best, best_n = [], None
    for r in range(n):
        for cut in itertools.combinations(range(1, n), r):
            b = [0] + list(cut) + [n]
            if all(sum(sizes[b[j]:b[j + 1]]) + overhead <= bound for j in range(len(b) - 1)):
                if best_n is None or r + 1 < best_n:
                    best, best_n = [[0] + list(cut)], r + 1
                elif r + 1 == best_n:
                    best.append([0] + list(cut))
        if best_n is not None:
            break
    return best


@pytest.mark.parametrize("seed", range(20))
def test_greedy_walk_is_feasible_maximal_and_uses_fewest_shards(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 9))
    sizes = [int(x) for x in rng.integers(1, 20, n)]
    overhead = int(rng.integers(0, 5))
    bound = max(sizes) + overhead + int(rng.integers(0, 30))
    fits = lambda a, b: sum(sizes[a:b + 1]) + overhead <= bound
    cuts = OP.partition(n, fits)
    b = cuts + [n]
    assert cuts[0] == 0 and b == sorted(set(b))
    for j in range(len(cuts)):
        assert fits(b[j], b[j + 1] - 1)                          # every shard fits
        if j + 1 < len(cuts):
            assert not fits(b[j], b[j + 1])                      # and could not take the next layer
    opt = _brute_force(sizes, overhead, bound)
    assert len(cuts) == len(opt[0])                              # no partition has fewer shards
    assert cuts in opt


def test_uniform_layers_closed_form_and_errors():
    # equal layers of size 3, bound 10, no overhead: shards of floor(10 / 3) = 3 layers
    fits = lambda a, b: 3 * (b - a + 1) <= 10
    assert OP.partition(8, fits) == [0, 3, 6]
    assert OP.equal_shard_size(8, [0, 3, 6]) == 2                # divisors of 8 that are <= 3: 1, 2
    assert OP.equal_shard_size(12, [0, 3, 6, 9]) == 3
    assert OP.partition(4, lambda a, b: True) == [0]
    assert OP.equal_shard_size(4, [0]) == 4
    with pytest.raises(MemoryError):
        OP.partition(3, lambda a, b: False)
    with pytest.raises(MemoryError):
        OP.partition(3, lambda a, b: (a, b) == (0, 0))           # layer 1 alone does not fit


@pytest.mark.parametrize("name", ["tiny", "gpt2s", "gpt2m", "gpt2xl", "gpt6b"])
def test_library_partitioner_equals_oracle_on_the_library_footprint(name):
    """The library's walk over its closed-form footprint against the oracle's walk over the same numbers."""
    cfg = SI.CONFIGS[name]
    desc = H.model_desc(cfg, 1e-4)
    L = cfg["L"]
    fp = [H.hydra_shard_footprint(desc, n) for n in range(L + 1)]
    assert all(fp[n + 1] > fp[n] for n in range(1, L))           # more layers, more memory
    for frac in (1.0, 2.5, 4.0, 7.3, float(L)):
        n_fit = max(1, min(L, int(frac)))
        bound = max(fp[n_fit], fp[0])
        fits = lambda a, b: fp[b - a + 1] <= bound
        want = OP.partition(L, fits)
        cuts, k = H.hydra_partition(desc, bound)
        assert cuts == want
        assert k == OP.equal_shard_size(L, want)
        assert L % k == 0 and fp[k] <= bound
    with pytest.raises(H.HydraError) as e:
        H.hydra_partition(desc, min(fp[1], fp[0]) - 1)
    assert e.value.code == H.E_NOMEM


def test_footprint_grows_with_the_parts_it_names():
    """18 bytes per parameter of shard buffer (fp32 w, m, v, g + one bf16 copy; the library keeps two) is a lower bound; micro-batches do
    not change it (activation memory is that of one micro-batch)."""
    cfg = SI.CONFIGS["gpt2s"]
    desc = H.model_desc(cfg, 1e-4)
    per_block = 12 * cfg["d"] ** 2 + 13 * cfg["d"]
    for n in (1, 2, 6):
        assert H.hydra_shard_footprint(desc, n) >= 18 * n * per_block
    d4 = H.model_desc(dict(cfg, n_micro=4), 1e-4)
    assert H.hydra_shard_footprint(d4, 2) == H.hydra_shard_footprint(desc, 2)
