"""rCache replacement simulation (Belady) and chunk-size search: oracle pins and product parity.  Host only."""
import functools
import time

import numpy as np
import pytest

import paper_2212_05339_amd as ex
from oracle import elixir_oracle as orc
from synth import gen


def min_misses_brute_force(seq, n_blocks):
    """Fewest misses any replacement policy can reach: exhaustive search over eviction choices."""
    seq = tuple(seq)

    @functools.lru_cache(maxsize=None)
    def go(i, cache):
        if i == len(seq):
            return 0
        c = seq[i]
        if c in cache:
            return go(i + 1, cache)
        if len(cache) < n_blocks:
            return 1 + go(i + 1, tuple(sorted(cache + (c,))))
        return 1 + min(go(i + 1, tuple(sorted(tuple(x for x in cache if x != v) + (c,)))) for v in cache)

    return go(0, ())


def test_oracle_belady_is_optimal_on_small_sequences():
    rng = np.random.default_rng(3)
    for _ in range(150):
        n_ids = int(rng.integers(2, 7))
        seq = [int(x) for x in rng.integers(0, n_ids, size=rng.integers(1, 14))]
        blocks = int(rng.integers(1, 5))
        misses, evictions = orc.rcache_simulate(seq, blocks)
        assert misses == min_misses_brute_force(seq, blocks)
        assert evictions == max(0, misses - blocks)        # the cache never shrinks: every miss beyond the first `blocks` evicts


def test_oracle_hand_worked_and_closed_form():
    # 2 blocks, sequence 0 1 2 0 1: miss 0, miss 1, miss 2 (0 is used at 3, 1 at 4: evict 1), hit 0, miss 1 (evict either)
    assert orc.rcache_simulate([0, 1, 2, 0, 1], 2) == (4, 2)
    # one training step over n chunks, forward then backward, B blocks: the last B chunks of the forward pass are
    # still cached when the backward pass starts, so misses = n + max(0, n - B)
    for n in range(1, 9):
        for B in range(1, 10):
            seq = list(range(n)) + list(range(n - 1, -1, -1))
            seq = [c for i, c in enumerate(seq) if i == 0 or seq[i - 1] != c]
            misses, ev = orc.rcache_simulate(seq, B)
            assert misses == n + max(0, n - B)
            assert ev == max(0, misses - B)
    with pytest.raises(ValueError):
        orc.rcache_simulate([0], 0)


def test_product_simulation_matches_oracle():
    rng = np.random.default_rng(4)
    for _ in range(300):
        n_ids = int(rng.integers(1, 30))
        seq = [int(x) for x in rng.integers(0, n_ids, size=rng.integers(0, 200))]
        blocks = int(rng.integers(1, 12))
        assert ex.elixir_rcache_simulate(seq, blocks) == orc.rcache_simulate(seq, blocks)
    for bad in (([0, -1], 2), ([0], 0), ([10 ** 9], 1)):
        with pytest.raises(ex.ElixirError) as e:
            ex.elixir_rcache_simulate(*bad)
        assert e.value.code == ex.ELIXIR_EINVAL


def test_step_sequence_hand_case():
    # the grouping example of the layout tests: numels 3 5 4 9 2, C = 8 -> chunks 0 0 1 2(+3) 3
    numels = [3, 5, 4, 9, 2]
    cid, off, _ = orc.layout_plan(numels, 8, orc.NEXT_FIT)
    assert orc.step_access_sequence(numels, 8, cid, off) == [0, 1, 2, 3, 2, 1, 0]


@pytest.mark.parametrize("policy", [0, 1, 2])
def test_search_matches_oracle_on_small_sets(policy):
    rng = np.random.default_rng(5 + policy)
    for _ in range(40):
        numels = [int(x) for x in rng.integers(0, 50, size=rng.integers(1, 25))]
        cands = sorted({int(x) for x in rng.integers(4, 60, size=5)})
        cache = float(rng.integers(16, 400))
        assert ex.elixir_chunk_size_search(numels, cands, cache, policy) == tuple(orc.chunk_size_search(numels, cands, cache, policy))


def test_search_on_the_gpt2_1p5b_set():
    cfg = gen.CONFIGS["gpt2_1p5b"]
    cands = gen.SWEEP_CHUNK_ELEMS
    cache = 2.0 * (1 << 30)                                    # a 2 GiB rCache
    t0 = time.perf_counter()
    best, replaced, padding = ex.elixir_chunk_size_search(cfg.numels(), cands, cache)
    dt = time.perf_counter() - t0
    assert (best, replaced, padding) == tuple(orc.chunk_size_search(cfg.numels(), cands, cache))
    assert dt < 0.5
    # a cache that holds every chunk replaces nothing, whatever the length; then padding decides
    best, replaced, padding = ex.elixir_chunk_size_search(cfg.numels(), cands, 1e12)
    assert not any(replaced) and padding[best] == min(padding)
