"""The grid-row planner of the batched kernels (csrc/row_plan.hpp), on the CPU: whatever it decides, every tile of every
item must be covered exactly once, by rows that fit their launch, start on the granule and respect the table size; and on
lists with the structure of a transformer it must find the common piece.  The planner is header-only C++; a small harness
(tests/native/row_plan_harness.cpp) is compiled with g++ and driven through stdin/stdout."""
import os
import subprocess

import numpy as np
import pytest

from oracle import elixir_oracle as orc
from synth import gen

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def harness(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("row_plan") / "harness")
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-Wall", "-o", exe, os.path.join(HERE, "native", "row_plan_harness.cpp")])
    return exe


def plan(exe, tiles, granule, max_rows, max_piece=1 << 22):
    text = f"{granule} {max_rows} {max_piece}\n" + " ".join(str(t) for t in tiles) + "\n"
    out = subprocess.run([exe], input=text, capture_output=True, text=True, check=True).stdout
    launches = []
    for line in out.splitlines():
        kind, *vals = line.split()
        if kind == "L":
            launches.append((int(vals[0]), []))
        else:
            launches[-1][1].append(tuple(int(v) for v in vals))
    return launches


def check(tiles, launches, granule, max_rows, max_piece):
    covered = [np.zeros(t, np.int32) for t in tiles]
    for row_length, rows in launches:
        assert 1 <= len(rows) <= max_rows
        assert row_length <= max_piece and row_length == max(n for _, _, n in rows)        # the grid is as long as its longest row
        for item, first, n in rows:
            assert n >= 1 and first % granule == 0 and first + n <= tiles[item]
            covered[item][first:first + n] += 1
    for t, c in zip(tiles, covered):
        assert (c == 1).all(), "a tile is covered twice or not at all"
    used = sum(tiles)
    grid = sum(length * len(rows) for length, rows in launches)
    return len(launches), (grid - used) / max(used, 1)


@pytest.mark.parametrize("granule,max_rows", [(1, 160), (16, 64), (1, 3), (16, 1)])
def test_every_tile_is_covered_exactly_once(harness, granule, max_rows):
    rng = np.random.default_rng(granule * 1000 + max_rows)
    for _ in range(60):
        kind = rng.integers(0, 4)
        n = int(rng.integers(1, 60))
        if kind == 0:
            tiles = [int(x) for x in rng.integers(0, 50, size=n)]
        elif kind == 1:
            tiles = [int(x) for x in rng.integers(1, 200_000, size=n)]
        elif kind == 2:                                   # a few sizes that are multiples of each other, plus tiny ones
            base = int(rng.integers(1, 4000)) * granule
            tiles = [int(base * rng.choice([1, 2, 3, 4])) for _ in range(n)] + [int(x) for x in rng.integers(1, 20, size=n)]
        else:
            tiles = [int(rng.integers(1, 1 << 20))] + [int(x) for x in rng.integers(0, 3000, size=n)]
        max_piece = int(rng.choice([1 << 22, 4096, 64])) // granule * granule
        check(tiles, plan(harness, tiles, granule, max_rows, max_piece), granule, max_rows, max_piece)
    assert plan(harness, [], granule, max_rows) == [] and plan(harness, [0, 0], granule, max_rows) == []


def test_more_items_than_one_window(harness):
    rng = np.random.default_rng(5)
    tiles = [int(x) for x in rng.integers(0, 300, size=9000)]       # the planner works through windows of 4096 items
    check(tiles, plan(harness, tiles, 1, 160), 1, 160, 1 << 22)


def test_transformer_shaped_lists_get_their_common_piece(harness):
    """The 581 tensor pieces of the 1.5B set in tiles of 256 elements: the weight matrices are 4x, 3x and 1x one
    common length, which becomes the row length, and the grid of the big launches has no idle tail."""
    cfg = gen.CONFIGS["gpt2_1p5b"]
    C = cfg.chunk_elems
    numels = cfg.numels()
    cid, off, _ = orc.layout_plan(numels, C, orc.NEXT_FIT, 1)
    pieces = []
    for i, n in enumerate(numels):
        c, o, left = cid[i], off[i], n
        while left > 0:
            take = min(left, C - o)
            pieces.append(take)
            left, c, o = left - take, c + 1, 0
    tiles = [(n // 4 + 63) // 64 for n in pieces]
    launches = plan(harness, tiles, 1, 160)
    n_launches, idle = check(tiles, launches, 1, 160, 1 << 22)
    assert launches[0][0] == 10_000                                   # 2,560,000 elements: the attention projection, a quarter of the MLP matrices
    assert n_launches <= 8 and idle < 0.02
    # the tiny set's seven ragged chunks in workgroups of 256 elements, whole state tiles per row: one launch, few idle workgroups
    tiny = gen.CONFIGS["tiny"]
    valid = orc.layout_plan(tiny.numels(), tiny.chunk_elems, orc.NEXT_FIT, 1)[2]
    blocks = [(n // 2 + 127) // 128 for n in valid]
    n_launches, idle = check(blocks, plan(harness, blocks, 16, 64), 16, 64, 1 << 22)
    assert n_launches == 1 and idle < 0.06
