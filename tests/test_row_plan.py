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


# ---- the compact table of rows (two bases per launch, 32-bit offsets)

def tables(exe, rows):
    text = "".join(f"{d} {s} {c}\n" for d, s, c in rows)
    out = subprocess.run([exe, "table"], input=text, capture_output=True, text=True, check=True).stdout
    got = []
    for line in out.splitlines():
        kind, *vals = line.split()
        assert kind != "P", "an unused entry of the table was not cleared"
        if kind == "T":
            got.append(([int(v) for v in vals], []))
        else:
            got[-1][1].append(tuple(int(v) for v in vals))
    return got


def check_tables(rows, got, max_rows=336):
    """Every row once, in the order given; offsets lead back to the addresses; launches within the table size."""
    NO_SOURCE = 0xFFFFFFFF
    k = 0
    for (n_rows, longest, dst_base, src_base), entries in got:
        assert 1 <= n_rows == len(entries) <= max_rows
        assert dst_base % 1024 == 0                            # so that dst_off mod 64 is the row's distance from a KiB boundary
        assert longest == max((c + d_off % 64 + 63) // 64 for d_off, _, c in entries)   # the first workgroup starts that many lanes in
        for d_off, s_off, count in entries:
            d, s, c = rows[k]
            assert dst_base + 16 * d_off == d and count == c
            if s == 0:
                assert s_off == NO_SOURCE
            else:
                assert s_off < NO_SOURCE and src_base + 8 * s_off == s
            k += 1
    assert k == len(rows)


def test_compact_table_keeps_every_row_and_its_addresses(harness):
    rng = np.random.default_rng(3)
    base_d, base_s = 0x7F0000000000, 0x7E0000000000
    rows = [(base_d + 16 * int(rng.integers(0, 1 << 28)), base_s + 8 * int(rng.integers(0, 1 << 28)), int(rng.integers(1, 1 << 20))) for _ in range(1000)]
    rows[5] = (rows[5][0], 0, 77)                      # rows without a source (fills) among the others
    rows[6] = (rows[6][0], 0, 1)
    got = tables(harness, rows)
    check_tables(rows, got)
    assert [t[0][0] for t in got] == [336, 336, 328]   # full tables, then the rest
    only_fills = [(base_d + 16 * i, 0, 64) for i in range(10)]
    got = tables(harness, only_fills)
    check_tables(only_fills, got)
    assert got[0][0][3] == 0                            # no source base when no row has a source


def test_compact_table_starts_a_new_launch_when_an_offset_would_not_fit(harness):
    GiB = 1 << 30
    d0, s0 = 0x7F0000000000, 0x7E0000000000
    # destinations 16-byte units: 2^32 units = 64 GiB; sources 8-byte units: 2^32 units = 32 GiB
    rows = [(d0, s0, 100), (d0 + 63 * GiB, s0 + 31 * GiB, 100),          # still one launch
            (d0 + 65 * GiB, s0, 100),                                     # destination too far from the lowest one
            (d0 + 65 * GiB + 16, s0 + 33 * GiB, 100),                     # source too far
            (d0 - 70 * GiB, s0 + 33 * GiB, 100),                          # below the base: the span counts, not the order
            (d0 - 70 * GiB + 16, 0, 100), (d0 - 70 * GiB + 32, s0 - 40 * GiB, 5)]   # a fill does not move the source span; the next source does
    got = tables(harness, rows)
    check_tables(rows, got)
    assert [t[0][0] for t in got] == [2, 1, 1, 2, 1]
    # exactly at the limit: the largest offset is 2^32 - 2 units (2^32 - 1 marks a row without a source)
    edge = [(d0, s0, 1), (d0 + 16 * 0xFFFFFFFE, s0 + 8 * 0xFFFFFFFE, 1), (d0 + 16 * 0xFFFFFFFF, s0, 1)]
    got = tables(harness, edge)
    check_tables(edge, got)
    assert [t[0][0] for t in got] == [2, 1]
