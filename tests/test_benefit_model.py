"""Offloading benefit model (paper Sec. 5.1, Eq. 1 and 2) and placement rule: oracle pins and product parity.  Host only."""
import itertools
import os
from fractions import Fraction as Fr

import numpy as np
import pytest

import paper_2212_05339_amd as ex
from oracle import elixir_oracle as orc

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
G = 10 ** 9


def paper_tables():
    rows = []
    with open(os.path.join(GOLD, "paper_hardware_tables.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            srv, n, c2g, g2c, vg, vc = line.split()
            rows.append((srv, int(n), Fr(int(c2g), 10) * G, Fr(int(g2c), 10) * G, Fr(int(vg), 10) * G, Fr(int(vc), 10) * G))
    return rows


def test_oracle_benefit_hand_computed_on_the_paper_table():
    # development server, n = 1: B_c2g = 22 GB/s, B_g2c = 16 GB/s, V_g = 50, V_c = 5 G elements/s; per element (C = 1):
    #   I = 1/2 (2/16e9 + 2/22e9) = 1/16e9 + 1/22e9 = 19/176e9
    #   J = 1/14 [ 4/22e9 + 2 I + 2/16e9 + 1/5e9 - 1/50e9 ] = 1/14 [ 2/11 + 19/88 + 1/8 + 9/50 ] / 1e9
    srv, n, c2g, g2c, vg, vc = paper_tables()[0]
    assert (srv, n) == ("dev", 1)
    I, J = orc.offload_benefit(1, 1, g2c, c2g, vg, vc)
    assert I == Fr(19, 176 * G)
    assert J == Fr(1, 14) * (Fr(2, 11) + Fr(19, 88) + Fr(1, 8) + Fr(9, 50)) / G
    assert I > J          # with these numbers one more cached block is worth more than one more uploaded chunk
    # both scale linearly with the chunk length
    I2, J2 = orc.offload_benefit(1, 1 << 20, g2c, c2g, vg, vc)
    assert I2 == I * (1 << 20) and J2 == J * (1 << 20)


def test_oracle_benefit_limits():
    # an infinitely fast link leaves only the update term; equal update velocities leave only traffic
    I, J = orc.offload_benefit(2, 100, 10 ** 30, 10 ** 30, 50 * G, 5 * G)
    assert float(I) < 1e-25 and float(J) == pytest.approx(2 / 14 * (100 / 5e9 - 100 / 50e9), rel=1e-12)
    I, J = orc.offload_benefit(1, 100, 16 * G, 22 * G, 7 * G, 7 * G)
    assert J == Fr(1, 14) * (Fr(400, 22 * G) + 2 * I + Fr(200, 16 * G))
    # a slower CPU update raises J and leaves I alone
    a = orc.offload_benefit(1, 100, 16 * G, 22 * G, 50 * G, 5 * G)
    b = orc.offload_benefit(1, 100, 16 * G, 22 * G, 50 * G, 1 * G)
    assert b[0] == a[0] and b[1] > a[1]


def test_product_benefit_matches_oracle_on_the_paper_tables_and_random_profiles():
    rng = np.random.default_rng(1)
    cases = [(n, 64 << 20, g2c, c2g, vg, vc) for _, n, c2g, g2c, vg, vc in paper_tables()]
    for _ in range(200):
        cases.append((int(rng.integers(1, 9)), int(rng.integers(1, 1 << 28)), *[Fr(float(x)) for x in rng.uniform(1e9, 1e12, size=4)]))
    for n, C, g2c, c2g, vg, vc in cases:
        I, J = orc.offload_benefit(n, C, g2c, c2g, vg, vc)
        gi, gj = ex.elixir_offload_benefit(n, C, float(g2c), float(c2g), float(vg), float(vc))
        assert gi == pytest.approx(float(I), rel=1e-13) and gj == pytest.approx(float(J), rel=1e-12)


def test_plan_brute_force_and_parity():
    """The rule is greedy on two constants, so it must (a) respect the budget, (b) give the preferred kind as much as
    fits before the other gets anything, (c) agree between oracle and product."""
    rng = np.random.default_rng(2)
    C = 1 << 20
    block, chunk = 2 * C, 14 * C
    for trial in range(300):
        n_chunks = int(rng.integers(0, 30))
        min_blocks = int(rng.integers(1, 5))
        budget = float(rng.integers(0, 40 * chunk))
        slow_cpu = trial % 2 == 0
        prof = dict(b_g2c=16e9, b_c2g=22e9, v_g=50e9, v_c=0.05e9 if slow_cpu else 5e9)
        I, J = orc.offload_benefit(1, C, prof["b_g2c"], prof["b_c2g"], prof["v_g"], prof["v_c"])
        assert (J > I) == slow_cpu
        blocks, up = orc.offload_plan(1, C, n_chunks, min_blocks, budget, **prof)
        assert (blocks, up) == ex.elixir_offload_plan(1, C, n_chunks, min_blocks, budget, **prof)
        base = max(1, min(min_blocks, n_chunks) if n_chunks else min_blocks)
        assert blocks >= base and 0 <= up <= n_chunks and blocks <= max(base, n_chunks)
        if budget >= base * block:
            assert blocks * block + up * chunk <= budget
            # brute force: among all feasible (blocks, up) the rule's answer maximises the preferred kind first
            feas = [(b, u) for b, u in itertools.product(range(base, max(base, n_chunks) + 1), range(n_chunks + 1))
                    if b * block + u * chunk <= budget]
            best = max(feas, key=(lambda t: (t[1], t[0])) if slow_cpu else (lambda t: (t[0], t[1])))
            assert (blocks, up) == best
        else:
            assert (blocks, up) == (base, 0)


def test_plan_with_this_box_profile():
    # measured here: 48.3 GB/s each way with both directions busy, GPU update 233 G elements/s, CPU update 13.9 G elements/s
    I, J = ex.elixir_offload_benefit(1, 128 << 20, 48.3e9, 48.3e9, 233e9, 13.9e9)
    assert I > J           # a fast host CPU makes uploading a chunk's update worth less than caching a block
    blocks, up = ex.elixir_offload_plan(1, 128 << 20, 152, 1, 100e9, 48.3e9, 48.3e9, 233e9, 13.9e9)
    assert blocks == 152 and up == (100e9 - 152 * 2 * (128 << 20)) // (14 * (128 << 20))


def test_benefit_errors():
    for args in ((0, 1, 1e9, 1e9, 1e9, 1e9), (1, 0, 1e9, 1e9, 1e9, 1e9), (1, 1, 0.0, 1e9, 1e9, 1e9), (1, 1, 1e9, 1e9, 1e9, -1.0)):
        with pytest.raises(ex.ElixirError) as e:
            ex.elixir_offload_benefit(*args)
        assert e.value.code == ex.ELIXIR_EINVAL
    with pytest.raises(ex.ElixirError):
        ex.elixir_offload_plan(1, 1, -1, 1, 1e9, 1e9, 1e9, 1e9, 1e9)


def test_product_plan_on_the_paper_rows_follows_the_larger_benefit():
    """The decision rule after Eq. 2 on the paper's own App. B.1 numbers, through the product: on both servers at n = 1
    I > J (a cached block is worth more than an uploaded chunk), so spare memory goes to rCache blocks first and chunks
    only get what is left; where J > I it is the other way round."""
    C, n_chunks = 64 << 20, 40
    for srv, n, c2g, g2c, vg, vc in paper_tables():
        I, J = ex.elixir_offload_benefit(n, C, float(g2c), float(c2g), float(vg), float(vc))
        if n == 1:
            assert I > J, (srv, n)
        # memory for the mandatory block plus five more blocks' worth: at n = 1 that is 5 blocks (10 C bytes) and no chunk,
        # since a chunk costs 14 C / n bytes
        allowed = 2.0 * C * 6
        blocks, chunks = ex.elixir_offload_plan(n, C, n_chunks, 1, allowed, float(g2c), float(c2g), float(vg), float(vc))
        assert (blocks, chunks) == tuple(orc.offload_plan(n, C, n_chunks, 1, int(allowed), g2c, c2g, vg, vc))
        if I > J:
            assert blocks == 6 and chunks == 0
        else:
            assert chunks == int(10 * C // (14 * C // n)) and blocks == 1 + (10 * C - chunks * (14 * C // n)) // (2 * C)
