"""The seeded input recipe (synth/gen.py, host side): the value distribution, the exact-zero lane, the property that
any slice can be regenerated on its own, and the GPT-2-shaped tensor lists.  No method arithmetic is involved."""
import numpy as np
import pytest

from synth import gen


def test_value_distribution_of_the_generator():
    n = 1 << 21
    x = gen.fill_f32(gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM), 0, n, 0.02).astype(np.float64)
    assert abs(x.mean()) < 4 * 0.02 / np.sqrt(n)
    assert x.std() == pytest.approx(0.02, rel=5e-3)
    assert np.abs(x).max() <= 0.02 * 2 * 65535 / gen.IRWIN_HALL_STD * 1.0001      # Irwin-Hall of four 16-bit fields: bounded at +-3.46 sigma
    assert (np.abs(x) < 0.02).mean() == pytest.approx(0.68, abs=0.02)              # bell-shaped, not uniform
    # mixed signs and magnitudes, no duplicates to speak of
    assert 0.49 < (x > 0).mean() < 0.51 and np.unique(x).size > 0.5 * n / 100


@pytest.mark.parametrize("zero_pct", [0, 1, 37])
def test_exact_zero_lane(zero_pct):
    n = 1 << 20
    g = gen.fill_bf16(gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, 0, 2), 0, n, 1e-3, zero_pct=zero_pct)
    zeros = (g == 0).mean()                      # +0 bit pattern
    # the forced zeros plus the values that truncate to zero by themselves (|x| below the smallest bf16 step around 0: none at this sigma)
    assert zeros == pytest.approx(zero_pct / 100, abs=2e-3)
    assert not (g == 0x8000).any() or zero_pct == 0


def test_any_slice_regenerates_on_its_own_and_blocks_do_not_matter():
    key = gen.stream_key(7, gen.TAG_GRAD, 3, 2, 4)
    whole = gen.fill_bf16(key, 1000, 100_000, 1e-3, zero_pct=1)
    for a, n in ((0, 1), (1, 4097), (12345, 50_000), (99_999, 1)):
        assert np.array_equal(gen.fill_bf16(key, 1000 + a, n, 1e-3, zero_pct=1), whole[a:a + n])
    assert np.array_equal(gen.fill_bf16(key, 1000, 100_000, 1e-3, zero_pct=1, block=777), whole)
    w32 = gen.fill_f32(key, 5, 10_000, 0.02)
    assert np.array_equal(gen.fill_f32(key, 5 + 300, 700, 0.02), w32[300:1000])
    # beyond 2^32 elements the index still matters (the 20B set has 2e10 elements)
    far = gen.fill_f32(key, (1 << 34) + 5, 1000, 0.02)
    assert not np.array_equal(far, w32[:1000]) and not np.array_equal(far, gen.fill_f32(key, 5 + (1 << 32), 1000, 0.02))


def test_streams_of_different_steps_micro_batches_and_kinds_are_unrelated():
    n = 200_000
    base = gen.fill_f32(gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, 0, 2), 0, n, 1.0).astype(np.float64)
    for other in (gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 2, 0, 2), gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, 1, 2),
                  gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, 1, 0, 2), gen.stream_key(gen.BASE_SEED + 1, gen.TAG_GRAD, 1, 0, 2),
                  gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, 0, 3)):
        y = gen.fill_f32(other, 0, n, 1.0).astype(np.float64)
        assert abs(np.corrcoef(base, y)[0, 1]) < 0.01
    assert gen.stream_key(1, 2, 3, 4, 5) == gen.stream_key(1, 2, 3, 4, 5)           # a pure function of its arguments
    shifted = gen.fill_f32(gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, 0, 2), 1, n - 1, 1.0).astype(np.float64)
    assert abs(np.corrcoef(base[:-1], shifted)[0, 1]) < 0.01                        # neighbours are unrelated too


def test_gpt2_shaped_tensor_lists():
    # (layers, hidden, vocab) -> total = (V + P) h + L (12 h^2 + 13 h) + 2 h with P = 1024
    for (L, h, V), total, tensors in (((2, 768, 8192), 21_255_168, 28), ((48, 1600, 50257), 1_557_611_200, 580),
                                      ((48, 3200, 50257), 6_064_342_400, 580), ((64, 5120, 50257), 20_399_488_000, 772)):
        lst = gen.gpt2_tensor_list(L, h, V)
        numels = [n for _, n in lst]
        assert len(lst) == tensors and sum(numels) == total == (V + 1024) * h + L * (12 * h * h + 13 * h) + 2 * h
        assert numels[0] == V * h and numels[1] == 1024 * h and numels[-2:] == [h, h]
        assert all(n % 64 == 0 for n in numels)                                     # tight packing keeps every tensor 128-bit aligned
        assert max(numels[2:]) == 4 * h * h
    assert [c.name for c in gen.CONFIGS.values()] and gen.CONFIGS["gpt2_1p5b"].chunk_elems == 64 * gen.Mi
    assert gen.SWEEP_CHUNK_ELEMS == [m * gen.Mi for m in (8, 16, 32, 64, 128, 256)]
