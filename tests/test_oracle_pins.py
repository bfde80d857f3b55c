"""Pins for the CPU oracle (no GPU): every oracle function is checked against something that is
not the oracle itself -- closed forms, brute force with exact rationals, IEEE fp32 arithmetic done
by numpy, hand-worked fixtures, and torch.optim.AdamW on the CPU as the library special case."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import elixir_oracle as orc
from synth import gen

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
F32 = np.float32
HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def f32d(x):
    """the double value of x after rounding to fp32 (what a float argument becomes)."""
    return float(F32(x))


def ulp_diff_f32(a, b):
    """distance in fp32 grid steps between arrays a and b (same-sign or tiny values)."""
    ia = a.view(np.int32).astype(np.int64)
    ib = b.view(np.int32).astype(np.int64)
    ia = np.where(ia < 0, -(ia & 0x7FFFFFFF), ia)
    ib = np.where(ib < 0, -(ib & 0x7FFFFFFF), ib)
    return np.abs(ia - ib)


def read_fixture(name):
    d = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            d[k] = [int(x) for x in v]
    return d


# --------------------------------------------------------------------------- bf16

def test_bf16_roundtrip_exhaustive():
    bits = np.arange(65536, dtype=np.uint16)
    f = orc.bf16_to_f32(bits)
    # widening = appending 16 zero bits
    assert np.array_equal(f.view(np.uint32), bits.astype(np.uint32) << 16)
    back = orc.f32_to_bf16(f)
    nan = np.isnan(f)
    assert np.array_equal(back[~nan], bits[~nan])
    assert np.all(np.isnan(orc.bf16_to_f32(back[nan])))


def test_bf16_ties_to_even_and_specials():
    u = np.array([0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF, 0x7F7FFFFF, 0x7F800000, 0xFF800000,
                  0x7FC00001, 0x7F800001, 0x00000000, 0x80000000, 0x00008000, 0x00018000], dtype=np.uint32)
    want = np.array([0x3F80, 0x3F82, 0x3F81, 0x3F80, 0x7F80, 0x7F80, 0xFF80,
                     0x7FC0, 0x7FC0, 0x0000, 0x8000, 0x0000, 0x0002], dtype=np.uint16)
    got = orc.f32_to_bf16(u.view(np.float32))
    assert np.array_equal(got, want)


def test_bf16_rne_matches_nearest_neighbour_brute_force():
    rng = np.random.default_rng(7)
    u = rng.integers(0, 1 << 32, size=1_000_000, dtype=np.uint64).astype(np.uint32)
    x = u.view(np.float32)
    finite = np.isfinite(x)
    u, x = u[finite], x[finite]
    got = orc.f32_to_bf16(x)
    # the two bf16 neighbours of x: truncation (towards zero) and the next pattern away from zero
    lo = (u >> 16).astype(np.uint32)
    hi = lo + 1
    xd = x.astype(np.float64)
    lod = (lo << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    hi_bits = (hi << 16).astype(np.uint32)
    hi_is_inf = (hi_bits & 0x7FFFFFFF) == 0x7F800000
    # for the comparison an overflowing neighbour counts as 2^128 (the value the grid would continue with)
    hid = np.where(hi_is_inf, np.sign(xd) * 2.0 ** 128, hi_bits.view(np.float32).astype(np.float64))
    dlo, dhi = np.abs(xd - lod), np.abs(hid - xd)
    want = np.where(dlo < dhi, lo, np.where(dhi < dlo, hi, np.where(lo & 1 == 0, lo, hi))).astype(np.uint16)
    assert np.array_equal(got, want)


# --------------------------------------------------------------------------- layout

def test_paper_byte_accounting():
    fx = read_fixture("paper_model_state_bytes.txt")
    assert fx["L_c"][0] == np.dtype(np.uint16).itemsize                      # low-precision params / grads
    assert fx["L_os"][0] * fx["F_os"][0] == 3 * np.dtype(np.float32).itemsize == fx["optimizer_state_bytes_per_element"][0]
    # a chunk pair of C elements: L_c*C + L_os*F_os*C bytes (N = 1)
    C = 4 * gen.Mi
    assert fx["L_c"][0] * C + fx["L_os"][0] * fx["F_os"][0] * C == 14 * C


def test_layout_hand_case():
    fx = read_fixture("layout_hand_case.txt")
    cid, off, valid = orc.layout_plan(fx["numel"], fx["chunk_elems"][0], orc.NEXT_FIT)
    assert cid == fx["chunk_id"] and off == fx["offset"] and valid == fx["valid_len"]
    assert len(valid) * fx["chunk_elems"][0] - sum(valid) == fx["padding"][0]


def test_layout_hand_cases_other_policies():
    # first-fit: the 2 goes back into chunk 1 (room 4) instead of behind the oversize tail
    cid, off, valid = orc.layout_plan([3, 5, 4, 9, 2], 8, orc.FIRST_FIT)
    assert (cid, off, valid) == ([0, 0, 1, 2, 1], [0, 3, 0, 0, 4], [8, 6, 8, 1])
    # dense: one running position, 23 elements -> 3 chunks, only the last padded
    cid, off, valid = orc.layout_plan([3, 5, 4, 9, 2], 8, orc.DENSE)
    assert (cid, off, valid) == ([0, 0, 1, 1, 2], [0, 3, 0, 4, 5], [8, 8, 7])
    # alignment 4: starts rounded up
    cid, off, valid = orc.layout_plan([3, 5, 4], 16, orc.NEXT_FIT, align=4)
    assert (cid, off, valid) == ([0, 0, 0], [0, 4, 12], [16])


def _occupancy(numels, C, cid, off, n_chunks):
    occ = np.zeros(n_chunks * C, dtype=np.int32)
    for i, n in enumerate(numels):
        a = cid[i] * C + off[i]
        occ[a:a + n] += 1
    return occ


@pytest.mark.parametrize("policy", [orc.NEXT_FIT, orc.FIRST_FIT, orc.DENSE])
def test_layout_invariants_random(policy):
    rng = np.random.default_rng(policy + 11)
    for trial in range(60):
        C = int(rng.integers(4, 64))
        numels = [int(x) for x in rng.integers(0, 3 * C, size=rng.integers(1, 40))]
        cid, off, valid = orc.layout_plan(numels, C, policy)
        occ = _occupancy(numels, C, cid, off, len(valid))
        assert occ.max(initial=0) <= 1, "slices overlap"
        assert occ.sum() == sum(numels)
        for c, v in enumerate(valid):
            assert 0 <= v <= C
            assert occ[c * C + v:(c + 1) * C].sum() == 0, "element beyond valid_len"
        starts = [cid[i] * C + off[i] for i in range(len(numels))]
        if policy != orc.FIRST_FIT:
            assert starts == sorted(starts), "order of use not preserved"
        if policy == orc.DENSE:
            assert occ[:sum(numels)].all()
        else:
            for i, n in enumerate(numels):
                if n <= C:
                    assert off[i] + n <= C, "a parameter that fits in a chunk must not straddle"
                else:
                    assert off[i] == 0


def test_layout_next_fit_is_brute_force_simulation():
    # independent simulation on an explicit cell grid: put each parameter right behind the
    # previous one if it fits before the next chunk boundary, else at the next boundary.
    rng = np.random.default_rng(5)
    for _ in range(50):
        C = int(rng.integers(3, 40))
        numels = [int(x) for x in rng.integers(1, 2 * C, size=30)]
        cid, off, _ = orc.layout_plan(numels, C, orc.NEXT_FIT)
        pos, opened = 0, False
        for i, n in enumerate(numels):
            boundary = -(-pos // C) * C
            room = boundary - pos if opened else 0
            if n > C or n > room:
                pos = boundary
            opened = True
            assert (pos // C, pos % C) == (cid[i], off[i])
            pos += n


def test_layout_table_regression_and_paper_waste_claim():
    rows = {}
    with open(os.path.join(GOLD, "layout_table.txt")) as f:
        for line in f:
            if line.startswith("#"):
                continue
            name, C, pol, n_chunks, pad = line.split()
            rows[(name, int(C), int(pol))] = (int(n_chunks), int(pad))
    for (name, C, pol), (n_chunks, pad) in rows.items():
        cfg = gen.CONFIGS[name]
        _, _, valid = orc.layout_plan(cfg.numels(), C, pol)
        assert (len(valid), len(valid) * C - sum(valid)) == (n_chunks, pad)
        assert sum(valid) == cfg.total_params()
    # the paper reports a packing waste below 4% at the searched chunk size (Sec. 4): the sweep must contain one
    best = min(pad / (n * C) for (name, C, pol), (n, pad) in rows.items() if name == "gpt2_1p5b" and pol == orc.NEXT_FIT)
    assert best < 0.04
    # parameter counts of the GPT-2-shaped sets: (V+P)h + L(12h^2+13h) + 2h
    assert gen.CONFIGS["tiny"].total_params() == 21_255_168
    assert gen.CONFIGS["gpt2_1p5b"].total_params() == 1_557_611_200


# --------------------------------------------------------------------------- pack / unpack

@pytest.mark.parametrize("dtype", [np.float32, np.uint16])
def test_pack_unpack_roundtrip_and_indexing(dtype):
    rng = np.random.default_rng(3)
    numels = [5, 1, 17, 0, 64, 9]
    C = 128
    cid, off, valid = orc.layout_plan(numels, C, orc.NEXT_FIT)
    assert len(valid) == 1
    tensors = [rng.integers(1, 60000, size=n).astype(dtype) for n in numels]
    chunk = np.full(C, 77, dtype=dtype)
    orc.chunk_pack(chunk, tensors, off)
    covered = np.zeros(C, bool)
    for t, o in zip(tensors, off):
        assert np.array_equal(chunk[o:o + t.size].view(np.uint8), t.view(np.uint8))
        covered[o:o + t.size] = True
    assert not chunk[~covered].view(np.uint8).any(), "padding must be zero bits"
    outs = [np.zeros_like(t) for t in tensors]
    orc.chunk_unpack(chunk, outs, off)
    for a, b in zip(tensors, outs):
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8))
    with pytest.raises(ValueError):
        orc.chunk_pack(chunk, [np.zeros(4, dtype)], [C - 3])


def test_pack_preserves_nan_payloads_and_negative_zero():
    u = np.array([0x7FC01234, 0xFFFFFFFF, 0x80000000, 0x00000001, 0x7F800000], dtype=np.uint32)
    t = u.view(np.float32)
    chunk = np.ones(8, np.float32)
    orc.chunk_pack(chunk, [t], [2])
    assert np.array_equal(chunk.view(np.uint32), np.array([0, 0, *u, 0], dtype=np.uint32))


# --------------------------------------------------------------------------- gradient reduction

def test_reduce_first_microbatch_is_exact_widening():
    bits = np.arange(65536, dtype=np.uint16)
    bits = bits[~np.isnan(orc.bf16_to_f32(bits))]
    g = np.full(bits.size + 10, 123.0, np.float32)
    orc.grad_reduce_into_chunk(g, 7, bits, 1.0, accumulate=False)
    # 0 + (-0) is +0 in IEEE arithmetic: the only pattern the first micro-batch does not keep
    want = np.where(bits == 0x8000, 0, bits.astype(np.uint32) << 16).astype(np.uint32)
    assert np.array_equal(g[7:7 + bits.size].view(np.uint32), want)
    assert np.all(g[:7] == 123.0) and np.all(g[7 + bits.size:] == 123.0)   # writes only its slice


@pytest.mark.parametrize("scale", [0.25, 1.0, 0.3])
def test_reduce_matches_sequential_ieee_fp32_sum(scale):
    # numpy float32 multiply/add are correctly rounded IEEE operations: an independent route to
    # fl32(acc + fl32(scale*g)) applied micro-batch by micro-batch in index order
    n, K = 4099, 4
    key = [gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, mb) for mb in range(K)]
    mbs = [gen.fill_bf16(k, 0, n, 1e-3, zero_pct=1) for k in key]
    got = np.full(n + 5, -1.0, np.float32)
    want = np.zeros(n, np.float32)
    for mb in range(K):
        orc.grad_reduce_into_chunk(got, 3, mbs[mb], scale, accumulate=mb > 0)
        gf = (mbs[mb].astype(np.uint32) << 16).view(np.float32)
        want = (want + F32(scale) * gf).astype(np.float32) if mb > 0 else (F32(0) + F32(scale) * gf).astype(np.float32)
    assert np.array_equal(got[3:3 + n].view(np.uint32), want.view(np.uint32))
    assert np.all(got[:3] == -1.0) and np.all(got[3 + n:] == -1.0)


def test_reduce_order_matters_only_through_rounding():
    # sum of 4 microbatches equals the exact rational sum to within 3 fp32 roundings
    n = 257
    mbs = [gen.fill_bf16(gen.stream_key(1, gen.TAG_GRAD, 0, mb), 0, n, 1e-3) for mb in range(4)]
    got = np.zeros(n, np.float32)
    for mb in range(4):
        orc.grad_reduce_into_chunk(got, 0, mbs[mb], 0.25, accumulate=mb > 0)
    for k in range(0, n, 16):
        exact = sum(Fraction(float(orc.bf16_to_f32(m[k:k + 1])[0])) for m in mbs) / 4
        assert abs(Fraction(float(got[k])) - exact) <= 3 * Fraction(2) ** -24 * max(abs(Fraction(float(orc.bf16_to_f32(m[k:k + 1])[0]))) for m in mbs)


# --------------------------------------------------------------------------- norm / clip

def test_norm_brute_force_exact_rationals():
    rng = np.random.default_rng(0)
    chunks = [rng.standard_normal(13).astype(np.float32) * F32(1e-3), rng.standard_normal(8).astype(np.float32)]
    valid = [11, 5]
    exact = sum(Fraction(float(x)) ** 2 for c, v in zip(chunks, valid) for x in c[:v])
    want = math.sqrt(exact)
    got = orc.grad_norm(chunks, valid)
    assert abs(got - want) <= 1e-14 * want
    # fsum of float squares as a second, independent route
    assert abs(got - math.sqrt(math.fsum(float(x) * float(x) for c, v in zip(chunks, valid) for x in c[:v]))) <= 1e-14 * want


def test_norm_closed_forms():
    n = 100_003
    c = F32(-0.0123)
    assert orc.grad_norm([np.full(n, c, np.float32)], [n]) == pytest.approx(abs(float(c)) * math.sqrt(n), rel=n * 2.0 ** -53)  # sequential double sum
    one_hot = np.zeros(n, np.float32)
    one_hot[77] = F32(-3.5)
    assert orc.grad_norm([one_hot], [n]) == 3.5
    # 3-4-5
    assert orc.grad_norm([np.array([3, 0], np.float32), np.array([4, 100], np.float32)], [2, 1]) == 5.0
    # padding (beyond valid_len) does not count
    a = np.array([1, 2, 2, 1e30], np.float32)
    assert orc.grad_norm([a], [3]) == 3.0
    assert orc.grad_norm([], []) == 0.0


def test_norm_partition_invariance():
    x = gen.fill_f32(gen.stream_key(2, gen.TAG_MISC), 0, 50_000, 1e-3)
    whole = orc.grad_norm([x], [x.size])
    parts = [np.ascontiguousarray(x[a:a + 7777]) for a in range(0, x.size, 7777)]
    split = orc.grad_norm(parts, [p.size for p in parts])
    assert abs(whole - split) <= 1e-12 * whole


def test_clip_coef():
    assert orc.clip_coef(0.5, 1.0) == 1.0                       # below max-norm: clamp to 1
    assert orc.clip_coef(1.0 - 1e-6, 1.0) == 1.0
    assert orc.clip_coef(38.9, 1.0) == pytest.approx(1.0 / (38.9 + 1e-6), rel=1e-15)
    assert orc.clip_coef(38.9, 1.0) * 38.9 == pytest.approx(1.0, rel=1e-6)
    assert orc.clip_coef(38.9, 0.0) == 1.0 and orc.clip_coef(38.9, -1.0) == 1.0   # no clipping requested
    assert orc.clip_coef(4.0, 2.0) == pytest.approx(2.0 / (4.0 + 1e-6), rel=1e-15)


# --------------------------------------------------------------------------- AdamW

def _state(n, seed=0, zero_moments=True):
    p = gen.fill_f32(gen.stream_key(seed, gen.TAG_PARAM), 0, n, 0.02)
    g = gen.fill_bf16(gen.stream_key(seed, gen.TAG_GRAD, 1), 0, n, 1e-3, zero_pct=1)
    if zero_moments:
        m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
    else:
        m = gen.fill_f32(gen.stream_key(seed, gen.TAG_MOMENT, 0), 0, n, 3e-4)
        v = np.square(gen.fill_f32(gen.stream_key(seed, gen.TAG_MOMENT, 1), 0, n, 1e-3)) + F32(1e-12)
    return p, m, v, g


def test_adam_first_step_closed_form():
    # m = v = 0, t = 1: m_hat = g, v_hat = g^2, so p1 = p0 (1 - lr wd) - lr g / (|g| + eps)
    n = 5000
    for wd in (0.0, 0.01):
        p, m, v, g = _state(n)
        p0 = p.copy()
        gf = orc.bf16_to_f32(g).astype(np.float64)
        hp = dict(HP, weight_decay=wd)
        out = np.zeros(n, np.uint16)
        orc.chunk_adam_step(p, m, v, g, out, step=1, **hp)
        lr, eps, b1, b2 = f32d(hp["lr"]), f32d(hp["eps"]), f32d(hp["beta1"]), f32d(hp["beta2"])
        want = p0.astype(np.float64) * (1 - lr * f32d(wd)) - lr * gf / (np.abs(gf) + eps)
        assert ulp_diff_f32(p, want.astype(np.float32)).max() <= 1
        assert (ulp_diff_f32(p, want.astype(np.float32)) == 0).mean() > 0.999
        assert ulp_diff_f32(m, ((1 - b1) * gf).astype(np.float32)).max() <= 1
        assert ulp_diff_f32(v, ((1 - b2) * gf * gf).astype(np.float32)).max() <= 1
        # with wd = 0 a zero gradient leaves the parameter untouched, a non-zero one moves it by ~lr against g
        if wd == 0.0:
            assert np.array_equal(p[gf == 0], p0[gf == 0])
            big = np.abs(gf) > 1e-4
            moved = p.astype(np.float64)[big] - p0.astype(np.float64)[big]
            assert np.all(np.sign(moved) == -np.sign(gf[big]))
            assert np.allclose(np.abs(moved), lr, rtol=1e-3)
        # low-precision copy is the rounding of the stored fp32 master
        assert np.array_equal(out, orc.f32_to_bf16(p))


def test_adam_constant_gradient_many_steps():
    # g_t = g: m_t = (1-b1^t) g, v_t = (1-b2^t) g^2, every step moves p by lr g / (|g| + eps)
    n, T = 2000, 25
    p, m, v, g = _state(n, seed=3)
    p0 = p.astype(np.float64)
    gf = orc.bf16_to_f32(g).astype(np.float64)
    hp = dict(HP, weight_decay=0.0)
    lr, eps, b1, b2 = f32d(hp["lr"]), f32d(hp["eps"]), f32d(hp["beta1"]), f32d(hp["beta2"])
    for t in range(1, T + 1):
        orc.chunk_adam_step(p, m, v, g, None, step=t, **hp)
        assert np.allclose(m, (1 - b1 ** t) * gf, rtol=3e-7 * 3, atol=0)
        assert np.allclose(v, (1 - b2 ** t) * gf * gf, rtol=3e-7 * 3, atol=0)
    want = p0 - T * lr * gf / (np.abs(gf) + eps)
    # T roundings of p to fp32, each at most half an ulp of |p| <= ~0.1
    assert np.max(np.abs(p.astype(np.float64) - want)) <= T * 2.0 ** -24 * 0.13
    # a wrong step count in the bias correction (t-1 or t+1) would move p by a different amount per step:
    # relative to the travelled distance T*lr the error must be far below 1/T
    nz = np.abs(gf) > 1e-5
    travelled = np.abs(p.astype(np.float64) - p0)[nz]
    assert np.allclose(travelled, T * lr, rtol=2e-3)


def test_adam_zero_gradient_invariants():
    n = 3000
    p, m, v, _ = _state(n, seed=4)
    g0 = np.zeros(n, np.uint16)
    p0 = p.copy()
    hp = dict(HP, weight_decay=0.0)
    for t in (1, 2, 3):
        orc.chunk_adam_step(p, m, v, g0, None, step=t, **hp)
    assert np.array_equal(p.view(np.uint32), p0.view(np.uint32))
    assert not m.view(np.uint32).any() and not v.view(np.uint32).any()
    # non-zero moments decay by exactly beta (one fp32 rounding)
    p, m, v, _ = _state(n, seed=5, zero_moments=False)
    m0, v0 = m.astype(np.float64), v.astype(np.float64)
    orc.chunk_adam_step(p, m, v, np.zeros(n, np.float32), None, step=7, **hp)
    assert np.array_equal(m, (f32d(0.9) * m0).astype(np.float32))
    assert np.array_equal(v, (f32d(0.999) * v0).astype(np.float32))
    # weight decay alone: p_T = p_0 (1 - lr wd)^T
    p, m, v, _ = _state(n, seed=6)
    p0 = p.astype(np.float64)
    T = 50
    hp = dict(HP, weight_decay=0.1, lr=1e-2)
    for t in range(1, T + 1):
        orc.chunk_adam_step(p, m, v, g0, None, step=t, **hp)
    want = p0 * (1 - f32d(1e-2) * f32d(0.1)) ** T
    assert np.allclose(p, want, rtol=T * 6e-8, atol=0)
    # padding invariant: all-zero state stays all-zero bits with weight decay on
    z = [np.zeros(64, np.float32) for _ in range(3)]
    out = np.ones(64, np.uint16)
    orc.chunk_adam_step(z[0], z[1], z[2], np.zeros(64, np.uint16), out, step=3, **HP)
    assert not any(a.view(np.uint32).any() for a in z) and not out.any()


def test_adam_sign_symmetry_bitwise():
    n = 4000
    p, m, v, g = _state(n, seed=8, zero_moments=False)
    gf = orc.bf16_to_f32(g)
    p2, m2, v2, g2 = -p, -m, v.copy(), -gf
    o1, o2 = np.zeros(n, np.uint16), np.zeros(n, np.uint16)
    orc.chunk_adam_step(p, m, v, gf, o1, step=4, **HP)
    orc.chunk_adam_step(p2, m2, v2, g2, o2, step=4, **HP)
    assert np.array_equal((-p2).view(np.uint32), p.view(np.uint32))
    assert np.array_equal((-m2).view(np.uint32), m.view(np.uint32))
    assert np.array_equal(v2.view(np.uint32), v.view(np.uint32))
    assert np.array_equal(o1 ^ np.uint16(0x8000), o2)


def test_adam_bf16_and_fp32_gradient_inputs_agree_and_grad_scale():
    n = 1000
    p, m, v, g = _state(n, seed=9, zero_moments=False)
    a = [p.copy(), m.copy(), v.copy()]
    b = [p.copy(), m.copy(), v.copy()]
    orc.chunk_adam_step(*a, g, None, step=2, **HP)
    orc.chunk_adam_step(*b, orc.bf16_to_f32(g), None, step=2, **HP)
    for x, y in zip(a, b):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    # grad_scale = 0.5 on g equals grad_scale = 1 on g/2 (exact halving)
    c = [p.copy(), m.copy(), v.copy()]
    d = [p.copy(), m.copy(), v.copy()]
    orc.chunk_adam_step(*c, orc.bf16_to_f32(g), None, step=2, grad_scale=0.5, **HP)
    orc.chunk_adam_step(*d, orc.bf16_to_f32(g) * F32(0.5), None, step=2, **HP)
    for x, y in zip(c, d):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    assert not np.array_equal(a[0], c[0])


def test_adam_matches_torch_adamw_single_steps():
    """Library special case: decoupled-weight-decay Adam as implemented by torch.optim.AdamW in float64
    on the CPU, started from the same stored fp32 state at an arbitrary step count."""
    torch = pytest.importorskip("torch")
    n = 4096
    for step, wd, seed in ((1, 0.01, 20), (2, 0.0, 21), (17, 0.1, 22), (1000, 0.01, 23)):
        p, m, v, g = _state(n, seed=seed, zero_moments=(step == 1))
        gf = orc.bf16_to_f32(g)
        hp = dict(HP, weight_decay=wd)
        tp = torch.nn.Parameter(torch.from_numpy(p.astype(np.float64)))
        opt = torch.optim.AdamW([tp], lr=f32d(hp["lr"]), betas=(f32d(hp["beta1"]), f32d(hp["beta2"])),
                                eps=f32d(hp["eps"]), weight_decay=f32d(wd), amsgrad=False, foreach=False)
        tp.grad = torch.from_numpy(gf.astype(np.float64))
        if step > 1:
            opt.state[tp] = {"step": torch.tensor(float(step - 1)),
                             "exp_avg": torch.from_numpy(m.astype(np.float64)),
                             "exp_avg_sq": torch.from_numpy(v.astype(np.float64))}
        opt.step()
        st = opt.state[tp]
        assert int(st["step"].item()) == step
        orc.chunk_adam_step(p, m, v, g, None, step=step, **hp)
        for got, want in ((p, tp.detach().numpy()), (m, st["exp_avg"].numpy()), (v, st["exp_avg_sq"].numpy())):
            d = ulp_diff_f32(got, want.astype(np.float32))
            assert d.max() <= 1 and (d == 0).mean() > 0.999


def test_adam_planted_mistakes_are_caught_by_the_closed_forms():
    """The closed forms above really discriminate: plausible wrong variants of the update, written out here
    in numpy, violate them.  (eps inside the square root's bias correction, decay applied after the step,
    bias correction with t-1.)"""
    lr, b1, b2, eps = 1e-4, 0.9, 0.999, 1e-8
    g = np.array([1e-3, -2e-3, 1e-7], np.float64)
    p0 = np.array([0.02, -0.01, 0.03], np.float64)
    closed = p0 - lr * g / (np.abs(g) + eps)

    def variant(eps_before_correction=False, t_off=0):
        m = (1 - b1) * g
        v = (1 - b2) * g * g
        t = 1 + t_off
        bc1, bc2 = 1 - b1 ** t, 1 - b2 ** t
        if eps_before_correction:
            return p0 - lr * (m / bc1) / ((np.sqrt(v) + eps) / math.sqrt(bc2))
        return p0 - lr * (m / bc1) / (np.sqrt(v / bc2) + eps)

    assert np.allclose(variant(), closed, rtol=1e-12)
    assert not np.allclose(variant(eps_before_correction=True), closed, rtol=1e-7)   # differs where |g| ~ eps
    assert not np.allclose(variant(t_off=1), closed, rtol=1e-3)


# --------------------------------------------------------------------------- fp16 (the paper's format) and loss scaling

def test_f16_conversions_against_numpy_float16():
    """numpy's float16 is IEEE binary16 with round-to-nearest-even conversions: an independent implementation."""
    bits = np.arange(65536, dtype=np.uint16)
    f = orc.f16_to_f32(bits)
    ref = bits.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(f[~nan].view(np.uint32), ref[~nan].view(np.uint32)) and np.all(np.isnan(f[nan]))
    assert np.array_equal(orc.f32_to_f16(f)[~nan], bits[~nan])
    rng = np.random.default_rng(11)
    x = rng.integers(0, 1 << 32, size=1_000_000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    y = (rng.standard_normal(1_000_000) * np.float32(10.0) ** rng.integers(-9, 6, size=1_000_000)).astype(np.float32)
    for v in (x[np.isfinite(x)], y):
        with np.errstate(over="ignore"):
            want = v.astype(np.float16).view(np.uint16)
        assert np.array_equal(orc.f32_to_f16(v), want)
    # ties to even, overflow threshold, subnormals, specials
    cases = {1.0 + 2.0 ** -11: 0x3C00, 1.0 + 3 * 2.0 ** -11: 0x3C02, 65504.0: 0x7BFF, 65519.996: 0x7BFF, 65520.0: 0x7C00,
             2.0 ** -24: 0x0001, 2.0 ** -25: 0x0000, 1.5 * 2.0 ** -24: 0x0002, -0.0: 0x8000, float("inf"): 0x7C00, -float("inf"): 0xFC00}
    for val, want in cases.items():
        assert int(orc.f32_to_f16(np.array([val], np.float32))[0]) == want, val
    assert np.isnan(orc.f16_to_f32(orc.f32_to_f16(np.array([np.nan], np.float32))))[0]


def test_f16_reduce_and_adam_variants():
    n = 3000
    bits = np.random.default_rng(12).integers(0, 0x7C00, size=n).astype(np.uint16)       # finite positive fp16 patterns
    bits[::2] |= 0x8000
    g = np.zeros(n, np.float32)
    orc.grad_reduce_into_chunk(g, 0, bits, 1.0, False, fmt=orc.FP16)
    assert np.array_equal(g, bits.view(np.float16).astype(np.float32) + np.float32(0))
    # fp16 gradients and fp32 gradients of the same values give the same update; the copy is the fp16 rounding of p
    p, m, v, _ = _state(n, seed=30)
    gh = (bits.view(np.float16).astype(np.float32) * np.float32(2.0 ** -8)).astype(np.float16)
    a, b = [p.copy(), m.copy(), v.copy()], [p.copy(), m.copy(), v.copy()]
    out = np.zeros(n, np.uint16)
    orc.chunk_adam_step(*a, gh.view(np.uint16), out, step=1, fmt=orc.FP16, **HP)
    orc.chunk_adam_step(*b, gh.astype(np.float32), None, step=1, **HP)
    for x, y in zip(a, b):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    assert np.array_equal(out, a[0].astype(np.float16).view(np.uint16))


def test_loss_scale_state_machine():
    # clean step: grad_scale = clip / S from the unscaled norm; counter advances
    s, good, skip, gs = orc.loss_scale_step(65536.0, 0, 65536.0 * 38.9, 1.0, growth_interval=3)
    assert (s, good, skip) == (65536.0, 1, False) and gs == pytest.approx(1.0 / (38.9 + 1e-6) / 65536.0, rel=1e-12)
    # no clipping requested, or norm below max-norm: pure unscaling
    assert orc.loss_scale_step(1024.0, 0, 1024.0 * 0.5, 1.0)[3] == 1.0 / 1024.0
    assert orc.loss_scale_step(1024.0, 0, 1e9, 0.0)[3] == 1.0 / 1024.0
    # overflow: skip, halve, reset
    assert orc.loss_scale_step(65536.0, 7, float("inf"), 1.0) == (32768.0, 0, True, 0.0)
    assert orc.loss_scale_step(65536.0, 7, float("nan"), 1.0) == (32768.0, 0, True, 0.0)
    # growth after `growth_interval` clean steps in a row
    s, good = 8.0, 0
    trace = []
    for norm in (1.0, 1.0, 1.0, float("inf"), 1.0, 1.0, 1.0, 1.0):
        s, good, skip, _ = orc.loss_scale_step(s, good, norm, 0.0, growth_interval=3)
        trace.append((s, good, skip))
    assert trace == [(8.0, 1, False), (8.0, 2, False), (16.0, 0, False), (8.0, 0, True), (8.0, 1, False), (8.0, 2, False),
                     (16.0, 0, False), (16.0, 1, False)]
