"""Helpers shared by the GPU parity tests (no method arithmetic here)."""
from concurrent.futures import ThreadPoolExecutor
import os

import numpy as np

from oracle import elixir_oracle as orc

HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def n_threads():
    return max(1, min(16, len(os.sched_getaffinity(0))))


def oracle_adam_parallel(p, m, v, g, out, *, step, grad_scale=1.0, hp=HP, threads=None):
    """The oracle's AdamW over slices of one chunk on several host threads (the update is elementwise)."""
    threads = threads or n_threads()
    n = p.size
    if n < (1 << 16) or threads == 1:
        orc.chunk_adam_step(p, m, v, g, out, step=step, grad_scale=grad_scale, **hp)
        return
    edges = np.linspace(0, n, threads + 1).astype(np.int64)

    def work(i):
        a, b = int(edges[i]), int(edges[i + 1])
        orc.chunk_adam_step(p[a:b], m[a:b], v[a:b], g[a:b], None if out is None else out[a:b], step=step,
                            grad_scale=grad_scale, **hp)

    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(work, range(threads)))


def sign_magnitude(bits_u16):
    """bf16 patterns on a line where neighbouring values differ by 1 (for the 1-ulp check)."""
    b = bits_u16.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b)


F32_FULL_PRECISION_MIN = 2.0 ** -102      # above this an fp32 value and its neighbours are normal numbers (2^-126 * 2^24)


def check_adam_close(got_p, got_m, got_v, ref_p, ref_m, ref_v, *, lr, gmax, steps=1, what="", hp=HP):
    """The fp32 state against the oracle's, element by element, at relative 1e-6:
      v: |err| <= 1e-6 * |ref| -- purely relative (v is a sum of non-negative terms, nothing cancels); only below the
         range where fp32 has its full precision an absolute 1e-6 * 2^-102 is allowed, and a zero stays exactly zero;
      m: |err| <= 1e-6 * (|ref| + (1 - beta1) * max|g|): where m cancels to ~0 a relative bound is meaningless, and the
         floor is the size of ONE update's contribution, whatever the number of steps;
      p: |err| <= 1e-6 * (|ref| + steps * lr): an update moves a weight by at most ~lr, its fp32 arithmetic (constants
         rounded to fp32, 1-ulp sqrt and rcp, fp32 m and v) is good to ~3e-7 of that, and the errors of `steps` updates add.
    Returns diagnostics in units of 1e-6: "p", "m", "v" = the largest err / bound (<= 1 by the assertions) and "p1" = the
    same for p with the floor of a single update (lr), to show how far the result is from a bound that does not grow with
    the number of steps."""
    b1 = hp["beta1"]
    out = {}
    for name, got, ref, floor in (("p", got_p, ref_p, steps * lr), ("m", got_m, ref_m, (1.0 - b1) * gmax),
                                  ("v", got_v, ref_v, F32_FULL_PRECISION_MIN)):
        got64, ref64 = got.astype(np.float64), ref.astype(np.float64)
        err = np.abs(got64 - ref64)
        scale = np.abs(ref64) + floor if name != "v" else np.maximum(np.abs(ref64), floor)
        bad = ~(err <= 1e-6 * scale)
        assert not bad.any(), (f"{what} {name}: {int(bad.sum())} of {bad.size} elements outside tolerance; worst "
                               f"err {err[bad].max():.3e} at ref {ref64[bad][np.argmax(err[bad])]:.6e} (floor {floor:.3e})")
        out[name] = float((err / scale).max(initial=0.0)) * 1e6
        if name == "p":
            out["p1"] = float((err / (np.abs(ref64) + lr)).max(initial=0.0)) * 1e6
    assert not got_v[ref_v == 0].any(), f"{what} v: a variance the oracle leaves at exactly 0 moved"
    return out


def check_bf16_copy(got_bits, got_p, ref_bits, ref_p, *, lr, steps=1, what="", fmt=0):
    """The low-precision copy (fmt 0 = bf16, 1 = fp16): (a) it is exactly the round-to-nearest-even rounding of the fp32
    master the GPU stored (checked bit for bit with the oracle's rounding); (b) it is within one low-precision ulp of
    the oracle's copy wherever |p| is large enough for an ulp to exceed the fp32 tolerance (below that the master
    weight is a cancellation residue and only (a) and the fp32 bound apply)."""
    conv = orc.f32_to_f16 if fmt else orc.f32_to_bf16
    own = conv(np.ascontiguousarray(got_p))
    finite = np.isfinite(got_p)
    assert np.array_equal(got_bits[finite], own[finite]), f"{what}: low-precision copy is not the RNE rounding of the stored master weight"
    big = np.abs(ref_p) > (1e-2 if fmt else 1e-3) * steps * lr
    d = np.abs(sign_magnitude(got_bits[big]) - sign_magnitude(ref_bits[big]))
    assert d.max(initial=0) <= 1, f"{what}: low-precision copy differs by {int(d.max())} ulp"
    return float((got_bits == ref_bits).mean()) if got_bits.size else 1.0
