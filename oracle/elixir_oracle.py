"""CPU oracle for the chunked mixed-precision AdamW step -- TEST INFRASTRUCTURE ONLY.

Only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py`
may import this module.  It shares no code with the GPU library and never
imports it.  The floating-point work is done by the plain C file next to this
one (double precision internally, one rounding per stored value); the chunk
layout planner below is plain Python on integers.

Citations (paper = arXiv 2212.05339):
  * chunk definition and grouping of parameters into chunks: Sec. 3 "Chunk",
    App. A.2 "Grouping Method";
  * parameter chunk + optimizer chunk, one optimizer update per chunk pair:
    Sec. 4.1;
  * fp32 master weight rounded to low precision after the update, 2+2+12
    bytes per parameter: Sec. 2 "Mixed Precision Training".
Every function is pinned by tests in tests/test_oracle_pins.py,
tests/test_benefit_model.py and tests/test_rcache_sim.py (closed forms, brute
force, hand-worked cases under tests/golden/, a library special case); none
is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "elixir_oracle.c")
_SO = os.path.join(_HERE, "libelixir_oracle.so")

NEXT_FIT, FIRST_FIT, DENSE = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _SO)
    return _SO


_lib = None


def _L():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        vp, i64, f32, f64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_double, ctypes.c_int
        L.orc_bf16_to_f32_array.argtypes = [vp, vp, i64]
        L.orc_f32_to_bf16_array.argtypes = [vp, vp, i64]
        L.orc_chunk_pack.argtypes = [vp, i64, ci, vp, vp, vp, ci]
        L.orc_chunk_unpack.argtypes = [vp, i64, ci, vp, vp, vp, ci]
        L.orc_grad_reduce_into_chunk.argtypes = [vp, i64, vp, i64, f32, ci]
        L.orc_sum_squares.argtypes = [vp, i64]
        L.orc_sum_squares.restype = f64
        L.orc_clip_coef.argtypes = [f64, f64]
        L.orc_clip_coef.restype = f64
        L.orc_chunk_adam_step.argtypes = [vp, vp, vp, vp, vp, vp, i64, f32, f32, f32, f32, f32, i64, f64]
        L.orc_chunk_adam_step_lp.argtypes = [vp, vp, vp, vp, vp, vp, ci, i64, f32, f32, f32, f32, f32, i64, f64]
        L.orc_grad_reduce_into_chunk_lp.argtypes = [vp, i64, vp, ci, i64, f32, ci]
        L.orc_f16_to_f32_array.argtypes = [vp, vp, i64]
        L.orc_f32_to_f16_array.argtypes = [vp, vp, i64]
        for n in ("orc_bf16_to_f32_array", "orc_f32_to_bf16_array", "orc_chunk_pack", "orc_chunk_unpack",
                  "orc_grad_reduce_into_chunk", "orc_chunk_adam_step", "orc_chunk_adam_step_lp", "orc_grad_reduce_into_chunk_lp",
                  "orc_f16_to_f32_array", "orc_f32_to_f16_array"):
            getattr(L, n).restype = None
        _lib = L
    return _lib


def _ptr(a: np.ndarray, dtype) -> int:
    if a.dtype != np.dtype(dtype) or not a.flags.c_contiguous:
        raise TypeError(f"expected C-contiguous {np.dtype(dtype)} array, got {a.dtype}")
    return a.ctypes.data


# ---------------------------------------------------------------------------
# bf16
# ---------------------------------------------------------------------------

def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    out = np.empty(bits.shape, np.float32)
    _L().orc_bf16_to_f32_array(_ptr(bits, np.uint16), out.ctypes.data, bits.size)
    return out


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    out = np.empty(x.shape, np.uint16)
    _L().orc_f32_to_bf16_array(_ptr(x, np.float32), out.ctypes.data, x.size)
    return out


BF16, FP16 = 0, 1   # low-precision formats: the benchmark's and the paper's


def f16_to_f32(bits: np.ndarray) -> np.ndarray:
    out = np.empty(bits.shape, np.float32)
    _L().orc_f16_to_f32_array(_ptr(bits, np.uint16), out.ctypes.data, bits.size)
    return out


def f32_to_f16(x: np.ndarray) -> np.ndarray:
    out = np.empty(x.shape, np.uint16)
    _L().orc_f32_to_f16_array(_ptr(x, np.float32), out.ctypes.data, x.size)
    return out


# ---------------------------------------------------------------------------
# Chunk layout (paper App. A.2): walk the parameters in order of use, keep one
# current chunk, append a parameter when it fits, otherwise close the chunk and
# open a new one.  Readings where the paper is silent:
#   * a parameter longer than a chunk closes the current chunk, starts at
#     offset 0 of a fresh chunk and runs through ceil(n/C) consecutive chunks;
#     the unused tail of its last chunk stays the current chunk;
#   * FIRST_FIT looks for room in every open chunk, oldest first, instead of
#     only the current one;
#   * DENSE lets parameters straddle chunk boundaries, so only the last chunk
#     is padded;
#   * `align` rounds every parameter's start up to a multiple of `align`.
# A parameter occupies the linear range [chunk_id*C + offset, +numel).
# ---------------------------------------------------------------------------

def layout_plan(numels, chunk_elems: int, policy: int = NEXT_FIT, align: int = 1):
    """Returns (chunk_id[T], offset[T], valid_len[n_chunks])."""
    C = int(chunk_elems)
    if C <= 0 or align <= 0 or C % align != 0:
        raise ValueError("chunk_elems must be a positive multiple of align")
    if policy not in (NEXT_FIT, FIRST_FIT, DENSE):
        raise ValueError("unknown policy")
    used = []  # elements in use per chunk, in chunk order
    chunk_id, offset = [], []

    def up(x):
        return (x + align - 1) // align * align

    def spill(n):
        """Lay n elements from offset 0 of a fresh chunk through as many chunks as needed."""
        while True:
            take = min(n, C)
            used.append(take)
            n -= take
            if n == 0:
                return

    for n in numels:
        n = int(n)
        if n < 0:
            raise ValueError("negative numel")
        if policy == DENSE:
            if not used:
                used.append(0)
            c = len(used) - 1
            start = up(used[c])
            if start >= C and n > 0:          # current chunk is full
                used.append(0)
                c, start = c + 1, 0
            chunk_id.append(c)
            offset.append(start)
            take = min(n, C - start)
            used[c] = start + take
            if n - take > 0:
                spill(n - take)
            continue
        if n > C:                             # longer than a chunk: fresh chunks
            chunk_id.append(len(used))
            offset.append(0)
            spill(n)
            continue
        candidates = range(len(used)) if policy == FIRST_FIT else range(max(len(used) - 1, 0), len(used))
        for c in candidates:
            if up(used[c]) + n <= C:
                chunk_id.append(c)
                offset.append(up(used[c]))
                used[c] = up(used[c]) + n
                break
        else:                                 # does not fit: close, open a new chunk
            chunk_id.append(len(used))
            offset.append(0)
            used.append(n)
    return chunk_id, offset, used


def padding_waste(valid_len, chunk_elems: int) -> float:
    """Padding elements divided by total chunk capacity."""
    cap = len(valid_len) * chunk_elems
    return 0.0 if cap == 0 else (cap - sum(valid_len)) / cap


# ---------------------------------------------------------------------------
# pack / unpack (paper Fig. 3 left)
# ---------------------------------------------------------------------------

def _tables(tensors, offsets, dtype):
    T = len(tensors)
    ptrs = (ctypes.c_void_p * T)(*[_ptr(t, dtype) for t in tensors])
    numel = (ctypes.c_int64 * T)(*[t.size for t in tensors])
    offs = (ctypes.c_int64 * T)(*[int(o) for o in offsets])
    return ptrs, numel, offs, T


def chunk_pack(chunk: np.ndarray, tensors, offsets) -> None:
    """chunk[offset_i + k] = tensor_i[k]; everything else becomes zero bits."""
    for t, o in zip(tensors, offsets):
        if o < 0 or o + t.size > chunk.size:
            raise ValueError("tensor slice outside the chunk")
    ptrs, numel, offs, T = _tables(tensors, offsets, chunk.dtype)
    _L().orc_chunk_pack(_ptr(chunk, chunk.dtype), chunk.size, chunk.dtype.itemsize, ptrs, numel, offs, T)


def chunk_unpack(chunk: np.ndarray, tensors, offsets) -> None:
    for t, o in zip(tensors, offsets):
        if o < 0 or o + t.size > chunk.size:
            raise ValueError("tensor slice outside the chunk")
    ptrs, numel, offs, T = _tables(tensors, offsets, chunk.dtype)
    _L().orc_chunk_unpack(_ptr(chunk, chunk.dtype), chunk.size, chunk.dtype.itemsize, ptrs, numel, offs, T)


# ---------------------------------------------------------------------------
# gradient reduction, norm, clip
# ---------------------------------------------------------------------------

def grad_reduce_into_chunk(gchunk: np.ndarray, offset: int, g_bf16: np.ndarray, scale: float, accumulate: bool,
                           fmt: int = BF16) -> None:
    if offset < 0 or offset + g_bf16.size > gchunk.size:
        raise ValueError("slice outside the chunk")
    _L().orc_grad_reduce_into_chunk_lp(_ptr(gchunk, np.float32), offset, _ptr(g_bf16, np.uint16), fmt, g_bf16.size,
                                       scale, 1 if accumulate else 0)


def sum_squares(g: np.ndarray) -> float:
    return _L().orc_sum_squares(_ptr(g, np.float32), g.size)


def grad_norm(grad_chunks, valid_len) -> float:
    """sqrt of the sum of squares over the valid part of every chunk (double)."""
    return math.sqrt(math.fsum(sum_squares(np.ascontiguousarray(c[:int(n)])) for c, n in zip(grad_chunks, valid_len)))


def clip_coef(norm: float, max_norm: float) -> float:
    return _L().orc_clip_coef(norm, max_norm)


# ---------------------------------------------------------------------------
# AdamW on one chunk
# ---------------------------------------------------------------------------

def chunk_adam_step(master, exp_avg, exp_avg_sq, grad, param_bf16, *, lr, beta1, beta2, eps, weight_decay, step,
                    grad_scale: float = 1.0, fmt: int = BF16) -> None:
    """In-place AdamW on fp32 master/m/v; `grad` is fp32 or bf16 bits (uint16); param_bf16 (uint16) may be None."""
    n = master.size
    if exp_avg.size != n or exp_avg_sq.size != n or grad.size != n or (param_bf16 is not None and param_bf16.size != n):
        raise ValueError("length mismatch")
    if step < 1:
        raise ValueError("step is 1-based")
    g32 = _ptr(grad, np.float32) if grad.dtype == np.float32 else None
    g16 = _ptr(grad, np.uint16) if grad.dtype == np.uint16 else None
    if g32 is None and g16 is None:
        raise TypeError("grad must be float32 or uint16 (bf16 bits)")
    out = _ptr(param_bf16, np.uint16) if param_bf16 is not None else None
    _L().orc_chunk_adam_step_lp(_ptr(master, np.float32), _ptr(exp_avg, np.float32), _ptr(exp_avg_sq, np.float32),
                                g32, g16, out, fmt, n, lr, beta1, beta2, eps, weight_decay, step, float(grad_scale))


# ---------------------------------------------------------------------------
# Offloading benefit model (paper Sec. 5.1, Eq. 1 and Eq. 2), in exact rationals.
#   I(n) = 1/L_c * ( L_c C / B_g2c + L_c C / B_c2g )
#   J(n) = n / (L_c + L_os F_os) * [ ( L_os C / B_c2g + L_c I + L_c C / B_g2c ) + ( C / V_c - C / V_g ) ]
# and the placement rule of the same section: what has the larger benefit gets the spare GPU memory first.
# ---------------------------------------------------------------------------

def offload_benefit(n, C, b_g2c, b_c2g, v_g, v_c, L_c=2, L_os=4, F_os=3):
    from fractions import Fraction as Fr
    C, b_g2c, b_c2g, v_g, v_c = (Fr(x) for x in (C, b_g2c, b_c2g, v_g, v_c))
    I = Fr(1, L_c) * (L_c * C / b_g2c + L_c * C / b_c2g)
    J = Fr(n, L_c + L_os * F_os) * ((L_os * C / b_c2g + L_c * I + L_c * C / b_g2c) + (C / v_c - C / v_g))
    return I, J


def offload_plan(n, C, n_chunks, min_blocks, allowed_bytes, b_g2c, b_c2g, v_g, v_c, L_c=2, L_os=4, F_os=3):
    """(rCache blocks, chunks moved to the GPU): start from min_blocks blocks and every chunk in CPU memory."""
    from fractions import Fraction as Fr
    I, J = offload_benefit(n, C, b_g2c, b_c2g, v_g, v_c, L_c, L_os, F_os)
    block = Fr(L_c * C)
    chunk = Fr((L_c + L_os * F_os) * C, n)
    blocks = max(1, min(min_blocks, n_chunks) if n_chunks else min_blocks)
    left = Fr(allowed_bytes) - blocks * block
    if left < 0:
        return blocks, 0
    up = 0
    order = ("chunks", "blocks") if J > I else ("blocks", "chunks")
    for what in order:
        if what == "chunks":
            k = max(0, min(n_chunks, int(left // chunk)))
            up += k
            left -= k * chunk
        else:
            k = max(0, min(n_chunks - blocks, int(left // block)))
            blocks += k
            left -= k * block
    return blocks, up


# ---------------------------------------------------------------------------
# rCache with Belady's replacement (paper Sec. 3 "rCache") and the chunk-size search of App. A.2, written as
# the definitions read: on a miss with a full cache, look ahead in the sequence for every cached chunk and
# evict the one used farthest in the future (never again first; ties: lowest id).
# ---------------------------------------------------------------------------

def rcache_simulate(seq, n_blocks):
    """(misses, evictions)."""
    if n_blocks < 1:
        raise ValueError("at least one block")
    cache, misses, evictions = [], 0, 0
    for i, c in enumerate(seq):
        if c in cache:
            continue
        misses += 1
        if len(cache) == n_blocks:
            def next_use(x):
                for j in range(i + 1, len(seq)):
                    if seq[j] == x:
                        return j
                return float("inf")
            victim = max(sorted(cache), key=next_use)      # max() keeps the first (lowest id) among equals
            cache.remove(victim)
            evictions += 1
        cache.append(c)
    return misses, evictions


def step_access_sequence(numels, chunk_elems, chunk_id, offset):
    """Chunks touched by one training step: parameters in order of use, then in reverse (paper Sec. 5.1)."""
    C = chunk_elems
    seq = []

    def touch(c):
        if not seq or seq[-1] != c:
            seq.append(c)

    spans = [(chunk_id[i], chunk_id[i] + (offset[i] + n - 1) // C) for i, n in enumerate(numels) if n > 0]
    for a, b in spans:
        for c in range(a, b + 1):
            touch(c)
    for a, b in reversed(spans):
        for c in range(b, a - 1, -1):
            touch(c)
    return seq


def chunk_size_search(numels, candidates, cache_bytes, policy=NEXT_FIT, align=1, L_c=2):
    """(best index, replaced bytes per candidate, padding per candidate): fewest bytes replaced in the rCache in one
    step; ties go to less padding, then to the longer chunk."""
    replaced, padding = [], []
    for C in candidates:
        cid, off, valid = layout_plan(numels, C, policy, align)
        seq = step_access_sequence(numels, C, cid, off)
        blocks = max(1, int(cache_bytes // (L_c * C)))
        _, ev = rcache_simulate(seq, blocks)
        replaced.append(ev * L_c * C)
        padding.append(len(valid) * C - sum(numels))
    best = min(range(len(candidates)), key=lambda k: (replaced[k], padding[k], -candidates[k]))
    return best, replaced, padding


# ---------------------------------------------------------------------------
# Dynamic loss scaling for fp16 gradients (Micikevicius et al., "Mixed Precision Training", Sec. 3.2, which the
# paper cites for its mixed-precision set-up; the paper itself gives no rule).  The loss is multiplied by S, so
# every gradient arrives multiplied by S.  A step whose gradients contain Inf/NaN is skipped and S shrinks;
# after `growth_interval` clean steps in a row S grows.
# ---------------------------------------------------------------------------

def loss_scale_step(scale, good_steps, norm_scaled, max_norm, growth_factor=2.0, backoff_factor=0.5, growth_interval=2000):
    """One step of the state machine.  norm_scaled = L2 norm of the (scaled) gradients; non-finite means overflow.
    Returns (new_scale, new_good_steps, skip, grad_scale) where grad_scale = clip_coef / scale multiplies the
    scaled gradients inside the update (clip_coef from the unscaled norm) and is 0 when the step is skipped."""
    if not math.isfinite(norm_scaled):
        return scale * backoff_factor, 0, True, 0.0
    coef = clip_coef(norm_scaled / scale, max_norm)
    good = good_steps + 1
    new_scale = scale
    if good >= growth_interval:
        new_scale, good = scale * growth_factor, 0
    return new_scale, good, False, coef / scale
