"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This module holds NO arithmetic of the method (no Adam, no rounding of master
weights, no packing, no norm).  It only
  * lists GPT-2-shaped tensor sizes for the benchmark configurations, and
  * turns (key, element index) into a number with a counter-based integer hash,
so that the CPU side (numpy, below) and the GPU side (gen.hip, same recipe in
device code) can regenerate any slice of any input independently and get the
same bits.

Value recipe (all steps exact, hence identical on every machine):
  h   = mix64(key + GOLD * (idx + 1))                 64-bit integer hash
  s   = sum of the four 16-bit fields of h - 131070   integer in [-131070, 131070]
        (Irwin-Hall n=4: bell shaped, std = sqrt((2^32 - 1) / 3) = 37837.2254...)
  x   = float32(s) * float32(scale)                   one int->float, one fp32 multiply
  f32 output: x.   bf16 output: the upper 16 bits of x (truncation, a bit operation).
Optional exact zeros: a second hash lane h2 = mix64(h ^ LANE2); the value is
replaced by +0 when h2 % 100 < zero_pct.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

MASK64 = (1 << 64) - 1
GOLD = 0x9E3779B97F4A7C15
LANE2 = 0xD6E8FEB86659FD93
IRWIN_HALL_STD = 37837.22543550504  # sqrt((2**32 - 1) / 3)
BASE_SEED = 20221205

# stream tags
TAG_PARAM = 1
TAG_GRAD = 2
TAG_MOMENT = 3
TAG_MISC = 4


def mix64(z: int) -> int:
    """64-bit finaliser (splitmix64's output function) on a Python int."""
    z &= MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def stream_key(seed: int, tag: int, step: int = 0, micro_batch: int = 0, cfg: int = 0) -> int:
    """One 64-bit key per (seed, config, kind of data, step, micro-batch)."""
    k = mix64(seed + GOLD)
    k = mix64(k ^ ((cfg & 0xFFFF) << 48 | (tag & 0xFFFF) << 32))
    k = mix64(k ^ ((step & 0xFFFFFFFF) << 16 | (micro_batch & 0xFFFF)))
    return k


def scale_for_std(std: float) -> np.float32:
    return np.float32(std / IRWIN_HALL_STD)


def _mix64_np(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def _values_f32(key: int, idx0: int, n: int, scale, zero_pct: int) -> np.ndarray:
    idx = np.arange(idx0 + 1, idx0 + 1 + n, dtype=np.uint64)
    with np.errstate(over="ignore"):
        h = _mix64_np(np.uint64(key) + np.uint64(GOLD) * idx)
        s = ((h & np.uint64(0xFFFF)) + ((h >> np.uint64(16)) & np.uint64(0xFFFF))
             + ((h >> np.uint64(32)) & np.uint64(0xFFFF)) + (h >> np.uint64(48))).astype(np.int64) - 131070
        x = s.astype(np.float32) * np.float32(scale)
        if zero_pct > 0:
            h2 = _mix64_np(h ^ np.uint64(LANE2))
            x[(h2 % np.uint64(100)) < np.uint64(zero_pct)] = np.float32(0.0)
    return x


def fill_f32(key: int, idx0: int, n: int, std: float, zero_pct: int = 0, block: int = 1 << 22) -> np.ndarray:
    """fp32 values for global element indices [idx0, idx0+n)."""
    out = np.empty(n, dtype=np.float32)
    sc = scale_for_std(std)
    for a in range(0, n, block):
        b = min(n, a + block)
        out[a:b] = _values_f32(key, idx0 + a, b - a, sc, zero_pct)
    return out


def fill_bf16(key: int, idx0: int, n: int, std: float, zero_pct: int = 0, block: int = 1 << 22) -> np.ndarray:
    """bf16 bit patterns (uint16) for global element indices [idx0, idx0+n)."""
    out = np.empty(n, dtype=np.uint16)
    sc = scale_for_std(std)
    for a in range(0, n, block):
        b = min(n, a + block)
        x = _values_f32(key, idx0 + a, b - a, sc, zero_pct)
        out[a:b] = (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    return out


# ---------------------------------------------------------------------------
# GPT-2-shaped parameter sets (generic decoder block, declaration order; the
# output head is tied to wte and therefore not a tensor of its own).
# ---------------------------------------------------------------------------

def gpt2_tensor_list(n_layer: int, hidden: int, vocab: int, n_pos: int = 1024):
    h = hidden
    t = [("wte", vocab * h), ("wpe", n_pos * h)]
    for i in range(n_layer):
        p = f"h.{i}."
        t += [
            (p + "ln_1.w", h), (p + "ln_1.b", h),
            (p + "attn.qkv.w", h * 3 * h), (p + "attn.qkv.b", 3 * h),
            (p + "attn.proj.w", h * h), (p + "attn.proj.b", h),
            (p + "ln_2.w", h), (p + "ln_2.b", h),
            (p + "mlp.fc.w", h * 4 * h), (p + "mlp.fc.b", 4 * h),
            (p + "mlp.proj.w", 4 * h * h), (p + "mlp.proj.b", h),
        ]
    t += [("ln_f.w", h), ("ln_f.b", h)]
    return t


Mi = 1 << 20


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    cfg_id: int
    n_layer: int
    hidden: int
    vocab: int
    n_pos: int
    chunk_elems: int
    steps: int
    micro_batches: int = 1
    grad_zero_pct: int = 0
    max_norm: float = 0.0
    host_fraction: float = 0.0
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    param_std: float = 0.02
    grad_std: float = 1e-3

    def tensors(self):
        return gpt2_tensor_list(self.n_layer, self.hidden, self.vocab, self.n_pos)

    def numels(self):
        return [n for _, n in self.tensors()]

    def total_params(self):
        return sum(self.numels())


CONFIGS = {
    "tiny": WorkloadConfig("gpt2-tiny-21M/C=4Mi", 1, 2, 768, 8192, 1024, 4 * Mi, steps=10),
    "gpt2_1p5b": WorkloadConfig("gpt2-1.5B/C=64Mi", 2, 48, 1600, 50257, 1024, 64 * Mi, steps=20, grad_zero_pct=1),
    "gpt2_6b_clip": WorkloadConfig("gpt2-6B/C=128Mi/4mb+clip", 4, 48, 3200, 50257, 1024, 128 * Mi, steps=1,
                                   micro_batches=4, max_norm=1.0),
    "gpt2_20b_offload": WorkloadConfig("gpt2-20B/C=128Mi/60%host", 5, 64, 5120, 50257, 1024, 128 * Mi, steps=1,
                                       host_fraction=0.6),
}
SWEEP_CHUNK_ELEMS = [8 * Mi, 16 * Mi, 32 * Mi, 64 * Mi, 128 * Mi, 256 * Mi]


# ---------------------------------------------------------------------------
# Device-side generator (same recipe, gen.hip).  Harness code: fills caller-owned
# device buffers so that multi-billion-element inputs never cross the host link.
# ---------------------------------------------------------------------------
_LIB = None


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsynth_gen.so")


def _lib():
    global _LIB
    if _LIB is None:
        p = lib_path()
        if not os.path.exists(p):
            raise RuntimeError(f"{p} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(p)
        for name in ("synth_fill_bf16", "synth_fill_f32"):
            f = getattr(L, name)
            f.restype = ctypes.c_int
            f.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int64,
                          ctypes.c_float, ctypes.c_int, ctypes.c_void_p]
        _LIB = L
    return _LIB


def fill_bf16_device(ptr: int, n: int, key: int, idx0: int, std: float, zero_pct: int = 0, stream: int = 0):
    """Fill n bf16 elements at device address `ptr` with the values fill_bf16(key, idx0, n, std, zero_pct) gives."""
    rc = _lib().synth_fill_bf16(ptr, n, key, idx0, float(scale_for_std(std)), zero_pct, stream)
    if rc != 0:
        raise RuntimeError(f"synth_fill_bf16 failed with HIP error {rc}")


def fill_f32_device(ptr: int, n: int, key: int, idx0: int, std: float, zero_pct: int = 0, stream: int = 0):
    rc = _lib().synth_fill_f32(ptr, n, key, idx0, float(scale_for_std(std)), zero_pct, stream)
    if rc != 0:
        raise RuntimeError(f"synth_fill_f32 failed with HIP error {rc}")
