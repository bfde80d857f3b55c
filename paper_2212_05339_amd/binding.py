"""ctypes binding of libelixir_chunk.so: one Python function per C entry point, same names.

Argument marshalling only -- every step of the path runs in the library's HIP kernels.
Device buffers are torch tensors (torch is used for device memory and streams only) or raw
integer addresses.  There is no CPU fallback: if the library is missing or a call fails an
exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libelixir_chunk.so")

ELIXIR_OK, ELIXIR_EINVAL, ELIXIR_EALIGN, ELIXIR_ENOSLOT, ELIXIR_EHIP, ELIXIR_ESTATE, ELIXIR_ECAP = 0, -1, -2, -3, -4, -5, -6
ELIXIR_LAYOUT_NEXT_FIT, ELIXIR_LAYOUT_FIRST_FIT, ELIXIR_LAYOUT_DENSE = 0, 1, 2
ELIXIR_LOWP_BF16, ELIXIR_LOWP_FP16 = 0, 1

EXPORTS = (
    "elixir_last_error", "elixir_ctx_create", "elixir_ctx_destroy", "elixir_layout_plan", "elixir_chunk_pack",
    "elixir_chunk_unpack", "elixir_grad_reduce_into_chunk", "elixir_chunk_grad_norm", "elixir_chunk_adam_step",
    "elixir_chunk_adam_step_multi",
    "elixir_host_alloc", "elixir_host_free", "elixir_offload_register_slots", "elixir_offload_copy_streams",
    "elixir_offload_set_evict_path",
    "elixir_chunk_prefetch",
    "elixir_chunk_wait_ready", "elixir_chunk_evict", "elixir_host_adam_step", "elixir_host_adam_isa", "elixir_copy_h2d_async",
    "elixir_copy_d2h_async", "elixir_stream_synchronize", "elixir_offload_benefit", "elixir_offload_plan",
    "elixir_rcache_simulate", "elixir_chunk_size_search", "elixir_grad_reduce_into_chunk_lp", "elixir_chunk_adam_step_lp",
    "elixir_chunk_adam_step_multi_lp", "elixir_loss_scale_init", "elixir_loss_scale_update",
    "elixir_grad_reduce_chunk_sumsq", "elixir_chunk_grad_norm_finish", "elixir_grad_reduce_multi_lp", "elixir_chunk_grad_norm_lp", "elixir_grad_reduce_sources_lp", "elixir_grad_reduce_sources_chunk_sumsq",
    "elixir_state_tiled_len", "elixir_state_tile", "elixir_state_untile", "elixir_chunk_adam_step_tiled_lp",
    "elixir_chunk_adam_step_tiled_multi_lp", "elixir_host_adam_step_tiled", "elixir_chunk_grad_norm_noalloc", "elixir_arena_plan",
    "elixir_chunks_pack", "elixir_chunks_unpack", "elixir_host_adam_step_lp", "elixir_host_adam_step_tiled_lp", "elixir_adam_step_state_init", "elixir_adam_step_state_advance", "elixir_chunk_adam_step_tiled_dev", "elixir_chunk_adam_step_tiled_multi_dev",
)


class ElixirError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libelixir_chunk status {code}: {message}")
        self.code = code


class elixir_hw_profile(ctypes.Structure):
    _fields_ = [("b_g2c", ctypes.c_double), ("b_c2g", ctypes.c_double), ("v_g", ctypes.c_double), ("v_c", ctypes.c_double)]


class elixir_arena_array(ctypes.Structure):
    _fields_ = [("bytes", ctypes.c_int64), ("count", ctypes.c_int32), ("region", ctypes.c_int32)]


class elixir_adam_hparams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("step", ctypes.c_int64)]


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the library built by `__graft_entry__.build()`; raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2212_05339_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, ci, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        pi64 = ctypes.POINTER(ctypes.c_int64)
        L.elixir_last_error.restype = ctypes.c_char_p
        L.elixir_last_error.argtypes = []
        sigs = {
            "elixir_ctx_create": [ctypes.POINTER(vp), ci, i64, ci],
            "elixir_ctx_destroy": [vp],
            "elixir_layout_plan": [pi64, ci, i64, ci, i64, pi64, pi64, pi64, pi64, i64],
            "elixir_chunk_pack": [vp, i64, ci, ctypes.POINTER(vp), pi64, pi64, ci, vp],
            "elixir_chunk_unpack": [vp, i64, ci, ctypes.POINTER(vp), pi64, pi64, ci, vp],
            "elixir_grad_reduce_into_chunk": [vp, i64, vp, i64, f32, ci, vp],
            "elixir_chunk_grad_norm": [vp, ctypes.POINTER(vp), pi64, ci, f32, vp, vp, vp],
            "elixir_chunk_adam_step": [vp, vp, vp, vp, vp, vp, i64, ctypes.POINTER(elixir_adam_hparams), vp, vp],
            "elixir_chunk_adam_step_multi": [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                             ctypes.POINTER(vp), ctypes.POINTER(vp), pi64, ctypes.POINTER(elixir_adam_hparams), vp, vp],
            "elixir_host_alloc": [ctypes.POINTER(vp), sz],
            "elixir_host_free": [vp],
            "elixir_offload_register_slots": [vp, ctypes.POINTER(vp), ci, sz],
            "elixir_offload_copy_streams": [vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(ci)],
            "elixir_offload_set_evict_path": [vp, ci],
            "elixir_chunk_prefetch": [vp, vp, sz, ctypes.POINTER(ci), vp],
            "elixir_chunk_wait_ready": [vp, ci, vp],
            "elixir_chunk_evict": [vp, ci, vp, sz, vp, vp],
        }
        sigs["elixir_chunk_grad_norm_noalloc"] = [ctypes.POINTER(vp), pi64, ci, f32, vp, vp, vp]
        sigs["elixir_chunks_pack"] = [ctypes.POINTER(vp), ci, i64, ci, ctypes.POINTER(vp), pi64, pi64, pi64, ci, vp]
        sigs["elixir_chunks_unpack"] = [ctypes.POINTER(vp), ci, i64, ci, ctypes.POINTER(vp), pi64, pi64, pi64, ci, vp]
        sigs["elixir_arena_plan"] = [ci, ctypes.POINTER(elixir_arena_array), ci, pi64, i64, pi64]
        sigs["elixir_adam_step_state_init"] = [vp, ctypes.POINTER(elixir_adam_hparams), vp]
        sigs["elixir_adam_step_state_advance"] = [vp, vp, vp]
        sigs["elixir_chunk_adam_step_tiled_dev"] = [vp, vp, vp, vp, ci, i64, vp, vp, vp, vp]
        sigs["elixir_chunk_adam_step_tiled_multi_dev"] = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                                          ci, pi64, vp, vp, vp, vp]
        sigs["elixir_host_adam_step"] = [vp, vp, vp, vp, vp, vp, i64, ctypes.POINTER(elixir_adam_hparams), f32, ci]
        sigs["elixir_host_adam_step_lp"] = [vp, vp, vp, vp, vp, vp, ci, i64, ctypes.POINTER(elixir_adam_hparams), f32, ci]
        sigs["elixir_host_adam_step_tiled_lp"] = [vp, vp, vp, vp, ci, i64, ctypes.POINTER(elixir_adam_hparams), f32, ci]
        sigs["elixir_host_adam_step_tiled"] = [vp, vp, vp, vp, i64, ctypes.POINTER(elixir_adam_hparams), f32, ci]
        sigs["elixir_copy_h2d_async"] = [vp, vp, sz, vp]
        sigs["elixir_copy_d2h_async"] = [vp, vp, sz, vp]
        sigs["elixir_stream_synchronize"] = [vp]
        pd = ctypes.POINTER(ctypes.c_double)
        sigs["elixir_grad_reduce_into_chunk_lp"] = [vp, i64, vp, ci, i64, f32, ci, vp]
        sigs["elixir_chunk_adam_step_lp"] = [vp, vp, vp, vp, vp, vp, ci, i64, ctypes.POINTER(elixir_adam_hparams), vp, vp, vp]
        sigs["elixir_chunk_adam_step_multi_lp"] = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                                   ctypes.POINTER(vp), ctypes.POINTER(vp), ci, pi64,
                                                   ctypes.POINTER(elixir_adam_hparams), vp, vp, vp]
        sigs["elixir_grad_reduce_chunk_sumsq"] = [vp, ci, vp, vp, ci, i64, i64, f32, ci, vp]
        sigs["elixir_chunk_grad_norm_finish"] = [vp, ci, f32, vp, vp, vp]
        sigs["elixir_grad_reduce_sources_lp"] = [vp, i64, ctypes.POINTER(vp), ci, ci, i64, f32, ci, vp]
        sigs["elixir_grad_reduce_sources_chunk_sumsq"] = [vp, ci, vp, ctypes.POINTER(vp), ci, ci, i64, i64, f32, ci, vp]
        sigs["elixir_chunk_grad_norm_lp"] = [vp, ctypes.POINTER(vp), ci, pi64, ci, f32, f32, vp, vp, vp]
        sigs["elixir_grad_reduce_multi_lp"] = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), pi64, ci, f32, ci, vp]
        sigs["elixir_state_tile"] = [vp, vp, vp, vp, i64, vp]
        sigs["elixir_state_untile"] = [vp, vp, vp, vp, i64, vp]
        sigs["elixir_chunk_adam_step_tiled_lp"] = [vp, vp, vp, vp, ci, i64, ctypes.POINTER(elixir_adam_hparams), vp, vp, vp]
        sigs["elixir_chunk_adam_step_tiled_multi_lp"] = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                                         ci, pi64, ctypes.POINTER(elixir_adam_hparams), vp, vp, vp]
        sigs["elixir_loss_scale_init"] = [vp, f32, vp]
        sigs["elixir_loss_scale_update"] = [vp, vp, f32, f32, f32, ci, vp]
        sigs["elixir_rcache_simulate"] = [pi64, i64, i64, pi64, pi64]
        sigs["elixir_chunk_size_search"] = [pi64, ci, pi64, ci, ci, i64, ctypes.c_double, ci, ctypes.POINTER(ci), pi64, pi64]
        sigs["elixir_offload_benefit"] = [ci, i64, ci, ci, ci, ctypes.POINTER(elixir_hw_profile), pd, pd]
        sigs["elixir_offload_plan"] = [ci, i64, i64, i64, ci, ci, ci, ctypes.POINTER(elixir_hw_profile), ctypes.c_double, pi64, pi64]
        L.elixir_host_adam_isa.restype = ctypes.c_char_p
        L.elixir_host_adam_isa.argtypes = []
        for name, argtypes in sigs.items():
            f = getattr(L, name)
            f.restype = ci
            f.argtypes = argtypes
        L.elixir_state_tiled_len.restype = i64
        L.elixir_state_tiled_len.argtypes = [i64]
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != ELIXIR_OK:
        raise ElixirError(rc, lib().elixir_last_error().decode())


def elixir_last_error() -> str:
    return lib().elixir_last_error().decode()


def _addr(x) -> Optional[int]:
    """Device/host address of a torch tensor, or the integer itself, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if not x.is_contiguous():       # the library sees a base address and an element count: a strided view would be read as dense
        raise ValueError("elixir: a non-contiguous tensor was passed where a dense buffer is expected")
    return x.data_ptr()


def _stream(stream) -> Optional[int]:
    """hipStream_t of a torch.cuda.Stream, a raw handle, or torch's current stream when None."""
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _i64_array(xs: Sequence[int]):
    if isinstance(xs, ctypes.Array):     # a table built ahead with elixir_i64_table
        return xs
    return (ctypes.c_int64 * len(xs))(*[int(x) for x in xs])


def _ptr_array(xs):
    if isinstance(xs, ctypes.Array):     # a table built ahead with elixir_ptr_table
        return xs
    return (ctypes.c_void_p * len(xs))(*[_addr(x) for x in xs])


def elixir_ptr_table(xs):
    """The host table of addresses a list-taking call builds from `xs` on every call, built once.  A tensor list that does
    not change from step to step (the gradients of a model, the chunks of a set) can be handed to those calls in this
    form; the caller keeps the tensors alive."""
    return _ptr_array(list(xs))


def elixir_i64_table(xs):
    """The host table of lengths / offsets / chunk indices a list-taking call takes, built once."""
    return _i64_array(list(xs))


# --------------------------------------------------------------------------- context

class Ctx:
    """Owner of an elixir_ctx handle."""

    def __init__(self, handle: int):
        self.handle = handle


def elixir_ctx_create(device: int, max_chunk_elems: int, max_chunks: int) -> Ctx:
    h = ctypes.c_void_p()
    _check(lib().elixir_ctx_create(ctypes.byref(h), device, max_chunk_elems, max_chunks))
    return Ctx(h.value)


def elixir_ctx_destroy(ctx: Ctx) -> None:
    if ctx.handle:
        h, ctx.handle = ctx.handle, None
        _check(lib().elixir_ctx_destroy(h))


# --------------------------------------------------------------------------- layout

def elixir_layout_plan(numel: Sequence[int], chunk_elems: int, policy: int = ELIXIR_LAYOUT_NEXT_FIT, align_elems: int = 1):
    """Returns (chunk_id, offset, valid_len) as Python lists."""
    T = len(numel)
    nm = _i64_array(numel)
    cid, off = (ctypes.c_int64 * max(T, 1))(), (ctypes.c_int64 * max(T, 1))()
    n_chunks = ctypes.c_int64(0)
    _check(lib().elixir_layout_plan(nm, T, chunk_elems, policy, align_elems, cid, off, ctypes.byref(n_chunks), None, 0))
    valid = (ctypes.c_int64 * max(n_chunks.value, 1))()
    _check(lib().elixir_layout_plan(nm, T, chunk_elems, policy, align_elems, cid, off, ctypes.byref(n_chunks), valid,
                                    n_chunks.value))
    return list(cid[:T]), list(off[:T]), list(valid[:n_chunks.value])


# --------------------------------------------------------------------------- placement of the chunk buffers

ELIXIR_ARENA_NEAR, ELIXIR_ARENA_FAR = 0, 1
ELIXIR_ARENA_GAP_BYTES = (4 << 20) + 8192


def elixir_arena_plan(n_chunks: int, arrays):
    """arrays: [(bytes, count, region)].  Returns (offsets[c][k], (region 0 bytes, region 1 bytes)); k counts the arrays
    of a chunk in the order given, an array with count > 1 taking `count` consecutive k."""
    arr = (elixir_arena_array * max(len(arrays), 1))(*[elixir_arena_array(int(b), int(n), int(r)) for b, n, r in arrays])
    K = sum(int(n) for _, n, _ in arrays)
    off = (ctypes.c_int64 * max(n_chunks * K, 1))()
    region = (ctypes.c_int64 * 2)()
    _check(lib().elixir_arena_plan(n_chunks, arr, len(arrays), off, n_chunks * K, region))
    return [list(off[c * K:(c + 1) * K]) for c in range(n_chunks)], (region[0], region[1])


# --------------------------------------------------------------------------- pack / unpack

def elixir_chunk_pack(chunk, chunk_elems: int, elem_size: int, tensors, numel, offset, stream=None) -> None:
    T = len(tensors)
    _check(lib().elixir_chunk_pack(_addr(chunk), chunk_elems, elem_size, _ptr_array(tensors), _i64_array(numel),
                                   _i64_array(offset), T, _stream(stream)))


def elixir_chunk_unpack(chunk, chunk_elems: int, elem_size: int, tensors, numel, offset, stream=None) -> None:
    T = len(tensors)
    _check(lib().elixir_chunk_unpack(_addr(chunk), chunk_elems, elem_size, _ptr_array(tensors), _i64_array(numel),
                                     _i64_array(offset), T, _stream(stream)))


def elixir_chunks_pack(chunks, chunk_elems: int, elem_size: int, tensors, numel, chunk_id, offset, stream=None) -> None:
    """Every tensor of a set into its place in the chunk sequence (chunk_id, offset as elixir_layout_plan returns them)."""
    _check(lib().elixir_chunks_pack(_ptr_array(chunks), len(chunks), chunk_elems, elem_size, _ptr_array(tensors), _i64_array(numel),
                                    _i64_array(chunk_id), _i64_array(offset), len(tensors), _stream(stream)))


def elixir_chunks_unpack(chunks, chunk_elems: int, elem_size: int, tensors, numel, chunk_id, offset, stream=None) -> None:
    _check(lib().elixir_chunks_unpack(_ptr_array(chunks), len(chunks), chunk_elems, elem_size, _ptr_array(tensors), _i64_array(numel),
                                      _i64_array(chunk_id), _i64_array(offset), len(tensors), _stream(stream)))


# --------------------------------------------------------------------------- reduce / norm / step

def elixir_grad_reduce_into_chunk(grad_chunk, offset: int, grad_bf16, n: int, scale: float, accumulate: bool,
                                  stream=None) -> None:
    _check(lib().elixir_grad_reduce_into_chunk(_addr(grad_chunk), offset, _addr(grad_bf16), n, scale,
                                               1 if accumulate else 0, _stream(stream)))


def elixir_chunk_grad_norm(ctx: Ctx, grad_chunks, valid_len, max_norm: float, d_norm_out, d_clip_coef_out,
                           stream=None) -> None:
    n = len(grad_chunks)
    _check(lib().elixir_chunk_grad_norm(ctx.handle, _ptr_array(grad_chunks), _i64_array(valid_len), n, max_norm,
                                        _addr(d_norm_out), _addr(d_clip_coef_out), _stream(stream)))


def elixir_chunk_grad_norm_noalloc(grad_chunks, valid_len, max_norm: float, d_norm_out, d_clip_coef_out, stream=None) -> None:
    """elixir_chunk_grad_norm without a context: the partial sums go to the library's static device array."""
    _check(lib().elixir_chunk_grad_norm_noalloc(_ptr_array(grad_chunks), _i64_array(valid_len), len(grad_chunks), max_norm,
                                                _addr(d_norm_out), _addr(d_clip_coef_out), _stream(stream)))


def elixir_chunk_grad_norm_lp(ctx: Ctx, grad_chunks_lowp, lowp_format: int, valid_len, scale: float, max_norm: float, d_norm_out,
                              d_grad_scale_out, stream=None) -> None:
    _check(lib().elixir_chunk_grad_norm_lp(ctx.handle, _ptr_array(grad_chunks_lowp), lowp_format, _i64_array(valid_len),
                                           len(grad_chunks_lowp), scale, max_norm, _addr(d_norm_out), _addr(d_grad_scale_out),
                                           _stream(stream)))


def make_hparams(lr: float, beta1: float, beta2: float, eps: float, weight_decay: float, step: int) -> elixir_adam_hparams:
    return elixir_adam_hparams(lr, beta1, beta2, eps, weight_decay, step)


def elixir_chunk_adam_step(master, exp_avg, exp_avg_sq, grad_fp32, grad_bf16, param_bf16, n: int,
                           hp: elixir_adam_hparams, d_grad_scale=None, stream=None) -> None:
    _check(lib().elixir_chunk_adam_step(_addr(master), _addr(exp_avg), _addr(exp_avg_sq), _addr(grad_fp32),
                                        _addr(grad_bf16), _addr(param_bf16), n, ctypes.byref(hp), _addr(d_grad_scale),
                                        _stream(stream)))


def elixir_chunk_adam_step_multi(master, exp_avg, exp_avg_sq, grad_fp32, grad_bf16, param_bf16, n, hp: elixir_adam_hparams,
                                 d_grad_scale=None, stream=None) -> None:
    """Lists of per-chunk buffers (grad_fp32 / grad_bf16 / param_bf16 may be None as a whole)."""
    k = len(master)
    tab = lambda xs: None if xs is None else _ptr_array(xs)
    _check(lib().elixir_chunk_adam_step_multi(k, _ptr_array(master), _ptr_array(exp_avg), _ptr_array(exp_avg_sq), tab(grad_fp32),
                                              tab(grad_bf16), tab(param_bf16), _i64_array(n), ctypes.byref(hp),
                                              _addr(d_grad_scale), _stream(stream)))


# --------------------------------------------------------------------------- offload

def elixir_host_alloc(nbytes: int) -> int:
    p = ctypes.c_void_p()
    _check(lib().elixir_host_alloc(ctypes.byref(p), nbytes))
    return p.value


def elixir_host_free(ptr: int) -> None:
    _check(lib().elixir_host_free(ptr))


def elixir_offload_register_slots(ctx: Ctx, d_slots, slot_bytes: int) -> None:
    _check(lib().elixir_offload_register_slots(ctx.handle, _ptr_array(d_slots), len(d_slots), slot_bytes))


def elixir_offload_copy_streams(ctx: Ctx, compute_stream=None, with_flag: bool = False):
    """Returns (h2d, d2h): raw handles of the library's two copy streams, measured to have hardware queues to themselves
    beside compute_stream.  Pass them as h2d_stream / d2h_stream.  with_flag: (h2d, d2h, full_duplex) -- whether an
    upload and a download issued together overlapped when the call looked."""
    up, down, flag = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_int(0)
    _check(lib().elixir_offload_copy_streams(ctx.handle, _stream(compute_stream), ctypes.byref(up), ctypes.byref(down), ctypes.byref(flag)))
    return (up.value, down.value, bool(flag.value)) if with_flag else (up.value, down.value)


ELIXIR_EVICT_DMA, ELIXIR_EVICT_KERNEL = 0, 1


def elixir_offload_set_evict_path(ctx: Ctx, path: int) -> None:
    """ELIXIR_EVICT_DMA (default) or ELIXIR_EVICT_KERNEL: how elixir_chunk_evict brings a slot back to its host block."""
    _check(lib().elixir_offload_set_evict_path(ctx.handle, path))


def elixir_chunk_prefetch(ctx: Ctx, h_block: int, nbytes: int, h2d_stream) -> int:
    slot = ctypes.c_int(-1)
    _check(lib().elixir_chunk_prefetch(ctx.handle, h_block, nbytes, ctypes.byref(slot), _stream(h2d_stream)))
    return slot.value


def elixir_chunk_wait_ready(ctx: Ctx, slot: int, compute_stream=None) -> None:
    _check(lib().elixir_chunk_wait_ready(ctx.handle, slot, _stream(compute_stream)))


def elixir_chunk_evict(ctx: Ctx, slot: int, h_block: Optional[int], nbytes: int, compute_stream, d2h_stream) -> None:
    _check(lib().elixir_chunk_evict(ctx.handle, slot, h_block, nbytes, _stream(compute_stream), _stream(d2h_stream)))


# --------------------------------------------------------------------------- CPU update of host-resident chunks

def _host_addr(x):
    """Address of a numpy array, a raw integer address, or None."""
    if x is None or isinstance(x, int):
        return x
    return x.ctypes.data


def elixir_host_adam_step(master, exp_avg, exp_avg_sq, grad_fp32, grad_bf16, param_bf16, n: int, hp: elixir_adam_hparams,
                          grad_scale: float = 1.0, n_threads: int = 0) -> None:
    """Host buffers are numpy arrays or raw addresses (e.g. from elixir_host_alloc)."""
    _check(lib().elixir_host_adam_step(_host_addr(master), _host_addr(exp_avg), _host_addr(exp_avg_sq), _host_addr(grad_fp32),
                                       _host_addr(grad_bf16), _host_addr(param_bf16), n, ctypes.byref(hp), grad_scale, n_threads))


def elixir_host_adam_step_tiled(state, grad_fp32, grad_bf16, param_bf16, n: int, hp: elixir_adam_hparams, grad_scale: float = 1.0,
                                n_threads: int = 0) -> None:
    """The CPU update on a tiled optimizer chunk in host memory (numpy array or raw address)."""
    _check(lib().elixir_host_adam_step_tiled(_host_addr(state), _host_addr(grad_fp32), _host_addr(grad_bf16), _host_addr(param_bf16), n,
                                             ctypes.byref(hp), grad_scale, n_threads))


def elixir_host_adam_step_lp(master, exp_avg, exp_avg_sq, grad_fp32, grad_lowp, param_lowp, lowp_format: int, n: int,
                             hp: elixir_adam_hparams, grad_scale: float = 1.0, n_threads: int = 0) -> None:
    _check(lib().elixir_host_adam_step_lp(_host_addr(master), _host_addr(exp_avg), _host_addr(exp_avg_sq), _host_addr(grad_fp32),
                                          _host_addr(grad_lowp), _host_addr(param_lowp), lowp_format, n, ctypes.byref(hp), grad_scale,
                                          n_threads))


def elixir_host_adam_step_tiled_lp(state, grad_fp32, grad_lowp, param_lowp, lowp_format: int, n: int, hp: elixir_adam_hparams,
                                   grad_scale: float = 1.0, n_threads: int = 0) -> None:
    _check(lib().elixir_host_adam_step_tiled_lp(_host_addr(state), _host_addr(grad_fp32), _host_addr(grad_lowp), _host_addr(param_lowp),
                                                lowp_format, n, ctypes.byref(hp), grad_scale, n_threads))


def elixir_host_adam_isa() -> str:
    return lib().elixir_host_adam_isa().decode()


def elixir_copy_h2d_async(d_dst, h_src: int, nbytes: int, stream=None) -> None:
    _check(lib().elixir_copy_h2d_async(_addr(d_dst), h_src, nbytes, _stream(stream)))


def elixir_copy_d2h_async(h_dst: int, d_src, nbytes: int, stream=None) -> None:
    _check(lib().elixir_copy_d2h_async(h_dst, _addr(d_src), nbytes, _stream(stream)))


def elixir_stream_synchronize(stream=None) -> None:
    _check(lib().elixir_stream_synchronize(_stream(stream)))


# --------------------------------------------------------------------------- benefit model

def elixir_offload_benefit(n_procs: int, chunk_elems: int, b_g2c: float, b_c2g: float, v_g: float, v_c: float,
                           L_c: int = 2, L_os: int = 4, F_os: int = 3):
    """Returns (I, J).  Bandwidths in bytes/s, velocities in elements/s."""
    hw = elixir_hw_profile(b_g2c, b_c2g, v_g, v_c)
    i, j = ctypes.c_double(), ctypes.c_double()
    _check(lib().elixir_offload_benefit(n_procs, chunk_elems, L_c, L_os, F_os, ctypes.byref(hw), ctypes.byref(i), ctypes.byref(j)))
    return i.value, j.value


def elixir_offload_plan(n_procs: int, chunk_elems: int, n_chunks: int, min_blocks: int, allowed_bytes: float, b_g2c: float,
                        b_c2g: float, v_g: float, v_c: float, L_c: int = 2, L_os: int = 4, F_os: int = 3):
    """Returns (n_blocks, n_gpu_chunks)."""
    hw = elixir_hw_profile(b_g2c, b_c2g, v_g, v_c)
    nb, ng = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().elixir_offload_plan(n_procs, chunk_elems, n_chunks, min_blocks, L_c, L_os, F_os, ctypes.byref(hw), allowed_bytes,
                                     ctypes.byref(nb), ctypes.byref(ng)))
    return nb.value, ng.value


# --------------------------------------------------------------------------- rCache simulation, chunk-size search

def elixir_rcache_simulate(seq: Sequence[int], n_blocks: int):
    """Returns (misses, evictions) of Belady's replacement."""
    m, e = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().elixir_rcache_simulate(_i64_array(seq), len(seq), n_blocks, ctypes.byref(m), ctypes.byref(e)))
    return m.value, e.value


def elixir_chunk_size_search(numel: Sequence[int], candidates: Sequence[int], cache_bytes: float, policy: int = ELIXIR_LAYOUT_NEXT_FIT,
                             align_elems: int = 1, L_c: int = 2):
    """Returns (best index, replaced bytes per candidate, padding elements per candidate)."""
    k = len(candidates)
    best = ctypes.c_int(-1)
    rep, pad = (ctypes.c_int64 * k)(), (ctypes.c_int64 * k)()
    _check(lib().elixir_chunk_size_search(_i64_array(numel), len(numel), _i64_array(candidates), k, policy, align_elems, cache_bytes,
                                          L_c, ctypes.byref(best), rep, pad))
    return best.value, list(rep), list(pad)


# --------------------------------------------------------------------------- fp16 / loss scaling

def elixir_grad_reduce_into_chunk_lp(grad_chunk, offset: int, grad_lowp, lowp_format: int, n: int, scale: float, accumulate: bool,
                                     stream=None) -> None:
    _check(lib().elixir_grad_reduce_into_chunk_lp(_addr(grad_chunk), offset, _addr(grad_lowp), lowp_format, n, scale,
                                                  1 if accumulate else 0, _stream(stream)))


def elixir_chunk_adam_step_lp(master, exp_avg, exp_avg_sq, grad_fp32, grad_lowp, param_lowp, lowp_format: int, n: int,
                              hp: elixir_adam_hparams, d_grad_scale=None, d_skip=None, stream=None) -> None:
    _check(lib().elixir_chunk_adam_step_lp(_addr(master), _addr(exp_avg), _addr(exp_avg_sq), _addr(grad_fp32), _addr(grad_lowp),
                                           _addr(param_lowp), lowp_format, n, ctypes.byref(hp), _addr(d_grad_scale), _addr(d_skip),
                                           _stream(stream)))


def elixir_chunk_adam_step_multi_lp(master, exp_avg, exp_avg_sq, grad_fp32, grad_lowp, param_lowp, lowp_format: int, n,
                                    hp: elixir_adam_hparams, d_grad_scale=None, d_skip=None, stream=None) -> None:
    tab = lambda xs: None if xs is None else _ptr_array(xs)
    _check(lib().elixir_chunk_adam_step_multi_lp(len(master), _ptr_array(master), _ptr_array(exp_avg), _ptr_array(exp_avg_sq),
                                                 tab(grad_fp32), tab(grad_lowp), tab(param_lowp), lowp_format, _i64_array(n),
                                                 ctypes.byref(hp), _addr(d_grad_scale), _addr(d_skip), _stream(stream)))


def elixir_grad_reduce_multi_lp(dst, grad_lowp, n, lowp_format: int, scale: float, accumulate: bool, stream=None) -> None:
    """dst[i]: the tensor's slice of its fp32 gradient chunk; grad_lowp[i]: its n[i] 16-bit gradients."""
    _check(lib().elixir_grad_reduce_multi_lp(len(dst), _ptr_array(dst), _ptr_array(grad_lowp), _i64_array(n), lowp_format, scale,
                                             1 if accumulate else 0, _stream(stream)))


# --------------------------------------------------------------------------- tiled optimizer chunk

ELIXIR_STATE_TILE = 4096


def elixir_state_tiled_len(n: int) -> int:
    """Floats a tiled optimizer chunk of n elements occupies."""
    return lib().elixir_state_tiled_len(n)


def elixir_state_tile(state, master, exp_avg, exp_avg_sq, n: int, stream=None) -> None:
    _check(lib().elixir_state_tile(_addr(state), _addr(master), _addr(exp_avg), _addr(exp_avg_sq), n, _stream(stream)))


def elixir_state_untile(state, master, exp_avg, exp_avg_sq, n: int, stream=None) -> None:
    _check(lib().elixir_state_untile(_addr(state), _addr(master), _addr(exp_avg), _addr(exp_avg_sq), n, _stream(stream)))


def elixir_chunk_adam_step_tiled_lp(state, grad_fp32, grad_lowp, param_lowp, lowp_format: int, n: int, hp: elixir_adam_hparams,
                                    d_grad_scale=None, d_skip=None, stream=None) -> None:
    _check(lib().elixir_chunk_adam_step_tiled_lp(_addr(state), _addr(grad_fp32), _addr(grad_lowp), _addr(param_lowp), lowp_format, n,
                                                 ctypes.byref(hp), _addr(d_grad_scale), _addr(d_skip), _stream(stream)))


def elixir_chunk_adam_step_tiled_multi_lp(state, grad_fp32, grad_lowp, param_lowp, lowp_format: int, n, hp: elixir_adam_hparams,
                                          d_grad_scale=None, d_skip=None, stream=None) -> None:
    tab = lambda xs: None if xs is None else _ptr_array(xs)
    _check(lib().elixir_chunk_adam_step_tiled_multi_lp(len(state), _ptr_array(state), tab(grad_fp32), tab(grad_lowp), tab(param_lowp),
                                                       lowp_format, _i64_array(n), ctypes.byref(hp), _addr(d_grad_scale), _addr(d_skip),
                                                       _stream(stream)))


ADAM_STEP_STATE_BYTES = 64      # elixir_adam_step_state: 5 floats, pad, int64 steps done (byte 24), 8 floats of constants
ADAM_STEP_STATE_STEP_OFFSET = 24


def elixir_adam_step_state_init(d_step_state, hp: elixir_adam_hparams, stream=None) -> None:
    _check(lib().elixir_adam_step_state_init(_addr(d_step_state), ctypes.byref(hp), _stream(stream)))


def elixir_adam_step_state_advance(d_step_state, d_skip=None, stream=None) -> None:
    _check(lib().elixir_adam_step_state_advance(_addr(d_step_state), _addr(d_skip), _stream(stream)))


def elixir_chunk_adam_step_tiled_dev(state, grad_fp32, grad_lowp, param_lowp, lowp_format: int, n: int, d_step_state,
                                     d_grad_scale=None, d_skip=None, stream=None) -> None:
    _check(lib().elixir_chunk_adam_step_tiled_dev(_addr(state), _addr(grad_fp32), _addr(grad_lowp), _addr(param_lowp), lowp_format, n,
                                                  _addr(d_step_state), _addr(d_grad_scale), _addr(d_skip), _stream(stream)))


def elixir_chunk_adam_step_tiled_multi_dev(state, grad_fp32, grad_lowp, param_lowp, lowp_format: int, n, d_step_state,
                                           d_grad_scale=None, d_skip=None, stream=None) -> None:
    tab = lambda xs: None if xs is None else _ptr_array(xs)
    _check(lib().elixir_chunk_adam_step_tiled_multi_dev(len(state), _ptr_array(state), tab(grad_fp32), tab(grad_lowp), tab(param_lowp),
                                                        lowp_format, _i64_array(n), _addr(d_step_state), _addr(d_grad_scale),
                                                        _addr(d_skip), _stream(stream)))


LOSS_SCALE_STATE_BYTES = 16   # float scale, int32 good_steps, int32 skip, float grad_scale
LOSS_SCALE_SKIP_OFFSET, LOSS_SCALE_GRAD_SCALE_OFFSET = 8, 12


def elixir_loss_scale_init(d_state, init_scale: float, stream=None) -> None:
    _check(lib().elixir_loss_scale_init(_addr(d_state), init_scale, _stream(stream)))


def elixir_loss_scale_update(d_state, d_norm_scaled, max_norm: float, growth_factor: float = 2.0, backoff_factor: float = 0.5,
                             growth_interval: int = 2000, stream=None) -> None:
    _check(lib().elixir_loss_scale_update(_addr(d_state), _addr(d_norm_scaled), max_norm, growth_factor, backoff_factor,
                                          growth_interval, _stream(stream)))


# --------------------------------------------------------------------------- reduction fused with the norm

def elixir_grad_reduce_chunk_sumsq(ctx: Ctx, chunk_index: int, grad_chunk, grad_lowp, lowp_format: int, chunk_elems: int,
                                   valid_len: int, scale: float, accumulate: bool, stream=None) -> None:
    _check(lib().elixir_grad_reduce_chunk_sumsq(ctx.handle, chunk_index, _addr(grad_chunk), _addr(grad_lowp), lowp_format,
                                                chunk_elems, valid_len, scale, 1 if accumulate else 0, _stream(stream)))


def elixir_grad_reduce_sources_lp(grad_chunk, offset: int, grads_lowp, lowp_format: int, n: int, scale: float, accumulate: bool,
                                  stream=None) -> None:
    """Several low-precision gradient arrays (a list) summed into the fp32 chunk in one pass."""
    _check(lib().elixir_grad_reduce_sources_lp(_addr(grad_chunk), offset, _ptr_array(grads_lowp), len(grads_lowp), lowp_format, n, scale,
                                               1 if accumulate else 0, _stream(stream)))


def elixir_grad_reduce_sources_chunk_sumsq(ctx: Ctx, chunk_index: int, grad_chunk, grads_lowp, lowp_format: int, chunk_elems: int,
                                           valid_len: int, scale: float, accumulate: bool, stream=None) -> None:
    _check(lib().elixir_grad_reduce_sources_chunk_sumsq(ctx.handle, chunk_index, _addr(grad_chunk), _ptr_array(grads_lowp), len(grads_lowp),
                                                        lowp_format, chunk_elems, valid_len, scale, 1 if accumulate else 0,
                                                        _stream(stream)))


def elixir_chunk_grad_norm_finish(ctx: Ctx, n_chunks: int, max_norm: float, d_norm_out, d_clip_coef_out, stream=None) -> None:
    _check(lib().elixir_chunk_grad_norm_finish(ctx.handle, n_chunks, max_norm, _addr(d_norm_out), _addr(d_clip_coef_out),
                                               _stream(stream)))
