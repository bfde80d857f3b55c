"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, its integer layout planner agrees with the oracle's, and bad arguments come back as status
codes before anything is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2212_05339_amd as ex
from oracle import elixir_oracle as orc
from synth import gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "elixir_chunk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(elixir_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 15
    L = ex.lib()
    for n in names:
        assert hasattr(L, n), f"{n} declared in the header but not exported"
    assert sorted(ex.EXPORTS) == names, "binding and header disagree on the entry points"
    for n in names:
        assert callable(getattr(ex, n)), f"binding lacks {n}"


def test_hparams_struct_layout_matches_header():
    # 5 floats, then an int64 aligned to 8 bytes
    assert ctypes.sizeof(ex.elixir_adam_hparams) == 32
    assert ex.elixir_adam_hparams.step.offset == 24


@pytest.mark.parametrize("policy", [0, 1, 2])
def test_planner_matches_oracle_on_random_inputs(policy):
    rng = np.random.default_rng(100 + policy)
    for _ in range(200):
        align = int(rng.choice([1, 1, 2, 4, 8]))
        C = int(rng.integers(1, 40)) * align
        numels = [int(x) for x in rng.integers(0, 3 * C + 2, size=rng.integers(0, 50))]
        assert ex.elixir_layout_plan(numels, C, policy, align) == tuple(orc.layout_plan(numels, C, policy, align))


def test_planner_matches_oracle_on_benchmark_sets():
    for name, cfg in gen.CONFIGS.items():
        sizes = gen.SWEEP_CHUNK_ELEMS if name == "gpt2_1p5b" else [cfg.chunk_elems]
        for C in sizes:
            for policy in (0, 1, 2):
                for align in (1, 64):
                    assert ex.elixir_layout_plan(cfg.numels(), C, policy, align) == tuple(orc.layout_plan(cfg.numels(), C, policy, align))


def test_planner_errors():
    for args in (([1, 2], 0, 0, 1), ([1, 2], 8, 7, 1), ([1, -2], 8, 0, 1), ([1, 2], 8, 0, 3), ([1], 8, 0, 0)):
        with pytest.raises(ex.ElixirError) as e:
            ex.elixir_layout_plan(*args)
        assert e.value.code == ex.ELIXIR_EINVAL
    # capacity of valid_len too small -> ECAP, with the chunk count reported
    L = ex.lib()
    nm = (ctypes.c_int64 * 3)(5, 5, 5)
    cid, off, valid = (ctypes.c_int64 * 3)(), (ctypes.c_int64 * 3)(), (ctypes.c_int64 * 1)()
    n = ctypes.c_int64()
    assert L.elixir_layout_plan(nm, 3, 8, 0, 1, cid, off, ctypes.byref(n), valid, 1) == ex.ELIXIR_ECAP
    assert n.value == 3 and b"3 chunks" in L.elixir_last_error()


def test_argument_errors_return_before_any_launch():
    hp = ex.make_hparams(1e-4, 0.9, 0.999, 1e-8, 0.01, 1)
    a = 4096  # stand-in addresses; never dereferenced because validation fails first
    cases = [
        (lambda: ex.elixir_chunk_adam_step(a, a, a, None, a, a, -1, hp, None, 0), ex.ELIXIR_EINVAL),          # negative n
        (lambda: ex.elixir_chunk_adam_step(a, a, a, a, a, a, 8, hp, None, 0), ex.ELIXIR_EINVAL),               # both grads
        (lambda: ex.elixir_chunk_adam_step(a, a, a, None, None, a, 8, hp, None, 0), ex.ELIXIR_EINVAL),         # no grad
        (lambda: ex.elixir_chunk_adam_step(None, a, a, None, a, a, 8, hp, None, 0), ex.ELIXIR_EINVAL),         # NULL master
        (lambda: ex.elixir_chunk_adam_step(a + 2, a, a, None, a, a, 8, hp, None, 0), ex.ELIXIR_EALIGN),        # fp32 at 2 mod 4
        (lambda: ex.elixir_chunk_adam_step(a, a, a, None, a + 1, a, 8, hp, None, 0), ex.ELIXIR_EALIGN),        # bf16 at odd address
        (lambda: ex.elixir_chunk_adam_step(a, a, a, None, a, a, 8, ex.make_hparams(1e-4, 0.9, 0.999, 1e-8, 0.0, 0), None, 0), ex.ELIXIR_EINVAL),  # step 0
        (lambda: ex.elixir_chunk_adam_step(a, a, a, None, a, a, 8, ex.make_hparams(1e-4, 1.0, 0.999, 1e-8, 0.0, 1), None, 0), ex.ELIXIR_EINVAL),  # beta1 = 1
        (lambda: ex.elixir_grad_reduce_into_chunk(a, -1, a, 8, 1.0, False, 0), ex.ELIXIR_EINVAL),
        (lambda: ex.elixir_grad_reduce_into_chunk(a, 0, None, 8, 1.0, False, 0), ex.ELIXIR_EINVAL),
        (lambda: ex.elixir_grad_reduce_into_chunk(a, 0, a + 1, 8, 1.0, False, 0), ex.ELIXIR_EALIGN),
        (lambda: ex.elixir_chunk_pack(a, 16, 3, [a], [4], [0], 0), ex.ELIXIR_EINVAL),                           # elem_size 3
        (lambda: ex.elixir_chunk_pack(a, 16, 4, [a], [4], [13], 0), ex.ELIXIR_EINVAL),                          # leaves the chunk
        (lambda: ex.elixir_chunk_pack(a, 16, 4, [a, a + 64], [8, 8], [0, 4], 0), ex.ELIXIR_EINVAL),             # overlap
        (lambda: ex.elixir_chunk_pack(a, 16, 4, [None], [4], [0], 0), ex.ELIXIR_EINVAL),                        # NULL tensor
        (lambda: ex.elixir_chunk_unpack(a, 16, 4, [a + 2], [4], [0], 0), ex.ELIXIR_EALIGN),
        (lambda: ex.elixir_chunk_unpack(a, 16, 2, [a], [4], [-1], 0), ex.ELIXIR_EINVAL),
        (lambda: ex.elixir_chunk_grad_norm(ex.Ctx(None), [a], [4], 1.0, a, a, 0), ex.ELIXIR_EINVAL),            # NULL ctx
        (lambda: ex.elixir_offload_register_slots(ex.Ctx(None), [a], 64), ex.ELIXIR_EINVAL),
        (lambda: ex.elixir_chunk_prefetch(ex.Ctx(None), a, 64, 0), ex.ELIXIR_EINVAL),
        (lambda: ex.elixir_chunk_wait_ready(ex.Ctx(None), 0, 0), ex.ELIXIR_EINVAL),
        (lambda: ex.elixir_chunk_evict(ex.Ctx(None), 0, a, 64, 0, 0), ex.ELIXIR_EINVAL),
        (lambda: ex.elixir_host_alloc(0), ex.ELIXIR_EINVAL),
        (lambda: ex.elixir_chunk_grad_norm_lp(ex.Ctx(None), [a], 0, [4], 1.0, 1.0, a, a, 0), ex.ELIXIR_EINVAL),   # NULL ctx
        (lambda: ex.elixir_grad_reduce_sources_lp(a, 0, [a, a], 5, 8, 1.0, False, 0), ex.ELIXIR_EINVAL),          # unknown format
        (lambda: ex.elixir_grad_reduce_sources_lp(a, 0, [a, None], 0, 8, 1.0, False, 0), ex.ELIXIR_EINVAL),       # NULL source
        (lambda: ex.elixir_grad_reduce_sources_lp(a, 0, [a, a + 1], 0, 8, 1.0, False, 0), ex.ELIXIR_EALIGN),
        (lambda: ex.elixir_grad_reduce_sources_lp(a + 2, 0, [a], 0, 8, 1.0, False, 0), ex.ELIXIR_EALIGN),
        (lambda: ex.elixir_grad_reduce_sources_chunk_sumsq(ex.Ctx(None), 0, a, [a], 0, 8, 8, 1.0, False, 0), ex.ELIXIR_EINVAL),
        (lambda: ex.elixir_chunk_adam_step_tiled_lp(a + 4, None, a, a, 0, 8, hp, None, None, 0), ex.ELIXIR_EALIGN),   # tiled chunk at 4 mod 8
        (lambda: ex.elixir_chunk_adam_step_tiled_lp(a, None, a, a, 3, 8, hp, None, None, 0), ex.ELIXIR_EINVAL),       # unknown format
    ]
    for i, (call, code) in enumerate(cases):
        with pytest.raises(ex.ElixirError) as e:
            call()
        assert e.value.code == code, f"case {i}: {e.value}"
        assert ex.elixir_last_error() != ""
    # zero-length work is a successful no-op and launches nothing
    ex.elixir_chunk_adam_step(a, a, a, None, a, a, 0, hp, None, 0)
    ex.elixir_grad_reduce_into_chunk(a, 0, a, 0, 1.0, False, 0)
    ex.elixir_chunk_pack(None, 0, 4, [], [], [], 0)
    ex.elixir_host_free(0)
    ex.elixir_grad_reduce_sources_lp(a, 0, [], 0, 8, 1.0, False, 0)
    ex.elixir_grad_reduce_sources_lp(a, 0, [a, a], 0, 0, 1.0, False, 0)
    ex.elixir_chunk_adam_step_tiled_lp(a, None, a, a, 0, 0, hp, None, None, 0)


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2212_05339_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    for f in ("elixir_oracle.py", "elixir_oracle.c"):
        text = open(os.path.join(ROOT, "oracle", f)).read()
        assert "paper_2212_05339_amd" not in text and "libelixir_chunk" not in text


def test_bench_refuses_more_than_one_gpu_and_the_product_fails_loudly_without_its_library():
    import subprocess
    import sys

    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU only" in r.stderr and r.stdout == ""
    # a missing library is an error, never a fallback: load the binding with the path pointing nowhere
    code = ("import paper_2212_05339_amd.binding as b\n"
            "b.LIB_PATH = '/nonexistent/libelixir_chunk.so'\n"
            "try:\n    b.lib()\nexcept RuntimeError as e:\n    print('raised:', e)\n")
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120, cwd=ROOT)
    assert r.returncode == 0 and "raised:" in r.stdout and "no fallback" in r.stdout


def test_binding_refuses_strided_tensors():
    torch = pytest.importorskip("torch")
    t = torch.zeros(8, 8)
    hp = ex.make_hparams(1e-4, 0.9, 0.999, 1e-8, 0.01, 1)
    with pytest.raises(ValueError):
        ex.elixir_chunk_adam_step(t[:, 0], t[:, 1], t[:, 2], t[:, 3], None, None, 8, hp, None, 0)


# --------------------------------------------------------------------------- placement of the chunk buffers

def test_arena_plan_offsets():
    GAP, GRAIN = ex.ELIXIR_ARENA_GAP_BYTES, 8192
    slot = lambda b: -(-b // GRAIN) * GRAIN + GAP
    # per chunk: one optimizer chunk of 1,000,000 bytes, three gradient sets of 12,345 bytes (near), one parameter copy (far)
    arrays = [(1_000_000, 1, ex.ELIXIR_ARENA_NEAR), (12_345, 3, ex.ELIXIR_ARENA_NEAR), (500_000, 1, ex.ELIXIR_ARENA_FAR)]
    off, (near, far) = ex.elixir_arena_plan(4, arrays)
    group = slot(1_000_000) + 3 * slot(12_345)
    assert near == 4 * group and far == 4 * slot(500_000)
    for c in range(4):
        assert off[c] == [c * group, c * group + slot(1_000_000), c * group + slot(1_000_000) + slot(12_345),
                          c * group + slot(1_000_000) + 2 * slot(12_345), c * slot(500_000)]
    # invariants on a random description: aligned, inside the region, disjoint, every array followed by the gap
    rng = np.random.default_rng(8)
    for _ in range(50):
        arrays = [(int(rng.integers(0, 1 << 28)), int(rng.integers(0, 4)), int(rng.integers(0, 2))) for _ in range(rng.integers(0, 6))]
        n_chunks = int(rng.integers(0, 7))
        off, region = ex.elixir_arena_plan(n_chunks, arrays)
        sizes = [b for b, n, r in arrays for _ in range(n)]
        regs = [r for b, n, r in arrays for _ in range(n)]
        for r in (0, 1):
            spans = sorted((off[c][k], sizes[k]) for c in range(n_chunks) for k in range(len(sizes)) if regs[k] == r)
            for (a, sa), (b, _) in zip(spans, spans[1:]):
                assert a + sa + GAP <= b
            assert all(a % GRAIN == 0 for a, _ in spans)
            assert (spans[-1][0] + spans[-1][1] + GAP <= region[r] + GRAIN) if spans else region[r] == 0
        # arrays whose sizes are equal never start a multiple of 1 MiB apart within a chunk's group
        for c in range(n_chunks):
            near_k = [k for k in range(len(sizes)) if regs[k] == 0]
            for i, j in zip(near_k, near_k[1:]):
                if sizes[i] % (1 << 20) == 0:
                    assert (off[c][j] - off[c][i]) % (1 << 20) != 0
    with pytest.raises(ex.ElixirError) as e:
        ex.elixir_arena_plan(2, [(16, 1, 7)])
    assert e.value.code == ex.ELIXIR_EINVAL
    with pytest.raises(ex.ElixirError) as e:
        ex.elixir_arena_plan(-1, [(16, 1, 0)])
    assert e.value.code == ex.ELIXIR_EINVAL
    region = (ctypes.c_int64 * 2)()
    arr = (ex.elixir_arena_array * 1)(ex.elixir_arena_array(100, 2, 0))
    assert ex.lib().elixir_arena_plan(3, arr, 1, None, 0, region) == ex.ELIXIR_ECAP and region[0] == 6 * slot(100)   # sizes first, offsets later
