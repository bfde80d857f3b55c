"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times: whole 64Mi- and
128Mi-element chunks of the GPT-2-shaped 1.5B / 6B / 20B sets.  The oracle checks sampled whole chunks
element by element (the update and the reduction are elementwise, so a chunk is a complete unit) and the
global norm in full.  Gradients are generated on the device by the seeded generator; what the oracle gets
is that buffer copied back, after slices of it have been checked against the host generator."""
import ctypes
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import paper_2212_05339_amd as ex
from oracle import elixir_oracle as orc
from synth import gen
from tests._util import HP, check_adam_close, check_bf16_copy, n_threads, oracle_adam_parallel

torch = pytest.importorskip("torch")
pytestmark = [pytest.mark.gpu, pytest.mark.timeout(400)]
DEV = "cuda:0"


def hp_struct(step):
    return ex.make_hparams(HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"], step)


def u16(t):
    return t.cpu().numpy().view(np.uint16)


def device_grads(buf, valid, key, idx0, std, zero_pct, rng):
    """Fill buf[:valid] on the device (padding zero), copy back, and spot-check slices against the host generator."""
    buf.zero_()
    gen.fill_bf16_device(buf.data_ptr(), valid, key, idx0, std, zero_pct)
    torch.cuda.synchronize()
    h = u16(buf)
    for a in [0, max(0, valid - 4096)] + [int(x) for x in rng.integers(0, max(1, valid - 4096), size=3)]:
        n = min(4096, valid - a)
        assert np.array_equal(h[a:a + n], gen.fill_bf16(key, idx0 + a, n, std, zero_pct)), "device generator differs from host"
    assert not h[valid:].any()
    return h


def test_gpt2_1p5b_sampled_chunks_twenty_steps():
    cfg = gen.CONFIGS["gpt2_1p5b"]
    C = cfg.chunk_elems
    cid, off, valid = ex.elixir_layout_plan(cfg.numels(), C, ex.ELIXIR_LAYOUT_NEXT_FIT, 1)
    assert (cid, off, valid) == tuple(orc.layout_plan(cfg.numels(), C, orc.NEXT_FIT, 1))
    nch = len(valid)
    assert nch == 26 and sum(valid) == 1_557_611_200
    rng = np.random.default_rng(2)
    sampled = [0, 1, int(rng.integers(2, nch - 1)), nch - 1]   # wte's full chunk, wte's tail + small tensors, a middle one, the ragged last
    assert valid[0] == C and valid[nch - 1] < C
    pkey = gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=cfg.cfg_id)
    state = torch.empty(3, C, dtype=torch.float32, device=DEV)
    tiled = torch.empty(ex.elixir_state_tiled_len(C), dtype=torch.float32, device=DEV)   # the optimizer chunk as bench.py holds it
    g = torch.empty(C, dtype=torch.int16, device=DEV)
    out = torch.empty(C, dtype=torch.int16, device=DEV)
    for c in sampled:
        state.zero_()
        out.zero_()
        # as bench.py launches it: over the chunk's valid prefix (the padding is never touched); the ragged last chunk is
        # launched over its padding as well, which pins that an update leaves all-zero padding all-zero
        n_launch = C if c == nch - 1 else valid[c]
        gen.fill_f32_device(state[0].data_ptr(), valid[c], pkey, c * C, cfg.param_std)
        torch.cuda.synchronize()
        ref = state.cpu().numpy()
        assert valid[c] >= 4096 and np.array_equal(ref[0, :4096], gen.fill_f32(pkey, c * C, 4096, cfg.param_std))
        rp, rm, rv = ref[0].copy(), ref[1].copy(), ref[2].copy()
        rout = np.zeros(C, np.uint16)
        ex.elixir_state_tile(tiled, state[0], state[1], state[2], C)
        for step in range(1, cfg.steps + 1):
            gkey = gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, step, 0, cfg.cfg_id)
            hg = device_grads(g, valid[c], gkey, c * C, cfg.grad_std, cfg.grad_zero_pct, rng)
            ex.elixir_chunk_adam_step_tiled_lp(tiled, None, g, out, ex.ELIXIR_LOWP_BF16, n_launch, hp_struct(step))
            oracle_adam_parallel(rp, rm, rv, hg, rout, step=step)
        ex.elixir_state_untile(tiled, state[0], state[1], state[2], C)
        torch.cuda.synchronize()
        got = state.cpu().numpy()
        err = check_adam_close(got[0], got[1], got[2], rp, rm, rv, lr=HP["lr"], gmax=3.5e-3, steps=cfg.steps,
                               what=f"1.5B chunk {c}")
        same = check_bf16_copy(u16(out), got[0], rout, rp, lr=HP["lr"], steps=cfg.steps, what=f"1.5B chunk {c}")
        assert not got[:, valid[c]:].view(np.uint32).any(), "padding moved"
        print(f"chunk {c}: valid {valid[c]}, max rel err {err}, bf16 identical {same:.6f}")


def _oracle_norm_streamed(chunks, valid):
    """sqrt(sum of squares) with the oracle, one chunk at a time from device memory, chunks spread over threads."""
    def one(i):
        h = chunks[i][:valid[i]].cpu().numpy()
        k = n_threads()
        edges = np.linspace(0, h.size, k + 1).astype(np.int64)
        return [orc.sum_squares(h[edges[j]:edges[j + 1]]) for j in range(k)]
    import math
    parts = []
    with ThreadPoolExecutor(4) as pool:
        for r in pool.map(one, range(len(chunks))):
            parts += r
    return math.sqrt(math.fsum(parts))


def test_gpt2_1p5b_clip_on_bf16_gradient_chunks_full_size():
    """One micro-batch with clipping, the paper's arrangement: the gradients sit in low-precision chunks (Sec. 4.1), the
    norm is taken over those 26 chunks directly (full, against the oracle on the widened values), and the tiled update
    reads them with the device-resident factor and writes the new parameters over them."""
    cfg = gen.CONFIGS["gpt2_1p5b"]
    C = cfg.chunk_elems
    _, _, valid = ex.elixir_layout_plan(cfg.numels(), C, ex.ELIXIR_LAYOUT_NEXT_FIT, 1)
    nch = len(valid)
    gkey = gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, 0, cfg.cfg_id)
    g = torch.zeros(nch, C, dtype=torch.int16, device=DEV)
    for c in range(nch):
        gen.fill_bf16_device(g[c].data_ptr(), valid[c], gkey, c * C, cfg.grad_std, cfg.grad_zero_pct)
    torch.cuda.synchronize()
    ctx = ex.elixir_ctx_create(0, C, nch)
    try:
        d_nc = torch.zeros(2, dtype=torch.float32, device=DEV)
        ex.elixir_chunk_grad_norm_lp(ctx, [g[c] for c in range(nch)], ex.ELIXIR_LOWP_BF16, valid, 1.0, 1.0, d_nc[0:1], d_nc[1:2])
        torch.cuda.synchronize()
        first = d_nc.cpu().numpy().copy()
        ex.elixir_chunk_grad_norm_lp(ctx, [g[c] for c in range(nch)], ex.ELIXIR_LOWP_BF16, valid, 1.0, 1.0, d_nc[0:1], d_nc[1:2])
        torch.cuda.synchronize()
        assert np.array_equal(first.view(np.uint32), d_nc.cpu().numpy().view(np.uint32)), "norm not reproducible"

        def one(c):
            h = orc.bf16_to_f32(u16(g[c][:valid[c]]))
            k = n_threads()
            edges = np.linspace(0, h.size, k + 1).astype(np.int64)
            return [orc.sum_squares(h[edges[j]:edges[j + 1]]) for j in range(k)]
        import math
        parts = []
        with ThreadPoolExecutor(4) as pool:
            for r in pool.map(one, range(nch)):
                parts += r
        want = math.sqrt(math.fsum(parts))
        want_coef = orc.clip_coef(want, 1.0)
        print(f"1.5B norm over bf16 chunks: gpu {first[0]:.6f} oracle {want:.6f}; factor gpu {first[1]:.8f} oracle {want_coef:.8f}")
        assert abs(first[0] - want) <= 1e-6 * want and abs(first[1] - want_coef) <= 1.2e-7 * want_coef   # one fp32 rounding
        assert 36.0 < want < 42.0                      # sigma 1e-3 on 99% of 1.56e9 elements: the clip is active
        pkey = gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=cfg.cfg_id)
        state = torch.empty(3, C, dtype=torch.float32, device=DEV)
        tiled = torch.empty(ex.elixir_state_tiled_len(C), dtype=torch.float32, device=DEV)
        for c in (1, nch - 1):
            state.zero_()
            gen.fill_f32_device(state[0].data_ptr(), valid[c], pkey, c * C, cfg.param_std)
            torch.cuda.synchronize()
            ref = state.cpu().numpy()
            hg = u16(g[c]).copy()
            assert np.array_equal(hg[:4096], gen.fill_bf16(gkey, c * C, 4096, cfg.grad_std, cfg.grad_zero_pct))
            ex.elixir_state_tile(tiled, state[0], state[1], state[2], C)
            ex.elixir_chunk_adam_step_tiled_lp(tiled, None, g[c], g[c], ex.ELIXIR_LOWP_BF16, valid[c], hp_struct(1), d_nc[1:2])
            ex.elixir_state_untile(tiled, state[0], state[1], state[2], C)
            torch.cuda.synchronize()
            rp, rm, rv, rout = ref[0].copy(), ref[1].copy(), ref[2].copy(), np.zeros(C, np.uint16)
            oracle_adam_parallel(rp, rm, rv, hg, rout, step=1, grad_scale=want_coef)      # the oracle's own norm and factor
            got = state.cpu().numpy()
            check_adam_close(got[0], got[1], got[2], rp, rm, rv, lr=HP["lr"], gmax=3.5e-3 * want_coef, what=f"1.5B clip chunk {c}")
            now = u16(g[c])
            check_bf16_copy(now[:valid[c]], got[0][:valid[c]], rout[:valid[c]], rp[:valid[c]], lr=HP["lr"], what=f"1.5B clip chunk {c}")
            assert not now[valid[c]:].any() and not got[:, valid[c]:].view(np.uint32).any()     # padding untouched
    finally:
        ex.elixir_ctx_destroy(ctx)


def test_gpt2_1p5b_sweep_shape_first_fit_8mi_chunks_in_batched_launches():
    """The launch shape of the chunk-size sweep at its smallest size: the 1.5B set placed first-fit into 8Mi-element chunks
    (251 of them, ragged), every chunk a tiled optimizer chunk, ONE batched call per step over the valid prefixes (four
    launches of up to 64 chunks inside, chunks regrouped by length).  Two steps; sampled chunks against the oracle, and
    every chunk's padding still all-zero bits."""
    cfg = gen.CONFIGS["gpt2_1p5b"]
    C = 8 * gen.Mi
    _, _, valid = ex.elixir_layout_plan(cfg.numels(), C, ex.ELIXIR_LAYOUT_FIRST_FIT, 1)
    assert tuple(valid) == tuple(orc.layout_plan(cfg.numels(), C, orc.FIRST_FIT, 1)[2])
    nch = len(valid)
    assert nch == 251 and sum(valid) == 1_557_611_200
    rng = np.random.default_rng(8)
    shortest = int(np.argmin(valid))
    sampled = sorted({0, nch - 1, shortest, *[int(x) for x in rng.integers(1, nch - 1, size=3)]})
    L = ex.elixir_state_tiled_len(C)
    tiled = torch.zeros(nch, L, dtype=torch.float32, device=DEV)                 # 25 GB
    g = torch.zeros(nch, C, dtype=torch.int16, device=DEV)
    out = torch.zeros(nch, C, dtype=torch.int16, device=DEV)
    pkey = gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=cfg.cfg_id)
    flat = torch.zeros(3, C, dtype=torch.float32, device=DEV)
    ref = {}
    for c in range(nch):
        flat[0].zero_()
        gen.fill_f32_device(flat[0].data_ptr(), valid[c], pkey, c * C, cfg.param_std)
        ex.elixir_state_tile(tiled[c], flat[0], flat[1], flat[2], C)
        if c in sampled:
            torch.cuda.synchronize()
            p = flat[0].cpu().numpy().copy()
            k = min(1024, valid[c])
            assert np.array_equal(p[:k], gen.fill_f32(pkey, c * C, k, cfg.param_std)), "device generator differs from host"
            ref[c] = [p, np.zeros(C, np.float32), np.zeros(C, np.float32), np.zeros(C, np.uint16)]
    for step in (1, 2):
        gkey = gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, step, 0, cfg.cfg_id)
        g.zero_()
        for c in range(nch):
            gen.fill_bf16_device(g[c].data_ptr(), valid[c], gkey, c * C, cfg.grad_std, cfg.grad_zero_pct)
        ex.elixir_chunk_adam_step_tiled_multi_lp([tiled[c] for c in range(nch)], None, [g[c] for c in range(nch)], [out[c] for c in range(nch)],
                                                 ex.ELIXIR_LOWP_BF16, valid, hp_struct(step))
        torch.cuda.synchronize()
        for c in sampled:
            hg = u16(g[c])
            a = int(rng.integers(0, max(1, valid[c] - 4096)))
            k = min(4096, valid[c] - a)
            assert np.array_equal(hg[a:a + k], gen.fill_bf16(gkey, c * C + a, k, cfg.grad_std, cfg.grad_zero_pct)), "device generator differs from host"
            oracle_adam_parallel(ref[c][0], ref[c][1], ref[c][2], hg, ref[c][3], step=step)
    for c in sampled:
        ex.elixir_state_untile(tiled[c], flat[0], flat[1], flat[2], C)
        torch.cuda.synchronize()
        got = flat.cpu().numpy()
        check_adam_close(got[0], got[1], got[2], ref[c][0], ref[c][1], ref[c][2], lr=HP["lr"], gmax=3.5e-3, steps=2, what=f"8Mi chunk {c}")
        check_bf16_copy(u16(out[c])[:valid[c]], got[0][:valid[c]], ref[c][3][:valid[c]], ref[c][0][:valid[c]], lr=HP["lr"], steps=2, what=f"8Mi chunk {c}")
    # padding: behind every chunk's valid prefix the state tiles and the parameter copy are still all-zero bits
    T = ex.ELIXIR_STATE_TILE
    e = torch.arange(C, device=DEV)
    for c in range(nch):
        if valid[c] == C:
            continue
        pad = e[valid[c]:]
        idx = 3 * T * (pad // T) + pad % T
        assert not bool(tiled[c].view(torch.int32)[idx].any()) and not bool(tiled[c].view(torch.int32)[idx + T].any()) \
            and not bool(tiled[c].view(torch.int32)[idx + 2 * T].any()) and not bool(out[c][valid[c]:].any()), f"padding of chunk {c} moved"


def test_gpt2_6b_accumulate_norm_clip_step_full_size():
    """Four micro-batches reduced into fp32 chunks (mean), global norm over all 50 chunks of 128Mi elements,
    clip to max-norm 1, AdamW with the clip coefficient taken from device memory."""
    cfg = gen.CONFIGS["gpt2_6b_clip"]
    C = cfg.chunk_elems
    cid, off, valid = ex.elixir_layout_plan(cfg.numels(), C, ex.ELIXIR_LAYOUT_NEXT_FIT, 1)
    nch = len(valid)
    assert nch == 50 and sum(valid) == 6_064_342_400
    K, scale = cfg.micro_batches, 0.25
    rng = np.random.default_rng(4)
    sampled = sorted({0, 1, nch - 1, int(rng.integers(2, nch - 1))})
    gch = torch.empty(nch, C, dtype=torch.float32, device=DEV)            # 26.8 GB
    stage = torch.empty(C, dtype=torch.int16, device=DEV)
    ref_g = {c: np.zeros(C, np.float32) for c in sampled}
    ctx = ex.elixir_ctx_create(0, C, nch)
    try:
        for mb in range(K):
            key = gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, mb, cfg.cfg_id)
            for c in range(nch):
                if c in sampled:
                    hg = device_grads(stage, valid[c], key, c * C, cfg.grad_std, 0, rng)
                    orc.grad_reduce_into_chunk(ref_g[c], 0, hg, scale, mb > 0)
                else:
                    stage.zero_()
                    gen.fill_bf16_device(stage.data_ptr(), valid[c], key, c * C, cfg.grad_std, 0)
                if mb < K - 1:
                    ex.elixir_grad_reduce_into_chunk(gch[c], 0, stage, C, scale, mb > 0)
                else:   # as bench.py runs it: the last pass also leaves the chunk's sum of squares in the context
                    ex.elixir_grad_reduce_chunk_sumsq(ctx, c, gch[c], stage, ex.ELIXIR_LOWP_BF16, C, valid[c], scale, True)
        d_fused = torch.zeros(2, dtype=torch.float32, device=DEV)
        ex.elixir_chunk_grad_norm_finish(ctx, nch, cfg.max_norm, d_fused[0:1], d_fused[1:2])
        torch.cuda.synchronize()
        fused_nc = d_fused.cpu().numpy().copy()
        for c in sampled:
            assert np.array_equal(gch[c].cpu().numpy().view(np.uint32), ref_g[c].view(np.uint32)), f"reduced chunk {c} differs"
        d_nc = torch.zeros(2, dtype=torch.float32, device=DEV)
        ex.elixir_chunk_grad_norm(ctx, [gch[c] for c in range(nch)], valid, cfg.max_norm, d_nc[0:1], d_nc[1:2])
        torch.cuda.synchronize()
        first = d_nc.cpu().numpy().copy()
        ex.elixir_chunk_grad_norm(ctx, [gch[c] for c in range(nch)], valid, cfg.max_norm, d_nc[0:1], d_nc[1:2])
        torch.cuda.synchronize()
        assert np.array_equal(first.view(np.uint32), d_nc.cpu().numpy().view(np.uint32)), "norm not reproducible"
        want = _oracle_norm_streamed([gch[c] for c in range(nch)], valid)
        want_coef = orc.clip_coef(want, cfg.max_norm)
        print(f"6B norm: gpu {first[0]:.6f} oracle {want:.6f}; clip gpu {first[1]:.8f} oracle {want_coef:.8f}")
        assert abs(first[0] - want) <= 1e-5 * want
        assert abs(first[1] - want_coef) <= 1.2e-7 * want_coef       # the device's coefficient is the oracle's, rounded once to fp32
        print(f"6B norm fused into the last reduction pass: {fused_nc[0]:.6f}, clip {fused_nc[1]:.8f}")
        assert abs(fused_nc[0] - want) <= 1e-5 * want and abs(fused_nc[1] - want_coef) <= 1e-5 * want_coef
        assert abs(float(fused_nc[0]) - float(first[0])) <= 2e-7 * want
        # mean of 4 gradients of sigma 1e-3 -> sigma 5e-4 per element -> norm ~ 5e-4*sqrt(6.06e9) ~ 38.9: clipping is active
        assert 35.0 < want < 43.0 and want_coef < 0.03
        # the norm of a single chunk (one-chunk call) against the oracle, and the per-chunk sums adding up to the global one
        sq = 0.0
        one = torch.zeros(1, dtype=torch.float32, device=DEV)
        for c in range(nch):
            ex.elixir_chunk_grad_norm(ctx, [gch[c]], [valid[c]], 0.0, one, None)
            torch.cuda.synchronize()
            sq += float(one.item()) ** 2
        assert abs(np.sqrt(sq) - first[0]) <= 2e-6 * first[0]
        # AdamW on the sampled chunks: the device reads its own coefficient from device memory, the oracle uses its own
        coef = want_coef
        pkey = gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=cfg.cfg_id)
        state = torch.empty(3, C, dtype=torch.float32, device=DEV)
        out = torch.empty(C, dtype=torch.int16, device=DEV)
        for c in sampled:
            state.zero_()
            gen.fill_f32_device(state[0].data_ptr(), valid[c], pkey, c * C, cfg.param_std)
            torch.cuda.synchronize()
            ref = state.cpu().numpy()
            ex.elixir_chunk_adam_step(state[0], state[1], state[2], gch[c], None, out, C, hp_struct(1), d_nc[1:2])
            torch.cuda.synchronize()
            rp, rm, rv, rout = ref[0].copy(), ref[1].copy(), ref[2].copy(), np.zeros(C, np.uint16)
            oracle_adam_parallel(rp, rm, rv, ref_g[c], rout, step=1, grad_scale=coef)
            got = state.cpu().numpy()
            check_adam_close(got[0], got[1], got[2], rp, rm, rv, lr=HP["lr"], gmax=3e-3 * coef, what=f"6B chunk {c}")
            check_bf16_copy(u16(out), got[0], rout, rp, lr=HP["lr"], what=f"6B chunk {c}")
            assert np.array_equal(gch[c].cpu().numpy().view(np.uint32), ref_g[c].view(np.uint32)), "gradients were rewritten"
        # all four micro-batches in ONE pass (bench.py --sources-per-pass 4), on the sampled chunks: the chunk bits of the
        # one-at-a-time order, and, the pass having refilled the chunk's slots with the same sums, the same fused norm
        del state, out
        four = torch.empty(K, C, dtype=torch.int16, device=DEV)
        once = torch.empty(C, dtype=torch.float32, device=DEV)
        for c in sampled:
            four.zero_()
            for mb in range(K):
                gen.fill_bf16_device(four[mb].data_ptr(), valid[c], gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, mb, cfg.cfg_id), c * C, cfg.grad_std, 0)
            once.fill_(7.0)
            ex.elixir_grad_reduce_sources_chunk_sumsq(ctx, c, once, [four[mb] for mb in range(K)], ex.ELIXIR_LOWP_BF16, C, valid[c], scale, False)
            torch.cuda.synchronize()
            assert torch.equal(once.view(torch.int32), gch[c].view(torch.int32)), f"one pass over four micro-batches differs on chunk {c}"
        ex.elixir_chunk_grad_norm_finish(ctx, nch, cfg.max_norm, d_fused[0:1], d_fused[1:2])
        torch.cuda.synchronize()
        assert np.array_equal(d_fused.cpu().numpy().view(np.uint32), fused_nc.view(np.uint32))
    finally:
        ex.elixir_ctx_destroy(ctx)


def test_gpt2_20b_offload_mix_full_size_chunks():
    """128Mi-element chunks of the 20B set: 60% of the sampled chunks live in pinned host memory (1.6 GB blocks),
    the rest in HBM; one AdamW step through two staging slots.  Host-resident and resident chunks must end up
    bitwise identical to the all-resident run, and that run matches the oracle on a sampled chunk."""
    cfg = gen.CONFIGS["gpt2_20b_offload"]
    C = cfg.chunk_elems
    cid, off, valid = ex.elixir_layout_plan(cfg.numels(), C, ex.ELIXIR_LAYOUT_NEXT_FIT, 1)
    nch = len(valid)
    assert nch == 194 and sum(valid) == 20_399_488_000
    rng = np.random.default_rng(5)
    chunks = sorted({0, 1, nch - 1, *[int(x) for x in rng.integers(2, nch - 1, size=2)]})   # 5 sampled chunks
    host_ids = chunks[:3]                                                               # 60% of them
    pkey = gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=cfg.cfg_id)
    gkey = gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, 0, cfg.cfg_id)
    nbytes = 3 * C * 4

    def fresh_state(c, t):
        t.zero_()
        gen.fill_f32_device(t[0].data_ptr(), valid[c], pkey, c * C, cfg.param_std)

    grads = {}
    for c in chunks:
        grads[c] = torch.zeros(C, dtype=torch.int16, device=DEV)
        gen.fill_bf16_device(grads[c].data_ptr(), valid[c], gkey, c * C, cfg.grad_std, 0)
    hp = hp_struct(1)
    # all-resident reference run on the GPU
    res = {c: torch.empty(3, C, dtype=torch.float32, device=DEV) for c in chunks}
    res_out = {c: torch.zeros(C, dtype=torch.int16, device=DEV) for c in chunks}
    for c in chunks:
        fresh_state(c, res[c])
        ex.elixir_chunk_adam_step(res[c][0], res[c][1], res[c][2], None, grads[c], res_out[c], C, hp)
    torch.cuda.synchronize()
    # oracle on one sampled chunk of the resident run
    c0 = chunks[-2]
    tmp = torch.empty(3, C, dtype=torch.float32, device=DEV)
    fresh_state(c0, tmp)
    torch.cuda.synchronize()
    ref = tmp.cpu().numpy()
    rout = np.zeros(C, np.uint16)
    hg = u16(grads[c0])
    assert np.array_equal(hg[:4096], gen.fill_bf16(gkey, c0 * C, 4096, cfg.grad_std))
    oracle_adam_parallel(ref[0], ref[1], ref[2], hg, rout, step=1)
    got = res[c0].cpu().numpy()
    check_adam_close(got[0], got[1], got[2], ref[0], ref[1], ref[2], lr=HP["lr"], gmax=3.5e-3, what=f"20B chunk {c0}")
    check_bf16_copy(u16(res_out[c0]), got[0], rout, ref[0], lr=HP["lr"], what=f"20B chunk {c0}")
    del ref, got
    # offloaded run
    ctx = ex.elixir_ctx_create(0, C, 8)
    blocks = {c: ex.elixir_host_alloc(nbytes) for c in host_ids}
    try:
        for c in host_ids:                                   # initial state goes to the host blocks
            fresh_state(c, tmp)
            torch.cuda.synchronize()
            h = tmp.cpu().numpy()
            ctypes.memmove(blocks[c], h.ctypes.data, nbytes)
        resident = {}
        for c in chunks:
            if c not in host_ids:
                resident[c] = torch.empty(3, C, dtype=torch.float32, device=DEV)
                fresh_state(c, resident[c])
        slots = [torch.full((3, C), float("nan"), dtype=torch.float32, device=DEV) for _ in range(2)]
        ex.elixir_offload_register_slots(ctx, slots, nbytes)
        out = {c: torch.zeros(C, dtype=torch.int16, device=DEV) for c in chunks}
        compute = torch.cuda.Stream()
        h2d, d2h = ex.elixir_offload_copy_streams(ctx, compute)
        torch.cuda.synchronize()
        pending, inflight = list(host_ids), []
        for c in chunks:
            while pending and len(inflight) < 2:
                inflight.append((pending[0], ex.elixir_chunk_prefetch(ctx, blocks[pending.pop(0)], nbytes, h2d)))
            if c in host_ids:
                cc, s = inflight.pop(0)
                assert cc == c
                ex.elixir_chunk_wait_ready(ctx, s, compute)
                ex.elixir_chunk_adam_step(slots[s][0], slots[s][1], slots[s][2], None, grads[c], out[c], C, hp, None, compute)
                ex.elixir_chunk_evict(ctx, s, blocks[c], nbytes, compute, d2h)
            else:
                r = resident[c]
                ex.elixir_chunk_adam_step(r[0], r[1], r[2], None, grads[c], out[c], C, hp, None, compute)
        torch.cuda.synchronize()
        for c in chunks:
            want = res[c].cpu().numpy()
            if c in host_ids:
                got = np.empty((3, C), np.float32)
                ctypes.memmove(got.ctypes.data, blocks[c], nbytes)
            else:
                got = resident[c].cpu().numpy()
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"chunk {c} differs from the resident run"
            assert torch.equal(out[c], res_out[c])
    finally:
        torch.cuda.synchronize()
        ex.elixir_offload_register_slots(ctx, [], 0)
        for b in blocks.values():
            ex.elixir_host_free(b)
        ex.elixir_ctx_destroy(ctx)


def test_gpt2_1p5b_tensor_list_reduce_and_whole_set_pack_full_size():
    """The batched reduction and the whole-set pack / unpack on the real tensor list of the 1.5B set, as
    `bench.py --workload tensor_lists` and `rows.grad_reduce_per_tensor` launch them: 580 tensors = 581 pieces in 26
    chunks of 64Mi elements, every tensor's gradient a slice of a chunk-shaped bf16 array.  Two micro-batches (overwrite,
    then accumulate); the oracle reduces sampled pieces from the seed (large ones at their head, middle and tail) and
    packs two whole chunks; everything no tensor covers must keep its preset pattern (reduction) or read zero (pack)."""
    cfg = gen.CONFIGS["gpt2_1p5b"]
    C = cfg.chunk_elems
    numels = cfg.numels()
    cid, off, valid = ex.elixir_layout_plan(numels, C, ex.ELIXIR_LAYOUT_NEXT_FIT, 1)
    nch = len(valid)
    rng = np.random.default_rng(8)
    pieces = []                                                       # (chunk, offset, length): a tensor that spans chunks in pieces
    for i, n in enumerate(numels):
        c, o, left = cid[i], off[i], n
        while left > 0:
            take = min(left, C - o)
            pieces.append((c, o, take))
            left, c, o = left - take, c + 1, 0
    assert len(pieces) == 581
    chunks = [torch.full((C,), 1.5, dtype=torch.float32, device=DEV) for _ in range(nch)]
    g16 = [torch.empty(C, dtype=torch.int16, device=DEV) for _ in range(nch)]
    keys = [gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, mb, cfg.cfg_id) for mb in range(2)]
    d32 = ex.elixir_ptr_table([chunks[c][o:o + n] for c, o, n in pieces])
    s16 = ex.elixir_ptr_table([g16[c][o:o + n] for c, o, n in pieces])
    lens = ex.elixir_i64_table([n for _, _, n in pieces])
    for mb, key in enumerate(keys):
        for c in range(nch):
            gen.fill_bf16_device(g16[c].data_ptr(), valid[c], key, c * C, cfg.grad_std, cfg.grad_zero_pct)
        ex.elixir_grad_reduce_multi_lp(d32, s16, lens, ex.ELIXIR_LOWP_BF16, 0.25, mb > 0)
        torch.cuda.synchronize()

    def windows(n):                                                   # what the oracle looks at of a piece of n elements
        if n <= 300_000:
            return [(0, n)]
        mid = int(rng.integers(100_000, n - 200_000)) // 4 * 4 + 1   # an odd start inside the piece
        return [(0, 100_000), (mid, 100_003), (n - 100_000, 100_000)]

    order = sorted(range(len(pieces)), key=lambda k: pieces[k][2])
    sampled = set(order[:6] + order[-4:] + [0, 1, 2, len(pieces) - 1] + [int(x) for x in rng.integers(0, len(pieces), size=24)])
    sampled |= {k for k, (c, o, n) in enumerate(pieces) if o == 0 or o + n == C}        # pieces of tensors that span chunks
    checked = 0
    for k in sorted(sampled):
        c, o, n = pieces[k]
        got = chunks[c][o:o + n].cpu().numpy()
        for a, m in windows(n):
            want = np.full(m, 1.5, np.float32)
            for mb, key in enumerate(keys):
                orc.grad_reduce_into_chunk(want, 0, gen.fill_bf16(key, c * C + o + a, m, cfg.grad_std, cfg.grad_zero_pct), 0.25, mb > 0)
            assert np.array_equal(got[a:a + m].view(np.uint32), want.view(np.uint32)), f"piece {k} (chunk {c}, offset {o}, {n} elements) at {a}"
            checked += m
    for c in range(nch):                                              # nothing outside the tensors was written
        tail = chunks[c][valid[c]:]
        assert tail.numel() == 0 or bool((tail == 1.5).all()), f"padding of chunk {c}"
    print(f"reduction: {len(sampled)} pieces, {checked} elements checked against the oracle")

    # ---- whole-set pack / unpack of fp32 data
    pkey = gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=cfg.cfg_id)
    data = [torch.zeros(C, dtype=torch.float32, device=DEV) for _ in range(nch)]        # tensor data, chunk-shaped like the gradients
    for c in range(nch):
        gen.fill_f32_device(data[c].data_ptr(), valid[c], pkey, c * C, cfg.param_std)
    views = ex.elixir_ptr_table([data[c][o:o + n] for c, o, n in pieces])
    p_c, p_o = ex.elixir_i64_table([c for c, _, _ in pieces]), ex.elixir_i64_table([o for _, o, _ in pieces])
    ex.elixir_chunks_pack(chunks, C, 4, views, lens, p_c, p_o)         # over the reduced values and the 1.5 pattern
    torch.cuda.synchronize()
    for c in (0, nch - 1):                                            # the oracle packs two whole chunks
        mine = [(o, n) for cc, o, n in pieces if cc == c]
        tensors = [gen.fill_f32(pkey, c * C + o, n, cfg.param_std) for o, n in mine]
        want = np.full(C, 7.0, np.float32)
        orc.chunk_pack(want, tensors, [o for o, _ in mine])
        assert np.array_equal(chunks[c].cpu().numpy().view(np.uint32), want.view(np.uint32)), f"packed chunk {c}"
    for c in range(nch):
        assert torch.equal(chunks[c][:valid[c]], data[c][:valid[c]]) and not bool(chunks[c][valid[c]:].any()), f"packed chunk {c}"
    back = [torch.full((C,), 3.0, dtype=torch.float32, device=DEV) for _ in range(nch)]
    ex.elixir_chunks_unpack(chunks, C, 4, ex.elixir_ptr_table([back[c][o:o + n] for c, o, n in pieces]), lens, p_c, p_o)
    torch.cuda.synchronize()
    for c in range(nch):
        assert torch.equal(back[c][:valid[c]], data[c][:valid[c]]) and bool((back[c][valid[c]:] == 3.0).all()), f"unpacked chunk {c}"


def test_one_chunk_past_four_gib_per_array():
    """A single chunk of 1.25 Gi + 3 elements: every fp32 array is longer than 4 GiB, so any 32-bit byte or element
    arithmetic in a kernel or in the host code would show.  Reduce (plain and fused with the sum of squares), norm,
    AdamW with fp32 and with bf16 gradients, and pack are run over the whole chunk; results are compared with the
    oracle on windows at the start, across the 4 GiB byte boundary, and at the odd end, and the norm in full."""
    n = (1 << 30) + (1 << 28) + 3
    W = 1 << 19
    windows = [(0, W), ((1 << 30) - W // 2, W), ((1 << 30) + 12345, W), (n - W - 3, W + 3)]
    pkey, gkey = gen.stream_key(99, gen.TAG_PARAM), gen.stream_key(99, gen.TAG_GRAD, 1)
    state = torch.zeros(3, n, dtype=torch.float32, device=DEV)
    g16 = torch.empty(n, dtype=torch.int16, device=DEV)
    gch = torch.full((n,), 7.0, dtype=torch.float32, device=DEV)
    out = torch.zeros(n, dtype=torch.int16, device=DEV)
    gen.fill_f32_device(state[0].data_ptr(), n, pkey, 0, 0.02)
    gen.fill_bf16_device(g16.data_ptr(), n, gkey, 0, 1e-3, 1)
    ctx = ex.elixir_ctx_create(0, n, 2)
    try:
        d_a = torch.zeros(2, dtype=torch.float32, device=DEV)
        d_b = torch.zeros(2, dtype=torch.float32, device=DEV)
        ex.elixir_grad_reduce_into_chunk(gch, 0, g16, n, 0.5, False)
        ex.elixir_grad_reduce_into_chunk(gch, 0, g16, n, 0.25, True)
        ex.elixir_grad_reduce_chunk_sumsq(ctx, 0, gch, g16, ex.ELIXIR_LOWP_BF16, 0, 0, 0.25, True)   # chunk 0 of the step is empty
        ex.elixir_grad_reduce_chunk_sumsq(ctx, 1, gch, g16, ex.ELIXIR_LOWP_BF16, n, n, 0.25, True)
        ex.elixir_chunk_grad_norm_finish(ctx, 2, 1.0, d_a[0:1], d_a[1:2])
        ex.elixir_chunk_grad_norm(ctx, [gch], [n], 1.0, d_b[0:1], d_b[1:2])
        torch.cuda.synchronize()
        ref_g = {}
        for a, w in windows:
            hg = u16(g16[a:a + w])
            assert np.array_equal(hg, gen.fill_bf16(gkey, a, w, 1e-3, 1)), f"gradients at {a}"
            r = np.full(w, 7.0, np.float32)
            orc.grad_reduce_into_chunk(r, 0, hg, 0.5, False)
            orc.grad_reduce_into_chunk(r, 0, hg, 0.25, True)
            orc.grad_reduce_into_chunk(r, 0, hg, 0.25, True)
            assert np.array_equal(gch[a:a + w].cpu().numpy().view(np.uint32), r.view(np.uint32)), f"reduced window at {a}"
            ref_g[a] = r
        want = _oracle_norm_streamed([gch], [n])
        fused, plain = d_a.cpu().numpy(), d_b.cpu().numpy()
        print(f"norm of {n} elements: oracle {want:.6f}, fused {fused[0]:.6f}, plain {plain[0]:.6f}")
        assert abs(fused[0] - want) <= 1e-5 * want and abs(plain[0] - want) <= 1e-5 * want
        assert abs(float(fused[0]) - float(plain[0])) <= 2e-7 * want
        assert want == pytest.approx(1e-3 * np.sqrt(0.99 * n), rel=0.01)       # sum of the three passes is 1.0 x g, 1% zeros
        coef = orc.clip_coef(want, 1.0)                                         # the oracle's own coefficient for its own update
        assert abs(float(plain[1]) - coef) <= 1.2e-7 * coef and abs(float(fused[1]) - coef) <= 1.2e-7 * coef
        # AdamW with the fp32 gradient chunk and the clip coefficient from device memory, then a second step with bf16 gradients
        before = {a: state[:, a:a + w].cpu().numpy() for a, w in windows}
        ex.elixir_chunk_adam_step(state[0], state[1], state[2], gch, None, out, n, hp_struct(1), d_b[1:2])
        ex.elixir_chunk_adam_step(state[0], state[1], state[2], None, g16, out, n, hp_struct(2))
        torch.cuda.synchronize()
        for a, w in windows:
            rp, rm, rv = (before[a][k].copy() for k in range(3))
            assert np.array_equal(rp, gen.fill_f32(pkey, a, w, 0.02)) and not rm.any() and not rv.any()
            rout = np.zeros(w, np.uint16)
            oracle_adam_parallel(rp, rm, rv, ref_g[a], rout, step=1, grad_scale=coef)
            oracle_adam_parallel(rp, rm, rv, u16(g16[a:a + w]), rout, step=2)
            got = state[:, a:a + w].cpu().numpy()
            check_adam_close(got[0], got[1], got[2], rp, rm, rv, lr=HP["lr"], gmax=4e-3, steps=2, what=f"window at {a}")
            check_bf16_copy(u16(out[a:a + w]), got[0], rout, rp, lr=HP["lr"], steps=2, what=f"window at {a}")
        # pack: the master array as one tensor into a chunk that starts 5 elements in (an unaligned 5 GiB copy)
        del gch
        torch.cuda.empty_cache()
        chunk = torch.zeros(n + 16, dtype=torch.float32, device=DEV)
        ex.elixir_chunk_pack(chunk, n + 16, 4, [state[0]], [n], [5])
        torch.cuda.synchronize()
        for a, w in windows:
            assert torch.equal(chunk[5 + a:5 + a + w], state[0, a:a + w]), f"packed window at {a}"
        assert not chunk[:5].any() and not chunk[5 + n:].any()
    finally:
        ex.elixir_ctx_destroy(ctx)
