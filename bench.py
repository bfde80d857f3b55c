#!/usr/bin/env python3
"""Benchmark of the chunked mixed-precision AdamW step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload at N=1: the GPT-2-shaped 1.5B parameter set (48 layers, hidden 1600, vocab 50257, 1024
positions; 1,557,611,200 parameters) grouped next-fit into 64Mi-element chunks (26 chunks), all
resident in HBM; bf16 gradients ~N(0, 1e-3) with 1% exact zeros, a fresh set per step, generated
on the device BEFORE the timed region; one step = the fused AdamW update of every chunk (fp32
master + two moments read and written, bf16 gradient read, bf16 parameter copy written).
Prints ONE JSON line: params/s over the valid parameters, the roofline of the dominant kernel
(measured with HIP events on the launch stream), and the CPU oracle timed on a bounded sample.

After the timed region the same line collects, under `rows`:
  side_rows()             pack, gradient reduction (whole set and tensor list), norms, fp16 update, a small offload pipeline
  naive_allocation_row()  the benchmark step with every array an allocation of its own
  other_configs()         short runs of the other benchmark configurations: run_offload (20B mix, first: it needs a link
                          nobody has disturbed), run_hybrid (CPU update + benefit model), the tiny set through
                          run_headline, run_sweep (chunk sizes), run_clip (6B accumulate + norm + clip)
Each run_* is also `--workload <name>` on its own, as is run_tensor_lists; a row that fails records its error and
leaves the line alone.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E bandwidth
BYTES_PER_ELEM = 28         # 2 (bf16 grad) + 12 (read p, m, v) + 12 (write p, m, v) + 2 (bf16 param)


STAGGER_BYTES = (4 << 20) + 8192   # gap between the arrays of a chunk, see chunk_buffers()


def chunk_buffers(torch, dev, nch, C, n32=3):
    """Device buffers of nch chunks: n32 fp32 arrays (master, m, v and, with n32=4, the fp32 gradient chunk) and two
    bf16 arrays (gradient, parameter copy) per chunk.
    Where the buffers sit is the caller's choice; arrays that start at the same offset modulo a few MiB make the
    eight streams of the AdamW kernel cross DRAM pages in phase and cost ~2% of bandwidth (measured), so every
    array is followed by a 4 MiB + 8 KiB gap.  Returns (state[c] = (master, m, v[, grad32]), grad16[c], out16[c])."""
    gap32, gap16 = STAGGER_BYTES // 4, STAGGER_BYTES // 2
    flat32 = torch.zeros(nch * n32 * (C + gap32), dtype=torch.float32, device=dev)
    flat16 = torch.zeros(nch * 2 * (C + gap16) + gap16, dtype=torch.int16, device=dev)
    state, g16, o16 = [], [], []
    for c in range(nch):
        b = c * n32 * (C + gap32)
        state.append(tuple(flat32[b + j * (C + gap32): b + j * (C + gap32) + C] for j in range(n32)))
        g = c * (C + gap16)
        g16.append(flat16[g: g + C])
        o = nch * (C + gap16) + gap16 // 2 + c * (C + gap16)
        o16.append(flat16[o: o + C])
    return state, g16, o16, (flat32, flat16)


def chunk_groups(torch, dev, nch, parts, far=False):
    """The arrays of nch chunks carved out of one allocation at the offsets elixir_arena_plan gives: parts =
    [(name, dtype, numel, count)], chunk after chunk, array after array, every array followed by the stagger gap.
    Returns ({name: [per chunk: tensor, or list of `count` tensors]}, the allocation).  far=True: the arrays are the
    write-only ones (parameter copies), which the plan puts into a region of their own; the caller allocates that region
    away from the others (out_of_the_way).

    Why: device memory on this part behaves as a few classes of large address ranges.  Measured on whole 64Mi-element
    launches: the AdamW launch takes 266-272 us when the gradient array lies next to the optimizer chunk and 280-283 us
    when it lies tens of GiB away; the accumulate pass of the reduction 99-102 us against 106-109 us for its bf16
    source; a write-only array next to the optimizer chunk costs 2% instead."""
    import paper_2212_05339_amd as ex
    esz = {torch.float32: 4, torch.int16: 2}
    region = ex.ELIXIR_ARENA_FAR if far else ex.ELIXIR_ARENA_NEAR
    offsets, region_bytes = ex.elixir_arena_plan(nch, [(n * esz[dt], cnt, region) for _, dt, n, cnt in parts])
    arena = torch.zeros(region_bytes[region], dtype=torch.uint8, device=dev)
    out = {name: [] for name, *_ in parts}
    for c in range(nch):
        k = 0
        for name, dt, n, cnt in parts:
            views = [arena[offsets[c][k + j]: offsets[c][k + j] + n * esz[dt]].view(dt) for j in range(cnt)]
            k += cnt
            out[name].append(views if cnt > 1 else views[0])
    return out, arena


def out_of_the_way(torch, dev, nbytes_needed, make):
    """Allocates what make() allocates behind a temporary spacer of up to 100 GiB, so that it lands far from what was
    allocated before (see chunk_groups); the spacer is freed again."""
    free_b, _ = torch.cuda.mem_get_info()
    room = int(free_b) - nbytes_needed - (8 << 30)
    spacer = torch.empty(min(100 << 30, room), dtype=torch.uint8, device=dev) if room > (16 << 30) else None
    res = make()
    del spacer
    return res


_COMPUTE_STREAM = None


def compute_stream(torch):
    """The one stream every workload of this process launches its kernels on.  The HIP runtime feeds all streams of a process
    through four hardware queues, and streams that share a queue hold each other back; the offload pipeline needs its
    compute stream and its two copy streams on three different queues, which is easy to keep while the process holds few
    streams (elixir_offload_copy_streams measures it)."""
    global _COMPUTE_STREAM
    if _COMPUTE_STREAM is None:
        _COMPUTE_STREAM = torch.cuda.Stream()
    return _COMPUTE_STREAM


SINK = None     # a list while the default run collects the lines of the other configurations, else lines are printed



def settled_copy_streams(ex, ctx, stream, limit_s=30.0):
    """The library's copy streams, taken once uploads and downloads overlap.  After device memory has been freed (by this
    process or by the one that ran before it on the box) downloads by DMA run at half rate for about 30 ms per GiB freed,
    uploads are not affected; measured: 16 GiB < 0.5 s, 64 GiB 2 s.  A benchmark waits that out (a trainer would rather
    let the slots come back by the store kernel, elixir_offload_set_evict_path).  Returns (h2d, d2h, full_duplex, waited_s)."""
    t0 = time.perf_counter()
    while True:
        h2d, d2h, duplex = ex.elixir_offload_copy_streams(ctx, stream, with_flag=True)
        if duplex or time.perf_counter() - t0 > limit_s:
            return h2d, d2h, duplex, time.perf_counter() - t0
        time.sleep(0.5)

def emit(line):
    """Prints one JSON line (or hands it to the collecting run); the keys every line of this program carries get their
    common values where a workload did not set them (one GPU, larger is better, nothing of the paper to compare with,
    synthetic inputs)."""
    for key, val in (("n_gpus", 1), ("higher_is_better", True), ("scaling", "weak"), ("vs_baseline", None), ("data", "synthetic")):
        line.setdefault(key, val)
    if SINK is not None:
        SINK.append(line)
    else:
        print(json.dumps(line), flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt2_1p5b",
                    help="gpt2_1p5b (default, the benchmark line), tiny, sweep (chunk sizes 8Mi..256Mi), gpt2_6b_clip, gpt2_20b_offload, gpt2_20b_hybrid (CPU update + streaming), tensor_lists (pack / unpack / reduction over the 580 tensors of the 1.5B set), link_after_free (the host link in the seconds after device memory has been freed)")
    ap.add_argument("--host-threads", type=int, default=0, help="gpt2_20b_hybrid: threads of the CPU update (default: all cores)")
    ap.add_argument("--host-chunks", type=int, default=0, help="gpt2_20b_offload: allocate only about this many host-resident chunks")
    ap.add_argument("--multi", action="store_true",
                    help="update all chunks of a step with elixir_chunk_adam_step_multi (always done for chunks of <= 16Mi elements, "
                         "which are launch-bound one call at a time)")
    ap.add_argument("--sources-per-pass", type=int, default=1,
                    help="gpt2_6b_clip: how many micro-batches one reduction pass takes (1 = one pass per micro-batch, as gradients "
                         "arrive; 2 or 4 need that many bf16 gradient sets resident at once and save the re-reads and re-writes of "
                         "the fp32 chunk in between: same bits)")
    ap.add_argument("--unfused-norm", action="store_true", help="gpt2_6b_clip: separate norm pass instead of the one fused into the last reduction")
    ap.add_argument("--host-order", choices=["interleaved", "first"], default="interleaved",
                    help="gpt2_20b_offload: which 60%% of the chunks live in host memory (every 3 of 5, or the first 60%% in schedule order)")
    ap.add_argument("--whole-chunks", action="store_true", help="update the zero padding behind a chunk's last tensor as well "
                                                                "(default: a launch covers the valid prefix of its chunk)")
    ap.add_argument("--params-over-grads", action="store_true",
                    help="gpt2_1p5b / tiny: write the bf16 parameters over the bf16 gradients they were computed from (the paper's "
                         "parameter chunk, which holds the gradients after the backward pass) instead of into an array of their own; "
                         "a gradient set then holds parameters when the ring comes round to it again, which the timing does not see")
    ap.add_argument("--max-norm", type=float, default=0.0,
                    help="gpt2_1p5b / tiny: clip every step to this gradient norm; the norm is taken directly over the bf16 gradient "
                         "chunks (2 more bytes per element) and the update reads the factor from device memory")
    ap.add_argument("--state-layout", choices=["tiled", "flat"], default="tiled",
                    help="optimizer chunk as one buffer of interleaved [master|m|v] tiles (default) or as three arrays")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-rows", action="store_true", help="skip the per-row side measurements")
    ap.add_argument("--evict-path", choices=["auto", "dma", "kernel"], default="auto",
                    help="offload workloads: how a staging slot comes back to its host block: the DMA engine, the library's store kernel, or "
                         "(auto) the kernel only where uploads and downloads by DMA take turns")
    ap.add_argument("--configs", default="1,3,4,5,f", help="gpt2_1p5b: which of the other benchmark configurations get their short runs (rows.config_*); "
                                                            "f: the CPU update of host-resident chunks with the split the benefit model chooses (rows.f1_f2_hybrid_20b)")
    ap.add_argument("--no-configs", action="store_true", help="gpt2_1p5b: skip the short runs of the other benchmark configurations "
                                                               "(tiny, sweep, 6B accumulate + clip, 20B offload mix) that fill rows.config_*")
    return ap.parse_args()


def cpu_baseline(cfg, valid0, budget_elems):
    """The oracle's AdamW, as it stands, on the host cores: the first chunk of the workload, several
    consecutive steps, slices of the chunk spread over the threads (the update is elementwise)."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    from oracle import elixir_oracle as orc
    from synth import gen

    threads = max(1, len(os.sched_getaffinity(0)))
    n = min(valid0, cfg.chunk_elems)
    steps = max(1, int(budget_elems // n))
    p = gen.fill_f32(gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=cfg.cfg_id), 0, n, cfg.param_std)
    m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
    g = gen.fill_bf16(gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, 0, cfg.cfg_id), 0, n, cfg.grad_std, cfg.grad_zero_pct)
    out = np.zeros(n, np.uint16)
    edges = np.linspace(0, n, threads + 1).astype(np.int64)
    hp = dict(lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, weight_decay=cfg.weight_decay)

    def work(args):
        i, step = args
        a, b = int(edges[i]), int(edges[i + 1])
        orc.chunk_adam_step(p[a:b], m[a:b], v[a:b], g[a:b], out[a:b], step=step, **hp)

    orc.chunk_adam_step(p[:1024].copy(), m[:1024].copy(), v[:1024].copy(), g[:1024], None, step=1, **hp)  # load the library
    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        for step in range(1, steps + 1):
            list(ex.map(work, [(i, step) for i in range(threads)]))
    dt = time.perf_counter() - t0
    n1 = min(n, 4 * gen.Mi)                                    # one thread alone, on the head of the same chunk
    t1 = time.perf_counter()
    for step in range(steps + 1, steps + 5):
        orc.chunk_adam_step(p[:n1], m[:n1], v[:n1], g[:n1], out[:n1], step=step, **hp)
    dt1 = time.perf_counter() - t1
    return {"value": n * steps / dt, "unit": "params/s", "cores": threads, "kind": "oracle",
            "sample": f"chunk 0 of the workload ({n} elements), {steps} consecutive AdamW steps with bf16 write-back, "
                      f"{dt:.2f} s wall on {threads} threads",
            "single_thread_value": 4 * n1 / dt1, "single_thread_sample": f"4 steps on the first {n1} elements, {dt1:.2f} s"}


def side_rows(ex, gen, torch, cfg, C, nch, valid, state, grads, out, stream, step_ms):
    """Throughput of the other rows of the path, measured after (outside) the timed region on the same
    buffers: pack (a plain copy), gradient reduction, global norm, and the offload pipeline."""
    sh = stream.cuda_stream
    dev = out[0].device

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    rows = {}
    # an fp32 chunk with an fp32 tensor and a bf16 gradient array allocated next to it (see chunk_groups)
    side, _keep_side = chunk_groups(torch, dev, 1, [("dst", torch.float32, C, 1), ("src", torch.float32, C, 1), ("g16", torch.int16, C, 1)])
    src, dst, g16 = side["src"][0], side["dst"][0], side["g16"][0]
    g16.copy_(grads[0][0])
    t = timed(lambda: ex.elixir_chunk_pack(dst, C, 4, [src], [C], [0], sh), 10)
    rows["pack"] = {"what": f"one fp32 tensor of {C} elements into a chunk (plain copy)", "bytes": 8 * C, "GB/s": 8 * C / t / 1e9}
    # the gradient reduction over the whole set, chunk after chunk as a step does it (repeating ONE chunk instead keeps hitting the
    # same 384 MiB, which measures 2 points lower): per chunk an fp32 gradient chunk with the bf16 gradients next to it
    rg, _keep_rg = chunk_groups(torch, dev, nch, [("g32", torch.float32, C, 1), ("g16", torch.int16, C, 1)])
    for c in range(nch):
        rg["g16"][c].copy_(grads[0][c])

    def reduce_set(acc):
        for c in range(nch):
            ex.elixir_grad_reduce_into_chunk(rg["g32"][c], 0, rg["g16"][c], valid[c], 0.25, acc, sh)

    n_valid = sum(valid)
    t = timed(lambda: reduce_set(False), 5)
    rows["grad_reduce_first"] = {"what": f"bf16 -> fp32 chunk, overwrite: the valid prefixes of the {nch} chunks, one call each", "bytes": 6 * n_valid,
                                 "GB/s": 6 * n_valid / t / 1e9, "ms": t * 1e3}
    t = timed(lambda: reduce_set(True), 5)
    rows["grad_reduce_accumulate"] = {"what": f"bf16 + fp32 chunk -> fp32 chunk: the valid prefixes of the {nch} chunks, one call each", "bytes": 10 * n_valid,
                                      "GB/s": 10 * n_valid / t / 1e9, "ms": t * 1e3}
    # the reduction as gradients really arrive, tensor by tensor (a tensor that spans chunks in pieces): one call each against
    # one batched call for all of them
    cid, off, _ = ex.elixir_layout_plan(cfg.numels(), C, ex.ELIXIR_LAYOUT_NEXT_FIT, 1)
    pieces = []
    for i, n in enumerate(cfg.numels()):
        c, o, left = cid[i], off[i], n
        while left > 0:
            take = min(left, C - o)
            pieces.append((rg["g32"][c][o:o + take], rg["g16"][c][o:o + take], take))
            left, c, o = left - take, c + 1, 0
    p_dst, p_src, p_n = [p[0] for p in pieces], [p[1] for p in pieces], [p[2] for p in pieces]

    def per_tensor():
        for d, g, n in pieces:
            ex.elixir_grad_reduce_into_chunk(d, 0, g, n, 0.25, False, sh)

    t_each = timed(per_tensor, 3)
    T_dst, T_src, T_n = ex.elixir_ptr_table(p_dst), ex.elixir_ptr_table(p_src), ex.elixir_i64_table(p_n)   # built once, as a trainer would
    t_multi = timed(lambda: ex.elixir_grad_reduce_multi_lp(T_dst, T_src, T_n, ex.ELIXIR_LOWP_BF16, 0.25, False, sh), 5)
    rows["grad_reduce_per_tensor"] = {"what": f"bf16 -> fp32, overwrite, the {len(pieces)} tensor pieces of the set: one call per tensor against "
                                              "one elixir_grad_reduce_multi_lp call", "bytes": 6 * sum(p_n),
                                      "one_call_per_tensor_ms": t_each * 1e3, "one_call_per_tensor_GB/s": 6 * sum(p_n) / t_each / 1e9,
                                      "ms": t_multi * 1e3, "GB/s": 6 * sum(p_n) / t_multi / 1e9}
    t_macc = timed(lambda: ex.elixir_grad_reduce_multi_lp(T_dst, T_src, T_n, ex.ELIXIR_LOWP_BF16, 0.25, True, sh), 5)
    rows["grad_reduce_per_tensor"].update({"accumulate_ms": t_macc * 1e3, "accumulate_bytes": 10 * sum(p_n),
                                           "accumulate_GB/s": 10 * sum(p_n) / t_macc / 1e9})
    del rg, _keep_rg, pieces, p_dst, p_src
    # the fp16 variant of the update (same traffic: 16-bit gradient in, 16-bit copy out), with the loss-scale state on the device
    lss = torch.zeros(4, dtype=torch.float32, device=dev)
    ex.elixir_loss_scale_init(lss, 65536.0, sh)
    hp16 = ex.make_hparams(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, 1)
    f16g, _keep_f16 = chunk_groups(torch, dev, 1, [("state", torch.float32, ex.elixir_state_tiled_len(C), 1), ("g", torch.int16, C, 1)])
    ex.elixir_state_tile(f16g["state"][0], state[0][0], state[0][1], state[0][2], C, sh)
    f16g["g"][0].copy_(g16)
    t = timed(lambda: ex.elixir_chunk_adam_step_tiled_lp(f16g["state"][0], None, f16g["g"][0], out[0], ex.ELIXIR_LOWP_FP16, C, hp16, lss[3:4],
                                                        lss[2:3].view(torch.int32), sh), 10)
    rows["adam_fp16_loss_scaled"] = {"what": "tiled optimizer chunk, fp16 gradient in, fp16 copy out, grad_scale and skip flag read from the device state",
                                     "bytes": 28 * C, "GB/s": 28 * C / t / 1e9}
    del f16g, _keep_f16
    ctx = ex.elixir_ctx_create(0, C, nch)
    try:
        d_nc = torch.zeros(2, dtype=torch.float32, device=dev)
        chunks = [state[c][1] for c in range(nch)]          # the momentum buffers stand in for fp32 gradient chunks
        t = timed(lambda: ex.elixir_chunk_grad_norm(ctx, chunks, valid, 1.0, d_nc[0:1], d_nc[1:2], sh), 5)
        rows["grad_norm"] = {"what": f"{nch} fp32 chunks, {sum(valid)} valid elements, two-stage fp64 tree",
                             "bytes": 4 * sum(valid), "GB/s": 4 * sum(valid) / t / 1e9, "ms": t * 1e3}
        t = timed(lambda: ex.elixir_chunk_grad_norm_lp(ctx, grads[0], ex.ELIXIR_LOWP_BF16, valid, 1.0, 1.0, d_nc[0:1], d_nc[1:2], sh), 5)
        rows["grad_norm_lowp"] = {"what": f"the same norm taken directly over the {nch} bf16 gradient chunks (single micro-batch: no fp32 gradient chunk)",
                                  "bytes": 2 * sum(valid), "GB/s": 2 * sum(valid) / t / 1e9, "ms": t * 1e3}
        # ---- offload pipeline: n_host chunks live in pinned host memory, the nch resident chunks are updated meanwhile
        n_host, n_slots = 12, 3
        nbytes = 3 * C * 4
        blocks = [ex.elixir_host_alloc(nbytes) for _ in range(n_host)]
        slots = [torch.zeros(3, C, dtype=torch.float32, device=dev) for _ in range(n_slots)]
        ex.elixir_offload_register_slots(ctx, slots, nbytes)
        h2d, d2h, duplex, waited = settled_copy_streams(ex, ctx, stream)   # two streams with hardware queues of their own beside `stream`
        if not duplex:          # uploads and downloads by DMA take turns in this process: the slots come back by the store kernel
            ex.elixir_offload_set_evict_path(ctx, ex.ELIXIR_EVICT_KERNEL)
        hp = ex.make_hparams(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, 1)
        try:
            for b in blocks:                                   # touch the host blocks once (first-touch, zero state)
                s = ex.elixir_chunk_prefetch(ctx, b, nbytes, h2d)
                ex.elixir_chunk_evict(ctx, s, b, nbytes, h2d, d2h)
            torch.cuda.synchronize()

            def wall(fn):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                fn()
                torch.cuda.synchronize()
                return time.perf_counter() - t0

            def only_h2d():
                for b in blocks:
                    s = ex.elixir_chunk_prefetch(ctx, b, nbytes, h2d)
                    ex.elixir_chunk_evict(ctx, s, None, 0, h2d, h2d)

            def only_d2h():
                # a slot must be held before it can be evicted: hold it with a 4 KiB upload, then copy the block back
                for b in blocks:
                    s = ex.elixir_chunk_prefetch(ctx, b, 4096, h2d)
                    ex.elixir_chunk_evict(ctx, s, b, nbytes, h2d, d2h)

            def both_ways():
                # bare bidirectional traffic, no kernels: uploads on one stream, downloads of another block on the other
                half = n_host // 2
                for k in range(half):
                    s = ex.elixir_chunk_prefetch(ctx, blocks[k], nbytes, h2d)          # upload block k
                    ex.elixir_chunk_evict(ctx, s, None, 0, h2d, h2d)
                    s2 = ex.elixir_chunk_prefetch(ctx, blocks[half + k], 4096, d2h)    # download into block half+k
                    ex.elixir_chunk_evict(ctx, s2, blocks[half + k], nbytes, d2h, d2h)

            def resident_step():
                for c in range(nch):
                    ex.elixir_chunk_adam_step(state[c][0], state[c][1], state[c][2], None, grads[0][c], out[c], C, hp, None, sh)

            def offload_step(with_resident):
                pending, inflight = list(range(n_host)), []
                for k in range(n_host):
                    while pending and len(inflight) < n_slots:
                        inflight.append((pending[0], ex.elixir_chunk_prefetch(ctx, blocks[pending.pop(0)], nbytes, h2d)))
                    j, s = inflight.pop(0)
                    ex.elixir_chunk_wait_ready(ctx, s, sh)
                    ex.elixir_chunk_adam_step(slots[s][0], slots[s][1], slots[s][2], None, grads[0][j % nch], out[j % nch], C, hp, None, sh)
                    ex.elixir_chunk_evict(ctx, s, blocks[j], nbytes, sh, d2h)
                    if with_resident:                           # resident chunks are updated between offloaded ones
                        for c in range(k * nch // n_host, (k + 1) * nch // n_host):
                            ex.elixir_chunk_adam_step(state[c][0], state[c][1], state[c][2], None, grads[0][c], out[c], C, hp, None, sh)

            # the pipeline first, the bare link afterwards
            t_res = min(wall(resident_step) for _ in range(2))
            t_off = min(wall(lambda: offload_step(False)) for _ in range(2))
            t_mix = min(wall(lambda: offload_step(True)) for _ in range(2))
            t_h2d = min(wall(only_h2d) for _ in range(2))
            t_d2h = min(wall(only_d2h) for _ in range(2))
            t_both = min(wall(both_ways) for _ in range(2))
            # the same pipeline with the slots coming back the other way (store kernel / DMA engine)
            ex.elixir_offload_set_evict_path(ctx, ex.ELIXIR_EVICT_KERNEL if duplex else ex.ELIXIR_EVICT_DMA)
            t_off_other = min(wall(lambda: offload_step(False)) for _ in range(2))
            moved = n_host * nbytes
            t_dma = max(t_h2d, t_d2h)
            rows["offload"] = {
                "what": f"{n_host} host-resident chunks of {C} elements ([master|m|v], {nbytes} bytes each) through {n_slots} "
                        f"staging slots, prefetch / AdamW / evict on three streams, with the {nch} resident chunks updated meanwhile",
                "uploads_and_downloads_overlap_at_start": duplex, "waited_s_for_downloads_at_full_rate": round(waited, 2),
                "evict_path": "DMA" if duplex else "store kernel", "h2d_alone_GB/s": moved / t_h2d / 1e9, "d2h_alone_GB/s": moved / t_d2h / 1e9,
                "pipeline_ms": t_off * 1e3, "pipeline_GB/s_each_way": moved / t_off / 1e9,
                ("pipeline_GB/s_each_way_evict_by_store_kernel" if duplex else "pipeline_GB/s_each_way_evict_by_DMA"): moved / t_off_other / 1e9,
                "bidirectional_GB/s_each_way": (n_host // 2) * nbytes / t_both / 1e9,
                "pipeline_frac_of_one_way_link": t_dma / t_off,
                "pipeline_frac_of_bidirectional_link": (moved / t_off) / ((n_host // 2) * nbytes / t_both),
                "with_resident_ms": t_mix * 1e3, "resident_alone_ms": t_res * 1e3,
                "overlap": 1.0 - (t_mix - max(t_off, t_res)) / min(t_off, t_res),
            }
        finally:
            torch.cuda.synchronize()
            ex.elixir_offload_register_slots(ctx, [], 0)
            for b in blocks:
                ex.elixir_host_free(b)
    finally:
        ex.elixir_ctx_destroy(ctx)
    return rows


def _event_time(torch, stream, fn, reps, warm=1):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(reps):
        fn()
    e1.record(stream)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps, e0.elapsed_time(e1) * 1e-3 / reps


def run_sweep(args, torch, ex, gen):
    """Chunk-size sweep on the 1.5B set: padding waste of the three grouping policies and AdamW throughput per chunk size
    with the tensors placed first-fit in declaration order (what the benchmark definition asks for) and next-fit (the
    paper's grouping); ragged final chunks included.  One JSON line per size; `value` is the first-fit figure."""
    cfg = gen.CONFIGS["gpt2_1p5b"]
    dev = torch.device("cuda:0")
    stream = compute_stream(torch)
    sh = stream.cuda_stream
    measured = {}
    for C in gen.SWEEP_CHUNK_ELEMS:
        plans = {name: ex.elixir_layout_plan(cfg.numels(), C, pol, 1)[2] for name, pol in
                 (("next_fit", ex.ELIXIR_LAYOUT_NEXT_FIT), ("first_fit", ex.ELIXIR_LAYOUT_FIRST_FIT), ("dense", ex.ELIXIR_LAYOUT_DENSE))}
        use_multi = args.multi or C <= 16 * gen.Mi
        timed = {}
        for policy in ("first_fit", "next_fit"):
            valid = plans[policy]
            same = [k for k, v in timed.items() if plans[k] == valid]
            if same:                                   # the same chunks: nothing new to time
                timed[policy] = dict(timed[same[0]], same_layout_as=same[0])
                continue
            nch = len(valid)
            state, grads, out, keep = chunk_buffers(torch, dev, nch, C)
            pkey = gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=3)
            gkey = gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, 0, 3)
            for c in range(nch):
                gen.fill_f32_device(state[c][0].data_ptr(), valid[c], pkey, c * C, cfg.param_std)
                gen.fill_bf16_device(grads[c].data_ptr(), valid[c], gkey, c * C, cfg.grad_std, cfg.grad_zero_pct)
            step_no = [0]
            lens = [C] * nch if args.whole_chunks else list(valid)     # padding is never touched unless asked for
            tiled = None
            if args.state_layout == "tiled":       # [tiled optimizer chunk | gradient] side by side, parameter copies elsewhere (see chunk_groups)
                groups, keep_t = chunk_groups(torch, dev, nch, [("state", torch.float32, ex.elixir_state_tiled_len(C), 1), ("grad", torch.int16, C, 1)])
                tiled = groups["state"]
                for c in range(nch):
                    ex.elixir_state_tile(tiled[c], state[c][0], state[c][1], state[c][2], C)
                    groups["grad"][c].copy_(grads[c])
                torch.cuda.synchronize()
                del state, grads, out, keep
                torch.cuda.empty_cache()
                grads = groups["grad"]
                out_far = out_of_the_way(torch, dev, nch * (2 * C + STAGGER_BYTES), lambda: chunk_groups(torch, dev, nch, [("out", torch.int16, C, 1)], far=True))
                out, keep, state = out_far[0]["out"], out_far[1], None

            def step():
                step_no[0] += 1
                hp = ex.make_hparams(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, step_no[0])
                if use_multi and tiled:
                    ex.elixir_chunk_adam_step_tiled_multi_lp(tiled, None, grads, out, ex.ELIXIR_LOWP_BF16, lens, hp, None, None, sh)
                    return
                if use_multi:
                    ex.elixir_chunk_adam_step_multi([st[0] for st in state], [st[1] for st in state], [st[2] for st in state], None,
                                                    grads, out, lens, hp, None, sh)
                    return
                for c in range(nch):
                    if tiled:
                        ex.elixir_chunk_adam_step_tiled_lp(tiled[c], None, grads[c], out[c], ex.ELIXIR_LOWP_BF16, lens[c], hp, None, None, sh)
                    else:
                        ex.elixir_chunk_adam_step(state[c][0], state[c][1], state[c][2], None, grads[c], out[c], lens[c], hp, None, sh)

            wall, ev = _event_time(torch, stream, step, args.steps, args.warmup)
            timed[policy] = {"n_chunks": nch, "ms_per_step": wall * 1e3, "params_per_s": sum(valid) / wall,
                             "elements_per_s": sum(lens) / wall, "ms_per_chunk": ev / nch * 1e3,
                             "GB/s": BYTES_PER_ELEM * sum(lens) / ev / 1e9}
            del state, grads, out, keep
            if tiled:
                del tiled, keep_t
            torch.cuda.empty_cache()
        ff = timed["first_fit"]
        measured[C] = timed["next_fit"]["params_per_s"]
        emit({
            "metric": "chunked AdamW params/sec", "value": ff["params_per_s"], "unit": "params/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": ff["ms_per_step"], "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"gpt2-1.5B sweep/C={C >> 20}Mi", "chunk_elems": C, "n_chunks": ff["n_chunks"], "layout": "first-fit",
                       "launch": ("multi, " if use_multi else "per chunk, ") + ("tiled optimizer chunk" if args.state_layout == "tiled" else "three arrays")},
            "padding_waste": {k: 1.0 - sum(v) / (len(v) * C) for k, v in plans.items()},
            "n_chunks_by_policy": {k: len(v) for k, v in plans.items()},
            "elements_per_s": ff["elements_per_s"], "by_layout": timed,
            "roofline": {"bound": "hbm", "achieved": ff["GB/s"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": ff["GB/s"] / HBM_PEAK_GBPS, "traffic": None, "ms_per_chunk": ff["ms_per_chunk"]}})
    # from report to choice: the paper picks the chunk length whose simulated rCache replaces the fewest bytes per step
    # (App. A.2; the paper's grouping, forward + backward sweep, Belady's replacement); the update throughput measured above
    # is printed beside it
    cache_bytes = float(2 << 30)
    sizes = list(gen.SWEEP_CHUNK_ELEMS)
    best, replaced, padding = ex.elixir_chunk_size_search(cfg.numels(), sizes, cache_bytes, ex.ELIXIR_LAYOUT_NEXT_FIT, 1, 2)
    emit({"metric": "chunk-size search (bytes replaced in the rCache per step)", "config": {"workload": "gpt2-1.5B sweep", "layout": "next-fit",
                      "rcache_bytes": cache_bytes, "candidates_elems": sizes},
                      "replaced_bytes_per_step": replaced, "padding_elems": padding, "chosen_chunk_elems": sizes[best],
                      "measured_update_params_per_s_next_fit": {str(c): measured[c] for c in sizes}})


def run_clip(args, torch, ex, gen):
    """Gradient accumulation + clipping on the 6B set: 4 bf16 micro-batches reduced into fp32 chunks, global
    norm, clip coefficient on the device, AdamW with fp32 gradients (30 bytes per element)."""
    cfg = gen.CONFIGS["gpt2_6b_clip"]
    dev = torch.device("cuda:0")
    C = cfg.chunk_elems
    valid = ex.elixir_layout_plan(cfg.numels(), C, ex.ELIXIR_LAYOUT_NEXT_FIT, 1)[2]
    nch, K = len(valid), cfg.micro_batches
    stream = compute_stream(torch)
    sh = stream.cuda_stream
    tiled = None
    pkey = gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=cfg.cfg_id)
    if args.state_layout == "tiled":
        # per chunk [tiled optimizer chunk | fp32 gradient chunk | the K micro-batch gradients] side by side (see chunk_groups);
        # the parameter copies elsewhere
        groups, _keep_g = chunk_groups(torch, dev, nch, [("state", torch.float32, ex.elixir_state_tiled_len(C), 1), ("gch", torch.float32, C, 1),
                                                       ("mb", torch.int16, C, K)])
        tiled, gch = groups["state"], groups["gch"]
        mbs = [[groups["mb"][c][mb] for c in range(nch)] for mb in range(K)]
        scratch = torch.zeros(3, C, dtype=torch.float32, device=dev)
        for c in range(nch):
            scratch[0].zero_()
            gen.fill_f32_device(scratch[0].data_ptr(), valid[c], pkey, c * C, cfg.param_std)
            ex.elixir_state_tile(tiled[c], scratch[0], scratch[1], scratch[2], C)
        torch.cuda.synchronize()
        del scratch
        out_far = out_of_the_way(torch, dev, nch * (2 * C + STAGGER_BYTES), lambda: chunk_groups(torch, dev, nch, [("out", torch.int16, C, 1)], far=True))
        out, _keep_o = out_far[0]["out"], out_far[1]
    else:
        state, _unused16, out, _keep = chunk_buffers(torch, dev, nch, C, n32=4)     # [master | m | v | fp32 gradient chunk]
        gch = [st[3] for st in state]
        mbs_flat = torch.zeros(K, nch, C, dtype=torch.int16, device=dev)
        mbs = [[mbs_flat[mb, c] for c in range(nch)] for mb in range(K)]
        for c in range(nch):
            gen.fill_f32_device(state[c][0].data_ptr(), valid[c], pkey, c * C, cfg.param_std)
    for c in range(nch):
        for mb in range(K):
            gen.fill_bf16_device(mbs[mb][c].data_ptr(), valid[c], gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, mb, cfg.cfg_id),
                                 c * C, cfg.grad_std)
    ctx = ex.elixir_ctx_create(0, C, nch)
    d_nc = torch.zeros(2, dtype=torch.float32, device=dev)
    chunks = [gch[c] for c in range(nch)]
    step_no = [0]
    parts = {}

    fused = not args.unfused_norm
    lens = [C] * nch if args.whole_chunks else list(valid)     # padding (all-zero gradients and state) is never touched unless asked for

    spp = max(1, min(args.sources_per_pass, K))
    passes = [list(range(a, min(a + spp, K))) for a in range(0, K, spp)]          # micro-batches taken by each pass

    def reduce_all():
        for which in passes:
            first, last = which[0] == 0, which[-1] == K - 1
            for c in range(nch):
                srcs = [mbs[mb][c] for mb in which]
                if fused and last:              # the last pass also leaves the chunk's sum of squares in the context
                    ex.elixir_grad_reduce_sources_chunk_sumsq(ctx, c, gch[c], srcs, ex.ELIXIR_LOWP_BF16, lens[c], valid[c], 1.0 / K, not first, sh)
                else:
                    ex.elixir_grad_reduce_sources_lp(gch[c], 0, srcs, ex.ELIXIR_LOWP_BF16, lens[c], 1.0 / K, not first, sh)

    def norm():
        if fused:
            ex.elixir_chunk_grad_norm_finish(ctx, nch, cfg.max_norm, d_nc[0:1], d_nc[1:2], sh)
        else:
            ex.elixir_chunk_grad_norm(ctx, chunks, valid, cfg.max_norm, d_nc[0:1], d_nc[1:2], sh)

    def adam():
        step_no[0] += 1
        hp = ex.make_hparams(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, step_no[0])
        for c in range(nch):
            if tiled:
                ex.elixir_chunk_adam_step_tiled_lp(tiled[c], gch[c], None, out[c], ex.ELIXIR_LOWP_BF16, lens[c], hp, d_nc[1:2], None, sh)
            else:
                ex.elixir_chunk_adam_step(state[c][0], state[c][1], state[c][2], gch[c], None, out[c], lens[c], hp, d_nc[1:2], sh)

    def step():
        reduce_all()
        norm()
        adam()

    try:
        wall, ev = _event_time(torch, stream, step, args.steps, args.warmup)
        for name, fn in (("reduce", reduce_all), ("norm", norm), ("adam", adam)):
            parts[name] = _event_time(torch, stream, fn, 2, 1)[1]
        n_el = sum(lens)
        reduce_bytes = sum(2 * len(w) + 4 + (4 if w[0] > 0 else 0) for w in passes)     # per element: sources read, chunk written (+ read)
        step_bytes = (reduce_bytes + 30) * n_el + (0 if fused else 4 * sum(valid))
        emit({
            "metric": "chunked AdamW params/sec (4 micro-batches reduced, global norm, clip, step)", "value": sum(valid) / wall,
            "unit": "params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3,
            "dtype": "f32", "data": "synthetic",
            "config": {"workload": cfg.name, "params": sum(valid), "chunk_elems": C, "n_chunks": nch, "micro_batches": K,
                       "processed_elems_per_step": n_el, "padding_updated": bool(args.whole_chunks),
                       "optimizer_chunk": "tiled [master|m|v], 4096-element tiles" if tiled else "three arrays",
                       "micro_batches_per_reduction_pass": spp, "max_norm": cfg.max_norm},
            "norm": float(d_nc[0].item()), "clip_coef": float(d_nc[1].item()),
            "phase_ms": {k: v * 1e3 for k, v in parts.items()},
            "norm_fused_into_last_reduction": fused,
            "phase_GB/s": {"reduce": reduce_bytes * n_el / parts["reduce"] / 1e9,
                           "norm": None if fused else 4 * sum(valid) / parts["norm"] / 1e9,
                           "adam_fp32_grad": 30 * n_el / parts["adam"] / 1e9},
            "roofline": {"bound": "hbm", "achieved": step_bytes / 1e9 / ev, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "traffic": None,
                         "frac": step_bytes / 1e9 / ev / HBM_PEAK_GBPS,
                         "note": f"whole step: {reduce_bytes} (reduce, {len(passes)} pass{'es' if len(passes) > 1 else ''}) + 30 (AdamW, fp32 gradient) bytes per element"
                                 + ("" if fused else " + 4 per valid element (norm)")}})
    finally:
        ex.elixir_ctx_destroy(ctx)


def run_offload(args, torch, ex, gen):
    """Offload mix on the 20B set: dense layout, 128Mi-element chunks; 60% of the chunks keep [master|m|v] in pinned
    host memory and are prefetched, updated on the GPU and evicted on side streams; 40% are updated in HBM meanwhile.
    --host-chunks limits how many host-resident chunks are really allocated (the split stays 60/40)."""
    cfg = gen.CONFIGS["gpt2_20b_offload"]
    dev = torch.device("cuda:0")
    C = cfg.chunk_elems
    valid_all = ex.elixir_layout_plan(cfg.numels(), C, ex.ELIXIR_LAYOUT_DENSE, 1)[2]
    n_all = len(valid_all)
    n_host_all = -(-3 * n_all // 5)
    if args.host_order == "first":
        is_host_all = [c < n_host_all for c in range(n_all)]                   # the first 60% in schedule order
    else:
        is_host_all = [(3 * c) % 5 < 3 for c in range(n_all)]                  # 60% of the chunks, interleaved
    nbytes = 3 * C * 4
    # pin host memory first: if the box refuses the full amount, the same 60/40 mix runs on as many chunks as fit
    want = args.host_chunks if args.host_chunks > 0 else sum(is_host_all)
    t0 = time.perf_counter()
    pinned, pinned_limit = [], None
    try:
        for _ in range(want):
            pinned.append(ex.elixir_host_alloc(nbytes))
    except ex.ElixirError:
        pinned_limit = len(pinned)
        for _ in range(min(3, len(pinned) - 1)):              # leave the runtime some room
            ex.elixir_host_free(pinned.pop())
        print(f"bench.py: the box pins at most {pinned_limit} blocks of {nbytes} bytes; running with {len(pinned)} host chunks",
              file=sys.stderr, flush=True)
    t_alloc = time.perf_counter() - t0
    if args.host_order == "first":                                             # H host chunks, then 2H/3 resident ones
        H = min(len(pinned), n_host_all)
        keep = n_all if H == n_host_all else min(n_all, H + round(H * 2 / 3))
        valid, is_host = valid_all[:keep], [c < H for c in range(keep)]
    else:
        keep, h = 0, 0
        for c in range(n_all):                                                 # first chunks, whole groups of 5
            h += is_host_all[c]
            keep = c + 1
            if h >= len(pinned) and (keep % 5 == 0 or keep == n_all):
                break
        valid, is_host = valid_all[:keep], is_host_all[:keep]
        while sum(is_host) > len(pinned):                                      # a partial last group: make its tail resident
            is_host[max(c for c in range(keep) if is_host[c])] = False
    nch = len(valid)
    host_ids = [c for c in range(nch) if is_host[c]]
    n_slots = 3
    compute = compute_stream(torch)
    sh = compute.cuda_stream
    pkey = gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=cfg.cfg_id)
    gkey = gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, 0, cfg.cfg_id)
    grads = torch.zeros(nch, C, dtype=torch.int16, device=dev)
    out = torch.empty(nch, C, dtype=torch.int16, device=dev)
    resident = {c: torch.zeros(3, C, dtype=torch.float32, device=dev) for c in range(nch) if not is_host[c]}
    slots = [torch.zeros(3, C, dtype=torch.float32, device=dev) for _ in range(n_slots)]
    ctx = ex.elixir_ctx_create(0, C, 8)
    blocks = {c: pinned[i] for i, c in enumerate(host_ids)}
    for extra in pinned[len(host_ids):]:
        ex.elixir_host_free(extra)
    try:
        ex.elixir_offload_register_slots(ctx, slots, nbytes)
        h2d, d2h, duplex, waited = settled_copy_streams(ex, ctx, compute)
        # where uploads and downloads by DMA take turns (a state that follows large frees, see elixir_offload_copy_streams) the
        # slots come back by the library's store kernel instead, which needs no DMA engine
        by_kernel = args.evict_path == "kernel" or (args.evict_path == "auto" and not duplex)
        ex.elixir_offload_set_evict_path(ctx, ex.ELIXIR_EVICT_KERNEL if by_kernel else ex.ELIXIR_EVICT_DMA)

        def wall_of(fn):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            return time.perf_counter() - t0

        # ---- the link itself (run after the timed steps): bare pinned copies of whole blocks, each direction alone and both at once
        probe = [blocks[c] for c in host_ids[:min(8, len(host_ids) // 2 * 2)]]
        half = len(probe) // 2

        def only_h2d():
            for k, b in enumerate(probe):
                ex.elixir_copy_h2d_async(slots[k % n_slots], b, nbytes, h2d)

        def only_d2h():
            for k, b in enumerate(probe):
                ex.elixir_copy_d2h_async(b, slots[k % n_slots], nbytes, d2h)

        def both_ways(piece=None):
            piece = piece or nbytes
            for k in range(half):
                for at in range(0, nbytes, piece):                              # a block as one copy, or in pieces as the pipeline issues it
                    n = min(piece, nbytes - at)
                    ex.elixir_copy_h2d_async(slots[0].data_ptr() + at, probe[k] + at, n, h2d)
                    ex.elixir_copy_d2h_async(probe[half + k] + at, slots[1].data_ptr() + at, n, d2h)

        def probe_link():
            only_d2h()                                                          # first touch of the host pages
            t_up = min(wall_of(only_h2d) for _ in range(3))
            t_down = min(wall_of(only_d2h) for _ in range(3))
            t_bi = min(wall_of(both_ways) for _ in range(3))
            by_piece = {f"{p >> 20} MiB": half * nbytes / min(wall_of(lambda: both_ways(p)) for _ in range(2)) / 1e9
                        for p in (16 << 20, 64 << 20, 256 << 20)}
            return {"h2d_alone_GB/s": len(probe) * nbytes / t_up / 1e9, "d2h_alone_GB/s": len(probe) * nbytes / t_down / 1e9,
                    "bidirectional_GB/s_each_way": half * nbytes / t_bi / 1e9,
                    "bidirectional_GB/s_each_way_by_piece": by_piece,
                    "what": f"bare pinned copies of {len(probe)} blocks of {nbytes} bytes (whole blocks; by_piece: the same blocks issued in pieces; "
                            "the pipeline issues 256 MiB pieces); probed after the timed steps"}

        for c in range(nch):
            gen.fill_bf16_device(grads[c].data_ptr(), valid[c], gkey, c * C, cfg.grad_std)
            if is_host[c]:                                     # initial state: generated in a slot, evicted to the host block
                s = ex.elixir_chunk_prefetch(ctx, blocks[c], 4096, h2d)
                ex.elixir_chunk_wait_ready(ctx, s, compute)
                with torch.cuda.stream(compute):
                    slots[s].zero_()
                gen.fill_f32_device(slots[s][0].data_ptr(), valid[c], pkey, c * C, cfg.param_std, 0, sh)
                ex.elixir_chunk_evict(ctx, s, blocks[c], nbytes, compute, d2h)
            else:
                gen.fill_f32_device(resident[c][0].data_ptr(), valid[c], pkey, c * C, cfg.param_std)
        torch.cuda.synchronize()
        step_no = [0]

        def step(update=True):
            step_no[0] += update
            hp = ex.make_hparams(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, max(step_no[0], 1))
            pending, inflight = list(host_ids), []
            for c in range(nch):
                while pending and len(inflight) < n_slots:
                    try:
                        inflight.append((pending[0], ex.elixir_chunk_prefetch(ctx, blocks[pending[0]], nbytes, h2d)))
                    except ex.ElixirError as e:
                        if e.code != ex.ELIXIR_ENOSLOT:
                            raise
                        break
                    pending.pop(0)
                if is_host[c]:
                    _, s = inflight.pop(0)
                    ex.elixir_chunk_wait_ready(ctx, s, compute)
                    if update:
                        ex.elixir_chunk_adam_step(slots[s][0], slots[s][1], slots[s][2], None, grads[c], out[c], C, hp, None, sh)
                    ex.elixir_chunk_evict(ctx, s, blocks[c], nbytes, compute, d2h)
                elif update:
                    r = resident[c]
                    ex.elixir_chunk_adam_step(r[0], r[1], r[2], None, grads[c], out[c], C, hp, None, sh)

        def compute_only():
            # the same updates with nothing to wait for: host-resident chunks are updated in whatever a slot holds
            hp = ex.make_hparams(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, 1)
            for c in range(nch):
                r = slots[c % n_slots] if is_host[c] else resident[c]
                ex.elixir_chunk_adam_step(r[0], r[1], r[2], None, grads[c], out[c], C, hp, None, sh)

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / args.steps
        moved = len(host_ids) * nbytes
        t_compute = min(wall_of(compute_only) for _ in range(2))
        t_dma = wall_of(lambda: step(update=False))                             # the same schedule of copies, no kernels
        overlap = min(1.0, 1.0 - (wall - max(t_dma, t_compute)) / min(t_dma, t_compute))   # 1: the shorter of the two is hidden
        # the link itself, after the pipeline has run:
        # the probe overwrites host blocks and slots whose contents no longer matter, the timed steps being over
        link = probe_link() if half >= 1 else None
        # ceiling of the pipeline: the best both-directions rate seen in this run, bare copies or the pipeline's own copies alone
        peak = max([moved / t_dma / 1e9] + ([link["bidirectional_GB/s_each_way"]] + list(link["bidirectional_GB/s_each_way_by_piece"].values()) if link else []))
        frac = (moved / wall / 1e9) / peak
        emit({
            "metric": "chunked AdamW params/sec with 60% of the chunks streamed from pinned host memory", "value": sum(valid) / wall,
            "unit": "params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3, "dtype": "f32",
            "data": "synthetic",
            "config": {"workload": cfg.name, "layout": "dense", "chunk_elems": C, "n_chunks": nch, "n_chunks_full_set": n_all,
                       "host_chunks": len(host_ids), "resident_chunks": nch - len(host_ids), "slots": n_slots,
                       "params": sum(valid), "pinned_GB": moved / 1e9, "pinned_alloc_s": t_alloc,
                       "copy_streams": "elixir_offload_copy_streams (hardware queues of their own beside the compute stream)",
                       "uploads_and_downloads_overlap_at_start": duplex, "waited_s_for_downloads_at_full_rate": round(waited, 2),
                       "evict_path": ("store kernel (elixir_offload_set_evict_path)" + ("" if duplex else ": uploads and downloads by DMA took turns "
                                      "when the run began")) if by_kernel else "DMA",
                       "host_order": args.host_order,
                       "pinned_blocks_the_box_allowed": pinned_limit},
            "offload_GB/s_each_way": moved / wall / 1e9, "link": link,
            "frac_of_one_way_link": (moved / wall / 1e9) / max(link["h2d_alone_GB/s"], link["d2h_alone_GB/s"]) if link else None,
            "compute_only_ms": t_compute * 1e3, "copies_only_ms": t_dma * 1e3, "overlap": overlap,
            "roofline": {"bound": "host link", "achieved": moved / wall / 1e9, "unit": "GB/s each way, both directions concurrent",
                         "peak": peak, "frac": frac, "traffic": None,
                         "note": "peak = the best both-directions rate measured in this run: bare pinned copies (whole blocks or pieces) or the "
                                 "pipeline's own copies without any kernel"}})
    finally:
        torch.cuda.synchronize()
        ex.elixir_offload_register_slots(ctx, [], 0)
        for b in blocks.values():
            ex.elixir_host_free(b)
        ex.elixir_ctx_destroy(ctx)


def run_hybrid(args, torch, ex, gen):
    """Host-resident chunks of the 20B set (128Mi elements) updated two ways at once: some are streamed to the GPU and
    back ([master|m|v], 12 + 12 bytes per element over the link), the others are updated by the host cores in place,
    the paper's own treatment (only bf16 gradients come down and bf16 parameters go up: 2 + 2 bytes per element).
    Sweeps the share of host chunks given to the CPU; the resident chunks are updated on the GPU meanwhile."""
    import threading

    cfg = gen.CONFIGS["gpt2_20b_offload"]
    dev = torch.device("cuda:0")
    C = cfg.chunk_elems
    n_host = args.host_chunks if args.host_chunks > 0 else 16
    n_res = max(1, round(n_host * 2 / 3))                                  # 60 / 40
    nbytes = 3 * C * 4
    cores = len(os.sched_getaffinity(0))
    threads = args.host_threads if args.host_threads > 0 else max(1, cores - 1)   # one core stays with the thread that drives the copies
    compute, gdown = compute_stream(torch), torch.cuda.Stream()
    pup = [torch.cuda.Stream(), torch.cuda.Stream()]                              # one upload stream per parameter buffer
    sh = compute.cuda_stream
    ctx = ex.elixir_ctx_create(0, C, 8)
    N = n_host + n_res                                                     # any split of the N chunks can be run
    blocks = [ex.elixir_host_alloc(nbytes) for _ in range(N)]
    hgrad = [ex.elixir_host_alloc(2 * C) for _ in range(2)]
    hparam = [ex.elixir_host_alloc(2 * C) for _ in range(2)]
    slots = [torch.zeros(3, C, dtype=torch.float32, device=dev) for _ in range(3)]
    grads = torch.zeros(n_host + n_res, C, dtype=torch.int16, device=dev)
    out = torch.zeros(n_host + n_res, C, dtype=torch.int16, device=dev)
    resident = [torch.zeros(3, C, dtype=torch.float32, device=dev) for _ in range(N)]
    pkey = gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=cfg.cfg_id)
    gkey = gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, 0, cfg.cfg_id)
    try:
        ex.elixir_offload_register_slots(ctx, slots, nbytes)
        h2d, d2h, duplex, waited = settled_copy_streams(ex, ctx, compute)
        by_kernel = args.evict_path == "kernel" or (args.evict_path == "auto" and not duplex)   # see run_offload
        ex.elixir_offload_set_evict_path(ctx, ex.ELIXIR_EVICT_KERNEL if by_kernel else ex.ELIXIR_EVICT_DMA)
        for c in range(N):
            gen.fill_bf16_device(grads[c].data_ptr(), C, gkey, c * C, cfg.grad_std)
        for c in range(N):
            gen.fill_f32_device(resident[c][0].data_ptr(), C, pkey, c * C, cfg.param_std)
        for c in range(N):                                                 # initial state of the host blocks
            slots[0].zero_()
            gen.fill_f32_device(slots[0][0].data_ptr(), C, pkey, c * C, cfg.param_std)
            torch.cuda.synchronize()
            ex.elixir_copy_d2h_async(blocks[c], slots[0], nbytes, d2h)
            torch.cuda.synchronize()
        step_no = [0]

        def cpu_path(chunks, hp):
            # double-buffered: gradients of the next chunk come down while the cores update the current one
            if not chunks:
                return
            ex.elixir_copy_d2h_async(hgrad[0], grads[chunks[0]], 2 * C, gdown.cuda_stream)
            for i, c in enumerate(chunks):
                b = i % 2
                ex.elixir_stream_synchronize(gdown.cuda_stream)            # gradients of chunk c are in hgrad[b]
                if i + 1 < len(chunks):
                    ex.elixir_copy_d2h_async(hgrad[1 - b], grads[chunks[i + 1]], 2 * C, gdown.cuda_stream)
                if i >= 2:
                    ex.elixir_stream_synchronize(pup[b].cuda_stream)       # hparam[b] (chunk i-2) has left for the GPU
                ex.elixir_host_adam_step(blocks[c], blocks[c] + 4 * C, blocks[c] + 8 * C, None, hgrad[b], hparam[b], C, hp, 1.0, threads)
                ex.elixir_copy_h2d_async(out[c], hparam[b], 2 * C, pup[b].cuda_stream)
            for q in pup:
                ex.elixir_stream_synchronize(q.cuda_stream)

        def step(n_cpu, n_gpu=n_res):
            """One step with the first n_cpu chunks updated by the host cores, the last n_gpu chunks resident in HBM and
            the chunks in between streamed through the staging slots."""
            step_no[0] += 1
            hp = ex.make_hparams(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, step_no[0])
            cpu_chunks = list(range(n_cpu))
            gpu_chunks = list(range(n_cpu, N - n_gpu))                      # streamed
            res_chunks = list(range(N - n_gpu, N))
            worker = threading.Thread(target=cpu_path, args=(cpu_chunks, hp))
            worker.start()
            pending, inflight, r = list(gpu_chunks), [], 0
            per = -(-n_gpu // max(1, len(gpu_chunks)))
            for _ in range(max(len(gpu_chunks), 1)):
                while pending and len(inflight) < 3:
                    inflight.append((pending[0], ex.elixir_chunk_prefetch(ctx, blocks[pending.pop(0)], nbytes, h2d)))
                if inflight:
                    c, s = inflight.pop(0)
                    ex.elixir_chunk_wait_ready(ctx, s, compute)
                    ex.elixir_chunk_adam_step(slots[s][0], slots[s][1], slots[s][2], None, grads[c], out[c], C, hp, None, sh)
                    ex.elixir_chunk_evict(ctx, s, blocks[c], nbytes, compute, d2h)
                for _ in range(per):                                       # resident chunks in between
                    if r < n_gpu:
                        st = resident[res_chunks[r]]
                        ex.elixir_chunk_adam_step(st[0], st[1], st[2], None, grads[res_chunks[r]], out[res_chunks[r]], C, hp, None, sh)
                        r += 1
            while r < n_gpu:
                st = resident[res_chunks[r]]
                ex.elixir_chunk_adam_step(st[0], st[1], st[2], None, grads[res_chunks[r]], out[res_chunks[r]], C, hp, None, sh)
                r += 1
            worker.join()
            torch.cuda.synchronize()

        def timed_step(n_cpu, n_gpu=n_res):
            step(n_cpu, n_gpu)
            t = []
            for _ in range(args.steps):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                step(n_cpu, n_gpu)
                t.append(time.perf_counter() - t0)
            return min(t)

        results = []
        for n_cpu in sorted({0, n_host // 4, n_host // 2, 2 * n_host // 3, 3 * n_host // 4, 5 * n_host // 6, n_host}):
            t = timed_step(n_cpu)
            results.append({"cpu_chunks": n_cpu, "streamed_chunks": n_host - n_cpu, "ms_per_step": t * 1e3,
                            "host_resident_G_elements_per_s": n_host * C / t / 1e9})
        # the CPU update alone: this box's V_c
        hp = ex.make_hparams(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, 1)
        vc = {}
        for T in sorted({1, threads // 2, threads, cores}):
            if T < 1:
                continue
            ex.elixir_host_adam_step(blocks[0], blocks[0] + 4 * C, blocks[0] + 8 * C, None, hgrad[0], hparam[0], C, hp, 1.0, T)
            t0 = time.perf_counter()
            ex.elixir_host_adam_step(blocks[0], blocks[0] + 4 * C, blocks[0] + 8 * C, None, hgrad[0], hparam[0], C, hp, 1.0, T)
            dt = time.perf_counter() - t0
            vc[str(T)] = {"G_elements_per_s": C / dt / 1e9, "host_GB/s": 28 * C / dt / 1e9}
        best = min(results, key=lambda r: r["ms_per_step"])
        # the paper's benefit model (Sec. 5.1, Eq. 1 and 2) on what this run measured: the link rate of the all-streamed row,
        # the GPU update rate of the resident chunks, the CPU update rate on all cores
        hp = ex.make_hparams(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, 2)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(compute)
        for r_ in range(n_host, N):
            st_ = resident[r_]
            ex.elixir_chunk_adam_step(st_[0], st_[1], st_[2], None, grads[r_], out[r_], C, hp, None, sh)
        e1.record(compute)
        torch.cuda.synchronize()
        v_g = n_res * C / (e0.elapsed_time(e1) * 1e-3)
        streamed = [r for r in results if r["cpu_chunks"] == 0][0]
        link = 12.0 * n_host * C / (streamed["ms_per_step"] * 1e-3)                 # bytes/s in each direction, fill and drain included
        v_c = vc[str(cores)]["G_elements_per_s"] * 1e9
        I, J = ex.elixir_offload_benefit(1, C, link, link, v_g, v_c)
        benefit = {"B_g2c_and_B_c2g_GB/s": link / 1e9, "V_g_G_elements_per_s": v_g / 1e9, "V_c_G_elements_per_s": v_c / 1e9,
                   "I": I, "J": J, "unit_of_I_and_J": "seconds saved per step for each byte per element of GPU memory spent (chunks of C elements)",
                   "reading": "I > J: a further rCache block saves more time per byte of GPU memory than moving a chunk's update to the GPU"
                              if I > J else "J > I: moving a chunk's update to the GPU saves more time per byte of GPU memory than a further rCache block"}
        # from report to choice (paper Sec. 5.1, the rule after Eq. 2): the GPU memory the fixed 60/40 split spends on resident
        # chunks (40% of the chunks at 14 bytes per element, plus the one mandatory rCache block) is handed to
        # elixir_offload_plan with the rates just measured; the split it returns is run with the paper's own treatment of
        # host-resident chunks (updated by the CPU in place) beside the fixed split
        allowed = n_res * 14.0 * C + 2.0 * C
        n_blocks_plan, n_gpu_plan = ex.elixir_offload_plan(1, C, N, 1, allowed, link, link, v_g, v_c)
        n_gpu_plan = min(int(n_gpu_plan), N)
        plan_t = timed_step(N - n_gpu_plan, n_gpu_plan)
        fixed_cpu = [r for r in results if r["cpu_chunks"] == n_host][0]
        plan = {"allowed_bytes": allowed, "n_chunks": N, "rcache_blocks": int(n_blocks_plan), "gpu_chunks": n_gpu_plan,
                "cpu_chunks": N - n_gpu_plan, "fixed_split_gpu_chunks": n_res,
                "note": "with I > J the rule spends memory on rCache blocks before chunks, so fewer chunks are resident than in the fixed "
                        "split; the optimizer step alone cannot show what the blocks buy (they save parameter gathers in the forward "
                        "and backward pass, which this build does not run), so plan_ms is an upper bound on the plan's cost"
                        if I > J else "with J > I the rule moves chunks to the GPU first"}
        emit({
            "metric": "host-resident chunk update rate, CPU update and GPU streaming combined", "value": best["host_resident_G_elements_per_s"] * 1e9,
            "unit": "params/s", "n_gpus": 1, "steps": args.steps, "warmup": 1, "ms_per_step": best["ms_per_step"], "dtype": "f32",
            "data": "synthetic",
            "config": {"workload": "gpt2-20B/C=128Mi hybrid offload", "chunk_elems": C, "host_chunks": n_host, "resident_chunks": n_res,
                       "host_threads": threads, "host_isa": ex.elixir_host_adam_isa()},
            "sweep": results, "cpu_update_alone": vc, "benefit_model": benefit,
            "plan": plan, "plan_ms": plan_t * 1e3, "fixed60_ms": fixed_cpu["ms_per_step"], "fixed60_streamed_ms": streamed["ms_per_step"],
            "best_sweep_ms": best["ms_per_step"],
            "link": {"uploads_and_downloads_overlap_at_start": duplex, "waited_s_for_downloads_at_full_rate": round(waited, 2),
                     "evict_path": "store kernel" if by_kernel else "DMA",
                     "GB/s_each_way_all_streamed": link / 1e9,
                     "state": ("full duplex" if duplex else
                               "uploads and downloads by DMA took turns when the run began (a state of the box that follows large frees, also a "
                               "previous process's)" + (": the slots came back by the store kernel instead" if by_kernel else
                                                        ": the streamed rows and B in the benefit model are half of what a fresh process measures"))},
            "roofline": {"bound": "host memory / host link", "achieved": None, "peak": None, "frac": None, "traffic": None}})
    finally:
        torch.cuda.synchronize()
        ex.elixir_offload_register_slots(ctx, [], 0)
        for b in blocks + hgrad + hparam:
            ex.elixir_host_free(b)
        ex.elixir_ctx_destroy(ctx)


def run_tensor_lists(args, torch, ex, gen):
    """Pack / unpack and the gradient reduction over the REAL tensor list of the 1.5B set (580 tensors, 581 pieces in 26
    chunks of 64Mi elements, next-fit): what a trainer calls when gradients arrive tensor by tensor and when parameters
    are packed at set-up.  Each is timed next to the same bytes moved as whole chunks (one slice per chunk), which is the
    ceiling the tensor list can reach.  One JSON line."""
    cfg = gen.CONFIGS["gpt2_1p5b"]
    dev = torch.device("cuda:0")
    C = cfg.chunk_elems
    numels = cfg.numels()
    cid, off, valid = ex.elixir_layout_plan(numels, C, ex.ELIXIR_LAYOUT_NEXT_FIT, 1)
    nch = len(valid)
    stream = compute_stream(torch)
    sh = stream.cuda_stream
    # per chunk, side by side: the fp32 chunk, an fp32 array and a bf16 array of the same length holding the tensors' data
    groups, _keep = chunk_groups(torch, dev, nch, [("chunk", torch.float32, C, 1), ("t32", torch.float32, C, 1), ("t16", torch.int16, C, 1),
                                                   ("c16", torch.int16, C, 1)])
    gkey = gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, 1, 0, cfg.cfg_id)
    for c in range(nch):
        gen.fill_bf16_device(groups["t16"][c].data_ptr(), valid[c], gkey, c * C, cfg.grad_std, cfg.grad_zero_pct)
        gen.fill_f32_device(groups["t32"][c].data_ptr(), valid[c], gkey, c * C, cfg.param_std)
    torch.cuda.synchronize()
    # the pieces: (chunk, offset, length); the data of a tensor lies in t32 / t16 at its chunk offset
    pieces = []
    for i, n in enumerate(numels):
        c, o, left = cid[i], off[i], n
        while left > 0:
            take = min(left, C - o)
            pieces.append((c, o, take))
            left, c, o = left - take, c + 1, 0
    by_chunk = [[p for p in pieces if p[0] == c] for c in range(nch)]
    n_valid = sum(valid)
    d32 = [groups["chunk"][c][o:o + n] for c, o, n in pieces]
    s16 = [groups["t16"][c][o:o + n] for c, o, n in pieces]
    p_n = [n for _, _, n in pieces]
    reps = max(3, args.steps)

    def t(fn):
        return _event_time(torch, stream, fn, reps, 2)[1]

    # host tables built once, as a trainer whose tensor list does not change would: the timed calls should not wait for Python
    T_d32, T_s16, T_n = ex.elixir_ptr_table(d32), ex.elixir_ptr_table(s16), ex.elixir_i64_table(p_n)

    def reduce_list(acc):
        ex.elixir_grad_reduce_multi_lp(T_d32, T_s16, T_n, ex.ELIXIR_LOWP_BF16, 0.25, acc, sh)

    def reduce_chunks(acc):
        for c in range(nch):
            ex.elixir_grad_reduce_into_chunk(groups["chunk"][c], 0, groups["t16"][c], valid[c], 0.25, acc, sh)

    seg_tables = {}
    for esz, data in ((4, groups["t32"]), (2, groups["t16"])):
        for per_tensor in (True, False):
            seg_tables[esz, per_tensor] = []
            for c in range(nch):
                segs = by_chunk[c] if per_tensor else [(c, 0, valid[c])]
                seg_tables[esz, per_tensor].append((ex.elixir_ptr_table([data[c][o:o + n] for _, o, n in segs]),
                                                    ex.elixir_i64_table([n for _, _, n in segs]), ex.elixir_i64_table([o for _, o, _ in segs])))

    def pack(esz, per_tensor, unpack=False):
        chunks = groups["chunk"] if esz == 4 else groups["c16"]
        fn = ex.elixir_chunk_unpack if unpack else ex.elixir_chunk_pack
        tabs = seg_tables[esz, per_tensor]
        for c in range(nch):
            fn(chunks[c], C, esz, tabs[c][0], tabs[c][1], tabs[c][2], sh)

    set_views = {4: ex.elixir_ptr_table([groups["t32"][c][o:o + n] for c, o, n in pieces]), 2: T_s16}
    set_chunks = {4: ex.elixir_ptr_table(groups["chunk"]), 2: ex.elixir_ptr_table(groups["c16"])}
    T_c, T_o = ex.elixir_i64_table([c for c, _, _ in pieces]), ex.elixir_i64_table([o for _, o, _ in pieces])

    def pack_set(esz, unpack=False):
        fn = ex.elixir_chunks_unpack if unpack else ex.elixir_chunks_pack
        fn(set_chunks[esz], C, esz, set_views[esz], T_n, T_c, T_o, sh)

    res = {}
    for name, fn, nbytes in (
            ("reduce_overwrite_tensor_list", lambda: reduce_list(False), 6 * n_valid),
            ("reduce_overwrite_whole_chunks", lambda: reduce_chunks(False), 6 * n_valid),
            ("reduce_accumulate_tensor_list", lambda: reduce_list(True), 10 * n_valid),
            ("reduce_accumulate_whole_chunks", lambda: reduce_chunks(True), 10 * n_valid),
            ("pack_fp32_tensor_list", lambda: pack(4, True), 8 * n_valid + 4 * (nch * C - n_valid)),
            ("pack_fp32_whole_chunks", lambda: pack(4, False), 8 * n_valid + 4 * (nch * C - n_valid)),
            ("pack_fp32_whole_set_one_call", lambda: pack_set(4), 8 * n_valid + 4 * (nch * C - n_valid)),
            ("unpack_fp32_whole_set_one_call", lambda: pack_set(4, True), 8 * n_valid),
            ("pack_bf16_whole_set_one_call", lambda: pack_set(2), 4 * n_valid + 2 * (nch * C - n_valid)),
            ("unpack_bf16_whole_set_one_call", lambda: pack_set(2, True), 4 * n_valid),
            ("unpack_fp32_tensor_list", lambda: pack(4, True, True), 8 * n_valid),
            ("unpack_fp32_whole_chunks", lambda: pack(4, False, True), 8 * n_valid),
            ("pack_bf16_tensor_list", lambda: pack(2, True), 4 * n_valid + 2 * (nch * C - n_valid)),
            ("pack_bf16_whole_chunks", lambda: pack(2, False), 4 * n_valid + 2 * (nch * C - n_valid)),
            ("unpack_bf16_tensor_list", lambda: pack(2, True, True), 4 * n_valid),
            ("unpack_bf16_whole_chunks", lambda: pack(2, False, True), 4 * n_valid)):
        sec = t(fn)
        res[name] = {"ms": sec * 1e3, "bytes": nbytes, "GB/s": nbytes / sec / 1e9, "frac": nbytes / sec / 1e9 / HBM_PEAK_GBPS}
    head = res["reduce_overwrite_tensor_list"]
    emit({"metric": "gradient reduction and pack / unpack over the tensor list of the set", "value": head["GB/s"], "unit": "GB/s",
          "steps": reps, "warmup": 2, "ms_per_step": head["ms"], "dtype": "f32",
          "config": {"workload": "gpt2-1.5B/C=64Mi tensor lists", "tensors": len(numels), "pieces": len(pieces), "n_chunks": nch,
                     "params": n_valid, "placement": "elixir_arena_plan: per chunk [fp32 chunk | fp32 data | bf16 data | bf16 chunk] side by side"},
          "rows": res,
          "roofline": {"bound": "hbm", "achieved": head["GB/s"], "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": head["frac"], "traffic": None,
                       "kernel": "reduce_multi_kernel<false, false> (bf16 -> fp32, overwrite, 6 bytes per element)"}})


def run_link_after_free(args, torch, ex, gen):
    """What a large hipFree does to the host link: bare pinned copies of 256 MiB (upload alone, download alone, both at
    once, on two streams of their own) every half second after 16, 64 and 128 GiB of device memory have been freed.
    One JSON line; the time series is what profiles/host_link_after_a_large_free.txt summarises."""
    dev = torch.device("cuda:0")
    n = 256 << 20
    h_up, h_dn = ex.elixir_host_alloc(n), ex.elixir_host_alloc(n)
    d_up = torch.zeros(n, dtype=torch.uint8, device=dev)
    d_dn = torch.zeros(n, dtype=torch.uint8, device=dev)
    s_up, s_dn = torch.cuda.Stream(), torch.cuda.Stream()

    def rate(up, dn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if up:
            ex.elixir_copy_h2d_async(d_up, h_up, n, s_up.cuda_stream)
        if dn:
            ex.elixir_copy_d2h_async(h_dn, d_dn, n, s_dn.cuda_stream)
        torch.cuda.synchronize()
        return n / (time.perf_counter() - t0) / 1e9

    try:
        for _ in range(3):
            rate(True, True)
        fresh = {"up_alone": rate(True, False), "down_alone": rate(False, True), "both_each_way": rate(True, True)}
        series = []
        for gib in (16, 64, 128):
            x = torch.zeros(gib << 30, dtype=torch.uint8, device=dev)
            torch.cuda.synchronize()
            del x
            t0 = time.perf_counter()
            torch.cuda.empty_cache()
            t_free = time.perf_counter() - t0
            rows, settled = [], None
            for k in range(40):
                t = time.perf_counter() - t0
                d, u, b = rate(False, True), rate(True, False), rate(True, True)
                rows.append({"t_s": round(t, 2), "down_alone": round(d, 1), "up_alone": round(u, 1), "both_each_way": round(b, 1)})
                if b > 0.9 * fresh["both_each_way"] and d > 0.9 * fresh["down_alone"]:
                    settled = settled if settled is not None else t
                    if k >= 3:
                        break
                time.sleep(0.5)
            series.append({"freed_GiB": gib, "hipFree_s": round(t_free, 4), "first_sample_at_full_rate_s": None if settled is None else round(settled, 2),
                           "samples": rows})
        emit({"metric": "host link after a large free", "value": fresh["both_each_way"], "unit": "GB/s each way, fresh", "steps": 1, "warmup": 0,
              "ms_per_step": None, "dtype": "u8", "config": {"workload": "host link after a large free", "copy_bytes": n}, "fresh": fresh, "after_free": series,
              "roofline": {"bound": "host link", "achieved": fresh["both_each_way"], "peak": None, "unit": "GB/s", "frac": None, "traffic": None}})
    finally:
        torch.cuda.synchronize()
        ex.elixir_host_free(h_up)
        ex.elixir_host_free(h_dn)


def naive_allocation_row(args, torch, ex, gen, cfg, valid, lens, dev, stream):
    """The same step with every array an ordinary allocation of its own (what a caller gets who does not plan where its
    buffers lie): per chunk one tiled optimizer chunk, two gradient sets, one parameter copy, each from torch's allocator."""
    C, nch, sh = cfg.chunk_elems, len(valid), stream.cuda_stream
    tiled = [torch.zeros(ex.elixir_state_tiled_len(C), dtype=torch.float32, device=dev) for _ in range(nch)]
    out = [torch.zeros(C, dtype=torch.int16, device=dev) for _ in range(nch)]
    sets = [[torch.zeros(C, dtype=torch.int16, device=dev) for _ in range(nch)] for _ in range(2)]
    pkey = gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=cfg.cfg_id)
    scratch = torch.zeros(3, C, dtype=torch.float32, device=dev)
    for c in range(nch):
        scratch[0].zero_()
        gen.fill_f32_device(scratch[0].data_ptr(), valid[c], pkey, c * C, cfg.param_std)
        ex.elixir_state_tile(tiled[c], scratch[0], scratch[1], scratch[2], C)
        for s_, g in enumerate(sets):
            gen.fill_bf16_device(g[c].data_ptr(), valid[c], gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, s_ + 1, 0, cfg.cfg_id), c * C,
                                 cfg.grad_std, cfg.grad_zero_pct)
    torch.cuda.synchronize()
    del scratch
    step_no = [0]

    def step():
        step_no[0] += 1
        hp = ex.make_hparams(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, step_no[0])
        g = sets[step_no[0] % 2]
        for c in range(nch):
            ex.elixir_chunk_adam_step_tiled_lp(tiled[c], None, g[c], out[c], ex.ELIXIR_LOWP_BF16, lens[c], hp, None, None, sh)

    wall, ev = _event_time(torch, stream, step, 6, 2)
    gbs = BYTES_PER_ELEM * sum(lens) / ev / 1e9
    return {"what": "the benchmark step with one ordinary allocation per array (tiled optimizer chunk, 2 gradient sets, parameter copy per chunk)",
            "ms_per_step": wall * 1e3, "params_per_s": sum(valid) / wall, "GB/s": gbs, "frac": gbs / HBM_PEAK_GBPS, "steps": 6}


def other_configs(args, torch, ex, gen):
    """Short runs of the other benchmark configurations, after the timed region of the benchmark line and with its buffers
    freed: the tiny set (one batched launch per step), the chunk-size sweep, gradient accumulation + clipping on the 6B
    set (one and four micro-batches per reduction pass) and the 20B offload mix (as many host chunks as the box pins).
    Each is the workload `--workload <name>` runs, with fewer steps; a failure is recorded and does not touch the line."""
    import gc
    global SINK
    rows = {}
    drop = ("n_gpus", "higher_is_better", "scaling", "vs_baseline", "data", "dtype", "rows", "cpu_baseline")

    def collect(name, fn, **over):
        global SINK
        sub = argparse.Namespace(**{**vars(args), **{k: v for k, v in over.items() if k != "free_after"}})
        SINK = []
        t0 = time.perf_counter()
        try:
            r = fn(sub, torch, ex, gen)
            if isinstance(r, dict):          # run_headline hands its line back instead of emitting it
                SINK.append(r)
            lines = [{k: v for k, v in ln.items() if k not in drop} for ln in SINK]
            rows[name] = {"lines": lines, "took_s": round(time.perf_counter() - t0, 1)}
        except Exception as e:  # noqa: BLE001
            rows[name] = {"error": f"{type(e).__name__}: {e}", "lines": SINK}
        finally:
            SINK = None
            gc.collect()
            torch.cuda.synchronize()
            if over.get("free_after", True):
                torch.cuda.empty_cache()

    dev = torch.device("cuda:0")
    want = set(args.configs.split(","))
    if "5" in want:
        # first, and with nothing large freed since the process began (torch keeps the benchmark line's buffers cached): after a
        # large hipFree the runtime makes uploads and downloads by DMA take turns for a while.  Should that state be there all
        # the same, the slots come back by the store kernel (--evict-path auto).
        collect("config_5_20b_offload_mix", run_offload, steps=2, warmup=1, free_after=False)
    if "f" in want:
        # the paper's own treatment of host-resident chunks (updated by the host cores) and the split its benefit model
        # chooses from what the run measures; it streams as well, so it too comes before anything large is freed
        collect("f1_f2_hybrid_20b", run_hybrid, steps=2, free_after=False)
    gc.collect()
    torch.cuda.empty_cache()
    if "1" in want:
        collect("config_1_tiny", lambda a, *rest: run_headline(a, *rest, dev), workload="tiny", no_rows=True, multi=True)
    if "3" in want:
        collect("config_3_sweep", run_sweep, steps=5, warmup=2)
    if "4" in want:
        collect("config_4_6b_accumulate_clip", run_clip, steps=3, warmup=1, sources_per_pass=1)
        collect("config_4_6b_accumulate_clip_4_per_pass", run_clip, steps=3, warmup=1, sources_per_pass=4)
    return rows


OTHER_WORKLOADS = {"link_after_free": run_link_after_free, "tensor_lists": run_tensor_lists, "sweep": run_sweep, "gpt2_6b_clip": run_clip, "gpt2_20b_offload": run_offload, "gpt2_20b_hybrid": run_hybrid}


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); the path would shard by giving "
              "each rank a 1/N slice of every chunk, which is not built here.", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2212_05339_amd as ex
    from synth import gen

    from paper_2212_05339_amd.build import ensure_built
    ensure_built()   # compiles only if no library is there
    ex.lib()         # fail loudly if the HIP library is still missing: there is no other path
    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload in OTHER_WORKLOADS:
        OTHER_WORKLOADS[args.workload](args, torch, ex, gen)
        return
    line = run_headline(args, torch, ex, gen, dev)
    if args.workload == "gpt2_1p5b" and not args.no_rows and not args.no_configs:
        line["rows"].update(other_configs(args, torch, ex, gen))
    if not args.no_cpu_baseline:
        try:
            cfg = gen.CONFIGS[args.workload]
            valid0 = ex.elixir_layout_plan(cfg.numels(), cfg.chunk_elems, ex.ELIXIR_LAYOUT_NEXT_FIT, 1)[2][0]
            line["cpu_baseline"] = cpu_baseline(cfg, valid0, budget_elems=32 * 64 * gen.Mi)
        except Exception as e:  # noqa: BLE001
            line["cpu_baseline_error"] = f"{type(e).__name__}: {e}"
    emit(line)


def run_headline(args, torch, ex, gen, dev):
    """The benchmark line: K AdamW steps over every chunk of the workload (gpt2_1p5b or tiny), then the side rows on the
    same buffers.  Returns the line; its buffers are gone when it returns."""
    cfg = gen.CONFIGS[args.workload]
    C = cfg.chunk_elems
    numels = cfg.numels()
    valid = ex.elixir_layout_plan(numels, C, ex.ELIXIR_LAYOUT_NEXT_FIT, 1)[2]
    nch = len(valid)
    K, W = args.steps, args.warmup
    if C <= 16 * gen.Mi:
        args.multi = True

    stream = compute_stream(torch)
    sh = stream.cuda_stream
    # ---- state, resident in HBM ----
    state, _g_unused, out, _keep = chunk_buffers(torch, dev, nch, C)
    pkey = gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=cfg.cfg_id)
    for c in range(nch):
        gen.fill_f32_device(state[c][0].data_ptr(), valid[c], pkey, c * C, cfg.param_std)
    # ---- gradients: a ring of sets that is cycled (each set is far larger than any cache) ----
    tiled = None
    if args.state_layout == "tiled":
        # per chunk [tiled optimizer chunk | gradient sets] side by side; the parameter copies elsewhere
        n_sets = max(1, min(K + W, 8))
        groups, _keep_g = chunk_groups(torch, dev, nch, [("state", torch.float32, ex.elixir_state_tiled_len(C), 1), ("grad", torch.int16, C, n_sets)])
        tiled = groups["state"]
        grads = [[(groups["grad"][c][s] if n_sets > 1 else groups["grad"][c]) for c in range(nch)] for s in range(n_sets)]
        for c in range(nch):
            ex.elixir_state_tile(tiled[c], state[c][0], state[c][1], state[c][2], C)
        out_far = out_of_the_way(torch, dev, nch * (2 * C + STAGGER_BYTES), lambda: chunk_groups(torch, dev, nch, [("out", torch.int16, C, 1)], far=True))
        out, _keep_o = out_far[0]["out"], out_far[1]
    else:
        free_b, _ = torch.cuda.mem_get_info()
        gstride = C + STAGGER_BYTES // 2
        set_bytes = nch * gstride * 2
        n_sets = max(1, min(K + W, int(0.8 * free_b // set_bytes)))
        gflat = torch.zeros(n_sets * nch * gstride, dtype=torch.int16, device=dev)   # padding stays zero
        grads = [[gflat[(s * nch + c) * gstride: (s * nch + c) * gstride + C] for c in range(nch)] for s in range(n_sets)]
    for s in range(n_sets):
        gkey = gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, s + 1, 0, cfg.cfg_id)
        for c in range(nch):
            gen.fill_bf16_device(grads[s][c].data_ptr(), valid[c], gkey, c * C, cfg.grad_std, cfg.grad_zero_pct)
    torch.cuda.synchronize()

    p_list, m_list, v_list = [st[0] for st in state], [st[1] for st in state], [st[2] for st in state]
    # what a launch covers: the chunk's valid prefix (padding is all-zero bits and an update would leave it so: never touched),
    # or, with --whole-chunks, the padding as well
    lens = [C] * nch if args.whole_chunks else list(valid)

    clip_ctx = ex.elixir_ctx_create(0, C, nch) if args.max_norm > 0 else None
    d_nc = torch.zeros(2, dtype=torch.float32, device=dev)
    gscale = d_nc[1:2] if clip_ctx is not None else None

    def one_step(step_no):
        hp = ex.make_hparams(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, step_no)
        g = grads[(step_no - 1) % n_sets]
        o = g if args.params_over_grads else out
        if clip_ctx is not None:
            ex.elixir_chunk_grad_norm_lp(clip_ctx, g, ex.ELIXIR_LOWP_BF16, valid, 1.0, args.max_norm, d_nc[0:1], d_nc[1:2], sh)
        if args.multi and tiled:
            ex.elixir_chunk_adam_step_tiled_multi_lp(tiled, None, g, o, ex.ELIXIR_LOWP_BF16, lens, hp, gscale, None, sh)
            return
        if args.multi:
            ex.elixir_chunk_adam_step_multi(p_list, m_list, v_list, None, g, o, lens, hp, gscale, sh)
            return
        for c in range(nch):
            if tiled:
                ex.elixir_chunk_adam_step_tiled_lp(tiled[c], None, g[c], o[c], ex.ELIXIR_LOWP_BF16, lens[c], hp, gscale, None, sh)
            else:
                ex.elixir_chunk_adam_step(state[c][0], state[c][1], state[c][2], None, g[c], o[c], lens[c], hp, gscale, sh)

    for w in range(W):
        one_step(w + 1)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for k in range(K):
        one_step(W + k + 1)
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = e0.elapsed_time(e1)

    # the same steps once more with an event after each, for the spread (kept out of the timed region above)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    marks[0].record(stream)
    for k in range(K):
        one_step(W + K + k + 1)
        marks[k + 1].record(stream)
    torch.cuda.synchronize()
    per_step_in_order = [marks[k].elapsed_time(marks[k + 1]) for k in range(K)]
    per_step = sorted(per_step_in_order)

    total_params = sum(valid)
    bpe = BYTES_PER_ELEM + (2 if clip_ctx is not None else 0)   # with clipping the norm's read of the bf16 gradients is in the region too
    if args.multi:
        # a batched call cuts the chunks into grid rows and may split a step over several launches: the library decides, so
        # no per-launch figure is derived here; the rate over the whole timed region is the same number
        launches, launch_s, per_launch_elems = None, None, None
        achieved = bpe * sum(lens) * K / (ev_ms * 1e-3) / 1e9
    else:
        launches = K * nch
        per_launch_elems = sum(lens) / nch                   # average over the launches of a step
        launch_s = ev_ms * 1e-3 / launches                   # average duration of one launch of the AdamW kernel
        achieved = bpe * per_launch_elems / launch_s / 1e9   # GB/s, algorithmic bytes of one launch
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "adam_step_traffic.json")
    if os.path.exists(tpath) and args.workload == "gpt2_1p5b" and clip_ctx is None and not args.multi:
        with open(tpath) as f:                                 # counters were read on whole-chunk launches: scale to this run's average launch
            t = json.load(f)
            traffic = round(t["hbm_bytes_per_launch"] / t["algorithmic_bytes_per_launch"] * BYTES_PER_ELEM * per_launch_elems)
            traffic_source = ("not read in this run: the HBM-bytes / algorithmic-bytes ratio of the rocprofv3 counter runs recorded in "
                              "profiles/adam_step_traffic.json times this run's bytes per launch")

    line = {
        "metric": "chunked AdamW params/sec", "value": total_params * K / wall, "unit": "params/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": wall * 1e3 / K, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "params": total_params, "chunk_elems": C, "n_chunks": nch,
                   "processed_elems_per_step": sum(lens), "padding_updated": bool(args.whole_chunks), "layout": "next-fit", "grad_dtype": "bf16",
                   "optimizer_chunk": "tiled [master|m|v], 4096-element tiles" if tiled else "three arrays",
                   "lowp_params": "written over the gradients" if args.params_over_grads else "an array of their own",
                   "clip": (f"max-norm {args.max_norm}: norm over the bf16 gradient chunks every step (2 more bytes per element, "
                            f"inside the timed region; last norm {float(d_nc[0].item()):.4f})") if clip_ctx is not None else "none",
                   "placement": ("elixir_arena_plan: per chunk [optimizer chunk | gradient sets] side by side in one allocation with "
                                 "4 MiB + 8 KiB gaps; the parameter copies in a second allocation made behind a temporary spacer of up to "
                                 "100 GiB (rows.naive_allocation: every array an allocation of its own)") if tiled else
                                "one allocation per kind of array, 4 MiB + 8 KiB gaps",
                   "grad_sets_resident": n_sets, "hparams": {"lr": cfg.lr, "betas": [cfg.beta1, cfg.beta2],
                                                             "eps": cfg.eps, "weight_decay": cfg.weight_decay}},
        "elements_per_s": sum(lens) * K / wall,
        "step_ms_device": {"median": per_step[K // 2], "min": per_step[0], "max": per_step[-1],
                           "in_order": [round(x, 4) for x in per_step_in_order], "grad_set_of_first": (W + K) % n_sets,
                           "what": "HIP events around each of K further steps"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": (("adam_multi_kernel<1, 1, true>" if tiled else "adam_multi_kernel<1, 1, false>") if args.multi else
                                "adam_tiled_kernel<1, 1>" if tiled else "adam_vec_kernel<1, 1>") + " (bf16 gradient in, bf16 copy out)" +
                               (" with the step's sumsq_lowp_kernel<false> shared out over its launches" if clip_ctx is not None else ""),
                     "bytes_per_launch": bpe * per_launch_elems if launches else None,
                     "launch_ms": launch_s * 1e3 if launches else None, "launches_timed": launches,
                     "timing": "HIP events on the launch stream around the timed region" + (" / launches" if launches else
                               " (batched calls: the library chooses the launches, the rate is bytes of the region / its duration)")},
    }
    if clip_ctx is not None:
        ex.elixir_ctx_destroy(clip_ctx)
    line["rows"] = {}
    if not args.no_rows:
        # the side measurements come after the timed region: if one of them cannot run on this machine (e.g. no pinned memory
        # left for the offload row) the benchmark line above still stands and says what happened
        try:
            line["rows"] = side_rows(ex, gen, torch, cfg, C, nch, valid, state, grads, out, stream, wall * 1e3 / K)
            if "pack" in line["rows"]:   # the plain device copy of this library, measured in the same run
                line["roofline"]["frac_of_measured_device_copy"] = achieved / line["rows"]["pack"]["GB/s"]
        except Exception as e:  # noqa: BLE001
            line["rows_error"] = f"{type(e).__name__}: {e}"
        if args.workload == "gpt2_1p5b" and tiled:
            try:
                line["rows"]["naive_allocation"] = naive_allocation_row(args, torch, ex, gen, cfg, valid, lens, dev, stream)
            except Exception as e:  # noqa: BLE001
                line["rows"]["naive_allocation"] = {"error": f"{type(e).__name__}: {e}"}
    return line


if __name__ == "__main__":
    main()
