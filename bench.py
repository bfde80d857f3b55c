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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt2_1p5b", help="gpt2_1p5b (default) or tiny")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-rows", action="store_true", help="skip the per-row side measurements")
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
    return {"value": n * steps / dt, "unit": "params/s", "cores": threads, "kind": "oracle",
            "sample": f"chunk 0 of the workload ({n} elements), {steps} consecutive AdamW steps with bf16 write-back, "
                      f"{dt:.2f} s wall on {threads} threads"}


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); the path would shard by giving "
              "each rank a 1/N slice of every chunk, which is not built here.", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2212_05339_amd as ex
    from synth import gen

    ex.lib()   # fail loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = gen.CONFIGS[args.workload]
    C = cfg.chunk_elems
    numels = cfg.numels()
    cid, off, valid = ex.elixir_layout_plan(numels, C, ex.ELIXIR_LAYOUT_NEXT_FIT, 1)
    nch = len(valid)
    K, W = args.steps, args.warmup

    stream = torch.cuda.Stream()
    sh = stream.cuda_stream
    # ---- state, resident in HBM ----
    state = torch.empty(nch, 3, C, dtype=torch.float32, device=dev)     # [chunk][master | m | v]
    state.zero_()
    out = torch.empty(nch, C, dtype=torch.int16, device=dev)
    pkey = gen.stream_key(gen.BASE_SEED, gen.TAG_PARAM, cfg=cfg.cfg_id)
    for c in range(nch):
        gen.fill_f32_device(state[c, 0].data_ptr(), valid[c], pkey, c * C, cfg.param_std)
    # ---- gradients: one set per step where memory allows, else a ring that is cycled ----
    free_b, _ = torch.cuda.mem_get_info()
    set_bytes = nch * C * 2
    n_sets = max(1, min(K + W, int(0.8 * free_b // set_bytes)))
    grads = torch.zeros(n_sets, nch, C, dtype=torch.int16, device=dev)   # padding stays zero
    for s in range(n_sets):
        gkey = gen.stream_key(gen.BASE_SEED, gen.TAG_GRAD, s + 1, 0, cfg.cfg_id)
        for c in range(nch):
            gen.fill_bf16_device(grads[s, c].data_ptr(), valid[c], gkey, c * C, cfg.grad_std, cfg.grad_zero_pct)
    torch.cuda.synchronize()

    def one_step(step_no):
        hp = ex.make_hparams(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, step_no)
        g = grads[(step_no - 1) % n_sets]
        for c in range(nch):
            ex.elixir_chunk_adam_step(state[c, 0], state[c, 1], state[c, 2], None, g[c], out[c], C, hp, None, sh)

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

    total_params = sum(valid)
    launches = K * nch
    launch_s = ev_ms * 1e-3 / launches                      # average duration of one launch of the AdamW kernel
    achieved = BYTES_PER_ELEM * C / launch_s / 1e9          # GB/s, algorithmic bytes of one launch
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "adam_step_traffic.json")
    if os.path.exists(tpath) and args.workload == "gpt2_1p5b":
        with open(tpath) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")

    line = {
        "metric": "chunked AdamW params/sec", "value": total_params * K / wall, "unit": "params/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": wall * 1e3 / K, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "params": total_params, "chunk_elems": C, "n_chunks": nch,
                   "processed_elems_per_step": nch * C, "layout": "next-fit", "grad_dtype": "bf16",
                   "grad_sets_resident": n_sets, "hparams": {"lr": cfg.lr, "betas": [cfg.beta1, cfg.beta2],
                                                             "eps": cfg.eps, "weight_decay": cfg.weight_decay}},
        "elements_per_s": nch * C * K / wall,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "kernel": "adam_vec_kernel<bf16 grad, bf16 out>", "bytes_per_launch": BYTES_PER_ELEM * C,
                     "launch_ms": launch_s * 1e3, "launches_timed": launches,
                     "timing": "HIP events on the launch stream around the timed region / launches"},
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg, valid[0], budget_elems=32 * 64 * gen.Mi)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
