#!/usr/bin/env python3
"""Benchmark of the batched KV-cache compression stage on one MI355X.

A step is one fc_compress_batch over the whole batch (score -> select ->
allocate -> gather -> reclaim) with every input already resident in HBM.
Between steps only the pool metadata (free stack, block tables, lengths) is
rewound, by two small device-side copies.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config4|config3|config2]
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak

# HBM bytes per launch of the dominant kernel, measured with rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE and scaled by what the same counters read for a plain
# 4 GiB copy (FETCH_SIZE x 2.000, WRITE_SIZE x 1.000 on this chip); summary and
# commands in profiles/fused_unit_kernel_config2_config3_config4.md.
MEASURED_TRAFFIC_BYTES = {
    ("config3_batched_mixed", "fused_unit"): 25.95e9,
    ("config4_multi_image", "fused_unit"): 214.57e9,
    # profiles/mlp_compress_kernel_config4_mlp.md
    ("config4_multi_image_mlp", "mlp_compress"): 211.99e9,
}


def cpu_baseline(dw, seconds=15.0, seed=0):
    """The CPU oracle, as it stands, timed on a bounded random sample of
    (request, layer, head) units of the same workload (bytes downloaded from
    the device pool; the download is not timed).  One thread."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_limits
    from oracle import fastcache_oracle as fo
    wl = dw.wl
    rng = np.random.Generator(np.random.PCG64(seed))
    n_lh = wl.n_layers * wl.n_heads
    bt0 = dw.bt0.cpu().numpy()
    spent, token_heads, units = 0.0, 0, 0
    with threadpool_limits(limits=1):
        while spent < seconds and units < 4096:
            r = int(rng.integers(wl.n_req))
            l = int(rng.integers(wl.n_layers))
            h = int(rng.integers(wl.n_heads))
            if wl.methods[r] == fo.METHOD_NONE:
                continue
            L, B = int(wl.seq_lens[r]), int(wl.budgets[r])
            n_old, n_new = fo.blocks_for(L, wl.block_size), fo.blocks_for(B, wl.block_size)
            ids = torch.from_numpy(bt0[r, :n_old].astype(np.int64)).to(dw.dev)
            mini = np.zeros((1, n_old + n_new, 2, 1, wl.block_size, wl.head_dim), np.float16)
            mini[0, :n_old, :, 0] = dw.kv[l, ids, :, h].cpu().numpy()
            q = dw.q[r:r + 1, l:l + 1, h:h + 1].cpu().numpy()
            st = fo.FreeStack(n_old + n_new)
            bt = st.alloc(n_old)[None, :].copy()
            lens = np.array([L], dtype=np.int32)
            t0 = time.perf_counter()
            status, _, _ = fo.compress_batch(mini, st, bt, lens, q, wl.window,
                                             wl.methods[r:r + 1], wl.budgets[r:r + 1],
                                             wl.pool_kernel)
            spent += time.perf_counter() - t0
            assert status is None
            token_heads += L
            units += 1
    return {
        "value": token_heads / n_lh / spent,
        "unit": "tokens/s",
        "cores": 1,
        "kind": "oracle",
        "sample": "%d random (request, layer, head) units of %s = %d token-heads in %.1f s, "
                  "scaled by 1/%d layer-heads per token" % (units, wl.name, token_heads, spent,
                                                            n_lh),
    }


MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X published dense fp16 MFMA peak


def cpu_baseline_mlp(dw, weights, k, img_b, img_e, seconds=15.0, seed=0):
    """The chunk-MLP oracle, as it stands, timed on random (request, layer,
    head, K|V) units of the same workload.  One thread."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_limits
    from oracle import fastcache_oracle as fo
    from oracle import mlp_compressor_oracle as mo
    wl = dw.wl
    rng = np.random.Generator(np.random.PCG64(seed))
    n_units = wl.n_layers * wl.n_heads * 2
    bt0 = dw.bt0.cpu().numpy()
    w = {kk: [t.cpu().numpy() for t in v] for kk, v in weights.items()}
    spent, tokens, units = 0.0, 0, 0
    with threadpool_limits(limits=1):
        while spent < seconds and units < 4096:
            r = int(rng.integers(wl.n_req))
            l = int(rng.integers(wl.n_layers))
            h = int(rng.integers(wl.n_heads))
            kv = int(rng.integers(2))
            L = int(wl.seq_lens[r])
            n_old = fo.blocks_for(L, wl.block_size)
            ids = torch.from_numpy(bt0[r, :n_old].astype(np.int64)).to(dw.dev)
            rows = dw.kv[l, ids, kv, h].cpu().numpy().reshape(-1, wl.head_dim)[:L].astype(np.float64)
            t0 = time.perf_counter()
            plan = mo.chunk_plan(L, int(img_b[r]), int(img_e[r]), k)
            mo.compress_rows(rows, plan, w, k)
            spent += time.perf_counter() - t0
            tokens += L
            units += 1
    return {
        "value": tokens / n_units / spent,
        "unit": "tokens/s",
        "cores": 1,
        "kind": "oracle",
        "sample": "%d random (request, layer, head, K|V) units of %s = %d token rows in %.1f s, "
                  "scaled by 1/%d units per token" % (units, wl.name, tokens, spent, n_units),
    }


def bench_mlp(args, wl):
    """The chunk-MLP compressor on the same batch: text 64 | image | text 64,
    k = 5, hidden 256, seeded random weights.  The roofline object names
    whichever of the two published peaks (HBM, dense fp16 MFMA) takes longer for
    this shape; the other fraction is reported under "path"."""
    import numpy as np
    import torch
    from paper_2503_08461_amd import fastcache as fc
    from paper_2503_08461_amd.device_setup import DeviceWorkload
    k, hidden, d = 5, 256, wl.head_dim
    wl.name += "_mlp"
    dw = DeviceWorkload(wl, verbose=True)
    gen = torch.Generator(device=dw.dev)
    gen.manual_seed(wl.seed + 5000)
    w1 = [(torch.randn((hidden, k * d), generator=gen, device=dw.dev) / (k * d) ** 0.5).half()
          for _ in range(2)]
    w2 = [(torch.randn((d, hidden), generator=gen, device=dw.dev) / hidden ** 0.5).half()
          for _ in range(2)]
    b1 = [0.1 * torch.randn(hidden, generator=gen, device=dw.dev) for _ in range(2)]
    b2 = [0.1 * torch.randn(d, generator=gen, device=dw.dev) for _ in range(2)]
    fc.fc_mlp_set_weights(dw.pool, k, w1, b1, w2, b2)
    img_b = np.full(wl.n_req, 64, dtype=np.int32)
    img_e = (wl.seq_lens - 64).astype(np.int32)

    def step():
        dw.rewind_async()
        fc.fc_compress_batch_mlp(dw.pool, dw.bt, dw.lens, img_b, img_e)

    for _ in range(args.warmup):
        step()
    fc.fc_set_profiling(dw.pool, True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    kms = fc.fc_get_kernel_times(dw.pool)
    n_units = wl.n_layers * wl.n_heads * 2
    tokens = int(wl.seq_lens.astype(np.int64).sum())
    chunks = int(sum(-(-64 // k) + -(-(int(L) - 128) // k) + -(-64 // k) for L in wl.seq_lens))
    flops = chunks * n_units * 2.0 * (k * d * hidden + hidden * d)
    bytes_ = n_units * (tokens + chunks) * 2 * d
    ksec = kms["mlp_compress"] * 1e-3
    tf, gbs = flops / ksec / 1e12, bytes_ / ksec / 1e9
    hbm_bound = bytes_ / (HBM_PEAK_GBPS * 1e9) >= flops / (MFMA_F16_PEAK_TFLOPS * 1e12)
    if hbm_bound:
        roof = {"kernel": "mlp_compress", "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": gbs / HBM_PEAK_GBPS,
                "traffic": MEASURED_TRAFFIC_BYTES.get((wl.name, "mlp_compress"))}
    else:
        roof = {"kernel": "mlp_compress", "bound": "mfma", "achieved": tf,
                "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / MFMA_F16_PEAK_TFLOPS, "traffic": None}
    out = {
        "metric": "KV tokens compressed/sec (all layers x heads), batched, chunk-MLP compressor",
        "value": tokens / sec, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": wl.name, "n_req": wl.n_req, "tokens": tokens, "k": k,
                   "hidden": hidden, "rows_out": chunks, "pool_GiB": round(wl.pool_bytes() / 2**30, 1)},
        "path": {"flops": flops, "algorithmic_bytes": bytes_,
                 "kernel_TFLOPs": tf, "mfma_frac": tf / MFMA_F16_PEAK_TFLOPS,
                 "kernel_GBps": gbs, "hbm_frac": gbs / HBM_PEAK_GBPS},
        "kernel_ms": {kk: round(v, 4) for kk, v in kms.items() if v > 0},
        "roofline": roof,
    }
    if args.cpu_seconds > 0:
        dw.rewind()
        out["cpu_baseline"] = cpu_baseline_mlp(dw, {"w1": w1, "b1": b1, "w2": w2, "b2": b2}, k,
                                               img_b, img_e, seconds=args.cpu_seconds)
    dw.close()
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config4",
                    choices=["config2", "config3", "config4", "config4_streaming", "config4_mlp"],
                    help="config4_streaming: the config-4 batch with every request using the "
                         "score-free sinks + recent rule (gather and pool work only); "
                         "config4_mlp: the config-4 batch through the chunk-MLP compressor "
                         "(k = 5, hidden 256, synthetic weights)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="CPU time budget of the oracle baseline (0 = skip)")
    ap.add_argument("--score-mode", default="auto", choices=["auto", "two_pass", "one_pass"],
                    help="which SnapKV score kernel the library uses")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of known size (reference for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the stage has no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2503_08461_amd import synth, fastcache as fc
    from paper_2503_08461_amd.device_setup import DeviceWorkload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if args.calibrate_copy:
        n = 4 << 30
        src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": True, "bytes_read_per_copy": n,
                          "bytes_written_per_copy": n, "copies": 5}), flush=True)
        return
    fc.load_library()
    wl = synth.make_workload(int(args.workload[6]))
    if args.workload.endswith("_streaming"):
        wl.methods[:] = synth.METHOD_STREAMING
        wl.name += "_streaming"
    need = wl.pool_bytes() + (8 << 30)
    total = torch.cuda.get_device_properties(0).total_memory
    if need > total:
        print("bench.py: %s needs %.0f GiB, device has %.0f GiB" % (
            wl.name, need / 2**30, total / 2**30), file=sys.stderr)
        sys.exit(2)

    if args.workload.endswith("_mlp"):
        bench_mlp(args, wl)
        return
    dw = DeviceWorkload(wl, verbose=True)
    fc.fc_set_score_mode(dw.pool, {"auto": 0, "two_pass": 1, "one_pass": 2}[args.score_mode])
    fc.fc_set_profiling(dw.pool, True)
    for _ in range(args.warmup):
        dw.rewind()
        dw.compress()
    torch.cuda.synchronize()

    # The K timed steps run back to back.  The metadata rewind between them is
    # two small device-side copies issued on the same stream, inside the timed
    # region (it costs a few microseconds and keeps the GPU from idling and
    # down-clocking between steps, as it would not in a serving loop).
    fc.fc_set_profiling(dw.pool, True)    # restart the per-kernel averages
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        dw.rewind_async()
        dw.compress()
    torch.cuda.synchronize()
    sec_per_step = (time.perf_counter() - t0) / args.steps
    kavg = fc.fc_get_kernel_times(dw.pool)  # HIP events around every kernel of those steps

    comp = wl.methods != synth.METHOD_NONE
    tokens = int(wl.seq_lens[comp].astype(np.int64).sum())
    path_bytes = dw.algorithmic_bytes()
    kbytes = dw.kernel_algorithmic_bytes(8192 if args.score_mode == "auto" else 0)
    # dominant kernel = the one with the largest average duration
    dom = max(kbytes, key=lambda k: kavg.get(k, 0.0))
    dom_gbps = kbytes[dom] / (kavg[dom] * 1e-3) / 1e9

    out = {
        "metric": "KV tokens compressed/sec (all layers x heads), batched",
        "value": tokens / sec_per_step,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": sec_per_step * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "dtype_note": "fp16 K/V/Q and MFMA inputs, fp32 accumulation, softmax and scores",
        "data": "synthetic",
        "config": {
            "workload": wl.name,
            "n_req": wl.n_req, "tokens": tokens, "n_layers": wl.n_layers,
            "n_heads": wl.n_heads, "head_dim": wl.head_dim, "window": wl.window,
            "pool_blocks": wl.n_blocks, "pool_GiB": round(wl.pool_bytes() / 2**30, 1),
            "kept_fraction": round(float(wl.budgets[comp].sum()) / tokens, 4),
            "score_mode": args.score_mode,
        },
        "path": {
            "algorithmic_bytes": path_bytes,
            "achieved_GBps": path_bytes / sec_per_step / 1e9,
            "frac_of_hbm_peak": path_bytes / sec_per_step / 1e9 / HBM_PEAK_GBPS,
        },
        "kernel_ms": {k: round(v, 4) for k, v in kavg.items()},
        "roofline": {
            "kernel": dom,
            "bound": "hbm",
            "achieved": dom_gbps,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": dom_gbps / HBM_PEAK_GBPS,
            "traffic": MEASURED_TRAFFIC_BYTES.get((wl.name, dom)) if args.score_mode == "auto"
            else None,
        },
    }
    if args.cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(dw, args.cpu_seconds)
    dw.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
