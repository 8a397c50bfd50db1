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

CSRC_DIR = os.path.join(ROOT, "paper_2503_08461_amd", "csrc")
PROFILES_DIR = os.path.join(ROOT, "profiles")


def csrc_digest():
    """Short hash of every kernel and host source of the library: a traffic
    figure measured with rocprofv3 belongs to the sources it was measured on."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC_DIR)):
        if name.endswith((".hip", ".h", ".cpp")):
            h.update(name.encode())
            with open(os.path.join(CSRC_DIR, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def kernel_symbol(slot, wl, pruning):
    """The kernel's name in a rocprofv3 trace for the library's timing slot
    `slot` on workload wl (None where a slot covers several kernels)."""
    nt = 1 if wl.window <= 16 else (2 if wl.window <= 32 else 4)
    if slot == "fused_unit":
        return "fc::%s<%d, %d>" % ("fused_bounded_kernel" if pruning else "fused_unit_kernel",
                                   wl.head_dim, nt)
    if slot == "snapkv_score":
        return "fc::snapkv_score_kernel<%d, %d>" % (wl.head_dim, nt)
    if slot in ("gather", "knorm_score"):
        return "fc::%s_kernel<%d>" % (slot, wl.head_dim)
    return None


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload` from the rocprofv3 counter
    summaries under profiles/ (FETCH_SIZE and WRITE_SIZE, each scaled by what it
    reads for a plain copy of known size).  A summary states its figure in a line
      traffic-record: workload=<name> kernel=<name> bytes=<float> csrc=<digest> commit=<hash>
    and the figure counts only while the library sources still hash to <digest>:
    returns (bytes, where it comes from), or (None, why not)."""
    import re
    now = csrc_digest()
    stale = None
    for name in sorted(os.listdir(PROFILES_DIR)) if os.path.isdir(PROFILES_DIR) else []:
        if not name.endswith((".md", ".txt")):
            continue
        with open(os.path.join(PROFILES_DIR, name)) as f:
            for line in f:
                m = re.match(r"\s*traffic-record:\s*workload=(\S+)\s+kernel=(\S+)\s+bytes=(\S+)"
                             r"\s+csrc=(\S+)\s+commit=(\S+)", line)
                if not m or m.group(1) != workload or m.group(2) != kernel:
                    continue
                if m.group(4) == now:
                    return float(m.group(3)), "profiles/%s (commit %s, csrc %s)" % (
                        name, m.group(5), now)
                stale = "profiles/%s was measured on other sources (csrc %s, now %s)" % (
                    name, m.group(4), now)
    return None, stale or "no rocprofv3 counter summary for this kernel and workload"


def _oracle_unit(job):
    """Worker of the all-cores baseline: one (request, layer, head) unit through
    the oracle, single-threaded.  Returns the unit's token count."""
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle import fastcache_oracle as fo
    mini, q, L, window, method, budget, pool_kernel, n_old = job
    st = fo.FreeStack(mini.shape[1])
    bt = st.alloc(n_old)[None, :].copy()
    lens = np.array([L], dtype=np.int32)
    with threadpool_limits(limits=1):
        status, _, _ = fo.compress_batch(mini, st, bt, lens, q, window,
                                         np.array([method], np.int32),
                                         np.array([budget], np.int32), pool_kernel)
    assert status is None
    return L


def _worker_ready(_):
    from oracle import fastcache_oracle  # noqa: F401  (import cost outside the timed region)
    return os.getpid()


def _sample_unit(dw, rng):
    """Inputs of one random (request, layer, head) unit, downloaded from the
    device pool as a one-layer, one-head pool of its own."""
    import numpy as np
    import torch
    from oracle import fastcache_oracle as fo
    wl = dw.wl
    while True:
        r = int(rng.integers(wl.n_req))
        if wl.methods[r] != fo.METHOD_NONE:
            break
    l = int(rng.integers(wl.n_layers))
    h = int(rng.integers(wl.n_heads))
    L, B = int(wl.seq_lens[r]), int(wl.budgets[r])
    n_old, n_new = fo.blocks_for(L, wl.block_size), fo.blocks_for(B, wl.block_size)
    ids = torch.from_numpy(dw.bt0_host[r, :n_old].astype(np.int64)).to(dw.dev)
    mini = np.zeros((1, n_old + n_new, 2, 1, wl.block_size, wl.head_dim), np.float16)
    mini[0, :n_old, :, 0] = dw.kv[l, ids, :, h].cpu().numpy()
    q = dw.q[r:r + 1, l:l + 1, h:h + 1].cpu().numpy()
    return (mini, q, L, wl.window, int(wl.methods[r]), B, wl.pool_kernel, n_old)


def cpu_baseline(dw, seconds=15.0, seed=0):
    """The CPU oracle, as it stands, timed on bounded random samples of
    (request, layer, head) units of the same workload (bytes downloaded from
    the device pool; the download is not timed): first on one core, then on all
    the cores this process may use, one single-threaded oracle per core over
    independent units (a process pool; the time includes handing the units to
    the workers).  `value` is the all-cores figure."""
    import multiprocessing as mp
    import numpy as np
    wl = dw.wl
    rng = np.random.Generator(np.random.PCG64(seed))
    n_lh = wl.n_layers * wl.n_heads
    dw.bt0_host = dw.bt0.cpu().numpy()
    # ---- one core
    spent, token_heads, units = 0.0, 0, 0
    while spent < 0.4 * seconds and units < 4096:
        job = _sample_unit(dw, rng)
        t0 = time.perf_counter()
        token_heads += _oracle_unit(job)
        spent += time.perf_counter() - t0
        units += 1
    one = {"value": token_heads / n_lh / spent, "unit": "tokens/s", "cores": 1,
           "sample": "%d units = %d token-heads in %.1f s" % (units, token_heads, spent)}
    # ---- all cores (the GPU machine gives a one-GPU job 16 of them, whatever nproc says)
    n_workers = max(1, min(16, len(os.sched_getaffinity(0))))
    spent, token_heads, units = 0.0, 0, 0
    with mp.get_context("spawn").Pool(n_workers) as pool:
        pool.map(_worker_ready, range(4 * n_workers), chunksize=1)
        while spent < 0.6 * seconds and units < 16384:
            jobs = [_sample_unit(dw, rng) for _ in range(3 * n_workers)]
            t0 = time.perf_counter()
            token_heads += sum(pool.map(_oracle_unit, jobs, chunksize=1))
            spent += time.perf_counter() - t0
            units += len(jobs)
    return {
        "value": token_heads / n_lh / spent,
        "unit": "tokens/s",
        "cores": n_workers,
        "kind": "oracle",
        "sample": "%d random (request, layer, head) units of %s = %d token-heads in %.1f s of "
                  "wall time on %d single-threaded worker processes, scaled by 1/%d layer-heads "
                  "per token" % (units, wl.name, token_heads, spent, n_workers, n_lh),
        "one_core": one,
    }


MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X published dense fp16 MFMA peak


def cpu_baseline_mlp(dw, weights, k, img_b, img_e, activation, seconds=15.0, seed=0):
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
            mo.compress_rows(rows, plan, w, k, activation)
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
    k, hidden, d = 5, args.mlp_hidden, wl.head_dim
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
    act = {"gelu_erf": fc.FC_ACT_GELU_ERF, "gelu_tanh": fc.FC_ACT_GELU_TANH}[args.mlp_activation]
    fc.fc_mlp_set_weights(dw.pool, k, w1, b1, w2, b2, act)
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
                "traffic": measured_traffic(wl.name, "mlp_compress")[0],
                "traffic_source": measured_traffic(wl.name, "mlp_compress")[1]}
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
                   "hidden": hidden, "activation": args.mlp_activation, "rows_out": chunks, "pool_GiB": round(wl.pool_bytes() / 2**30, 1)},
        "path": {"flops": flops, "algorithmic_bytes": bytes_,
                 "kernel_TFLOPs": tf, "mfma_frac": tf / MFMA_F16_PEAK_TFLOPS,
                 "kernel_GBps": gbs, "hbm_frac": gbs / HBM_PEAK_GBPS},
        "kernel_ms": {kk: round(v, 4) for kk, v in kms.items() if v > 0},
        "roofline": roof,
    }
    if args.cpu_seconds > 0:
        dw.rewind()
        out["cpu_baseline"] = cpu_baseline_mlp(dw, {"w1": w1, "b1": b1, "w2": w2, "b2": b2}, k,
                                               img_b, img_e, args.mlp_activation,
                                               seconds=args.cpu_seconds)
    dw.close()
    print(json.dumps(out), flush=True)


def bench_replay(args):
    """Replay of a Poisson arrival trace through the compress stage (Algorithm
    1's loop around `kv_c <- C(kv, lambda)`): requests with the config-4 length
    mix arrive already prefilled (their blocks are taken from the pool at
    arrival, or they wait for admission), the C-ABI scheduler forms batches
    from the pool's free count, every batch is really compressed on the GPU
    (SnapKV, window 64, keep 20 %) and its measured time advances the simulated
    clock; a compressed request then holds its blocks for a modelled decode
    residence and releases them.  Prefill and decode are a stage-time MODEL
    (constants below), the compress times are measurements."""
    import numpy as np
    import torch
    from paper_2503_08461_amd import synth, fastcache as fc
    dev = torch.device("cuda:0")
    n_layers, n_heads, d, W = 32, 32, 128, 64
    n_blocks = 8192                      # 64 GiB pool
    B_MIN, B_MAX, MAX_WAIT_US = 2, 32, 50_000
    DECODE_RESIDENCE_US = 2_000_000      # model: 64 output tokens at about 30 ms per step
    N_REQ = 200
    RESERVE = 1024                       # blocks that admission leaves free, so that compression
                                         # (which needs new blocks) can always proceed
    kv = torch.empty((n_layers, n_blocks, 2, n_heads, 16, d), dtype=torch.float16, device=dev)
    for l in range(n_layers):
        kv[l].normal_(0.0, 1.0)
    q = torch.randn((B_MAX, n_layers, n_heads, W, d), device=dev).half()
    pool = fc.fc_pool_create(kv, n_blocks, n_layers, n_heads, d)
    max_blocks = synth.blocks_for(576 * 12 + 128)
    out = []
    for rate in (1, 5, 10, 20, 40, 200, 1000):
        rng = np.random.Generator(np.random.PCG64(4000 + rate))
        arrivals = np.cumsum(rng.exponential(1e6 / rate, size=N_REQ)).astype(np.int64)
        lens = (576 * rng.integers(2, 13, size=N_REQ) + 128).astype(np.int32)
        budgets = np.maximum(lens // 5, W).astype(np.int32)
        sched = fc.Scheduler(B_MIN, B_MAX, MAX_WAIT_US)
        rows = {}                        # id -> device tensor of block ids
        admission, holding = [], []      # waiting ids; (release time, id)
        waits, batch_sizes, busy_us, now = [], [], 0, 0
        nxt, done, peak_used, adm_waits = 0, 0, 0, 0
        admitted_at = {}

        last_submit = [0]

        def admit(i, t):
            need = synth.blocks_for(int(lens[i]))
            if fc.fc_pool_num_free(pool) < need + RESERVE:
                return False
            rows[i] = fc.fc_pool_alloc(pool, need)
            # the compress queue takes submissions in time order: a request that
            # arrived while an earlier one was being admitted enters right after it
            t = max(t, last_submit[0])
            last_submit[0] = t
            admitted_at[i] = t
            assert sched.submit(i, t, int(lens[i]), int(budgets[i]))
            return True

        spins = 0
        while done < N_REQ:
            spins += 1
            if spins > 3_000_000:
                raise RuntimeError("replay cannot make progress at %d req/s" % rate)
            # next event: arrival, release, or the wait-time trigger
            cand = []
            if nxt < N_REQ:
                cand.append(int(arrivals[nxt]))
            if holding:
                cand.append(holding[0][0])
            if sched.pending() and not sched.ready(now):
                cand.append(now + 1000)  # poll the trigger every millisecond of simulated time
            if not sched.ready(now) and cand:
                now = max(now, min(cand))
            while holding and holding[0][0] <= now:
                _, i = holding.pop(0)
                fc.fc_pool_free(pool, rows.pop(i))
                done += 1
            still = []
            for i in admission:
                if not admit(i, now):
                    still.append(i)
            admission = still
            while nxt < N_REQ and arrivals[nxt] <= now:
                if admission or not admit(nxt, int(arrivals[nxt])):
                    admission.append(nxt)
                    adm_waits += 1
                nxt += 1
            peak_used = max(peak_used, n_blocks - fc.fc_pool_num_free(pool))
            batch = sched.form_batch(now, fc.fc_pool_num_free(pool))
            if not batch:
                if sched.ready(now) and not holding and not admission and nxt >= N_REQ:
                    raise RuntimeError("replay cannot make progress: pool too small")
                if sched.ready(now):
                    # nothing fits: wait for the next release
                    now = max(now, holding[0][0]) if holding else now + 1000
                continue
            n = len(batch)
            bt = torch.full((n, max_blocks), -1, dtype=torch.int32, device=dev)
            for r, i in enumerate(batch):
                bt[r, :rows[i].shape[0]] = rows[i]
            blens = lens[batch].copy()
            meth = np.full(n, synth.METHOD_SNAPKV, np.int32)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fc.fc_compress_batch(pool, bt, blens, q[:n], W, meth, budgets[batch].copy(), 7)
            torch.cuda.synchronize()
            dt = max(1, int((time.perf_counter() - t0) * 1e6))
            for r, i in enumerate(batch):
                waits.append(now - admitted_at[i])
                rows[i] = bt[r, :synth.blocks_for(int(budgets[i]))].clone()
                holding.append((now + dt + DECODE_RESIDENCE_US, i))
            holding.sort()
            now += dt
            busy_us += dt
            batch_sizes.append(n)
            sched.adjust(dt)
        sched.close()
        w = np.array(waits, dtype=np.float64) / 1e3
        out.append({"rate_req_s": rate, "batches": len(batch_sizes),
                    "mean_batch": round(float(np.mean(batch_sizes)), 2),
                    "mean_wait_ms": round(float(w.mean()), 3),
                    "p95_wait_ms": round(float(np.percentile(w, 95)), 3),
                    "compress_ms_per_request": round(busy_us / 1e3 / N_REQ, 3),
                    "compress_busy_frac": round(busy_us / max(now, 1), 5),
                    "peak_pool_occupancy": round(peak_used / n_blocks, 3),
                    "arrivals_that_waited_for_admission": adm_waits})
        assert fc.fc_pool_num_free(pool) == n_blocks
    fc.fc_pool_destroy(pool)
    print(json.dumps({
        "metric": "compress-stage queueing under Poisson arrivals (C-ABI scheduler, measured "
                  "compress times, modelled decode residence)",
        "unit": "ms", "n_gpus": 1, "data": "synthetic", "dtype": "f16",
        "config": {"workload": "replay_config4_mix", "requests_per_rate": N_REQ,
                   "pool_blocks": n_blocks, "admission_reserve_blocks": RESERVE, "b_min": B_MIN, "b_max": B_MAX,
                   "max_wait_ms": MAX_WAIT_US / 1e3,
                   "decode_residence_ms_model": DECODE_RESIDENCE_US / 1e3},
        "rates": out}), flush=True)


def bench_decode(args, wl):
    """Decode-side traffic on the config-4 batch: the single-query attention of
    one decode step over the paged cache before and after the batch is
    compressed (same kernel, same pool; after compression every head's kept
    rows are dense in the new blocks), and the one-token append."""
    import numpy as np
    import torch
    from paper_2503_08461_amd import fastcache as fc
    from paper_2503_08461_amd.device_setup import DeviceWorkload
    wl.name += "_decode"
    dw = DeviceWorkload(wl, verbose=True)
    n_lh = wl.n_layers * wl.n_heads
    d = wl.head_dim
    gen = torch.Generator(device=dw.dev)
    gen.manual_seed(wl.seed + 6000)
    q = torch.randn((wl.n_req, wl.n_layers, wl.n_heads, d), generator=gen, device=dw.dev).half()
    new_kv = torch.randn((wl.n_req, wl.n_layers, 2, wl.n_heads, d), generator=gen,
                         device=dw.dev).half()
    out = torch.empty((wl.n_req, wl.n_layers, wl.n_heads, d), dtype=torch.float32, device=dw.dev)
    fc.fc_set_profiling(dw.pool, True)

    def timed_attention():
        for _ in range(args.warmup):
            fc.fc_decode_attention(dw.pool, dw.bt, dw.lens, q, out)
        fc.fc_set_profiling(dw.pool, True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fc.fc_decode_attention(dw.pool, dw.bt, dw.lens, q, out)
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / args.steps
        ms = fc.fc_get_kernel_times(dw.pool)["decode_attention"]
        tokens = int(dw.lens.astype(np.int64).sum())
        bytes_ = tokens * n_lh * 4 * d                    # every K and V row once
        return {"tokens": tokens, "ms_per_step": sec * 1e3, "kernel_ms": ms,
                "algorithmic_bytes": bytes_, "kernel_GBps": bytes_ / (ms * 1e-3) / 1e9,
                "frac_of_hbm_peak": bytes_ / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}

    before = timed_attention()
    kept = torch.empty(int(wl.budgets.astype(np.int64).sum()) * n_lh, dtype=torch.int32,
                       device=dw.dev)
    dw.compress(None, kept)
    torch.cuda.synchronize()
    after = timed_attention()

    # the counterfactual: the same kept tokens read in place from the uncompacted
    # cache (the old blocks are intact: compaction writes only into free blocks)
    def timed_kept():
        call = lambda: fc.fc_decode_attention_kept(dw.pool, dw.bt0, wl.seq_lens, wl.budgets, kept,
                                                   q, out)
        for _ in range(args.warmup):
            call()
        fc.fc_set_profiling(dw.pool, True)
        torch.cuda.synchronize()
        for _ in range(args.steps):
            call()
        torch.cuda.synchronize()
        ms = fc.fc_get_kernel_times(dw.pool)["decode_attention"]
        bytes_ = after["algorithmic_bytes"]
        return {"tokens": after["tokens"], "kernel_ms": ms, "algorithmic_bytes": bytes_,
                "kernel_GBps": bytes_ / (ms * 1e-3) / 1e9,
                "frac_of_hbm_peak": bytes_ / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}

    uncompacted = timed_kept()
    # the append: one step (every further step would move the lengths)
    lens = dw.lens.copy()
    fc.fc_set_profiling(dw.pool, True)
    fc.fc_append_batch(dw.pool, dw.bt, lens, new_kv)
    torch.cuda.synchronize()
    app_ms = fc.fc_get_kernel_times(dw.pool)["append"]
    app_bytes = wl.n_req * n_lh * 2 * d * 2 * 2          # rows read and written
    print(json.dumps({
        "metric": "cached tokens attended/sec in one decode step (all layers x heads), "
                  "after compression",
        "value": after["tokens"] / (after["ms_per_step"] * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": after["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": wl.name, "n_req": wl.n_req, "pool_GiB": round(wl.pool_bytes() / 2**30, 1)},
        "decode_attention_before_compression": before,
        "decode_attention_after_compression": after,
        "decode_attention_kept_tokens_without_compaction": uncompacted,
        "append": {"kernel_ms": app_ms, "algorithmic_bytes": app_bytes,
                   "kernel_GBps": app_bytes / (app_ms * 1e-3) / 1e9},
        "roofline": {"kernel": "decode_attention", "bound": "hbm",
                     "achieved": after["kernel_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": after["frac_of_hbm_peak"],
                     "traffic": measured_traffic(wl.name, "decode_attention")[0],
                     "traffic_source": measured_traffic(wl.name, "decode_attention")[1],
                     "note": "the launch over the compressed caches"},
    }), flush=True)
    dw.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config4",
                    choices=["config2", "config3", "config4", "config3_precall70", "config3_lse",
                             "config4_lse",
                             "config4_streaming", "config4_mlp", "config4_decode", "replay"],
                    help="config3_precall70: the config-3 batch in a pool that is 70 %% full BEFORE "
                         "the call, compressed as two half-batches (one call would need more "
                         "free blocks than there are); configN_lse: the batch of config N with the window rows' log-sum-exp "
                         "supplied as an input (computed before the timed region, as the "
                         "prefill's attention kernel would have), one pass over K; "
                         "config4_streaming: the config-4 batch with every request using the "
                         "score-free sinks + recent rule (gather and pool work only); "
                         "config4_mlp: the config-4 batch through the chunk-MLP compressor "
                         "(k = 5, hidden 256, synthetic weights)")
    ap.add_argument("--mlp-activation", default="gelu_erf", choices=["gelu_erf", "gelu_tanh"],
                    help="activation of the chunk-MLP workload")
    ap.add_argument("--mlp-hidden", type=int, default=256, choices=[128, 256],
                    help="hidden width of the chunk-MLP workload")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="CPU time budget of the oracle baseline (0 = skip)")
    ap.add_argument("--score-mode", default="auto", choices=["auto", "two_pass"],
                    help="scheduling: fused per-unit kernel, or separate kernels for everything")
    ap.add_argument("--score-pruning", type=int, default=1, choices=[0, 1],
                    help="1: fc_set_score_pruning (the fused kernel bounds the column sums in its "
                         "first pass over K and re-reads only the rows that can decide the selection)")
    ap.add_argument("--with-lse-variant", action="store_true",
                    help="also time the same batch through fc_compress_batch_lse (row log-sum-exp "
                         "supplied, computed before the timed region) and report it beside the value")
    ap.add_argument("--csrc-digest", action="store_true",
                    help="print the hash of the library sources that a traffic-record line "
                         "in profiles/ has to carry, and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of known size (reference for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.csrc_digest:
        print(csrc_digest())
        return
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
    if args.workload == "replay":
        bench_replay(args)
        return
    wl = synth.make_workload(int(args.workload[6]))
    if args.workload.endswith("_precall70"):
        synth.precall_occupancy_variant(wl, 0.70)
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
    if args.workload.endswith("_decode"):
        bench_decode(args, wl)
        return
    out = run_stage(args, wl, args.cpu_seconds, lse_variant=args.with_lse_variant)
    if args.workload == "config4":
        # the default run also carries config 3 (the benchmark spec sets its bar on both)
        torch.cuda.empty_cache()
        c3 = run_stage(args, synth.make_workload(3), 0.0, lse_variant=False)
        out["config3"] = {k: c3[k] for k in ("value", "unit", "ms_per_step", "config", "path",
                                             "call_ms", "kernel_ms", "roofline")}
    print(json.dumps(out), flush=True)


def run_stage(args, wl, cpu_seconds, lse_variant=False):
    """Times fc_compress_batch on one workload; returns the result object."""
    import numpy as np
    import torch
    from paper_2503_08461_amd import synth, fastcache as fc
    from paper_2503_08461_amd.device_setup import DeviceWorkload
    dw = DeviceWorkload(wl, verbose=True)
    fc.fc_set_score_mode(dw.pool, {"auto": 0, "two_pass": 1}[args.score_mode])
    fc.fc_set_score_pruning(dw.pool, bool(args.score_pruning))
    fc.fc_set_profiling(dw.pool, True)
    lse_ms = None
    if args.workload.endswith("_precall70"):
        dw.parts = 2
    if args.workload.endswith("_lse"):
        wl.name += "_lse_supplied"
        dw.compute_lse()
        dw.compute_lse()
        lse_ms = fc.fc_get_kernel_times(dw.pool)["window_lse"]
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

    # the same call timed one at a time (HIP events on the stream it runs on,
    # metadata rewound outside the events): median and minimum
    call_ms = []
    for _ in range(args.steps):
        dw.rewind()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        dw.compress()
        e1.record()
        torch.cuda.synchronize()
        call_ms.append(e0.elapsed_time(e1))
    call_ms.sort()

    comp = wl.methods != synth.METHOD_NONE
    tokens = int(wl.seq_lens[comp].astype(np.int64).sum())
    path_bytes = dw.algorithmic_bytes()
    kbytes = dw.kernel_algorithmic_bytes(args.score_mode)
    # dominant kernel = the one with the largest average duration
    dom = max(kbytes, key=lambda k: kavg.get(k, 0.0))
    # (a batch issued as several calls launches the kernel once per call:
    # the average launch moves that share of the bytes)
    dom_gbps = kbytes[dom] / dw.parts / (kavg[dom] * 1e-3) / 1e9
    # (records of the fused kernel without the pruned second pass are kept under a name of their own)
    traffic, traffic_source = measured_traffic(
        wl.name, dom if args.score_pruning or dom != "fused_unit" else "fused_unit_two_pass")
    if args.score_mode != "auto":
        traffic, traffic_source = None, "counters are kept for the default scheduling only"

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
            "score_pruning": bool(args.score_pruning),
        },
        "path": {
            "algorithmic_bytes": path_bytes,
            "achieved_GBps": path_bytes / sec_per_step / 1e9,
            "frac_of_hbm_peak": path_bytes / sec_per_step / 1e9 / HBM_PEAK_GBPS,
        },
        "call_ms": {"median": call_ms[len(call_ms) // 2], "min": call_ms[0],
                    "note": "one call at a time, HIP events around it"},
        "kernel_ms": {k: round(v, 4) for k, v in kavg.items()},
        "roofline": {
            "kernel": dom,
            # the name rocprofv3 shows for it (profiles/ summaries are keyed by that name)
            # (a call that brings the row log-sum-exps has no second pass to prune)
            "kernel_symbol": kernel_symbol(dom, wl, bool(args.score_pruning)
                                           and not args.workload.endswith("_lse")),
            "bound": "hbm",
            "achieved": dom_gbps,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": dom_gbps / HBM_PEAK_GBPS,
            "traffic": traffic,
            "traffic_source": traffic_source,
        },
    }
    if dw.parts > 1:
        out["config"]["calls_per_step"] = dw.parts
    if lse_variant and lse_ms is None and dw.parts == 1 and \
            bool((wl.methods == synth.METHOD_SNAPKV).any()):
        # the same batch when the caller hands over the window rows' log-sum-exp
        # (one pass over K); reported beside the headline value, never as it
        dw.compute_lse()
        for _ in range(2):
            dw.rewind()
            dw.compress()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            dw.rewind_async()
            dw.compress()
        torch.cuda.synchronize()
        sec_lse = (time.perf_counter() - t0) / args.steps
        dw.lse = None
        out["with_row_lse_supplied"] = {
            "entry_point": "fc_compress_batch_lse",
            "ms_per_step": sec_lse * 1e3,
            "value": tokens / sec_lse,
            "achieved_GBps": path_bytes / sec_lse / 1e9,
            "frac_of_hbm_peak": path_bytes / sec_lse / 1e9 / HBM_PEAK_GBPS,
            "note": "log-sum-exp input computed before the timed region (fc_window_lse)",
        }
    if lse_ms is not None:
        out["config"]["lse_input"] = ("fc_window_lse before the timed region, %.3f ms "
                                      "(not part of value)" % lse_ms)
    if cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(dw, cpu_seconds)
    dw.close()
    del dw
    return out


if __name__ == "__main__":
    main()
