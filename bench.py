#!/usr/bin/env python3
"""Benchmark of the HashAttention decode layer-step on one MI355X.

A step is one pass of the whole hot path over one layer: encode query -> SCORE + TOPK ->
GATHER-ATT (preceded by the one-token append where the workload has one).  Steps walk a ring of
distinct layers (own K/V, codes and mapping weights) whose codes and weights alone exceed the 256 MB
Infinity Cache, so a step reads everything from HBM, as a decode that streams the model's weights
between two visits of a layer does.  A whole sweep over the ring is
captured in one HIP graph and replayed, which removes the host's launch cost from the step as a
serving loop would.

Prints ONE JSON line: whole-step effective GB/s (algorithmic bytes = key codes + gathered K/V rows
+ Q/O), the roofline record of the dominant kernel (GATHER-ATT) from HIP-event timing, the speed-up
over the in-house dense decode kernel on the same buffers, and the CPU oracle timed on the host.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
METRIC = "µs/layer decode step + effective HBM GB/s (% of peak), 32× sparsity, 1 GPU"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=640)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", default="C1", choices=list(WORKLOADS),
                    help="C1 = Llama-3.1-8B layer, B=1, N=32768, k=1024 (the headline configuration)")
    ap.add_argument("--ring", type=int, default=0, help="distinct layers walked by the steps (0 = per workload)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--score-table", action="store_true",
                    help="also time SCORE + TOPK alone on uniform random codes of 32..512 bits at this workload's shape")
    ap.add_argument("--sink", type=int, default=0, help="always keep this many first tokens (k counts the rest)")
    ap.add_argument("--local", type=int, default=0, help="always keep this many most recent tokens")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for scaling rocprofv3 byte counters)")
    return ap.parse_args()


# workload name -> (config factory, ring length): the steps walk a ring of distinct layers whose key codes and mapping weights
# alone exceed the 256 MB Infinity Cache (the K/V rows are loaded with the non-temporal hint and do not
# displace them), so that every read of a step comes from HBM, as it does in a model that streams its
# weights between two visits of a layer.  Measured: C1 takes 23.9 us per step on a ring of 32 layers
# (codes and weights stay cached) and 25.7 us from 128 layers on.
WORKLOADS = {
    "C1": (lambda W: W.c1(), 128),
    "C1-128K": (lambda W: W.scaled(W.c1(context=131072), name="C1-128K"), 64),
    "C2": (lambda W: W.c2(), 5),
    "C3": (lambda W: W.c3(), 20),
    "C3-16x": (lambda W: W.scaled(W.c3(k=32768), name="C3-16x"), 20),
    "C4": (lambda W: W.c4(), 7),
}


def workload_config(name):
    import workloads as W
    make, ring = WORKLOADS[name]
    return make(W), ring


def device_layer_from_host(L, torch, ha):
    """Layer 0 of the ring: the numpy arrays of workloads.make_layer, so the oracle sees the same bytes."""
    from paper_2412_14468_amd.runner import LayerState
    dev = "cuda:0"
    as_bf16 = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    return LayerState(as_bf16(L.q), as_bf16(L.k), as_bf16(L.v), torch.from_numpy(L.seq_lens.copy()).to(dev),
                      int(L.seq_lens.max()), [torch.from_numpy(w).to(dev) for w in L.w_q],
                      [torch.from_numpy(w).to(dev) for w in L.w_kv], None, int(L.k_per_seq.max()))


def device_layer_synthetic(cfg, seed, torch):
    """Ring layers drawn on the device by the same recipe (workloads.device_tensors)."""
    import workloads as W
    from paper_2412_14468_amd.runner import layer_from_tensors
    t = W.device_tensors(cfg, seed)
    s = layer_from_tensors(t)
    s.lens_host, s.k_host = t["seq_lens_host"], t["k_per_seq_host"]
    return s


def describe_lengths(v):
    return str(v[0]) if min(v) == max(v) else f"{min(v)}..{max(v)} (sum {sum(v)})"


def stored_traffic(workload):
    """HBM bytes per GATHER-ATT launch from the committed rocprofv3 --pmc summary, if there is one
    (counters cannot be read from inside this process)."""
    path = os.path.join(ROOT, "profiles", "gather_attend_traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload)
    except (OSError, ValueError):
        return None


def time_region(torch, fn, reps):
    """Wall-clock seconds of reps calls of fn, bracketed by device synchronisation."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def capture(torch, body):
    """Capture body() (launches on torch's current stream) into a HIP graph; returns a replay callable."""
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        body()                                   # first run outside capture: lazy module loads happen here
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        body()
    return graph.replay


def event_time_us(torch, fn, reps):
    """Average microseconds of one fn() on the current stream, from HIP events around reps calls."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the decode hot path of one attention layer); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2412_14468_amd as ha
    from paper_2412_14468_amd import runner
    import workloads as W

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    ha.load()
    cfg, ring_default = workload_config(args.workload)
    ring = args.ring or ring_default
    B, Hq, Hkv, d, N = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.context
    host_layer0 = args.workload == "C1" and not args.no_cpu_baseline      # numpy layer 0 feeds the oracle too

    t_setup = time.perf_counter()
    layers = []
    L0 = None
    if host_layer0:
        L0 = W.make_layer(cfg)
        s0 = device_layer_from_host(L0, torch, ha)
        s0.lens_host, s0.k_host = L0.seq_lens.copy(), L0.k_per_seq.copy()
        layers.append(s0)
    while len(layers) < ring:
        layers.append(device_layer_synthetic(cfg, W.BASE_SEED + 1000 * cfg.index + len(layers), torch))
    n_cap = max(int(s.k.shape[2]) if s.page_table is None else int(s.page_table.shape[1]) * cfg.page_size for s in layers)
    k_max = max(s.k_max for s in layers)
    ctx = ha.Context(Hq, Hkv, B, n_cap, k_max + args.sink + args.local, page_size=cfg.page_size)
    for s in layers:
        if args.sink or args.local:
            s.set_window(args.sink, args.local)
        runner.build_key_codes(ctx, s)
        s.lens0_dev = s.seq_lens.clone()
        s.max_len0 = s.cache.max_seq_len
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup
    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").random_(0, 255)
        torch.empty_like(src).copy_(src)
        torch.cuda.synchronize()
        del src

    def one_step(s):
        if cfg.append:                       # every step appends to a cache that holds N - 1 tokens (the copy is timed too)
            s.seq_lens.copy_(s.lens0_dev)
            s.cache.max_seq_len = s.max_len0
        runner.decode_step(ctx, s, append=cfg.append)

    def sweep(n_steps, start=0):
        for i in range(n_steps):
            one_step(layers[(start + i) % ring])

    # ---- whole-step timing: W warm-up steps, then exactly K timed steps
    K, Wm = args.steps, args.warmup
    if args.no_graph:
        sweep(Wm)
        seconds = time_region(torch, lambda: sweep(K), 1)
        launch = "eager launches"
    else:
        full = capture(torch, lambda: sweep(ring))
        rem_k = capture(torch, lambda: sweep(K % ring)) if K % ring else None
        for _ in range(max(1, (Wm + ring - 1) // ring)):
            full()

        def timed():
            for _ in range(K // ring):
                full()
            if rem_k:
                rem_k()
        seconds = time_region(torch, timed, 1)
        launch = f"HIP graph of {ring} layer-steps"
    us_per_step = seconds * 1e6 / K
    lens_final = [int(n) + (1 if cfg.append else 0) for n in layers[0].lens_host]
    ks = [int(x) for x in layers[0].k_host]
    if args.sink or args.local:          # tokens attended per head: always-kept ones plus the retrieved budget
        def attended(n, kk):
            lo = min(args.sink, n)
            hi = max(lo, n - args.local)
            return lo + min(kk, hi - lo) + (n - hi)
        ks = [attended(n, kk) for n, kk in zip(lens_final, ks)]
    alg_bytes = W.algorithmic_bytes(Hkv, Hq, d, lens_final, ks)
    gbs = alg_bytes / (us_per_step * 1e-6) / 1e9
    k = k_max

    # ---- dominant kernel (GATHER-ATT) by HIP events on its own graph of `ring` launches
    def gather_sweep():
        for s in layers:
            runner.gather_attend(ctx, s)
    gather_bytes = W.gathered_bytes(Hq, d, lens_final, ks)
    if args.no_graph:
        gather_us = event_time_us(torch, gather_sweep, 10) / ring
    else:
        g_replay = capture(torch, gather_sweep)
        g_replay()
        gather_us = event_time_us(torch, g_replay, 10) / ring
    gather_gbs = gather_bytes / (gather_us * 1e-6) / 1e9

    def stage_us(body):
        if args.no_graph:
            return event_time_us(torch, body, 10) / ring
        rp = capture(torch, body)
        rp()
        return event_time_us(torch, rp, 10) / ring

    def topk_sweep():
        for s in layers:
            runner.score_topk(ctx, s)

    def encq_sweep():
        for s in layers:
            ctx.hashattn_encode_query(s.phi_q, s.q, s.B, s.q_codes)
    topk_us, encq_us = stage_us(topk_sweep), stage_us(encq_sweep)

    # ---- prefill side: rebuilding the whole key-code store of one layer (not part of the decode step)
    def rebuild():
        runner.build_key_codes(ctx, layers[0])
    rebuild()
    enc_us = event_time_us(torch, rebuild, 3)
    n_vec = sum(int(n) for n in layers[0].lens_host) * Hkv
    dims = cfg.mlp_dims
    mlp_flop = 2 * sum(a * b for a, b in zip(dims[:-1], dims[1:]))
    key_encode = {"us": round(enc_us, 1), "Mvectors_per_s": round(n_vec / enc_us, 1),
                  "algorithmic_TFLOPs": round(n_vec * mlp_flop / (enc_us * 1e-6) / 1e12, 1),
                  "key_read_GBps": round(n_vec * d * 2 / (enc_us * 1e-6) / 1e9, 1),
                  "note": "fp32-equivalent flops of the mapping; run as 2-3 bf16 MFMA passes per layer"}

    # ---- SCORE + TOPK alone for signatures of 32..512 bits (the paper's SCORE latency table lists 64..512)
    score_table = None
    if args.score_table:
        score_table = {}
        gen = torch.Generator(device="cuda:0")
        gen.manual_seed(W.BASE_SEED + 512)
        s0 = layers[0]
        for bits in (32, 64, 128, 256, 512):
            words = bits // 32
            wctx = ctx if bits == 32 else ha.Context(Hq, Hkv, B, n_cap, k_max, page_size=cfg.page_size, bits=bits)
            n_ring = max(2, min(ring, (1 << 30) // max(1, s0.codes.numel() * 4 * words)))
            shape = tuple(s0.codes.shape) + ((words,) if words > 1 else ())
            rings = [(torch.randint(-2 ** 31, 2 ** 31 - 1, shape, dtype=torch.int32, device="cuda:0", generator=gen),
                      torch.randint(-2 ** 31, 2 ** 31 - 1, (B, Hq) + ((words,) if words > 1 else ()), dtype=torch.int32,
                                    device="cuda:0", generator=gen)) for _ in range(n_ring)]
            caches = [ha.KvCache(s0.k, s0.v, cds, s0.seq_lens, s0.cache.max_seq_len, page_table=s0.page_table) for cds, _ in rings]

            def wide_sweep():
                for cache_w, (_, qcw) in zip(caches, rings):
                    wctx.hashattn_score_topk(qcw, cache_w, B, s0.k_per_seq, s0.k_max, s0.idx, s0.count, s0.threshold)
            rp = capture(torch, wide_sweep) if not args.no_graph else wide_sweep
            rp()
            us = event_time_us(torch, rp, 10) / n_ring
            code_bytes = sum(int(n) for n in s0.lens_host) * Hkv * 4 * words
            score_table[str(bits)] = {"us": round(us, 2), "code_GBps": round(code_bytes / (us * 1e-6) / 1e9, 1)}
            del rings, caches

    # ---- in-house dense decode on the same ring
    dense = None
    if not args.no_dense:
        def dense_sweep():
            for s in layers:
                runner.dense_step(ctx, s)
        dense_us = stage_us(dense_sweep)
        dense_bytes = sum(2 * Hkv * n * d * 2 + 2 * Hq * d * 2 for n in lens_final)
        dense = {"us_per_layer": round(dense_us, 3), "GBps": round(dense_bytes / (dense_us * 1e-6) / 1e9, 1),
                 "speedup_sparse_vs_dense": round(dense_us / us_per_step, 3)}

    # ---- CPU oracle on the host cores, same arrays as ring layer 0
    cpu = None
    parity = None
    if host_layer0:
        import oracle
        ok, ov = L0.k.copy(), L0.v.copy()
        codes = np.zeros(ok.shape[:3], dtype=np.uint32)
        ocache = oracle.Cache(ok, ov, codes, L0.seq_lens.copy())
        phi_q, phi_kv = oracle.Mlp(L0.w_q), oracle.Mlp(L0.w_kv)
        oracle.encode_keys(phi_kv, ocache, None, None, N)            # prefill-side, not timed
        scale = 1.0 / math.sqrt(d)
        times, res = [], None
        t_all = time.perf_counter()
        while len(times) < 3 or (time.perf_counter() - t_all < 10.0 and len(times) < 40):
            t0 = time.perf_counter()
            res = oracle.decode_step(phi_q, phi_kv, ocache, L0.q, L0.k_per_seq, scale, n_sink=args.sink, n_local=args.local)
            times.append(time.perf_counter() - t0)
        cpu_s = float(np.median(times))
        cores = oracle.num_threads()
        oracle.set_threads(1)                                        # the same step on one host thread, for reference
        one = []
        for _ in range(3):
            t0 = time.perf_counter()
            oracle.decode_step(phi_q, phi_kv, ocache, L0.q, L0.k_per_seq, scale, n_sink=args.sink, n_local=args.local)
            one.append(time.perf_counter() - t0)
        oracle.set_threads(cores)
        cpu = {"value": round(alg_bytes / cpu_s / 1e9, 4), "unit": "GB/s", "us_per_layer_step": round(cpu_s * 1e6, 1),
               "cores": cores, "kind": "oracle",
               "sample": f"whole {cfg.name} layer-step (all {B * Hq} (sequence, head) pairs), median of {len(times)} runs",
               "one_thread_us_per_layer_step": round(float(np.median(one)) * 1e6, 1)}
        # parity of ring layer 0 against the oracle, staged as in tests/: the GPU's own codes are compared
        # bit by bit (they may differ where the pre-sign activation is within rounding of 0), then SCORE +
        # TOPK + GATHER-ATT run on the oracle's codes, where index sets must be identical
        s0 = layers[0]
        runner.build_key_codes(ctx, s0)
        ctx.hashattn_encode_query(s0.phi_q, s0.q, s0.B, s0.q_codes)
        torch.cuda.synchronize()
        gpu_codes = s0.codes.cpu().numpy().view(np.uint32)
        diff_bits = int(sum(bin(int(x)).count("1") for x in (gpu_codes ^ codes)[gpu_codes != codes]))
        q_same = bool(np.array_equal(s0.q_codes.cpu().numpy().view(np.uint32), res["q_codes"]))
        s0.codes.copy_(torch.from_numpy(codes.view(np.int32)).to("cuda:0"))
        s0.q_codes.copy_(torch.from_numpy(res["q_codes"].view(np.int32)).to("cuda:0"))
        runner.score_topk(ctx, s0)
        runner.gather_attend(ctx, s0)
        torch.cuda.synchronize()
        got = s0.out.float().cpu().numpy().astype(np.float64)
        n_att = int(res["count"].max())
        same_sets = bool(np.array_equal(s0.count.cpu().numpy(), res["count"]) and
                         np.array_equal(s0.idx.cpu().numpy()[:, :, :n_att], res["idx"][:, :, :n_att]))
        err = np.abs(got - res["out"])
        parity = {"key_code_bits_differing": diff_bits, "key_code_bits_total": int(codes.size) * 32,
                  "query_codes_equal": q_same, "index_sets_equal_on_oracle_codes": same_sets,
                  "out_within_tol": bool(np.all(err <= 2e-3 + 1e-2 * np.abs(res["out"]))) if same_sets else None,
                  "max_abs_err": float(err.max()) if same_sets else None}

    line = {
        "metric": METRIC, "value": round(gbs, 2), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(us_per_step * 1e-3, 6), "us_per_layer_step": round(us_per_step, 3),
        "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: Llama-3.1-8B-shaped decode layer, B={B}, N={describe_lengths(lens_final)}, "
                               f"k={describe_lengths(ks)} ({round(sum(lens_final) / max(sum(ks), 1))}x sparsity), "
                               f"{Hq} q heads / {Hkv} KV heads, d={d}, mapping MLPs {'-'.join(map(str, cfg.mlp_dims))} fp32"
                               + (", paged KV (16 tokens/page)" if cfg.page_size else "")
                               + (", one-token append per step" if cfg.append else "")
                               + (f", first {args.sink} and last {args.local} tokens always kept (k counts them here)"
                                  if args.sink or args.local else ""),
                   "batch": B, "context": max(lens_final), "k": k, "ring_layers": ring, "launch": launch,
                   "algorithmic_bytes_per_step": alg_bytes},
        "roofline": {"bound": "hbm", "kernel": "hashattn_gather_attend = gather_attend_kernel + merge_partials_kernel",
                     "achieved": round(gather_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gather_gbs / HBM_PEAK_GBS, 4), "traffic": stored_traffic(args.workload),
                     "us_per_launch": round(gather_us, 3), "algorithmic_bytes_per_launch": gather_bytes},
        "cpu_baseline": cpu,
        "stages_us": {"encode_query": round(encq_us, 3), "score_topk": round(topk_us, 3),
                      "gather_attend": round(gather_us, 3)},
        "dense_baseline": dense, "key_encode_bulk": key_encode, "score_topk_by_bits": score_table, "parity_layer0": parity, "setup_s": round(t_setup, 1),
    }
    print(json.dumps(line, ensure_ascii=False))


if __name__ == "__main__":
    main()
