#!/usr/bin/env python3
"""Benchmark of the HashAttention decode layer-step on one MI355X.

A step is one pass of the whole hot path over one layer: [one-token append ->] encode query ->
SCORE + TOPK -> GATHER-ATT.  Steps walk a ring of distinct layers (own K/V, codes and mapping
weights) whose codes and weights alone exceed the 256 MB Infinity Cache, so a step reads everything
from HBM, as a decode that streams the model's weights between two visits of a layer does.  A whole
sweep over the ring is captured in one HIP graph and replayed, which removes the host's launch cost
from the step as a serving loop would.

The headline workload is the largest single-GPU configuration (C2: 16 sequences of 131072 tokens,
k = 4096, with the one-token append).  Prints ONE JSON line for it: whole-step effective GB/s
(algorithmic bytes = key codes + gathered K/V rows + Q/O), the roofline record of the dominant kernel
(GATHER-ATT), the speed-up over the in-house dense decode kernel on the same buffers, the CPU oracle
timed on a stated sample of the same layer, a parity check of that sample, and (key "other_workloads")
the step times of the other configurations measured in the same process.
"""
from __future__ import annotations

import argparse
import gc
import glob
import hashlib
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
DEV = "cuda:0"

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
HEADLINE = "C2"
OTHERS_DEFAULT = "C1,C1-128K,C3,C4"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=640)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", default=HEADLINE, choices=list(WORKLOADS),
                    help="C2 = Llama-3.1-8B layer, B=16, N=131072, k=4096, one-token append (the headline: the "
                         "largest single-GPU configuration)")
    ap.add_argument("--also", default=None,
                    help="comma-separated workloads whose step time is added under 'other_workloads' "
                         f"(default '{OTHERS_DEFAULT}' when the headline workload runs, none otherwise; '' = none)")
    ap.add_argument("--ring", type=int, default=0, help="distinct layers walked by the steps (0 = per workload)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--score-table", action="store_true",
                    help="also time SCORE + TOPK alone on uniform random codes of 32..512 bits at this workload's shape")
    ap.add_argument("--sink", type=int, default=0, help="always keep this many first tokens (k counts the rest)")
    ap.add_argument("--local", type=int, default=0, help="always keep this many most recent tokens")
    ap.add_argument("--planted", type=int, default=-1,
                    help="planted pivotal tokens per query head (default: the workload's 64); 0 skips them, which leaves "
                         "every byte count unchanged and is used for counter runs under rocprofv3, to keep set-up short")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for scaling rocprofv3 byte counters)")
    return ap.parse_args()


def workload_config(name):
    import workloads as W
    make, ring = WORKLOADS[name]
    return make(W), ring


def device_layer_synthetic(cfg, seed, lens_view=None):
    """One ring layer drawn on the device by the recipe of workloads.device_tensors.  lens_view: where the
    layer's sequence lengths live (a row of one tensor for the whole ring), if given."""
    import workloads as W
    from paper_2412_14468_amd.runner import layer_from_tensors
    t = W.device_tensors(cfg, seed)
    if lens_view is not None:
        lens_view.copy_(t["seq_lens"])
        t["seq_lens"] = lens_view
    s = layer_from_tensors(t)
    s.lens_host, s.k_host = t["seq_lens_host"], t["k_per_seq_host"]
    return s


def describe_lengths(v):
    return str(v[0]) if min(v) == max(v) else f"{min(v)}..{max(v)} (sum {sum(v)})"


def source_id():
    """Identity of the kernel sources a profile was taken with (first 16 hex digits of their SHA-256)."""
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(ROOT, "paper_2412_14468_amd", "csrc", "*")))
    for path in files + [os.path.join(ROOT, "include", "hashattn.h")]:
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def stored_profile(workload):
    """What the committed rocprofv3 summaries hold for this workload (profiles/kernel_profiles.json):
    average duration of the dominant kernel alone and HBM bytes per launch from the --pmc runs.  Counters
    cannot be read from inside this process, so these are stored figures; `current` says whether the
    kernel sources are still the ones they were measured with."""
    path = os.path.join(ROOT, "profiles", "kernel_profiles.json")
    try:
        with open(path) as f:
            rec = json.load(f).get(workload)
    except (OSError, ValueError):
        return None
    if rec:
        rec = dict(rec)
        rec["current"] = rec.get("source_id") == source_id()
    return rec


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


# ------------------------------------------------------------------ host copies of sampled sequences
def bits_of(torch, t):
    """bf16 / int32 device tensor -> numpy bit patterns."""
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy().view(np.uint32)


def sequence_rows(torch, s, tensor, b, n, page_size):
    """Rows of the first n tokens of sequence b, all KV heads, in token order: [H_kv][n][...]."""
    if s.page_table is None:
        return tensor[b, :, :n]
    t = torch.arange(n, device=DEV)
    return tensor[s.page_table[b, t // page_size].long(), :, t % page_size].transpose(0, 1)


def put_sequence_codes(torch, s, b, codes_host, page_size):
    """codes_host [H_kv][n] uint32 -> the code store of sequence b."""
    n = codes_host.shape[1]
    src = torch.from_numpy(np.ascontiguousarray(codes_host).view(np.int32)).to(DEV)
    if s.page_table is None:
        s.codes[b, :, :n] = src
    else:
        t = torch.arange(n, device=DEV)
        s.codes[s.page_table[b, t // page_size].long(), :, t % page_size] = src.transpose(0, 1)


def oracle_leg(torch, ha, runner, W, ctx, cfg, s0, args, alg_bytes_all, budget_s=12.0):
    """CPU oracle on a bounded sample of ring layer 0 (its first sequences, every head), timed on the
    host cores, and the parity of the HIP path with it on that sample.

    The sampled sequences' K/V rows, queries and mapping weights are copied back from the device
    tensors the timed steps ran on; the oracle builds its own key codes from them (untimed: prefill
    side) and runs whole layer-steps.  Parity is staged as in tests/: the GPU's own codes are
    compared bit by bit (they may differ where the pre-sign activation is within rounding of 0), then
    SCORE + TOPK + GATHER-ATT run on the oracle's codes, where index sets must be identical."""
    import oracle
    B, Hq, Hkv, d, ps = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.page_size
    nb = min(B, 2)
    seqs = list(range(nb))
    lens0 = np.array([int(s0.lens_host[b]) for b in seqs], dtype=np.int32)
    step_new = 1 if cfg.append else 0
    cap = int(lens0.max()) + step_new
    cap += (-cap) % 4
    k_host = np.zeros((nb, Hkv, cap, d), dtype=np.uint16)
    v_host = np.zeros_like(k_host)
    for i, b in enumerate(seqs):
        n0 = int(lens0[i])
        k_host[i, :, :n0] = bits_of(torch, sequence_rows(torch, s0, s0.k, b, n0, ps))
        v_host[i, :, :n0] = bits_of(torch, sequence_rows(torch, s0, s0.v, b, n0, ps))
    codes = np.zeros((nb, Hkv, cap), dtype=np.uint32)
    olens = lens0.copy()
    ocache = oracle.Cache(k_host, v_host, codes, olens)
    phi_q = oracle.Mlp([w.cpu().numpy() for w in s0.phi_q.weights])
    phi_kv = oracle.Mlp([w.cpu().numpy() for w in s0.phi_kv.weights])
    q_host = bits_of(torch, s0.q[:nb])
    kps = np.array([int(s0.k_host[b]) for b in seqs], dtype=np.int32)
    kw = {}
    if cfg.append:
        kw = dict(k_new=bits_of(torch, s0.k_new[:nb, :, 0]), v_new=bits_of(torch, s0.v_new[:nb, :, 0]))
    t0 = time.perf_counter()
    oracle.encode_keys(phi_kv, ocache, None, None, max(int(lens0.max()), 1))          # prefill side, not timed
    prefill_s = time.perf_counter() - t0
    scale = 1.0 / math.sqrt(d)

    def step():
        olens[:] = lens0                     # an append step starts from the same cache state every time
        return oracle.decode_step(phi_q, phi_kv, ocache, q_host, kps, scale, n_sink=args.sink, n_local=args.local, **kw)

    times, res = [], None
    t_all = time.perf_counter()
    while len(times) < 3 or (time.perf_counter() - t_all < budget_s and len(times) < 40):
        t0 = time.perf_counter()
        res = step()
        times.append(time.perf_counter() - t0)
    cpu_s = float(np.median(times))
    threads = oracle.num_threads()
    cores = min(threads, nb * Hq)            # the step runs one (sequence, head) pair per thread
    one_s = None
    if cpu_s * min(threads, nb * Hq) < 6.0:  # the same step on one host thread, for reference, when it is short
        oracle.set_threads(1)
        t0 = time.perf_counter()
        step()
        one_s = time.perf_counter() - t0
        oracle.set_threads(threads)
    lens1 = [int(n) + step_new for n in lens0]

    def attended(n, kk):
        lo = min(args.sink, n)
        hi = max(lo, n - args.local)
        return lo + min(kk, hi - lo) + (n - hi)
    sample_bytes = W.algorithmic_bytes(Hkv, Hq, d, lens1, [attended(n, int(kk)) for n, kk in zip(lens1, kps)])
    whole_s = cpu_s * alg_bytes_all / sample_bytes
    cpu = {"value": round(sample_bytes / cpu_s / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
           "sample": (f"sequence{'s' if nb > 1 else ''} {', '.join(map(str, seqs))} of {B} of ring layer 0, all {Hq} query heads "
                      f"each ({nb * Hq} (sequence, head) pairs, {sample_bytes} algorithmic bytes), whole layer-step"
                      f"{' incl. the append' if cfg.append else ''}, median of {len(times)} runs of {round(cpu_s * 1e3, 1)} ms; "
                      f"rows copied back from the device tensors of the timed steps"),
           "us_per_layer_step_sample": round(cpu_s * 1e6, 1),
           "us_per_layer_step_scaled_to_workload": round(whole_s * 1e6, 1),
           "one_thread_us_per_layer_step_sample": None if one_s is None else round(one_s * 1e6, 1),
           "oracle_prefill_encode_s": round(prefill_s, 2)}

    # ---- parity of the sample: GPU codes first, then the rest of the step on the oracle's codes
    s0.seq_lens.copy_(s0.lens0_dev)
    s0.cache.max_seq_len = s0.max_len0
    runner.build_key_codes(ctx, s0)
    if cfg.append:
        ctx.hashattn_encode_keys(s0.phi_kv, s0.k_new, s0.v_new, s0.B, 1, s0.cache)
    ctx.hashattn_encode_query(s0.phi_q, s0.q, s0.B, s0.q_codes)
    torch.cuda.synchronize()
    diff_bits = total_bits = 0
    for i, b in enumerate(seqs):
        n1 = lens1[i]
        gpu_codes = bits_of(torch, sequence_rows(torch, s0, s0.codes, b, n1, ps))
        x = gpu_codes ^ codes[i, :, :n1]
        diff_bits += int(np.unpackbits(x[x != 0].view(np.uint8)).sum())
        total_bits += int(x.size) * 32
        put_sequence_codes(torch, s0, b, codes[i, :, :n1], ps)
    q_same = bool(np.array_equal(bits_of(torch, s0.q_codes[:nb]), res["q_codes"]))
    s0.q_codes[:nb] = torch.from_numpy(res["q_codes"].view(np.int32)).to(DEV)
    runner.score_topk(ctx, s0)
    runner.gather_attend(ctx, s0)
    torch.cuda.synchronize()
    got = s0.out[:nb].float().cpu().numpy().astype(np.float64)
    cnt_gpu, idx_gpu = s0.count[:nb].cpu().numpy(), s0.idx[:nb].cpu().numpy()
    same_sets = bool(np.array_equal(cnt_gpu, res["count"]))
    if same_sets:
        for i in range(nb):
            for h in range(Hq):
                c = int(res["count"][i, h])
                same_sets = same_sets and bool(np.array_equal(idx_gpu[i, h, :c], res["idx"][i, h, :c]))
    err = np.abs(got - res["out"])
    ref16 = W.bf16_bits_to_f32(W.f32_to_bf16_bits(res["out"].astype(np.float32))).astype(np.float64)
    parity = {"sample": f"sequences {seqs} of ring layer 0, all heads", "key_code_bits_differing": diff_bits,
              "key_code_bits_total": total_bits, "query_codes_equal": q_same,
              "index_sets_equal_on_oracle_codes": same_sets,
              "out_within_tol": bool(np.all(err <= 2e-3 + 1e-2 * np.abs(res["out"]))) if same_sets else None,
              "max_abs_err": float(err.max()) if same_sets else None,
              "max_abs_err_vs_oracle_rounded_to_bf16": float(np.abs(got - ref16).max()) if same_sets else None}
    return cpu, parity


# ------------------------------------------------------------------ one workload
def run_workload(name, args, headline):
    import torch
    import paper_2412_14468_amd as ha
    from paper_2412_14468_amd import runner
    import workloads as W

    cfg, ring_default = workload_config(name)
    if args.planted >= 0:
        cfg = W.scaled(cfg, planted=args.planted)
    ring = (args.ring if headline else 0) or ring_default
    B, Hq, Hkv, d = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim

    t_setup = time.perf_counter()
    # the sequence lengths of all ring layers sit in one tensor, so that an append workload puts them back
    # to "N - 1 tokens cached" with one small copy per sweep over the ring
    lens_all = torch.zeros((ring, B), dtype=torch.int32, device=DEV)
    layers = [device_layer_synthetic(cfg, W.BASE_SEED + 1000 * cfg.index + i, lens_all[i]) for i in range(ring)]
    n_cap = max(int(s.k.shape[2]) if s.page_table is None else int(s.page_table.shape[1]) * cfg.page_size for s in layers)
    k_max = max(s.k_max for s in layers)
    ctx = ha.Context(Hq, Hkv, B, n_cap, k_max + args.sink + args.local, page_size=cfg.page_size)
    for s in layers:
        if args.sink or args.local:
            s.set_window(args.sink, args.local)
        runner.build_key_codes(ctx, s)
        s.lens0_dev = s.seq_lens.clone()
        s.max_len0 = s.cache.max_seq_len
    lens0_all = lens_all.clone()
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup
    if headline and args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=DEV).random_(0, 255)
        torch.empty_like(src).copy_(src)
        torch.cuda.synchronize()
        del src

    def one_step(s):
        if cfg.append:                       # every step appends to a cache that holds N - 1 tokens
            s.cache.max_seq_len = s.max_len0
        runner.decode_step(ctx, s, append=cfg.append)

    def sweep(n_steps, start=0):
        for i in range(n_steps):
            if cfg.append and (i == 0 or (start + i) % ring == 0):
                lens_all.copy_(lens0_all)    # one copy of ring x B lengths per sweep (timed with the steps)
            one_step(layers[(start + i) % ring])

    # ---- whole-step timing: W warm-up steps, then exactly K timed steps
    K, Wm = args.steps, args.warmup
    if args.no_graph:
        sweep(Wm)
        seconds = time_region(torch, lambda: sweep(K), 1)
        launch = "eager launches"
    else:
        # the K timed steps are as few graph launches as possible (one for K <= 256): a launch costs a few
        # microseconds of idle GPU, which would count against a short run
        full = capture(torch, lambda: sweep(ring))
        chunk = min(K, max(ring, 256 // ring * ring))
        g_chunk = full if chunk == ring else capture(torch, lambda: sweep(chunk))
        g_rem = capture(torch, lambda: sweep(K % chunk)) if K % chunk else None
        for _ in range(max(1, (Wm + ring - 1) // ring)):
            full()
        # the graphs of the timed region are replayed once before it as well: the first replay of a graph
        # uploads it, which is no part of a step (so the warm-up is W steps or more, never fewer)
        if g_chunk is not full:
            g_chunk()
        if g_rem:
            g_rem()

        def timed():
            for _ in range(K // chunk):
                g_chunk()
            if g_rem:
                g_rem()
        seconds = time_region(torch, timed, 1)
        launch = f"HIP graphs of {chunk} layer-steps over a ring of {ring} layers"
    us_per_step = seconds * 1e6 / K
    # bytes per step: the mean over the ring's layers (their lengths differ in the mixed-length workload)
    step_new = 1 if cfg.append else 0

    def attended(n, kk):
        lo = min(args.sink, n)
        hi = max(lo, n - args.local)
        return lo + min(kk, hi - lo) + (n - hi)

    def layer_shape(s):
        lens = [int(n) + step_new for n in s.lens_host]
        return lens, [attended(n, int(kk)) for n, kk in zip(lens, s.k_host)]
    shapes = [layer_shape(s) for s in layers]
    lens_final, ks = shapes[0]
    alg_bytes = round(sum(W.algorithmic_bytes(Hkv, Hq, d, ln, kk) for ln, kk in shapes) / ring)
    gbs = alg_bytes / (us_per_step * 1e-6) / 1e9

    def stage_us(body):
        if args.no_graph:
            return event_time_us(torch, body, 10) / ring
        rp = capture(torch, body)
        rp()
        return event_time_us(torch, rp, 10) / ring

    # ---- the entry points one by one, by HIP events on their own graphs of `ring` launches
    def gather_sweep():
        for s in layers:
            runner.gather_attend(ctx, s)

    def topk_sweep():
        for s in layers:
            runner.score_topk(ctx, s)

    def encq_sweep():
        for s in layers:
            ctx.hashattn_encode_query(s.phi_q, s.q, s.B, s.q_codes)
    gather_bytes = round(sum(W.gathered_bytes(Hq, d, ln, kk) for ln, kk in shapes) / ring)
    code_bytes = round(sum(4 * Hkv * sum(ln) for ln, _ in shapes) / ring)
    def enc_topk_sweep():           # the combined entry point the whole step calls
        for s in layers:
            ctx.hashattn_encode_score_topk(s.phi_q, s.q, s.cache, s.B, s.k_per_seq, s.k_max, s.n_sink, s.n_local,
                                           s.q_codes, s.idx, s.count, s.threshold)
    gather_us, topk_us, encq_us = stage_us(gather_sweep), stage_us(topk_sweep), stage_us(encq_sweep)
    enc_topk_us = stage_us(enc_topk_sweep)
    gather_gbs = gather_bytes / (gather_us * 1e-6) / 1e9

    dense = None
    if not args.no_dense:
        def dense_sweep():
            for s in layers:
                runner.dense_step(ctx, s)
        dense_us = stage_us(dense_sweep)
        dense_bytes = sum(sum(2 * Hkv * n * d * 2 + 2 * Hq * d * 2 for n in ln) for ln, _ in shapes) / ring
        dense = {"us_per_layer": round(dense_us, 3), "GBps": round(dense_bytes / (dense_us * 1e-6) / 1e9, 1),
                 "speedup_sparse_vs_dense": round(dense_us / us_per_step, 3)}

    rec = {"name": cfg.name, "cfg": cfg, "ring": ring, "launch": launch, "us_per_step": us_per_step, "gbs": gbs,
           "alg_bytes": alg_bytes, "lens_final": lens_final, "ks": ks, "k_max": k_max, "gather_us": gather_us,
           "gather_bytes": gather_bytes, "gather_gbs": gather_gbs, "topk_us": topk_us, "encq_us": encq_us, "enc_topk_us": enc_topk_us,
           "code_bytes": code_bytes, "dense": dense, "setup_s": t_setup}
    if not headline:
        del layers, ctx
        gc.collect()
        torch.cuda.empty_cache()
        return rec

    # ---- prefill side: rebuilding the whole key-code store of one layer (not part of the decode step)
    def rebuild():
        runner.build_key_codes(ctx, layers[0])
    rebuild()
    enc_us = event_time_us(torch, rebuild, 3)
    n_vec = sum(int(n) for n in layers[0].lens_host) * Hkv       # the rebuild is timed on ring layer 0 alone
    dims = cfg.mlp_dims
    mlp_flop = 2 * sum(a * b for a, b in zip(dims[:-1], dims[1:]))
    rec["key_encode"] = {"us": round(enc_us, 1), "Mvectors_per_s": round(n_vec / enc_us, 1),
                         "algorithmic_TFLOPs": round(n_vec * mlp_flop / (enc_us * 1e-6) / 1e12, 1),
                         "key_read_GBps": round(n_vec * d * 2 / (enc_us * 1e-6) / 1e9, 1),
                         "note": "fp32-equivalent flops of the mapping; run as 2-3 bf16 MFMA passes per layer"}

    # ---- SCORE + TOPK alone for signatures of 32..512 bits (the paper's SCORE latency table lists 64..512)
    rec["score_table"] = None
    if args.score_table:
        score_table = {}
        gen = torch.Generator(device=DEV)
        gen.manual_seed(W.BASE_SEED + 512)
        s0 = layers[0]
        for bits in (32, 64, 128, 256, 512):
            words = bits // 32
            wctx = ctx if bits == 32 else ha.Context(Hq, Hkv, B, n_cap, k_max, page_size=cfg.page_size, bits=bits)
            n_ring = max(2, min(ring, (1 << 30) // max(1, s0.codes.numel() * 4 * words)))
            shape = tuple(s0.codes.shape) + ((words,) if words > 1 else ())
            rings = [(torch.randint(-2 ** 31, 2 ** 31 - 1, shape, dtype=torch.int32, device=DEV, generator=gen),
                      torch.randint(-2 ** 31, 2 ** 31 - 1, (B, Hq) + ((words,) if words > 1 else ()), dtype=torch.int32,
                                    device=DEV, generator=gen)) for _ in range(n_ring)]
            caches = [ha.KvCache(s0.k, s0.v, cds, s0.seq_lens, s0.cache.max_seq_len, page_table=s0.page_table) for cds, _ in rings]

            def wide_sweep():
                for cache_w, (_, qcw) in zip(caches, rings):
                    wctx.hashattn_score_topk(qcw, cache_w, B, s0.k_per_seq, s0.k_max, s0.idx, s0.count, s0.threshold)
            rp = capture(torch, wide_sweep) if not args.no_graph else wide_sweep
            rp()
            us = event_time_us(torch, rp, 10) / n_ring
            cb = sum(int(n) for n in s0.lens_host) * Hkv * 4 * words
            score_table[str(bits)] = {"us": round(us, 2), "code_GBps": round(cb / (us * 1e-6) / 1e9, 1)}
            del rings, caches
        rec["score_table"] = score_table

    # ---- CPU oracle on the host cores and parity, on a sample of ring layer 0
    rec["cpu"] = rec["parity"] = None
    if not args.no_cpu_baseline:
        rec["cpu"], rec["parity"] = oracle_leg(torch, ha, runner, W, ctx, cfg, layers[0], args, alg_bytes)
    del layers, ctx
    gc.collect()
    torch.cuda.empty_cache()
    return rec


def workload_text(r, args):
    cfg = r["cfg"]
    return (f"{cfg.name}: Llama-3.1-8B-shaped decode layer, B={cfg.batch}, N={describe_lengths(r['lens_final'])}, "
            f"k={describe_lengths(r['ks'])} ({round(sum(r['lens_final']) / max(sum(r['ks']), 1))}x sparsity), "
            f"{cfg.n_q_heads} q heads / {cfg.n_kv_heads} KV heads, d={cfg.head_dim}, "
            f"mapping MLPs {'-'.join(map(str, cfg.mlp_dims))} fp32"
            + (" in ring layer 0 (every ring layer draws its own lengths; bytes per step are the mean over the ring)"
               if cfg.mixed_lengths else "")
            + (", paged KV (16 tokens/page)" if cfg.page_size else "")
            + (", one-token append per step" if cfg.append else "")
            + (f", first {args.sink} and last {args.local} tokens always kept (k counts them here)"
               if args.sink or args.local else ""))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the decode hot path of one attention layer); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2412_14468_amd as ha

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    ha.load()
    r = run_workload(args.workload, args, headline=True)
    also = args.also if args.also is not None else (OTHERS_DEFAULT if args.workload == HEADLINE else "")
    others = {}
    for name in [w for w in also.split(",") if w]:
        if name not in WORKLOADS or name == args.workload:
            continue
        o = run_workload(name, args, headline=False)
        sg_us = o["topk_us"] + o["gather_us"]
        others[name] = {"workload": workload_text(o, args), "us_per_layer_step": round(o["us_per_step"], 3),
                        "GBps": round(o["gbs"], 1), "pct_of_hbm_peak": round(100.0 * o["gbs"] / HBM_PEAK_GBS, 2),
                        "algorithmic_bytes_per_step": o["alg_bytes"], "ring_layers": o["ring"],
                        "stages_us": {"encode_query": round(o["encq_us"], 3), "score_topk": round(o["topk_us"], 3),
                                      "encode_score_topk": round(o["enc_topk_us"], 3),
                                      "gather_attend": round(o["gather_us"], 3)},
                        "score_plus_gather_pct_of_hbm_peak":
                            round(100.0 * (o["code_bytes"] + o["gather_bytes"]) / (sg_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 2),
                        "dense_baseline": o["dense"], "setup_s": round(o["setup_s"], 1)}

    cfg = r["cfg"]
    prof = stored_profile(args.workload)
    frac_kernel = traffic = None
    if prof:
        if prof.get("gather_attend_kernel_avg_us"):
            frac_kernel = round(r["gather_bytes"] / (prof["gather_attend_kernel_avg_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
        if prof.get("fetch_bytes") is not None:
            traffic = {"fetch_bytes": prof["fetch_bytes"], "write_bytes": prof.get("write_bytes"),
                       "total_bytes": prof["fetch_bytes"] + (prof.get("write_bytes") or 0),
                       "measured_with_source_id": prof.get("source_id"), "current": prof["current"],
                       "note": prof.get("traffic_note")}
    sg_us = r["topk_us"] + r["gather_us"]
    line = {
        "metric": METRIC, "value": round(r["gbs"], 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(r["us_per_step"] * 1e-3, 6), "us_per_layer_step": round(r["us_per_step"], 3),
        "pct_of_hbm_peak": round(100.0 * r["gbs"] / HBM_PEAK_GBS, 2), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": workload_text(r, args), "batch": cfg.batch, "context": max(r["lens_final"]), "k": r["k_max"],
                   "ring_layers": r["ring"], "launch": r["launch"], "algorithmic_bytes_per_step": r["alg_bytes"]},
        "roofline": {"bound": "hbm", "kernel": "gather_attend_kernel",
                     "achieved": round(r["gather_gbs"], 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(r["gather_gbs"] / HBM_PEAK_GBS, 4),
                     "frac_entry": round(r["gather_gbs"] / HBM_PEAK_GBS, 4), "frac_kernel": frac_kernel,
                     "traffic": traffic, "us_per_launch": round(r["gather_us"], 3),
                     "algorithmic_bytes_per_launch": r["gather_bytes"],
                     "note": ("achieved, frac and frac_entry: algorithmic bytes of GATHER-ATT / HIP-event time of the entry point "
                              "hashattn_gather_attend in this run (gather_attend_kernel followed by the small merge_partials_kernel); "
                              "frac_kernel: the same bytes / the rocprofv3 average of gather_attend_kernel alone from "
                              "profiles/kernel_profiles.json"
                              + ("" if not prof else (", taken with these kernel sources" if prof["current"] else
                                                      ", taken with OLDER kernel sources than this build")))},
        "cpu_baseline": r["cpu"],
        "stages_us": {"encode_query": round(r["encq_us"], 3), "score_topk": round(r["topk_us"], 3),
                      "encode_score_topk": round(r["enc_topk_us"], 3),
                      "gather_attend": round(r["gather_us"], 3)},
        "score_plus_gather_pct_of_hbm_peak":
            round(100.0 * (r["code_bytes"] + r["gather_bytes"]) / (sg_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 2),
        "dense_baseline": r["dense"], "key_encode_bulk": r["key_encode"], "score_topk_by_bits": r["score_table"],
        "parity_sample": r["parity"], "other_workloads": others or None, "kernel_source_id": source_id(),
        "setup_s": round(r["setup_s"], 1),
    }
    print(json.dumps(line, ensure_ascii=False))


if __name__ == "__main__":
    main()
