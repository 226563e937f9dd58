"""Recall of the selected index sets against the true pivotal tokens, on synthetic data (the paper's
quality proxy that needs no dataset: recall(I_n, I_true,k) of section 4, I_true,k ranked by
a_i ||v_i||_2 per the lemma of section 4.2; its figure on recall rates uses the top-32 tokens at 16x
sparsity).

The index sets come from the HIP path (encode keys and query, SCORE + TOPK through the C ABI); the
true pivotal tokens and the recall come from the CPU oracle.  Two mappings are compared on the same
keys: sign random projections shared between queries and keys (a locality-sensitive hash of the angle,
so keys planted along the query get codes close to the query's) and the workload's independent
random-init MLPs (no relation between query and key codes: recall near n / N).

Run as a script for a table:  python tests/recall_harness.py [context ...]
"""
import math
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

import oracle
import workloads as W


def measure(context: int, sparsity: int = 16, k_true: int = 32, mapping: str = "shared-projection",
            seed: int = W.BASE_SEED + 77, heads=None, n_sink: int = 0, n_local: int = 0, oracle_codes: bool = False):
    """Mean recall over query heads of one Llama-shaped layer (B = 1).  Returns (mean, per-head list).

    oracle_codes: the key and query codes are computed by the oracle and uploaded (instead of the HIP
    mapping kernels), and a third value is returned: the per-head recall of index sets computed wholly
    by the oracle from those same codes.  SCORE + TOPK are exact integer work, so the HIP path's index
    sets, and with them the recall, must then equal the oracle's exactly."""
    import torch
    import gpu_util as gu

    n_sel = max(context // sparsity, 1)
    cfg = W.scaled(W.c1(context=context, k=n_sel), name="recall")
    L = W.make_layer(cfg, seed)
    if mapping == "shared-projection":
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence(seed + 1)))
        L.w_q, L.w_kv = W.shared_projection_weights(rng, cfg.n_q_heads, cfg.n_kv_heads)
    elif mapping != "independent-mlp":
        raise ValueError(mapping)
    pitch = n_sel + n_sink + n_local
    D = gu.DeviceLayer(L, max_k=pitch)
    ocache, ocodes, _ = D.oracle_cache()
    if oracle_codes:
        oracle.encode_keys(oracle.Mlp(L.w_kv), ocache, None, None, context)
        oq, _ = oracle.encode_query(oracle.Mlp(L.w_q), L.q)
        D.set_codes(ocodes)
        qc = gu.u32_dev(oq)
    else:
        D.ctx.hashattn_encode_keys(D.phi_kv, None, None, D.B, context, D.cache)
        qc = torch.zeros((D.B, D.Hq), dtype=torch.int32, device=gu.DEV)
        D.ctx.hashattn_encode_query(D.phi_q, D.q, D.B, qc)
    idx = torch.zeros((D.B, D.Hq, pitch), dtype=torch.int32, device=gu.DEV)
    count = torch.zeros((D.B, D.Hq), dtype=torch.int32, device=gu.DEV)
    D.ctx.hashattn_score_topk_window(qc, D.cache, D.B, None, n_sel, n_sink, n_local, idx, count, None)
    torch.cuda.synchronize()
    idx_h, count_h = idx.cpu().numpy(), count.cpu().numpy()

    scale = 1.0 / math.sqrt(cfg.head_dim)
    per_head, per_head_oracle = [], []
    for h in (heads if heads is not None else range(cfg.n_q_heads)):
        truth = oracle.true_topk(ocache, 0, h // cfg.group, L.q[0, h], context, k_true, scale)
        per_head.append(oracle.recall(idx_h[0, h, :count_h[0, h]], truth))
        if oracle_codes:
            sc = oracle.scores(int(oq[0, h]), ocodes[0, h // cfg.group, :context])
            chosen, _, _ = oracle.topk_window(sc, n_sel, n_sink, n_local)
            per_head_oracle.append(oracle.recall(chosen, truth))
    if oracle_codes:
        return float(np.mean(per_head)), per_head, per_head_oracle
    return float(np.mean(per_head)), per_head


def main(argv):
    contexts = [int(a) for a in argv] or [4096, 16384, 65536]
    print("context  sparsity  mapping             recall(top-32)   chance n/N")
    for n in contexts:
        for sp in (16, 32):
            for m in ("shared-projection", "independent-mlp"):
                r, _ = measure(n, sp, 32, m)
                print(f"{n:7d}  {sp:7d}x  {m:18s}  {r:14.3f}   {1.0 / sp:10.3f}", flush=True)


if __name__ == "__main__":
    main(sys.argv[1:])
