"""hashattn_gather_attend_noalloc (GATHER-ATT with its split partials in the library's static device
array, for callers that cannot allocate) against hashattn_gather_attend on the same inputs, and both
against the oracle: two calls in a row, the second on a smaller input, so that whatever the first call
left in the shared array must not leak into the second."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W

pytestmark = pytest.mark.gpu


def one_case(cfg, seed, lens=None, ks=None):
    import gpu_util as gu
    import paper_2412_14468_amd as ha
    L = W.make_layer(cfg, seed=seed)
    if lens is not None:
        L.seq_lens[:] = lens
    if ks is not None:
        L.k_per_seq[:] = ks
    D = gu.DeviceLayer(L)
    g = D.Hq // D.Hkv
    ocache, codes, lens_h = D.oracle_cache()
    oracle.encode_keys(oracle.Mlp(L.w_kv), ocache, None, None, max(int(L.seq_lens.max()), 1))
    qc, _ = oracle.encode_query(oracle.Mlp(L.w_q), L.q)
    D.set_codes(codes)
    idx, count, thr, out_ctx = D.new_outputs()
    D.ctx.hashattn_score_topk(gu.u32_dev(qc), D.cache, D.B, D.k_per_seq, D.k_max, idx, count, thr)
    D.ctx.hashattn_gather_attend(D.q, D.cache, idx, count, D.B, D.k_max, D.scale, out_ctx)
    out_static = torch.full_like(out_ctx, float("nan"))
    ha.hashattn_gather_attend_noalloc(D.Hq, D.Hkv, cfg.page_size, D.q, D.cache, idx, count, D.B, D.k_max, D.scale, out_static)
    torch.cuda.synchronize()
    idx_h, count_h = idx.cpu().numpy(), count.cpu().numpy()
    ref = np.zeros((D.B, D.Hq, D.d))
    for b in range(D.B):
        for h in range(D.Hq):
            c = int(count_h[b, h])
            if c:
                ref[b, h] = oracle.gather_attend(ocache, b, h // g, L.q[b, h], idx_h[b, h, :c], D.scale)
    gu.assert_out_close(out_ctx, ref, "gather_attend")
    gu.assert_out_close(out_static, ref, "gather_attend_noalloc")
    # same kernels; only the number of splits may differ (it follows the scratch size), so the two
    # agree to within the rounding of a different summation order
    a, b_ = gu.bf16_host_f64(out_static), gu.bf16_host_f64(out_ctx)
    assert np.all(np.abs(a - b_) <= 2.0 ** -7 * np.abs(b_) + 5e-5)
    return out_static


def test_noalloc_matches_gather_attend_on_two_calls_in_a_row():
    big = W.scaled(W.c1(), context=40000, k=2500, batch=3, planted=16)           # split path, several splits per head
    one_case(big, seed=91, lens=[40000, 1, 23017], ks=[2500, 2500, 700])
    small = W.scaled(W.c1(), context=3000, k=90, batch=2, planted=4)              # fewer heads, shorter lists
    one_case(small, seed=92, lens=[3000, 0], ks=[90, 90])
    paged = W.scaled(W.c4(batch=5, lo=200, hi=6000), planted=4)                   # paged layout, per-sequence k
    one_case(paged, seed=93)
    direct = W.scaled(W.c1(), context=2000, k=64, batch=6, planted=4)             # >= 128 heads, short lists: no partials
    one_case(direct, seed=94)


def test_noalloc_rejects_what_the_static_scratch_cannot_hold():
    import gpu_util as gu
    import paper_2412_14468_amd as ha
    L = W.make_layer(W.scaled(W.c0(), context=256, k=16))
    D = gu.DeviceLayer(L)
    idx, count, thr, out = D.new_outputs()
    with pytest.raises(ha.HashAttnError, match="static scratch") as e:
        ha.hashattn_gather_attend_noalloc(32, 8, 0, D.q, D.cache, idx, count, 500, 16, D.scale, out)   # 16000 pairs
    assert e.value.status == ha.SCRATCH_TOO_SMALL
    with pytest.raises(ha.HashAttnError) as e:
        ha.hashattn_gather_attend_noalloc(32, 5, 0, D.q, D.cache, idx, count, 1, 16, D.scale, out)
    assert e.value.status == ha.INVALID_ARG
    with pytest.raises(ha.HashAttnError) as e:
        ha.hashattn_gather_attend_noalloc(1, 1, 0, None, D.cache, idx, count, 1, 16, D.scale, out)
    assert e.value.status == ha.INVALID_ARG
    assert torch.all(torch.isnan(out.float()))            # nothing was enqueued
