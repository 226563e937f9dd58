"""GPU parity of hashattn_decode_step (the whole layer-step in one call: [append,] ENCODE-Q, SCORE, TOPK,
GATHER-ATT; section 4, section 4.1) against the oracle's decode step, through the C ABI.

The cached keys' codes are the oracle's (put on the device before the call).  The call's own codes (the query
codes and, with an append, the new token's key code) must equal the oracle's wherever the activation decides the
bit; for every (sequence, head) whose codes are the oracle's, ids, count and threshold must be the oracle's bit
for bit and the output within the tolerance.  Shapes cover the shared append + query launch (context or batch
beyond the one-launch SCORE + TOPK), its absence (short context; mappings of different or other shapes), no
append, the paged layout, the kept window and a budget per sequence."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
import gpu_util as gu

pytestmark = pytest.mark.gpu


def step_case(cfg, seed, lens=None, k_per_seq=None, n_sink=0, n_local=0, append=True, dims_kv=None, check_heads=None):
    import paper_2412_14468_amd as ha
    L = W.make_layer(cfg, seed=seed)
    if lens is not None:
        L.seq_lens[:] = lens
    if k_per_seq is not None:
        L.k_per_seq[:] = k_per_seq
    w_kv = L.w_kv
    if dims_kv is not None:                               # a key mapping of another shape than the query mapping
        rng = np.random.default_rng(seed + 7)
        w_kv = [(rng.uniform(-1, 1, size=(cfg.n_kv_heads, dims_kv[l], dims_kv[l + 1])) / np.sqrt(dims_kv[l])).astype(np.float32)
                for l in range(len(dims_kv) - 1)]
    k_max = int(L.k_per_seq.max())
    pitch = k_max + n_sink + n_local
    D = gu.DeviceLayer(L, max_k=pitch, extra_rows=4)
    phi_kv_dev = ha.Mlp([torch.from_numpy(w).to(gu.DEV) for w in w_kv])
    g = D.Hq // D.Hkv
    ocache, codes, lns = D.oracle_cache()
    phi_q_o, phi_kv_o = oracle.Mlp(L.w_q), oracle.Mlp(w_kv)
    oracle.encode_keys(phi_kv_o, ocache, None, None, max(int(L.seq_lens.max()), 1))
    D.set_codes(codes)                                    # cached keys: the oracle's codes
    lens0 = lns.copy()
    kw = {}
    if append:
        assert L.k_new is not None
        kw = dict(k_new=L.k_new, v_new=L.v_new)
    ref = oracle.decode_step(phi_q_o, phi_kv_o, ocache, L.q, L.k_per_seq, D.scale, n_sink=n_sink, n_local=n_local, **kw)
    _, act_q = oracle.encode_query(phi_q_o, L.q)

    idx = torch.full((D.B, D.Hq, pitch), -7, dtype=torch.int32, device=gu.DEV)
    count = torch.full((D.B, D.Hq), -7, dtype=torch.int32, device=gu.DEV)
    thr = torch.full((D.B, D.Hq), 255, dtype=torch.uint8, device=gu.DEV)
    qc = torch.zeros((D.B, D.Hq), dtype=torch.int32, device=gu.DEV)
    out = torch.full((D.B, D.Hq, D.d), float("nan"), dtype=torch.bfloat16, device=gu.DEV)
    kps = None if k_per_seq is None else D.k_per_seq
    D.ctx.hashattn_decode_step(phi_kv_dev if append else None, gu.bf16_dev(L.k_new) if append else None,
                               gu.bf16_dev(L.v_new) if append else None, D.phi_q, D.q, D.cache, D.B, kps, k_max,
                               n_sink, n_local, D.scale, qc, idx, count, thr, out)
    torch.cuda.synchronize()
    lens1 = lens0 + (1 if append else 0)
    assert D.seq_lens.cpu().tolist() == lens1.tolist() == lns.tolist()
    assert D.cache.max_seq_len == int(L.seq_lens.max()) + (1 if append else 0)
    qc_h = gu.u32_host(qc)
    gu.assert_codes_match(qc_h, ref["q_codes"], act_q, "query codes")
    gpu_codes = gu.u32_host(D.codes)
    new_ok = np.ones((D.B, D.Hkv), dtype=bool)            # the appended token's code equals the oracle's
    if append:
        for b in range(D.B):
            pos = int(lens0[b])
            for h in range(D.Hkv):
                if L.page_table is None:
                    got, want = gpu_codes[b, h, pos], codes[b, h, pos]
                else:
                    pg, sl = L.page_table[b, pos // cfg.page_size], pos % cfg.page_size
                    got, want = gpu_codes[pg, h, sl], codes[pg, h, sl]
                _, a_new = oracle.encode_vec(phi_kv_o, h, L.k_new[b, h])
                gu.assert_codes_match(np.array([got]), np.array([want]), a_new[None, :], f"appended key code b={b} h={h}")
                new_ok[b, h] = got == want
        # the appended rows themselves
        kh, vh = D.k.view(torch.int16).cpu().numpy().view(np.uint16), D.v.view(torch.int16).cpu().numpy().view(np.uint16)
        for b in range(D.B):
            pos = int(lens0[b])
            for h in range(D.Hkv):
                if L.page_table is None:
                    rk, rv = kh[b, h, pos], vh[b, h, pos]
                else:
                    pg, sl = L.page_table[b, pos // cfg.page_size], pos % cfg.page_size
                    rk, rv = kh[pg, h, sl], vh[pg, h, sl]
                np.testing.assert_array_equal(rk, L.k_new[b, h])
                np.testing.assert_array_equal(rv, L.v_new[b, h])
    idx_h, count_h, thr_h = idx.cpu().numpy(), count.cpu().numpy(), thr.cpu().numpy()
    compared = 0
    heads = check_heads if check_heads is not None else [(b, h) for b in range(D.B) for h in range(D.Hq)]
    for (b, h) in heads:
        if qc_h[b, h] != ref["q_codes"][b, h] or not new_ok[b, h // g]:
            continue
        compared += 1
        cnt = int(ref["count"][b, h])
        assert count_h[b, h] == cnt, (b, h, count_h[b, h], cnt)
        np.testing.assert_array_equal(idx_h[b, h, :cnt], ref["idx"][b, h, :cnt], err_msg=f"idx b={b} h={h}")
        assert np.all(idx_h[b, h, cnt:] == -7)
        assert thr_h[b, h] == ref["threshold"][b, h]
        gu.assert_out_close(out[b, h:h + 1], ref["out"][b, h][None], f"out b={b} h={h}")
    assert len(heads) - compared <= max(2, len(heads) // 10), f"only {compared} of {len(heads)} heads had the oracle's codes"


def test_append_and_query_share_a_launch_long_context():
    """Context beyond the one-launch SCORE + TOPK: append and ENCODE-Q in one launch, then the two-launch select."""
    cfg = W.scaled(W.c2(batch=3, context=40001), planted=8)
    step_case(cfg, seed=701, check_heads=[(b, h) for b in range(3) for h in (0, 5, 17, 31)])


@pytest.mark.parametrize("dims", [(128, 32), (128, 128, 32), (128, 128, 128, 32)])
def test_append_and_query_share_a_launch_many_sequences(dims):
    """More (sequence, head) pairs than the one-launch SCORE + TOPK takes; 1, 2 and 3 layers; ragged lengths and budgets."""
    cfg = W.scaled(W.c2(batch=17, context=1500), k=47, planted=4, mlp_dims=dims)
    lens = [1499, 0, 1, 700, 1024, 1499, 33, 1499, 256, 1499, 5, 1499, 1499, 64, 1499, 1000, 1499]
    kps = [47, 47, 47, 10, 47, 1, 47, 47, 47, 0, 47, 47, 47, 47, 47, 47, 47]
    step_case(cfg, seed=702, lens=lens, k_per_seq=kps)


def test_short_context_append_then_one_launch_select():
    cfg = W.scaled(W.c2(batch=2, context=5003), planted=8)
    step_case(cfg, seed=703, n_sink=16, n_local=32)


def test_no_append():
    step_case(W.scaled(W.c1(), context=9000, k=282, batch=2, planted=8), seed=704, append=False)
    step_case(W.scaled(W.c1(), context=40000, k=1250, batch=1, planted=8), seed=705, append=False,
              check_heads=[(0, h) for h in (0, 9, 31)])


def test_mappings_of_different_shapes_take_separate_launches():
    cfg = W.scaled(W.c2(batch=17, context=900), planted=4)
    step_case(cfg, seed=706, dims_kv=(128, 128, 128, 32))
    step_case(cfg, seed=707, dims_kv=(128, 256, 32))


@pytest.mark.parametrize("batch", [3, 20])
def test_paged_append(batch):
    cfg = W.scaled(W.c4(batch=batch, lo=40, hi=6000), planted=4, k_divisor=16, append=True)
    L = W.make_layer(cfg, seed=708 + batch)
    step_case(cfg, seed=708 + batch, k_per_seq=L.k_per_seq.copy())


def test_argument_errors():
    import paper_2412_14468_amd as ha
    cfg = W.scaled(W.c2(batch=2, context=300), k=16, planted=0)
    L = W.make_layer(cfg, seed=709)
    D = gu.DeviceLayer(L, extra_rows=4)
    idx, count, thr, out = D.new_outputs()
    qc = torch.zeros((2, 32), dtype=torch.int32, device=gu.DEV)
    kn, vn = gu.bf16_dev(L.k_new), gu.bf16_dev(L.v_new)
    with pytest.raises(ha.HashAttnError, match="both"):
        D.ctx.hashattn_decode_step(D.phi_kv, kn, None, D.phi_q, D.q, D.cache, 2, None, 16, 0, 0, D.scale, qc, idx, count, thr, out)
    with pytest.raises(ha.HashAttnError, match="NULL|mapping|phi"):
        D.ctx.hashattn_decode_step(None, kn, vn, D.phi_q, D.q, D.cache, 2, None, 16, 0, 0, D.scale, qc, idx, count, thr, out)
    assert D.seq_lens.cpu().tolist() == [299, 299]          # nothing was launched
