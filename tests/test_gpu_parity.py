"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Staged so that a sign flip of a near-zero activation cannot cascade:
  codes      bit-exact wherever |pre-sign activation| > 1e-3
  TOPK       index sets, counts and thresholds bit-exact on identical (oracle) codes
  GATHER-ATT |gpu - oracle| <= 2e-3 + 1e-2 |oracle| on identical (oracle) index sets
"""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

gu = None


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    global gu
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import gpu_util
    gu = gpu_util
    yield


def oracle_topk_all(codes, lens, q_codes, k_per_seq, g, layer):
    """Oracle SCORE + TOPK for every (b, h): lists of idx arrays and thresholds."""
    B, Hq = q_codes.shape
    out = {}
    cache = None
    for b in range(B):
        n = int(lens[b])
        for h in range(Hq):
            if layer.page_table is None:
                kc = codes[b, h // g, :n]
            else:
                ps = layer.cfg.page_size
                t = np.arange(n)
                kc = codes[layer.page_table[b, t // ps], h // g, t % ps]
            sc = oracle.scores(int(q_codes[b, h]), np.ascontiguousarray(kc))
            out[(b, h)] = oracle.topk_sort(sc, int(k_per_seq[b])) if n > 0 else (np.zeros(0, np.int32), 0)
    return out


def check_topk(D, q_codes_host, ref, k_per_seq=None):
    idx, count, thr, _ = D.new_outputs()
    qc = gu.u32_dev(q_codes_host)
    D.ctx.hashattn_score_topk(qc, D.cache, D.B, D.k_per_seq if k_per_seq is None else k_per_seq, D.k_max,
                              idx, count, thr)
    torch.cuda.synchronize()
    idx_h, count_h, thr_h = idx.cpu().numpy(), count.cpu().numpy(), thr.cpu().numpy()
    for (b, h), (want, T) in ref.items():
        assert count_h[b, h] == len(want), (b, h, count_h[b, h], len(want))
        np.testing.assert_array_equal(idx_h[b, h, :len(want)], want, err_msg=f"idx of (b={b}, h={h})")
        assert np.all(idx_h[b, h, len(want):] == -7), "slots past count must stay untouched"
        if len(want):
            assert thr_h[b, h] == T, (b, h, thr_h[b, h], T)
    return idx, count


def check_gather(D, ocache, idx_dev, count_dev, ref_topk, heads=None):
    _, _, _, out = D.new_outputs()
    D.ctx.hashattn_gather_attend(D.q, D.cache, idx_dev, count_dev, D.B, D.k_max, D.scale, out)
    torch.cuda.synchronize()
    g = D.Hq // D.Hkv
    ref = np.zeros((D.B, D.Hq, D.d))
    pairs = heads or list(ref_topk.keys())
    for (b, h) in pairs:
        ref[b, h] = oracle.gather_attend(ocache, b, h // g, D.L.q[b, h], ref_topk[(b, h)][0], D.scale)
    got = out.clone()
    if heads:
        mask = torch.zeros((D.B, D.Hq), dtype=torch.bool)
        for (b, h) in pairs:
            mask[b, h] = True
        sel = mask.to(got.device)
        gu.assert_out_close(got[sel], ref[mask.numpy()], "gather_attend")
    else:
        gu.assert_out_close(got, ref, "gather_attend")
    return out


def check_combined_entry(D, qc_ref, act_q, ref, n_sink=0, n_local=0, min_compared=0.9):
    """hashattn_encode_score_topk on the device's current key codes (the oracle's): its query codes against
    the oracle's where the activation decides the bit, and for every head whose code is the oracle's, ids,
    count and threshold against `ref` (the oracle's result for the oracle's codes)."""
    pitch = D.k_max + n_sink + n_local
    idx = torch.full((D.B, D.Hq, pitch), -7, dtype=torch.int32, device=gu.DEV)
    count = torch.full((D.B, D.Hq), -7, dtype=torch.int32, device=gu.DEV)
    thr = torch.full((D.B, D.Hq), 255, dtype=torch.uint8, device=gu.DEV)
    qc = torch.zeros((D.B, D.Hq), dtype=torch.int32, device=gu.DEV)
    D.ctx.hashattn_encode_score_topk(D.phi_q, D.q, D.cache, D.B, D.k_per_seq, D.k_max, n_sink, n_local, qc, idx, count, thr)
    torch.cuda.synchronize()
    qc_h, idx_h, count_h, thr_h = gu.u32_host(qc), idx.cpu().numpy(), count.cpu().numpy(), thr.cpu().numpy()
    flips = gu.assert_codes_match(qc_h, qc_ref, act_q, "query codes (combined entry point)")
    compared = 0
    for (b, h), (want, T) in ref.items():
        if qc_h[b, h] != qc_ref[b, h]:
            continue                                   # a bit within rounding of zero: another query code, another set
        compared += 1
        assert count_h[b, h] == len(want), (b, h, count_h[b, h], len(want))
        np.testing.assert_array_equal(idx_h[b, h, :len(want)], want, err_msg=f"combined entry: idx of (b={b}, h={h})")
        assert np.all(idx_h[b, h, len(want):] == -7)
        if len(want):
            assert thr_h[b, h] == T
    assert len(ref) - compared <= max(2, (1 - min_compared) * len(ref)), \
        f"only {compared} of {len(ref)} heads had the oracle's query code"
    return flips


# ---------------------------------------------------------------- C0: single head, random codes
def test_c0_score_topk_and_gather():
    L = W.make_layer(W.c0())
    D = gu.DeviceLayer(L)
    D.set_codes(L.k_codes)
    ocache, codes, lens = D.oracle_cache()
    codes[...] = L.k_codes
    ref = oracle_topk_all(codes, lens, L.q_codes, L.k_per_seq, 1, L)
    assert ref[(0, 0)][1] == 20
    idx, count = check_topk(D, L.q_codes, ref)
    check_gather(D, ocache, idx, count, ref)


def test_k_equals_n_is_dense_sdpa():
    L = W.make_layer(W.scaled(W.c0(), context=1000, k=1000))
    D = gu.DeviceLayer(L)
    D.set_codes(L.k_codes)
    ocache, codes, lens = D.oracle_cache()
    codes[...] = L.k_codes
    ref = oracle_topk_all(codes, lens, L.q_codes, L.k_per_seq, 1, L)
    assert ref[(0, 0)][0].tolist() == list(range(1000))
    idx, count = check_topk(D, L.q_codes, ref)
    sparse = check_gather(D, ocache, idx, count, ref)
    _, _, _, dense = D.new_outputs()
    D.ctx.hashattn_dense_attend(D.q, D.cache, D.B, D.scale, dense)
    torch.cuda.synchronize()
    want = oracle.dense_attend(ocache, 0, 0, L.q[0, 0], 1000, D.scale)
    gu.assert_out_close(dense, want[None, None], "dense_attend")
    gu.assert_out_close(sparse, want[None, None], "gather_attend with k = N")


# ---------------------------------------------------------------- mapping
@pytest.mark.parametrize("dims,batch", [((128, 128, 32), 1), ((128, 128, 128, 32), 3), ((128, 32), 9),
                                        ((128, 256, 64, 32), 2),
                                        ((128, 128, 32), 40), ((128, 128, 128, 32), 131)])   # 4 and 8 vectors per block
def test_encode_query_codes(dims, batch):
    cfg = W.scaled(W.c1(), context=64, k=4, batch=batch, planted=0, mlp_dims=dims)
    L = W.make_layer(cfg, seed=11 + batch)
    D = gu.DeviceLayer(L)
    qc = torch.zeros((D.B, D.Hq), dtype=torch.int32, device=gu.DEV)
    D.ctx.hashattn_encode_query(D.phi_q, D.q, D.B, qc)
    torch.cuda.synchronize()
    want, act = oracle.encode_query(oracle.Mlp(L.w_q), L.q)
    flips = gu.assert_codes_match(gu.u32_host(qc), want, act, "encode_query")
    assert flips <= 2 + batch // 16


def test_encode_query_with_bias():
    cfg = W.scaled(W.c1(), context=64, k=4, batch=2, planted=0)
    L = W.make_layer(cfg, seed=5)
    rng = np.random.default_rng(6)
    biases = [rng.uniform(-0.3, 0.3, size=(32, w.shape[2])).astype(np.float32) for w in L.w_q]
    D = gu.DeviceLayer(L)
    import paper_2412_14468_amd as ha
    b_dev = [torch.from_numpy(b).to(gu.DEV) for b in biases]
    phi = ha.Mlp(D.wq_dev, b_dev)
    qc = torch.zeros((D.B, D.Hq), dtype=torch.int32, device=gu.DEV)
    D.ctx.hashattn_encode_query(phi, D.q, D.B, qc)
    torch.cuda.synchronize()
    want, act = oracle.encode_query(oracle.Mlp(L.w_q, biases), L.q)
    gu.assert_codes_match(gu.u32_host(qc), want, act, "encode_query with bias")
    nobias, _ = oracle.encode_query(oracle.Mlp(L.w_q), L.q)
    assert (want != nobias).any()          # the bias matters in this case


@pytest.mark.parametrize("dims", [(128, 128, 32), (128, 128, 128, 32), (128, 256, 64, 32)])
def test_encode_keys_in_place_ragged(dims):
    cfg = W.scaled(W.c1(), context=1237, k=16, batch=2, planted=8, mlp_dims=dims)
    L = W.make_layer(cfg, seed=21)
    L.seq_lens[1] = 700
    D = gu.DeviceLayer(L)
    D.ctx.hashattn_encode_keys(D.phi_kv, None, None, D.B, 1237, D.cache)
    torch.cuda.synchronize()
    ocache, codes, lens = D.oracle_cache()
    act = oracle.encode_keys(oracle.Mlp(L.w_kv), ocache, None, None, 1237, want_act=True)
    got = gu.u32_host(D.codes)
    for b, n in enumerate(lens):
        n = int(n)
        gu.assert_codes_match(got[b, :, :n], codes[b, :, :n], act[b, :, :n], f"encode_keys b={b}")
        assert np.all(got[b, :, n:] == 0), "codes past seq_len must stay untouched"
    # partial rebuild: only the last 100 tokens
    D.codes.zero_()
    D.ctx.hashattn_encode_keys(D.phi_kv, None, None, D.B, 100, D.cache)
    torch.cuda.synchronize()
    got = gu.u32_host(D.codes)
    for b, n in enumerate(lens):
        n = int(n)
        assert np.all(got[b, :, :n - 100] == 0)
        gu.assert_codes_match(got[b, :, n - 100:n], codes[b, :, n - 100:n], act[b, :, n - 100:n], "tail rebuild")
    assert D.seq_lens.cpu().tolist() == lens.tolist()


@pytest.mark.parametrize("n_new", [1, 3, 70])
def test_encode_keys_append(n_new):
    cfg = W.scaled(W.c1(), context=300, k=16, batch=3, planted=0)
    L = W.make_layer(cfg, seed=31)
    L.seq_lens[:] = [300, 17, 0]
    D = gu.DeviceLayer(L, extra_rows=n_new)
    rng = np.random.default_rng(32)
    k_new = W.f32_to_bf16_bits(rng.standard_normal((3, 8, n_new, 128), dtype=np.float32))
    v_new = W.f32_to_bf16_bits(rng.standard_normal((3, 8, n_new, 128), dtype=np.float32))
    k_before = D.k.clone()
    D.ctx.hashattn_encode_keys(D.phi_kv, gu.bf16_dev(k_new), gu.bf16_dev(v_new), D.B, n_new, D.cache)
    torch.cuda.synchronize()
    assert D.cache.max_seq_len == 300 + n_new
    ocache, codes, lens = D.oracle_cache()
    act = oracle.encode_keys(oracle.Mlp(L.w_kv), ocache, k_new, v_new, n_new, want_act=True)
    assert D.seq_lens.cpu().tolist() == lens.tolist() == [300 + n_new, 17 + n_new, n_new]
    got_codes = gu.u32_host(D.codes)
    k_after = D.k.view(torch.int16).cpu().numpy().view(np.uint16)
    v_after = D.v.view(torch.int16).cpu().numpy().view(np.uint16)
    np.testing.assert_array_equal(k_after, ocache.k)          # rows copied, nothing else touched
    np.testing.assert_array_equal(v_after, ocache.v)
    for b, start in enumerate((300, 17, 0)):
        sl = slice(start, start + n_new)
        gu.assert_codes_match(got_codes[b, :, sl], codes[b, :, sl], act[b], f"append b={b}")
        assert np.all(got_codes[b, :, :start] == 0) and np.all(got_codes[b, :, start + n_new:] == 0)
    assert torch.equal(k_before[:2, :, :17], D.k[:2, :, :17])


@pytest.mark.parametrize("heads,batch", [(64, 20), (128, 32)])        # 4 and 8 vectors per block in the append kernel
def test_encode_keys_append_many_heads(heads, batch):
    cfg = W.scaled(W.c1(), context=40, k=4, batch=batch, planted=0, n_q_heads=heads, n_kv_heads=heads)
    L = W.make_layer(cfg, seed=33)
    L.seq_lens[:] = np.arange(batch) % 37
    D = gu.DeviceLayer(L, extra_rows=4)
    rng = np.random.default_rng(34)
    k_new = W.f32_to_bf16_bits(rng.standard_normal((batch, heads, 1, 128), dtype=np.float32))
    v_new = W.f32_to_bf16_bits(rng.standard_normal((batch, heads, 1, 128), dtype=np.float32))
    D.ctx.hashattn_encode_keys(D.phi_kv, gu.bf16_dev(k_new), gu.bf16_dev(v_new), D.B, 1, D.cache)
    torch.cuda.synchronize()
    ocache, codes, lens = D.oracle_cache()
    lens0 = lens.copy()
    act = oracle.encode_keys(oracle.Mlp(L.w_kv), ocache, k_new, v_new, 1, want_act=True)
    assert D.seq_lens.cpu().tolist() == lens.tolist() == (lens0 + 1).tolist()
    got_codes = gu.u32_host(D.codes)
    np.testing.assert_array_equal(D.k.view(torch.int16).cpu().numpy().view(np.uint16), ocache.k)
    np.testing.assert_array_equal(D.v.view(torch.int16).cpu().numpy().view(np.uint16), ocache.v)
    for b in range(batch):
        p0 = int(lens0[b])
        gu.assert_codes_match(got_codes[b, :, p0:p0 + 1], codes[b, :, p0:p0 + 1], act[b], f"append b={b}")
        assert np.all(got_codes[b, :, :p0] == 0) and np.all(got_codes[b, :, p0 + 1:] == 0)


def test_append_reports_a_counter_left_behind_by_an_unfinished_launch():
    """The decode-time append moves the lengths from inside its kernel through a block counter that is
    zero between calls.  With the counter set as an unfinished earlier launch would leave it, the next
    append notices (its blocks count past the grid) and every later call on the context fails with a
    message; a fresh context on the same cache works."""
    import paper_2412_14468_amd as ha
    cfg = W.scaled(W.c1(), context=300, k=16, batch=3, planted=0)
    L = W.make_layer(cfg, seed=35)
    D = gu.DeviceLayer(L, extra_rows=8)                 # contiguous cache with room: every row written stays inside it
    rng = np.random.default_rng(36)
    k_new = gu.bf16_dev(W.f32_to_bf16_bits(rng.standard_normal((3, 8, 1, 128), dtype=np.float32)))
    v_new = gu.bf16_dev(W.f32_to_bf16_bits(rng.standard_normal((3, 8, 1, 128), dtype=np.float32)))
    D.ctx.hashattn_encode_keys(D.phi_kv, k_new, v_new, D.B, 1, D.cache)          # a normal append: lengths move by one
    torch.cuda.synchronize()
    assert D.seq_lens.cpu().tolist() == [301, 301, 301]
    D.ctx.hashattn_selftest_set_append_counter(5)
    D.ctx.hashattn_encode_keys(D.phi_kv, k_new, v_new, D.B, 1, D.cache)          # runs to its end, reports the state
    torch.cuda.synchronize()
    qc = torch.zeros((D.B, D.Hq), dtype=torch.int32, device=gu.DEV)
    with pytest.raises(ha.HashAttnError, match="beyond its grid") as e:
        D.ctx.hashattn_encode_query(D.phi_q, D.q, D.B, qc)
    assert e.value.status == ha.HIP_ERROR
    with pytest.raises(ha.HashAttnError, match="beyond its grid"):
        D.ctx.hashattn_encode_keys(D.phi_kv, k_new, v_new, D.B, 1, D.cache)
    D.ctx.hashattn_selftest_set_append_counter(0)
    D.ctx.close()
    D.seq_lens.copy_(torch.tensor([301, 301, 301], dtype=torch.int32))
    D.cache.max_seq_len = 301
    ctx2 = ha.Context(D.Hq, D.Hkv, D.B, 308, 16)
    ctx2.hashattn_encode_keys(D.phi_kv, k_new, v_new, D.B, 1, D.cache)
    ctx2.hashattn_encode_query(D.phi_q, D.q, D.B, qc)
    torch.cuda.synchronize()
    assert D.seq_lens.cpu().tolist() == [302, 302, 302]


# ---------------------------------------------------------------- whole step, Llama shape, ragged
def run_whole_step(L, extra_rows=0, gather_heads=None):
    """Stages: GPU codes vs oracle codes; GPU TOPK on oracle codes; GPU GATHER-ATT on oracle sets;
    then the chained GPU step, which must agree end to end whenever no code bit differed."""
    D = gu.DeviceLayer(L, extra_rows=extra_rows)
    g = D.Hq // D.Hkv
    ocache, codes, lens = D.oracle_cache()
    phi_q_o, phi_kv_o = oracle.Mlp(L.w_q), oracle.Mlp(L.w_kv)
    n_all = int(L.seq_lens.max())
    act_k = oracle.encode_keys(phi_kv_o, ocache, None, None, max(n_all, 1), want_act=True)
    D.ctx.hashattn_encode_keys(D.phi_kv, None, None, D.B, max(n_all, 1), D.cache)
    torch.cuda.synchronize()
    gpu_codes = gu.u32_host(D.codes).copy()
    flips = 0
    for b in range(D.B):
        n = int(L.seq_lens[b])
        if L.page_table is None:
            flips += gu.assert_codes_match(gpu_codes[b, :, :n], codes[b, :, :n], act_k[b, :, :n], "key codes")
        else:
            ps = L.cfg.page_size
            t = np.arange(n)
            pg, sl = L.page_table[b, t // ps], t % ps
            flips += gu.assert_codes_match(gpu_codes[pg, :, sl], codes[pg, :, sl],
                                           np.moveaxis(act_k[b, :, :n], 0, 1), "key codes (paged)")
    k_new = v_new = None
    if L.k_new is not None:
        k_new, v_new = L.k_new[:, :, None, :].copy(), L.v_new[:, :, None, :].copy()
        oracle.encode_keys(phi_kv_o, ocache, k_new, v_new, 1)
        D.ctx.hashattn_encode_keys(D.phi_kv, gu.bf16_dev(k_new), gu.bf16_dev(v_new), D.B, 1, D.cache)
        torch.cuda.synchronize()
        assert D.seq_lens.cpu().tolist() == lens.tolist()
    qc_gpu = torch.zeros((D.B, D.Hq), dtype=torch.int32, device=gu.DEV)
    D.ctx.hashattn_encode_query(D.phi_q, D.q, D.B, qc_gpu)
    torch.cuda.synchronize()
    qc_ref, act_q = oracle.encode_query(phi_q_o, L.q)
    flips += gu.assert_codes_match(gu.u32_host(qc_gpu), qc_ref, act_q, "query codes")

    # TOPK and GATHER-ATT on the oracle's codes
    gpu_codes_after = gu.u32_host(D.codes).copy()
    D.set_codes(codes)
    ref = oracle_topk_all(codes, lens, qc_ref, L.k_per_seq, g, L)
    idx, count = check_topk(D, qc_ref, ref)
    out_staged = check_gather(D, ocache, idx, count, ref, heads=gather_heads)
    flips += check_combined_entry(D, qc_ref, act_q, ref)

    # chained GPU step on the GPU's own codes
    D.set_codes(gpu_codes_after)
    idx2, count2, _, out2 = D.new_outputs()
    D.ctx.hashattn_score_topk(qc_gpu, D.cache, D.B, D.k_per_seq, D.k_max, idx2, count2, None)
    D.ctx.hashattn_gather_attend(D.q, D.cache, idx2, count2, D.B, D.k_max, D.scale, out2)
    torch.cuda.synchronize()
    same_codes = np.array_equal(gpu_codes_after, codes) and np.array_equal(gu.u32_host(qc_gpu), qc_ref)
    if same_codes:
        assert torch.equal(idx2, idx) and torch.equal(count2, count)
        assert torch.equal(out2.view(torch.int16), out_staged.view(torch.int16))
    return flips


def test_llama_shape_ragged_batch():
    cfg = W.scaled(W.c1(), context=5003, k=157, batch=3, planted=16)
    L = W.make_layer(cfg, seed=41)
    L.seq_lens[:] = [5003, 1, 2049]
    L.k_per_seq[:] = [157, 157, 64]
    run_whole_step(L)


def test_many_heads_short_lists_single_block_path():
    """k <= 1024 with at least 128 (sequence, head) pairs: GATHER-ATT runs one block per head."""
    cfg = W.scaled(W.c1(), context=3001, k=97, batch=5, planted=8)
    L = W.make_layer(cfg, seed=42)
    L.seq_lens[:] = [3001, 0, 17, 2048, 96]
    L.k_per_seq[:] = [97, 97, 97, 1, 96]
    run_whole_step(L)


def test_c1_full_size():
    """Llama-3.1-8B-shaped layer, N = 32768, k = 1024: every head against the oracle."""
    L = W.make_layer(W.c1())
    flips = run_whole_step(L)
    assert flips < 2000          # ~0.5 % of bits sit within 1e-3 of zero; only a few of those flip


def test_c2_shape_append_then_step():
    cfg = W.scaled(W.c2(batch=3, context=4097), planted=8)
    L = W.make_layer(cfg, seed=43)
    run_whole_step(L)


def test_c4_paged_mixed_lengths():
    cfg = W.scaled(W.c4(batch=6, lo=100, hi=3000), planted=4)
    L = W.make_layer(cfg, seed=44)
    run_whole_step(L)


# ---------------------------------------------------------------- TOPK edge cases on chosen codes
def topk_case(n, k, codes_fn, batch=1, Hq=4, Hkv=1, k_per_seq=None, lens=None):
    cfg = W.Config("edge", 9, batch, Hq, Hkv, 128, n, k, mlp_dims=None, planted=0)
    L = W.make_layer(cfg, seed=1000 + n + k)
    if lens is not None:
        L.seq_lens[:] = lens
    if k_per_seq is not None:
        L.k_per_seq[:] = k_per_seq
    L.k_codes[...] = codes_fn(L.k_codes.shape)
    D = gu.DeviceLayer(L)
    D.set_codes(np.pad(L.k_codes, ((0, 0), (0, 0), (0, D.k_host.shape[2] - L.k_codes.shape[2]))))
    ocache, codes, lns = D.oracle_cache()
    codes[:, :, :L.k_codes.shape[2]] = L.k_codes
    ref = oracle_topk_all(codes, lns, L.q_codes, L.k_per_seq, Hq // Hkv, L)
    idx, count = check_topk(D, L.q_codes, ref)
    check_gather(D, ocache, idx, count, ref)


def test_topk_all_codes_equal_takes_index_prefix():
    topk_case(3000, 100, lambda s: np.full(s, 0xDEADBEEF, np.uint32))


def test_topk_two_valued_codes_heavy_ties():
    rng = np.random.default_rng(3)
    topk_case(70001, 2500, lambda s: np.where(rng.random(s) < 0.5, 0x0F0F0F0F, 0x0F0F0F1F).astype(np.uint32))


def test_topk_k_larger_than_n_and_k_one():
    rng = np.random.default_rng(4)
    topk_case(77, 200, lambda s: rng.integers(0, 2 ** 32, size=s, dtype=np.uint64).astype(np.uint32))
    topk_case(513, 1, lambda s: rng.integers(0, 2 ** 32, size=s, dtype=np.uint64).astype(np.uint32))
    topk_case(1, 1, lambda s: rng.integers(0, 2 ** 32, size=s, dtype=np.uint64).astype(np.uint32))


def test_topk_empty_and_mixed_sequences_per_seq_k():
    rng = np.random.default_rng(5)
    topk_case(2000, 300, lambda s: rng.integers(0, 2 ** 32, size=s, dtype=np.uint64).astype(np.uint32),
              batch=4, Hq=8, Hkv=2, lens=[0, 2000, 255, 1025], k_per_seq=[5, 300, 256, 1])


def test_topk_group_sizes():
    rng = np.random.default_rng(6)
    for Hq, Hkv in ((2, 2), (4, 2), (8, 1)):
        topk_case(4500, 140, lambda s: rng.integers(0, 2 ** 32, size=s, dtype=np.uint64).astype(np.uint32),
                  Hq=Hq, Hkv=Hkv)


def test_topk_is_repeatable():
    L = W.make_layer(W.scaled(W.c0(), context=100000, k=3125))
    D = gu.DeviceLayer(L)
    D.set_codes(L.k_codes)
    qc = gu.u32_dev(L.q_codes)
    outs = []
    for _ in range(3):
        idx, count, thr, out = D.new_outputs()
        D.ctx.hashattn_score_topk(qc, D.cache, 1, None, D.k_max, idx, count, thr)
        D.ctx.hashattn_gather_attend(D.q, D.cache, idx, count, 1, D.k_max, D.scale, out)
        torch.cuda.synchronize()
        outs.append((idx.clone(), out.clone()))
    for idx, out in outs[1:]:
        assert torch.equal(idx, outs[0][0]) and torch.equal(out.view(torch.int16), outs[0][1].view(torch.int16))


# ---------------------------------------------------------------- argument errors (nothing is launched)
def test_argument_errors_are_status_codes():
    import paper_2412_14468_amd as ha
    L = W.make_layer(W.scaled(W.c0(), context=256, k=16))
    D = gu.DeviceLayer(L)
    idx, count, thr, out = D.new_outputs()
    qc = gu.u32_dev(L.q_codes)
    with pytest.raises(ha.HashAttnError) as e:
        D.ctx.hashattn_score_topk(None, D.cache, 1, None, 16, idx, count, thr)
    assert e.value.status == ha.INVALID_ARG
    with pytest.raises(ha.HashAttnError) as e:
        D.ctx.hashattn_score_topk(qc, D.cache, 1, None, 17, idx, count, thr)
    assert e.value.status == ha.SCRATCH_TOO_SMALL
    with pytest.raises(ha.HashAttnError) as e:
        D.ctx.hashattn_score_topk(qc, D.cache, 2, None, 16, idx, count, thr)
    assert e.value.status == ha.SCRATCH_TOO_SMALL
    with pytest.raises(ha.HashAttnError) as e:
        D.ctx.hashattn_score_topk(qc, D.cache, 1, None, 0, idx, count, thr)
    assert e.value.status == ha.INVALID_ARG
    with pytest.raises(ha.HashAttnError) as e:
        D.ctx.hashattn_gather_attend(D.q.data_ptr() + 2, D.cache, idx, count, 1, 16, 0.1, out)
    assert e.value.status == ha.INVALID_ARG          # misaligned q
    with pytest.raises(ha.HashAttnError) as e:
        D.ctx.hashattn_gather_attend(D.q, D.cache, idx, count, 1, 16, float("nan"), out)
    assert e.value.status == ha.INVALID_ARG
    D.cache.max_seq_len = 10 ** 6
    with pytest.raises(ha.HashAttnError) as e:
        D.ctx.hashattn_dense_attend(D.q, D.cache, 1, 0.1, out)
    assert e.value.status == ha.SCRATCH_TOO_SMALL
    D.cache.max_seq_len = 256
    with pytest.raises(ha.HashAttnError) as e:
        ha.Context(32, 8, 1, 1024, 32, head_dim=64)
    assert e.value.status == ha.UNSUPPORTED
    with pytest.raises(ha.HashAttnError) as e:
        ha.Context(32, 5, 1, 1024, 32)
    assert e.value.status == ha.INVALID_ARG
    # outputs were never touched by the failed calls
    assert torch.all(idx == -7) and torch.all(count == -7)
