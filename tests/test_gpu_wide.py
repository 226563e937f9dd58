"""GPU parity for signatures wider than 32 bits (b = 32 W bits, W = 2, 4, 8, 16; the paper's bit-width
ablation and its SCORE latency table) against the oracle, through the C ABI: SCORE + TOPK bit-exact on
the same codes (with and without the always-kept window), codes from the mapping kernels bit-exact
where |activation| > 1e-3, GATHER-ATT over the selected sets within the output tolerance."""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as W
import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = gu.DEV


def rand_words(rng, shape):
    return rng.integers(0, 2 ** 32, size=shape, dtype=np.uint64).astype(np.uint32)


def topk_wide_case(words, n, k, batch=1, Hq=4, Hkv=1, n_sink=0, n_local=0, lens=None, k_per_seq=None,
                   codes_fn=None, paged=False, seed=0):
    import paper_2412_14468_amd as ha
    rng = np.random.default_rng(1000 * words + n + k + seed)
    g = Hq // Hkv
    lens = np.array(lens if lens is not None else [n] * batch, dtype=np.int32)
    kps = np.array(k_per_seq if k_per_seq is not None else [k] * batch, dtype=np.int32)
    k_max = int(kps.max())
    pitch = k_max + n_sink + n_local
    n_max = n + (-n) % 4
    if paged:
        pages_per_seq = (n_max + 15) // 16
        n_pages = batch * pages_per_seq
        table = rng.permutation(n_pages).astype(np.int32).reshape(batch, pages_per_seq)
        codes = codes_fn(rng, (n_pages, Hkv, 16, words)) if codes_fn else rand_words(rng, (n_pages, Hkv, 16, words))
        kshape = (n_pages, Hkv, 16, 128)
    else:
        table = None
        codes = codes_fn(rng, (batch, Hkv, n_max, words)) if codes_fn else rand_words(rng, (batch, Hkv, n_max, words))
        kshape = (batch, Hkv, n_max, 128)
    q_codes = rand_words(rng, (batch, Hq, words))
    kz = torch.zeros(kshape, dtype=torch.bfloat16, device=DEV)
    codes_dev = gu.u32_dev(codes)
    cache = ha.KvCache(kz, kz, codes_dev, torch.from_numpy(lens).to(DEV), int(lens.max()),
                       page_table=None if table is None else torch.from_numpy(table).to(DEV))
    ctx = ha.Context(Hq, Hkv, batch, max(n_max, 1), max(pitch, 1), page_size=16 if paged else 0, bits=32 * words)
    idx = torch.full((batch, Hq, pitch), -7, dtype=torch.int32, device=DEV)
    count = torch.full((batch, Hq), -7, dtype=torch.int32, device=DEV)
    thr = torch.full((batch, Hq), 255, dtype=torch.uint8, device=DEV)
    ctx.hashattn_score_topk_window(gu.u32_dev(q_codes), cache, batch, None if k_per_seq is None else torch.from_numpy(kps).to(DEV),
                                   k_max, n_sink, n_local, idx, count, thr)
    torch.cuda.synchronize()
    idx_h, count_h, thr_h = idx.cpu().numpy(), count.cpu().numpy(), thr.cpu().numpy()
    for b in range(batch):
        nb = int(lens[b])
        t = np.arange(nb)
        for h in range(Hq):
            if paged:
                kc = codes[table[b, t // 16], h // g, t % 16]
            else:
                kc = codes[b, h // g, :nb]
            sc = oracle.scores_wide(q_codes[b, h], np.ascontiguousarray(kc).reshape(nb, words))
            ref, rthr, got = oracle.topk_window(sc, int(kps[b]), n_sink, n_local)
            assert count_h[b, h] == len(ref), (b, h, count_h[b, h], len(ref))
            np.testing.assert_array_equal(idx_h[b, h, :len(ref)], ref, err_msg=f"W={words} b={b} h={h}")
            assert np.all(idx_h[b, h, len(ref):] == -7)
            assert thr_h[b, h] == min(rthr, 255)


@pytest.mark.parametrize("words", [2, 4, 8, 16])
def test_topk_wide_random_codes(words):
    topk_wide_case(words, 20000, 625, Hq=8, Hkv=2)
    topk_wide_case(words, 5000, 100, n_sink=128, n_local=128)
    topk_wide_case(words, 777, 2000)                       # k larger than the sequence
    topk_wide_case(words, 1, 1)


@pytest.mark.parametrize("words", [2, 4, 16])
def test_topk_wide_heavy_ties_and_ragged_batches(words):
    def few_codes(rng, shape):
        base = rand_words(rng, (3, shape[-1]))
        base[1] = base[0]; base[1, 0] ^= 1                  # one bit apart: adjacent scores, huge tie buckets
        pick = rng.integers(0, 3, size=shape[:-1])
        return base[pick]
    topk_wide_case(words, 70001, 2500, codes_fn=few_codes)
    topk_wide_case(words, 9000, 700, n_sink=300, n_local=17, codes_fn=lambda rng, s: np.broadcast_to(rand_words(rng, (s[-1],)), s).copy())
    topk_wide_case(words, 40000, 1200, batch=5, Hq=8, Hkv=2, n_sink=128, n_local=128,
                   lens=[0, 40000, 255, 1025, 17000], k_per_seq=[5, 1200, 256, 1, 0])


@pytest.mark.parametrize("words,Hq,Hkv", [(4, 2, 2), (4, 4, 2), (2, 8, 1), (8, 8, 1)])
def test_topk_wide_group_sizes_and_paged(words, Hq, Hkv):
    topk_wide_case(words, 4500, 140, Hq=Hq, Hkv=Hkv)
    topk_wide_case(words, 4500, 140, batch=3, Hq=Hq, Hkv=Hkv, paged=True, lens=[4500, 100, 2047], k_per_seq=[140, 140, 9])


def test_topk_wide_long_context_units_of_512_and_1024():
    topk_wide_case(4, 600000, 4000, Hq=2, Hkv=1, n_sink=5000, n_local=9000)        # pitch forces units of 512
    topk_wide_case(2, 40000, 1000, batch=64, Hq=2, Hkv=1)                           # many lanes: units of 1024
    topk_wide_case(2, 600001, 3000, Hq=4, Hkv=1, n_sink=7, n_local=1000)            # 64 bits in units of 512
    topk_wide_case(4, 30000, 900, batch=40, Hq=2, Hkv=1)                            # 128 bits in units of 1024 (step-mask select)


@pytest.mark.parametrize("bits,dims", [(64, (128, 128, 64)), (128, (128, 128)), (256, (128, 64, 128, 256)),
                                       (512, (128, 128, 512)), (512, (128, 512))])
def test_wide_mapping_and_whole_step(bits, dims):
    """encode_keys (bulk and append), encode_query, SCORE + TOPK, GATHER-ATT with b-bit signatures."""
    import paper_2412_14468_amd as ha
    words = bits // 32
    n, k, batch = 3000, 96, 2
    cfg = W.scaled(W.c1(context=n, k=k, batch=batch), name="wide", mlp_dims=dims, planted=8)
    L = W.make_layer(cfg, seed=300 + bits)
    L.seq_lens[1] = 1234
    g, Hq, Hkv = cfg.group, cfg.n_q_heads, cfg.n_kv_heads
    n_max = n + 4
    pad = np.zeros((batch, Hkv, 4, 128), dtype=np.uint16)
    k_host, v_host = np.concatenate([L.k, pad], axis=2), np.concatenate([L.v, pad], axis=2)
    kd, vd, qd = gu.bf16_dev(k_host), gu.bf16_dev(v_host), gu.bf16_dev(L.q)
    codes_dev = torch.zeros((batch, Hkv, n_max, words), dtype=torch.int32, device=DEV)
    lens_dev = torch.from_numpy(L.seq_lens.copy()).to(DEV)
    cache = ha.KvCache(kd, vd, codes_dev, lens_dev, int(L.seq_lens.max()))
    ctx = ha.Context(Hq, Hkv, batch, n_max, k, bits=bits)
    wq = [torch.from_numpy(w).to(DEV) for w in L.w_q]
    wkv = [torch.from_numpy(w).to(DEV) for w in L.w_kv]
    phi_q, phi_kv = ha.Mlp(wq), ha.Mlp(wkv)

    # oracle twin
    ok, ov = k_host.copy(), v_host.copy()
    olens = L.seq_lens.copy()
    ocache = oracle.Cache(ok, ov, np.zeros(ok.shape[:3], dtype=np.uint32), olens)
    ocodes = np.zeros((batch, Hkv, n_max, words), dtype=np.uint32)
    o_q, o_kv = oracle.Mlp(L.w_q), oracle.Mlp(L.w_kv)

    # 1. bulk rebuild
    ctx.hashattn_encode_keys(phi_kv, None, None, batch, n, cache)
    torch.cuda.synchronize()
    act = oracle.encode_keys_wide(o_kv, ocache, ocodes, None, None, n, want_act=True)
    got = gu.u32_host(codes_dev)
    for b in range(batch):
        nb = int(olens[b])
        for w in range(words):
            gu.assert_codes_match(got[b, :, :nb, w], ocodes[b, :, :nb, w], act[b, :, :nb, 32 * w:32 * w + 32], f"bulk b={b} w={w}")
        assert not got[b, :, nb:].any()
    # 2. append one token (decode-time kernel)
    rng = np.random.default_rng(bits)
    k_new = W.f32_to_bf16_bits(rng.standard_normal((batch, Hkv, 1, 128), dtype=np.float32))
    v_new = W.f32_to_bf16_bits(rng.standard_normal((batch, Hkv, 1, 128), dtype=np.float32))
    ctx.hashattn_encode_keys(phi_kv, gu.bf16_dev(k_new), gu.bf16_dev(v_new), batch, 1, cache)
    torch.cuda.synchronize()
    lens0 = olens.copy()
    act1 = oracle.encode_keys_wide(o_kv, ocache, ocodes, k_new, v_new, 1, want_act=True)
    assert lens_dev.cpu().tolist() == olens.tolist() == (lens0 + 1).tolist()
    got = gu.u32_host(codes_dev)
    for b in range(batch):
        p = int(lens0[b])
        for w in range(words):
            gu.assert_codes_match(got[b, :, p:p + 1, w], ocodes[b, :, p:p + 1, w], act1[b, :, :, 32 * w:32 * w + 32], f"append b={b} w={w}")
    np.testing.assert_array_equal(kd.view(torch.int16).cpu().numpy().view(np.uint16), ok)
    # 3. query codes
    qc_dev = torch.zeros((batch, Hq, words), dtype=torch.int32, device=DEV)
    ctx.hashattn_encode_query(phi_q, qd, batch, qc_dev)
    torch.cuda.synchronize()
    oqc, oqa = oracle.encode_query_wide(o_q, L.q, words)
    for w in range(words):
        gu.assert_codes_match(gu.u32_host(qc_dev)[:, :, w], oqc[:, :, w], oqa[:, :, 32 * w:32 * w + 32], f"query w={w}")
    # 4. SCORE + TOPK + GATHER-ATT on the oracle's codes
    codes_dev.copy_(gu.u32_dev(ocodes))
    scale = 1.0 / math.sqrt(128)
    kps = np.full(batch, k, dtype=np.int32)
    res = oracle.decode_step_wide(None, None, ocache, ocodes, L.q, kps, scale, q_codes=oqc)
    idx = torch.full((batch, Hq, k), -7, dtype=torch.int32, device=DEV)
    count = torch.zeros((batch, Hq), dtype=torch.int32, device=DEV)
    thr = torch.zeros((batch, Hq), dtype=torch.uint8, device=DEV)
    out = torch.zeros((batch, Hq, 128), dtype=torch.bfloat16, device=DEV)
    ctx.hashattn_score_topk(gu.u32_dev(oqc), cache, batch, None, k, idx, count, thr)
    ctx.hashattn_gather_attend(qd, cache, idx, count, batch, k, scale, out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(count.cpu().numpy(), res["count"])
    np.testing.assert_array_equal(idx.cpu().numpy(), res["idx"])
    np.testing.assert_array_equal(thr.cpu().numpy(), np.minimum(res["threshold"], 255))
    gu.assert_out_close(out, res["out"], f"gather_attend, {bits}-bit signatures")


def test_bad_widths_rejected():
    import paper_2412_14468_amd as ha
    with pytest.raises(ha.HashAttnError, match="bits"):
        ha.Context(4, 1, 1, 1024, 16, bits=96)
    ctx = ha.Context(4, 1, 1, 1024, 16, bits=512)
    q = torch.zeros((1, 4, 128), dtype=torch.bfloat16, device=DEV)
    qc = torch.zeros((1, 4, 16), dtype=torch.int32, device=DEV)
    w = [torch.zeros((4, 128, 256), dtype=torch.float32, device=DEV)]              # 256 outputs in a 512-bit context
    with pytest.raises(ha.HashAttnError, match="512 outputs"):
        ctx.hashattn_encode_query(ha.Mlp(w), q, 1, qc)
    w = [torch.zeros((4, 128, 512), dtype=torch.float32, device=DEV),             # hidden layers stop at 256
         torch.zeros((4, 512, 512), dtype=torch.float32, device=DEV)]
    with pytest.raises(ha.HashAttnError, match="hidden width"):
        ctx.hashattn_encode_query(ha.Mlp(w), q, 1, qc)
