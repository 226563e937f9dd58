"""GPU parity at the full sizes of the benchmark configurations (C2, C3, C4), in the launch
configuration bench.py times, on sampled (sequence, KV head) pairs.

Inputs are drawn on the device (seeded); for every sampled pair the K/V rows of that head are copied
to the host and the oracle runs the whole step on them as a one-head contiguous cache (also for the
paged configuration, which thereby checks the page-table addressing).  Stages as in the small tests:
codes bit-exact outside |activation| <= 1e-3, then TOPK and GATHER-ATT on the oracle's codes.  The dense
baseline kernel (hashattn_dense_attend) runs on the same cache and is compared with the oracle's dense
SDPA for the same sampled pairs.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def bits_of(t):                      # bf16 / int32 device tensor -> numpy bit patterns
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy().view(np.uint32)


class HeadView:
    """Logical (token-ordered) access to one (sequence, KV head) of a device cache."""

    def __init__(self, s, b, kvh, page_size):
        self.s, self.b, self.kvh, self.ps = s, b, kvh, page_size

    def _sel(self, n):
        if self.s.page_table is None:
            return None
        t = torch.arange(n, device=DEV)
        return self.s.page_table[self.b, t // self.ps].long(), t % self.ps

    def rows(self, tensor, n):
        if self.s.page_table is None:
            return tensor[self.b, self.kvh, :n]
        pg, sl = self._sel(n)
        return tensor[pg, self.kvh, sl]

    def put_codes(self, codes_host):
        n = codes_host.shape[0]
        src = torch.from_numpy(codes_host.view(np.int32)).to(DEV)
        if self.s.page_table is None:
            self.s.codes[self.b, self.kvh, :n] = src
        else:
            pg, sl = self._sel(n)
            self.s.codes[pg, self.kvh, sl] = src


def run_sampled(cfg, seed, pairs, extra_rows=0):
    import paper_2412_14468_amd as ha
    from paper_2412_14468_amd import runner
    from gpu_util import assert_codes_match, assert_out_close

    t = W.device_tensors(cfg, seed, extra_rows=extra_rows)
    s = runner.layer_from_tensors(t)
    g = cfg.group
    n_cap = t["n_max"]
    ctx = ha.Context(cfg.n_q_heads, cfg.n_kv_heads, cfg.batch, n_cap, s.k_max, page_size=cfg.page_size)
    lens0 = t["seq_lens_host"].copy()
    scale = 1.0 / math.sqrt(cfg.head_dim)

    # ---- the GPU's own whole step (prefill codes, [append], encode, TOPK, GATHER-ATT)
    runner.build_key_codes(ctx, s)
    runner.decode_step(ctx, s, append=cfg.append)
    torch.cuda.synchronize()
    lens1 = lens0 + (1 if cfg.append else 0)
    assert s.seq_lens.cpu().tolist() == lens1.tolist()
    gpu_q_codes = bits_of(s.q_codes)

    # ---- oracle per sampled pair; its codes replace the GPU's for the staged TOPK / GATHER-ATT run
    refs = {}
    flips = 0
    qc_dev = s.q_codes.clone()
    for (b, kvh) in pairs:
        hv = HeadView(s, b, kvh, cfg.page_size)
        n0, n1 = int(lens0[b]), int(lens1[b])
        cap = n1 + (-n1) % 4
        k_host = np.zeros((1, 1, cap, cfg.head_dim), dtype=np.uint16)
        v_host = np.zeros_like(k_host)
        # rows before the step come from the generator's tensors: after an append the device cache holds
        # the new row as well, which the oracle must produce itself from k_new
        k_host[0, 0, :n0] = bits_of(hv.rows(s.k, n0))
        v_host[0, 0, :n0] = bits_of(hv.rows(s.v, n0))
        codes = np.zeros((1, 1, cap), dtype=np.uint32)
        olens = np.array([n0], dtype=np.int32)
        ocache = oracle.Cache(k_host, v_host, codes, olens)
        phi_kv = oracle.Mlp([w[kvh:kvh + 1].cpu().numpy() for w in t["w_kv"]])
        phi_q = oracle.Mlp([w[kvh * g:(kvh + 1) * g].cpu().numpy() for w in t["w_q"]])
        act_k = oracle.encode_keys(phi_kv, ocache, None, None, max(n0, 1), want_act=True)
        q_host = bits_of(s.q[b:b + 1, kvh * g:(kvh + 1) * g])
        kw = {}
        if cfg.append:
            kw = dict(k_new=bits_of(t["k_new"][b:b + 1, kvh:kvh + 1, 0]), v_new=bits_of(t["v_new"][b:b + 1, kvh:kvh + 1, 0]))
        res = oracle.decode_step(phi_q, phi_kv, ocache, q_host, t["k_per_seq_host"][b:b + 1].copy(), scale, **kw)
        assert olens[0] == n1
        _, act_q = oracle.encode_query(phi_q, q_host)
        gpu_codes = bits_of(hv.rows(s.codes, n1))
        flips += assert_codes_match(gpu_codes[:n0], codes[0, 0, :n0], act_k[0, 0, :n0], f"key codes (b={b}, kvh={kvh})")
        if cfg.append:       # the appended token's code: compare where its activation is decisive
            _, a_new = oracle.encode_vec(phi_kv, 0, k_host[0, 0, n0])
            flips += assert_codes_match(gpu_codes[n0:n1], codes[0, 0, n0:n1], a_new[None, :], "appended key code")
            np.testing.assert_array_equal(bits_of(hv.rows(s.k, n1))[n0], k_host[0, 0, n0])
            np.testing.assert_array_equal(bits_of(hv.rows(s.v, n1))[n0], v_host[0, 0, n0])
        flips += assert_codes_match(gpu_q_codes[b, kvh * g:(kvh + 1) * g], res["q_codes"][0], act_q[0], "query codes")
        hv.put_codes(codes[0, 0, :n1])
        qc_dev[b, kvh * g:(kvh + 1) * g] = torch.from_numpy(res["q_codes"][0].view(np.int32)).to(DEV)
        # dense SDPA over all n1 tokens of this head (section 3.1): what hashattn_dense_attend must give
        res["dense"] = np.stack([oracle.dense_attend(ocache, 0, 0, q_host[0, j], n1, scale) for j in range(g)])
        refs[(b, kvh)] = res

    idx = torch.full_like(s.idx, -7)
    count = torch.full_like(s.count, -7)
    thr = torch.full_like(s.threshold, 255)
    out = torch.zeros_like(s.out)
    ctx.hashattn_score_topk(qc_dev, s.cache, s.B, s.k_per_seq, s.k_max, idx, count, thr)
    ctx.hashattn_gather_attend(s.q, s.cache, idx, count, s.B, s.k_max, s.scale, out)
    dense = torch.full_like(s.out, float("nan"))
    ctx.hashattn_dense_attend(s.q, s.cache, s.B, s.scale, dense)        # the split shape bench.py times
    torch.cuda.synchronize()
    idx_h, count_h, thr_h = idx.cpu().numpy(), count.cpu().numpy(), thr.cpu().numpy()
    for (b, kvh), res in refs.items():
        for j in range(g):
            h = kvh * g + j
            cnt = int(res["count"][0, j])
            assert count_h[b, h] == cnt
            np.testing.assert_array_equal(idx_h[b, h, :cnt], res["idx"][0, j, :cnt], err_msg=f"idx (b={b}, h={h})")
            assert np.all(idx_h[b, h, cnt:] == -7)
            assert thr_h[b, h] == res["threshold"][0, j]
        assert_out_close(out[b, kvh * g:(kvh + 1) * g], res["out"][0], f"gather_attend (b={b}, kvh={kvh})")
        assert_out_close(dense[b, kvh * g:(kvh + 1) * g], res["dense"], f"dense_attend (b={b}, kvh={kvh})")
    assert torch.isfinite(dense.float()).all()
    return flips


def test_c3_full_size_sampled_heads():
    """B = 1, N = 524288, k = 16384 (32x): two of the eight KV heads, all their query heads."""
    run_sampled(W.c3(), W.BASE_SEED + 3003, [(0, 1), (0, 6)])


def test_c3_16x_full_size_sampled_head():
    run_sampled(W.scaled(W.c3(k=32768), name="C3-16x"), W.BASE_SEED + 3004, [(0, 4)])


def test_c2_full_size_sampled_pairs_with_append():
    """B = 16, N = 131072 (cache holds N - 1, the step appends one token), k = 4096."""
    run_sampled(W.c2(), W.BASE_SEED + 2002, [(0, 0), (9, 3), (15, 7)])


def test_c4_full_size_sampled_pairs_paged():
    """64 sequences, lengths log-uniform in [4096, 65536], page size 16, k = ceil(N / 16)."""
    cfg = W.c4()
    t_lens = W.draw_lengths(np.random.Generator(np.random.PCG64(np.random.SeedSequence(W.BASE_SEED + 4004))), 64, 4096, 65536)
    longest, shortest = int(np.argmax(t_lens)), int(np.argmin(t_lens))
    run_sampled(cfg, W.BASE_SEED + 4004, [(longest, 2), (shortest, 5), (31, 0)])


def codes_only_case(n, k, Hq, Hkv, seed, batch=1):
    """SCORE + TOPK on uniform random codes (K/V are not touched), every query head against the oracle."""
    import paper_2412_14468_amd as ha
    import gpu_util as gu
    rng = np.random.default_rng(seed)
    codes = rng.integers(0, 2 ** 32, size=(batch, Hkv, n), dtype=np.uint64).astype(np.uint32)
    q_codes = rng.integers(0, 2 ** 32, size=(batch, Hq), dtype=np.uint64).astype(np.uint32)
    kz = torch.zeros((batch, Hkv, 4, 128), dtype=torch.bfloat16, device=DEV)
    cache = ha.KvCache(kz, kz, gu.u32_dev(codes), torch.full((batch,), n, dtype=torch.int32, device=DEV), n)
    cache.c.n_max = n                                                         # the code store has n rows
    ctx = ha.Context(Hq, Hkv, batch, n, k)
    idx = torch.full((batch, Hq, k), -7, dtype=torch.int32, device=DEV)
    count = torch.zeros((batch, Hq), dtype=torch.int32, device=DEV)
    thr = torch.zeros((batch, Hq), dtype=torch.uint8, device=DEV)
    ctx.hashattn_score_topk(gu.u32_dev(q_codes), cache, batch, None, k, idx, count, thr)
    torch.cuda.synchronize()
    idx_h, count_h, thr_h = idx.cpu().numpy(), count.cpu().numpy(), thr.cpu().numpy()
    for b in range(batch):
        for h in range(Hq):
            sc = oracle.scores(int(q_codes[b, h]), codes[b, h // (Hq // Hkv)])
            ref, rthr = oracle.topk_hist(sc, k)
            assert int(count_h[b, h]) == k and int(thr_h[b, h]) == rthr
            np.testing.assert_array_equal(idx_h[b, h], ref)


def test_topk_at_the_context_limit():
    """The largest context a 32-bit context accepts (4 Mi tokens: 256 blocks of 8 units of 2048 tokens per
    sequence), k = N / 32, one KV head with two query heads."""
    import paper_2412_14468_amd as ha
    n = 4 * 1024 * 1024
    codes_only_case(n, 131072, 2, 1, W.BASE_SEED + 4096)
    with pytest.raises(ha.HashAttnError, match="max_context"):
        ha.Context(2, 1, 1, n + 1, 131072)


def test_topk_groups_of_eight_at_512k():
    """64 query heads on 8 KV heads at 512K tokens: units of 2048 tokens with eight heads per block."""
    codes_only_case(524288, 16384, 64, 8, W.BASE_SEED + 4097)


def test_topk_many_sequences_units_of_2048():
    """130 sequences of 140000 tokens: 8-wave blocks of 1024-token units would be more than 2048 blocks, so the
    units are 2048 tokens (two chunks per wave in the select)."""
    codes_only_case(140000, 4375, 2, 1, W.BASE_SEED + 4098, batch=130)
