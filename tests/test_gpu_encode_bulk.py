"""GPU parity of the bulk (prefill-side) key encoder, which runs on the matrix cores for the paper's
mapping shapes (section 4.1, eq. 2; 128-128-128-32 of section 5.2), against the fp64 oracle: codes
bit-exact wherever the pre-sign activation exceeds 1e-3 in magnitude.  Also measures how far below
that bound the disagreements really start (the bf16 hi/lo operand split keeps about 16 bits)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
import gpu_util as gu

pytestmark = pytest.mark.gpu


def disagreement_margin(gpu_codes, ref_codes, act):
    """Largest |activation| among the bits on which GPU and oracle disagree (0 if none)."""
    diff = (gpu_codes ^ ref_codes).astype(np.uint32)
    bits = ((diff[..., None] >> np.arange(32, dtype=np.uint32)) & 1).astype(bool)
    return float(np.abs(act)[bits].max()) if bits.any() else 0.0


@pytest.mark.parametrize("dims", [(128, 32), (128, 128, 32), (128, 128, 128, 32)])
@pytest.mark.parametrize("with_bias", [False, True])
def test_bulk_encode_shapes_bias_and_margin(dims, with_bias):
    import paper_2412_14468_amd as ha
    n = 5000                                       # several blocks of 256 tokens, ragged last tile
    cfg = W.scaled(W.c1(), context=n, k=16, batch=2, planted=8, mlp_dims=dims)
    L = W.make_layer(cfg, seed=41 + len(dims))
    L.seq_lens[1] = 3333
    D = gu.DeviceLayer(L)
    biases = None
    phi = D.phi_kv
    if with_bias:
        rng = np.random.default_rng(7)
        biases = [rng.uniform(-0.3, 0.3, size=(8, w.shape[2])).astype(np.float32) for w in L.w_kv]
        b_dev = [torch.from_numpy(b).to(gu.DEV) for b in biases]
        phi = ha.Mlp(D.wkv_dev, b_dev)
    D.ctx.hashattn_encode_keys(phi, None, None, D.B, n, D.cache)
    torch.cuda.synchronize()
    ocache, codes, lens = D.oracle_cache()
    act = oracle.encode_keys(oracle.Mlp(L.w_kv, biases), ocache, None, None, n, want_act=True)
    got = gu.u32_host(D.codes)
    worst = 0.0
    for b, nb in enumerate(lens):
        nb = int(nb)
        gu.assert_codes_match(got[b, :, :nb], codes[b, :, :nb], act[b, :, :nb], f"bulk encode b={b}")
        worst = max(worst, disagreement_margin(got[b, :, :nb], codes[b, :, :nb], act[b, :, :nb]))
        assert np.all(got[b, :, nb:] == 0), "codes past seq_len must stay untouched"
    assert worst < 1e-4, f"a code bit differs at |activation| = {worst:.2e}: the operand split lost precision"
    if with_bias:
        plain = np.zeros_like(codes)
        c2 = oracle.Cache(ocache.k, ocache.v, plain, lens.copy())
        oracle.encode_keys(oracle.Mlp(L.w_kv), c2, None, None, n)
        assert (plain != codes).any()              # the bias matters in this case


def test_bulk_encode_paged_and_partial_rebuild():
    cfg = W.scaled(W.c4(batch=3, lo=700, hi=3000), name="paged-bulk")
    L = W.make_layer(cfg, seed=51)
    D = gu.DeviceLayer(L)
    n_cap = L.max_pages_per_seq * cfg.page_size
    D.ctx.hashattn_encode_keys(D.phi_kv, None, None, D.B, n_cap, D.cache)
    torch.cuda.synchronize()
    ocache, codes, lens = D.oracle_cache()
    oracle.encode_keys(oracle.Mlp(L.w_kv), ocache, None, None, n_cap)
    got_full = gu.u32_host(D.codes).copy()
    # compare in logical token order through the page table
    for b, nb in enumerate(lens):
        nb = int(nb)
        t = np.arange(nb)
        pg, sl = L.page_table[b, t // cfg.page_size], t % cfg.page_size
        for h in range(cfg.n_kv_heads):
            phi = oracle.Mlp([w[h:h + 1] for w in L.w_kv])
            acts = np.stack([oracle.encode_vec(phi, 0, ocache.k[pg[i], h, sl[i]])[1] for i in range(0, nb, 97)])
            gu.assert_codes_match(got_full[pg[::97], h, sl[::97]], codes[pg[::97], h, sl[::97]], acts, f"paged b={b} h={h}")
    # last 300 tokens only
    D.codes.zero_()
    D.ctx.hashattn_encode_keys(D.phi_kv, None, None, D.B, 300, D.cache)
    torch.cuda.synchronize()
    got = gu.u32_host(D.codes)
    for b, nb in enumerate(lens):
        nb = int(nb)
        t = np.arange(nb)
        pg, sl = L.page_table[b, t // cfg.page_size], t % cfg.page_size
        head = got[pg[:nb - 300], :, sl[:nb - 300]]
        assert np.all(head == 0)
        np.testing.assert_array_equal(got[pg[nb - 300:], :, sl[nb - 300:]], got_full[pg[nb - 300:], :, sl[nb - 300:]])


def test_bulk_append_many_tokens():
    """Append of a long chunk (prefill in pieces): rows copied, codes by the matrix-core kernel."""
    n_new = 1000
    cfg = W.scaled(W.c1(), context=300, k=16, batch=3, planted=0)
    L = W.make_layer(cfg, seed=61)
    L.seq_lens[:] = [300, 17, 0]
    D = gu.DeviceLayer(L, extra_rows=n_new)
    rng = np.random.default_rng(62)
    k_new = W.f32_to_bf16_bits(rng.standard_normal((3, 8, n_new, 128), dtype=np.float32))
    v_new = W.f32_to_bf16_bits(rng.standard_normal((3, 8, n_new, 128), dtype=np.float32))
    D.ctx.hashattn_encode_keys(D.phi_kv, gu.bf16_dev(k_new), gu.bf16_dev(v_new), D.B, n_new, D.cache)
    torch.cuda.synchronize()
    ocache, codes, lens = D.oracle_cache()
    act = oracle.encode_keys(oracle.Mlp(L.w_kv), ocache, k_new, v_new, n_new, want_act=True)
    assert D.seq_lens.cpu().tolist() == lens.tolist() == [300 + n_new, 17 + n_new, n_new]
    got = gu.u32_host(D.codes)
    np.testing.assert_array_equal(D.k.view(torch.int16).cpu().numpy().view(np.uint16), ocache.k)
    for b, start in enumerate((300, 17, 0)):
        sl = slice(start, start + n_new)
        gu.assert_codes_match(got[b, :, sl], codes[b, :, sl], act[b], f"bulk append b={b}")
        assert np.all(got[b, :, :start] == 0) and np.all(got[b, :, start + n_new:] == 0)
