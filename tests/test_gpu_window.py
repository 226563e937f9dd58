"""GPU parity of hashattn_score_topk_window (always-kept first / most recent tokens, section 5 protocol)
against the oracle, through the C ABI: index sets, counts and thresholds bit-exact on the same codes,
GATHER-ATT over the windowed sets within the output tolerance."""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as W
import gpu_util as gu

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("topk_path")]


def random_codes(rng):
    return lambda s: rng.integers(0, 2 ** 32, size=s, dtype=np.uint64).astype(np.uint32)


def window_case(n, k, n_sink, n_local, codes_fn, batch=1, Hq=4, Hkv=1, lens=None, k_per_seq=None, check_out=True):
    cfg = W.Config("window", 9, batch, Hq, Hkv, 128, n, k, mlp_dims=None, planted=0)
    L = W.make_layer(cfg, seed=2000 + n + k + n_sink)
    if lens is not None:
        L.seq_lens[:] = lens
    if k_per_seq is not None:
        L.k_per_seq[:] = k_per_seq
    L.k_codes[...] = codes_fn(L.k_codes.shape)
    k_max = int(L.k_per_seq.max())
    pitch = k_max + n_sink + n_local
    D = gu.DeviceLayer(L, max_k=pitch)
    D.set_codes(np.pad(L.k_codes, ((0, 0), (0, 0), (0, D.k_host.shape[2] - L.k_codes.shape[2]))))
    ocache, codes, lns = D.oracle_cache()
    codes[:, :, :L.k_codes.shape[2]] = L.k_codes
    g = Hq // Hkv

    idx = torch.full((batch, Hq, pitch), -7, dtype=torch.int32, device=gu.DEV)
    count = torch.full((batch, Hq), -7, dtype=torch.int32, device=gu.DEV)
    thr = torch.full((batch, Hq), 255, dtype=torch.uint8, device=gu.DEV)
    out = torch.zeros((batch, Hq, 128), dtype=torch.bfloat16, device=gu.DEV)
    kps = None if k_per_seq is None else D.k_per_seq
    D.ctx.hashattn_score_topk_window(gu.u32_dev(L.q_codes), D.cache, batch, kps, k_max, n_sink, n_local, idx, count, thr)
    D.ctx.hashattn_gather_attend(D.q, D.cache, idx, count, batch, pitch, D.scale, out)
    torch.cuda.synchronize()
    idx_h, count_h, thr_h = idx.cpu().numpy(), count.cpu().numpy(), thr.cpu().numpy()
    for b in range(batch):
        nb = int(lns[b])
        for h in range(Hq):
            sc = oracle.scores(int(L.q_codes[b, h]), codes[b, h // g, :nb])
            ref, rthr, got = oracle.topk_window(sc, int(L.k_per_seq[b]), n_sink, n_local)
            assert count_h[b, h] == len(ref), (b, h, count_h[b, h], len(ref))
            np.testing.assert_array_equal(idx_h[b, h, :len(ref)], ref, err_msg=f"idx b={b} h={h}")
            assert np.all(idx_h[b, h, len(ref):] == -7)
            assert thr_h[b, h] == rthr
            if check_out:
                o = oracle.gather_attend(ocache, b, h // g, L.q[b, h], ref, D.scale)
                gu.assert_out_close(out[b, h:h + 1], o[None], f"gather over window set b={b} h={h}")


def test_window_128_128_llama_group():
    rng = np.random.default_rng(1)
    window_case(20000, 625, 128, 128, random_codes(rng), Hq=8, Hkv=2)


@pytest.mark.parametrize("n,k,s,l", [(5000, 100, 128, 128),   # several waves, unit 256
                                     (5000, 100, 0, 128), (5000, 100, 128, 0),
                                     (5000, 100, 3, 5),       # edges inside a lane's run
                                     (300, 40, 128, 128),     # middle shorter than a wave
                                     (256, 40, 128, 128),     # empty middle
                                     (100, 40, 128, 128),     # window larger than the sequence
                                     (1, 1, 1, 1),
                                     (70001, 2500, 1000, 3000),  # window spans units and blocks; ragged tail
                                     (5000, 6000, 128, 128)])    # k larger than the middle
def test_window_shapes(n, k, s, l):
    rng = np.random.default_rng(n + k)
    window_case(n, k, s, l, random_codes(rng), check_out=(n <= 5000))


def test_window_heavy_ties_quota_inside_middle():
    rng = np.random.default_rng(3)
    two = lambda s: np.where(rng.random(s) < 0.5, 0x0F0F0F0F, 0x0F0F0F1F).astype(np.uint32)
    window_case(70001, 2500, 128, 128, two, check_out=False)
    window_case(9000, 700, 300, 17, lambda s: np.full(s, 0xDEADBEEF, np.uint32), check_out=False)


def test_window_mixed_batch_per_sequence_k():
    rng = np.random.default_rng(5)
    window_case(40000, 1200, 128, 128, random_codes(rng), batch=5, Hq=8, Hkv=2,
                lens=[0, 40000, 255, 1025, 17000], k_per_seq=[5, 1200, 256, 1, 0], check_out=False)


def test_window_big_units():
    """Units of 512, 1024 and 2048 tokens (several 16-byte loads per lane, two chunks per wave) with a
    window that spans units."""
    rng = np.random.default_rng(6)
    window_case(600000, 4000, 5000, 9000, random_codes(rng), Hq=2, Hkv=1, check_out=False)           # 512
    window_case(40000, 1000, 700, 1500, random_codes(rng), batch=64, Hq=2, Hkv=1, check_out=False)    # 1024
    window_case(20000, 600, 128, 3000, random_codes(rng), batch=130, Hq=1, Hkv=1, check_out=False)    # 2048


def test_no_window_equals_plain_entry_point():
    rng = np.random.default_rng(7)
    cfg = W.Config("plain", 9, 2, 8, 2, 128, 30000, 900, mlp_dims=None, planted=0)
    L = W.make_layer(cfg, seed=77)
    D = gu.DeviceLayer(L)
    D.set_codes(np.pad(L.k_codes, ((0, 0), (0, 0), (0, D.k_host.shape[2] - L.k_codes.shape[2]))))
    qc = gu.u32_dev(L.q_codes)
    a = D.new_outputs(); b = D.new_outputs()
    D.ctx.hashattn_score_topk(qc, D.cache, 2, None, D.k_max, a[0], a[1], a[2])
    D.ctx.hashattn_score_topk_window(qc, D.cache, 2, None, D.k_max, 0, 0, b[0], b[1], b[2])
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])


def test_window_argument_errors():
    import paper_2412_14468_amd as ha
    L = W.make_layer(W.scaled(W.c0(), context=256, k=16))
    D = gu.DeviceLayer(L, max_k=64)
    qc = gu.u32_dev(L.q_codes)
    idx, count, thr, _ = D.new_outputs()
    with pytest.raises(ha.HashAttnError, match="negative"):
        D.ctx.hashattn_score_topk_window(qc, D.cache, 1, None, 16, -1, 0, idx, count, thr)
    with pytest.raises(ha.HashAttnError, match="exceeds max_k"):
        D.ctx.hashattn_score_topk_window(qc, D.cache, 1, None, 16, 40, 40, idx, count, thr)
