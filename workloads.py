"""Seeded synthetic inputs for the HashAttention decode path.

This module only *draws inputs*: random K/V/Q rows, random-init mapping
weights, random key codes, context lengths, page tables and planted tokens.
It contains none of the method's arithmetic (no encoding, scoring, selection
or attention) and is the only module shared by the CPU oracle's tests and the
HIP path's tests/bench.

Everything is numpy; bf16 tensors are carried as uint16 bit patterns (numpy
has no bf16 type).  The stand-in shapes follow the paper's efficiency setup
(Llama-3.1-8B attention shapes, 32-bit signatures, 32x sparsity; section 5.2
and the KV-cache sizing in section 1): the paper measures on a trained model
with real prompts, which are not available here.

Streams: one numpy PCG64 generator per tensor, spawned in a fixed order from
SeedSequence(BASE_SEED + config index), so adding a tensor at the end never
changes earlier ones.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional

import numpy as np

BASE_SEED = 241214468
BITS = 32

_STREAMS = ("q", "k", "v", "plant_pos", "plant_noise", "w_q", "w_kv",
            "codes", "lengths", "page_table", "k_new", "v_new")


# --------------------------------------------------------------------------
# bf16 <-> fp32 as storage conversion (round-to-nearest-even), on bit patterns
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (RNE) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32)
            << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# configuration
# --------------------------------------------------------------------------
@dataclasses.dataclass
class Config:
    name: str
    index: int                       # seed offset
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int                     # N (max over sequences for mixed batches)
    k: int                           # tokens selected per query head (uniform case)
    mlp_dims: Optional[tuple] = (128, 128, 32)   # None -> uniform random codes
    planted: int = 64                # planted pivotal tokens per query head
    page_size: int = 0               # 0 = contiguous KV, else tokens per page
    mixed_lengths: Optional[tuple] = None   # (lo, hi): log-uniform context lengths
    k_divisor: int = 0               # if >0, per-sequence k = ceil(N_b / k_divisor)
    append: bool = False             # the step appends one token before scoring

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


def c0() -> Config:
    """Single head, N=4096, k=256, uniform random codes (no mapping)."""
    return Config("C0", 0, 1, 1, 1, 128, 4096, 256, mlp_dims=None, planted=0)


def c1(context: int = 32768, k: Optional[int] = None, batch: int = 1) -> Config:
    """Llama-3.1-8B-shaped decode layer, batch 1, 32x sparsity."""
    return Config("C1", 1, batch, 32, 8, 128, context, k or context // 32)


def c2(batch: int = 16, context: int = 131072) -> Config:
    return Config("C2", 2, batch, 32, 8, 128, context, context // 32, append=True)


def c3(k: int = 16384, context: int = 524288) -> Config:
    return Config("C3", 3, 1, 32, 8, 128, context, k)


def c4(batch: int = 64, lo: int = 4096, hi: int = 65536) -> Config:
    return Config("C4", 4, batch, 32, 8, 128, hi, (hi + 15) // 16,
                  page_size=16, mixed_lengths=(lo, hi), k_divisor=16)


def scaled(cfg: Config, **kw) -> Config:
    """A copy of a config with some fields replaced (used for small test cases)."""
    return dataclasses.replace(cfg, **kw)


# --------------------------------------------------------------------------
# generated layer
# --------------------------------------------------------------------------
@dataclasses.dataclass
class Layer:
    cfg: Config
    q: np.ndarray                    # [B,Hq,d] bf16 bits
    k: np.ndarray                    # contiguous [B,Hkv,Nmax,d] | paged [P,Hkv,page,d]  (bf16 bits)
    v: np.ndarray
    seq_lens: np.ndarray             # [B] int32 (length *before* any append)
    k_per_seq: np.ndarray            # [B] int32
    n_max: int                       # row capacity per sequence (contiguous) or pages*page_size
    w_q: Optional[List[np.ndarray]]  # per layer [Hq,in,out] fp32
    w_kv: Optional[List[np.ndarray]] # per layer [Hkv,in,out] fp32
    k_codes: Optional[np.ndarray]    # only when cfg.mlp_dims is None: same layout as k minus d (uint32)
    q_codes: Optional[np.ndarray]    # only when cfg.mlp_dims is None: [B,Hq] uint32
    page_table: Optional[np.ndarray] # [B,max_pages] int32
    k_new: Optional[np.ndarray]      # [B,Hkv,d] bf16 bits (append configs)
    v_new: Optional[np.ndarray]
    planted_pos: Optional[np.ndarray]  # [B,Hq,planted] int32 logical positions

    @property
    def max_pages_per_seq(self) -> int:
        return 0 if self.page_table is None else int(self.page_table.shape[1])


def _rngs(cfg: Config, seed: Optional[int]):
    ss = np.random.SeedSequence(BASE_SEED + cfg.index if seed is None else seed)
    kids = ss.spawn(len(_STREAMS))
    return {name: np.random.Generator(np.random.PCG64(kid))
            for name, kid in zip(_STREAMS, kids)}


def _normal_bf16(rng, shape) -> np.ndarray:
    return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))


def mapping_weights(rng, n_heads: int, dims) -> List[np.ndarray]:
    """Random-init mapping MLP: layer l is [n_heads, dims[l], dims[l+1]] fp32,
    U(-1/sqrt(fan_in), 1/sqrt(fan_in)), applied as y = x @ W."""
    out = []
    for l in range(len(dims) - 1):
        bound = 1.0 / math.sqrt(dims[l])
        out.append(rng.uniform(-bound, bound,
                               size=(n_heads, dims[l], dims[l + 1])).astype(np.float32))
    return out


def shared_projection_weights(rng, n_q_heads: int, n_kv_heads: int, d: int = 128, bits: int = 32):
    """One-layer mappings that share a Gaussian projection between a KV head and the query heads of its
    group: sign random projections, the locality-sensitive hash of the angle (used by the recall
    harness as a mapping whose quality is known without training).  Returns (w_q, w_kv)."""
    w_kv = rng.standard_normal((n_kv_heads, d, bits)).astype(np.float32)
    w_q = np.repeat(w_kv, n_q_heads // n_kv_heads, axis=0)
    return [np.ascontiguousarray(w_q)], [w_kv]


def draw_lengths(rng, batch: int, lo: int, hi: int) -> np.ndarray:
    """Context lengths log-uniform in [lo, hi]."""
    u = rng.uniform(math.log(lo), math.log(hi), size=batch)
    return np.clip(np.floor(np.exp(u)), lo, hi).astype(np.int32)


def make_layer(cfg: Config, seed: Optional[int] = None) -> Layer:
    """Draw all inputs of one decode layer-step for `cfg`."""
    r = _rngs(cfg, seed)
    B, Hq, Hkv, d = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim

    if cfg.mixed_lengths is not None:
        seq_lens = draw_lengths(r["lengths"], B, *cfg.mixed_lengths)
    else:
        seq_lens = np.full(B, cfg.context, dtype=np.int32)
    if cfg.append:
        seq_lens = seq_lens - 1      # cache holds N-1 rows; the step appends the N-th
    final_lens = seq_lens + (1 if cfg.append else 0)
    if cfg.k_divisor > 0:
        k_per_seq = ((final_lens + cfg.k_divisor - 1) // cfg.k_divisor).astype(np.int32)
    else:
        k_per_seq = np.full(B, cfg.k, dtype=np.int32)

    q = _normal_bf16(r["q"], (B, Hq, d))

    page_table = None
    if cfg.page_size > 0:
        ps = cfg.page_size
        pages_per_seq = (final_lens + ps - 1) // ps
        max_pages = int(pages_per_seq.max())
        total_pages = int(pages_per_seq.sum())
        perm = r["page_table"].permutation(total_pages).astype(np.int32)
        page_table = np.full((B, max_pages), -1, dtype=np.int32)
        off = 0
        for b in range(B):
            n = int(pages_per_seq[b])
            page_table[b, :n] = perm[off:off + n]
            off += n
        k = _normal_bf16(r["k"], (total_pages, Hkv, ps, d))
        v = _normal_bf16(r["v"], (total_pages, Hkv, ps, d))
        n_max = max_pages * ps
    else:
        n_max = int(final_lens.max())
        k = _normal_bf16(r["k"], (B, Hkv, n_max, d))
        v = _normal_bf16(r["v"], (B, Hkv, n_max, d))

    # planted pivotal tokens: key row = 4 q/|q| + N(0, 0.1^2) noise, per query head,
    # positions disjoint inside a KV head, V rows untouched
    planted_pos = None
    if cfg.planted > 0:
        g = cfg.group
        planted_pos = np.zeros((B, Hq, cfg.planted), dtype=np.int32)
        qf = bf16_bits_to_f32(q)
        for b in range(B):
            n_b = int(seq_lens[b])
            per_kv = min(cfg.planted * g, n_b)
            for hk in range(Hkv):
                pos = r["plant_pos"].choice(n_b, size=per_kv, replace=False).astype(np.int32)
                for j in range(g):
                    hq = hk * g + j
                    mine = pos[j * cfg.planted:(j + 1) * cfg.planted]
                    planted_pos[b, hq, :len(mine)] = mine
                    if len(mine) < cfg.planted:
                        planted_pos[b, hq, len(mine):] = -1
                    if len(mine) == 0:
                        continue
                    qv = qf[b, hq]
                    base = 4.0 * qv / max(float(np.linalg.norm(qv)), 1e-12)
                    noise = r["plant_noise"].standard_normal((len(mine), d), dtype=np.float32) * 0.1
                    rows = f32_to_bf16_bits((base[None, :] + noise).astype(np.float32))
                    if page_table is None:
                        k[b, hk, mine] = rows
                    else:
                        ps = cfg.page_size
                        k[page_table[b, mine // ps], hk, mine % ps] = rows

    w_q = w_kv = k_codes = q_codes = None
    if cfg.mlp_dims is not None:
        w_q = mapping_weights(r["w_q"], Hq, cfg.mlp_dims)
        w_kv = mapping_weights(r["w_kv"], Hkv, cfg.mlp_dims)
    else:
        k_codes = r["codes"].integers(0, 2 ** 32, size=k.shape[:-1], dtype=np.uint64).astype(np.uint32)
        q_codes = r["codes"].integers(0, 2 ** 32, size=(B, Hq), dtype=np.uint64).astype(np.uint32)

    k_new = v_new = None
    if cfg.append:
        k_new = _normal_bf16(r["k_new"], (B, Hkv, d))
        v_new = _normal_bf16(r["v_new"], (B, Hkv, d))

    return Layer(cfg, q, k, v, seq_lens.astype(np.int32), k_per_seq, n_max, w_q, w_kv,
                 k_codes, q_codes, page_table, k_new, v_new, planted_pos)


# --------------------------------------------------------------------------
# the same recipe drawn on the device (large configurations: drawing GiB of normals with numpy
# would take minutes).  Inputs only: a seeded torch generator, no arithmetic of the method.
# --------------------------------------------------------------------------
def device_tensors(cfg: Config, seed: int, device: str = "cuda:0", extra_rows: int = 0) -> dict:
    """K, V, Q ~ N(0,1) in bf16, planted keys 4 q/|q| + 0.1 N(0,1), U(-1/sqrt(fan_in), 1/sqrt(fan_in))
    fp32 weights, as torch tensors on `device`.  Contiguous or paged layout as cfg says; for append
    configs the cache holds N-1 rows and k_new/v_new carry the N-th."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    B, Hq, Hkv, d = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    grp = Hq // Hkv
    host_rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence(seed)))
    if cfg.mixed_lengths is not None:
        final_lens = draw_lengths(host_rng, B, *cfg.mixed_lengths)
    else:
        final_lens = np.full(B, cfg.context, dtype=np.int32)
    seq_lens = final_lens - (1 if cfg.append else 0)
    if cfg.k_divisor > 0:
        k_per_seq = ((final_lens + cfg.k_divisor - 1) // cfg.k_divisor).astype(np.int32)
    else:
        k_per_seq = np.full(B, cfg.k, dtype=np.int32)

    def normal_bf16(shape):
        return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)

    q = normal_bf16((B, Hq, d))
    page_table = None
    if cfg.page_size > 0:
        ps = cfg.page_size
        pages_per_seq = (final_lens + ps - 1) // ps
        max_pages, total_pages = int(pages_per_seq.max()), int(pages_per_seq.sum())
        perm = host_rng.permutation(total_pages).astype(np.int32)
        table = np.full((B, max_pages), -1, dtype=np.int32)
        off = 0
        for b in range(B):
            table[b, :pages_per_seq[b]] = perm[off:off + pages_per_seq[b]]
            off += int(pages_per_seq[b])
        page_table = torch.from_numpy(table).to(device)
        k = torch.empty((total_pages, Hkv, ps, d), device=device, dtype=torch.bfloat16)
        v = torch.empty_like(k)
        step = 4096
        for t in (k, v):
            for p0 in range(0, total_pages, step):
                p1 = min(total_pages, p0 + step)
                t[p0:p1] = normal_bf16((p1 - p0, Hkv, ps, d))
        n_max = max_pages * ps
    else:
        n_max = int(final_lens.max()) + extra_rows
        n_max += (-n_max) % 4
        k = torch.empty((B, Hkv, n_max, d), device=device, dtype=torch.bfloat16)
        v = torch.empty_like(k)
        for t in (k, v):
            for b in range(B):
                for h in range(Hkv):
                    t[b, h] = normal_bf16((n_max, d))
    if cfg.planted > 0:
        for b in range(B):
            n_b = int(seq_lens[b])
            per_kv = min(cfg.planted * grp, n_b)
            for hk in range(Hkv):
                pos = torch.randperm(n_b, generator=g, device=device)[:per_kv]
                for j in range(grp):
                    mine = pos[j * cfg.planted:(j + 1) * cfg.planted]
                    if mine.numel() == 0:
                        continue
                    qv = q[b, hk * grp + j].float()
                    rows = 4.0 * qv / qv.norm() + 0.1 * torch.randn((mine.numel(), d), generator=g, device=device)
                    if page_table is None:
                        k[b, hk, mine] = rows.to(torch.bfloat16)
                    else:
                        k[page_table[b, mine // cfg.page_size].long(), hk, mine % cfg.page_size] = rows.to(torch.bfloat16)

    def weights(n_heads):
        out = []
        for l in range(len(cfg.mlp_dims) - 1):
            bound = 1.0 / math.sqrt(cfg.mlp_dims[l])
            w = (torch.rand((n_heads, cfg.mlp_dims[l], cfg.mlp_dims[l + 1]), generator=g, device=device) * 2 - 1) * bound
            out.append(w.contiguous())
        return out

    out = dict(q=q, k=k, v=v, seq_lens_host=seq_lens.astype(np.int32), k_per_seq_host=k_per_seq,
               seq_lens=torch.from_numpy(seq_lens.astype(np.int32)).to(device),
               k_per_seq=torch.from_numpy(k_per_seq).to(device), page_table=page_table, n_max=n_max,
               w_q=weights(Hq), w_kv=weights(Hkv), k_new=None, v_new=None)
    if cfg.append:
        out["k_new"] = normal_bf16((B, Hkv, 1, d))
        out["v_new"] = normal_bf16((B, Hkv, 1, d))
    return out


# --------------------------------------------------------------------------
# byte accounting used by the benchmark report (sizes only, no arithmetic of
# the method): key codes + gathered K/V rows + Q and O
# --------------------------------------------------------------------------
def algorithmic_bytes(n_kv_heads: int, n_q_heads: int, head_dim: int,
                      seq_lens, k_per_seq) -> int:
    total = 0
    for n, k in zip(seq_lens, k_per_seq):
        kk = min(int(k), int(n))
        total += 4 * n_kv_heads * int(n)                 # uint32 key codes
        total += n_q_heads * kk * 2 * head_dim * 2       # gathered K and V rows (bf16)
        total += 2 * n_q_heads * head_dim * 2            # Q read + O write (bf16)
    return total


def gathered_bytes(n_q_heads: int, head_dim: int, seq_lens, k_per_seq) -> int:
    """Bytes the GATHER-ATT kernel must move: selected K/V rows + Q + O."""
    total = 0
    for n, k in zip(seq_lens, k_per_seq):
        kk = min(int(k), int(n))
        total += n_q_heads * kk * 2 * head_dim * 2 + 2 * n_q_heads * head_dim * 2
    return total


def kv_cache_bytes_per_token(n_layers: int, n_kv_heads: int, head_dim: int) -> int:
    """bf16 K and V rows of one token over all layers."""
    return n_layers * n_kv_heads * head_dim * 2 * 2
