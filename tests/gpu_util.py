"""Helpers of the GPU parity tests: move a generated layer to the device, run the
HIP path through the C ABI binding, run the oracle on the same arrays."""
from __future__ import annotations

import math

import numpy as np
import torch

import oracle
import paper_2412_14468_amd as ha
import workloads as W

ATOL, RTOL = 2e-3, 1e-2          # attention outputs, bf16 inputs (spec tolerance)
ACT_EPS = 1e-3                   # code bits are compared where |pre-sign activation| > ACT_EPS
DEV = "cuda:0"


def bf16_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)


def u32_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(a.view(np.int32)).to(DEV)


def u32_host(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def bf16_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


class DeviceLayer:
    """Device copy of a workloads.Layer plus the library objects that refer to it."""

    def __init__(self, L: W.Layer, max_k: int | None = None, extra_rows: int = 0):
        cfg = L.cfg
        self.L = L
        self.B, self.Hq, self.Hkv, self.d = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
        self.paged = cfg.page_size > 0
        k_host, v_host = L.k, L.v
        if not self.paged and (k_host.shape[2] + extra_rows) % 4:
            extra_rows += 4 - (k_host.shape[2] + extra_rows) % 4       # capacity must be a multiple of 4
        if extra_rows and not self.paged:
            pad = np.zeros((self.B, self.Hkv, extra_rows, self.d), dtype=np.uint16)
            k_host = np.concatenate([k_host, pad], axis=2)
            v_host = np.concatenate([v_host, pad], axis=2)
        self.k_host, self.v_host = np.ascontiguousarray(k_host), np.ascontiguousarray(v_host)
        self.q = bf16_dev(L.q)
        self.k = bf16_dev(self.k_host)
        self.v = bf16_dev(self.v_host)
        self.codes = torch.zeros(self.k_host.shape[:3], dtype=torch.int32, device=DEV)
        self.seq_lens = torch.from_numpy(L.seq_lens.copy()).to(DEV)
        self.k_per_seq = torch.from_numpy(L.k_per_seq.copy()).to(DEV)
        self.page_table = None if L.page_table is None else torch.from_numpy(L.page_table).to(DEV)
        self.k_max = int(L.k_per_seq.max())
        n_cap = int(self.k_host.shape[2]) if not self.paged else L.max_pages_per_seq * cfg.page_size
        self.cache = ha.KvCache(self.k, self.v, self.codes, self.seq_lens, int(L.seq_lens.max()),
                                page_table=self.page_table)
        self.ctx = ha.Context(self.Hq, self.Hkv, self.B, max(n_cap, 1), max(max_k or self.k_max, 1),
                              page_size=cfg.page_size)
        self.phi_q = self.phi_kv = None
        if L.w_q is not None:
            self.wq_dev = [torch.from_numpy(w).to(DEV) for w in L.w_q]
            self.wkv_dev = [torch.from_numpy(w).to(DEV) for w in L.w_kv]
            self.phi_q = ha.Mlp(self.wq_dev)
            self.phi_kv = ha.Mlp(self.wkv_dev)
        self.scale = 1.0 / math.sqrt(self.d)

    # host-side twin of the cache for the oracle (own copies, so appends do not alias)
    def oracle_cache(self):
        k, v = self.k_host.copy(), self.v_host.copy()
        codes = np.zeros(k.shape[:3], dtype=np.uint32)
        lens = self.L.seq_lens.copy()
        return oracle.Cache(k, v, codes, lens, page_table=self.L.page_table,
                            page_size=self.L.cfg.page_size), codes, lens

    def set_codes(self, codes_host: np.ndarray):
        self.codes.copy_(u32_dev(codes_host))

    def new_outputs(self):
        idx = torch.full((self.B, self.Hq, self.k_max), -7, dtype=torch.int32, device=DEV)
        count = torch.full((self.B, self.Hq), -7, dtype=torch.int32, device=DEV)
        thr = torch.full((self.B, self.Hq), 255, dtype=torch.uint8, device=DEV)
        out = torch.full((self.B, self.Hq, self.d), float("nan"), dtype=torch.bfloat16, device=DEV)
        return idx, count, thr, out


def assert_codes_match(gpu_codes: np.ndarray, ref_codes: np.ndarray, act: np.ndarray, what: str):
    """Bit j must agree wherever |activation_j| > ACT_EPS.  act has a trailing axis of 32."""
    diff = (gpu_codes ^ ref_codes).astype(np.uint32)
    if not diff.any():
        return 0
    bits = ((diff[..., None] >> np.arange(32, dtype=np.uint32)) & 1).astype(bool)
    sure = np.abs(act) > ACT_EPS
    bad = bits & sure
    assert not bad.any(), f"{what}: {int(bad.sum())} code bits differ where |activation| > {ACT_EPS}"
    return int(bits.sum())


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp64 values rounded to the nearest bf16 (ties to even), returned as fp64."""
    return W.bf16_bits_to_f32(W.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))).astype(np.float64)


# The output is bf16, so half a bf16 unit of rounding (up to 2^-9 |ref|, 1.95e-3 at 1.0) sits in every
# comparison with the fp64 oracle.  Against the oracle's value rounded to bf16 only the kernel's own
# error is left: an fp32 result within rounding of the true value rounds to the same bf16 number or,
# when the true value lies next to a rounding boundary, to its neighbour (one unit, at most 2^-7 |ref|);
# OWN_FLOOR covers outputs near zero, where fp32 accumulation error exceeds the tiny bf16 unit.
OWN_RTOL, OWN_FLOOR = 2.0 ** -7, 5e-5


def assert_out_close(gpu_out_bf16: torch.Tensor, ref: np.ndarray, what: str):
    got = bf16_host_f64(gpu_out_bf16)
    err = np.abs(got - ref)
    tol = ATOL + RTOL * np.abs(ref)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    worst = float((err - tol).max())
    assert worst <= 0, f"{what}: max |err| {float(err.max()):.3e} exceeds {ATOL} + {RTOL}|ref| by {worst:.3e}"
    ref16 = round_to_bf16(ref)
    own = np.abs(got - ref16)
    own_tol = OWN_RTOL * np.abs(ref16) + OWN_FLOOR
    worst_own = float((own - own_tol).max())
    assert worst_own <= 0, (f"{what}: kernel's own error (against the oracle rounded to bf16) {float(own.max()):.3e} "
                            f"exceeds one bf16 unit + {OWN_FLOOR} by {worst_own:.3e}")
    return {"max_abs_err": float(err.max()), "max_own_err": float(own.max()),
            "same_bf16_frac": float((own == 0).mean())}
