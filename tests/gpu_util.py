"""Helpers shared by the GPU parity tests (marshalling and comparison only)."""
from __future__ import annotations

import numpy as np
import torch

from oracle import hack_oracle as ho
from paper_2504_09261_amd import workload as wl
from paper_2504_09261_amd.binding import Cache, Hack

DEV = torch.device("cuda", 0)


def to_dev(x_f32: np.ndarray, dtype: str) -> torch.Tensor:
    """float32 host values (already bf16-representable for bf16 configs) -> device tensor."""
    t = torch.from_numpy(np.ascontiguousarray(x_f32, dtype=np.float32))
    if dtype == "bf16":
        tb = t.to(torch.bfloat16)
        assert torch.equal(tb.to(torch.float32), t), "bf16 inputs must be exactly representable"
        t = tb
    return t.to(DEV).contiguous()


def from_dev(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rand_values(rng, shape, dtype: str) -> np.ndarray:
    x = rng.standard_normal(shape).astype(np.float32)
    if dtype == "bf16":
        x = wl.bf16_to_f32(wl.bf16_round(x))
    return x


def aligned_offsets(lens, pad_rows=0):
    """Row offsets (multiples of 8) for ragged units, with optional slack between them."""
    off, r = [], 0
    for n in lens:
        off.append(r)
        r += (int(n) + pad_rows + 7) // 8 * 8
    return np.asarray(off, np.int64), max(r, 8)


def build_cache(rows_per_unit, d, dtype, pad_rows=0, fill=None):
    """rows_per_unit: list of (K [L,d], V [L,d]) float32 arrays -> (Cache, off)."""
    lens = [k.shape[0] for k, _ in rows_per_unit]
    off, total = aligned_offsets(lens, pad_rows)
    K = np.zeros((total, d), np.float32) if fill is None else np.full((total, d), fill, np.float32)
    V = K.copy()
    for (k, v), o, n in zip(rows_per_unit, off, lens):
        K[o:o + n] = k
        V[o:o + n] = v
    return Cache(to_dev(K, dtype), to_dev(V, dtype), off, np.asarray(lens, np.int32)), off


def make_hack(cfg_or_none=None, *, heads=None, head_dim=None, dtype=None, max_units=None, max_cache_len=None,
              max_queries=None, n_obs=32, attention=None) -> Hack:
    """attention: None = the library's own choice between its two bf16 attention kernels per launch;
    "split" / "tile128" = force the key-split (32-query items) or the 128-query-tile kernel for every
    launch of this context (the library reads the override when the context is created)."""
    import os
    saved = os.environ.get("HACK_ATTN_SPLIT_ITEMS")
    if attention is not None:
        os.environ["HACK_ATTN_SPLIT_ITEMS"] = {"split": "2000000000", "tile128": "0"}[attention]
    try:
        if cfg_or_none is not None:
            c = cfg_or_none
            return Hack(c.heads, c.head_dim, c.dtype, c.n_units, c.T_K, max(c.N), c.n_obs)
        return Hack(heads, head_dim, dtype, max_units, max_cache_len, max_queries, n_obs)
    finally:
        if attention is not None:
            if saved is None:
                del os.environ["HACK_ATTN_SPLIT_ITEMS"]
            else:
                os.environ["HACK_ATTN_SPLIT_ITEMS"] = saved


def kept_set_verdict(I_gpu: np.ndarray, I_ref: np.ndarray, imp_ref: np.ndarray, sel_lo: int, sel_hi: int, m: int):
    """'exact', 'excused' (every differing index is a near-tie: oracle importance
    within 1e-6 relative of the oracle's m-th largest of the ranked segment) or 'mismatch'."""
    if np.array_equal(I_gpu, I_ref):
        return "exact"
    if len(I_gpu) != len(I_ref) or np.any(np.diff(I_gpu) <= 0):
        return "mismatch"
    diff = np.setxor1d(I_gpu, I_ref)
    if np.any(diff < sel_lo) or np.any(diff >= sel_hi) or m <= 0:
        return "mismatch"
    seg = np.sort(imp_ref[sel_lo:sel_hi])[::-1]
    thr = seg[m - 1]
    ok = np.all(np.abs(imp_ref[diff] - thr) <= 1e-6 * abs(thr))
    return "excused" if ok else "mismatch"


def ranked_segment(head_type: int, T: int, b: int, n_init: int, N_k: int):
    """(sel_lo, sel_hi, m) of the ranked segment, restated from Sec. 4.4 for the verdict helper."""
    if head_type == ho.CONTEXTUAL:
        return 0, T, b
    n0 = min(n_init, T - N_k)
    M = b - n0 - N_k
    if M >= 0:
        return n0, T - N_k, M
    return T - N_k, T, b - min(n0, b)
