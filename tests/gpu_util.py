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
    """Device tensor -> float64 host array.  Call it on the rows a unit owns (slices of a slab
    that was allocated uninitialised hold arbitrary bit patterns outside those rows)."""
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
    """attention: None = the library's own choice between its bf16 attention kernels per launch;
    "split" / "tile128" = force the key-split (32-query items) or the 128-query-tile kernel (the
    deeper software pipeline, one work item per work-group) for every launch of this context;
    "stream" = that kernel in its streamed form (the launch cut into equal runs of key blocks) for
    every launch; "cut" = that kernel with every single work item cut in two that the library's
    pair model likes, however small the gain; "tile128_plain" = 128-query tiles through the plain one-block pipeline (the
    library reads the overrides when the context is created)."""
    import os
    env = {}
    if attention is not None:
        env["HACK_ATTN_SPLIT_ITEMS"] = {"split": "2000000000", "tile128": "0", "tile128_plain": "0", "stream": "0", "cut": "0"}[attention]
        env["HACK_ATTN_PIPE"] = "0" if attention == "tile128_plain" else "1"
        env["HACK_ATTN_STREAM"] = {"stream": "1", "cut": "4"}.get(attention, "0")
    saved = {k: os.environ.get(k) for k in env}
    os.environ.update(env)
    try:
        if cfg_or_none is not None:
            c = cfg_or_none
            return Hack(c.heads, c.head_dim, c.dtype, c.n_units, c.T_K, max(c.N), c.n_obs)
        return Hack(heads, head_dim, dtype, max_units, max_cache_len, max_queries, n_obs)
    finally:
        for k, v in saved.items():
            if v is None:
                del os.environ[k]
            else:
                os.environ[k] = v


# the verdict rules live with the oracle-side checker (pure numpy)
from oracle.parity import kept_set_verdict, ranked_segment  # noqa: E402,F401
