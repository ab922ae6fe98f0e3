"""Seeded synthetic VAR / Infinity-shaped workloads (inputs only).

This module produces the *inputs* of the hot path -- per-scale Q/K/V tensors,
head-type masks and integer budgets -- for both the HIP library and the CPU
oracle.  It contains none of the method's arithmetic (no softmax, no top-k,
no gather): it is a data recipe.

Shapes follow next-scale prediction (paper, Preliminaries): step k emits
N_k = side_k^2 tokens and the uncompressed cache length is T_k = sum_{i<=k} N_i.
Value structure stands in for the two head classes of the paper (Introduction;
Sec. 4.1 Observation 1):
  * contextual heads attend to a few sink keys  -> vertical pattern,
  * structural heads attend to spatially aligned keys of every scale
    -> multi-diagonal pattern.
Budgets follow Sec. 4.3 (B = alpha*B_C + (1-alpha)*B_S) and the supplementary
implementation details (rho = 1 - B/T_K; B_C : B_S = 1 : 2 for the 1024^2
models; B_C given as a fraction of T_K for the 256^2 model).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Sequence

import numpy as np

SEED_BASE = 250409261
NO_COMPRESSION = 1 << 30  # budget value meaning "never compress this unit"

SIDES_10 = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)                    # 680 tokens
SIDES_13 = (1, 2, 4, 6, 8, 12, 16, 20, 24, 32, 40, 48, 64)      # 10521 tokens

CONTEXTUAL = 0
STRUCTURAL = 1


@dataclass(frozen=True)
class Config:
    """One workload family (a row of the benchmark's `configs`)."""
    cfg_id: int
    name: str
    heads: int
    head_dim: int
    batch: int
    dtype: str                      # "f32" | "bf16"
    sides: Sequence[int]
    layers: int
    r_C: float                      # contextual budget as a fraction of T_K
    r_S: float                      # structural budget as a fraction of T_K
    head_rule: str                  # "first_half" | "bernoulli" | "count"
    n_contextual: int = 0           # used by head_rule == "count"
    gate_step: int = 4              # compression allowed from this 1-based step
    n_obs: int = 32                 # observation queries (suppl., Compression Setting)
    n_init_scales: int = 2          # structural heads always keep the first two scales
    sinks_lo: int = 12              # sink keys per contextual head (inclusive range)
    sinks_hi: int = 12
    budget_jitter: float = 0.0      # +-fraction applied per (layer, head)
    sink_gain_k: float = 3.0
    sink_gain_q: float = 1.0
    pos_gain: float = 2.0

    @property
    def N(self) -> List[int]:
        return [s * s for s in self.sides]

    @property
    def T(self) -> List[int]:
        return list(np.cumsum(self.N))

    @property
    def T_K(self) -> int:
        return int(sum(self.N))

    @property
    def n_steps(self) -> int:
        return len(self.sides)

    @property
    def n_units(self) -> int:
        return self.batch * self.heads

    @property
    def n_init(self) -> int:
        return int(sum(self.N[: self.n_init_scales]))

    @property
    def scale(self) -> float:
        # exactly the float32 the library receives, so both sides scale alike
        return float(np.float32(1.0 / math.sqrt(self.head_dim)))

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2


def _split_ratios(keep: float, alpha: float):
    """1:2 split with mean `keep`: keep = alpha*r_C + (1-alpha)*2*r_C."""
    r_C = keep / (alpha + 2.0 * (1.0 - alpha))
    return r_C, min(1.0, 2.0 * r_C)


def get_config(cfg_id: int, *, keep: float = 0.3, ctx_frac: float = 0.5,
               batch: Optional[int] = None) -> Config:
    """The five benchmark workload families."""
    if cfg_id == 0:
        c = Config(0, "cfg0-var-f32-1layer", 16, 64, 1, "f32", SIDES_10, 1,
                   0.15, 0.45, "first_half")
    elif cfg_id == 1:
        c = Config(1, "cfg1-var-d30", 30, 64, 32, "bf16", SIDES_10, 30,
                   0.15, 0.45, "bernoulli")
    elif cfg_id == 2:
        # keep = retained fraction of the cache, averaged over heads (compression ratio rho = 1 - keep);
        # the benchmark workload is rho = 70 %, other ratios give the other points of a latency-vs-rho curve
        r_C, r_S = _split_ratios(keep, 6.0 / 16.0)
        name = "cfg2-infinity-2b-1024" if keep == 0.3 else f"cfg2-infinity-2b-1024-keep{keep:g}"
        c = Config(2, name, 16, 128, 2, "bf16", SIDES_13, 32,
                   r_C, r_S, "count", n_contextual=6)
    elif cfg_id == 3:
        c = Config(3, "cfg3-8b-1024", 32, 128, 2, "bf16", SIDES_13, 40,
                   0.15, 0.45, "count", n_contextual=16)
    elif cfg_id == 4:
        n_c = int(round(ctx_frac * 16))
        r_C, r_S = _split_ratios(keep, n_c / 16.0)
        c = Config(4, f"cfg4-ragged-keep{keep:g}-ctx{ctx_frac:g}", 16, 128, 8, "bf16",
                   SIDES_13, 32, r_C, r_S, "count", n_contextual=n_c,
                   sinks_lo=4, sinks_hi=64, budget_jitter=0.2)
    else:
        raise ValueError(f"unknown config {cfg_id}")
    if batch is not None:
        c = replace(c, batch=batch)
    return c


# --------------------------------------------------------------------------
# random streams
# --------------------------------------------------------------------------
_TENSOR_ID = {"Q": 1, "K": 2, "V": 3, "heads": 4, "sinks": 5, "budget": 6}


def _rng(cfg: Config, layer: int, what: str, step: int = 0) -> np.random.Generator:
    seed = SEED_BASE + 1000 * cfg.cfg_id + layer
    ss = np.random.SeedSequence([seed, _TENSOR_ID[what], step])
    return np.random.Generator(np.random.Philox(ss))


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bfloat16 (ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# head classes and budgets
# --------------------------------------------------------------------------
def head_types(cfg: Config, layer: int) -> np.ndarray:
    """uint8[H]: 0 = contextual, 1 = structural."""
    H = cfg.heads
    if cfg.head_rule == "first_half":
        t = np.ones(H, np.uint8)
        t[: H // 2] = CONTEXTUAL
    elif cfg.head_rule == "bernoulli":
        t = (_rng(cfg, layer, "heads").random(H) >= 0.5).astype(np.uint8)
    elif cfg.head_rule == "count":
        t = np.ones(H, np.uint8)
        ctx = _rng(cfg, layer, "heads").permutation(H)[: cfg.n_contextual]
        t[ctx] = CONTEXTUAL
    else:
        raise ValueError(cfg.head_rule)
    return t


def head_budgets(cfg: Config, layer: int) -> np.ndarray:
    """int32[H]: B_p of each head, fixed over the schedule (B_p = ceil(r_p * T_K))."""
    t = head_types(cfg, layer)
    r = np.where(t == CONTEXTUAL, cfg.r_C, cfg.r_S).astype(np.float64)
    if cfg.budget_jitter > 0:
        j = _rng(cfg, layer, "budget").uniform(1 - cfg.budget_jitter, 1 + cfg.budget_jitter, cfg.heads)
        r = r * j
    b = np.ceil(r * cfg.T_K - 1e-9).astype(np.int64)
    b = np.clip(b, cfg.n_init + 1, cfg.T_K)
    return b.astype(np.int32)


def step_budgets(cfg: Config, layer: int, k: int) -> np.ndarray:
    """int32[B*H] budgets handed to the library at 1-based step k.

    Before the gate step no unit may compress; the library reads any budget
    >= T_in as "leave this unit alone".
    """
    if k < cfg.gate_step:
        return np.full(cfg.n_units, NO_COMPRESSION, np.int32)
    return np.tile(head_budgets(cfg, layer), cfg.batch).astype(np.int32)


def planned_lengths(cfg: Config, layer: int):
    """Host arithmetic only: per step, per unit (L_before, T_in, len_out).

    len_out = min(budget, T_in); this mirrors the trigger "compress when the
    cache exceeds its budget" (Sec. 4.3) and is what lets every launch shape be
    computed without reading device memory.
    """
    U = cfg.n_units
    L = np.zeros(U, np.int64)
    out = []
    for k in range(1, cfg.n_steps + 1):
        Nk = cfg.N[k - 1]
        t_in = L + Nk
        b = step_budgets(cfg, layer, k).astype(np.int64)
        len_out = np.minimum(b, t_in)
        out.append((L.copy(), t_in.copy(), len_out.copy()))
        L = len_out
    return out


# --------------------------------------------------------------------------
# tensors
# --------------------------------------------------------------------------
def positional_code(side: int) -> np.ndarray:
    """float32[side*side, 64]: 16 frequencies x (sin,cos) x (row,col) of the
    token's normalised grid position; identical for aligned positions of
    different scales, which is what makes structural heads multi-diagonal."""
    r, c = np.divmod(np.arange(side * side), side)
    x = (r / side).astype(np.float64)[:, None]
    y = (c / side).astype(np.float64)[:, None]
    w = (np.pi * (np.arange(16) + 1.0))[None, :]
    e = np.empty((side * side, 16, 4), np.float64)
    e[:, :, 0] = np.sin(w * x)
    e[:, :, 1] = np.cos(w * x)
    e[:, :, 2] = np.sin(w * y)
    e[:, :, 3] = np.cos(w * y)
    return e.reshape(side * side, 64).astype(np.float32)


def sink_plan(cfg: Config, layer: int):
    """Per head: (unit direction u float32[d], sorted global sink token ids)."""
    rng = _rng(cfg, layer, "sinks")
    plan = []
    for _ in range(cfg.heads):
        u = rng.standard_normal(cfg.head_dim)
        u = (u / np.linalg.norm(u)).astype(np.float32)
        s = int(rng.integers(cfg.sinks_lo, cfg.sinks_hi + 1))
        ids = np.sort(rng.choice(cfg.T_K, size=s, replace=False))
        plan.append((u, ids))
    return plan


@dataclass
class StepTensors:
    """Inputs of one scale step, as the library receives them.

    q, k, v: float32 [B, H, N_k, d] holding exactly the values the device sees
    (for bf16 configs they are already rounded, so the oracle and the GPU read
    identical numbers); *_bits are the uint16 bfloat16 encodings (None for f32).
    """
    k_index: int
    N_k: int
    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    q_bits: Optional[np.ndarray] = None
    k_bits: Optional[np.ndarray] = None
    v_bits: Optional[np.ndarray] = None


def gen_step(cfg: Config, layer: int, k: int, types: Optional[np.ndarray] = None,
             sinks=None) -> StepTensors:
    """Generate Q_k, K_k, V_k of 1-based step k."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    side = cfg.sides[k - 1]
    Nk = side * side
    t0 = int(sum(cfg.N[: k - 1]))            # global id of the first token of this scale
    types = head_types(cfg, layer) if types is None else types
    sinks = sink_plan(cfg, layer) if sinks is None else sinks
    shape = (B, H, Nk, d)
    q = _rng(cfg, layer, "Q", k).standard_normal(shape, dtype=np.float32)
    kk = _rng(cfg, layer, "K", k).standard_normal(shape, dtype=np.float32)
    v = _rng(cfg, layer, "V", k).standard_normal(shape, dtype=np.float32)
    e = positional_code(side) * np.float32(cfg.pos_gain)
    for h in range(H):
        if types[h] == CONTEXTUAL:
            u, ids = sinks[h]
            q[:, h] += np.float32(cfg.sink_gain_q) * u
            loc = ids[(ids >= t0) & (ids < t0 + Nk)] - t0
            if loc.size:
                kk[:, h, loc] += np.float32(cfg.sink_gain_k) * u
        else:
            q[:, h, :, :64] += e
            kk[:, h, :, :64] += e
    if cfg.dtype == "bf16":
        qb, kb, vb = bf16_round(q), bf16_round(kk), bf16_round(v)
        return StepTensors(k, Nk, bf16_to_f32(qb), bf16_to_f32(kb), bf16_to_f32(vb), qb, kb, vb)
    return StepTensors(k, Nk, q, kk, v)


def gen_layer(cfg: Config, layer: int, steps: Optional[Sequence[int]] = None) -> Dict[int, StepTensors]:
    types = head_types(cfg, layer)
    sinks = sink_plan(cfg, layer)
    ks = range(1, cfg.n_steps + 1) if steps is None else steps
    return {k: gen_step(cfg, layer, k, types, sinks) for k in ks}


# --------------------------------------------------------------------------
# algorithmic work model (what the method itself has to move / compute)
# --------------------------------------------------------------------------
def work_model(cfg: Config, layer: int = 0):
    """Per step: algorithmic flop / bytes of each stage, from the planned lengths.

    attend : 4*N_k*b*d flop, (2*N_k*d + 2*b*d)*e bytes        per unit
    score  : 2*n_obs*T_in*d flop, (T_in*d + n_obs*d)*e + 4*T_in bytes (compressing units)
    select : 4*T_in + 4*b bytes
    compact: 2*(2*b*d*e) bytes
    append : 4*N_k*d*e bytes (units that do not compress)
    """
    d, e = cfg.head_dim, cfg.elem_bytes
    rows = []
    for k, (L, t_in, len_out) in enumerate(planned_lengths(cfg, layer), start=1):
        Nk = cfg.N[k - 1]
        comp = len_out < t_in
        n_obs = min(cfg.n_obs, Nk)
        rows.append(dict(
            k=k, N_k=Nk, n_compress=int(comp.sum()),
            attn_flop=float((4.0 * Nk * len_out * d).sum()),
            attn_bytes=float(((2.0 * Nk * d + 2.0 * len_out * d) * e).sum()),
            score_flop=float((2.0 * n_obs * t_in[comp] * d).sum()),
            score_bytes=float(((t_in[comp] * d + n_obs * d) * e + 4.0 * t_in[comp]).sum()),
            select_bytes=float((4.0 * t_in[comp] + 4.0 * len_out[comp]).sum()),
            compact_bytes=float((4.0 * len_out[comp] * d * e).sum()),
            append_bytes=float((4.0 * Nk * d * e) * int((~comp).sum())),
            full_attn_flop=float(4.0 * Nk * cfg.T[k - 1] * d * cfg.n_units),
        ))
    return rows
