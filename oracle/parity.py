"""Step-by-step comparison of a device run with the CPU oracle (test infrastructure).

TEST INFRASTRUCTURE ONLY, like hack_oracle.py: used by tests/, the smoke check
and the benchmark's cpu_baseline leg.  It never calls the HIP library; the
caller hands it what the device produced as numpy arrays.

The checker walks one layer's scale schedule for a sample of units.  At every
step it advances the oracle (hack_oracle.unit_step) from the oracle's own cache
state and compares what the device produced for the same step:

  kept indices   bit-exact, except near-ties: a device set that differs from the
                 oracle's is "excused" only if every index in the symmetric
                 difference has oracle importance within 1e-6 relative of the
                 oracle's threshold value (the m-th largest of the ranked
                 segment); anything else is a "mismatch";
  token ids      of the retained rows, bit-exact;
  attention out  max |O_device - O_oracle| against the tolerance.

After an excused difference the two caches differ by a near-tied row, and both
are valid results of the method.  So that the unit stays under test, the
oracle's state for that unit is then re-seeded with the DEVICE's kept set:
K^ = K[I_device], V^ = V[I_device] formed by the oracle's own gather from the
oracle's own concatenated cache, and the attention of that step recomputed over
it.  Nothing else ever flows from the device into the oracle, and every
re-seed is counted.
"""
from __future__ import annotations

import numpy as np

from . import hack_oracle as ho

NEAR_TIE = 1e-6


def ranked_segment(head_type: int, T: int, b: int, n_init: int, N_k: int):
    """(sel_lo, sel_hi, m): the rows that are ranked by importance and how many of
    them are kept (Sec. 4.4: all rows for a contextual head; the intermediate rows
    for a structural head, or the current scale when the budget is below N_init + N_k)."""
    if head_type == ho.CONTEXTUAL:
        return 0, T, b
    n0 = min(n_init, T - N_k)
    M = b - n0 - N_k
    if M >= 0:
        return n0, T - N_k, M
    return T - N_k, T, b - min(n0, b)


def kept_set_verdict(I_dev: np.ndarray, I_ref: np.ndarray, imp_ref: np.ndarray, sel_lo: int, sel_hi: int, m: int):
    """'exact', 'excused' or 'mismatch' (see the module header)."""
    if np.array_equal(I_dev, I_ref):
        return "exact"
    if len(I_dev) != len(I_ref) or np.any(np.diff(I_dev) <= 0):
        return "mismatch"
    diff = np.setxor1d(I_dev, I_ref)
    if np.any(diff < sel_lo) or np.any(diff >= sel_hi) or m <= 0:
        return "mismatch"
    seg = np.sort(imp_ref[sel_lo:sel_hi])[::-1]
    thr = seg[m - 1]
    ok = np.all(np.abs(imp_ref[diff] - thr) <= NEAR_TIE * abs(thr))
    return "excused" if ok else "mismatch"


class ScheduleChecker:
    """Oracle-side walk of one layer's schedule for `units` (ids u = b*H + h)."""

    def __init__(self, heads: int, head_dim: int, head_types, n_init: int, scale: float, n_obs: int, units, tol: float):
        self.H, self.d = int(heads), int(head_dim)
        self.types = np.asarray(head_types)
        self.n_init, self.scale, self.n_obs, self.tol = int(n_init), float(scale), int(n_obs), float(tol)
        self.units = [int(u) for u in units]
        self.state = {u: (np.zeros((0, head_dim)), np.zeros((0, head_dim)), np.zeros(0, np.int64)) for u in self.units}
        self.pos0 = 0
        self.step_no = 0
        self.stats = dict(units=len(self.units), steps=0, compress_events=0, exact=0, excused=0, mismatch=0,
                          reseeded=0, max_abs_dO=0.0, pos_mismatch=0, out_of_tol=0)
        self.failures = []

    def step(self, Q, K, V, budgets, device, final_merge=False):
        """Q, K, V: host arrays [B, H, N_k, d] of this scale (the values the device received).
        final_merge: this is the last generation step (contextual units merge what they discard).
        budgets: int array [B*H].  device: dict unit -> dict with
          'I'   int array, the device's kept indices (only read when the unit compresses),
          'pos' int array, token ids of the rows the device retains after the step (or None),
          'O'   float array [N_k, d], the device's attention output."""
        self.step_no += 1
        self.stats["steps"] += 1
        N_k = Q.shape[2]
        for u in self.units:
            b, h = divmod(u, self.H)
            Kc, Vc, Pc = self.state[u]
            Qk = np.asarray(Q[b, h], np.float64)
            Kk = np.asarray(K[b, h], np.float64)
            Vk = np.asarray(V[b, h], np.float64)
            t = int(self.types[h])
            r = ho.unit_step(Kc, Vc, Pc, Qk, Kk, Vk, self.pos0, t, int(budgets[u]), self.n_init, self.scale, self.n_obs,
                             final_merge=final_merge)
            dev = device[u]
            if r["compressed"]:
                self.stats["compress_events"] += 1
                T_in = Kc.shape[0] + N_k
                I_dev = np.asarray(dev["I"], np.int64)
                lo, hi, m = ranked_segment(t, T_in, len(r["I"]), self.n_init, N_k)
                verdict = kept_set_verdict(I_dev, r["I"], r["imp"], lo, hi, m)
                self.stats[verdict] += 1
                if verdict == "mismatch":
                    self.failures.append(("kept set", self.step_no, u))
                    # keep walking from the oracle's own state; later differences of this unit are consequences
                elif verdict == "excused":
                    # both sets are valid; continue this unit from the device's choice (oracle arithmetic only)
                    K_in = np.concatenate([Kc, Kk], axis=0)
                    V_in = np.concatenate([Vc, Vk], axis=0)
                    P_in = np.concatenate([Pc, self.pos0 + np.arange(N_k, dtype=np.int64)])
                    if final_merge and t == ho.CONTEXTUAL:
                        K2, V2, _, _ = ho.merge_final(K_in, V_in, I_dev)
                    else:
                        K2, V2 = ho.compact(K_in, V_in, I_dev)
                    r = dict(r, K=K2, V=V2, pos=P_in[I_dev], O=ho.attention(Qk, K2, V2, self.scale), I=I_dev)
                    self.stats["reseeded"] += 1
            self.state[u] = (r["K"], r["V"], r["pos"])
            if dev.get("pos") is not None and not np.array_equal(np.asarray(dev["pos"], np.int64), r["pos"]):
                self.stats["pos_mismatch"] += 1
                self.failures.append(("token ids", self.step_no, u))
            err = float(np.abs(np.asarray(dev["O"], np.float64) - r["O"]).max())
            self.stats["max_abs_dO"] = max(self.stats["max_abs_dO"], err)
            if not err < self.tol:
                self.stats["out_of_tol"] += 1
                self.failures.append(("attention output %.3e" % err, self.step_no, u))
        self.pos0 += N_k

    def final_cache(self, u: int):
        """(K, V, pos) the oracle holds for unit u after the steps walked so far."""
        return self.state[int(u)]

    def summary(self) -> dict:
        s = dict(self.stats)
        s["tolerance"] = self.tol
        s["near_tie_rel"] = NEAR_TIE
        return s
