"""The oracle-side schedule checker (oracle/parity.py) on the CPU: a stand-in for the device is
played by the oracle's own primitives, once faithfully, once taking the other row of an exact tie
(must be excused, re-seeded and then followed), once taking a clearly worse row (must be flagged)."""
import numpy as np

from oracle import hack_oracle as ho
from oracle.parity import ScheduleChecker, kept_set_verdict, ranked_segment


def _schedule(seed=3, H=2, d=16, sizes=(4, 9, 16, 25)):
    rng = np.random.default_rng(seed)
    steps = []
    for n in sizes:
        q, k, v = (rng.standard_normal((1, H, n, d)) for _ in range(3))
        steps.append([q, k, v])
    # rows 1 and 2 of the second scale of head 0 are the same key: an exact tie in importance
    steps[1][1][0, 0, 2] = steps[1][1][0, 0, 1]
    return steps


def _play_device(steps, types, budgets, n_init, scale, n_obs, tamper=None):
    """Walks the schedule with oracle primitives; tamper(step, unit, I, imp) may return another kept set."""
    H = steps[0][0].shape[1]
    d = steps[0][0].shape[3]
    state = {u: (np.zeros((0, d)), np.zeros((0, d)), np.zeros(0, np.int64)) for u in range(H)}
    pos0, out = 0, []
    for s, (Q, K, V) in enumerate(steps):
        N_k = Q.shape[2]
        res = {}
        for u in range(H):
            Kc, Vc, Pc = state[u]
            r = ho.unit_step(Kc, Vc, Pc, Q[0, u], K[0, u], V[0, u], pos0, int(types[u]), int(budgets[s][u]), n_init, scale, n_obs)
            if r["compressed"] and tamper is not None:
                I2 = tamper(s, u, r["I"], r["imp"])
                if I2 is not None:
                    K_in, V_in = np.concatenate([Kc, K[0, u]]), np.concatenate([Vc, V[0, u]])
                    P_in = np.concatenate([Pc, pos0 + np.arange(N_k)])
                    K2, V2 = ho.compact(K_in, V_in, I2)
                    r = dict(r, I=I2, K=K2, V=V2, pos=P_in[I2], O=ho.attention(Q[0, u], K2, V2, scale))
            state[u] = (r["K"], r["V"], r["pos"])
            res[u] = dict(I=r["I"], pos=r["pos"], O=r["O"])
        out.append(res)
        pos0 += N_k
    return out, state


def _check(steps, types, budgets, n_init, scale, n_obs, device):
    chk = ScheduleChecker(len(types), steps[0][0].shape[3], types, n_init, scale, n_obs, range(len(types)), 1e-9)
    for s, (Q, K, V) in enumerate(steps):
        chk.step(Q, K, V, budgets[s], device[s])
    return chk


def test_checker_exact_excused_and_mismatch():
    steps = _schedule()
    types = np.array([0, 1], np.uint8)
    n_init, scale, n_obs = 5, 0.25, 8
    budgets = [np.array([1 << 30, 1 << 30]), np.array([7, 1 << 30]), np.array([9, 24]), np.array([12, 40])]
    device, state = _play_device(steps, types, budgets, n_init, scale, n_obs)
    chk = _check(steps, types, budgets, n_init, scale, n_obs, device)
    st = chk.summary()
    assert not chk.failures and st["mismatch"] == 0 and st["excused"] == 0 and st["exact"] == st["compress_events"] == 5
    for u in range(2):
        assert np.array_equal(chk.final_cache(u)[0], state[u][0])

    # the tied pair sits at cache rows 5 and 6 (scale 2 starts at row 4) of unit 0 at step 2: make the pair
    # straddle the cut by choosing the budget, then let the stand-in device take the higher index instead
    seen = {}

    def other_of_tie(s, u, I, imp):
        if s == 1 and u == 0:
            seen["imp"] = imp
            if 5 in I and 6 not in I:
                return np.sort(np.concatenate([I[I != 5], [6]]))
        return None

    for b in range(3, 12):
        budgets[1] = np.array([b, 1 << 30])
        seen.clear()
        device, state = _play_device(steps, types, budgets, n_init, scale, n_obs, tamper=other_of_tie)
        if not np.array_equal(device[1][0]["I"], ho.select(seen["imp"], 0, b, n_init, 9)):
            break
    else:
        raise AssertionError("no budget put the tied rows on the cut")
    assert seen["imp"][5] == seen["imp"][6]
    chk = _check(steps, types, budgets, n_init, scale, n_obs, device)
    st = chk.summary()
    assert not chk.failures, chk.failures
    assert st["excused"] == 1 and st["reseeded"] == 1 and st["mismatch"] == 0
    assert np.array_equal(chk.final_cache(0)[2], state[0][2])      # the checker followed the device's choice

    # a swap that is no tie: drop the best ranked row for the worst one
    def worse(s, u, I, imp):
        if s == 2 and u == 0:
            rest = np.setdiff1d(np.arange(imp.shape[0]), I)
            best, worst = I[np.argmax(imp[I])], rest[np.argmin(imp[rest])]
            return np.sort(np.concatenate([I[I != best], [worst]]))
        return None

    device, _ = _play_device(steps, types, budgets, n_init, scale, n_obs, tamper=worse)
    chk = _check(steps, types, budgets, n_init, scale, n_obs, device)
    # flagged at the step where it happens (the steps after it differ as a consequence)
    assert chk.summary()["mismatch"] >= 1 and chk.failures[0] == ("kept set", 3, 0)


def test_verdict_rules():
    imp = np.array([5.0, 1.0, 1.0 + 5e-7, 0.2, 3.0])
    lo, hi, m = ranked_segment(ho.CONTEXTUAL, 5, 3, 5, 2)
    assert (lo, hi, m) == (0, 5, 3)
    I_ref = ho.select(imp, ho.CONTEXTUAL, 3, 5, 2)
    assert list(I_ref) == [0, 2, 4]
    assert kept_set_verdict(np.array([0, 2, 4]), I_ref, imp, lo, hi, m) == "exact"
    assert kept_set_verdict(np.array([0, 1, 4]), I_ref, imp, lo, hi, m) == "excused"      # 5e-7 apart
    assert kept_set_verdict(np.array([0, 3, 4]), I_ref, imp, lo, hi, m) == "mismatch"
    assert kept_set_verdict(np.array([0, 4, 2]), I_ref, imp, lo, hi, m) == "mismatch"     # not ascending
    assert ranked_segment(ho.STRUCTURAL, 100, 40, 5, 20) == (5, 80, 15)
    assert ranked_segment(ho.STRUCTURAL, 100, 22, 5, 20) == (80, 100, 17)
