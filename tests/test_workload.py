"""Host-side checks of the synthetic workload recipe (no GPU, no method arithmetic)."""
import numpy as np
import torch

from paper_2504_09261_amd import workload as wl
from oracle import hack_oracle as ho


def test_schedules_and_budgets():
    c0, c2, c3 = wl.get_config(0), wl.get_config(2), wl.get_config(3)
    assert c0.T_K == 680 and c2.T_K == 10521 and c0.n_init == 5 and c2.n_init == 5
    assert sorted(set(wl.head_budgets(c0, 0))) == [102, 306]
    assert sorted(set(wl.head_budgets(c2, 0))) == [1943, 3885]
    assert sorted(set(wl.head_budgets(c3, 0))) == [1579, 4735]
    t2 = wl.head_types(c2, 3)
    assert t2.sum() == 10 and (t2 == 0).sum() == 6
    # mean budget equals the target keep ratio: B = alpha*B_C + (1-alpha)*B_S
    assert abs(wl.head_budgets(c2, 0).mean() / c2.T_K - 0.3) < 2e-4
    assert abs(wl.head_budgets(c3, 0).mean() / c3.T_K - 0.3) < 2e-4


def test_planned_lengths_table():
    c = wl.get_config(0)
    plan = wl.planned_lengths(c, 0)
    types = np.tile(wl.head_types(c, 0), c.batch)
    ctx, st = np.where(types == 0)[0][0], np.where(types == 1)[0][0]
    assert [int(p[1][ctx]) for p in plan] == [1, 5, 14, 30, 55, 91, 155, 202, 271, 358]
    assert [int(p[2][ctx]) for p in plan] == [1, 5, 14, 30, 55, 91, 102, 102, 102, 102]
    assert [int(p[1][st]) for p in plan] == [1, 5, 14, 30, 55, 91, 155, 255, 424, 562]
    assert [int(p[2][st]) for p in plan] == [1, 5, 14, 30, 55, 91, 155, 255, 306, 306]
    c = wl.get_config(2)
    plan = wl.planned_lengths(c, 0)
    types = np.tile(wl.head_types(c, 0), c.batch)
    ctx, st = np.where(types == 0)[0][0], np.where(types == 1)[0][0]
    assert [int(p[1][ctx]) for p in plan][9:] == [2521, 3543, 4247, 6039]
    assert [int(p[1][st]) for p in plan][9:] == [2521, 4121, 6189, 7981]


def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(0).standard_normal(4096).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -3.0, 65504.0]        # exact ties and plain values
    bits = wl.bf16_round(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    assert np.array_equal(wl.bf16_round(wl.bf16_to_f32(bits)), bits)


def test_generator_is_seeded_and_structured():
    c = wl.get_config(0)
    a, b = wl.gen_step(c, 0, 5), wl.gen_step(c, 0, 5)
    assert np.array_equal(a.q, b.q) and np.array_equal(a.k, b.k) and np.array_equal(a.v, b.v)
    assert a.q.shape == (1, 16, 25, 64) and a.q.dtype == np.float32
    assert not np.array_equal(a.q, wl.gen_step(c, 1, 5).q)
    c1 = wl.get_config(1, batch=2)
    s = wl.gen_step(c1, 0, 3)
    assert s.q_bits.dtype == np.uint16 and np.array_equal(wl.bf16_to_f32(s.q_bits), s.q)
    # aligned positions of two scales share the positional code
    e2, e4 = wl.positional_code(2), wl.positional_code(4)
    assert np.allclose(e2[1], e4[2])          # (0, 1/2) in both grids
    assert np.allclose(e2[3], e4[10])         # (1/2, 1/2)


def test_oracle_lengths_follow_the_plan():
    c = wl.get_config(0)
    layer = wl.gen_layer(c, 0)
    steps = [(layer[k].q, layer[k].k, layer[k].v) for k in range(1, c.n_steps + 1)]
    budgets = [wl.step_budgets(c, 0, k) for k in range(1, c.n_steps + 1)]
    units = [0, 7, 8, 15]
    trace = ho.run_schedule(steps, wl.head_types(c, 0), budgets, c.n_init, c.scale, c.n_obs,
                            units=units, keep_outputs=False)
    plan = wl.planned_lengths(c, 0)
    for k, res in enumerate(trace):
        for u in units:
            assert res[u]["len"] == plan[k][2][u]
            assert res[u]["compressed"] == bool(plan[k][2][u] < plan[k][1][u])
