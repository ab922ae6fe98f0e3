"""Per-kernel GPU-vs-oracle parity through the C ABI (ctypes binding).

Bars: kept-index sets and compaction bit-exact; importance within a few float32
ulp of the fp64 oracle; attention within 2e-2 max-abs (bf16) / 1e-4 (fp32).
"""
import numpy as np
import pytest
import torch

from oracle import hack_oracle as ho
from paper_2504_09261_amd import workload as wl
from paper_2504_09261_amd.binding import Cache, HackError

pytestmark = pytest.mark.gpu


def _u():
    from tests import gpu_util
    return gpu_util


# ---------------------------------------------------------------------------
# a3 compact
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 64)])
def test_compact_bit_exact_two_sources_and_pos(dtype, d):
    u = _u()
    rng = np.random.default_rng(42 + d)
    H, B, Nk = 4, 2, 37
    U = H * B
    lens = [0, 1, 63, 64, 65, 300, 7, 129]
    hk = u.make_hack(heads=H, head_dim=d, dtype=dtype, max_units=U, max_cache_len=512, max_queries=64)
    rows = [(u.rand_values(rng, (n, d), dtype), u.rand_values(rng, (n, d), dtype)) for n in lens]
    cin, off_in = u.build_cache(rows, d, dtype, pad_rows=3)
    pos_in = np.full(cin.rows, -7, np.int32)
    for o, n in zip(off_in, lens):
        pos_in[o:o + n] = 1000 + np.arange(n)
    cin.pos = torch.from_numpy(pos_in).to(u.DEV)
    k_new, v_new = u.rand_values(rng, (B, H, Nk, d), dtype), u.rand_values(rng, (B, H, Nk, d), dtype)
    keep = [min(n + Nk, k) for n, k in zip(lens, [5, 38, 1, 101, 64, 200, 44, 0])]
    idx_stride = 256
    idx = np.zeros((U, idx_stride), np.int32)
    sel = []
    for uu, (n, k) in enumerate(zip(lens, keep)):
        I = np.sort(rng.choice(n + Nk, size=k, replace=False)).astype(np.int32)
        sel.append(I)
        idx[uu, :k] = I
    off_out, total_out = u.aligned_offsets(keep, pad_rows=5)
    sentinel = 3.0
    Kout = torch.full((total_out, d), sentinel, dtype=hk.torch_dtype, device=u.DEV)
    Vout = torch.full((total_out, d), sentinel, dtype=hk.torch_dtype, device=u.DEV)
    Pout = torch.full((total_out,), -1, dtype=torch.int32, device=u.DEV)
    cout = Cache(Kout, Vout, off_out, np.asarray(keep, np.int32), Pout)
    hk.compact(B, Nk, cin, torch.from_numpy(idx).to(u.DEV), cout, u.to_dev(k_new, dtype), u.to_dev(v_new, dtype),
               pos_new=5000)
    torch.cuda.synchronize()
    Kg, Vg, Pg = u.from_dev(Kout), u.from_dev(Vout), Pout.cpu().numpy()
    touched = np.zeros(total_out, bool)
    for uu in range(U):
        b, h = divmod(uu, H)
        K_in = np.concatenate([rows[uu][0], k_new[b, h]]).astype(np.float64)
        V_in = np.concatenate([rows[uu][1], v_new[b, h]]).astype(np.float64)
        P_in = np.concatenate([1000 + np.arange(lens[uu]), 5000 + np.arange(Nk)])
        Kh, Vh = ho.compact(K_in, V_in, sel[uu])
        o, n = off_out[uu], keep[uu]
        assert np.array_equal(Kg[o:o + n], Kh) and np.array_equal(Vg[o:o + n], Vh)
        assert np.array_equal(Pg[o:o + n], P_in[sel[uu]])
        touched[o:o + n] = True
    assert np.all(Kg[~touched] == sentinel) and np.all(Pg[~touched] == -1)   # nothing written outside
    hk.close()


def test_compact_rejects_overlap_and_bad_ranges():
    u = _u()
    hk = u.make_hack(heads=1, head_dim=64, dtype="bf16", max_units=1, max_cache_len=64, max_queries=8)
    K = torch.zeros((64, 64), dtype=torch.bfloat16, device=u.DEV)
    idx = torch.zeros((1, 64), dtype=torch.int32, device=u.DEV)
    cin = Cache(K, K.clone(), [0], [16])
    with pytest.raises(HackError):       # output on top of rows that are read
        hk.compact(1, 1, cin, idx, Cache(K, cin.v, [8], [4]))
    with pytest.raises(HackError):       # output beyond the array
        hk.compact(1, 1, cin, idx, Cache(K.clone(), K.clone(), [56], [16]))
    with pytest.raises(HackError):       # keeps more rows than exist
        hk.compact(1, 1, cin, idx, Cache(K.clone(), K.clone(), [0], [17]))
    with pytest.raises(HackError):       # misaligned offset
        hk.compact(1, 1, Cache(K, K.clone(), [3], [4]), idx, Cache(K.clone(), K.clone(), [0], [2]))
    hk.close()


# ---------------------------------------------------------------------------
# a2 select
# ---------------------------------------------------------------------------
def _select_case(u, hk, imp_rows, t_in, head_type, budget, n_init, n_recent, H):
    U = len(t_in)
    stride = int(max(t_in))
    stride = (stride + 63) // 64 * 64
    imp = np.zeros((U, stride), np.float32)
    for i, r in enumerate(imp_rows):
        imp[i, :len(r)] = r
    kept = torch.full((U, stride), -1, dtype=torch.int32, device=u.DEV)
    len_out = hk.select(U // H, torch.from_numpy(imp).to(u.DEV), t_in, head_type, budget, n_init, n_recent, kept)
    torch.cuda.synchronize()
    kept = kept.cpu().numpy()
    for i in range(U):
        want = ho.select(imp_rows[i].astype(np.float64), int(head_type[i % H]), int(budget[i]), n_init, n_recent)
        assert len_out[i] == len(want) == min(budget[i], t_in[i])
        assert np.array_equal(kept[i, :len_out[i]], want), f"unit {i}: T={t_in[i]} b={budget[i]} type={head_type[i % H]}"
        assert np.all(kept[i, len_out[i]:] == -1)


def test_select_bit_exact_random_ragged():
    u = _u()
    rng = np.random.default_rng(5)
    H = 8
    hk = u.make_hack(heads=H, head_dim=64, dtype="bf16", max_units=32, max_cache_len=8831, max_queries=4096)
    head_type = np.array([0, 1, 0, 1, 1, 0, 1, 0], np.uint8)
    n_init, n_recent = 5, 64
    t_in = np.array([8831, 8831, 6039, 7981, 65, 64, 1025, 300,  70, 69, 1023, 1024, 4121, 2521, 100, 77], np.int32)
    budget = np.array([1579, 4735, 1943, 3885, 65, 1, 700, 299,   1, 69, 1022, 9999, 3885, 1943, 69, 76], np.int32)
    rows = []
    for T in t_in:
        r = rng.random(T).astype(np.float32) * np.float32(32.0 / T)
        dup = rng.integers(0, T, max(2, T // 10))           # plant exact duplicates around the threshold
        r[dup] = r[dup[0]]
        rows.append(r)
    _select_case(u, hk, rows, t_in, head_type, budget, n_init, n_recent, H)
    # swapped classes
    _select_case(u, hk, rows, t_in, 1 - head_type, budget, n_init, n_recent, H)
    hk.close()


def test_select_ties_and_degenerate_segments():
    u = _u()
    H = 2
    hk = u.make_hack(heads=H, head_dim=64, dtype="bf16", max_units=8, max_cache_len=2048, max_queries=256)
    head_type = np.array([0, 1], np.uint8)
    T = 1500
    flat = np.full(T, np.float32(32.0 / T))
    two = flat.copy()
    two[::3] *= 2
    zeros = np.zeros(T, np.float32)
    tiny = np.full(T, np.float32(1e-39))              # subnormal importance
    rows = [flat, flat, two, two, zeros, zeros, tiny, tiny]
    t_in = np.full(8, T, np.int32)
    for budget in (1, 5, 69, 70, 500, 501, 1499):
        _select_case(u, hk, rows, t_in, head_type, np.full(8, budget, np.int32), 5, 64, H)
    # structural budget below init + recent (small-budget reading) and n_init > T - n_recent
    _select_case(u, hk, rows, t_in, head_type, np.full(8, 40, np.int32), 5, 64, H)
    _select_case(u, hk, [r[:66] for r in rows], np.full(8, 66, np.int32), head_type, np.full(8, 65, np.int32), 5, 64, H)
    hk.close()


def test_select_rejects_bad_arguments():
    u = _u()
    hk = u.make_hack(heads=1, head_dim=64, dtype="bf16", max_units=1, max_cache_len=128, max_queries=16)
    imp = torch.zeros((1, 128), device=u.DEV)
    kept = torch.zeros((1, 128), dtype=torch.int32, device=u.DEV)
    with pytest.raises(HackError):
        hk.select(1, imp, [100], [0], [0], 5, 16, kept)           # budget < 1
    with pytest.raises(HackError):
        hk.select(1, imp, [129], [0], [10], 5, 16, kept)          # T above max_cache_len
    with pytest.raises(HackError):
        hk.select(1, imp, [100], [2], [10], 5, 16, kept)          # bad head class
    with pytest.raises(HackError):
        hk.select(1, imp, [10], [1], [5], 5, 16, kept)            # n_recent > T
    hk.close()


# ---------------------------------------------------------------------------
# a1 score
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,d,Nk,lens", [
    ("bf16", 128, 256, [0, 1, 255, 256, 257, 1500, 31, 700]),
    ("bf16", 64, 100, [5, 30, 462, 202, 0, 91, 255, 256]),
    ("bf16", 128, 9, [21, 57, 0, 4, 1000, 250, 256, 3]),        # N_k < 32: every query observes
    ("f32", 64, 100, [5, 30, 462, 202, 0, 91, 255, 256]),
])
def test_score_matches_oracle(dtype, d, Nk, lens):
    u = _u()
    rng = np.random.default_rng(11 + Nk + d)
    H, B = 4, 2
    U = H * B
    hk = u.make_hack(heads=H, head_dim=d, dtype=dtype, max_units=U, max_cache_len=2048, max_queries=256)
    scale = float(np.float32(1.0 / np.sqrt(d)))
    rows = [(u.rand_values(rng, (n, d), dtype), u.rand_values(rng, (n, d), dtype)) for n in lens]
    cin, _ = u.build_cache(rows, d, dtype, pad_rows=2, fill=100.0)      # poison between units
    q = u.rand_values(rng, (B, H, Nk, d), dtype) * 2.0
    k_new = u.rand_values(rng, (B, H, Nk, d), dtype)
    if dtype == "bf16":
        q = wl.bf16_to_f32(wl.bf16_round(q))
    stride = 2048
    imp = torch.full((U, stride), -1.0, device=u.DEV)
    hk.score(torch.from_numpy(q).to(hk.torch_dtype).to(u.DEV), cin, scale, imp, k_new=u.to_dev(k_new, dtype))
    torch.cuda.synchronize()
    got = imp.cpu().numpy().astype(np.float64)
    obs = ho.observation_rows(Nk, 32)
    worst = 0.0
    for uu in range(U):
        b, h = divmod(uu, H)
        K_in = np.concatenate([rows[uu][0], k_new[b, h]]).astype(np.float64)
        want = ho.importance(q[b, h][obs].astype(np.float64), K_in, scale)
        T = K_in.shape[0]
        rel = np.abs(got[uu, :T] - want) / want
        worst = max(worst, rel.max())
        assert np.all(got[uu, T:] == -1.0)
        assert abs(got[uu, :T].sum() - len(obs)) < 1e-4 * len(obs)
    assert worst < (2e-7 if dtype == "f32" else 1e-6), worst
    hk.close()


def test_score_many_units_split_into_launch_groups_and_repeated_calls():
    """More score work items than the device holds at once: the library must cut
    the launch into groups of whole units.  Calling twice on the same context
    also checks that the normaliser workspace is left clean."""
    u = _u()
    rng = np.random.default_rng(5)
    H, B, d, Nk, dtype = 16, 6, 128, 32, "bf16"
    U = H * B
    lens = [int(x) for x in rng.integers(3900, 4200, U)]
    lens[7], lens[50] = 1, 130                                         # short units among long ones
    hk = u.make_hack(heads=H, head_dim=d, dtype=dtype, max_units=U, max_cache_len=4352, max_queries=Nk)
    scale = float(np.float32(1.0 / np.sqrt(d)))
    rows = [(u.rand_values(rng, (n, d), dtype), None) for n in lens]
    rows = [(k, k) for k, _ in rows]
    cin, _ = u.build_cache(rows, d, dtype)
    q = u.rand_values(rng, (B, H, Nk, d), dtype) * 2.0
    k_new = u.rand_values(rng, (B, H, Nk, d), dtype)
    stride = 4352
    obs = ho.observation_rows(Nk, 32)
    qd, kd = u.to_dev(q, dtype), u.to_dev(k_new, dtype)
    for rep in range(2):
        imp = torch.full((U, stride), -1.0, device=u.DEV)
        hk.score(qd, cin, scale, imp, k_new=kd)
        torch.cuda.synchronize()
        got = imp.cpu().numpy().astype(np.float64)
        T_all = np.array(lens) + Nk
        sums = np.array([got[uu, :T_all[uu]].sum() for uu in range(U)])
        assert np.all(np.abs(sums - len(obs)) < 1e-4 * len(obs)), (rep, sums.min(), sums.max())
        for uu in (0, 7, 50, 51, U // 2, U - 1):
            b, h = divmod(uu, H)
            K_in = np.concatenate([rows[uu][0], k_new[b, h]]).astype(np.float64)
            want = ho.importance(q[b, h][obs].astype(np.float64), K_in, scale)
            assert float(np.max(np.abs(got[uu, :len(want)] - want) / want)) < 1e-6, (rep, uu)
            assert np.all(got[uu, len(want):] == -1.0)
    hk.close()


def test_score_extreme_logits_bf16():
    """Logits of a few hundred nats: the row normalisers live in fp64, so peaked
    rows must still follow the fp64 oracle over 100+ orders of magnitude (entries
    that underflow float32 are compared absolutely; the relative bar is the one
    the arithmetic supports at this logit magnitude, not the 1e-6 of ordinary data).  Beyond +-354 nats the parked logits are clamped: the
    library must say so instead of returning a silently different answer."""
    u = _u()
    rng = np.random.default_rng(21)
    H, B, d, Nk, dtype = 2, 1, 128, 40, "bf16"
    hk = u.make_hack(heads=H, head_dim=d, dtype=dtype, max_units=2, max_cache_len=1024, max_queries=Nk)
    rows = [(u.rand_values(rng, (n, d), dtype) * 4.0, u.rand_values(rng, (n, d), dtype)) for n in (700, 333)]
    cin, _ = u.build_cache(rows, d, dtype)
    q = wl.bf16_to_f32(wl.bf16_round(u.rand_values(rng, (B, H, Nk, d), dtype) * 4.0))
    k_new = u.rand_values(rng, (B, H, Nk, d), dtype) * 4.0
    obs = ho.observation_rows(Nk, 32)
    qd, kd = torch.from_numpy(q).to(hk.torch_dtype).to(u.DEV), u.to_dev(k_new, dtype)
    peak = max(float(np.abs(q[0, uu][obs].astype(np.float64) @ np.concatenate([rows[uu][0], k_new[0, uu]]).T.astype(np.float64)).max())
               for uu in range(2))
    scale = float(np.float32(300.0 / peak))                            # largest |logit| = 300 nats
    imp = torch.full((2, 1024), -1.0, device=u.DEV)
    hk.score(qd, cin, scale, imp, k_new=kd)
    torch.cuda.synchronize()
    hk.check()
    got = imp.cpu().numpy().astype(np.float64)
    for uu in range(2):
        K_in = np.concatenate([rows[uu][0], k_new[0, uu]]).astype(np.float64)
        want = ho.importance(q[0, uu][obs].astype(np.float64), K_in, scale)
        err = np.abs(got[uu, :len(want)] - want)
        # float32 slices of a dot product of magnitude 300 / scale carry ~2.5e-8 * |logit| of absolute
        # error into the logit, i.e. that much relative error into exp(logit): 1e-5 at 300 nats
        assert np.all(err <= 1e-5 * want + 1e-37), (uu, float((err / np.maximum(want, 1e-300)).max()))
        assert abs(got[uu, :len(want)].sum() - len(obs)) < 1e-4 * len(obs)
    # 500 nats: outside the supported range -> reported once, context stays usable
    hk.score(qd, cin, float(np.float32(500.0 / peak)), imp, k_new=kd)
    torch.cuda.synchronize()
    with pytest.raises(HackError) as ei:
        hk.check()
    assert ei.value.status == -3
    hk.check()
    hk.score(qd, cin, scale, imp, k_new=kd)
    torch.cuda.synchronize()
    hk.check()
    hk.close()


def test_score_cache_only_custom_rows_and_inactive_units():
    u = _u()
    rng = np.random.default_rng(3)
    H, B, d, Nk, dtype = 2, 1, 128, 64, "bf16"
    hk = u.make_hack(heads=H, head_dim=d, dtype=dtype, max_units=2, max_cache_len=1024, max_queries=64)
    rows = [(u.rand_values(rng, (n, d), dtype), u.rand_values(rng, (n, d), dtype)) for n in (513, 40)]
    cin, _ = u.build_cache(rows, d, dtype)
    q = u.rand_values(rng, (B, H, Nk, d), dtype)
    q_idx = np.array([63, 0, 5, 5, 17], np.int32)                     # arbitrary rows, repeats allowed
    imp = torch.full((2, 1024), -1.0, device=u.DEV)
    hk.score(u.to_dev(q, dtype), cin, 0.11, imp, q_idx=q_idx, n_obs=5, active=[1, 0])
    torch.cuda.synchronize()
    got = imp.cpu().numpy().astype(np.float64)
    want = ho.importance(q[0, 0][q_idx].astype(np.float64), rows[0][0].astype(np.float64), float(np.float32(0.11)))
    assert float(np.max(np.abs(got[0, :513] - want) / want)) < 1e-6
    assert np.all(got[1] == -1.0)                                     # inactive unit untouched
    with pytest.raises(HackError):
        hk.score(u.to_dev(q, dtype), cin, 0.11, imp, q_idx=[64], n_obs=1)
    with pytest.raises(HackError):
        hk.score(u.to_dev(q, dtype), cin, -1.0, imp)
    hk.close()


# ---------------------------------------------------------------------------
# a4 attention
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,d,Nk,lens,tol,kernel", [
    ("bf16", 128, 300, [1, 2, 63, 64, 65, 1943, 127, 700], 2e-2, "tile128"),
    ("bf16", 128, 300, [1, 2, 63, 64, 65, 1943, 127, 700], 2e-2, "split"),
    ("bf16", 64, 100, [102, 306, 1, 33, 562, 91, 128, 129], 2e-2, "tile128"),
    ("bf16", 64, 100, [102, 306, 1, 33, 562, 91, 128, 129], 2e-2, "split"),
    ("bf16", 128, 1, [1, 5, 21, 57, 121, 265, 64, 32], 2e-2, "tile128"),
    ("bf16", 128, 1, [1, 5, 21, 57, 121, 265, 64, 32], 2e-2, "split"),
    ("bf16", 64, 33, [3, 31, 32, 96, 97, 160, 2000, 129], 2e-2, "split"),
    ("bf16", 128, 300, [1, 2, 63, 64, 65, 1943, 127, 700], 2e-2, None),
    ("bf16", 128, 300, [1, 2, 63, 64, 65, 1943, 127, 700], 2e-2, "tile128_plain"),
    ("bf16", 64, 100, [102, 306, 1, 33, 562, 91, 128, 129], 2e-2, "tile128_plain"),
    ("bf16", 128, 130, [96, 97, 192, 193, 224, 225, 256, 289], 2e-2, "tile128"),      # 3 .. 10 key blocks: every
    ("bf16", 64, 130, [96, 97, 192, 193, 224, 225, 256, 289], 2e-2, "tile128"),       # way in and out of the steady loop
    ("bf16", 128, 130, [320, 321, 351, 352, 353, 384, 416, 449], 2e-2, "tile128"),
    ("bf16", 128, 300, [1, 2, 63, 64, 65, 1943, 127, 700], 2e-2, "stream"),           # work items cut into segments,
    ("bf16", 64, 100, [102, 306, 1, 33, 562, 91, 128, 129], 2e-2, "stream"),          # partial results added up by the
    ("bf16", 128, 130, [96, 97, 192, 193, 224, 225, 256, 289], 2e-2, "stream"),       # work-group that finishes last
    ("bf16", 64, 130, [320, 321, 351, 352, 353, 384, 416, 449], 2e-2, "stream"),
    ("bf16", 128, 1, [1, 5, 21, 57, 121, 265, 64, 32], 2e-2, "stream"),
    ("bf16", 128, 300, [1, 2, 63, 64, 65, 1943, 127, 700], 2e-2, "cut"),              # whole work items, the longest halved
    ("bf16", 64, 100, [102, 306, 1, 33, 562, 91, 128, 129], 2e-2, "cut"),
    ("bf16", 128, 130, [320, 321, 351, 352, 1353, 384, 416, 2047], 2e-2, "cut"),
    ("f32", 64, 100, [102, 306, 1, 33, 562, 91, 128, 129], 1e-4, None),
    ("f32", 128, 70, [1, 2, 63, 64, 65, 300, 127, 31], 1e-4, None),
])
def test_attention_matches_oracle(dtype, d, Nk, lens, tol, kernel):
    """Both bf16 attention kernels (128-query tiles; 32-query items with the keys split
    over the waves) on the same ragged shapes: fewer keys than waves, one key, block
    boundaries +-1, many blocks per wave, a last query tile with a single query."""
    u = _u()
    rng = np.random.default_rng(17 + Nk + d)
    H, B = 4, 2
    U = H * B
    hk = u.make_hack(heads=H, head_dim=d, dtype=dtype, max_units=U, max_cache_len=2048, max_queries=512,
                     attention=kernel)
    scale = float(np.float32(1.0 / np.sqrt(d)))
    rows = [(u.rand_values(rng, (n, d), dtype) * 1.5, u.rand_values(rng, (n, d), dtype)) for n in lens]
    if dtype == "bf16":
        rows = [(wl.bf16_to_f32(wl.bf16_round(k)), v) for k, v in rows]
    cache, _ = u.build_cache(rows, d, dtype, pad_rows=1, fill=50.0)
    q = u.rand_values(rng, (B, H, Nk, d), dtype)
    # twice with different queries: the second launch reuses whatever scratch the first one left
    for rep in range(2):
        out = torch.full((B, H, Nk, d), 7.0, dtype=hk.torch_dtype, device=u.DEV)
        hk.attn(u.to_dev(q, dtype), cache, scale, out)
        torch.cuda.synchronize()
        got = u.from_dev(out)
        for uu in range(U):
            b, h = divmod(uu, H)
            want = ho.attention(q[b, h].astype(np.float64), rows[uu][0].astype(np.float64),
                                rows[uu][1].astype(np.float64), scale)
            err = np.abs(got[b, h] - want).max()
            assert err < tol, (rep, uu, lens[uu], err)
        q = u.rand_values(rng, (B, H, Nk, d), dtype)
    hk.close()


def test_cut_and_streamed_attention_launches_agree_with_whole_work_items():
    """Random unit counts, cache lengths and query counts: the 128-query kernel with every cut the pair
    model likes, and in its streamed form (equal runs of key blocks), against the same kernel on whole
    work items.  The partial results of a cut work item are added up in float32, so the outputs agree to
    a bf16 rounding of the output; each form runs many times on its context (every launch meets the
    counters and partial-result slots the one before it left)."""
    u = _u()
    rng = np.random.default_rng(2024)
    for case in range(8):
        d = int(rng.choice([64, 128]))
        H, B = int(rng.integers(1, 9)), int(rng.integers(1, 6))
        U = H * B
        Nk = int(rng.integers(1, 900))
        lens = rng.integers(1, int(rng.choice([64, 700, 6000])) + 1, size=U).astype(np.int32)
        off = np.concatenate([[0], np.cumsum((lens + 7) // 8 * 8)])[:-1].astype(np.int64)
        rows = int(((lens + 7) // 8 * 8).sum())
        K = (torch.randn((rows, d), device=u.DEV) * 1.5).to(torch.bfloat16)
        V = torch.randn((rows, d), device=u.DEV).to(torch.bfloat16)
        q = torch.randn((B, H, Nk, d), device=u.DEV).to(torch.bfloat16)
        # Many launches back to back, alternating between two sets of queries: a part that was read before its
        # writer's stores had arrived would be the other query set's, far outside the tolerance.
        q2 = torch.randn((B, H, Nk, d), device=u.DEV).to(torch.bfloat16)
        outs = {}
        for kernel in ("tile128", "cut", "stream"):
            hk = u.make_hack(heads=H, head_dim=d, dtype="bf16", max_units=U, max_cache_len=6000, max_queries=900,
                             attention=kernel)
            o, o2 = torch.full_like(q, 7.0), torch.full_like(q, 7.0)
            first = None
            for it in range(1 if kernel == "tile128" else 24):
                hk.attn(q, Cache(K, V, off, lens), float(1.0 / np.sqrt(d)), o)
                hk.attn(q2, Cache(K, V, off, lens), float(1.0 / np.sqrt(d)), o2)
                if first is None:
                    first = (o.clone(), o2.clone())
                else:      # the parts are added up in a fixed order: every launch gives the same bits
                    assert torch.equal(o, first[0]) and torch.equal(o2, first[1]), (case, kernel, it)
                o.fill_(7.0)
                o2.fill_(7.0)
            o, o2 = first
            torch.cuda.synchronize()
            outs[kernel] = (o.float().cpu().numpy(), o2.float().cpu().numpy())
            hk.close()
        for kernel in ("cut", "stream"):
            for which in (0, 1):
                assert np.isfinite(outs[kernel][which]).all(), (case, kernel)
                err = float(np.abs(outs[kernel][which] - outs["tile128"][which]).max())
                assert err < 2e-2, (case, kernel, which, d, U, Nk, int(lens.max()), err)


def test_attention_rejects_empty_unit_and_bad_scale():
    u = _u()
    hk = u.make_hack(heads=1, head_dim=64, dtype="bf16", max_units=1, max_cache_len=64, max_queries=8)
    K = torch.zeros((64, 64), dtype=torch.bfloat16, device=u.DEV)
    q = torch.zeros((1, 1, 8, 64), dtype=torch.bfloat16, device=u.DEV)
    with pytest.raises(HackError):
        hk.attn(q, Cache(K, K.clone(), [0], [0]), 0.1, q.clone())
    with pytest.raises(HackError):
        hk.attn(q, Cache(K, K.clone(), [0], [8]), float("nan"), q.clone())
    with pytest.raises(HackError):
        hk.attn(torch.zeros((1, 1, 9, 64), dtype=torch.bfloat16, device=u.DEV), Cache(K, K.clone(), [0], [8]), 0.1, q)
    hk.close()


def test_attention_variant_query_matches_the_documented_rule():
    u = _u()
    hk = u.make_hack(heads=16, head_dim=128, dtype="bf16", max_units=32, max_cache_len=256, max_queries=4096)
    # 32-query work items of a launch: B*H*ceil(N_k/32); the key-split kernel serves launches up to 512 of them at d = 128
    assert [hk.attn_variant(2, n) for n in (1, 64, 400, 512, 513, 576, 4096)] == [1, 1, 1, 1, 0, 0, 0]
    assert hk.attn_variant(1, 1024) == 1 and hk.attn_variant(1, 1025) == 0
    hk.close()
    hk = u.make_hack(heads=30, head_dim=64, dtype="bf16", max_units=960, max_cache_len=256, max_queries=256)
    assert hk.attn_variant(32, 64) == 1 and hk.attn_variant(32, 100) == 0     # 1920 and 3840 items against 2048 at d = 64
    hk.close()
    hk = u.make_hack(heads=2, head_dim=64, dtype="f32", max_units=2, max_cache_len=64, max_queries=16)
    assert hk.attn_variant(1, 1) == 0                                          # fp32 contexts have one attention kernel
    with pytest.raises(HackError):
        hk.attn_variant(0, 4)
    hk.close()


def test_score_give_up_is_contained_reported_and_recovered(monkeypatch):
    """The in-kernel wait of the fused bf16 score kernel is bounded.  A host-side test hook makes
    one work-group of every fused launch withhold its row sums and sets a small poll limit, so the
    work-groups of that unit give up deterministically while every kernel still exits normally.
    Then: the condition is raised; a fused launch queued after the failing one does not consume
    what it left in the exchange slots (it writes nothing); the call that reports the failure
    re-arms the workspace and switches the context to the two-pass form; the same context then
    gives the right importance again."""
    u = _u()
    monkeypatch.setenv("HACK_SCORE_SPIN_LIMIT", "8")
    monkeypatch.setenv("HACK_SCORE_TEST_SKIP_PUBLISH", "3")
    rng = np.random.default_rng(9)
    H, d, dtype, Nk, L = 4, 128, "bf16", 64, 8000
    hk = u.make_hack(heads=H, head_dim=d, dtype=dtype, max_units=H, max_cache_len=8192, max_queries=Nk)
    monkeypatch.delenv("HACK_SCORE_SPIN_LIMIT")
    monkeypatch.delenv("HACK_SCORE_TEST_SKIP_PUBLISH")
    assert hk.score_mode() == 0
    K = u.rand_values(rng, (H * L, d), dtype)
    Kd = u.to_dev(K, dtype)
    cin = Cache(Kd, Kd, np.arange(H, dtype=np.int64) * L, np.full(H, L, np.int32))
    q = u.rand_values(rng, (1, H, Nk, d), dtype)
    qd = u.to_dev(q, dtype)
    scale = 0.05
    imp1 = torch.full((H, 8192), -1.0, device=u.DEV)
    imp2 = torch.full((H, 8192), -1.0, device=u.DEV)
    # a few milliseconds of other work first, so that both score calls are queued before the first one runs
    # (the host looks at the fault word at every entry)
    big = torch.randn((8192, 8192), device=u.DEV, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    for _ in range(8):
        big = (big @ big).clamp_(-1, 1)
    hk.score(qd, cin, scale, imp1)           # one unit of this launch never gets all its sums
    hk.score(qd, cin, scale, imp2)           # queued behind it: must leave without reading the slots
    torch.cuda.synchronize()
    assert torch.all(imp2 == -1.0)           # nothing was formed from stale sums
    with pytest.raises(HackError) as ei:
        hk.check()
    assert ei.value.status == -4
    assert hk.score_mode() == 1              # recovered into the form without in-kernel waits
    hk.check()                               # reported once
    imp3 = torch.full((H, 8192), -1.0, device=u.DEV)
    hk.score(qd, cin, scale, imp3)
    torch.cuda.synchronize()
    hk.check()
    got = imp3.cpu().numpy().astype(np.float64)
    obs = ho.observation_rows(Nk, 32)
    for uu in range(H):
        want = ho.importance(q[0, uu][obs].astype(np.float64), K[uu * L:(uu + 1) * L].astype(np.float64), scale)
        assert float(np.max(np.abs(got[uu, :L] - want) / want)) < 1e-6, uu
        assert np.all(got[uu, L:] == -1.0)
    hk.close()
    # a fresh context without the hook works in the fused form on the same inputs, with the same bits
    hk = u.make_hack(heads=H, head_dim=d, dtype=dtype, max_units=H, max_cache_len=8192, max_queries=Nk)
    imp4 = torch.full((H, 8192), -1.0, device=u.DEV)
    hk.score(qd, cin, scale, imp4)
    torch.cuda.synchronize()
    hk.check()
    assert hk.score_mode() == 0 and torch.equal(imp3, imp4)
    hk.close()


def test_score_two_pass_form_matches_fused_bit_for_bit_and_holds_any_number_of_items():
    """hack_set_score_mode: the two-pass form (no in-kernel waits) gives the same importance bit
    for bit, also where the fused form has to cut the work into several launches, and switching
    back and forth leaves the exchange workspace usable."""
    u = _u()
    rng = np.random.default_rng(15)
    H, B, d, Nk, dtype = 16, 5, 128, 48, "bf16"
    U = H * B
    lens = [int(x) for x in rng.integers(3500, 4200, U)]
    lens[3], lens[40] = 0, 77
    hk = u.make_hack(heads=H, head_dim=d, dtype=dtype, max_units=U, max_cache_len=4352, max_queries=Nk)
    rows = [(u.rand_values(rng, (n, d), dtype),) * 2 for n in lens]
    cin, _ = u.build_cache(rows, d, dtype)
    q, k_new = u.rand_values(rng, (B, H, Nk, d), dtype) * 1.5, u.rand_values(rng, (B, H, Nk, d), dtype)
    qd, kd = u.to_dev(wl.bf16_to_f32(wl.bf16_round(q)), dtype), u.to_dev(k_new, dtype)
    scale = float(np.float32(1.0 / np.sqrt(d)))
    out = []
    for mode in (0, 1, 0, 1):
        hk.set_score_mode(mode)
        imp = torch.full((U, 4352), -1.0, device=u.DEV)
        hk.score(qd, cin, scale, imp, k_new=kd)
        torch.cuda.synchronize()
        hk.check()
        out.append(imp)
    for o in out[1:]:
        assert torch.equal(out[0], o)
    got = out[1].cpu().numpy().astype(np.float64)
    obs = ho.observation_rows(Nk, 32)
    qh = wl.bf16_to_f32(wl.bf16_round(q))
    for uu in (0, 3, 40, U - 1):
        b, h = divmod(uu, H)
        K_in = np.concatenate([rows[uu][0], k_new[b, h]]).astype(np.float64)
        want = ho.importance(qh[b, h][obs].astype(np.float64), K_in, scale)
        assert float(np.max(np.abs(got[uu, :len(want)] - want) / want)) < 1e-6, uu
    hk.close()
