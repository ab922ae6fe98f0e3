"""hack_score_static (the entry point that allocates nothing: kernel scratch in a fixed device array
of the library) against hack_score through the C ABI: same importance bit for bit, on two calls in a
row, the second with a smaller input; beyond its stated maximum it refuses."""
import numpy as np
import pytest
import torch

from paper_2504_09261_amd.binding import HackError

pytestmark = pytest.mark.gpu


def test_score_static_matches_score_on_two_calls_in_a_row():
    from tests import gpu_util as u
    rng = np.random.default_rng(2026)
    H, d, dtype = 8, 128, "bf16"
    hk = u.make_hack(heads=H, head_dim=d, dtype=dtype, max_units=80, max_cache_len=8192, max_queries=512)
    scale = float(np.float32(1.0 / np.sqrt(d)))
    # first call: 4 x 8 = 32 units, long ragged caches + new rows; second call: 1 x 8 units, short caches, no new rows,
    # explicit observation rows and two inactive units
    cases = [
        dict(B=4, Nk=400, lens=[int(x) for x in rng.integers(2000, 7700, 32)], new=True, q_idx=None, active=None),
        dict(B=1, Nk=40, lens=[1, 17, 128, 129, 511, 512, 513, 1000], new=False,
             q_idx=np.array([39, 0, 7, 7, 20], np.int32), active=np.array([1, 1, 0, 1, 1, 1, 0, 1], np.uint8)),
    ]
    for case in cases:
        B, Nk, lens = case["B"], case["Nk"], case["lens"]
        U = B * H
        rows = [(u.rand_values(rng, (n, d), dtype),) * 2 for n in lens]
        cin, _ = u.build_cache(rows, d, dtype, pad_rows=3, fill=9.0)
        q = u.to_dev(u.rand_values(rng, (B, H, Nk, d), dtype), dtype)
        kn = u.to_dev(u.rand_values(rng, (B, H, Nk, d), dtype), dtype) if case["new"] else None
        n_obs = None if case["q_idx"] is None else len(case["q_idx"])
        want = torch.full((U, 8192), -1.0, device=u.DEV)
        got = torch.full((U, 8192), -1.0, device=u.DEV)
        hk.score(q, cin, scale, want, k_new=kn, q_idx=case["q_idx"], n_obs=n_obs, active=case["active"])
        hk.score_static(q, cin, scale, got, k_new=kn, q_idx=case["q_idx"], n_obs=n_obs, active=case["active"])
        torch.cuda.synchronize()
        hk.check()
        assert torch.equal(want, got)
        T = np.array(lens) + (Nk if case["new"] else 0)
        for uu in range(U):
            if case["active"] is not None and not case["active"][uu]:
                assert torch.all(got[uu] == -1.0)
            else:
                s = float(got[uu, :T[uu]].sum())
                assert abs(s - (32 if n_obs is None else n_obs)) < 1e-3, (uu, s)
    # more units than the fixed array is laid out for: refused, nothing launched
    lens = [8] * 80
    rows = [(u.rand_values(rng, (n, d), dtype),) * 2 for n in lens]
    cin, _ = u.build_cache(rows, d, dtype)
    q = u.to_dev(u.rand_values(rng, (10, H, 32, d), dtype), dtype)
    imp = torch.full((80, 8192), -1.0, device=u.DEV)
    with pytest.raises(HackError) as ei:
        hk.score_static(q, cin, scale, imp)
    assert ei.value.status == -2
    torch.cuda.synchronize()
    assert torch.all(imp == -1.0)
    act = np.zeros(80, np.uint8)
    act[:64] = 1
    hk.score_static(q, cin, scale, imp, active=act)     # a slice of 64 units is within the limit
    torch.cuda.synchronize()
    assert torch.all(imp[64:] == -1.0) and abs(float(imp[63, :8].sum()) - 32.0) < 1e-3
    hk.close()
