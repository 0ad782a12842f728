"""The allocation-free form of fg_lookup_prune (its scratch memory is a device array of the library) against
fg_lookup_prune with a caller's workspace: bit-identical outputs, on two calls in a row of which the second is smaller."""
import numpy as np
import pytest

from oracle import freshgnn_oracle as O

pytestmark = pytest.mark.gpu


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _block(r, n, n_src, max_deg):
    deg = r.integers(0, max_deg + 1, n)
    start = np.cumsum(np.concatenate([[0], deg[:-1]])).astype(np.int32) if n else np.zeros(0, np.int32)
    end = (start + deg).astype(np.int32)
    nnz = int(end[-1]) if n else 0
    col = r.integers(0, max(n_src, 1), max(nnz, 1)).astype(np.int32)
    return start, end, col, nnz


def test_lookup_prune_static_equals_lookup_prune_on_two_calls_in_a_row():
    import torch
    from paper_2301_07482_amd import binding as B
    assert torch.cuda.is_available()
    r = np.random.default_rng(5)
    N, cap, t_stale = 200000, 8192, 6
    cache = B.fg_cache_create(N, [cap], [4], B.FG_F32, t_stale, None)
    oc = O.HistoricalCache(N, cap, 4, t_stale)
    try:
        # fill the cache: a few updates through the ordinary entry points, the same ones on the oracle
        pool = r.permutation(N)[:6000].astype(np.int32)
        for it in range(3):
            ids_a = r.permutation(pool)[:3000]
            n_a = len(ids_a)
            gn = np.exp(r.standard_normal(n_a)).astype(np.float32)
            rows = np.zeros((n_a, 4), np.float32)
            wsb = max(B.fg_workspace_bytes(B.FG_WS_LOOKUP_PRUNE, n_a), B.fg_workspace_bytes(B.FG_WS_CACHE_UPDATE, n_a))
            ws = torch.zeros(wsb, dtype=torch.uint8, device="cuda")
            t_ids, t_hit = dev(torch, ids_a), torch.zeros(n_a, dtype=torch.uint8, device="cuda")
            t_l = [torch.zeros(n_a, dtype=torch.int32, device="cuda") for _ in range(3)]
            t_cnt, t_stats = torch.zeros(3, dtype=torch.int64, device="cuda"), torch.zeros(4, dtype=torch.int64, device="cuda")
            B.fg_lookup_prune(cache, 1, it, t_ids, n_a, None, None, None, None, 0, 0, None, t_hit, t_l[0], t_l[1], t_l[2], None,
                              t_cnt, ws, wsb, None)
            B.fg_cache_update(cache, 1, it, t_ids, n_a, None, t_hit, dev(torch, gn), 0.7, dev(torch, rows), 16, t_stats, ws, wsb, None)
            look = O.lookup_prune(oc, it, ids_a, None, None, None, None, 0)
            O.cache_update(oc, it, ids_a, None, look["hit"], gn, 0.7, rows)
        torch.cuda.synchronize()
        total_hits = 0
        # two calls in a row, the second with a smaller input (3 tiles and a ragged tail, then less than one tile)
        for n, n_src, max_deg in ((5000, 21000, 9), (700, 2500, 4)):
            ids = np.concatenate([r.permutation(pool)[:n // 2], r.permutation(N)[:n]])
            ids = ids[np.sort(np.unique(ids, return_index=True)[1])][:n].astype(np.int32)
            live = r.random(n) < 0.8
            start, end, col, nnz = _block(r, n, n_src, max_deg)
            got = {}
            for which in ("workspace", "static"):
                t_end = dev(torch, end)
                t_live_src = torch.full((n_src,), 3, dtype=torch.uint8, device="cuda")
                t_hit = torch.full((n,), 9, dtype=torch.uint8, device="cuda")
                t_hp, t_hs, t_np, t_ni = (torch.full((n,), -7, dtype=torch.int32, device="cuda") for _ in range(4))
                t_cnt = torch.zeros(3, dtype=torch.int64, device="cuda")
                args = (cache, 1, 3, dev(torch, ids), n, dev(torch, live.astype(np.uint8)), dev(torch, start), t_end, dev(torch, col),
                        nnz, n_src, t_live_src, t_hit, t_hp, t_hs, t_np, t_ni, t_cnt)
                if which == "workspace":
                    wsb = B.fg_workspace_bytes(B.FG_WS_LOOKUP_PRUNE, n)
                    ws = torch.zeros(wsb, dtype=torch.uint8, device="cuda")
                    B.fg_lookup_prune(*args, ws, wsb, None)
                else:
                    B.fg_lookup_prune_static(*args, None)
                torch.cuda.synchronize()
                got[which] = [t.cpu().numpy() for t in (t_cnt, t_hit, t_hp, t_hs, t_np, t_ni, t_end, t_live_src)]
            for a, b in zip(got["workspace"], got["static"]):
                assert np.array_equal(a, b)
            # and both are the oracle's result
            want_end = end.copy()
            want = O.lookup_prune(oc, 3, ids, live, start, want_end, col, n_src)
            cnt = got["static"][0]
            assert tuple(int(c) for c in cnt) == want["counts"]
            assert np.array_equal(got["static"][2][:cnt[1]], want["hit_pos"]) and np.array_equal(got["static"][3][:cnt[1]], want["hit_slot"])
            assert np.array_equal(got["static"][4][:cnt[2]], want["normal_pos"]) and np.array_equal(got["static"][6], want_end)
            assert np.array_equal(got["static"][7].astype(bool), want["live_src"])
            total_hits += int(cnt[1])
        assert total_hits > 0
        # beyond the built-in scratch memory the call refuses, before anything is launched
        with pytest.raises(B.FgError) as e:
            B.fg_lookup_prune_static(cache, 1, 3, 1, B.FG_LOOKUP_PRUNE_STATIC_MAX_N + 1, None, None, None, None, 0, 0, None, 1, 1, 1, 1,
                                     None, 1, None)
        assert e.value.code == B.FG_ERR_SHAPE
    finally:
        B.fg_cache_destroy(cache)
