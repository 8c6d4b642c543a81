"""The entry point that allocates nothing (ffsplit_select_heavy_static), called through the C
ABI: same indices, permutation and flag as ffsplit_select_heavy, bit for bit, on two calls in
a row that share the library's static scratch, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _both(ff, scores_h, k):
    L = ff.lib
    n = len(scores_h)
    sd = torch.from_numpy(scores_h).cuda()
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    out = []
    for static in (False, True):
        idx = torch.full((max(k, 1),), -1, dtype=torch.int32, device="cuda")
        perm = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        flag = torch.full((1,), 99, dtype=torch.int32, device="cuda")
        st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        if static:
            rc = L.ffsplit_select_heavy_static(vp(sd), n, k, vp(idx), vp(perm), vp(flag), st)
        else:
            ws = torch.empty(int(L.ffsplit_workspace_bytes(ctypes.byref(ff.make_desc(8, n)), ff.WS_SELECT, 0)),
                             dtype=torch.uint8, device="cuda")
            rc = L.ffsplit_select_heavy(vp(sd), n, k, vp(idx), vp(perm), vp(flag), vp(ws), ws.numel(), st)
        assert rc == 0, (static, rc)
        torch.cuda.synchronize()
        out.append((idx[:k].cpu().numpy(), perm.cpu().numpy(), int(flag.item())))
    return out


def test_static_select_matches_the_workspace_entry_point_twice_in_a_row():
    import paper_2401_04044_amd as ff
    from oracle import ffsplit_oracle as orc
    rng = np.random.default_rng(7)
    big = rng.random(50000).astype(np.float32)
    big[rng.integers(0, 50000, 9000)] = 0.75                      # many equal scores across the cut
    small = (rng.integers(0, 40, 3000) / 8.0).astype(np.float32)
    for scores, k in ((big, 2000), (small, 154), (big, 50000), (small, 0)):
        (i0, p0, f0), (i1, p1, f1) = _both(ff, scores, k)
        assert np.array_equal(i0, i1) and np.array_equal(p0, p1) and f0 == f1 == 0
        assert np.array_equal(i1, orc.select_heavy(scores, k))
        assert np.array_equal(p1, orc.neuron_permutation(i1, len(scores)))
    # a NaN raises the flag on both paths
    bad = small.copy()
    bad[17] = np.nan
    (i0, p0, f0), (i1, p1, f1) = _both(ff, bad, 10)
    assert f0 == f1 == -7 and np.array_equal(i0, i1) and np.array_equal(p0, p1)


def test_static_select_rejects_sizes_beyond_its_scratch():
    import paper_2401_04044_amd as ff
    fake = ctypes.c_void_p(0x1000)
    assert ff.lib.ffsplit_select_heavy_static(fake, ff.SELECT_STATIC_MAX_DFF + 1, 5, fake, None, None, None) == -9
    assert "scratch" in ff.status_string(-9)
