"""The allocation-free TopK entry point (dash_decide_topk_static: scratch in a device array of the library image
instead of a caller's workspace) against dash_decide_topk, bit for bit, through the C ABI: two calls in a row, the
second on a smaller input (the shared array still holds the first call's state and tie counts), then a larger one
again, both directions, with ties and protected ranks; and the size limit."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2604_18103_amd import binding as B

pytestmark = pytest.mark.gpu


def _both(p, s, n, keep_low):
    gs = torch.from_numpy(s).cuda()
    n_chunks = (n + 63) // 64
    out = []
    for static in (False, True):
        halt = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
        counts = torch.full((n_chunks,), -1, dtype=torch.int32, device="cuda")
        if static:
            B.dash_decide_topk_static(p, gs, n, keep_low, halt, counts)
        else:
            ws = torch.empty((256 + 4 * n_chunks + 64,), dtype=torch.uint8, device="cuda")
            B.dash_decide_topk(p, gs, n, keep_low, halt, counts, ws)
        torch.cuda.synchronize()
        out.append((halt.cpu().numpy(), counts.cpu().numpy()))
    return out


def test_static_scratch_topk_equals_workspace_topk_on_calls_in_a_row():
    rng = np.random.default_rng(4242)
    p = B.make_params(256, 4, 2, 64)
    for n, k_keep, first, last, ties in ((20000, 7000, 64, 32, True), (3001, 1200, 0, 0, True), (130, 1, 3, 2, False),
                                         (52428, 26214, 0, 0, False), (1, 1, 0, 0, False), (777, 0, 0, 0, True)):
        s = (np.abs(rng.standard_normal(n)) * np.exp(1.5 * rng.standard_normal(n))).astype(np.float32)
        if ties:
            s = (np.round(s * 3) / 3).astype(np.float32)
        p.k_keep, p.keep_first_n, p.keep_last_n = k_keep, first, last
        for keep_low in (False, True):
            (h_ws, c_ws), (h_st, c_st) = _both(p, s, n, keep_low)
            np.testing.assert_array_equal(h_st, h_ws)
            np.testing.assert_array_equal(c_st, c_ws)
            assert set(np.unique(h_st)) <= {0, 1}
            assert int(c_st.sum()) == int((h_st == 0).sum()) == max(k_keep, min(n, first + last))


def test_static_scratch_topk_rejects_sizes_beyond_its_array():
    L = B.lib()
    p = B.make_params(256, 4, 2, 64, k_keep=5)
    fake = 0x7F0000001000
    too_many = B.TOPK_STATIC_MAX_ROWS + 1
    assert L.dash_decide_topk_static(C.byref(p), fake, too_many, 0, fake, fake, None) == -2      # unsupported
    assert L.dash_decide_topk_static(C.byref(p), fake, -1, 0, fake, fake, None) == -1
    assert L.dash_decide_topk_static(C.byref(p), None, 10, 0, fake, fake, None) == -1
    assert L.dash_decide_topk_static(C.byref(p), fake, 0, 0, fake, fake, None) == 0              # nothing to do
    # at the limit itself the call runs
    n = B.TOPK_STATIC_MAX_ROWS
    s = np.random.default_rng(1).random(n).astype(np.float32)
    p.k_keep = n // 3
    (h_ws, c_ws), (h_st, c_st) = _both(p, s, n, False)
    np.testing.assert_array_equal(h_st, h_ws)
    np.testing.assert_array_equal(c_st, c_ws)
    assert int((h_st == 0).sum()) == n // 3
