"""dct_threshold_compact_static (the entry point that takes no workspace and allocates nothing)
against dct_threshold_compact on the same inputs: count, indices and values bit for bit, on two
calls in a row, the second with a smaller input, and against the oracle on the first."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu


def test_static_workspace_call_matches_the_workspace_call():
    import paper_2010_08899_amd as dct
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    assert 0 < dct.dct_threshold_compact_static_scratch_bytes() < (1 << 20)
    first = True
    for n, k, seed in ((3_000_017, 30_001, 11), (70_001, 3_000, 12)):  # the second call is the smaller one
        g = si.gaussian_gradient(n, dev, si.BASE_SEED + seed)
        thr = torch.zeros(4, dtype=torch.int32, device=dev)
        dct.dct_select_threshold(g, k, thr, dct.new_select_workspace(g))
        ws = dct.new_compact_workspace(g)
        for mode in (dct.DCT_GE_TAU, dct.DCT_EXACT_K):
            cap = 2 * k
            out = []
            for static in (False, True):
                idx = torch.full((cap + 64,), -7, dtype=torch.int32, device=dev)
                val = torch.full((cap + 64,), 123.0, dtype=torch.float32, device=dev)
                cnt = torch.zeros(1, dtype=torch.int64, device=dev)
                if static:
                    dct.dct_threshold_compact_static(g, thr, mode, idx, val, cnt, capacity=cap)
                else:
                    dct.dct_threshold_compact(g, thr, mode, idx, val, cnt, ws, capacity=cap)
                out.append((dct.read_count(cnt, capacity=cap), idx.cpu().numpy(), val.cpu().numpy().view(np.uint32)))
            (c0, i0, v0), (c1, i1, v1) = out
            assert c0 == c1
            assert np.array_equal(i0, i1)  # the guard zone past the survivors included
            assert np.array_equal(v0, v1)
            if first:
                gh = g.cpu().numpy()
                eidx, eval_, ecnt = oracle.threshold_compact(gh, oracle.select_threshold(gh, k), mode)
                assert c1 == ecnt and np.array_equal(i1[:c1], eidx)
                assert np.array_equal(v1[:c1], eval_.view(np.uint32))
        first = False
    # sizes beyond the int32 index range are refused on the host, before anything is enqueued
    lib = dct.lib()
    assert lib.dct_threshold_compact_static(1, 0, 1 << 31, 1, 0, None, None, 0, 1, None) == 1
