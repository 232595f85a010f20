"""GPU checks at the largest sizes the interface admits: a vector of 2^31 - 1 elements
(indices are int32) and matrices of more than 2^32 elements (row offsets need 64 bits).

The CPU oracle cannot sort vectors of this length in a test's time.  The whole result is
therefore checked against the DEFINITIONS, evaluated with plain torch operations on the
device (comparisons, counts, nonzero, gather: none of the library's kernels): the
threshold record is the unique one with n_gt < k <= n_gt + n_eq, the survivors are the keys
above tau plus the tie_quota lowest-index ties, in ascending index order, values copied bit
for bit.  On top of that the oracle itself checks slices it can do in seconds: the last 2^20
elements of the vector (GE_TAU survivors of a slice do not depend on the rest), and rows at
the start of each matrix and around its 2^32-nd element.
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu

DEV = torch.device("cuda:0")
CHUNK = 1 << 28  # torch.nonzero and friends are applied to pieces of at most this many elements


@pytest.fixture(scope="module")
def dct():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2010_08899_amd as m
    m.lib()
    return m


def host(t):
    return oracle.as_numpy(t.detach().cpu())


def bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a.view(np.uint16)


def keys_of(v):
    if v.dtype == torch.bfloat16:
        return v.view(torch.int16).to(torch.int32) & 0x7FFF
    return v.view(torch.int32) & 0x7FFFFFFF


def count_where(keys, tau, op):
    total = 0
    for lo in range(0, keys.numel(), CHUNK):
        c = keys[lo:lo + CHUNK]
        total += int((c > tau).sum() if op == "gt" else (c == tau).sum())
    return total


def indices_where(keys, tau, op, limit=None):
    """Ascending indices (int64) of the keys that compare `op` with tau; at most `limit` of them."""
    parts, have = [], 0
    for lo in range(0, keys.numel(), CHUNK):
        c = keys[lo:lo + CHUNK]
        m = {"gt": c > tau, "eq": c == tau, "ge": c >= tau}[op]
        parts.append(torch.nonzero(m).flatten() + lo)
        have += parts[-1].numel()
        if limit is not None and have >= limit:
            break
    out = torch.cat(parts)
    return out if limit is None else out[:limit]


def check_threshold_record(keys, k, thr):
    n_gt = count_where(keys, thr.tau_key, "gt")
    n_eq = count_where(keys, thr.tau_key, "eq")
    assert n_gt < k <= n_gt + n_eq                      # tau_key IS the k-th largest key
    assert (thr.n_gt, thr.n_eq, thr.tie_quota) == (n_gt, n_eq, k - n_gt)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_dp_longest_vector(dct, dtype):
    n = (1 << 31) - 1
    k = n // 200
    g = si.gaussian_gradient(n, DEV, 3100)
    # a planted value near the 0.5 % quantile (2.807 sigma): tau lands on it, with two million ties to ration
    # (bf16 has ties by the million without any planting: 2^31 elements share 2^15 keys)
    tie_value = float(torch.tensor(2.82e-3).to(dtype))
    g[::1000] = tie_value
    g[n - 1] = -tie_value
    g = g.to(dtype)
    keys = keys_of(g)
    it = torch.int32 if dtype == torch.float32 else torch.int16

    thr_t = torch.zeros(4, dtype=torch.int32, device=DEV)
    dct.dct_select_threshold(g, k, thr_t, dct.new_select_workspace(g))
    thr = oracle.Threshold(*dct.read_threshold(thr_t))
    check_threshold_record(keys, k, thr)
    assert thr.tau_key == int(keys[0])
    assert 1 < thr.tie_quota < thr.n_eq

    cap = thr.n_gt + thr.n_eq + 16
    idx = torch.full((cap,), -7, dtype=torch.int32, device=DEV)
    val = torch.zeros(cap, dtype=dtype, device=DEV)
    cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    ws = dct.new_compact_workspace(g)

    # EXACT_K: everything above tau, and the lowest-index ties
    dct.dct_threshold_compact(g, thr_t, dct.DCT_EXACT_K, idx, val, cnt, ws)
    assert dct.read_count(cnt) == k
    want = torch.cat([indices_where(keys, thr.tau_key, "gt"),
                      indices_where(keys, thr.tau_key, "eq", limit=thr.tie_quota)]).sort().values
    assert want.numel() == k and torch.equal(idx[:k].long(), want)
    assert torch.equal(val[:k].view(it), g[want].view(it))
    assert bool((idx[k:] == -7).all())

    # GE_TAU: the paper's mask
    idx.fill_(-7)
    dct.dct_threshold_compact(g, thr_t, dct.DCT_GE_TAU, idx, val, cnt, ws)
    c = dct.read_count(cnt)
    assert c == thr.n_gt + thr.n_eq
    want = indices_where(keys, thr.tau_key, "ge")
    assert torch.equal(idx[:c].long(), want)
    assert torch.equal(val[:c].view(it), g[want].view(it))
    assert int(idx[c - 1]) == n - 1 and bool((idx[c:] == -7).all())  # the very last element is a tie

    # the oracle on the last 2^20 elements
    lo = n - (1 << 20)
    eidx, eval_, ecnt = oracle.threshold_compact(host(g[lo:]), thr, dct.DCT_GE_TAU)
    first = int(torch.searchsorted(idx[:c], torch.tensor([lo], dtype=torch.int32, device=DEV))[0])
    assert c - first == ecnt
    assert np.array_equal(host(idx[first:c]) - lo, eidx)
    assert np.array_equal(bits(host(val[first:c])), bits(eval_))

    # decompression: a dense vector with the survivors in place
    dense = torch.full((n,), 5.0, dtype=dtype, device=DEV)
    dct.dct_scatter(idx, val, cnt, dense)
    expect = torch.zeros(n, dtype=dtype, device=DEV)
    expect[want] = g[want]
    assert torch.equal(dense.view(it), expect.view(it))


def test_dp_ef_longest_vector(dct):
    n = (1 << 31) - 1
    k = n // 100
    g = si.gaussian_gradient(n, DEV, 3200)
    e = si.residual_vector(n, DEV, 3201)
    w = g + e  # one IEEE fp32 addition per element, as the method prescribes
    keys = keys_of(w)

    thr_t = torch.zeros(4, dtype=torch.int32, device=DEV)
    dct.dct_ef_select_threshold(g, e, k, thr_t, dct.new_select_workspace(g))
    thr = oracle.Threshold(*dct.read_threshold(thr_t))
    check_threshold_record(keys, k, thr)

    cap = thr.n_gt + thr.n_eq + 16
    idx = torch.full((cap,), -7, dtype=torch.int32, device=DEV)
    val = torch.zeros(cap, dtype=torch.float32, device=DEV)
    cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    e_out = torch.full((n,), 123.0, device=DEV)
    dct.dct_ef_threshold_compact(g, e, e_out, thr_t, dct.DCT_GE_TAU, idx, val, cnt, dct.new_compact_workspace(g))
    c = dct.read_count(cnt)
    assert c == thr.n_gt + thr.n_eq
    want = indices_where(keys, thr.tau_key, "ge")
    assert torch.equal(idx[:c].long(), want)
    assert torch.equal(val[:c].view(torch.int32), w[want].view(torch.int32))
    assert bool((idx[c:] == -7).all())
    # the residual: the sum where nothing was sent, +0 where a pair was
    expect = w.clone()
    expect[want] = 0.0
    assert torch.equal(e_out.view(torch.int32), expect.view(torch.int32))
    del expect

    # the oracle on the last 2^20 elements
    lo = n - (1 << 20)
    eidx, eval_, ecnt, e_exp = oracle.ef_threshold_compact(host(g[lo:]), host(e[lo:]), thr, dct.DCT_GE_TAU)
    first = int(torch.searchsorted(idx[:c], torch.tensor([lo], dtype=torch.int32, device=DEV))[0])
    assert c - first == ecnt
    assert np.array_equal(host(idx[first:c]) - lo, eidx)
    assert np.array_equal(bits(host(val[first:c])), bits(eval_))
    assert np.array_equal(bits(host(e_out[lo:])), bits(e_exp))

    # conservation: message + residual is the sum, exactly
    dense = torch.empty(n, device=DEV)
    dct.dct_scatter(idx, val, cnt, dense)
    assert torch.equal(dense + e_out, w)


ROW_BLOCK = 1 << 17


def expected_keep(xb, k):
    """[rows, D] bool: the k largest |x| of every row, ties to the lower column (plain torch)."""
    if xb.dtype == torch.bfloat16:
        kb = xb.view(torch.int16).to(torch.int32) & 0x7FFF
    else:
        kb = xb.view(torch.int32) & 0x7FFFFFFF
    tau = kb.topk(k, dim=1).values[:, -1:]
    gt = kb > tau
    eq = kb == tau
    quota = k - gt.sum(1, keepdim=True)
    keep = gt | (eq & (eq.cumsum(1, dtype=torch.int32) <= quota))
    return keep, tau.flatten()


@pytest.mark.parametrize("dtype,B,D,k", [
    (torch.bfloat16, (1 << 21) + 5, 2048, 102),   # one row per wavefront
    (torch.bfloat16, (1 << 23) + 3, 512, 26),     # four rows per wavefront
    (torch.float32, (1 << 20) + 3, 4096, 204),
])
def test_mp_more_than_2_to_32_elements(dct, dtype, B, D, k):
    assert B * D > 1 << 32
    x = si.relu_activations(B, D, DEV, 3300, dtype=dtype)
    dy = si.normal_matrix(B, D, DEV, 3301, dtype=dtype)
    idx = torch.full((B, k), -7, dtype=torch.int32, device=DEV)
    val = torch.zeros(B, k, dtype=dtype, device=DEV)
    tau = torch.zeros(B, dtype=dtype, device=DEV)
    dval = torch.zeros(B, k, dtype=dtype, device=DEV)
    dct.dct_rowtopk_fwd(x, k, idx, val, tau)
    dct.dct_rowtopk_bwd(dy, idx, dval)
    dense = torch.full((B, D), 3.0, dtype=dtype, device=DEV)
    dct.dct_rowtopk_scatter(idx, val, dense)
    it, kmask = (torch.int16, 0x7FFF) if dtype == torch.bfloat16 else (torch.int32, 0x7FFFFFFF)

    for r0 in range(0, B, ROW_BLOCK):
        r1 = min(r0 + ROW_BLOCK, B)
        xb = x[r0:r1]
        keep, tau_key = expected_keep(xb, k)
        assert bool((keep.sum(1) == k).all())
        cols = torch.nonzero(keep)[:, 1].view(r1 - r0, k)  # ascending within each row
        ib = idx[r0:r1].long()
        assert torch.equal(ib, cols), f"rows {r0}..{r1}"
        assert torch.equal(val[r0:r1].view(it), torch.gather(xb, 1, cols).view(it))
        assert torch.equal(tau[r0:r1].view(it).to(torch.int32) & kmask, tau_key)
        assert torch.equal(dval[r0:r1].view(it), torch.gather(dy[r0:r1], 1, cols).view(it))
        want = torch.where(keep, xb, torch.zeros((), dtype=dtype, device=DEV))
        assert torch.equal(dense[r0:r1].view(it), want.view(it))

    # the other two encodings of the mask carry the same survivors
    idx16 = torch.zeros(B, k, dtype=torch.int16, device=DEV)
    val2 = torch.zeros_like(val)
    dct.dct_rowtopk_fwd_idx16(x, k, idx16, val2, None)
    assert torch.equal(idx16.to(torch.int32) & 0xFFFF, idx) and torch.equal(val2.view(it), val.view(it))
    dval2 = torch.zeros_like(dval)
    dct.dct_rowtopk_bwd_idx16(dy, idx16, dval2)
    assert torch.equal(dval2.view(it), dval.view(it))
    dense2 = torch.full((B, D), 3.0, dtype=dtype, device=DEV)
    dct.dct_rowtopk_scatter_idx16(idx16, val, dense2)
    assert torch.equal(dense2.view(it), dense.view(it))
    del idx16
    mask = torch.zeros(B, D // 32, dtype=torch.int32, device=DEV)
    val2.zero_()
    dct.dct_rowtopk_fwd_bitmask(x, k, mask, val2, None)
    assert torch.equal(val2.view(it), val.view(it))
    dval2.zero_()
    dct.dct_rowtopk_bwd_bitmask(dy, mask, dval2)
    assert torch.equal(dval2.view(it), dval.view(it))
    dense2.fill_(3.0)
    dct.dct_rowtopk_scatter_bitmask(mask, val, dense2)
    assert torch.equal(dense2.view(it), dense.view(it))
    # ... and the bitmap has bit c % 32 of word c / 32 set for exactly the surviving columns
    for r0 in range(0, B, ROW_BLOCK * 8):
        r1 = min(r0 + ROW_BLOCK * 8, B)
        words = torch.zeros(r1 - r0, D // 32, dtype=torch.int64, device=DEV)
        cols = idx[r0:r1].long()
        words.scatter_add_(1, cols >> 5, torch.ones((), dtype=torch.int64, device=DEV) << (cols & 31))
        assert torch.equal(words, mask[r0:r1].long() & 0xFFFFFFFF)
    del mask, dense2, dval2, val2

    # the oracle on the first rows and on the last ones, which lie on both sides of element 2^32
    assert B - 24 < (1 << 32) // D < B
    for r0, r1 in ((0, 24), (B - 24, B)):
        eidx, eval_, etau = oracle.rowtopk_fwd(host(x[r0:r1]), k)
        assert np.array_equal(host(idx[r0:r1]), eidx)
        assert np.array_equal(bits(host(val[r0:r1])), bits(eval_))
        assert np.array_equal(bits(host(tau[r0:r1])), bits(etau))
        assert np.array_equal(bits(host(dval[r0:r1])), bits(oracle.rowtopk_bwd(host(dy[r0:r1]), eidx)))
        assert np.array_equal(bits(host(dense[r0:r1])), bits(oracle.rowscatter(eidx, eval_, D)))
