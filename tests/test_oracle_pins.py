"""Pins for the CPU oracle: none of the expected values below comes from the
oracle itself or from the HIP path.

  * O(N^2) rank counting on tiny inputs (every k), over random, tie-heavy and
    special-value vectors;
  * hand-worked fixtures of Algorithm 1 and Algorithm 2 (tests/golden/);
  * closed forms (signed permutation of 1..N, all-equal, alternating sign);
  * library routines on tie-free data (numpy argsort / torch.topk / kthvalue);
  * the invariants that characterise the answer (count, tau separates kept
    from dropped, tie rule, ascending order, bit-copied values);
  * property tests over random sizes, k, dtypes and strides;
  * error feedback: a hand-worked two-iteration fixture with hand-rounded sums,
    numpy's float32 addition, rank counting on the summed vector, and the
    conservation law (delivered + residual == corrected gradient, bit for bit).
"""
import os

import numpy as np
import pytest
import torch
from hypothesis import given, settings, strategies as st

import oracle
import synth_inputs as si

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
CPU = torch.device("cpu")


# ------------------------------------------------------------------ helpers
def keys_of(a: np.ndarray) -> np.ndarray:
    """Sign-cleared bit patterns, written independently of the oracle's C++."""
    if a.dtype == np.float32:
        return a.view(np.uint32) & np.uint32(0x7FFFFFFF)
    assert a.dtype == np.uint16
    return (a & np.uint16(0x7FFF)).astype(np.uint32)


def brute_rank(keys: np.ndarray) -> np.ndarray:
    """rank[i] = number of positions that precede i (larger key, or equal key and
    lower position), by counting: O(N^2)."""
    n = keys.size
    rank = np.zeros(n, dtype=np.int64)
    for i in range(n):
        c = 0
        for j in range(n):
            if keys[j] > keys[i] or (keys[j] == keys[i] and j < i):
                c += 1
        rank[i] = c
    return rank


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, rest = line.partition(":")
            out[key.strip()] = rest.split()
    return out


def f32(words):
    return np.array([float(w) for w in words], dtype=np.float32)


def f32x(words):
    """Like f32, but also reads C99 hexadecimal floats (exact by construction)."""
    def one(w):
        return float.fromhex(w) if "0x" in w else float(w)
    vals = [one(w) for w in words]
    out = np.array(vals, dtype=np.float32)
    assert all(float(o) == v or (v != v) for o, v in zip(out, vals)), "fixture value is not a binary32 number"
    return out


def i32(words):
    return np.array([int(w) for w in words], dtype=np.int32)


def bits(a: np.ndarray) -> np.ndarray:
    return a.view(np.uint32) if a.dtype == np.float32 else a.view(np.uint16)


def to_bf16_bits(a32: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(a32)).to(torch.bfloat16)
    return oracle.as_numpy(t).copy()


def tiny_vectors(n, seed):
    vs = [(name, t.numpy().astype(np.float32)) for name, t in si.adversarial_vectors(n, CPU, seed)]
    rng = np.random.default_rng(seed)
    vs.append(("random", rng.standard_normal(n).astype(np.float32)))
    nanv = rng.standard_normal(n).astype(np.float32)
    if n >= 3:
        nanv[n // 3] = np.nan
        nanv[0] = np.inf
    vs.append(("nan_inf", nanv))
    return vs


# ------------------------------------------------------------------ brute force (DP)
@pytest.mark.parametrize("n", [1, 2, 5, 17, 40])
def test_dp_against_rank_counting(n):
    for name, g in tiny_vectors(n, 1000 + n):
        for g_any in (g, to_bf16_bits(g)):
            keys = keys_of(g_any)
            rank = brute_rank(keys)
            for k in range(1, n + 1):
                exp_idx = np.nonzero(rank < k)[0]
                tau = int(keys[np.nonzero(rank == k - 1)[0][0]])
                thr = oracle.select_threshold(g_any, k)
                assert thr.tau_key == tau, (name, n, k)
                assert thr.n_gt == int((keys > tau).sum())
                assert thr.n_eq == int((keys == tau).sum())
                assert thr.tie_quota == k - thr.n_gt
                assert oracle.select_threshold(g_any, k, method="nth") == thr
                idx, val, cnt = oracle.threshold_compact(g_any, thr, oracle.EXACT_K)
                assert cnt == k and np.array_equal(idx, exp_idx), (name, n, k)
                assert np.array_equal(bits(val), bits(g_any[exp_idx]))
                ge_idx = np.nonzero(keys >= tau)[0]
                idx, val, cnt = oracle.threshold_compact(g_any, thr, oracle.GE_TAU)
                assert cnt == ge_idx.size and np.array_equal(idx, ge_idx)
                assert np.array_equal(bits(val), bits(g_any[ge_idx]))


# ------------------------------------------------------------------ brute force (MP)
@pytest.mark.parametrize("d", [1, 3, 8, 33])
def test_mp_against_rank_counting(d):
    B = 5
    rng = np.random.default_rng(77 + d)
    rows = []
    vecs = tiny_vectors(d, 2000 + d)
    for b in range(B):
        rows.append(vecs[(b * 3) % len(vecs)][1])
    x = np.stack(rows).astype(np.float32)
    x[B - 1] = np.maximum(rng.standard_normal(d), 0).astype(np.float32)
    dy = rng.standard_normal((B, d)).astype(np.float32)
    for xa, dya in ((x, dy), (to_bf16_bits(x), to_bf16_bits(dy))):
        for k in range(1, d + 1):
            idx, val, tau = oracle.rowtopk_fwd(xa, k)
            dval = oracle.rowtopk_bwd(dya, idx)
            for b in range(B):
                keys = keys_of(xa[b])
                rank = brute_rank(keys)
                exp = np.nonzero(rank < k)[0]
                assert np.array_equal(idx[b], exp), (d, k, b)
                assert np.array_equal(bits(val[b]), bits(xa[b][exp]))
                assert int(keys_of(tau[b:b + 1])[0]) == int(keys[np.nonzero(rank == k - 1)[0][0]])
                assert int(bits(tau[b:b + 1])[0]) == int(keys_of(tau[b:b + 1])[0])  # tau >= +0
                assert np.array_equal(bits(dval[b]), bits(dya[b][exp]))


# ------------------------------------------------------------------ hand-worked fixtures
def test_golden_alg1():
    gd = read_golden("alg1_worked.txt")
    g = f32(gd["g"])
    k = int(gd["k"][0])
    thr = oracle.select_threshold(g, k)
    tau = np.array([thr.tau_key], dtype=np.uint32).view(np.float32)[0]
    assert tau == float(gd["tau"][0])
    assert (thr.n_gt, thr.n_eq, thr.tie_quota) == (int(gd["n_gt"][0]), int(gd["n_eq"][0]), int(gd["tie_quota"][0]))
    idx, val, cnt = oracle.threshold_compact(g, thr, oracle.GE_TAU)
    assert cnt == len(gd["ge_idx"]) and np.array_equal(idx, i32(gd["ge_idx"]))
    assert np.array_equal(bits(val), bits(f32(gd["ge_val"])))
    idx, val, cnt = oracle.threshold_compact(g, thr, oracle.EXACT_K)
    assert cnt == k and np.array_equal(idx, i32(gd["exact_idx"]))
    assert np.array_equal(bits(val), bits(f32(gd["exact_val"])))
    # same instance in bf16 (every value is exactly representable)
    gb = to_bf16_bits(g)
    thr_b = oracle.select_threshold(gb, k)
    assert thr_b.tau_key == int(to_bf16_bits(np.array([1.0], dtype=np.float32))[0])
    idx, val, cnt = oracle.threshold_compact(gb, thr_b, oracle.EXACT_K)
    assert np.array_equal(idx, i32(gd["exact_idx"]))
    assert np.array_equal(val, to_bf16_bits(f32(gd["exact_val"])))


def test_golden_alg2():
    gd = read_golden("alg2_worked.txt")
    k = int(gd["k"][0])
    x = np.stack([f32(gd[f"x{b}"]) for b in range(3)])
    dy = np.stack([f32(gd[f"dy{b}"]) for b in range(3)])
    for conv in (lambda a: a, to_bf16_bits):
        idx, val, tau = oracle.rowtopk_fwd(conv(x), k)
        dval = oracle.rowtopk_bwd(conv(dy), idx)
        for b in range(3):
            assert np.array_equal(idx[b], i32(gd[f"idx{b}"]))
            assert np.array_equal(bits(val[b]), bits(conv(f32(gd[f"val{b}"]))))
            assert np.array_equal(bits(dval[b]), bits(conv(f32(gd[f"dval{b}"]))))
        assert np.array_equal(bits(tau), bits(conv(f32(gd["tau"]))))


def test_capacity_prefix_and_zero_count():
    gd = read_golden("alg1_worked.txt")
    g = f32(gd["g"])
    thr = oracle.select_threshold(g, 4)
    idx, val, cnt = oracle.threshold_compact(g, thr, oracle.GE_TAU, capacity=2)
    assert cnt == 5 and np.array_equal(idx, i32(gd["ge_idx"])[:2])
    assert np.array_equal(val, f32(gd["ge_val"])[:2])
    stale = oracle.Threshold(int(np.array([10.0], dtype=np.float32).view(np.uint32)[0]), 0, 0, 0)
    idx, val, cnt = oracle.threshold_compact(g, stale, oracle.GE_TAU)
    assert cnt == 0 and idx.size == 0


def test_invalid_arguments():
    g = np.ones(4, dtype=np.float32)
    for k in (0, 5):
        with pytest.raises(ValueError):
            oracle.select_threshold(g, k)
    with pytest.raises(ValueError):
        oracle.rowtopk_fwd(np.ones((2, 4), dtype=np.float32), 5)


# ------------------------------------------------------------------ closed forms
@pytest.mark.parametrize("n,k", [(1000, 1), (1000, 10), (1000, 999), (1000, 1000), (4097, 41)])
def test_signed_permutation_closed_form(n, k):
    rng = np.random.default_rng(n * 7 + k)
    mags = rng.permutation(n) + 1
    g = (mags * rng.choice([-1, 1], n)).astype(np.float32)
    thr = oracle.select_threshold(g, k)
    assert np.array([thr.tau_key], dtype=np.uint32).view(np.float32)[0] == float(n - k + 1)
    assert (thr.n_gt, thr.n_eq, thr.tie_quota) == (k - 1, 1, 1)
    exp = np.nonzero(mags >= n - k + 1)[0]
    for mode in (oracle.GE_TAU, oracle.EXACT_K):
        idx, val, cnt = oracle.threshold_compact(g, thr, mode)
        assert cnt == k and np.array_equal(idx, exp) and np.array_equal(val, g[exp])


@pytest.mark.parametrize("value", [0.75, 0.0, -0.0])
def test_all_equal_closed_form(value):
    n, k = 257, 19
    g = np.full(n, value, dtype=np.float32)
    thr = oracle.select_threshold(g, k)
    assert thr.tau_key == int(np.abs(g[:1]).view(np.uint32)[0])
    assert (thr.n_gt, thr.n_eq, thr.tie_quota) == (0, n, k)
    idx, val, cnt = oracle.threshold_compact(g, thr, oracle.EXACT_K)
    assert cnt == k and np.array_equal(idx, np.arange(k)) and np.array_equal(bits(val), bits(g[:k]))
    idx, _, cnt = oracle.threshold_compact(g, thr, oracle.GE_TAU)
    assert cnt == n and np.array_equal(idx, np.arange(n))


def test_alternating_sign_ties_resolve_by_index():
    n, k = 64, 9
    g = np.array([3.0 if i % 2 == 0 else -3.0 for i in range(n)], dtype=np.float32)
    thr = oracle.select_threshold(g, k)
    idx, val, cnt = oracle.threshold_compact(g, thr, oracle.EXACT_K)
    assert cnt == k and np.array_equal(idx, np.arange(k)) and np.array_equal(val, g[:k])


def test_k_equals_n_keeps_everything():
    rng = np.random.default_rng(5)
    g = rng.standard_normal(513).astype(np.float32)
    thr = oracle.select_threshold(g, g.size)
    assert thr.tau_key == int(keys_of(g).min())
    idx, val, cnt = oracle.threshold_compact(g, thr, oracle.EXACT_K)
    assert cnt == g.size and np.array_equal(idx, np.arange(g.size)) and np.array_equal(bits(val), bits(g))


# ------------------------------------------------------------------ library routines (tie-free data)
@pytest.mark.parametrize("n,k", [(5000, 50), (65536, 656), (100003, 1)])
def test_dp_against_library_on_distinct_magnitudes(n, k):
    rng = np.random.default_rng(n + k)
    g = rng.standard_normal(n + n // 8).astype(np.float32)
    _, first = np.unique(np.abs(g), return_index=True)  # drop repeated magnitudes: tie-free data,
    g = g[np.sort(first)[:n]]                           # so the library's tie order is irrelevant
    mag = np.abs(g)
    assert g.size == n and np.unique(mag).size == n
    order = np.argsort(-mag.astype(np.float64), kind="stable")
    exp = np.sort(order[:k])
    thr = oracle.select_threshold(g, k)
    tau = np.array([thr.tau_key], dtype=np.uint32).view(np.float32)[0]
    assert tau == mag[order[k - 1]]
    assert tau == torch.kthvalue(torch.from_numpy(mag), n - k + 1).values.item()
    idx, val, cnt = oracle.threshold_compact(g, thr, oracle.EXACT_K)
    assert cnt == k and np.array_equal(idx, exp) and np.array_equal(val, g[exp])
    top = torch.topk(torch.from_numpy(mag), k).indices.numpy()
    assert np.array_equal(np.sort(top), idx)


def test_mp_against_library_on_distinct_magnitudes():
    rng = np.random.default_rng(11)
    B, D, k = 64, 300, 15
    x = rng.standard_normal((B, D)).astype(np.float32)
    dy = rng.standard_normal((B, D)).astype(np.float32)
    assert all(np.unique(np.abs(r)).size == D for r in x)
    idx, val, tau = oracle.rowtopk_fwd(x, k)
    top = torch.topk(torch.from_numpy(np.abs(x)), k, dim=1)
    exp = np.sort(top.indices.numpy(), axis=1)
    assert np.array_equal(idx, exp)
    assert np.array_equal(val, np.take_along_axis(x, exp, axis=1))
    assert np.array_equal(tau, top.values.numpy()[:, -1])
    dval = oracle.rowtopk_bwd(dy, idx)
    assert np.array_equal(dval, dy[np.arange(B)[:, None], exp])


def test_mp_row_stride():
    rng = np.random.default_rng(12)
    B, D, S, k = 7, 50, 64, 5
    buf = np.full((B, S), 1e4, dtype=np.float32)
    buf[:, :D] = rng.standard_normal((B, D)).astype(np.float32)
    x = buf[:, :D]
    idx, val, tau = oracle.rowtopk_fwd(x, k)
    idx2, val2, tau2 = oracle.rowtopk_fwd(np.ascontiguousarray(x), k)
    assert np.array_equal(idx, idx2) and np.array_equal(val, val2) and np.array_equal(tau, tau2)
    assert np.array_equal(oracle.rowtopk_bwd(x, idx), val)


# ------------------------------------------------------------------ invariants as properties
def check_dp_invariants(g, k, thr, idx, val, cnt, mode):
    keys = keys_of(g)
    tau = thr.tau_key
    assert np.all(np.diff(idx.astype(np.int64)) > 0)
    assert np.array_equal(bits(val), bits(g[idx]))
    kept = np.zeros(g.size, dtype=bool)
    kept[idx] = True
    assert np.all(keys[kept] >= tau) and np.all(keys[~kept] <= tau)
    assert thr.n_gt == int((keys > tau).sum()) and thr.n_eq == int((keys == tau).sum())
    assert 1 <= thr.tie_quota <= thr.n_eq and thr.tie_quota == k - thr.n_gt
    if mode == oracle.EXACT_K:
        assert cnt == k == idx.size
        ties = np.nonzero(keys == tau)[0]
        assert np.array_equal(np.nonzero(kept & (keys == tau))[0], ties[:thr.tie_quota])
    else:
        assert cnt == thr.n_gt + thr.n_eq == idx.size == int((keys >= tau).sum())


@settings(max_examples=120, deadline=None)
@given(n=st.integers(1, 3000), frac=st.floats(0.0, 1.0), levels=st.sampled_from([0, 2, 3, 17, 1000]),
       seed=st.integers(0, 2 ** 31), bf16=st.booleans())
def test_dp_invariants_property(n, frac, levels, seed, bf16):
    rng = np.random.default_rng(seed)
    g = rng.standard_normal(n).astype(np.float32)
    if levels:
        g = (np.round(g * levels / 3.0) * (3.0 / levels)).astype(np.float32)  # few distinct magnitudes
    ga = to_bf16_bits(g) if bf16 else g
    k = min(n, max(1, int(round(frac * n))))
    thr = oracle.select_threshold(ga, k)
    for mode in (oracle.GE_TAU, oracle.EXACT_K):
        idx, val, cnt = oracle.threshold_compact(ga, thr, mode)
        check_dp_invariants(ga, k, thr, idx, val, cnt, mode)
    if thr.n_eq == thr.tie_quota:
        a = oracle.threshold_compact(ga, thr, oracle.GE_TAU)
        b = oracle.threshold_compact(ga, thr, oracle.EXACT_K)
        assert np.array_equal(a[0], b[0]) and a[2] == b[2]


@settings(max_examples=80, deadline=None)
@given(B=st.integers(1, 12), D=st.integers(1, 400), frac=st.floats(0.0, 1.0), pad=st.integers(0, 9),
       seed=st.integers(0, 2 ** 31), bf16=st.booleans(), relu=st.booleans())
def test_mp_invariants_property(B, D, frac, pad, seed, bf16, relu):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, D + pad)).astype(np.float32)
    if relu:
        x = np.maximum(x, 0)
    dy = rng.standard_normal((B, D + pad)).astype(np.float32)
    xa = (to_bf16_bits(x) if bf16 else x)[:, :D]
    dya = (to_bf16_bits(dy) if bf16 else dy)[:, :D]
    k = min(D, max(1, int(round(frac * D))))
    idx, val, tau = oracle.rowtopk_fwd(xa, k)
    dval = oracle.rowtopk_bwd(dya, idx)
    assert idx.shape == (B, k)
    for b in range(B):
        keys = keys_of(np.ascontiguousarray(xa[b]))
        t = int(keys_of(tau[b:b + 1])[0])
        assert np.all(np.diff(idx[b].astype(np.int64)) > 0) and idx[b].min() >= 0 and idx[b].max() < D
        kept = np.zeros(D, dtype=bool)
        kept[idx[b]] = True
        assert np.all(keys[kept] >= t) and np.all(keys[~kept] <= t) and t in keys[kept]
        ties = np.nonzero(keys == t)[0]
        quota = k - int((keys > t).sum())
        assert np.array_equal(np.nonzero(kept & (keys == t))[0], ties[:quota])
        assert np.array_equal(bits(val[b]), bits(np.ascontiguousarray(xa[b])[idx[b]]))
        assert np.array_equal(bits(dval[b]), bits(np.ascontiguousarray(dya[b])[idx[b]]))


# ------------------------------------------------------------------ generators + k: statistical sanity
def test_keep_counts():
    assert si.C1_K == 10486 and si.C2_K == 51 and si.C3_K == 25000
    assert si.C4_K == 1342178 and si.C4_NZ_ROWS == 209715 and si.C5_K == 204
    assert si.C1_N - (si.C1_N * 99) // 100 == si.C1_K  # N - floor(N*eta), eta = 0.99 (Algorithm 1)


def tau_value(thr):
    return float(np.array([thr.tau_key], dtype=np.uint32).view(np.float32)[0])


def test_c1_threshold_is_the_normal_quantile():
    g, k = si.config_c1(CPU)
    thr = oracle.select_threshold(g.numpy(), k)
    assert abs(tau_value(thr) / 2.5758e-3 - 1) < 0.02  # two-sided 1 % point of N(0, 1e-3^2)
    idx, _, cnt = oracle.threshold_compact(g.numpy(), thr, oracle.EXACT_K)
    assert cnt == k


def test_c3_threshold_is_the_student_t_quantile_and_reuse_counts_fluctuate():
    n = 1_000_000  # c3's distribution at a size the CPU suite affords
    k = si.ceil_frac(n, 1, 1000)
    g0 = si.config_c3_draw(CPU, 0, n).numpy()
    thr = oracle.select_threshold(g0, k)
    assert abs(tau_value(thr) / 12.92e-3 - 1) < 0.08  # two-sided 0.1 % point of t(3) * 1e-3
    g1 = si.config_c3_draw(CPU, 1, n).numpy()
    assert not np.array_equal(g0, g1)
    _, _, cnt = oracle.threshold_compact(g1, thr, oracle.GE_TAU)
    assert cnt != k and abs(cnt - k) < 6 * (k ** 0.5) * 2  # stale tau: count near k, not equal


def test_c4_structure_and_quantile():
    rows = 1 << 16
    g, k = si.config_c4(CPU, rows)
    t = g.view(rows, si.C4_DIM)
    nz_rows = (t != 0).any(dim=1).sum().item()
    assert nz_rows == (rows * 5) // 100
    assert (t == 0).all(dim=1).sum().item() == rows - nz_rows
    thr = oracle.select_threshold(g.numpy(), k)
    assert abs(tau_value(thr) / 1.645 - 1) < 0.03  # keeps 10 % of the non-zeros of N(0,1)


def test_c2_c5_shape_sanity():
    x, dy, k = si.config_c2(CPU)
    assert x.shape == (si.C2_B, si.C2_D) and abs((x == 0).float().mean().item() - 0.5) < 0.01
    _, _, tau = oracle.rowtopk_fwd(x.numpy()[:256], k)
    assert abs(tau.mean() / 1.64 - 1) < 0.05  # 10 % point of the half-normal non-zeros
    xb, dyb, kb = si.config_c5(CPU, b=64)
    assert xb.dtype == torch.bfloat16 and xb.shape == (64, si.C5_D) and kb == 204
    idx, val, taub = oracle.rowtopk_fwd(oracle.as_numpy(xb), kb)
    tau_f = torch.from_numpy(taub.view(np.int16)).view(torch.bfloat16).float()
    assert abs(tau_f.mean().item() / 1.64 - 1) < 0.05
    # bf16 makes ties at tau the normal case
    keys = keys_of(oracle.as_numpy(xb))
    n_eq = [(keys[b] == (int(taub[b]) & 0x7FFF)).sum() for b in range(64)]
    assert np.mean(n_eq) > 1.5


# ------------------------------------------------------------------ error feedback (Algorithm 1 with E_grad)
def scatter(n, idx, val):
    out = np.zeros(n, dtype=np.float32)
    out[idx] = val
    return out


def test_golden_error_feedback_two_iterations():
    gd = read_golden("alg1_error_feedback_worked.txt")
    g1, e0, g2 = f32x(gd["g1"]), f32x(gd["e0"]), f32x(gd["g2"])
    k = int(gd["k"][0])
    # iteration 1: add the residual, select, mask, new residual
    assert np.array_equal(bits(oracle.ef_accumulate(g1, e0)), bits(f32x(gd["w1"])))
    thr = oracle.ef_select_threshold(g1, e0, k)
    tau = np.array([thr.tau_key], dtype=np.uint32).view(np.float32)[0]
    assert tau == float(gd["tau"][0])
    assert (thr.n_gt, thr.n_eq, thr.tie_quota) == (int(gd["n_gt"][0]), int(gd["n_eq"][0]), int(gd["tie_quota"][0]))
    for mode in (oracle.GE_TAU, oracle.EXACT_K):
        idx, val, cnt, e1 = oracle.ef_threshold_compact(g1, e0, thr, mode)
        assert cnt == k and np.array_equal(idx, i32(gd["idx1"]))
        assert np.array_equal(bits(val), bits(f32x(gd["val1"])))
        assert np.array_equal(bits(e1), bits(f32x(gd["e1"])))
    # iteration 2 reuses the threshold of iteration 1
    assert np.array_equal(bits(oracle.ef_accumulate(g2, e1)), bits(f32x(gd["w2"])))
    idx, val, cnt, e2 = oracle.ef_threshold_compact(g2, e1, thr, oracle.GE_TAU)
    assert cnt == len(gd["ge_idx2"]) and np.array_equal(idx, i32(gd["ge_idx2"]))
    assert np.array_equal(bits(val), bits(f32x(gd["ge_val2"])))
    assert np.array_equal(bits(e2), bits(f32x(gd["ge_e2"])))
    idx, val, cnt, e2 = oracle.ef_threshold_compact(g2, e1, thr, oracle.EXACT_K)
    assert np.array_equal(idx, i32(gd["exact_idx2"]))
    assert np.array_equal(bits(val), bits(f32x(gd["exact_val2"])))
    assert np.array_equal(bits(e2), bits(f32x(gd["exact_e2"])))
    # survivors that do not fit stay in the residual
    idx, val, cnt, e2 = oracle.ef_threshold_compact(g2, e1, thr, oracle.GE_TAU, capacity=2)
    assert cnt == int(gd["cap2_count"][0]) and np.array_equal(idx, i32(gd["cap2_idx"]))
    assert np.array_equal(bits(e2), bits(f32x(gd["cap2_e2"])))


def test_golden_error_feedback_rounding():
    gd = read_golden("alg1_error_feedback_worked.txt")
    g, e, w = f32x(gd["round_g"]), f32x(gd["round_e"]), f32x(gd["round_w"])
    assert np.array_equal(bits(oracle.ef_accumulate(g, e)), bits(w))
    assert np.array_equal(bits(oracle.ef_accumulate(e, g)), bits(w))  # the sum is commutative


def ef_vectors(n, seed):
    """(g, e) pairs with cancellation, wide exponent ranges, denormals and exact ties in the sum."""
    rng = np.random.default_rng(seed)
    out = []
    g = rng.standard_normal(n).astype(np.float32)
    out.append(("normal", g, (0.3 * rng.standard_normal(n)).astype(np.float32)))
    out.append(("cancelling", g, (-g + (rng.integers(-2, 3, n) * 2.0 ** -20).astype(np.float32)).astype(np.float32)))
    scale = (2.0 ** rng.integers(-40, 40, n)).astype(np.float32)
    out.append(("wide_exponents", (g * scale).astype(np.float32),
                (rng.standard_normal(n) * 2.0 ** rng.integers(-40, 40, n)).astype(np.float32)))
    den = rng.integers(1, 1 << 22, n).astype(np.uint32).view(np.float32)
    out.append(("denormals", den * np.where(rng.random(n) < 0.5, -1, 1).astype(np.float32),
                rng.integers(0, 1 << 22, n).astype(np.uint32).view(np.float32)))
    q = rng.integers(-3, 4, n).astype(np.float32) * 0.25
    out.append(("quantised_ties", q, rng.integers(-3, 4, n).astype(np.float32) * 0.25))
    out.append(("zero_residual", g, np.zeros(n, dtype=np.float32)))
    return out


@pytest.mark.parametrize("n", [1, 7, 33])
def test_error_feedback_against_rank_counting(n):
    for name, g, e in ef_vectors(n, 100 + n):
        w = g + e  # numpy's float32 addition: an IEEE-754 library routine, not the oracle's code
        assert np.array_equal(bits(oracle.ef_accumulate(g, e)), bits(w)), name
        keys = keys_of(w)
        rank = brute_rank(keys)
        for k in sorted({1, (n + 1) // 2, n}):
            thr = oracle.ef_select_threshold(g, e, k)
            tau = int(keys[np.nonzero(rank == k - 1)[0][0]])
            assert thr.tau_key == tau, (name, k)
            assert thr.n_gt == int((keys > tau).sum()) and thr.n_eq == int((keys == tau).sum())
            idx, val, cnt, e_out = oracle.ef_threshold_compact(g, e, thr, oracle.EXACT_K)
            want = np.nonzero(rank < k)[0]
            assert cnt == k and np.array_equal(idx, want.astype(np.int32)), (name, k)
            assert np.array_equal(bits(val), bits(w[want]))
            expect_e = w.copy()
            expect_e[want] = 0.0
            assert np.array_equal(bits(e_out), bits(expect_e)), (name, k)
            idx, val, cnt, e_out = oracle.ef_threshold_compact(g, e, thr, oracle.GE_TAU)
            want = np.nonzero(keys >= tau)[0]
            assert cnt == want.size and np.array_equal(idx, want.astype(np.int32))
            expect_e = w.copy()
            expect_e[want] = 0.0
            assert np.array_equal(bits(e_out), bits(expect_e)), (name, k)


@settings(max_examples=40, deadline=None)
@given(n=st.integers(1, 3000), frac=st.floats(0.001, 1.0), seed=st.integers(0, 2**31 - 1),
       which=st.integers(0, 5), cap_frac=st.floats(0.0, 1.5))
def test_error_feedback_conservation_property(n, frac, seed, which, cap_frac):
    """Nothing is lost and nothing is invented: what is delivered plus what stays
    in the residual is the corrected gradient, bit for bit, at every position; a
    delivered position has residual +0; with zero residual the result is that of
    the plain path."""
    name, g, e = ef_vectors(n, seed)[which]
    w = g + e
    k = max(1, min(n, int(round(frac * n))))
    thr = oracle.ef_select_threshold(g, e, k)
    assert thr == oracle.select_threshold(w, k)
    cap = int(cap_frac * n)
    for mode in (oracle.GE_TAU, oracle.EXACT_K):
        idx, val, cnt, e_out = oracle.ef_threshold_compact(g, e, thr, mode, capacity=cap)
        pidx, pval, pcnt = oracle.threshold_compact(w, thr, mode, capacity=cap)
        assert cnt == pcnt and np.array_equal(idx, pidx) and np.array_equal(bits(val), bits(pval))
        delivered = np.zeros(n, dtype=bool)
        delivered[idx] = True
        assert np.all(bits(e_out)[delivered] == 0)
        assert np.array_equal(bits(e_out)[~delivered], bits(w)[~delivered])
        assert np.array_equal(bits(val), bits(w[idx]))
        finite = np.isfinite(w)
        total = scatter(n, idx, val) + e_out  # one of the two terms is +0 at every position
        assert np.array_equal(total[finite], w[finite])


def test_error_feedback_residual_is_eventually_delivered():
    """The point of the residual (Fig. 3): a coordinate whose gradient is always
    below the threshold is still delivered once its accumulated value crosses it."""
    n, k = 64, 4
    g = np.full(n, 0.125, dtype=np.float32)
    g[:4] = 1.0                       # four large coordinates fix tau = 1.0
    e = np.zeros(n, dtype=np.float32)
    thr = oracle.ef_select_threshold(g, e, k)
    assert thr.tau_key == int(np.float32(1.0).view(np.uint32))
    first_delivery = None
    for it in range(1, 10):
        idx, val, cnt, e = oracle.ef_threshold_compact(g, e, thr, oracle.GE_TAU)
        if first_delivery is None and cnt > 4:
            first_delivery = it
            assert cnt == n and np.all(val[4:] == 1.0)   # 8 * 0.125, summed exactly
            assert np.all(e == 0.0)
    assert first_delivery == 8


# ------------------------------------------------------------------ receiver side: decompression
def test_scatter_hand_worked():
    """The message of iteration 1 of the error-feedback fixture, put back into a dense vector."""
    out = oracle.scatter(i32(["1", "4"]), f32(["-1.5", "-1.25"]), 8)
    assert np.array_equal(bits(out), bits(f32("0 -1.5 0 0 -1.25 0 0 0".split())))
    # server-side accumulation of two workers' messages (distinct positions, then a shared one)
    acc = np.zeros(8, dtype=np.float32)
    oracle.scatter(i32(["1", "4"]), f32(["-1.5", "-1.25"]), 8, out=acc, mode=oracle.SCATTER_ADD)
    oracle.scatter(i32(["0", "4", "7"]), f32(["0.5", "0.25", "2"]), 8, out=acc, mode=oracle.SCATTER_ADD)
    assert np.array_equal(bits(acc), bits(f32("0.5 -1.5 0 0 -1.0 0 0 2".split())))
    # nothing to deliver: all zeros; indices outside the vector are skipped
    assert np.all(bits(oracle.scatter(i32([]), f32([]), 5)) == 0)
    out = oracle.scatter(i32(["-1", "2", "5"]), f32(["9", "3", "9"]), 5)
    assert np.array_equal(out, f32("0 0 3 0 0".split()))


@pytest.mark.parametrize("bf16", [False, True])
def test_scatter_against_numpy_indexing(bf16):
    rng = np.random.default_rng(5)
    for n, c in [(1, 1), (10, 3), (1000, 0), (1000, 1000), (70_001, 700)]:
        idx = np.sort(rng.choice(n, size=c, replace=False)).astype(np.int32)
        val = rng.standard_normal(c).astype(np.float32)
        if bf16:
            val = to_bf16_bits(val)
        want = np.zeros(n, dtype=val.dtype)
        want[idx] = val  # numpy fancy indexing: a library routine
        assert np.array_equal(bits(oracle.scatter(idx, val, n)), bits(want))
        if not bf16:
            base = rng.standard_normal(n).astype(np.float32)
            want = base.copy()
            want[idx] += val
            got = oracle.scatter(idx, val, n, out=base.copy(), mode=oracle.SCATTER_ADD)
            assert np.array_equal(bits(got), bits(want))
    with pytest.raises(ValueError):
        oracle.scatter(i32(["0"]), to_bf16_bits(f32(["1"])), 4, out=np.zeros(4, dtype=np.uint16),
                       mode=oracle.SCATTER_ADD)


@settings(max_examples=30, deadline=None)
@given(n=st.integers(1, 3000), frac=st.floats(0.001, 1.0), seed=st.integers(0, 2**31 - 1), bf16=st.booleans())
def test_compress_then_decompress_is_the_masked_gradient(n, frac, seed, bf16):
    """Decompressing the message gives W_grad . M, and with error feedback the
    decompressed message plus the new residual is the corrected gradient."""
    rng = np.random.default_rng(seed)
    g = (rng.integers(-6, 7, n) * 0.25).astype(np.float32) if seed % 2 else rng.standard_normal(n).astype(np.float32)
    gq = to_bf16_bits(g) if bf16 else g
    k = max(1, min(n, int(round(frac * n))))
    thr = oracle.select_threshold(gq, k)
    idx, val, cnt = oracle.threshold_compact(gq, thr, oracle.GE_TAU)
    mask = keys_of(gq) >= thr.tau_key
    want = np.where(mask, gq, np.zeros_like(gq))
    assert np.array_equal(bits(oracle.scatter(idx, val, n)), bits(want))
    if not bf16:
        e = (0.5 * rng.standard_normal(n)).astype(np.float32)
        thr = oracle.ef_select_threshold(g, e, k)
        idx, val, cnt, e_out = oracle.ef_threshold_compact(g, e, thr, oracle.EXACT_K)
        assert np.array_equal(oracle.scatter(idx, val, n) + e_out, g + e)


def test_rowscatter_against_numpy_and_round_trip():
    rng = np.random.default_rng(9)
    B, D, k = 7, 40, 6
    x = np.maximum(rng.standard_normal((B, D)), 0).astype(np.float32)
    x[3, :] = 0
    x[3, 5] = -2.0
    for xq in (x, to_bf16_bits(x.reshape(-1)).reshape(B, D)):
        idx, val, tau = oracle.rowtopk_fwd(xq, k)
        want = np.zeros_like(xq)
        np.put_along_axis(want, idx.astype(np.int64), val, axis=1)  # library routine
        got = oracle.rowscatter(idx, val, D)
        assert np.array_equal(bits(got.reshape(-1)), bits(want.reshape(-1)))
        # the dense result is X_act . M: kept entries equal x, the rest is zero
        keep = np.zeros((B, D), dtype=bool)
        np.put_along_axis(keep, idx.astype(np.int64), True, axis=1)
        assert np.array_equal(bits(got[keep]), bits(xq[keep])) and np.all(bits(got[~keep]) == 0)
        # gathering the dense result through the same mask returns the values
        assert np.array_equal(bits(oracle.rowtopk_bwd(got, idx).reshape(-1)), bits(val.reshape(-1)))
    # a wider output buffer: the padding is not touched; columns outside [0, D) are skipped
    buf = np.full((B, D + 8), 7, dtype=np.float32)
    idx, val, _ = oracle.rowtopk_fwd(x, k)
    idx2 = idx.copy()
    idx2[0, 0] = D + 3
    oracle.rowscatter(idx2, val, D, out=buf[:, :D])
    assert np.all(buf[:, D:] == 7)
    want = np.zeros((B, D), dtype=np.float32)
    np.put_along_axis(want, idx.astype(np.int64), val, axis=1)
    want[0, idx[0, 0]] = 0
    assert np.array_equal(buf[:, :D], want)


# ------------------------------------------------------------------ Algorithm 2 with the mask as a bitmap
def test_bitmask_hand_worked():
    """Rows of the Algorithm 2 fixture: the mask words follow from the kept columns by hand."""
    gd = read_golden("alg2_worked.txt")
    k = int(gd["k"][0])
    x = np.stack([f32(gd[f"x{b}"]) for b in range(3)])
    mask, val, tau = oracle.rowtopk_fwd_bitmask(x, k)
    assert mask.shape == (3, 1)
    for b in range(3):
        cols = [int(c) for c in gd[f"idx{b}"]]
        word = 0
        for c in cols:            # bit c of the row's only word (D <= 32 in the fixture)
            word |= 1 << c
        assert int(mask[b, 0]) == word, b
        assert np.array_equal(bits(val[b]), bits(f32(gd[f"val{b}"])))
    # a row of 40 columns with columns 0, 31, 32 and 39 kept: words 0x80000001 and 0x00000081
    x = np.zeros((1, 40), dtype=np.float32)
    x[0, [0, 31, 32, 39]] = [4.0, -3.0, 2.0, 1.0]
    mask, val, _ = oracle.rowtopk_fwd_bitmask(x, 4)
    assert [int(w) for w in mask[0]] == [0x80000001, 0x00000081]
    assert val[0].tolist() == [4.0, -3.0, 2.0, 1.0]


@pytest.mark.parametrize("bf16", [False, True])
def test_bitmask_against_numpy_packbits_and_index_form(bf16):
    rng = np.random.default_rng(17)
    for B, D, k in [(5, 33, 7), (4, 64, 64), (6, 1000, 50), (3, 4096, 204)]:
        x = np.maximum(rng.standard_normal((B, D)), 0).astype(np.float32)
        dy = rng.standard_normal((B, D)).astype(np.float32)
        if bf16:
            x = to_bf16_bits(x.reshape(-1)).reshape(B, D)
            dy = to_bf16_bits(dy.reshape(-1)).reshape(B, D)
        idx, val, tau = oracle.rowtopk_fwd(x, k)
        mask, mval, mtau = oracle.rowtopk_fwd_bitmask(x, k)
        keep = np.zeros((B, ((D + 31) // 32) * 32), dtype=np.uint8)
        np.put_along_axis(keep, idx.astype(np.int64), 1, axis=1)
        want = np.packbits(keep, axis=1, bitorder="little").view(np.uint32)  # library routine
        assert np.array_equal(mask, want)
        assert np.array_equal(bits(mval.reshape(-1)), bits(val.reshape(-1))) and np.array_equal(mtau, tau)
        assert np.all(np.unpackbits(mask.view(np.uint8), axis=1).sum(axis=1) == k)
        # backward and decompression agree with the index form
        assert np.array_equal(oracle.rowtopk_bwd_bitmask(dy, mask, k), oracle.rowtopk_bwd(dy, idx))
        assert np.array_equal(oracle.rowscatter_bitmask(mask, mval, D), oracle.rowscatter(idx, val, D))
    # a mask with fewer set bits than k: the remaining slots are zero
    m = np.array([[0b1010]], dtype=np.uint32)
    d = oracle.rowtopk_bwd_bitmask(f32("1 2 3 4 5".split()).reshape(1, 5), m, 3)
    assert d.tolist() == [[2.0, 4.0, 0.0]]


# ------------------------------------------------------------------ Algorithm 2 with 16-bit column indices
def test_idx16_hand_worked_and_limits():
    """The fixture's kept columns, stored in 16 bits; the widest row whose last column still fits."""
    gd = read_golden("alg2_worked.txt")
    k = int(gd["k"][0])
    x = np.stack([f32(gd[f"x{b}"]) for b in range(3)])
    idx, val, tau = oracle.rowtopk_fwd_idx16(x, k)
    assert idx.dtype == np.uint16
    for b in range(3):
        assert idx[b].tolist() == [int(c) for c in gd[f"idx{b}"]], b
        assert np.array_equal(bits(val[b]), bits(f32(gd[f"val{b}"])))
    # D = 65536: column 65535 is the largest magnitude and must come back as 0xFFFF
    x = np.zeros((1, 65536), dtype=np.float32)
    x[0, 65535] = -9.0
    x[0, 32768] = 5.0
    x[0, 7] = 1.0
    idx, val, tau = oracle.rowtopk_fwd_idx16(x, 3)
    assert idx[0].tolist() == [7, 32768, 65535] and val[0].tolist() == [1.0, 5.0, -9.0] and tau[0] == 1.0
    with pytest.raises(ValueError):
        oracle.rowtopk_fwd_idx16(np.zeros((1, 65537), dtype=np.float32), 3)
    with pytest.raises(ValueError):   # an index past the row's end is an error of the backward pass
        oracle.rowtopk_bwd_idx16(np.zeros((1, 8), dtype=np.float32), np.array([[8]], dtype=np.uint16))
    # decompression skips such an index
    out = oracle.rowscatter_idx16(np.array([[1, 9]], dtype=np.uint16), f32(["2", "3"]).reshape(1, 2), 8)
    assert out.tolist() == [[0, 2.0, 0, 0, 0, 0, 0, 0]]


@pytest.mark.parametrize("bf16", [False, True])
def test_idx16_against_numpy_stable_sort_gather_and_put(bf16):
    rng = np.random.default_rng(23)
    for B, D, k in [(5, 33, 7), (4, 64, 64), (6, 1000, 50), (2, 40000, 123)]:
        x = np.maximum(rng.standard_normal((B, D)), 0).astype(np.float32)
        dy = rng.standard_normal((B, D)).astype(np.float32)
        if bf16:
            x = to_bf16_bits(x.reshape(-1)).reshape(B, D)
            dy = to_bf16_bits(dy.reshape(-1)).reshape(B, D)
            keys = (x & 0x7FFF).astype(np.int64)
        else:
            keys = (x.view(np.uint32) & 0x7FFFFFFF).astype(np.int64)
        # library routines: a stable sort by descending key keeps the lower column first among equals
        order = np.argsort(-keys, axis=1, kind="stable")[:, :k]
        want_idx = np.sort(order, axis=1)
        idx, val, tau = oracle.rowtopk_fwd_idx16(x, k)
        assert np.array_equal(idx.astype(np.int64), want_idx)
        assert np.array_equal(val, np.take_along_axis(x, want_idx, axis=1))
        assert np.array_equal(oracle.rowtopk_bwd_idx16(dy, idx), np.take_along_axis(dy, want_idx, axis=1))
        dense = np.zeros((B, D), dtype=val.dtype)
        np.put_along_axis(dense, want_idx, val, axis=1)
        assert np.array_equal(oracle.rowscatter_idx16(idx, val, D), dense)
