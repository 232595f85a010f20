"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Everything is integer / bit-copy work, so the bar is
bit-exact: threshold words, counts, indices and copied values (0 ULP).
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dct():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2010_08899_amd as m
    m.lib()
    return m


DEV = torch.device("cuda:0")


def host(t):
    return oracle.as_numpy(t.detach().cpu())


def bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a.view(np.uint16)


class DP:
    """Buffers for one vector size; reused across calls like a training loop would."""

    def __init__(self, dct, g, capacity=None):
        self.dct, self.g = dct, g
        n = g.numel()
        self.cap = n if capacity is None else capacity
        self.thr = torch.zeros(4, dtype=torch.int32, device=g.device)
        self.idx = torch.full((max(self.cap, 1),), -7, dtype=torch.int32, device=g.device)
        self.val = torch.zeros(max(self.cap, 1), dtype=g.dtype, device=g.device)
        self.count = torch.zeros(1, dtype=torch.int64, device=g.device)
        self.sel_ws = dct.new_select_workspace(g)
        self.ws = dct.new_compact_workspace(g)

    def select(self, k, g=None):
        self.dct.dct_select_threshold(self.g if g is None else g, k, self.thr, self.sel_ws)
        return oracle.Threshold(*self.dct.read_threshold(self.thr))

    def compact(self, mode, g=None, capacity=None):
        cap = self.cap if capacity is None else capacity
        self.idx.fill_(-7)
        self.dct.dct_threshold_compact(self.g if g is None else g, self.thr, mode, self.idx, self.val, self.count,
                                       self.ws, capacity=cap)
        c = self.dct.read_count(self.count)
        m = min(c, cap)
        return host(self.idx[:m]), host(self.val[:m]), c, host(self.idx[m:m + 16])


def check_dp(dct, g, k, modes=(0, 1), select_method="sort"):
    gh = host(g)
    dp = DP(dct, g)
    thr = dp.select(k)
    exp = oracle.select_threshold(gh, k, method=select_method)
    assert thr == exp, (thr, exp)
    for mode in modes:
        idx, val, cnt, guard = dp.compact(mode)
        eidx, eval_, ecnt = oracle.threshold_compact(gh, exp, mode)
        assert cnt == ecnt
        assert np.array_equal(idx, eidx)
        assert np.array_equal(bits(val), bits(eval_))
        assert np.all(guard == -7)  # nothing written past the survivors
    return dp, exp


# ------------------------------------------------------------------ DP: sizes, tails, alignment
@pytest.mark.parametrize("n", [1, 2, 5, 63, 64, 1000, 8191, 8192, 8193, 3 * 8192 + 17, 100_003, 1_000_000])
def test_dp_sizes(dct, n):
    g = si.gaussian_gradient(n, DEV, 100 + n)
    for k in sorted({1, max(1, n // 100), max(1, n // 2), n}):
        check_dp(dct, g, k)


@pytest.mark.parametrize("shift", [1, 2, 3])
def test_dp_misaligned_base(dct, shift):
    buf = si.gaussian_gradient(50_000 + shift, DEV, 7)
    g = buf[shift:]
    assert g.data_ptr() % 16 != 0
    check_dp(dct, g, 500)
    check_dp(dct, g[:5], 2)


@pytest.mark.parametrize("n", [40, 20_000])
def test_dp_adversarial_values(dct, n):
    for name, g in si.adversarial_vectors(n, DEV, 900 + n):
        for k in sorted({1, 3, n // 7 + 1, n // 2, n}):
            check_dp(dct, g.contiguous(), k)
    g = si.gaussian_gradient(n, DEV, 5)
    g[n // 3] = float("nan")
    g[0] = float("inf")
    check_dp(dct, g, 3)


def test_dp_bf16(dct):
    for n in (10, 16384, 16385, 70_001):
        g = si.gaussian_gradient(n, DEV, 300 + n, scale=1.0).to(torch.bfloat16)
        for k in (1, max(1, n // 100), n):
            check_dp(dct, g, k)
    check_dp(dct, g[1:], 100)  # 2-byte-aligned base


@pytest.mark.parametrize("frac", [0.02, 0.05, 0.10, 0.25, 0.50, 0.90, 0.999])
def test_dp_low_sparsity_levels(dct, frac):
    """The paper's lower compression levels (a quarter of the vector kept, and beyond): sampled
    selection with many candidates, compaction with more survivors than fit on chip."""
    n = 5_000_011
    g = si.gaussian_gradient(n, DEV, 2200)
    check_dp(dct, g, int(n * frac), select_method="nth")
    t3 = si.student_t3_gradient(n, DEV, 2201)
    check_dp(dct, t3, int(n * frac), modes=(0,), select_method="nth")


def test_dp_c1_full(dct):
    g, k = si.config_c1(DEV)
    dp, thr = check_dp(dct, g, k)
    assert abs(np.array([thr.tau_key], dtype=np.uint32).view(np.float32)[0] / 2.5758e-3 - 1) < 0.02
    # determinism: a second run gives the same bits
    a = dp.compact(1)
    b = dp.compact(1)
    assert np.array_equal(a[0], b[0]) and np.array_equal(bits(a[1]), bits(b[1])) and a[2] == b[2] == k


def test_dp_overflow_prefix_and_empty(dct):
    g = si.gaussian_gradient(200_000, DEV, 11)
    gh = host(g)
    dp = DP(dct, g)
    thr = dp.select(2000)
    full = oracle.threshold_compact(gh, thr, oracle.GE_TAU)
    idx, val, cnt, guard = dp.compact(0, capacity=777)
    assert cnt == full[2] == 2000 and np.array_equal(idx, full[0][:777]) and np.array_equal(val, full[1][:777])
    assert np.all(guard == -7)
    with pytest.raises(dct.DctError):
        dct.read_count(dp.count, capacity=777)
    idx, val, cnt, _ = dp.compact(1, capacity=0)
    assert cnt == 2000 and idx.size == 0
    # a stale threshold that nothing reaches: count 0, nothing written
    dp.thr.copy_(torch.tensor([0x7F000000, 0, 0, 0], dtype=torch.int32))
    idx, val, cnt, guard = dp.compact(0)
    assert cnt == 0 and np.all(guard == -7)
    # a stale threshold of zero keeps everything
    dp.thr.zero_()
    idx, val, cnt, _ = dp.compact(0)
    assert cnt == g.numel() and np.array_equal(idx, np.arange(g.numel())) and np.array_equal(bits(val), bits(gh))


def test_dp_argument_and_workspace_errors(dct):
    g = si.gaussian_gradient(10_000, DEV, 12)
    dp = DP(dct, g)
    for k in (0, g.numel() + 1):
        with pytest.raises(dct.DctError) as e:
            dp.select(k)
        assert e.value.status == 1
    small = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(dct.DctError) as e:
        dct.dct_select_threshold(g, 5, dp.thr, small)
    assert e.value.status == 2
    dp.select(100)
    with pytest.raises(dct.DctError) as e:
        dct.dct_threshold_compact(g, dp.thr, 0, dp.idx, dp.val, dp.count, small[:16])
    assert e.value.status == 2
    with pytest.raises(dct.DctError):
        dct.dct_threshold_compact(g, dp.thr, 5, dp.idx, dp.val, dp.count, dp.ws)
    # a workspace that was never initialised is reported through the count, no hang
    raw = torch.zeros(dp.ws.numel(), dtype=torch.uint8, device=DEV)
    dct.dct_threshold_compact(g, dp.thr, 0, dp.idx, dp.val, dp.count, raw)
    with pytest.raises(dct.DctError) as e:
        dct.read_count(dp.count)
    assert e.value.status == 2
    # and the initialised one still works afterwards
    idx, val, cnt, _ = dp.compact(1)
    assert cnt == 100


# ------------------------------------------------------------------ DP: large vectors (sampled select) and its fallback
@pytest.mark.parametrize("case", ["gauss", "k1", "kn", "all_equal", "few_levels", "spike_block", "misaligned"])
def test_dp_sampled_select_and_fallback(dct, case):
    # n is above the size from which the threshold is bracketed from a sample and the radix passes
    # run over the candidates; several cases make the bracket fail (ties wider than the candidate
    # buffer, k = n) so that the device-side fallback to passes over the whole vector is taken.
    n = (1 << 22) + 12345
    g = si.gaussian_gradient(n, DEV, 4242)
    k = n // 200
    sel = "nth"
    if case == "k1":
        k = 1
    elif case == "kn":
        k = n
    elif case == "all_equal":
        g = torch.full((n,), -0.125, device=DEV)
    elif case == "few_levels":
        g = (torch.randint(0, 5, (n,), device=DEV, generator=torch.Generator(device=DEV).manual_seed(7)).float() - 2.0)
        k = n // 3
    elif case == "spike_block":
        # the k largest magnitudes all sit in one short block that a stratified sample barely sees
        g = g * 1e-3
        g[1_000_000:1_000_000 + 3000] = 5.0 + torch.arange(3000, device=DEV) * 1e-3
        k = 2500
    elif case == "misaligned":
        g = g[3:]
    dp, thr = check_dp(dct, g.contiguous() if case != "misaligned" else g, k, select_method=sel)
    assert thr == oracle.select_threshold(host(g), k, method="sort")


@pytest.mark.parametrize("case", ["gauss", "all_equal", "few_levels", "mostly_zero", "misaligned"])
def test_dp_sampled_select_long_vectors(dct, case):
    """The same from 2^26 elements on, where the partition pass takes 8 KiB pieces: candidates, candidate overflow
    (the passes then run over the keys of the vector inside the bounds) and a misaligned base."""
    n = (1 << 26) + 12345
    g = si.gaussian_gradient(n, DEV, 4343)
    k = n // 200
    if case == "all_equal":
        g = torch.full((n,), 0.375, device=DEV)
    elif case == "few_levels":
        g = (torch.randint(0, 5, (n,), device=DEV, generator=torch.Generator(device=DEV).manual_seed(8)).float() - 2.0)
        k = n // 3
    elif case == "mostly_zero":
        g[torch.rand(n, device=DEV, generator=torch.Generator(device=DEV).manual_seed(9)) < 0.9] = 0.0
        k = n // 5       # beyond the non-zeros: tau = 0
    elif case == "misaligned":
        g = g[1:]
    check_dp(dct, g, k, select_method="nth")


# ------------------------------------------------------------------ DP: c3 (select once, reuse on fresh draws)
@pytest.mark.parametrize("chunk", range(4))
def test_dp_c3_reuse(dct, chunk):
    draws_per_chunk = si.C3_DRAWS // 4
    g0 = si.config_c3_draw(DEV, 0)
    dp = DP(dct, g0, capacity=si.C3_CAPACITY)
    thr = dp.select(si.C3_K)
    if chunk == 0:
        exp = oracle.select_threshold(host(g0), si.C3_K)
        assert thr == exp
        tau = np.array([thr.tau_key], dtype=np.uint32).view(np.float32)[0]
        assert abs(tau / 12.92e-3 - 1) < 0.03
    else:
        assert thr == oracle.select_threshold(host(g0), si.C3_K, method="nth")
    del g0
    counts = []
    for j in range(1 + chunk * draws_per_chunk, 1 + (chunk + 1) * draws_per_chunk):
        g = si.config_c3_draw(DEV, j)
        idx, val, cnt, guard = dp.compact(0, g=g)
        eidx, eval_, ecnt = oracle.threshold_compact(host(g), thr, oracle.GE_TAU, capacity=si.C3_CAPACITY)
        assert cnt == ecnt <= si.C3_CAPACITY, j
        assert np.array_equal(idx, eidx) and np.array_equal(bits(val), bits(eval_)), j
        counts.append(cnt)
    counts = np.array(counts)
    assert abs(counts.mean() / si.C3_K - 1) < 0.05 and counts.std() > 10  # fluctuates around k


# ------------------------------------------------------------------ DP: c4 (embedding-shaped, 95 % exact zeros)
def test_dp_c4_reduced_full_sort(dct):
    g, k = si.config_c4(DEV, rows=1 << 18)  # N = 2^24: the oracle's full sort takes seconds
    check_dp(dct, g, k)
    # k larger than the number of non-zeros: tau = 0 and the lowest-index zeros fill up
    check_dp(dct, g, g.numel() // 10, modes=(1,))


def test_dp_c4_full(dct):
    g, k = si.config_c4(DEV)
    assert g.numel() == 1 << 28 and k == 1342178
    dp, thr = check_dp(dct, g, k, modes=(1,), select_method="nth")
    tau = np.array([thr.tau_key], dtype=np.uint32).view(np.float32)[0]
    assert abs(tau / 1.645 - 1) < 0.01


# ------------------------------------------------------------------ MP
def check_mp(dct, x, dy, k, with_tau=True):
    B, D = x.shape
    idx = torch.full((B, k), -7, dtype=torch.int32, device=DEV)
    val = torch.zeros(B, k, dtype=x.dtype, device=DEV)
    tau = torch.zeros(B, dtype=x.dtype, device=DEV) if with_tau else None
    dval = torch.zeros(B, k, dtype=x.dtype, device=DEV)
    dct.dct_rowtopk_fwd(x, k, idx, val, tau)
    dct.dct_rowtopk_bwd(dy, idx, dval)
    xh, dyh = host(x), host(dy)
    eidx, eval_, etau = oracle.rowtopk_fwd(xh, k)
    edval = oracle.rowtopk_bwd(dyh, eidx)
    assert np.array_equal(host(idx), eidx)
    assert np.array_equal(bits(host(val)), bits(eval_))
    if with_tau:
        assert np.array_equal(bits(host(tau)), bits(etau))
    assert np.array_equal(bits(host(dval)), bits(edval))
    return idx, val, dval


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("D", [1, 3, 64, 65, 500, 1000, 1024, 2048, 4096, 5000])
def test_mp_shapes(dct, dtype, D):
    B = 37
    for stride in (None, D + 3, D + 8):
        x = si.relu_activations(B, D, DEV, 40 + D, dtype=dtype, row_stride=stride)
        dy = si.normal_matrix(B, D, DEV, 41 + D, dtype=dtype, row_stride=stride)
        for k in sorted({1, max(1, D // 20), max(1, D // 2), D}):
            check_mp(dct, x, dy, k, with_tau=(k % 2 == 1))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_mp_signed_and_tie_heavy_rows(dct, dtype):
    D = 777
    rows = [t for _, t in si.adversarial_vectors(D, DEV, 55)]
    x = torch.stack(rows).to(dtype)
    dy = si.normal_matrix(x.shape[0], D, DEV, 56, dtype=dtype)
    for k in (1, 38, 400, D):
        check_mp(dct, x, dy, k)
    xs = si.normal_matrix(64, 1024, DEV, 57, dtype=dtype)  # split before the activation: signed entries
    check_mp(dct, xs, si.normal_matrix(64, 1024, DEV, 58, dtype=dtype), 51)


@pytest.mark.parametrize("D", [1024, 4096])
def test_mp_bf16_on_chip_kernel_hard_rows(dct, D):
    # rows that defeat the previous-row threshold prediction of the on-chip bf16 kernel (wildly
    # different scales from row to row), rows of ties, zeros, infinities and NaNs, fewer than k non-zeros
    rows = [t for _, t in si.adversarial_vectors(D, DEV, 71)]
    scales = [1e-30, 1e30, 1.0, 1e-3, 3e4, 1e-10]
    gen = torch.Generator(device=DEV).manual_seed(72)
    for s_ in scales:
        rows.append(torch.randn(D, device=DEV, generator=gen) * s_)
    sparse = torch.zeros(D, device=DEV)
    sparse[5::97] = 2.0
    rows.append(sparse)
    nanrow = torch.randn(D, device=DEV, generator=gen)
    nanrow[7] = float("nan")
    nanrow[D - 1] = float("nan")
    rows.append(nanrow)
    rows.append(torch.full((D,), float("nan"), device=DEV))
    x = torch.stack(rows * 3).to(torch.bfloat16)
    x = x[torch.randperm(x.shape[0], device=DEV, generator=gen)].contiguous()
    dy = si.normal_matrix(x.shape[0], D, DEV, 73, dtype=torch.bfloat16)
    for k in (1, 7, D // 20, D // 2, D):
        check_mp(dct, x, dy, k)


@pytest.mark.parametrize("dtype,B,D,k", [
    (torch.float32, 16390, 256, 12), (torch.float32, 16384, 512, 25), (torch.float32, 20000, 200, 10),
    (torch.bfloat16, 16400, 1024, 200), (torch.bfloat16, 16385, 2048, 102), (torch.float32, 16401, 1024, 51),
    # 8 KiB rows on both sides of the batch size from which the large workgroups are used
    (torch.bfloat16, 16383, 4096, 204), (torch.bfloat16, 16385, 4096, 204), (torch.float32, 16390, 2048, 102)])
def test_mp_many_rows_of_up_to_4_kib(dct, dtype, B, D, k):
    """From 16 k rows on the one-row-per-wavefront kernel runs as one workgroup of 16 wavefronts per CU that take
    their rows from a counter (rows of up to 2 KiB and of 8 KiB; 4 KiB rows keep the small workgroups)."""
    x = si.relu_activations(B, D, DEV, 2800 + D, dtype=dtype)
    x[3] = 0.5
    x[B - 2] = 0.0
    dy = si.normal_matrix(B, D, DEV, 2801 + D, dtype=dtype)
    check_mp(dct, x, dy, k)


@pytest.mark.parametrize("D", [256, 1024, 2048, 4096])
def test_mp_fp32_on_chip_kernel_hard_rows(dct, D):
    """fp32 rows for the on-chip kernel: its search runs on the upper halves of the keys, so the hard
    cases are many keys that share an upper half -- with equal lower halves (constants, zeros), with
    distinct ones (a narrow band of values), a handful of them, and more than a wavefront of them."""
    gen = torch.Generator(device=DEV).manual_seed(172)
    rows = [t for _, t in si.adversarial_vectors(D, DEV, 171)]
    for s_ in (1e-30, 1e30, 1.0, 1e-3):
        rows.append(torch.randn(D, device=DEV, generator=gen) * s_)
    step = torch.arange(D, device=DEV, dtype=torch.float32)
    perm = torch.randperm(D, device=DEV, generator=gen)
    rows.append(1.0 + step[perm] * 2.0 ** -20)                     # every key in one upper-half bin, all distinct
    rows.append(-(1.0 + (step[perm] % 37) * 2.0 ** -18))           # the same with repeats
    band = torch.randn(D, device=DEV, generator=gen)
    band[perm[: min(50, D // 4)]] = 3.0 + step[: min(50, D // 4)] * 2.0 ** -21     # a handful sharing the top bin
    rows.append(band)
    band2 = torch.randn(D, device=DEV, generator=gen) * 0.1
    band2[perm[: D // 2]] = 2.0 + step[: D // 2] * 2.0 ** -22                       # more than 64 sharing it
    rows.append(band2)
    sparse = torch.zeros(D, device=DEV)
    sparse[5::97] = 2.0
    rows.append(sparse)
    nanrow = torch.randn(D, device=DEV, generator=gen)
    nanrow[7] = float("nan")
    rows.append(nanrow)
    x = torch.stack(rows * 3).contiguous()
    x = x[torch.randperm(x.shape[0], device=DEV, generator=gen)].contiguous()
    dy = si.normal_matrix(x.shape[0], D, DEV, 173)
    for k in (1, 7, D // 20, D // 2, D):
        check_mp(dct, x, dy, k)


def test_mp_c2_full(dct):
    x, dy, k = si.config_c2(DEV)
    idx, val, dval = check_mp(dct, x, dy, k)
    idx2 = torch.zeros_like(idx)
    val2 = torch.zeros_like(val)
    dct.dct_rowtopk_fwd(x, k, idx2, val2, None)
    assert torch.equal(idx, idx2) and torch.equal(val.view(torch.int32), val2.view(torch.int32))


def test_mp_c5_full(dct):
    x, dy, k = si.config_c5(DEV)
    assert x.shape == (65536, 4096) and k == 204
    check_mp(dct, x, dy, k)


def test_mp_bwd_out_of_range_index_is_not_dereferenced(dct):
    dy = si.normal_matrix(4, 100, DEV, 60)
    idx = torch.tensor([[0, 5, 99], [1, 100, 2], [-1, 3, 4], [7, 8, 2 ** 31 - 1]], dtype=torch.int32, device=DEV)
    dval = torch.full((4, 3), 9.0, device=DEV)
    dct.dct_rowtopk_bwd(dy, idx, dval)
    d = dval.cpu()
    dyh = dy.cpu()
    assert d[0].tolist() == [dyh[0, 0].item(), dyh[0, 5].item(), dyh[0, 99].item()]
    assert d[1, 1] == 0 and d[2, 0] == 0 and d[3, 2] == 0 and d[1, 0] == dyh[1, 1]


@pytest.mark.parametrize("dtype,B,D,k,pad,idx16", [
    (torch.bfloat16, 16384, 4096, 204, 0, False), (torch.bfloat16, 16391, 2048, 300, 0, True),
    (torch.float32, 16385, 1024, 40, 8, False), (torch.float32, 16400, 2048, 700, 0, True),
    (torch.bfloat16, 20000, 3000, 100, 8, False)])
def test_mp_bwd_many_rows_dense_lists(dct, dtype, B, D, k, pad, idx16):
    """Backward over many rows of 4 to 8 KiB with k >= D / 32: the rows are streamed through LDS (bad indices
    give 0 there too; lists longer than the 256 entries that are fetched ahead; padded rows; both index widths)."""
    dy = si.normal_matrix(B, D, DEV, 2700 + D, dtype=dtype, row_stride=D + pad if pad else None)
    g = torch.Generator(device=DEV)
    g.manual_seed(2701 + D)
    idx = torch.rand(B, D, device=DEV, generator=g).argsort(1)[:, :k].sort(1).values.to(torch.int32)
    clean = idx.clone()     # the oracle takes valid lists only: the three bad entries are checked by hand
    idx[5, 0] = D           # just past the row
    idx[7, k - 1] = 65535 if idx16 else -1
    idx[B - 1, k // 2] = D + 7
    dval = torch.full((B, k), 3.0, device=DEV).to(dtype)
    if idx16:
        dct.dct_rowtopk_bwd_idx16(dy, idx.to(torch.int16), dval)
        want = oracle.rowtopk_bwd_idx16(oracle.as_numpy(dy.cpu()), clean.to(torch.int16).cpu().numpy().view(np.uint16))
    else:
        dct.dct_rowtopk_bwd(dy, idx, dval)
        want = oracle.rowtopk_bwd(oracle.as_numpy(dy.cpu()), clean.cpu().numpy())
    want[5, 0] = want[7, k - 1] = want[B - 1, k // 2] = 0
    got = host(dval)
    assert np.array_equal(bits(got.reshape(-1)), bits(want.reshape(-1)))
    assert got[5, 0] == 0 and got[7, k - 1] == 0 and got[B - 1, k // 2] == 0


@pytest.mark.parametrize("dtype,B,D,k", [
    (torch.bfloat16, 16384, 4096, 204), (torch.float32, 16390, 1024, 51), (torch.bfloat16, 16400, 2048, 512),
    (torch.bfloat16, 16385, 3008, 100), (torch.float32, 16384, 2048, 64)])
def test_mp_bwd_bitmask_many_rows_dense_masks(dct, dtype, B, D, k):
    """Backward through the bitmap over many rows of 4 to 8 KiB: the rows are streamed through LDS.  Masks with
    fewer set bits than k (zeros at the end of the list) and with more (the first k count) are among them."""
    x = si.relu_activations(B, D, DEV, 2900 + D, dtype=dtype)
    dy = si.normal_matrix(B, D, DEV, 2901 + D, dtype=dtype)
    mask = torch.zeros(B, (D + 31) // 32, dtype=torch.int32, device=DEV)
    val = torch.zeros(B, k, dtype=dtype, device=DEV)
    dct.dct_rowtopk_fwd_bitmask(x, k, mask, val, None)
    mask[5, 0] = 0                      # fewer kept columns than k
    mask[9] = 0                         # none at all
    mask[7, -1] = -1                    # more than k
    mask[B - 1, 1] |= 0x0F0F0F0F
    dval = torch.full((B, k), 3.0, device=DEV).to(dtype)
    dct.dct_rowtopk_bwd_bitmask(dy, mask, dval)
    want = oracle.rowtopk_bwd_bitmask(host(dy), mask.cpu().numpy().view(np.uint32), k)
    assert np.array_equal(bits(host(dval).reshape(-1)), bits(want.reshape(-1)))


def test_mp_argument_errors(dct):
    x = si.relu_activations(4, 100, DEV, 61)
    idx = torch.zeros(4, 101, dtype=torch.int32, device=DEV)
    val = torch.zeros(4, 101, device=DEV)
    with pytest.raises(dct.DctError) as e:
        dct.dct_rowtopk_fwd(x, 101, idx, val)
    assert e.value.status == 1
    with pytest.raises(dct.DctError):
        dct.dct_rowtopk_fwd(x, 0, idx[:, :0].contiguous(), val[:, :0].contiguous())


# ------------------------------------------------------------------ DP with error feedback
class EF:
    """Buffers of the error-feedback calls for one vector size."""

    def __init__(self, dct, n, capacity=None, device=DEV):
        self.dct, self.n = dct, n
        self.cap = n if capacity is None else capacity
        self.thr = torch.zeros(4, dtype=torch.int32, device=device)
        self.idx = torch.full((max(self.cap, 1),), -7, dtype=torch.int32, device=device)
        self.val = torch.zeros(max(self.cap, 1), dtype=torch.float32, device=device)
        self.count = torch.zeros(1, dtype=torch.int64, device=device)
        proto = torch.empty(n, dtype=torch.float32, device=device)
        self.sel_ws = dct.new_select_workspace(proto)
        self.ws = dct.new_compact_workspace(proto)

    def select(self, g, e, k):
        self.dct.dct_ef_select_threshold(g, e, k, self.thr, self.sel_ws)
        return oracle.Threshold(*self.dct.read_threshold(self.thr))

    def compact(self, g, e_in, e_out, mode, capacity=None):
        cap = self.cap if capacity is None else capacity
        self.idx.fill_(-7)
        self.dct.dct_ef_threshold_compact(g, e_in, e_out, self.thr, mode, self.idx, self.val, self.count, self.ws,
                                          capacity=cap)
        c = self.dct.read_count(self.count)
        m = min(c, cap)
        return host(self.idx[:m]), host(self.val[:m]), c, host(self.idx[m:m + 16])


def check_ef(dct, g, e, k, modes=(0, 1), capacity=None, in_place=True):
    """Select and compact g + e on the GPU and on the oracle; the residual is
    written to a fresh buffer and, in a second run, over e itself."""
    gh, eh = host(g), host(e)
    ef = EF(dct, g.numel(), capacity)
    thr = ef.select(g, e, k)
    exp = oracle.ef_select_threshold(gh, eh, k)
    assert thr == exp, (thr, exp)
    for mode in modes:
        eidx, eval_, ecnt, e_exp = oracle.ef_threshold_compact(gh, eh, exp, mode, capacity=capacity)
        for place in ((False, True) if in_place else (False,)):
            off = (g.data_ptr() % 16) // 4  # all three vectors sit at the same offset within 16 bytes
            e_in = torch.empty(g.numel() + off, device=g.device)[off:].copy_(e)
            e_out = e_in if place else torch.full((g.numel() + off,), 123.0, device=g.device)[off:]
            idx, val, cnt, guard = ef.compact(g, e_in, e_out, mode)
            assert cnt == ecnt
            assert np.array_equal(idx, eidx)
            assert np.array_equal(bits(val), bits(eval_))
            assert np.all(guard == -7)
            assert np.array_equal(bits(host(e_out)), bits(e_exp)), (mode, place)
            if not place:
                assert torch.equal(e_in.view(torch.int32), e.view(torch.int32))  # the input residual is untouched
    return ef, exp



@pytest.mark.parametrize("n", [1, 2, 5, 63, 64, 1000, 8191, 8193, 3 * 8192 + 17, 100_003, 1_000_000])
def test_dp_ef_sizes(dct, n):
    g = si.gaussian_gradient(n, DEV, 400 + n)
    e = si.residual_vector(n, DEV, 500 + n)
    for k in sorted({1, max(1, n // 100), max(1, n // 2), n}):
        check_ef(dct, g, e, k)


@pytest.mark.parametrize("n", [40, 30_000])
def test_dp_ef_awkward_sums(dct, n):
    """Cancellation to zero, exponents far apart, denormal sums (not flushed), many equal sums."""
    for name, g, e in si.error_feedback_pairs(n, DEV, 700 + n):
        for k in sorted({1, 3, n // 7 + 1, n // 2, n}):
            check_ef(dct, g, e, k)


@pytest.mark.parametrize("shift", [1, 2, 3])
def test_dp_ef_misaligned_base(dct, shift):
    n = 50_000
    gb, eb = si.gaussian_gradient(n + shift, DEV, 17), si.residual_vector(n + shift, DEV, 18)
    g, e = gb[shift:], eb[shift:]
    assert g.data_ptr() % 16 != 0 and g.data_ptr() % 16 == e.data_ptr() % 16
    ef = EF(dct, n)
    gh, eh = host(g), host(e)
    thr = ef.select(g, e, 500)
    exp = oracle.ef_select_threshold(gh, eh, 500)
    assert thr == exp
    ob = torch.full((n + shift,), 5.0, device=DEV)
    idx, val, cnt, _ = ef.compact(g, e, ob[shift:], 1)
    eidx, eval_, ecnt, e_exp = oracle.ef_threshold_compact(gh, eh, exp, 1)
    assert cnt == ecnt and np.array_equal(idx, eidx) and np.array_equal(bits(val), bits(eval_))
    assert np.array_equal(bits(host(ob[shift:])), bits(e_exp))
    assert torch.all(ob[:shift] == 5.0)  # nothing written before the vector
    # vectors at different offsets within 16 bytes are refused
    with pytest.raises(dct.DctError):
        ef.select(g, eb[:n], 500)
    with pytest.raises(dct.DctError):
        ef.compact(g, e, ob[:n], 1)


def test_dp_ef_capacity_keeps_the_rest_in_the_residual(dct):
    n = 200_000
    g, e = si.gaussian_gradient(n, DEV, 21), si.residual_vector(n, DEV, 22)
    check_ef(dct, g, e, 2000, capacity=777)
    check_ef(dct, g, e, 2000, capacity=0)


def test_dp_ef_dense_survivors_second_pass(dct):
    """More survivors than the on-chip staging holds: the kernel re-reads the
    corrected gradient from the new residual, also when that overwrites e_in."""
    n = 3_000_000
    g, e = si.gaussian_gradient(n, DEV, 31), si.residual_vector(n, DEV, 32)
    check_ef(dct, g, e, n // 2)
    check_ef(dct, g, e, n // 3, capacity=n // 10)
    q = (torch.randint(-1, 2, (n,), device=DEV, generator=si._gen(DEV, 33)).float() * 0.5)
    check_ef(dct, q, q.roll(1), n // 3)  # sums in {-1, -.5, 0, .5, 1}: a tie value covers much of the vector


def test_dp_ef_sampled_select(dct):
    """Large enough for the sampled selection (the partition pass reads both vectors)."""
    n = 6_000_011
    g = si.student_t3_gradient(n, DEV, 41)
    e = si.residual_vector(n, DEV, 42)
    check_ef(dct, g, e, n // 1000, in_place=False)
    check_ef(dct, g[1:], e[1:], n // 50, modes=(1,), in_place=False)
    name, qg, qe = si.error_feedback_pairs(n, DEV, 43)[4]   # quantised: the bounds collapse onto one key
    check_ef(dct, qg, qe, n // 10, modes=(1,), in_place=False)


def test_dp_ef_training_loop_with_reuse(dct):
    """Five iterations of Algorithm 1 at a reduced c3 size: iteration 0 selects,
    the others reuse tau; the residual is updated in place on the GPU and carried
    from iteration to iteration on both sides."""
    n, k = 2_500_000, 2_500
    ef = EF(dct, n, capacity=4 * k)
    e_gpu = torch.zeros(n, device=DEV)
    e_ref = np.zeros(n, dtype=np.float32)
    counts = []
    for it in range(5):
        g = si.config_c3_draw(DEV, it, n)
        gh = host(g)
        if it == 0:
            thr = ef.select(g, e_gpu, k)
            exp = oracle.ef_select_threshold(gh, e_ref, k)
            assert thr == exp
        idx, val, cnt, guard = ef.compact(g, e_gpu, e_gpu, 0)
        eidx, eval_, ecnt, e_ref = oracle.ef_threshold_compact(gh, e_ref, exp, 0, capacity=4 * k)
        assert cnt == ecnt and np.array_equal(idx, eidx) and np.array_equal(bits(val), bits(eval_))
        assert np.array_equal(bits(host(e_gpu)), bits(e_ref)), it
        counts.append(cnt)
    assert counts[0] == k and counts[1] > counts[0]  # the carried residual pushes more entries over tau


def test_dp_ef_argument_errors(dct):
    n = 4096
    g, e = si.gaussian_gradient(n, DEV, 51), si.residual_vector(n, DEV, 52)
    ef = EF(dct, n)
    ef.select(g, e, 10)
    lib = dct.lib()
    args = lambda gg, ei, eo, dt: lib.dct_ef_threshold_compact(  # noqa: E731
        gg, ei, eo, dt, n, ef.thr.data_ptr(), 0, ef.idx.data_ptr(), ef.val.data_ptr(), n, ef.count.data_ptr(),
        ef.ws.data_ptr(), ef.ws.numel(), None)
    out = torch.zeros(n, device=DEV)
    assert args(g.data_ptr(), e.data_ptr(), out.data_ptr(), 0) == 0
    assert args(g.data_ptr(), e.data_ptr(), out.data_ptr(), 1) == 1       # bf16: not defined
    assert args(g.data_ptr(), None, out.data_ptr(), 0) == 1
    assert args(g.data_ptr(), e.data_ptr(), None, 0) == 1
    assert args(g.data_ptr(), e.data_ptr(), g.data_ptr(), 0) == 1         # g overlaps e_out
    assert args(g.data_ptr(), e.data_ptr(), e.data_ptr() + 16, 0) == 1    # e_in partially overlaps e_out
    assert lib.dct_ef_select_threshold(g.data_ptr(), None, 0, n, 10, ef.thr.data_ptr(), ef.sel_ws.data_ptr(),
                                       ef.sel_ws.numel(), None) == 1
    assert lib.dct_ef_select_threshold(g.data_ptr(), e.data_ptr(), 1, n, 10, ef.thr.data_ptr(),
                                       ef.sel_ws.data_ptr(), ef.sel_ws.numel(), None) == 1
    torch.cuda.synchronize()


# ------------------------------------------------------------------ receiver side: decompression
def check_scatter(dct, g, k, mode=0, capacity=None, shift=0):
    """compress on the GPU, decompress on the GPU (the count stays on the device), compare the dense
    result with the oracle's decompression of the oracle's message."""
    n = g.numel()
    dp = DP(dct, g, capacity=capacity)
    thr = dp.select(k)
    idx, val, cnt, _ = dp.compact(mode)
    gh = host(g)
    eidx, eval_, ecnt = oracle.threshold_compact(gh, thr, mode, capacity=capacity)
    buf = torch.full((n + shift,), 3.0, device=DEV).to(g.dtype)
    out = buf[shift:]
    dct.dct_scatter(dp.idx, dp.val, dp.count, out, dct.DCT_SCATTER_ASSIGN, capacity=dp.cap)
    want = oracle.scatter(eidx, eval_, n)
    assert np.array_equal(bits(host(out)), bits(want))
    if shift:
        assert torch.all(buf[:shift] == 3.0)
    return dp


@pytest.mark.parametrize("n", [1, 5, 4095, 4096, 4097, 100_003, 1_000_000, 5_000_011])
def test_scatter_sizes(dct, n):
    g = si.gaussian_gradient(n, DEV, 600 + n)
    for k in sorted({1, max(1, n // 100), max(1, n // 2), n}):
        check_scatter(dct, g, k)
    check_scatter(dct, g.to(torch.bfloat16), max(1, n // 50), mode=1)


def test_scatter_structure_and_edges(dct):
    g, k = si.config_c4(DEV, rows=si.C4_ROWS // 64)   # clustered survivors: whole tiles without any pair
    check_scatter(dct, g, k // 64 + 1, mode=1)
    g = si.gaussian_gradient(300_000, DEV, 61)
    check_scatter(dct, g, 3000, capacity=777)          # count > capacity: only the written pairs are applied
    check_scatter(dct, g, 3000, capacity=0)            # nothing delivered: all zeros
    for shift in (1, 2, 3):                             # output not 16-byte aligned
        check_scatter(dct, g, 3000, shift=shift)
    dp = check_scatter(dct, g, 3000)
    # a failed compaction (error sentinel in the count) decompresses to zeros; no count pointer = all pairs
    out = torch.full((g.numel(),), 3.0, device=DEV)
    dp.count.fill_(-1)
    dct.dct_scatter(dp.idx, dp.val, dp.count, out)
    assert torch.all(out.view(torch.int32) == 0)
    idx = torch.tensor([2, 5, 400_000, -3, 7], dtype=torch.int32, device=DEV)   # out-of-range indices are skipped
    val = torch.tensor([1.0, 2.0, 9.0, 9.0, 3.0], device=DEV)
    out = torch.full((10,), 3.0, device=DEV)
    dct.dct_scatter(idx, val, None, out, dct.DCT_SCATTER_ADD)
    assert host(out).tolist() == [3, 3, 4, 3, 3, 5, 3, 6, 3, 3]


def test_scatter_add_server_accumulate(dct):
    """Two workers' sparse gradients summed into one dense fp32 vector, against the oracle."""
    n = 700_001
    acc = si.gaussian_gradient(n, DEV, 71)
    ref = host(acc).copy()
    for w in range(2):
        g = si.gaussian_gradient(n, DEV, 72 + w)
        dp = DP(dct, g)
        thr = dp.select(n // 100)
        dp.compact(0)
        dct.dct_scatter(dp.idx, dp.val, dp.count, acc, dct.DCT_SCATTER_ADD)
        eidx, eval_, _ = oracle.threshold_compact(host(g), thr, 0)
        oracle.scatter(eidx, eval_, n, out=ref, mode=oracle.SCATTER_ADD)
        assert np.array_equal(bits(host(acc)), bits(ref))
    lib = dct.lib()
    bf = acc.to(torch.bfloat16)
    assert lib.dct_scatter(dp.idx.data_ptr(), bf.data_ptr(), None, 8, 1, bf.data_ptr(), n, 1, None) == 1  # bf16 add
    assert lib.dct_scatter(dp.idx.data_ptr(), acc.data_ptr(), None, 8, 0, None, n, 0, None) == 1
    assert lib.dct_scatter(dp.idx.data_ptr(), acc.data_ptr(), None, 8, 0, acc.data_ptr(), n, 2, None) == 1


def test_scatter_after_error_feedback_conserves_the_gradient(dct):
    n, k = 1_200_000, 6000
    g, e = si.gaussian_gradient(n, DEV, 81), si.residual_vector(n, DEV, 82)
    ef = EF(dct, n)
    ef.select(g, e, k)
    e_out = torch.empty_like(e)
    ef.compact(g, e, e_out, 1)
    dense = torch.empty_like(g)
    dct.dct_scatter(ef.idx, ef.val, ef.count, dense)
    w = host(g) + host(e)
    assert np.array_equal(host(dense) + host(e_out), w)


@pytest.mark.parametrize("dtype,B,D,k,pad", [
    (torch.float32, 33, 1024, 51, 0), (torch.float32, 5, 40, 6, 0), (torch.float32, 9, 1000, 50, 24),
    (torch.bfloat16, 64, 4096, 204, 0), (torch.bfloat16, 7, 520, 26, 8), (torch.bfloat16, 3, 12_000, 600, 0),
    (torch.float32, 3, 5000, 250, 0), (torch.bfloat16, 10, 33, 33, 1),
    # narrow dense rows: several rows per step, ragged last block, k = D
    (torch.bfloat16, 1000, 256, 12, 0), (torch.bfloat16, 2077, 512, 25, 0), (torch.float32, 300, 128, 128, 0),
    (torch.float32, 4097, 256, 13, 0), (torch.bfloat16, 129, 8, 3, 0)])
def test_rowtopk_scatter(dct, dtype, B, D, k, pad):
    x = si.relu_activations(B, D, DEV, 900 + D, dtype=dtype)
    idx = torch.zeros(B, k, dtype=torch.int32, device=DEV)
    val = torch.zeros(B, k, dtype=dtype, device=DEV)
    dct.dct_rowtopk_fwd(x, k, idx, val, None)
    buf = torch.full((B, D + pad), 3.0, device=DEV).to(dtype)
    out = buf[:, :D]
    dct.dct_rowtopk_scatter(idx, val, out)
    want = oracle.rowscatter(host(idx), host(val), D)
    assert np.array_equal(bits(host(out.contiguous()).reshape(-1)), bits(want.reshape(-1)))
    if pad:
        assert torch.all(buf[:, D:] == 3.0)
    # the dense rows gathered through the same mask give the values back
    dval = torch.zeros_like(val)
    dct.dct_rowtopk_bwd(out, idx, dval)
    assert torch.equal(dval.view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                       val.view(torch.int16 if dtype == torch.bfloat16 else torch.int32))


@pytest.mark.parametrize("dtype,B,D,k,pad,idx16", [
    (torch.bfloat16, 16390, 4096, 300, 8, False), (torch.float32, 16384, 1024, 51, 0, False),
    (torch.bfloat16, 16385, 2048, 102, 0, True), (torch.float32, 16400, 2048, 400, 4, True)])
def test_rowtopk_scatter_many_rows(dct, dtype, B, D, k, pad, idx16):
    """Decompression of many rows of 4 to 8 KiB: long lists, padded output rows, out-of-range columns (dropped),
    both index widths."""
    g = torch.Generator(device=DEV)
    g.manual_seed(3000 + D)
    idx = torch.rand(B, D, device=DEV, generator=g).argsort(1)[:, :k].sort(1).values.to(torch.int32)
    val = si.normal_matrix(B, k, DEV, 3001 + D, dtype=dtype)
    clean = idx.clone()
    bad = [(5, 0, D), (7, k - 1, 65535 if idx16 else -1), (B - 1, k // 2, D + 9)]
    for r, c, v in bad:
        idx[r, c] = v
    buf = torch.full((B, D + pad), 3.0, device=DEV).to(dtype)
    out = buf[:, :D]
    if idx16:
        dct.dct_rowtopk_scatter_idx16(idx.to(torch.int16), val, out)
    else:
        dct.dct_rowtopk_scatter(idx, val, out)
    want = oracle.rowscatter(clean.cpu().numpy(), host(val), D)
    for r, c, _ in bad:                       # the oracle takes valid lists only: a dropped pair leaves a zero
        want[r, int(clean[r, c])] = 0
    assert np.array_equal(bits(host(out.contiguous()).reshape(-1)), bits(want.reshape(-1)))
    if pad:
        assert torch.all(buf[:, D:] == 3.0)


def test_rowtopk_scatter_c5_block(dct):
    x, dy, k = si.config_c5(DEV, b=2048)
    B, D = x.shape
    idx = torch.zeros(B, k, dtype=torch.int32, device=DEV)
    val = torch.zeros(B, k, dtype=x.dtype, device=DEV)
    dct.dct_rowtopk_fwd(x, k, idx, val, None)
    out = torch.empty_like(x)
    dct.dct_rowtopk_scatter(idx, val, out)
    want = oracle.rowscatter(host(idx), host(val), D)
    assert np.array_equal(host(out), want)


# ------------------------------------------------------------------ DCT-DP, many tensors per call
def make_segments(sizes, ks, caps, gap=3):
    """Segments laid out one after another with `gap` unused elements between them (odd offsets)."""
    segs, off, out = [], 1, 0
    for n, k, cap in zip(sizes, ks, caps):
        segs.append((off, n, k, out, cap))
        off += n + gap
        out += cap + 2          # two guard slots after every segment's range
    return segs, off, out


def check_batched(dct, g, segs, out_len, modes=(0, 1)):
    table = dct.segment_table(segs)
    ws = dct.new_batched_workspace(g, table)
    n_seg = len(segs)
    thr = torch.zeros(n_seg, 4, dtype=torch.int32, device=DEV)
    dct.dct_select_threshold_batched(g, table, thr, ws)
    thr_h = thr.cpu().numpy().view(np.uint32)
    gh = host(g)
    exp_thr = []
    for s, (off, n, k, out_off, cap) in enumerate(segs):
        e = oracle.select_threshold(gh[off:off + n], k)
        assert tuple(int(v) for v in thr_h[s]) == tuple(e), (s, n, k)
        exp_thr.append(e)
    for mode in modes:
        idx = torch.full((out_len,), -7, dtype=torch.int32, device=DEV)
        val = torch.zeros(out_len, dtype=g.dtype, device=DEV)
        cnt = torch.zeros(n_seg, dtype=torch.int64, device=DEV)
        dct.dct_threshold_compact_batched(g, table, thr, mode, idx, val, cnt, ws)
        idx_h, val_h, cnt_h = host(idx), host(val), cnt.cpu().numpy()
        written = np.zeros(out_len, dtype=bool)
        for s, (off, n, k, out_off, cap) in enumerate(segs):
            eidx, eval_, ecnt = oracle.threshold_compact(gh[off:off + n], exp_thr[s], mode, capacity=cap)
            assert int(cnt_h[s]) == ecnt, (s, mode)
            m = min(ecnt, cap)
            assert np.array_equal(idx_h[out_off:out_off + m], eidx), (s, mode)
            assert np.array_equal(bits(val_h[out_off:out_off + m]), bits(eval_)), (s, mode)
            written[out_off:out_off + m] = True
        assert np.all(idx_h[~written] == -7)  # nothing outside the survivors' slots
    return thr


def test_batched_layers_like_a_small_model(dct):
    """Tensors from a few elements to a few million, odd offsets, 1 % kept (sizes of FC weights and biases)."""
    sizes = [512 * 256, 256, 1024 * 1024, 1024, 8191, 65536, 65537, 1, 5, 3_000_001, 13 * 64]
    ks = [max(1, n // 100) for n in sizes]
    caps = [2 * k for k in ks]
    segs, total, out_len = make_segments(sizes, ks, caps)
    g = si.gaussian_gradient(total, DEV, 1234)
    thr = check_batched(dct, g, segs, out_len)
    # every segment agrees with the single-tensor call on the same slice
    for s in (0, 2, 9):
        off, n, k, _, _ = segs[s]
        dp = DP(dct, g[off:off + n])
        assert dp.select(k) == oracle.Threshold(*(int(v) & 0xFFFFFFFF for v in thr[s].cpu().tolist()))


def test_batched_ties_overflow_and_many_segments(dct):
    # heavy ties and special values per segment; capacities that cut the output short or are zero
    vecs = [v for _, v in si.adversarial_vectors(20_000, DEV, 77)] + [v for _, v in si.adversarial_vectors(40, DEV, 78)]
    sizes = [v.numel() for v in vecs]
    ks = [max(1, n // 7) for n in sizes]
    caps = [(0 if i % 5 == 0 else (k // 2 if i % 3 == 0 else n)) for i, (n, k) in enumerate(zip(sizes, ks))]
    segs, total, out_len = make_segments(sizes, ks, caps, gap=1)
    g = torch.zeros(total, device=DEV)
    for (off, n, *_), v in zip(segs, vecs):
        g[off:off + n] = v
    check_batched(dct, g, segs, out_len)
    # more segments than one table upload carries
    sizes = [17 + 37 * (i % 11) for i in range(150)]
    ks = [1 + (i % 5) for i in range(150)]
    segs, total, out_len = make_segments(sizes, ks, [n for n in sizes], gap=0)
    check_batched(dct, si.gaussian_gradient(total, DEV, 4321), segs, out_len)


def test_batched_bf16(dct):
    sizes = [70_001, 16384, 3, 262_144]
    ks = [max(1, n // 50) for n in sizes]
    segs, total, out_len = make_segments(sizes, ks, [3 * k for k in ks])
    g = si.gaussian_gradient(total, DEV, 99, scale=1.0).to(torch.bfloat16)
    check_batched(dct, g, segs, out_len)


def test_batched_argument_errors(dct):
    g = si.gaussian_gradient(10_000, DEV, 5)
    lib = dct.lib()
    import ctypes
    ok = dct.segment_table([(0, 5000, 50, 0, 100), (5000, 5000, 50, 100, 100)])
    ws = dct.new_batched_workspace(g, ok)
    thr = torch.zeros(2, 4, dtype=torch.int32, device=DEV)
    call = lambda tab, n_seg, wsb: lib.dct_select_threshold_batched(  # noqa: E731
        g.data_ptr(), 0, ctypes.cast(tab, ctypes.c_void_p), n_seg, thr.data_ptr(), ws.data_ptr(), wsb, None)
    assert call(ok, 2, ws.numel()) == 0
    assert call(ok, 0, ws.numel()) == 1
    assert call(ok, 2000, ws.numel()) == 1
    assert call(dct.segment_table([(0, 0, 1, 0, 0)]), 1, ws.numel()) == 1       # empty segment
    assert call(dct.segment_table([(0, 10, 11, 0, 0)]), 1, ws.numel()) == 1     # k > n
    assert call(ok, 2, 256) == 2                                                  # workspace too small
    assert lib.dct_batched_workspace_bytes(0, None, 1) == 0
    with pytest.raises(ValueError):
        dct.dct_select_threshold_batched(g, dct.segment_table([(9000, 5000, 5, 0, 0)]), thr[:1], ws)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ DCT-MP, the mask as a bitmap
@pytest.mark.parametrize("dtype,B,D,k,pad", [
    (torch.bfloat16, 70, 4096, 204, 0), (torch.bfloat16, 33, 2048, 102, 0), (torch.bfloat16, 9, 1024, 51, 8),
    (torch.bfloat16, 17, 512, 25, 0), (torch.bfloat16, 5, 264, 13, 0), (torch.bfloat16, 6, 40, 7, 0),
    (torch.bfloat16, 4, 8, 8, 0), (torch.bfloat16, 3, 12_000, 600, 0), (torch.bfloat16, 5, 1001, 50, 0),
    (torch.float32, 33, 1024, 51, 0), (torch.float32, 7, 33, 5, 3), (torch.float32, 2, 5000, 250, 0),
    # more survivors than the backward kernel lists on chip (1024 per row): its direct path
    (torch.bfloat16, 5, 4096, 2000, 0), (torch.float32, 3, 2304, 1500, 0), (torch.bfloat16, 3, 9000, 1025, 0)])
def test_mp_bitmask_encoding(dct, dtype, B, D, k, pad):
    x = si.relu_activations(B, D, DEV, 1300 + D, dtype=dtype, row_stride=D + pad if pad else None)
    dy = si.normal_matrix(B, D, DEV, 1400 + D, dtype=dtype)
    words = (D + 31) // 32
    mask = torch.full((B, words), -1, dtype=torch.int32, device=DEV)
    val = torch.zeros(B, k, dtype=dtype, device=DEV)
    tau = torch.zeros(B, dtype=dtype, device=DEV)
    dct.dct_rowtopk_fwd_bitmask(x, k, mask, val, tau)
    xh = host(x.contiguous()) if not pad else oracle.as_numpy(x.cpu())
    emask, eval_, etau = oracle.rowtopk_fwd_bitmask(xh, k)
    assert np.array_equal(mask.cpu().numpy().view(np.uint32), emask)
    assert np.array_equal(bits(host(val).reshape(-1)), bits(eval_.reshape(-1)))
    assert np.array_equal(bits(host(tau)), bits(etau))
    # the index form of the same call keeps the same set
    idx = torch.zeros(B, k, dtype=torch.int32, device=DEV)
    val2 = torch.zeros_like(val)
    dct.dct_rowtopk_fwd(x, k, idx, val2, None)
    assert torch.equal(val.view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                       val2.view(torch.int16 if dtype == torch.bfloat16 else torch.int32))
    # backward and decompression through the bitmap
    dval = torch.full((B, k), 3.0, device=DEV).to(dtype)
    dct.dct_rowtopk_bwd_bitmask(dy, mask, dval)
    assert np.array_equal(bits(host(dval).reshape(-1)), bits(oracle.rowtopk_bwd_bitmask(host(dy), emask, k).reshape(-1)))
    buf = torch.full((B, D + 5), 3.0, device=DEV).to(dtype)
    dct.dct_rowtopk_scatter_bitmask(mask, val, buf[:, :D])
    assert np.array_equal(bits(host(buf[:, :D].contiguous()).reshape(-1)),
                          bits(oracle.rowscatter_bitmask(emask, eval_, D).reshape(-1)))
    assert torch.all(buf[:, D:] == 3.0)


def test_mp_bitmask_hard_rows_and_short_masks(dct):
    # ties across the quota boundary, all-equal rows, all-zero rows (the bitmap must pick the lowest columns)
    B, D, k = 12, 4096, 204
    x = si.relu_activations(B, D, DEV, 1500, dtype=torch.bfloat16)
    x[0] = 0.75
    x[1] = 0.0
    x[2, ::2] = 1.0
    x[3] = (torch.arange(D, device=DEV) % 7).to(torch.bfloat16)
    mask = torch.zeros(B, D // 32, dtype=torch.int32, device=DEV)
    val = torch.zeros(B, k, dtype=torch.bfloat16, device=DEV)
    dct.dct_rowtopk_fwd_bitmask(x, k, mask, val, None)
    emask, eval_, _ = oracle.rowtopk_fwd_bitmask(host(x), k)
    assert np.array_equal(mask.cpu().numpy().view(np.uint32), emask)
    assert np.array_equal(host(val), eval_)
    # a mask with fewer / more set bits than k (not produced by the forward pass): defined behaviour
    dy = si.normal_matrix(B, D, DEV, 1501, dtype=torch.bfloat16)
    m2 = mask.clone()
    m2[0] = 0
    m2[0, 3] = 0b1011
    m2[1] = -1
    dval = torch.full((B, k), 3.0, device=DEV).to(torch.bfloat16)
    dct.dct_rowtopk_bwd_bitmask(dy, m2, dval)
    want = oracle.rowtopk_bwd_bitmask(host(dy), m2.cpu().numpy().view(np.uint32), k)
    assert np.array_equal(host(dval), want)
    out = torch.full((B, D), 3.0, device=DEV).to(torch.bfloat16)
    dct.dct_rowtopk_scatter_bitmask(m2, val, out)
    assert np.array_equal(host(out), oracle.rowscatter_bitmask(m2.cpu().numpy().view(np.uint32), host(val), D))


def test_mp_bitmask_c5_block(dct):
    x, dy, k = si.config_c5(DEV, b=4096)
    B, D = x.shape
    mask = torch.zeros(B, D // 32, dtype=torch.int32, device=DEV)
    val = torch.zeros(B, k, dtype=x.dtype, device=DEV)
    dct.dct_rowtopk_fwd_bitmask(x, k, mask, val, None)
    emask, eval_, _ = oracle.rowtopk_fwd_bitmask(host(x), k)
    assert np.array_equal(mask.cpu().numpy().view(np.uint32), emask) and np.array_equal(host(val), eval_)
    dval = torch.zeros_like(val)
    dct.dct_rowtopk_bwd_bitmask(dy, mask, dval)
    assert np.array_equal(host(dval), oracle.rowtopk_bwd_bitmask(host(dy), emask, k))


# ------------------------------------------------------------------ MP: bf16 rows of 4096 ... 8192 columns (four bitmap words per lane)
@pytest.mark.parametrize("B,D,k,enc", [(37, 8192, 409, 0), (20, 5120, 256, 1), (9, 6144, 300, 2), (5, 8192, 512, 0),
                                       (6, 4104, 1, 0), (4, 8192, 8192, 0), (11, 7168, 1000, 2),
                                       # enough rows for the workgroups of 8 wavefronts that share a row counter
                                       (8200, 8192, 409, 0), (8195, 5120, 256, 1), (8192, 6144, 300, 2)])
def test_mp_bf16_wide_rows(dct, B, D, k, enc):
    x = si.relu_activations(B, D, DEV, 1980 + D + k, dtype=torch.bfloat16)
    cols = torch.arange(D, device=DEV)
    x[0] = 0.75                                    # all equal: the k lowest columns
    x[1] = 0.0
    x[2] = torch.where(cols % 2 == 0, 1.0, 2.0).to(torch.bfloat16)
    x[3] = (cols % 5).to(torch.bfloat16)           # ties across the quota boundary in every word of a lane
    val = torch.zeros(B, k, dtype=torch.bfloat16, device=DEV)
    tau = torch.zeros(B, dtype=torch.bfloat16, device=DEV)
    xh = host(x)
    ei, ev, et = oracle.rowtopk_fwd(xh, k)
    if enc == 2:
        mask = torch.full((B, (D + 31) // 32), -1, dtype=torch.int32, device=DEV)
        dct.dct_rowtopk_fwd_bitmask(x, k, mask, val, tau)
        em, _, _ = oracle.rowtopk_fwd_bitmask(xh, k)
        assert np.array_equal(mask.cpu().numpy().view(np.uint32), em)
    else:
        idx = torch.full((B, k), -1, dtype=torch.int16 if enc == 1 else torch.int32, device=DEV)
        (dct.dct_rowtopk_fwd_idx16 if enc == 1 else dct.dct_rowtopk_fwd)(x, k, idx, val, tau)
        got = idx.cpu().numpy()
        got = got.view(np.uint16).astype(np.int32) if enc == 1 else got
        bad = np.nonzero((got != ei).any(axis=1))[0]
        assert bad.size == 0, (bad[:10], got[bad[0]][:20], ei[bad[0]][:20])
    assert np.array_equal(host(val), ev) and np.array_equal(host(tau), et)


# ------------------------------------------------------------------ MP: many narrow bf16 rows (four rows per wavefront)
@pytest.mark.parametrize("B,D,k,pad,idx16", [
    (8192, 256, 12, 0, False), (8193, 512, 25, 0, False), (10_000, 1024, 51, 0, False), (8200, 128, 6, 0, True),
    (9001, 264, 13, 8, False), (8192, 1000, 128, 0, False), (8195, 64, 64, 0, True), (8190 + 9, 8, 3, 0, False),
    (8192, 1024, 1, 0, False), (8194, 520, 100, 16, True),
    # 64 k rows and more: one workgroup of 16 wavefronts per CU takes the groups from a counter
    (65536, 256, 12, 0, False), (65539, 512, 25, 0, True), (70_001, 1024, 51, 0, False), (131_075, 64, 3, 0, False),
    (65_537, 264, 13, 8, False),
    # rows of up to 256 columns, 128 k rows and more: eight rows per wavefront
    (131_083, 256, 12, 0, False), (140_001, 128, 6, 0, True), (131_073, 200, 64, 0, False),
    (131_077, 256, 13, 8, True), (131_072, 8, 3, 0, False), (131_079, 256, 1, 0, False)])
def test_mp_many_narrow_rows(dct, B, D, k, pad, idx16):
    x = si.relu_activations(B, D, DEV, 1900 + D + k, dtype=torch.bfloat16, row_stride=D + pad if pad else None)
    # hard rows among the ordinary ones, spread over the slots of a group of four: all equal, all zero, two
    # values alternating, few distinct values, NaN, signed, ties straddling the quota
    gen = torch.Generator(device=DEV).manual_seed(77)
    cols = torch.arange(D, device=DEV)
    x[0] = 0.75
    x[5] = 0.0
    x[10] = torch.where(cols % 2 == 0, 1.0, 2.0).to(torch.bfloat16)
    x[15] = (cols % 7).to(torch.bfloat16)
    x[16] = torch.randn(D, device=DEV, generator=gen).to(torch.bfloat16)
    x[17, D // 2] = float("nan")
    x[22] = -x[23].clone()
    x[B - 1] = 3.0
    x[B - 2] = (cols % 3).to(torch.bfloat16)
    idx = torch.full((B, k), -1, dtype=torch.int16 if idx16 else torch.int32, device=DEV)
    val = torch.zeros(B, k, dtype=torch.bfloat16, device=DEV)
    tau = torch.zeros(B, dtype=torch.bfloat16, device=DEV)
    (dct.dct_rowtopk_fwd_idx16 if idx16 else dct.dct_rowtopk_fwd)(x, k, idx, val, tau)
    xh = host(x.contiguous()) if not pad else oracle.as_numpy(x.cpu())
    eidx, eval_, etau = oracle.rowtopk_fwd(xh, k)
    got = idx.cpu().numpy()
    got = got.view(np.uint16).astype(np.int32) if idx16 else got
    bad = np.nonzero((got != eidx).any(axis=1))[0]
    assert bad.size == 0, (bad[:10], got[bad[0]], eidx[bad[0]])
    assert np.array_equal(bits(host(val).reshape(-1)), bits(eval_.reshape(-1)))
    assert np.array_equal(bits(host(tau)), bits(etau))


def _hard_rows(kind, B, D, seed):
    """Rows whose thresholds jump, tie, or sit at the ends of the key range: what the prediction window, its
    neighbour step, the gallop and the clamps at both ends of the key space have to get right."""
    gen = torch.Generator(device=DEV).manual_seed(seed)
    x = torch.randn(B, D, device=DEV, generator=gen)
    rows = torch.arange(B, device=DEV)
    if kind == "scales":      # consecutive rows nine orders of magnitude apart
        sc = torch.where(rows % 3 == 0, 1e-3, torch.where(rows % 3 == 1, 1.0, 3e4))
        x = torch.relu(x) * sc[:, None]
    elif kind == "quant":     # few distinct values: ties by the dozen at every threshold
        x = torch.round(x * 2) / 2
    elif kind == "tiny":      # denormals: the window is clamped at key 0
        x = x * 1e-39
    elif kind == "huge":      # the top of the key range, infinities and NaNs
        x = x * 1e38
        x[::7, ::5] = float("inf")
        x[3::11, 1] = float("nan")
    elif kind == "drift":     # thresholds drifting over 17 orders of magnitude
        x = torch.relu(x) * torch.exp(torch.linspace(-20, 20, B, device=DEV))[:, None]
    return x.to(torch.bfloat16).contiguous()


@pytest.mark.parametrize("kind", ["scales", "quant", "tiny", "huge", "drift"])
@pytest.mark.parametrize("B,D,k,enc", [(131_077, 256, 12, 0), (131_075, 128, 6, 2), (70_001, 512, 25, 0),
                                       (66_003, 1024, 51, 1), (9_001, 512, 25, 2)])
def test_mp_narrow_rows_hard_distributions(dct, kind, B, D, k, enc):
    x = _hard_rows(kind, B, D, 4242 + D + enc)
    val = torch.zeros(B, k, dtype=torch.bfloat16, device=DEV)
    tau = torch.zeros(B, dtype=torch.bfloat16, device=DEV)
    xh = host(x)
    if enc == 1:
        mask = torch.full((B, (D + 31) // 32), -1, dtype=torch.int32, device=DEV)
        dct.dct_rowtopk_fwd_bitmask(x, k, mask, val, tau)
        emask, eval_, etau = oracle.rowtopk_fwd_bitmask(xh, k)
        assert np.array_equal(mask.cpu().numpy().view(np.uint32), emask)
    else:
        idx = torch.full((B, k), -1, dtype=torch.int16 if enc == 2 else torch.int32, device=DEV)
        (dct.dct_rowtopk_fwd_idx16 if enc == 2 else dct.dct_rowtopk_fwd)(x, k, idx, val, tau)
        eidx, eval_, etau = oracle.rowtopk_fwd(xh, k)
        got = idx.cpu().numpy()
        got = got.view(np.uint16).astype(np.int32) if enc == 2 else got
        bad = np.nonzero((got != eidx).any(axis=1))[0]
        assert bad.size == 0, (bad[:10], got[bad[0]], eidx[bad[0]])
    assert np.array_equal(bits(host(val).reshape(-1)), bits(np.asarray(eval_).reshape(-1)))
    assert np.array_equal(bits(host(tau)), bits(np.asarray(etau)))


@pytest.mark.parametrize("B,D,k", [(8192, 256, 12), (8199, 64, 5), (8193, 128, 9), (9000, 1024, 51), (8192, 520, 26),
                                   (65541, 256, 12), (66000, 1024, 51), (131_079, 256, 12), (131_075, 128, 9),
                                   (131_073, 72, 5)])
def test_mp_many_narrow_rows_bitmask(dct, B, D, k):
    x = si.relu_activations(B, D, DEV, 1950 + D, dtype=torch.bfloat16)
    x[3] = 0.5
    x[B - 1] = 0.0
    mask = torch.full((B, (D + 31) // 32), -1, dtype=torch.int32, device=DEV)
    val = torch.zeros(B, k, dtype=torch.bfloat16, device=DEV)
    dct.dct_rowtopk_fwd_bitmask(x, k, mask, val, None)
    emask, eval_, _ = oracle.rowtopk_fwd_bitmask(host(x), k)
    assert np.array_equal(mask.cpu().numpy().view(np.uint32), emask)
    assert np.array_equal(host(val), eval_)


@pytest.mark.parametrize("dtype,B,D,k", [
    (torch.bfloat16, 1000, 256, 12), (torch.bfloat16, 77, 32, 5), (torch.bfloat16, 513, 1024, 51),
    (torch.float32, 300, 64, 64), (torch.float32, 1025, 512, 25), (torch.bfloat16, 9, 128, 1)])
def test_mp_bitmask_consumers_narrow_rows(dct, dtype, B, D, k):
    """Masks of 1 ... 32 words per row (a power of two): several rows per wavefront, one lane per word."""
    x = si.relu_activations(B, D, DEV, 1960 + D, dtype=dtype)
    dy = si.normal_matrix(B, D, DEV, 1961 + D, dtype=dtype)
    mask = torch.zeros(B, D // 32, dtype=torch.int32, device=DEV)
    val = torch.zeros(B, k, dtype=dtype, device=DEV)
    dct.dct_rowtopk_fwd_bitmask(x, k, mask, val, None)
    emask, eval_, _ = oracle.rowtopk_fwd_bitmask(host(x), k)
    assert np.array_equal(mask.cpu().numpy().view(np.uint32), emask)
    # masks the forward pass would not produce: fewer set bits than k, more than k, none
    m2 = mask.clone()
    m2[0] = 0
    m2[1] = -1
    if B > 5:
        m2[5] = 0
        m2[5, 0] = 0b101
    m2h = m2.cpu().numpy().view(np.uint32)
    dval = torch.full((B, k), 3.0, device=DEV).to(dtype)
    dct.dct_rowtopk_bwd_bitmask(dy, m2, dval)
    assert np.array_equal(bits(host(dval).reshape(-1)), bits(oracle.rowtopk_bwd_bitmask(host(dy), m2h, k).reshape(-1)))
    out = torch.full((B, D), 3.0, device=DEV).to(dtype)
    dct.dct_rowtopk_scatter_bitmask(m2, val, out)
    assert np.array_equal(bits(host(out).reshape(-1)), bits(oracle.rowscatter_bitmask(m2h, host(val), D).reshape(-1)))


# ------------------------------------------------------------------ Algorithm 2, the mask as 16-bit indices
def _u16(t):
    return t.cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("dtype,B,D,k,pad", [
    (torch.bfloat16, 17, 512, 25, 0), (torch.bfloat16, 5, 264, 13, 0), (torch.bfloat16, 6, 40, 7, 0),
    (torch.bfloat16, 4, 8, 8, 0), (torch.bfloat16, 3, 12_000, 600, 0), (torch.bfloat16, 5, 1001, 50, 0),
    (torch.bfloat16, 9, 4096, 300, 8), (torch.bfloat16, 70, 2048, 102, 0),
    (torch.float32, 33, 1024, 51, 0), (torch.float32, 7, 33, 5, 3), (torch.float32, 2, 5000, 250, 0),
    (torch.float32, 6, 4096, 204, 0)])
def test_mp_idx16_encoding(dct, dtype, B, D, k, pad):
    x = si.relu_activations(B, D, DEV, 1600 + D, dtype=dtype, row_stride=D + pad if pad else None)
    dy = si.normal_matrix(B, D, DEV, 1700 + D, dtype=dtype)
    idx = torch.full((B, k), -1, dtype=torch.int16, device=DEV)
    val = torch.zeros(B, k, dtype=dtype, device=DEV)
    tau = torch.zeros(B, dtype=dtype, device=DEV)
    dct.dct_rowtopk_fwd_idx16(x, k, idx, val, tau)
    xh = host(x.contiguous()) if not pad else oracle.as_numpy(x.cpu())
    eidx, eval_, etau = oracle.rowtopk_fwd_idx16(xh, k)
    assert np.array_equal(_u16(idx), eidx)
    assert np.array_equal(bits(host(val).reshape(-1)), bits(eval_.reshape(-1)))
    assert np.array_equal(bits(host(tau)), bits(etau))
    dval = torch.full((B, k), 3.0, device=DEV).to(dtype)
    dct.dct_rowtopk_bwd_idx16(dy, idx, dval)
    assert np.array_equal(bits(host(dval).reshape(-1)), bits(oracle.rowtopk_bwd_idx16(host(dy), eidx).reshape(-1)))
    buf = torch.full((B, D + 5), 3.0, device=DEV).to(dtype)
    dct.dct_rowtopk_scatter_idx16(idx, val, buf[:, :D])
    assert np.array_equal(bits(host(buf[:, :D].contiguous()).reshape(-1)),
                          bits(oracle.rowscatter_idx16(eidx, eval_, D).reshape(-1)))
    assert torch.all(buf[:, D:] == 3.0)


def test_mp_idx16_widest_row_hard_rows_and_bad_indices(dct):
    # D = 65536: the last column (0xFFFF) is kept in row 0; D = 65537 does not fit 16 bits
    B, D, k = 3, 65536, 300
    x = si.relu_activations(B, D, DEV, 1800, dtype=torch.bfloat16)
    x[0, D - 1] = -100.0
    x[1] = 0.5          # all equal: the k lowest columns
    idx = torch.zeros(B, k, dtype=torch.int16, device=DEV)
    val = torch.zeros(B, k, dtype=torch.bfloat16, device=DEV)
    dct.dct_rowtopk_fwd_idx16(x, k, idx, val, None)
    eidx, eval_, _ = oracle.rowtopk_fwd_idx16(host(x), k)
    assert np.array_equal(_u16(idx), eidx) and np.array_equal(host(val), eval_)
    assert int(eidx[0, -1]) == 0xFFFF and eidx[1].tolist() == list(range(k))
    dy = si.normal_matrix(B, D, DEV, 1801, dtype=torch.bfloat16)
    dval = torch.zeros_like(val)
    dct.dct_rowtopk_bwd_idx16(dy, idx, dval)
    assert np.array_equal(host(dval), oracle.rowtopk_bwd_idx16(host(dy), eidx))
    out = torch.full((B, D), 3.0, device=DEV).to(torch.bfloat16)
    dct.dct_rowtopk_scatter_idx16(idx, val, out)
    assert np.array_equal(host(out), oracle.rowscatter_idx16(eidx, eval_, D))
    wide = torch.zeros(1, 65537, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(dct.DctError):
        dct.dct_rowtopk_fwd_idx16(wide, 4, torch.zeros(1, 4, dtype=torch.int16, device=DEV),
                                  torch.zeros(1, 4, dtype=torch.bfloat16, device=DEV), None)
    # an index past the row's end: zero in the backward pass, skipped by the decompression
    D2, k2 = 1000, 4
    dy2 = si.normal_matrix(2, D2, DEV, 1802, dtype=torch.float32)
    bad = torch.tensor([[1, 5, 1000, 65535], [0, 2, 3, 999]], dtype=torch.int32).to(torch.uint16).to(DEV)
    dv = torch.full((2, k2), 3.0, device=DEV)
    dct.dct_rowtopk_bwd_idx16(dy2, bad, dv)
    want = torch.stack([torch.stack([dy2[0, 1], dy2[0, 5], dy2.new_zeros(()), dy2.new_zeros(())]),
                        dy2[1, [0, 2, 3, 999]]])
    assert torch.equal(dv, want)
    v2 = torch.arange(1, 9, dtype=torch.float32, device=DEV).reshape(2, 4)
    o2 = torch.full((2, D2), 3.0, device=DEV)
    dct.dct_rowtopk_scatter_idx16(bad, v2, o2)
    assert np.array_equal(host(o2), oracle.rowscatter_idx16(_u16(bad), host(v2), D2))


def test_mp_idx16_c5_block_matches_the_int32_form(dct):
    x, dy, k = si.config_c5(DEV, b=4096)
    B, D = x.shape
    idx = torch.zeros(B, k, dtype=torch.int16, device=DEV)
    val = torch.zeros(B, k, dtype=x.dtype, device=DEV)
    dct.dct_rowtopk_fwd_idx16(x, k, idx, val, None)
    eidx, eval_, _ = oracle.rowtopk_fwd_idx16(host(x), k)
    assert np.array_equal(_u16(idx), eidx) and np.array_equal(host(val), eval_)
    idx32 = torch.zeros(B, k, dtype=torch.int32, device=DEV)
    val32 = torch.zeros_like(val)
    dct.dct_rowtopk_fwd(x, k, idx32, val32, None)
    assert np.array_equal(idx32.cpu().numpy(), eidx.astype(np.int32))
    dval = torch.zeros_like(val)
    dct.dct_rowtopk_bwd_idx16(dy, idx, dval)
    assert np.array_equal(host(dval), oracle.rowtopk_bwd_idx16(host(dy), eidx))


@pytest.mark.parametrize("frac", [0.05, 0.25])
def test_dp_ef_low_sparsity_levels(dct, frac):
    """Error feedback with more survivors than the grid holds on chip: the compaction runs in several
    rounds, in which every workgroup waits on all workgroups of the earlier rounds (both modes)."""
    n = 5_000_011
    g = si.gaussian_gradient(n, DEV, 2300)
    e = si.residual_vector(n, DEV, 2301)
    check_ef(dct, g, e, int(n * frac), in_place=False)


# ------------------------------------------------------------------ side stream, HIP graph
def test_calls_on_a_side_stream_and_in_a_captured_graph(dct):
    """The calls launch on the stream they are given and allocate nothing, so a training loop can
    capture them: one DP step (select + exactly-k compaction, 5 M elements: the sampled selection
    with its four launches) and one MP step (forward + backward) are captured once and replayed on
    fresh data, with eager work and synchronisations in between; every replay is checked against the oracle."""
    n, k = 5_000_003, 25_000
    B, D, kk = 300, 1024, 51
    g = torch.empty(n, device=DEV)
    x = torch.empty(B, D, dtype=torch.bfloat16, device=DEV)
    dy = torch.empty(B, D, dtype=torch.bfloat16, device=DEV)
    thr = torch.zeros(4, dtype=torch.int32, device=DEV)
    sws, cws = dct.new_select_workspace(g), dct.new_compact_workspace(g)
    idx = torch.zeros(k, dtype=torch.int32, device=DEV)
    val = torch.zeros(k, device=DEV)
    cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    ridx = torch.zeros(B, kk, dtype=torch.int32, device=DEV)
    rval = torch.zeros(B, kk, dtype=torch.bfloat16, device=DEV)
    dval = torch.zeros_like(rval)

    def step():
        dct.dct_select_threshold(g, k, thr, sws)
        dct.dct_threshold_compact(g, thr, dct.DCT_EXACT_K, idx, val, cnt, cws)
        dct.dct_rowtopk_fwd(x, kk, ridx, rval, None)
        dct.dct_rowtopk_bwd(dy, ridx, dval)

    def fill(seed):
        g.copy_(si.gaussian_gradient(n, DEV, seed))
        x.copy_(si.relu_activations(B, D, DEV, seed + 1, dtype=torch.bfloat16))
        dy.copy_(si.normal_matrix(B, D, DEV, seed + 2, dtype=torch.bfloat16))

    def check():
        torch.cuda.synchronize()
        gh = host(g)
        exp = oracle.select_threshold(gh, k, method="nth")
        assert dct.read_threshold(thr) == exp
        eidx, eval_, ecnt = oracle.threshold_compact(gh, exp, oracle.EXACT_K)
        assert cnt.item() == ecnt == k
        assert np.array_equal(idx.cpu().numpy(), eidx) and np.array_equal(bits(host(val)), bits(eval_))
        ei, ev, _ = oracle.rowtopk_fwd(host(x), kk)
        assert np.array_equal(ridx.cpu().numpy(), ei) and np.array_equal(host(rval), ev)
        assert np.array_equal(host(dval), oracle.rowtopk_bwd(host(dy), ei))

    side = torch.cuda.Stream()
    fill(3000)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):   # eager, not the default stream
        step()
    torch.cuda.current_stream().wait_stream(side)
    check()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for r in range(3):
        fill(3100 + 10 * r)         # eager work between the replays
        idx.fill_(-1)
        val.zero_()
        graph.replay()
        check()


# ------------------------------------------------------------------ seeded random configurations
def test_dp_selections_on_four_streams_at_once(dct):
    """Selections that run at the same time on different streams: the last kernel of each waits at grid
    barriers, and every waiting workgroup has to find room next to those of the other selections.
    Inputs of all kinds (radix passes over the vector, over the candidates, over the keys inside the
    bounds after a candidate overflow), 20 rounds, every record checked against the oracle."""
    inputs = [(si.gaussian_gradient(1 << 20, DEV, 2600), 10_486),
              (si.gaussian_gradient(3_000_001, DEV, 2601), 30_000),
              (si.student_t3_gradient(5_000_003, DEV, 2602), 5_000)]
    z = si.gaussian_gradient(4_500_000, DEV, 2603)
    z[torch.rand(z.numel(), device=DEV) < 0.9] = 0.0
    inputs.append((z, z.numel() // 5))  # k beyond the non-zeros: tau = 0 with four million ties
    expected = [oracle.select_threshold(host(g), k, method="nth") for g, k in inputs]
    assert expected[3].tau_key == 0
    streams = [torch.cuda.Stream() for _ in inputs]
    thr = [torch.zeros(4, dtype=torch.int32, device=DEV) for _ in inputs]
    ws = [dct.new_select_workspace(g) for g, _ in inputs]
    for rnd in range(20):
        torch.cuda.synchronize()  # the inputs, and the cleared records of the previous round, are in place
        for i, (g, k) in enumerate(inputs):
            with torch.cuda.stream(streams[i]):
                dct.dct_select_threshold(g, k, thr[i], ws[i])
        torch.cuda.synchronize()
        for i in range(len(inputs)):
            assert oracle.Threshold(*dct.read_threshold(thr[i])) == expected[i], (rnd, i)
            thr[i].zero_()


def _raw_count(cnt):
    return int(cnt.cpu().item()) & ((1 << 64) - 1)


COUNT_ERROR = (1 << 64) - 1


def test_dp_ef_compaction_next_to_long_kernels_on_another_stream(dct):
    """Algorithm 1 with error feedback while unrelated kernels hold compute units on another stream (a trainer
    that overlaps compression with its backward pass).  The residual is training state: the call must give the
    oracle's result, or -- had one of its bounded waits run out -- report so through the count with NO pair
    delivered and the corrected gradient g + e left in the residual.  Sparse and dense survivors (the dense
    case streams its chunks a second time), residual updated in place, five rounds each."""
    n = 6_000_011
    side = torch.cuda.Stream()
    a = torch.randn(4096, 4096, device=DEV)
    b = torch.randn(4096, 4096, device=DEV)
    for keep in (0.01, 0.30):
        k = int(n * keep)
        ef = EF(dct, n, capacity=n)
        for rnd in range(5):
            g = si.gaussian_gradient(n, DEV, 4100 + rnd)
            e = si.residual_vector(n, DEV, 4200 + rnd)
            gh, eh = host(g), host(e)
            thr = ef.select(g, e, k)
            exp = oracle.ef_select_threshold(gh, eh, k)
            assert thr == exp
            eidx, eval_, ecnt, e_exp = oracle.ef_threshold_compact(gh, eh, exp, oracle.GE_TAU)
            torch.cuda.synchronize()
            with torch.cuda.stream(side):       # a few hundred microseconds of matrix products per launch
                for _ in range(6):
                    a = torch.tanh(a @ b)
            ef.idx.fill_(-7)
            dct.dct_ef_threshold_compact(g, e, e, ef.thr, dct.DCT_GE_TAU, ef.idx, ef.val, ef.count, ef.ws)
            torch.cuda.synchronize()
            c = _raw_count(ef.count)
            if c == COUNT_ERROR:                # the documented state: nothing sent, nothing lost
                assert np.array_equal(bits(host(e)), bits(oracle.ef_accumulate(gh, eh)))
                pytest.fail("a bounded wait of dct_ef_threshold_compact ran out next to ordinary kernels")
            assert c == ecnt
            assert np.array_equal(host(ef.idx[:c]), eidx) and np.array_equal(bits(host(ef.val[:c])), bits(eval_))
            assert np.array_equal(bits(host(e)), bits(e_exp))


def test_dp_ef_give_up_delivers_nothing_and_keeps_the_corrected_gradient(dct):
    """The give-up path of the error-feedback compaction, reached from the host with a wait limit of one poll
    (every kernel still runs to its end).  Whatever the outcome, the documented state must hold: either the
    oracle's result, or count = DCT_COUNT_WORKSPACE_ERROR with e_out = g + e_in bit for bit (nothing delivered);
    the workspace then refuses further calls the same way, without losing anything, until it is initialised
    again."""
    n, k = 2_000_003, 20_000
    g = si.gaussian_gradient(n, DEV, 4300)
    e0 = si.residual_vector(n, DEV, 4301)
    gh, eh = host(g), host(e0)
    w = oracle.ef_accumulate(gh, eh)
    ef = EF(dct, n, capacity=n)
    exp = oracle.ef_select_threshold(gh, eh, k)
    assert ef.select(g, e0, k) == exp
    eidx, eval_, ecnt, e_exp = oracle.ef_threshold_compact(gh, eh, exp, oracle.EXACT_K)
    gave_up = 0
    try:
        dct.dct_set_wait_limit(1)
        for attempt in range(4):
            e = e0.clone()
            dct.dct_ef_threshold_compact(g, e, e, ef.thr, dct.DCT_EXACT_K, ef.idx, ef.val, ef.count, ef.ws)
            torch.cuda.synchronize()
            c = _raw_count(ef.count)
            if c != COUNT_ERROR:
                assert c == ecnt and np.array_equal(host(ef.idx[:c]), eidx)
                assert np.array_equal(bits(host(e)), bits(e_exp))
                continue
            gave_up += 1
            assert np.array_equal(bits(host(e)), bits(w))
            # the workspace now refuses: again nothing delivered, nothing lost (not in place this time)
            e_out = torch.full((n,), 5.0, device=DEV)
            dct.dct_ef_threshold_compact(g, e0, e_out, ef.thr, dct.DCT_EXACT_K, ef.idx, ef.val, ef.count, ef.ws)
            torch.cuda.synchronize()
            assert _raw_count(ef.count) == COUNT_ERROR
            assert np.array_equal(bits(host(e_out)), bits(w))
            cnt2 = torch.zeros(1, dtype=torch.int64, device=DEV)
            dct.dct_threshold_compact(g, ef.thr, dct.DCT_GE_TAU, ef.idx, ef.val, cnt2, ef.ws)
            assert _raw_count(cnt2) == COUNT_ERROR
            dct.dct_threshold_compact_workspace_init(ef.ws)
    finally:
        dct.dct_set_wait_limit(0)
    # back to the default limit and an initialised workspace: the call works
    e = e0.clone()
    idx, val, cnt, _ = ef.compact(g, e, e, dct.DCT_EXACT_K)
    assert cnt == ecnt and np.array_equal(idx, eidx) and np.array_equal(bits(val), bits(eval_))
    assert np.array_equal(bits(host(e)), bits(e_exp))
    print(f"gave up in {gave_up} of 4 attempts")


def test_dp_give_up_paths_of_select_and_compact_leave_a_verdict(dct):
    """With a wait limit of one poll the grid barriers of the selection and the count exchange of the
    compaction may give up.  Every kernel still ends, and the outputs always carry a verdict: the oracle's
    result or the error sentinel, never what the buffers held before."""
    cases = [(si.gaussian_gradient(1_000_003, DEV, 4400), 10_000),     # radix passes over the vector: grid barriers
             (si.student_t3_gradient(5_000_001, DEV, 4401), 5_000)]   # sample, partition, passes over candidates
    try:
        dct.dct_set_wait_limit(1)
        for g, k in cases:
            gh = host(g)
            exp = oracle.select_threshold(gh, k, method="nth")
            sws, cws = dct.new_select_workspace(g), dct.new_compact_workspace(g)
            good = torch.tensor([exp.tau_key, exp.n_gt, exp.n_eq, exp.tie_quota], dtype=torch.int64).to(torch.int32).to(DEV)
            eidx, eval_, ecnt = oracle.threshold_compact(gh, exp, oracle.GE_TAU)
            idx = torch.zeros(ecnt + 8, dtype=torch.int32, device=DEV)
            val = torch.zeros(ecnt + 8, device=DEV)
            for attempt in range(3):
                thr = torch.full((4,), 0x12345678, dtype=torch.int32, device=DEV)
                dct.dct_select_threshold(g, k, thr, sws)
                torch.cuda.synchronize()
                rec = [v & 0xFFFFFFFF for v in thr.cpu().tolist()]
                assert rec == [exp.tau_key, exp.n_gt, exp.n_eq, exp.tie_quota] or rec == [0xFFFFFFFF, 0, 0, 0], rec
                cnt = torch.full((1,), 77, dtype=torch.int64, device=DEV)
                dct.dct_threshold_compact(g, good, dct.DCT_GE_TAU, idx, val, cnt, cws)
                torch.cuda.synchronize()
                c = _raw_count(cnt)
                assert c in (ecnt, COUNT_ERROR)
                if c == ecnt:
                    assert np.array_equal(host(idx[:c]), eidx) and np.array_equal(bits(host(val[:c])), bits(eval_))
                else:
                    dct.dct_threshold_compact_workspace_init(cws)
    finally:
        dct.dct_set_wait_limit(0)


def test_random_mp_configurations(dct):
    """Forty seeded draws of (dtype, B, D, k, encoding, value structure): every forward kernel and every
    consumer against the oracle.  Value structures: post-ReLU, signed, four distinct values (ties everywhere),
    rows whose scale varies by orders of magnitude (the window prediction keeps missing), mostly zero rows,
    constant rows among ordinary ones."""
    rng = np.random.default_rng(20100889)
    for case in range(40):
        dtype = torch.bfloat16 if rng.random() < 0.7 else torch.float32
        D = int(rng.choice([8, 16, 24, 64, 72, 128, 200, 256, 264, 512, 520, 1000, 1024, 1032, 2048, 4096, 5120, 8192]))
        B = int(rng.integers(8192, 10000)) if rng.random() < 0.5 else int(rng.integers(1, 400))
        B = min(B, max(1, 12_000_000 // D))
        k = min(D, [1, max(1, D // 20), max(1, D // 3), D][int(rng.integers(0, 4))])
        kind, enc = int(rng.integers(0, 6)), int(rng.integers(0, 3))
        gen = torch.Generator(device=DEV).manual_seed(int(rng.integers(1 << 30)))
        x = torch.randn(B, D, device=DEV, generator=gen)
        if kind == 0:
            x = torch.relu(x)
        elif kind == 2:
            x = torch.randint(0, 4, (B, D), device=DEV, generator=gen).float() * 0.5
        elif kind == 3:
            x = torch.relu(x) * torch.exp(4 * torch.randn(B, 1, device=DEV, generator=gen))
        elif kind == 4:
            x = torch.relu(x - 1.5)
        elif kind == 5:
            x[::3] = 0.25
        x = x.to(dtype).contiguous()
        dy = torch.randn(B, D, device=DEV, generator=gen).to(dtype)
        val = torch.zeros(B, k, dtype=dtype, device=DEV)
        tau = torch.zeros(B, dtype=dtype, device=DEV)
        dval = torch.full((B, k), 3.0, device=DEV).to(dtype)
        out = torch.full((B, D), 3.0, device=DEV).to(dtype)
        xh, dyh = host(x), host(dy)
        ei, ev, et = oracle.rowtopk_fwd(xh, k)
        what = dict(case=case, dtype=dtype, B=B, D=D, k=k, kind=kind, enc=enc)
        if enc == 2:
            mask = torch.full((B, (D + 31) // 32), -1, dtype=torch.int32, device=DEV)
            dct.dct_rowtopk_fwd_bitmask(x, k, mask, val, tau)
            em, _, _ = oracle.rowtopk_fwd_bitmask(xh, k)
            assert np.array_equal(mask.cpu().numpy().view(np.uint32), em), what
            dct.dct_rowtopk_bwd_bitmask(dy, mask, dval)
            dct.dct_rowtopk_scatter_bitmask(mask, val, out)
        else:
            idx = torch.full((B, k), -1, dtype=torch.int16 if enc == 1 else torch.int32, device=DEV)
            (dct.dct_rowtopk_fwd_idx16 if enc == 1 else dct.dct_rowtopk_fwd)(x, k, idx, val, tau)
            got = idx.cpu().numpy()
            got = got.view(np.uint16).astype(np.int32) if enc == 1 else got
            assert np.array_equal(got, ei), what
            (dct.dct_rowtopk_bwd_idx16 if enc == 1 else dct.dct_rowtopk_bwd)(dy, idx, dval)
            (dct.dct_rowtopk_scatter_idx16 if enc == 1 else dct.dct_rowtopk_scatter)(idx, val, out)
        assert np.array_equal(bits(host(val).reshape(-1)), bits(ev.reshape(-1))), what
        assert np.array_equal(bits(host(tau)), bits(et)), what
        assert np.array_equal(bits(host(dval).reshape(-1)), bits(oracle.rowtopk_bwd(dyh, ei).reshape(-1))), what
        assert np.array_equal(bits(host(out).reshape(-1)), bits(oracle.rowscatter(ei, ev, D).reshape(-1))), what


def test_random_dp_configurations(dct):
    """Thirty seeded draws of (size, kept fraction, dtype, error feedback, mode, capacity, base offset, value
    structure: Gaussian, 95 % zeros, seven distinct values, log-normal magnitudes, sorted)."""
    rng = np.random.default_rng(889)
    for case in range(30):
        n = int(rng.integers(4_200_000, 7_000_000)) if rng.random() < 0.4 else int(rng.integers(1, 300_000))
        bf16 = rng.random() < 0.25
        ef = (not bf16) and rng.random() < 0.4
        k = min(n, max(1, int(n * float(rng.choice([1e-4, 1e-3, 5e-3, 0.02, 0.1, 0.3, 0.6, 1.0])))))
        kind, mode = int(rng.integers(0, 5)), int(rng.integers(0, 2))
        gen = torch.Generator(device=DEV).manual_seed(int(rng.integers(1 << 30)))
        g = torch.randn(n, device=DEV, generator=gen)
        if kind == 0:
            g = g * 1e-3
        elif kind == 1:
            g = g * (torch.rand(n, device=DEV, generator=gen) < 0.05)
        elif kind == 2:
            g = torch.randint(-3, 4, (n,), device=DEV, generator=gen).float()
        elif kind == 3:
            g = torch.exp(6 * g) * torch.sign(torch.randn(n, device=DEV, generator=gen))
        else:
            g = torch.sort(g)[0]
        off = 0 if ef else int(rng.integers(0, 4))
        buf = torch.zeros(n + 8, device=DEV, dtype=torch.bfloat16 if bf16 else torch.float32)
        buf[off:off + n] = g.to(buf.dtype)
        g = buf[off:off + n]
        gh = host(g)
        cap = int(min(n, max(16, k * float(rng.choice([0.5, 1.0, 2.0])))))
        what = dict(case=case, n=n, k=k, bf16=bf16, ef=ef, kind=kind, off=off, cap=cap, mode=mode)
        if ef:
            e = torch.randn(n, device=DEV, generator=gen) * 1e-3
            eh = host(e)
            efb = EF(dct, n, capacity=cap)
            thr = efb.select(g, e, k)
            exp = oracle.ef_select_threshold(gh, eh, k)
            assert thr == exp, what
            e_out = torch.empty_like(e)
            idx, val, cnt, guard = efb.compact(g, e, e_out, mode)
            ei, ev, ec, ee = oracle.ef_threshold_compact(gh, eh, exp, mode, capacity=cap)
            assert np.array_equal(bits(host(e_out)), bits(ee)), what
        else:
            dp = DP(dct, g, capacity=cap)
            thr = dp.select(k)
            exp = oracle.select_threshold(gh, k, method="nth")
            assert thr == exp, what
            idx, val, cnt, guard = dp.compact(mode)
            ei, ev, ec = oracle.threshold_compact(gh, exp, mode, capacity=cap)
        assert cnt == ec and np.array_equal(idx, ei) and np.array_equal(bits(val), bits(ev)), what
        assert np.all(guard == -7), what


# ------------------------------------------------------------------ the wider rows at the benchmark's full sizes
def test_ef_and_decompress_c4_full(dct):
    """Error feedback and decompression on the full c4 gradient (N = 2^28), the launch shape the
    benchmark times.  The oracle's threshold comes from its nth_element selection on its own sum."""
    g, k = si.config_c4(DEV)
    n = g.numel()
    e = si.residual_vector(n, DEV, 2100)
    ef = EF(dct, n, capacity=2 * k)
    thr = ef.select(g, e, k)
    gh, eh = host(g), host(e)
    w = oracle.ef_accumulate(gh, eh)
    exp = oracle.select_threshold(w, k, method="nth")
    assert thr == exp
    e_out = torch.empty_like(e)
    idx, val, cnt, guard = ef.compact(g, e, e_out, 1)
    eidx, eval_, ecnt, e_exp = oracle.ef_threshold_compact(gh, eh, exp, 1, capacity=2 * k)
    assert cnt == ecnt == k and np.array_equal(idx, eidx) and np.array_equal(bits(val), bits(eval_))
    assert np.all(guard == -7)
    assert np.array_equal(bits(host(e_out)), bits(e_exp))
    del e_exp, eh
    # decompress the message (count stays on the device) and check conservation on the device
    dense = torch.empty_like(g)
    dct.dct_scatter(ef.idx, ef.val, ef.count, dense)
    assert np.array_equal(bits(host(dense)), bits(oracle.scatter(eidx, eval_, n)))
    assert torch.equal(dense + e_out, torch.from_numpy(w).to(DEV))


def test_bitmask_and_decompress_c5_full(dct):
    x, dy, k = si.config_c5(DEV)
    B, D = x.shape
    assert (B, D, k) == (65536, 4096, 204)
    mask = torch.zeros(B, D // 32, dtype=torch.int32, device=DEV)
    val = torch.zeros(B, k, dtype=x.dtype, device=DEV)
    dct.dct_rowtopk_fwd_bitmask(x, k, mask, val, None)
    xh = host(x)
    emask, eval_, _ = oracle.rowtopk_fwd_bitmask(xh, k)
    assert np.array_equal(mask.cpu().numpy().view(np.uint32), emask) and np.array_equal(host(val), eval_)
    dval = torch.zeros_like(val)
    dct.dct_rowtopk_bwd_bitmask(dy, mask, dval)
    assert np.array_equal(host(dval), oracle.rowtopk_bwd_bitmask(host(dy), emask, k))
    out = torch.empty_like(x)
    dct.dct_rowtopk_scatter_bitmask(mask, val, out)
    want = oracle.rowscatter_bitmask(emask, eval_, D)
    assert np.array_equal(host(out), want)
    # the index form decompresses to the same dense matrix
    idx = torch.zeros(B, k, dtype=torch.int32, device=DEV)
    dct.dct_rowtopk_fwd(x, k, idx, val, None)
    out2 = torch.empty_like(x)
    dct.dct_rowtopk_scatter(idx, val, out2)
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))
