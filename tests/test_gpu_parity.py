"""GPU parity: libskm (through the C ABI) against the CPU oracle on the same seeded inputs.

Tolerances are those of the build's contract: assignments agree on >= 99.9 % of the points and
every disagreement is a near-tie (fp64 distances of the two centroids within 1e-4 relative);
centroids within 1e-3 relative L2; objective within 1e-4 relative.  Integer by-products (cluster
sizes, sampled indices) must be bit-exact; survivor counters within 0.1 %.
"""
import numpy as np
import pytest
import torch

from parity import EPS0, check_assignment, check_centroids, rel_l2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def skm():
    from paper_2603_20009_amd import skm as m
    m.lib()
    assert torch.cuda.is_available()
    return m


@pytest.fixture(scope="module")
def dg():
    from paper_2603_20009_amd import datagen
    return datagen


def cuda(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------ rotation
@pytest.mark.parametrize("n,d", [(300, 80), (1000, 128), (257, 100), (130, 75), (64, 1536), (1, 16)])
def test_rotation_gemm(skm, orc, dg, n, d):
    say("rotate", n, d)
    X = dg.mixture(n, d, 10, 1, "linear").numpy()
    R = orc.random_rotation(d, 3)
    got = skm.rotate(cuda(X), cuda(R)).cpu().numpy()
    assert np.abs(got - orc.rotate(X, R)).max() < 2e-6
    back = skm.rotate(cuda(got), cuda(R), True).cpu().numpy()     # (X R) R^T = X
    assert np.abs(back - X).max() < 4e-6
    want_t = X.astype(np.float64) @ R.astype(np.float64).T
    assert np.abs(skm.rotate(cuda(X), cuda(R), True).cpu().numpy() - want_t).max() < 2e-6


@pytest.mark.parametrize("scale", [1e-30, 1e-6, 1.0, 1e6, 1e30])
def test_split_gemm_keeps_fp32_accuracy_over_the_dynamic_range(skm, orc, scale):
    """The GEMMs multiply fp32 operands as scaled pairs of fp16 numbers.  The error against fp64 must stay at the
    fp32 level relative to the largest output whatever the magnitude of the inputs, also when a few columns are a
    thousand times larger than the rest, and zero inputs must give exact zeros."""
    rng = np.random.default_rng(7)
    n, d = 700, 256
    X = rng.standard_normal((n, d)).astype(np.float32)
    X[:, :5] *= 1000.0                      # a few dominant columns
    X[::7] *= 1e-3                          # and some tiny rows
    X = (X * np.float32(scale)).astype(np.float32)
    R = orc.random_rotation(d, 9)
    want = X.astype(np.float64) @ R.astype(np.float64)
    got = skm.rotate(cuda(X), cuda(R)).cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= 2e-6 * np.abs(want).max()
    # the tiny rows keep a relative accuracy of their own largest entry: 22-bit operands, not a global absolute error
    tiny = np.arange(n)[::7]
    assert (np.abs(got[tiny] - want[tiny]).max(1) <= 1e-4 * np.abs(want[tiny]).max(1)).all()
    Z = np.zeros((n, d), dtype=np.float32)
    assert not skm.rotate(cuda(Z), cuda(R)).cpu().numpy().any()
    # exact assignment on the same data agrees with fp64 except at near-ties (where squared distances fit fp32 at all)
    if not 1e-7 < scale < 1e7:
        return
    Y = X[rng.choice(n, 40, replace=False)]
    a, _ = skm.assign_exact(cuda(X), cuda(Y))
    ao, _ = orc.assign_full(X.astype(np.float64), Y.astype(np.float64))
    check_assignment(a.cpu().numpy(), ao, X, Y, min_agree=0.995)


def test_library_rotation_is_orthogonal_and_seeded(skm):
    for d in (16, 100, 384):
        R = skm.make_rotation(d, 5).cpu().numpy().astype(np.float64)
        assert np.abs(R @ R.T - np.eye(d)).max() < 1e-6
        assert np.abs(np.linalg.det(R)) == pytest.approx(1.0, abs=1e-4)
    # at the benchmark's size, several seeds: the error is that of rounding the fp64 matrix to fp32
    for seed in (0, 1, 2):
        R = skm.make_rotation(1536, seed).cpu().numpy().astype(np.float64)
        assert np.abs(R @ R.T - np.eye(1536)).max() < 1e-7 and np.abs(R.T @ R - np.eye(1536)).max() < 1e-7
    a = skm.make_rotation(64, 1).cpu().numpy()
    b = skm.make_rotation(64, 1).cpu().numpy()
    c = skm.make_rotation(64, 2).cpu().numpy()
    assert np.array_equal(a, b) and np.abs(a - c).max() > 0.05
    # entries of a Haar matrix have variance 1/d
    assert np.var(skm.make_rotation(384, 3).cpu().numpy()) == pytest.approx(1.0 / 384, rel=0.02)


# ------------------------------------------------------------------ exact assignment (iteration 1)
@pytest.mark.parametrize("n,d,k", [(1000, 128, 300), (257, 208, 129), (5000, 64, 17), (129, 16, 1), (3, 100, 3),
                                   (700, 75, 130)])
def test_exact_assignment(skm, orc, dg, n, d, k):
    say("exact", n, d, k)
    rng = np.random.default_rng(n + d + k)
    X = dg.mixture(n, d, 20, 2, "linear").numpy()
    Y = X[rng.choice(n, k, replace=False)] + (0.01 * rng.standard_normal((k, d))).astype(np.float32)
    a, dist = skm.assign_exact(cuda(X), cuda(Y))
    a = a.cpu().numpy()
    ao, do = orc.assign_full(X.astype(np.float64), Y.astype(np.float64))
    check_assignment(a, ao, X, Y, min_agree=0.999)
    same = a == ao
    assert np.abs(dist.cpu().numpy()[same] - do[same]).max() < 1e-6 * max(1.0, do.max())


# ------------------------------------------------------------------ one pruned step
def pruned_case(orc, dg, n, d, k, seed, recipe):
    rng = np.random.default_rng(seed)
    X = dg.mixture(n, d, 30, seed, recipe).numpy()
    R = orc.random_rotation(d, seed + 1)
    Y = X[rng.choice(n, k, replace=False)] + (0.01 * rng.standard_normal((k, d))).astype(np.float32)
    Xr = orc.rotate(X, R)
    Yr = orc.rotate(Y, R)
    prev = orc.assign_full(Xr, Yr)[0]
    prev[::4] = rng.integers(0, k, len(prev[::4]))          # a quarter of the points start from a poor incumbent
    return X, R, Y, Xr, Yr, prev.astype(np.int32)


@pytest.mark.parametrize("dense", [0.0125, 1.0, 0.0, 0.3])   # default, hand-over after the first test, dense tiles only
@pytest.mark.parametrize("n,d,k,dp,budget", [
    (2000, 128, 100, 0, 0),
    (3000, 208, 257, 0, 0),          # d' = 32, trailing 176 = 2 x 64 + 48 (short tail block)
    (1000, 1536, 64, 0, 0),          # d' = 192, 21 full blocks
    (1500, 1536, 300, 160, 0),       # d' not a multiple of 64: last block holds 32 dims
    (4000, 100, 50, 48, 0),          # d not a multiple of 16: padded rows
    (3000, 128, 130, 128, 0),        # d' = d: the first test is the exact comparison, no trailing block
    (5000, 128, 129, 0, 5248),       # hand-over list sized for 8 row tiles: 5 chunks of rows
])
def test_pruned_step(skm, orc, dg, n, d, k, dp, budget, dense):
    say("pruned", n, d, k, dp, budget, dense)
    X, R, Y, Xr, Yr, prev = pruned_case(orc, dg, n, d, k, n + k, "linear" if d < 512 else "embed")
    dp = dp or orc.dprime_init(d)
    ref = orc.assign_pruned(Xr, Yr, prev, dp, EPS0, 0)
    opts = skm.FitOptions(R=cuda(R), block_stats=True, pair_budget=budget, dense_frac=dense)
    a, dist, row = skm.assign(cuda(X), cuda(Y), cuda(prev), dp, opts)
    a = a.cpu().numpy()
    check_assignment(a, ref.assign, Xr, Yr)
    same = a == ref.assign
    # a distance finished inside a dense tile comes from the norm expansion accumulated in fp32 over d terms
    assert np.abs(dist.cpu().numpy()[same] - ref.dist[same]).max() < 2e-5 * max(1.0, ref.dist.max())
    surv_ref = n * (k - 1) - ref.pruned_first
    assert abs(row["survivors"] - surv_ref) <= max(2, 1e-3 * surv_ref)
    assert row["dprime"] == dp and row["nblocks"] == len(ref.enter) - 1
    for m in range(row["nblocks"]):
        assert abs(row["enter"][m] - ref.enter[m]) <= max(2, 1e-3 * ref.enter[m])
    assert abs(row["completed"] - ref.enter[-1]) <= max(2, 1e-3 * ref.enter[-1])
    assert row["objective"] == pytest.approx(ref.dist.sum(), rel=1e-5)
    assert row["changed"] == int((a != prev).sum())
    # every (pair, block) step ran either inside a dense tile or in the gather kernel
    if row["nblocks"] <= 32:
        assert row["dense_pair_blocks"] + row["gather_pair_blocks"] == sum(row["enter"][: row["nblocks"]])
    assert (row["gather_pairs"] == 0) == (row["gather_pair_blocks"] == 0) and row["gather_pairs"] <= row["survivors"]
    if dense == 0.0:
        assert row["gather_pairs"] == 0
    if dense == 1.0 and row["nblocks"] > 0:
        assert row["gather_pairs"] == row["survivors"] and row["dense_pair_blocks"] == 0


@pytest.mark.parametrize("dense", [0.0125, 1.0])
@pytest.mark.parametrize("n,d,k,dp,budget", [
    (2000, 128, 100, 0, 0),
    (3000, 208, 257, 0, 0),          # d' = 32; three column tiles, the last with one centroid
    (1000, 1536, 64, 0, 0),
    (1500, 1536, 300, 160, 0),       # d' = 160: the first slab starts 16 dimensions before the row
    (4000, 100, 50, 48, 0),          # padded rows
    (5000, 128, 129, 0, 5248),       # 5 chunks of rows
    (6000, 64, 1100, 16, 0),         # nine column tiles: most are dead for a row tile
])
def test_pruned_step_with_low_precision_filter(skm, orc, dg, n, d, k, dp, budget, dense):
    """The same step with the one-product first filter in front (params->screen = 1): the exact kernel then only sees
    the centroids that filter lists for a row tile.  Nothing that Algorithm 1's first test keeps may be lost: labels,
    distances and every counter must match the oracle exactly as without the filter."""
    say("screened", n, d, k, dp, budget, dense)
    X, R, Y, Xr, Yr, prev = pruned_case(orc, dg, n, d, k, n + k, "linear" if d < 512 else "embed")
    dp = dp or orc.dprime_init(d)
    ref = orc.assign_pruned(Xr, Yr, prev, dp, EPS0, 0)
    opts = skm.FitOptions(R=cuda(R), block_stats=True, pair_budget=budget, dense_frac=dense, screen=1)
    a, dist, row = skm.assign(cuda(X), cuda(Y), cuda(prev), dp, opts)
    a = a.cpu().numpy()
    check_assignment(a, ref.assign, Xr, Yr)
    same = a == ref.assign
    assert np.abs(dist.cpu().numpy()[same] - ref.dist[same]).max() < 2e-5 * max(1.0, ref.dist.max())
    surv_ref = n * (k - 1) - ref.pruned_first
    assert abs(row["survivors"] - surv_ref) <= max(2, 1e-3 * surv_ref)
    for m in range(row["nblocks"]):
        assert abs(row["enter"][m] - ref.enter[m]) <= max(2, 1e-3 * ref.enter[m])
    assert abs(row["completed"] - ref.enter[-1]) <= max(2, 1e-3 * ref.enter[-1])
    assert row["objective"] == pytest.approx(ref.dist.sum(), rel=1e-5)
    assert row["changed"] == int((a != prev).sum())
    nrt, nct = -(-n // 128), -(-k // 128)
    assert row["screen_dims"] > 0 and 0 < row["listed_tiles"] <= nrt * nct
    # without the filter the step gives the same labels (the tests applied to a pair are the same)
    b, _, row0 = skm.assign(cuda(X), cuda(Y), cuda(prev), dp, skm.FitOptions(R=cuda(R), block_stats=True,
                                                                              pair_budget=budget, dense_frac=dense, screen=-1))
    assert row0["screen_dims"] == 0 and row0["listed_tiles"] == 0
    assert row0["survivors"] == row["survivors"] and row0["enter"] == row["enter"] and row0["completed"] == row["completed"]
    assert (b.cpu().numpy() != a).sum() <= 1


@pytest.mark.parametrize("screen", [-1, 1])
def test_steps_on_rows_of_heavy_tailed_norm(skm, orc, dg, screen):
    """The split-fp16 operands share one power-of-two scale per matrix: an entry keeps 22 significant bits while it
    is at least 2^-18 of the matrix's largest entry, below that an absolute error of 2^-40 of the largest.  Rows whose
    norms span five orders of magnitude (log-normal factors, clipped to 1e-3 .. 1e2) must still meet the near-tie
    contract in the exact step and in a pruned step, with and without the low-precision first filter."""
    say("heavy-tailed norms, screen", screen)
    n, d, k = 6000, 256, 300
    rng = np.random.default_rng(77)
    scale = np.clip(np.exp(2.5 * rng.standard_normal(n)), 1e-3, 1e2).astype(np.float32)
    X = (dg.mixture(n, d, 30, 5, "linear").numpy() * scale[:, None]).astype(np.float32)
    pick = rng.choice(n, k, replace=False)
    Y = (X[pick] * (1.0 + 0.01 * rng.standard_normal((k, d)))).astype(np.float32)
    assert np.linalg.norm(X, axis=1).max() / np.linalg.norm(X, axis=1).min() > 3e4
    R = orc.random_rotation(d, 78)
    Xr, Yr = orc.rotate(X, R), orc.rotate(Y, R)
    # exact step: iteration 1 of a fit (its centroids are the seeded sample of the rows), behind the filter or not
    fr = skm.fit(cuda(X), k, 1, 3, skm.FitOptions(R=cuda(R), final_assign=False, screen=screen))
    assert (fr.trace[0]["screen_dims"] > 0) == (screen > 0)
    idx = orc.sample_rows(3, n, k)
    ao, _ = orc.assign_full(Xr, Xr[idx])
    check_assignment(fr.assign.cpu().numpy(), ao, Xr, Xr[idx])
    # pruned step from a partly poor incumbent
    prev = orc.assign_full(Xr, Yr)[0].astype(np.int32)
    prev[::4] = rng.integers(0, k, len(prev[::4]))
    dp = orc.dprime_init(d)
    ref = orc.assign_pruned(Xr, Yr, prev, dp, EPS0, 0)
    b, _, row = skm.assign(cuda(X), cuda(Y), cuda(prev), dp, skm.FitOptions(R=cuda(R), block_stats=True, screen=screen))
    check_assignment(b.cpu().numpy(), ref.assign, Xr, Yr)
    surv_ref = n * (k - 1) - ref.pruned_first
    assert abs(row["survivors"] - surv_ref) <= max(2, 1e-3 * surv_ref)
    assert abs(row["completed"] - ref.enter[-1]) <= max(2, 1e-3 * ref.enter[-1])


@pytest.mark.parametrize("case", range(14))
def test_filtered_steps_over_seeded_shapes(skm, orc, dg, case):
    """Seeded odd shapes through the filtered step and the filtered incumbent search: point and centroid counts around the
    edges of the 128- and 256-wide tiles, d not a multiple of 16, d' anywhere between 16 and d."""
    rng = np.random.default_rng(1000 + case)
    n = int(rng.choice([1, 2, 127, 129, 255, 257, 300, 1000, 2049, 3000]))
    k = int(min(rng.choice([1, 2, 3, 127, 128, 129, 255, 256, 257, 513, 700]), max(n, 1)))
    d = int(rng.choice([16, 20, 48, 100, 128, 200, 272, 400]))
    ds = (d + 15) // 16 * 16
    dp = int(rng.integers(1, max(d // 16, 1) + 1)) * 16
    dp = min(dp, (d // 16) * 16) if d >= 16 else 16
    say("filtered step, seeded shape", case, n, d, k, dp)
    X = dg.mixture(n, d, 12, 50 + case, "linear").numpy()
    R = orc.random_rotation(d, 60 + case)
    Y = X[rng.choice(n, k, replace=False)] + (0.01 * rng.standard_normal((k, d))).astype(np.float32)
    Xr, Yr = orc.rotate(X, R), orc.rotate(Y, R)
    prev = orc.assign_full(Xr, Yr)[0].astype(np.int32)
    prev[::3] = rng.integers(0, k, len(prev[::3]))
    for pv in (prev, None):
        ref = orc.assign_pruned(Xr, Yr, pv, dp, EPS0, 0)
        a, dist, row = skm.assign(cuda(X), cuda(Y), None if pv is None else cuda(pv), dp,
                                  skm.FitOptions(R=cuda(R), block_stats=True, screen=1))
        a = a.cpu().numpy()
        check_assignment(a, ref.assign, Xr, Yr, min_agree=0.995 if n < 2000 else 0.999)
        surv_ref = n * (k - 1) - ref.pruned_first
        assert abs(row["survivors"] - surv_ref) <= max(2, 1e-3 * surv_ref)
        assert abs(row["completed"] - ref.enter[-1]) <= max(2, 1e-3 * ref.enter[-1])
        assert row["objective"] == pytest.approx(ref.dist.sum(), rel=1e-5, abs=1e-9)


def test_pruned_step_without_previous_assignment(skm, orc, dg):
    X, R, Y, Xr, Yr, _ = pruned_case(orc, dg, 2500, 128, 90, 5, "linear")
    ref = orc.assign_pruned(Xr, Yr, None, 16, EPS0, 0)
    a, dist, _ = skm.assign(cuda(X), cuda(Y), None, 16, skm.FitOptions(R=cuda(R)))
    check_assignment(a.cpu().numpy(), ref.assign, Xr, Yr)


@pytest.mark.parametrize("n,d,k,dp", [(6000, 208, 300, 48), (3000, 128, 257, 16), (5000, 1536, 300, 192),
                                      (4000, 100, 130, 80)])
def test_step_without_previous_assignment_finds_its_incumbents_through_the_filter(skm, orc, dg, n, d, k, dp):
    """A step that comes without incumbents takes, for every point, the centroid nearest on the first d' dimensions.  With
    the first filter on, that search is the one-product multiply over d' dimensions plus exact distances for the few
    candidates (d' not a multiple of 64: the last gathered block is cut at d').  Same oracle, same contract, and the
    same counters as the search by the three-product GEMM."""
    say("no incumbents, filtered search", n, d, k, dp)
    X, R, Y, Xr, Yr, _ = pruned_case(orc, dg, n, d, k, n + d, "linear" if d < 512 else "embed")
    ref = orc.assign_pruned(Xr, Yr, None, dp, EPS0, 0)
    a1, d1, row1 = skm.assign(cuda(X), cuda(Y), None, dp, skm.FitOptions(R=cuda(R), block_stats=True, screen=1))
    a0, d0, row0 = skm.assign(cuda(X), cuda(Y), None, dp, skm.FitOptions(R=cuda(R), block_stats=True, screen=-1))
    for a, dist, row in ((a1, d1, row1), (a0, d0, row0)):
        a = a.cpu().numpy()
        check_assignment(a, ref.assign, Xr, Yr)
        same = a == ref.assign
        assert np.abs(dist.cpu().numpy()[same] - ref.dist[same]).max() < 2e-5 * max(1.0, ref.dist.max())
        surv_ref = n * (k - 1) - ref.pruned_first
        assert abs(row["survivors"] - surv_ref) <= max(2, 1e-3 * surv_ref)
        assert abs(row["completed"] - ref.enter[-1]) <= max(2, 1e-3 * ref.enter[-1])
        assert row["objective"] == pytest.approx(ref.dist.sum(), rel=1e-5)
    assert row1["screen_dims"] > 0 and row0["screen_dims"] == 0
    # the two searches may pick different incumbents only at ties of the partial distance: a handful of points
    assert abs(row1["survivors"] - row0["survivors"]) <= max(2, 1e-4 * row0["survivors"])
    assert (a1 != a0).sum().item() <= 2


def test_pruned_step_without_statistical_test_is_exact(skm, orc, dg):
    X, R, Y, Xr, Yr, prev = pruned_case(orc, dg, 3000, 144, 77, 9, "linear")
    exact, _ = orc.assign_full(Xr, Yr)
    a, dist, row = skm.assign(cuda(X), cuda(Y), cuda(prev), 0, skm.FitOptions(R=cuda(R), eps0=float("inf")))
    check_assignment(a.cpu().numpy(), exact, Xr, Yr, min_agree=0.9995)
    # and the same with no rotation at all (R = I)
    a2, _, _ = skm.assign(cuda(X), cuda(Y), cuda(prev), 0, skm.FitOptions(rotate=False, eps0=float("inf")))
    check_assignment(a2.cpu().numpy(), orc.assign_full(X.astype(np.float64), Y.astype(np.float64))[0], X, Y,
                     min_agree=0.9995)


def test_default_entry_points(skm, orc, dg):
    """skm_assign / skm_fit (defaults, library's own rotation): checked through properties."""
    n, d, k = 6000, 128, 40
    X = dg.mixture(n, d, 50, 21, "linear")
    Xc = X.cuda()
    cent, a = skm.fit_default(Xc, k, 6, 3)
    Xn = X.numpy().astype(np.float64)
    Yn = cent.cpu().numpy().astype(np.float64)
    D = ((Xn[:, None, :] - Yn[None, :, :]) ** 2).sum(2)
    an = a.cpu().numpy()
    assert (an == D.argmin(1)).mean() > 0.995                      # final pass: nearest centroid, rare false prunes
    ref = orc.fit(X.numpy(), k, 6, 3, orc.FitParams(eps0=EPS0), R=orc.random_rotation(d, 3))
    assert D.min(1).sum() == pytest.approx(ref.trace[-1]["objective"], rel=0.02)   # same quality, other rotation
    a2, dist2 = skm.assign_default(Xc, cent, a)
    assert (a2.cpu().numpy() == an).mean() > 0.999
    assert np.allclose(dist2.cpu().numpy(), D[np.arange(n), a2.cpu().numpy()], rtol=1e-4, atol=1e-6)


def test_bad_labels_are_refused(skm, dg):
    X = dg.mixture(500, 32, 5, 1, "linear").cuda()
    Y = X[:7].clone()
    prev = torch.full((500,), 7, dtype=torch.int32, device="cuda")
    with pytest.raises(skm.SkmError):
        skm.assign(X, Y, prev)
    with pytest.raises(skm.SkmError):
        skm.update(X, prev, Y)


def test_argument_errors_return_codes_and_leave_outputs_untouched(skm, dg):
    """Straight through the C ABI: every argument error comes back as SKM_EINVAL (a workspace that is too small as
    SKM_ENOMEM) with a message, before anything is enqueued, and the output arrays keep what they held."""
    import ctypes as C
    L = skm.lib()
    n, d, k = 2000, 64, 20
    X = dg.mixture(n, d, 8, 2, "linear").cuda()
    cent = torch.full((k, d), 7.0, device="cuda")
    assign = torch.full((n,), -9, dtype=torch.int32, device="cuda")
    dist = torch.full((n,), -3.0, device="cuda")
    vp = lambda t: C.c_void_p(t.data_ptr())

    def params(**kw):
        p = skm.Params()
        L.skm_params_default(C.byref(p))
        for name, v in kw.items():
            setattr(p, name, v)
        return p

    def fit(nn=n, dd=d, kk=k, iters=3, p=None, x=X, c=cent):
        return L.skm_fit_ex(None if x is None else vp(x), nn, dd, kk, iters, C.c_uint64(1), None if p is None else C.byref(p),
                            None if c is None else vp(c), vp(assign), vp(dist))

    ws = torch.empty(1024, dtype=torch.uint8, device="cuda")
    cases = [
        (fit(kk=n + 1), -1), (fit(kk=0), -1), (fit(nn=0), -1), (fit(dd=0), -1), (fit(dd=20000), -1), (fit(iters=0), -1),
        (fit(x=None), -1), (fit(c=None), -1),
        (fit(p=params(dprime_frac=0.0)), -1), (fit(p=params(dprime_frac=1.5)), -1), (fit(p=params(eps0=-1.0)), -1),
        (fit(p=params(tau_group=5)), -1), (fit(p=params(conv_tol=2.0)), -1),
        (fit(p=params(sample_frac=0.5, final_assign=0)), -1), (fit(p=params(angular=1, sample_frac=0.5)), -1),
        (fit(p=params(workspace=ws.data_ptr(), workspace_bytes=1024)), -2),
        (L.skm_assign_ex(vp(X), n, d, vp(cent), k, None, 0, C.byref(params(tau_group=3)), vp(assign), vp(dist)), -1),
        (L.skm_assign_ex(vp(X), n, d, vp(cent), k, None, 0, C.byref(params(workspace=ws.data_ptr(), workspace_bytes=1024)),
                         vp(assign), vp(dist)), -2),
        (L.skm_assign_ex(vp(X), n, d, None, k, None, 0, None, vp(assign), vp(dist)), -1),
        (L.skm_fit_hierarchical(vp(X), n, d, k, 0, 5, C.c_uint64(1), None, vp(cent), vp(assign), vp(dist), None, None), -1),
        (L.skm_fit_hierarchical(vp(X), n, d, k, 3, 5, C.c_uint64(1), C.byref(params(etr=1)), vp(cent), vp(assign), vp(dist),
                                None, None), -1),
        (L.skm_assign_exact_static(vp(X), n, d + 1, vp(cent), k, None, vp(assign), vp(dist)), -1),
        (L.skm_etr_ground_truth(vp(X), n, d, vp(X), 10, 0, None, vp(assign)), -1),
    ]
    for i, (rc, want) in enumerate(cases):
        assert rc == want, f"case {i}: returned {rc}, expected {want}"
    assert L.skm_last_error().decode() != ""
    assert L.skm_strerror(-1).decode() != L.skm_strerror(-2).decode() != ""
    torch.cuda.synchronize()
    assert (assign == -9).all() and (dist == -3.0).all() and (cent == 7.0).all()
    # and the same buffers take a good call afterwards
    assert fit() == 0
    torch.cuda.synchronize()
    assert (assign >= 0).all() and (assign < k).all() and (dist >= 0).all() and not (cent == 7.0).all()


# ------------------------------------------------------------------ update
@pytest.mark.parametrize("n,d,k", [(5000, 128, 100), (3000, 100, 37), (40_000, 64, 5), (2000, 1536, 700)])
def test_update(skm, orc, dg, n, d, k):
    say("update", n, d, k)
    rng = np.random.default_rng(n + k)
    X = dg.mixture(n, d, 30, 4, "linear").numpy()
    a = rng.integers(0, max(k - 2, 1), n).astype(np.int32)     # the last two clusters stay empty
    if k == 5:
        a[: n * 3 // 4] = 1                                    # one cluster above the in-LDS sort limit
    Y0 = rng.standard_normal((k, d)).astype(np.float32)
    Yg = cuda(Y0)
    cnt = skm.update(cuda(X), cuda(a), Yg).cpu().numpy()
    Yo, co = orc.update(X.astype(np.float64), a, Y0.astype(np.float64))
    assert (cnt == co).all()                                   # integer work: bit-exact
    assert np.abs(Yg.cpu().numpy() - Yo).max() < 1e-6
    assert np.array_equal(Yg.cpu().numpy()[co == 0], Y0[co == 0])


# ------------------------------------------------------------------ whole fit
def fit_pair(skm, orc, X, k, iters, seed, R, init_idx=None, **kw):
    kw.setdefault("eps0", EPS0)
    idx = orc.sample_rows(seed, len(X), k) if init_idx is None else np.asarray(init_idx, dtype=np.int64)
    okw = {a: b for a, b in kw.items() if a != "screen"}     # an execution choice of the library, not of the method
    ref = orc.fit(X, k, iters, seed, orc.FitParams(**okw), R=R, init_idx=idx)
    # without init_idx the library draws the same initial rows from the seed
    opts = skm.FitOptions(R=None if R is None else cuda(R), rotate=R is not None, block_stats=True,
                          init_idx=None if init_idx is None else list(idx), **kw)
    got = skm.fit(cuda(X), k, iters, seed, opts)
    return ref, got


def test_fit_c1_full_parity(skm, orc, dg):
    """Workload C1 (20 000 x 128, k = 100, 10 iterations), free-running: objective, d', empty clusters and prune fraction
    at every step; labels and centroids under the whole-fit rule (a disagreement is a near-tie under the oracle's
    centroids, or the nearest centroid under the library's own after the two runs split at a tie; the centroid bound over
    the clusters with the same members).  test_lockstep_fit_c1 holds every step to the strict rule."""
    X = dg.config_data("C1").numpy()
    R = orc.random_rotation(128, 42)
    ref, got = fit_pair(skm, orc, X, 100, 10, 42, R, adjust_dprime=False)
    Xr = orc.rotate(X, R)
    check_assignment(got.assign.cpu().numpy(), ref.assign, Xr, ref.centroids_rot, own=(X, got.centroids.cpu().numpy()))
    clean = check_centroids(got.centroids.cpu().numpy(), ref.centroids, got.assign.cpu().numpy(), ref.assign)
    assert got.iters_run == ref.iters_run == 10 and len(got.trace) == len(ref.trace) == 11
    for g, r in zip(got.trace, ref.trace):
        assert g["objective"] == pytest.approx(r["objective"], rel=1e-4)
        assert g["dprime"] == r["dprime"] and g["nempty"] == r["nempty"]
        assert g["prune_frac"] == pytest.approx(r["prune_frac"], abs=1e-3)
    obj = [g["objective"] for g in got.trace]
    assert all(b <= a * (1 + 1e-6) for a, b in zip(obj, obj[1:]))          # Lloyd objective never increases
    same = (got.assign.cpu().numpy() == ref.assign) & np.isin(ref.assign, clean)   # clusters with the same members
    assert same.mean() > 0.97
    assert np.abs(got.dist.cpu().numpy()[same] - ref.dist[same]).max() < 1e-5


def test_fit_with_dprime_adjustment(skm, orc, dg):
    X = dg.mixture(12_000, 256, 64, 8, "embed").numpy()
    R = orc.random_rotation(256, 8)
    ref, got = fit_pair(skm, orc, X, 64, 8, 5, R, adjust_dprime=True)
    assert [g["dprime"] for g in got.trace] == [r["dprime"] for r in ref.trace]
    assert len({g["dprime"] for g in got.trace[1:]}) > 1                    # the controller did move d'
    assert got.trace[-1]["objective"] == pytest.approx(ref.trace[-1]["objective"], rel=1e-4)
    check_assignment(got.assign.cpu().numpy(), ref.assign, orc.rotate(X, R), ref.centroids_rot,
                     own=(X, got.centroids.cpu().numpy()))
    check_centroids(got.centroids.cpu().numpy(), ref.centroids, got.assign.cpu().numpy(), ref.assign)


def test_fit_without_rotation_or_final_pass(skm, orc, dg):
    X = dg.mixture(5000, 96, 20, 3, "linear").numpy()
    ref, got = fit_pair(skm, orc, X, 24, 5, 11, None, adjust_dprime=False, final_assign=False)
    check_assignment(got.assign.cpu().numpy(), ref.assign, X, ref.centroids_rot)
    assert rel_l2(got.centroids.cpu().numpy(), ref.centroids) < 1e-3
    # centroids are the means of the returned (last in-loop) assignment
    a = got.assign.cpu().numpy()
    S = np.zeros((24, 96))
    np.add.at(S, a, X.astype(np.float64))
    assert np.abs(got.centroids.cpu().numpy() - S / np.bincount(a, minlength=24)[:, None]).max() < 1e-6


@pytest.mark.parametrize("screen", [0, 1])
def test_fit_splits_empty_clusters_like_the_oracle(skm, orc, dg, screen):
    """Repeated initial rows leave clusters empty after iteration 1 (identical centroids tie and the
    lowest index wins on both sides, also when the low-precision filter picks the candidates of iteration 1);
    the split must re-seed them from the same donors."""
    X = dg.mixture(6000, 64, 24, 10, "linear").numpy()
    R = orc.random_rotation(64, 10)
    idx = orc.sample_rows(1, 6000, 12)
    idx[1] = idx[0]
    idx[2] = idx[0]
    idx[7] = idx[6]
    ref, got = fit_pair(skm, orc, X, 12, 5, 1, R, init_idx=idx, adjust_dprime=False, screen=screen)
    assert [g["nempty"] for g in got.trace] == [r["nempty"] for r in ref.trace] and ref.trace[0]["nempty"] == 3
    check_assignment(got.assign.cpu().numpy(), ref.assign, orc.rotate(X, R), ref.centroids_rot,
                     own=(X, got.centroids.cpu().numpy()))
    assert rel_l2(got.centroids.cpu().numpy(), ref.centroids) < 1e-3
    assert (np.bincount(got.assign.cpu().numpy(), minlength=12) > 0).all()


@pytest.mark.parametrize("screen", [0, 1])
@pytest.mark.parametrize("case", range(8))
def test_fit_over_seeded_shapes(skm, orc, dg, case, screen):
    """Whole fits on shapes drawn from a seed: d not a multiple of 16 or 64, k below, at and above one tile, row
    counts that leave ragged tiles, with and without rotation and d' adjustment."""
    rng = np.random.default_rng(1000 + case)
    n = int(rng.integers(150, 6000))
    d = int(rng.choice([16, 24, 40, 72, 100, 129, 200, 333]))
    k = int(min(rng.choice([2, 7, 31, 127, 128, 129, 260]), n // 3))
    iters = int(rng.integers(2, 6))
    kind = ["linear", "embed"][case % 2]
    rotate = case % 3 != 2
    X = dg.mixture(n, d, max(k // 2, 3), 50 + case, kind).numpy()
    R = orc.random_rotation(d, case) if rotate else None
    say("fit shape", case, n, d, k, iters, kind, "rotate" if rotate else "plain")
    # screen = 1: the low-precision filter in front of iteration 1 and of every pruned step
    ref, got = fit_pair(skm, orc, X, k, iters, 77 + case, R, adjust_dprime=case % 2 == 0, screen=screen)
    assert (got.trace[0]["screen_dims"] > 0) == (screen == 1)
    Xr = orc.rotate(X, R) if rotate else X
    check_assignment(got.assign.cpu().numpy(), ref.assign, Xr, ref.centroids_rot, own=(X, got.centroids.cpu().numpy()))
    check_centroids(got.centroids.cpu().numpy(), ref.centroids, got.assign.cpu().numpy(), ref.assign)
    assert [g["dprime"] for g in got.trace] == [r["dprime"] for r in ref.trace]
    assert got.trace[-1]["objective"] == pytest.approx(ref.trace[-1]["objective"], rel=1e-4)
    assert np.array_equal(np.bincount(got.assign.cpu().numpy(), minlength=k) == 0,
                          np.bincount(ref.assign, minlength=k) == 0)


def test_fit_regroups_points_across_row_chunks(skm, orc, dg):
    """From the third step on a long fit works on the points grouped by cluster (labels and distances come back in the
    caller's order).  With a small pair budget the rows are also processed in several chunks; the result must follow
    the oracle like any other fit, and must not depend on the budget beyond near-ties."""
    X = dg.mixture(9000, 100, 60, 31, "embed").numpy()
    R = orc.random_rotation(100, 4)
    idx = orc.sample_rows(19, 9000, 70)
    ref = orc.fit(X, 70, 7, 19, orc.FitParams(eps0=EPS0, adjust_dprime=True), R=R, init_idx=idx)
    Xr = orc.rotate(X, R)
    fits = []
    for budget in (0, 150_000):     # default, and about 2000 rows (16 row tiles) per chunk
        got = skm.fit(cuda(X), 70, 7, 19, skm.FitOptions(R=cuda(R), eps0=EPS0, adjust_dprime=True, pair_budget=budget))
        a = got.assign.cpu().numpy()
        check_assignment(a, ref.assign, Xr, ref.centroids_rot, own=(X, got.centroids.cpu().numpy()))
        clean = check_centroids(got.centroids.cpu().numpy(), ref.centroids, a, ref.assign)
        assert [g["dprime"] for g in got.trace] == [r["dprime"] for r in ref.trace]
        assert got.trace[-1]["objective"] == pytest.approx(ref.trace[-1]["objective"], rel=1e-4)
        same = (a == ref.assign) & np.isin(ref.assign, clean)
        assert same.mean() > 0.97
        assert np.abs(got.dist.cpu().numpy()[same] - ref.dist[same]).max() < 1e-5      # distances sit with their points
        assert float(got.dist.sum()) == pytest.approx(got.trace[-1]["objective"], rel=1e-5)
        fits.append(a)
    assert (fits[0] == fits[1]).mean() >= 0.999


def test_fit_stops_at_convergence_like_the_oracle(skm, orc, dg):
    """conv_tol: the fit stops after the first iteration t >= 2 in which at most that share of the labels changed."""
    X = dg.mixture(8000, 64, 12, 6, "linear").numpy()
    R = orc.random_rotation(64, 6)
    for tol in (0.01, 1e-4, 1.0):
        ref, got = fit_pair(skm, orc, X, 12, 40, 6, R, conv_tol=tol)
        assert got.iters_run == ref.iters_run and len(got.trace) == len(ref.trace) == ref.iters_run + 1
        assert ref.iters_run < 40 and (tol < 1.0 or ref.iters_run == 2)
        assert got.trace[got.iters_run - 1]["changed"] <= tol * len(X)
        check_assignment(got.assign.cpu().numpy(), ref.assign, orc.rotate(X, R), ref.centroids_rot,
                         own=(X, got.centroids.cpu().numpy()))
        check_centroids(got.centroids.cpu().numpy(), ref.centroids, got.assign.cpu().numpy(), ref.assign)
    with pytest.raises(skm.SkmError):
        skm.fit(cuda(X), 12, 3, 6, skm.FitOptions(R=cuda(R), tau_group=5))      # only the frozen threshold is built
    skm.fit(cuda(X), 12, 2, 6, skm.FitOptions(R=cuda(R), tau_group=12))         # ... which is what G = k says


def test_update_after_a_split_that_moved_no_point(skm, orc, dg):
    """Ten distinct points, fifty copies each, twelve centroids: two clusters are empty after iteration 1 and every
    split re-seeds them next to a donor whose members are all equidistant from the two perturbed rows (exact ties:
    which way they fall is rounding, so the labels are not compared with the oracle here).  Whenever no label changes
    in the step after a split, the update must still put the donor back on the mean of its members before the next
    split perturbs it again (Algorithm 1 updates, then splits): at the end every cluster with members sits on their
    mean, or on the mean perturbed once, never twice."""
    eps = 1.0 / 1024.0
    base = dg.mixture(10, 32, 4, 2, "linear").numpy()
    X = np.repeat(base, 50, axis=0)
    idx = list(range(0, 500, 50)) + [101, 102]                # all ten points, and two more copies of the third
    # seven iterations: in this run the seventh is one that changes no label after the split of the sixth, so the
    # centroids returned are those of the update in question
    got = skm.fit(cuda(X), 12, 7, 5, skm.FitOptions(rotate=False, init_idx=idx, adjust_dprime=False,
                                                     final_assign=False))
    assert got.trace[0]["nempty"] == 2 and got.trace[-1]["changed"] == 0 and got.trace[-2]["nempty"] > 0
    quiet_after_split = [t for t in range(1, len(got.trace)) if got.trace[t]["changed"] == 0 and got.trace[t - 1]["nempty"] > 0]
    say("steps without a label change after a split:", quiet_after_split, [(g["changed"], g["nempty"]) for g in got.trace])
    assert quiet_after_split, "the scenario did not occur in this run (pick other points)"
    a = got.assign.cpu().numpy()
    Y = got.centroids.cpu().numpy().astype(np.float64)
    s = np.where(np.arange(32) % 2 == 0, 1.0, -1.0)
    for c in range(12):
        if (a == c).any():
            mean = X[a == c].astype(np.float64).mean(0)
            errs = [np.abs(Y[c] - mean * f).max() for f in (1.0, 1.0 + eps * s, 1.0 - eps * s)]
            assert min(errs) < 1e-6, (c, errs)


def test_filtered_first_iteration_is_the_exact_assignment(skm, orc, dg):
    """Iteration 1 behind the low-precision filter: among the candidates the one-product multiply leaves for a point
    the exact nearest centroid must always be present.  Several thousand centroids (the regime it is for), a ragged
    last tile in both directions, and rows of very different length (the bound scales with the row's norm)."""
    rng = np.random.default_rng(17)
    n, d, k = 30_100, 96, 2300
    X = dg.mixture(n, d, 300, 9, "embed").numpy() * rng.uniform(0.05, 20.0, (n, 1)).astype(np.float32)
    R = orc.random_rotation(d, 5)
    idx = orc.sample_rows(3, n, k)
    got = skm.fit(cuda(X), k, 1, 3, skm.FitOptions(R=cuda(R), final_assign=False))          # screen = 0: on from 2048 centroids
    off = skm.fit(cuda(X), k, 1, 3, skm.FitOptions(R=cuda(R), final_assign=False, screen=-1))
    assert got.trace[0]["screen_dims"] > 0 and got.trace[0]["gather_pairs"] >= n and off.trace[0]["screen_dims"] == 0
    say("candidates per point:", got.trace[0]["gather_pairs"] / n)
    Xr = orc.rotate(X, R)
    a_ref, d_ref = orc.assign_full(Xr, Xr[idx])
    for fr in (got, off):
        a = fr.assign.cpu().numpy()
        check_assignment(a, a_ref, Xr, Xr[idx], min_agree=0.9995)
        same = a == a_ref
        assert np.abs(fr.dist.cpu().numpy()[same] - d_ref[same]).max() < 2e-5 * d_ref.max()
        assert fr.trace[0]["objective"] == pytest.approx(d_ref.sum(), rel=1e-5)
    assert (got.assign != off.assign).sum() <= 3
    assert got.trace[0]["gather_pairs"] < 40 * n      # a handful of candidates per point, not the k of a full scan


def test_filtered_first_iteration_falls_back_when_the_candidates_flood_the_list(skm, orc):
    """A blob so tight that every centroid lies inside every point's rounding band: the one-product pass cannot rule out
    anything, the candidate list (16 slots per point and list part) overflows, and the step must notice and run the
    full three-product GEMM instead, with the exact result."""
    rng = np.random.default_rng(23)
    n, d, k = 4000, 64, 400
    u = rng.standard_normal(d)
    u /= np.linalg.norm(u)
    X = (u[None, :] + 0.045 * rng.standard_normal((n, d)) / np.sqrt(d)).astype(np.float32)   # pairwise ||x - y||^2 ~ 0.004
    R = orc.random_rotation(d, 6)
    idx = orc.sample_rows(3, n, k)
    got = skm.fit(cuda(X), k, 1, 3, skm.FitOptions(R=cuda(R), final_assign=False, screen=1))
    assert got.trace[0]["screen_dims"] == 0 and got.trace[0]["gather_pairs"] == 0      # the fallback's counters
    Xr = orc.rotate(X, R)
    a_ref, d_ref = orc.assign_full(Xr, Xr[idx])
    a = got.assign.cpu().numpy()
    check_assignment(a, a_ref, Xr, Xr[idx], min_agree=0.995)
    same = a == a_ref
    assert np.abs(got.dist.cpu().numpy()[same] - d_ref[same]).max() < 2e-5 * max(1.0, d_ref.max())
    # half as many centroids fit the list: the filtered path then runs to the end and agrees as well
    k2 = 100
    got2 = skm.fit(cuda(X), k2, 1, 3, skm.FitOptions(R=cuda(R), final_assign=False, screen=1))
    assert got2.trace[0]["screen_dims"] > 0 and got2.trace[0]["gather_pairs"] > 50 * n
    idx2 = orc.sample_rows(3, n, k2)
    a2_ref, _ = orc.assign_full(Xr, Xr[idx2])
    check_assignment(got2.assign.cpu().numpy(), a2_ref, Xr, Xr[idx2], min_agree=0.995)


def test_lent_workspace_changes_nothing_and_a_small_one_is_refused(skm, dg):
    """A fit in a workspace lent by the caller (whatever bytes it holds) gives the bits of a fit that allocates its
    own; a workspace below skm_workspace_bytes is refused with the out-of-memory code before anything runs."""
    X = cuda(dg.mixture(20_000, 128, 60, 3, "linear").numpy())
    k, iters = 300, 6
    own = skm.fit(X, k, iters, 5, skm.FitOptions(own_workspace=True))
    need = skm.workspace_bytes(20_000, 128, k)
    ws = torch.randint(0, 256, (need,), dtype=torch.uint8, device="cuda")     # garbage: nothing may be assumed zero
    lent = skm.fit(X, k, iters, 5, skm.FitOptions(workspace=ws))
    assert torch.equal(own.assign, lent.assign) and torch.equal(own.centroids, lent.centroids)
    assert torch.equal(own.dist, lent.dist)
    assert [t["survivors"] for t in own.trace] == [t["survivors"] for t in lent.trace]
    again = skm.fit(X, k, iters, 5, skm.FitOptions(workspace=ws))             # and on what the last call left behind
    assert torch.equal(own.assign, again.assign) and torch.equal(own.centroids, again.centroids)
    with pytest.raises(skm.SkmError, match="memory"):
        skm.fit(X, k, iters, 5, skm.FitOptions(workspace=ws[: need // 2]))
    # the step call takes a workspace of its own size the same way
    prev = own.assign
    a0, d0, _ = skm.assign(X, own.centroids, prev, 0, skm.FitOptions(own_workspace=True))
    a1, d1, _ = skm.assign(X, own.centroids, prev, 0, skm.FitOptions(workspace=ws))
    assert torch.equal(a0, a1) and torch.equal(d0, d1)
    # the sampled fit: one workspace for the fit on the sample and the assignment of all rows
    so = skm.fit(X, 64, 5, 5, skm.FitOptions(sample_frac=0.25, own_workspace=True))
    p = skm._params(skm.FitOptions(sample_frac=0.25), [], None)
    need_s = skm.workspace_bytes(20_000, 128, 64, p)
    wss = torch.randint(0, 256, (need_s,), dtype=torch.uint8, device="cuda")
    sl = skm.fit(X, 64, 5, 5, skm.FitOptions(sample_frac=0.25, workspace=wss))
    assert torch.equal(so.assign, sl.assign) and torch.equal(so.centroids, sl.centroids)
    with pytest.raises(skm.SkmError, match="memory"):
        skm.fit(X, 64, 5, 5, skm.FitOptions(sample_frac=0.25, workspace=wss[: need_s // 3]))
    # the hierarchical fit: every fine fit's share comes out of the workspace; with room for fewer than eight shares
    # fewer fits run side by side, with the same result; without room for one the call is refused
    ho, sizes_o, counts_o = skm.fit_hierarchical(X, 64, 13, 3, 5, skm.FitOptions(own_workspace=True))
    need_h = skm.hier_workspace_bytes(20_000, 128, 64)
    wsh = torch.randint(0, 256, (need_h,), dtype=torch.uint8, device="cuda")
    hl, sizes_l, counts_l = skm.fit_hierarchical(X, 64, 13, 3, 5, skm.FitOptions(workspace=wsh))
    assert sizes_o == sizes_l and counts_o == counts_l
    assert torch.equal(ho.assign, hl.assign) and torch.equal(ho.centroids, hl.centroids)
    with pytest.raises(skm.SkmError, match="memory"):
        skm.fit_hierarchical(X, 64, 13, 3, 5, skm.FitOptions(workspace=wsh[: need_h // 4]))


def test_fit_with_the_library_rotation_matches_the_oracle_run_with_that_matrix(skm, orc, dg):
    """A fit that makes its rotation matrix itself (from the seed, on the device) must match the oracle run with the
    very matrix skm_make_rotation returns for that seed, and a fit that is handed that matrix, at every step."""
    n, d, k, iters, seed = 70_000, 256, 50, 5, 11
    X = dg.mixture(n, d, 40, 8, "linear").numpy()
    R = skm.make_rotation(d, seed)
    ref = orc.fit(X, k, iters, seed, orc.FitParams(eps0=EPS0), R=R.cpu().numpy())
    got = skm.fit(cuda(X), k, iters, seed, skm.FitOptions(eps0=EPS0))                 # R from the seed, inside the fit
    given = skm.fit(cuda(X), k, iters, seed, skm.FitOptions(eps0=EPS0, R=R))
    assert got.timing["ms_rotate"] > 0
    Xr = orc.rotate(X, R.cpu().numpy())
    for fr in (got, given):
        a = fr.assign.cpu().numpy()
        Yg = fr.centroids.cpu().numpy()
        check_assignment(a, ref.assign, Xr, ref.centroids_rot, own=(X, Yg), max_far=20)
        check_centroids(Yg, ref.centroids, a, ref.assign)
        for g, r in zip(fr.trace, ref.trace):
            assert g["objective"] == pytest.approx(r["objective"], rel=1e-4) and g["dprime"] == r["dprime"]
    assert (got.assign != given.assign).sum().item() <= 20
    assert got.trace[0]["objective"] == pytest.approx(given.trace[0]["objective"], rel=1e-6)
    # and the labels of iteration 1 alone (a fit of one iteration without the final pass returns them)
    one = skm.fit(cuda(X), k, 1, seed, skm.FitOptions(eps0=EPS0, final_assign=False))
    ref1 = orc.fit(X, k, 1, seed, orc.FitParams(eps0=EPS0, final_assign=False), R=R.cpu().numpy())
    check_assignment(one.assign.cpu().numpy(), ref1.assign, Xr, Xr[orc.sample_rows(seed, n, k)])
    assert rel_l2(one.centroids.cpu().numpy(), ref1.centroids) < 1e-5


def test_fit_is_bitwise_reproducible(skm, orc, dg):
    X = cuda(dg.mixture(30_000, 128, 64, 12, "linear").numpy())
    R = cuda(orc.random_rotation(128, 2))
    a = skm.fit(X, 200, 5, 9, skm.FitOptions(R=R))
    b = skm.fit(X, 200, 5, 9, skm.FitOptions(R=R))
    assert torch.equal(a.assign, b.assign) and torch.equal(a.centroids, b.centroids) and torch.equal(a.dist, b.dist)
    assert [r["survivors"] for r in a.trace] == [r["survivors"] for r in b.trace]


# ------------------------------------------------------------------ ETR
def test_etr_ground_truth_recall_and_stop(skm, orc, dg):
    n, d, k, nq, K = 20_000, 64, 50, 40, 10
    X = dg.mixture(n, d, 30, 3, "linear").numpy()
    Q = dg.mixture(nq, d, 30, 4, "linear").numpy()
    R = orc.random_rotation(d, 6)
    idx = orc.sample_rows(2, n, k)
    kw = dict(etr=True, topk=K, probe_frac=0.1, adjust_dprime=False)
    for tol, want_stop in ((0.5, True), (-1.0, False)):
        ref = orc.fit(X, k, 6, 2, orc.FitParams(eps0=EPS0, etr_tol=tol, **kw), R=R, init_idx=idx, queries=Q)
        got = skm.fit(cuda(X), k, 6, 2, skm.FitOptions(R=cuda(R), queries=cuda(Q), etr_tol=tol, **kw))
        assert got.iters_run == ref.iters_run and (got.iters_run == 3) == want_stop
        for g, r in zip(got.trace[: got.iters_run], ref.trace):
            assert g["recall"] == pytest.approx(r["recall"], abs=2.0 / (nq * K))
    # user-supplied ground truth gives the same recalls as the computed one
    gt = orc.ground_truth(X, Q, K)
    got2 = skm.fit(cuda(X), k, 6, 2, skm.FitOptions(R=cuda(R), queries=cuda(Q), gt=cuda(gt), etr_tol=-1.0, **kw))
    assert [g["recall"] for g in got2.trace[:6]] == [g["recall"] for g in got.trace[:6]]
    # queries sampled from X by the library: every query finds itself, recall stays high
    got3 = skm.fit(cuda(X), k, 3, 2, skm.FitOptions(R=cuda(R), etr=True, nq=25, topk=1, probe_frac=0.02,
                                                    etr_tol=-1.0, adjust_dprime=False))
    assert all(g["recall"] >= 0.9 for g in got3.trace[:3])


def check_ground_truth(gt, ref, X, Q, tol=2e-6):
    """Index by index; where the two lists differ, the fp64 distances of the two points named at that rank must tie to
    the rounding of an fp32 score (the library orders by ||x||^2 - 2 q.x computed in fp32)."""
    gt = np.asarray(gt)
    ref = np.asarray(ref)
    assert gt.shape == ref.shape and gt.min() >= 0 and gt.max() < len(X)
    assert all(len(set(r.tolist())) == len(r) for r in gt)          # no point twice in a list
    qs, ranks = np.nonzero(gt != ref)
    say(f"ground truth: {gt.size} entries, {len(qs)} differ")
    assert len(qs) <= 0.01 * gt.size
    for q, r in zip(qs, ranks):
        dq = Q[q].astype(np.float64)
        a = ((dq - X[gt[q, r]].astype(np.float64)) ** 2).sum()
        b = ((dq - X[ref[q, r]].astype(np.float64)) ** 2).sum()
        scale = (dq ** 2).sum() + (X[ref[q, r]].astype(np.float64) ** 2).sum()
        assert abs(a - b) <= tol * scale, (q, r, a, b)


def test_etr_ground_truth_merges_score_chunks(skm, orc, dg):
    """The ground truth is selected from scores computed 65 536 points at a time.  150 000 points are three chunks
    (the last one ragged): the running lists are full after the first, so the later chunks go through the filtered
    merge (only columns below the list's largest key are candidates)."""
    n, d, nq, K = 150_000, 64, 64, 10
    X = dg.mixture(n, d, 30, 3, "linear").numpy()
    Q = dg.mixture(nq, d, 30, 3, "linear", sample_seed=99).numpy()
    gt = skm.etr_ground_truth(cuda(X), cuda(Q), K).cpu().numpy()
    check_ground_truth(gt, orc.ground_truth(X, Q, K), X, Q)
    # K = 1 and K larger than a wavefront
    for K2 in (1, 100):
        gt2 = skm.etr_ground_truth(cuda(X[:70_000]), cuda(Q[:8]), K2).cpu().numpy()
        check_ground_truth(gt2, orc.ground_truth(X[:70_000], Q[:8], K2), X, Q[:8])


def test_etr_ground_truth_when_a_chunk_floods_the_candidate_buffer(skm, orc):
    """The filtered merge keeps at most 4096 candidate columns; a chunk with more columns below the running list's
    largest key must fall back to selecting over the whole chunk.  First chunk: far points; second chunk: 60 000 points
    all nearer to every query than anything before."""
    rng = np.random.default_rng(5)
    d, nq, K = 32, 16, 10
    far = (rng.standard_normal((65_536, d)) * 0.1 + 3.0).astype(np.float32)
    near = (rng.standard_normal((60_000, d)) * 0.1).astype(np.float32)
    X = np.concatenate([far, near])
    Q = (rng.standard_normal((nq, d)) * 0.1).astype(np.float32)
    gt = skm.etr_ground_truth(cuda(X), cuda(Q), K).cpu().numpy()
    assert gt.min() >= 65_536                                   # every neighbour comes from the second chunk
    check_ground_truth(gt, orc.ground_truth(X, Q, K), X, Q)
    # fewer points than K: the lists end with -1
    gt3 = skm.etr_ground_truth(cuda(X[:4]), cuda(Q[:2]), K).cpu().numpy()
    assert (gt3[:, 4:] == -1).all() and (np.sort(gt3[:, :4], axis=1) == np.arange(4)).all()


def test_c3_full_size_etr(skm, orc, dg):
    """Workload C3 (1 000 000 x 768, k = 4096, 1000 held-out queries, top-10, 41 probed centroids) as the fit runs it:
    the ground truth over 16 score chunks against the oracle (a sample of the queries, index by index), and the recall
    of every step against the oracle's recall formula on all 1000 queries."""
    torch.cuda.empty_cache()
    n, d, k, nq, K = 1_000_000, 768, 4096, 1000, 10
    say("generating C3")
    X = dg.config_data("C3", device="cuda")
    Q = dg.config_queries("C3", device="cuda")
    Rn = orc.random_rotation(d, 42)
    R = cuda(Rn)
    say("ground truth")
    gt = skm.etr_ground_truth(X, Q, K)
    rng = np.random.default_rng(2)
    qs = np.sort(rng.choice(nq, 96, replace=False))
    Xn = X.cpu().numpy()
    Qn = Q.cpu().numpy()
    say("oracle ground truth of 96 queries")
    check_ground_truth(gt.cpu().numpy()[qs], orc.ground_truth(Xn, Qn[qs], K), Xn, Qn[qs])
    nprobe = orc.nprobe(k, 0.01)
    assert nprobe == 41
    Qr = orc.rotate(Qn, Rn)
    say("fits")
    base = dict(R=R, etr=True, queries=Q, adjust_dprime=True)
    full = skm.fit(X, k, 10, 42, skm.FitOptions(**base))                      # the library computes the ground truth
    given = skm.fit(X, k, 10, 42, skm.FitOptions(gt=gt, **base))              # ... or is handed it
    assert [r["recall"] for r in full.trace] == [r["recall"] for r in given.trace]
    assert 2 <= full.iters_run <= 10 and len(full.trace) == full.iters_run + 1
    gtn = gt.cpu().numpy()
    for t in range(1, full.iters_run + 1):
        # recall of step t: centroids Y_(t-1) (a fit of t - 1 iterations returns them; t = 1: the initial rows) and the
        # labels a_t (a fit of t iterations without the final pass returns them); fits are reproducible bit by bit
        if t == 1:
            Yprev = Xn[orc.sample_rows(42, n, k)]
        else:
            Yprev = skm.fit(X, k, t - 1, 42, skm.FitOptions(etr_tol=-1.0, final_assign=False, **base)).centroids.cpu().numpy()
        a_t = skm.fit(X, k, t, 42, skm.FitOptions(etr_tol=-1.0, final_assign=False, **base)).assign.cpu().numpy()
        want = orc.recall(Qr, orc.rotate(Yprev, Rn), nprobe, gtn, a_t)
        say(f"C3 step {t}: recall {full.trace[t - 1]['recall']:.5f} oracle {want:.5f}")
        assert full.trace[t - 1]["recall"] == pytest.approx(want, abs=3.0 / (nq * K))
    # the stop rule on the recalls it saw
    rec = [r["recall"] for r in full.trace[: full.iters_run]]
    best, streak, stop_at = rec[0], 0, None
    for t in range(2, len(rec) + 1):
        streak = streak + 1 if rec[t - 1] - best <= 0.005 else 0
        best = max(best, rec[t - 1])
        if streak >= 2:
            stop_at = t
            break
    if full.iters_run < 10:
        assert stop_at == full.iters_run
    else:
        assert stop_at in (None, 10)
    del X, Q, full, given
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ full size, bench launch configuration
def check_counters_on_rows(skm, ref, Xs, Y, prev_s, dp, R):
    """The same pruned step on the sampled rows alone, with per-block statistics: every counter within 0.1 % of the
    oracle's for those rows (the full-size run can only be compared in density: it counts over other points)."""
    a, dist, row = skm.assign(Xs, Y, prev_s, dp, skm.FitOptions(R=R, block_stats=True))
    ns, k = Xs.shape[0], Y.shape[0]
    surv_ref = ns * (k - 1) - ref.pruned_first
    assert abs(row["survivors"] - surv_ref) <= max(2, 1e-3 * surv_ref), (row["survivors"], surv_ref)
    for m in range(min(row["nblocks"], 32)):
        assert abs(row["enter"][m] - ref.enter[m]) <= max(2, 1e-3 * ref.enter[m]), (m, row["enter"][m], ref.enter[m])
    assert abs(row["completed"] - ref.enter[-1]) <= max(2, 1e-3 * ref.enter[-1])
    assert (a.cpu().numpy() != ref.assign).sum() <= max(1, 1e-3 * ns)
    return row


def test_c2_full_size_sampled_parity(skm, orc, dg):
    """Workload C2 (1 000 000 x 1536, k = 1024) exactly as bench.py runs it; the oracle checks
    a sample of the rows one by one (pruned step and exact step) and a sample of the clusters."""
    torch.cuda.empty_cache()
    n, d, k = 1_000_000, 1536, 1024
    say("generating C2")
    X = dg.config_data("C2", device="cuda")
    Rn = orc.random_rotation(d, 42)
    R = cuda(Rn)
    say("fit 2 iterations")
    fr = skm.fit(X, k, 2, 42, skm.FitOptions(R=R, final_assign=False, adjust_dprime=False))
    assert fr.trace[1]["survivors"] > 0
    say("assign step")
    a3, d3, row = skm.assign(X, fr.centroids, fr.assign, 0, skm.FitOptions(R=R))
    rng = np.random.default_rng(0)
    rows = np.sort(rng.choice(n, 1536, replace=False))
    Xs = X[torch.from_numpy(rows).cuda()].cpu().numpy()
    Y = fr.centroids.cpu().numpy()
    Xr = orc.rotate(Xs, Rn)
    Yr = orc.rotate(Y, Rn)
    say("oracle on the sample")
    ref = orc.assign_pruned(Xr, Yr, fr.assign.cpu().numpy()[rows], orc.dprime_init(d), EPS0, 0)
    check_assignment(a3.cpu().numpy()[rows], ref.assign, Xr, Yr, min_agree=0.998)
    same = a3.cpu().numpy()[rows] == ref.assign
    assert np.abs(d3.cpu().numpy()[rows][same] - ref.dist[same]).max() < 1e-5
    surv_ref = len(rows) * (k - 1) - ref.pruned_first
    assert row["survivors"] / n == pytest.approx(surv_ref / len(rows), rel=0.1)     # same survivor density (sampling error)
    ridx = torch.from_numpy(rows).cuda()
    check_counters_on_rows(skm, ref, X[ridx].contiguous(), fr.centroids, fr.assign[ridx].contiguous(), orc.dprime_init(d), R)
    say("exact step on the sample")
    ae, de = skm.assign_exact(X, fr.centroids)
    ao, do = orc.assign_full(Xs.astype(np.float64), Y.astype(np.float64))
    check_assignment(ae.cpu().numpy()[rows], ao, Xs, Y, min_agree=0.998)
    say("update on sampled clusters")
    Yn = fr.centroids.clone()
    cnt = skm.update(X, a3, Yn).cpu().numpy()
    assert cnt.sum() == n and (cnt == np.bincount(a3.cpu().numpy(), minlength=k)).all()
    for c in rng.choice(k, 6, replace=False):
        members = torch.nonzero(a3 == int(c)).flatten()
        if len(members) == 0:
            continue
        mean = X[members].cpu().numpy().astype(np.float64).mean(0)
        assert np.abs(Yn[int(c)].cpu().numpy() - mean).max() < 1e-6
    del X, fr
    torch.cuda.empty_cache()


def test_c2_full_fit_as_benchmarked_keeps_labels_with_their_points(skm, orc, dg):
    """The whole C2 fit as bench.py times it (10 iterations + final pass, points regrouped by cluster from the third
    step on).  On sampled rows the returned label must be the nearest of the returned centroids (up to near-ties and
    the pruning's rare losses), the returned distance the direct one, and the distances must add up to the objective
    of the final pass: a label or a distance that came back at the wrong row would break all three."""
    torch.cuda.empty_cache()
    n, d, k = 1_000_000, 1536, 1024
    X = dg.config_data("C2", device="cuda")
    Rn = orc.random_rotation(d, 42)
    say("full C2 fit")
    fr = skm.fit(X, k, 10, 42, skm.FitOptions(R=cuda(Rn)))
    assert fr.iters_run == 10 and len(fr.trace) == 11
    a = fr.assign.cpu().numpy()
    dist = fr.dist.cpu().numpy()
    assert np.bincount(a, minlength=k).sum() == n and a.min() >= 0 and a.max() < k
    assert float(dist.astype(np.float64).sum()) == pytest.approx(fr.trace[-1]["objective"], rel=1e-5)
    rng = np.random.default_rng(5)
    rows = np.sort(rng.choice(n, 1536, replace=False))
    Xs = X[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    Y = fr.centroids.cpu().numpy().astype(np.float64)
    ao, do = orc.assign_full(Xs, Y)
    check_assignment(a[rows], ao, Xs, Y, min_agree=0.998)
    direct = ((Xs - Y[a[rows]]) ** 2).sum(1)
    assert np.abs(dist[rows] - direct).max() < 1e-5
    obj = [t["objective"] for t in fr.trace]
    assert all(b <= x * (1 + 1e-6) for x, b in zip(obj, obj[1:]))
    del X, fr
    torch.cuda.empty_cache()


def test_c4_full_size_sampled_parity(skm, orc, dg):
    """Workload C4 (1 000 000 x 1536, k = 16 384): the large-k regime, where a step is a million tiles of one to
    three slabs.  Pruned steps at d' = 192 and at d' = 64 (what the d' rule reaches on this workload), checked by
    the oracle on a sample of the rows one by one."""
    torch.cuda.empty_cache()
    n, d, k = 1_000_000, 1536, 16_384
    say("generating C4")
    X = dg.config_data("C4", device="cuda")
    Rn = orc.random_rotation(d, 42)
    R = cuda(Rn)
    say("fit 3 iterations")
    fr = skm.fit(X, k, 3, 42, skm.FitOptions(R=R, final_assign=False, adjust_dprime=False))
    rng = np.random.default_rng(1)
    rows = np.sort(rng.choice(n, 3072, replace=False))
    Xr = orc.rotate(X[torch.from_numpy(rows).cuda()].cpu().numpy(), Rn)
    say("rotating the centroids on the host")
    Yr = orc.rotate(fr.centroids.cpu().numpy(), Rn)
    prev = fr.assign.cpu().numpy()[rows]
    for dp in (192, 64):
        say("assign step at d' =", dp)
        a, dist, row = skm.assign(X, fr.centroids, fr.assign, dp, skm.FitOptions(R=R))
        ref = orc.assign_pruned(Xr, Yr, prev, dp, EPS0, 0)
        check_assignment(a.cpu().numpy()[rows], ref.assign, Xr, Yr, min_agree=0.995)
        same = a.cpu().numpy()[rows] == ref.assign
        assert np.abs(dist.cpu().numpy()[rows][same] - ref.dist[same]).max() < 1e-5
        surv_ref = len(rows) * (k - 1) - ref.pruned_first
        assert row["survivors"] / n == pytest.approx(surv_ref / len(rows), rel=0.2)    # same survivor density (a heavy-tailed count per point)
        assert row["dprime"] == dp
        ridx = torch.from_numpy(rows).cuda()
        check_counters_on_rows(skm, ref, X[ridx].contiguous(), fr.centroids, fr.assign[ridx].contiguous(), dp, R)
    del X, fr
    torch.cuda.empty_cache()


def test_c5_full_size_sampled_parity(skm, orc, dg):
    """Workload C5 (10 000 000 x 384, k = 32 768): the large-N regime.  Three iterations as the fit runs them (at the
    default pair budget the rows of a pruned step go through the tile kernel in eight chunks), then pruned steps at
    d' = 48 (the initial value: the last trailing block holds 16 dimensions) and d' = 64, checked by the oracle on a
    sample of the rows one by one."""
    torch.cuda.empty_cache()
    n, d, k = 10_000_000, 384, 32_768
    say("generating C5")
    X = dg.config_data("C5", device="cuda")
    Rn = orc.random_rotation(d, 42)
    R = cuda(Rn)
    say("fit 3 iterations")
    fr = skm.fit(X, k, 3, 42, skm.FitOptions(R=R, final_assign=False, adjust_dprime=False))
    assert fr.trace[1]["dprime"] == 48 and fr.trace[1]["nblocks"] == 6
    cnt = torch.bincount(fr.assign.long(), minlength=k)
    assert int(cnt.sum()) == n
    rng = np.random.default_rng(4)
    rows = np.sort(rng.choice(n, 3072, replace=False))
    ridx = torch.from_numpy(rows).cuda()
    Xs = X[ridx].contiguous()
    Xr = orc.rotate(Xs.cpu().numpy(), Rn)
    Yr = orc.rotate(fr.centroids.cpu().numpy(), Rn)
    prev = fr.assign.cpu().numpy()[rows]
    for dp in (48, 64):
        say("assign step at d' =", dp)
        a, dist, row = skm.assign(X, fr.centroids, fr.assign, dp, skm.FitOptions(R=R))
        ref = orc.assign_pruned(Xr, Yr, prev, dp, EPS0, 0)
        check_assignment(a.cpu().numpy()[rows], ref.assign, Xr, Yr, min_agree=0.995)
        same = a.cpu().numpy()[rows] == ref.assign
        assert np.abs(dist.cpu().numpy()[rows][same] - ref.dist[same]).max() < 1e-5
        surv_ref = len(rows) * (k - 1) - ref.pruned_first
        # survivors per point are heavy-tailed here (a few points with a poor incumbent keep thousands of pairs), so
        # 3072 rows estimate the density of ten million only roughly; the exact comparison is on the rows themselves
        assert 0.5 < (row["survivors"] / n) / (surv_ref / len(rows)) < 2.0
        assert row["dprime"] == dp and row["changed"] == int((a != fr.assign).sum())
        check_counters_on_rows(skm, ref, Xs, fr.centroids, fr.assign[ridx].contiguous(), dp, R)
    say("update on sampled clusters")
    Yn = fr.centroids.clone()
    cnt2 = skm.update(X, a, Yn).cpu().numpy()
    assert cnt2.sum() == n
    for c in rng.choice(k, 6, replace=False):
        members = torch.nonzero(a == int(c)).flatten()
        if len(members):
            mean = X[members].cpu().numpy().astype(np.float64).mean(0)
            assert np.abs(Yn[int(c)].cpu().numpy() - mean).max() < 1e-6
    del X, fr
    torch.cuda.empty_cache()


def test_tall_problems_are_cut_into_bands_of_row_tiles(skm, orc, dg):
    """A launch holds at most 2^24 - 1 tiles; with the limit lowered (skm_debug_gemm_config) the banding of the GEMM
    launches runs on a small input."""
    X = dg.mixture(3000, 64, 20, 2, "linear").numpy()
    Y = X[:300].copy()
    R = orc.random_rotation(64, 1)
    skm.debug_gemm_config(max_tiles=7)   # 3 column tiles -> bands of 2 row tiles
    try:
        a, dist = skm.assign_exact(cuda(X), cuda(Y))
        out = skm.rotate(cuda(X), cuda(R)).cpu().numpy()
    finally:
        skm.debug_gemm_config()
    ao, do = orc.assign_full(X.astype(np.float64), Y.astype(np.float64))
    assert (a.cpu().numpy() == ao).mean() > 0.999
    assert np.abs(out - orc.rotate(X, R)).max() < 2e-6


@pytest.mark.parametrize("max_tiles", [0, 5])
def test_wide_tile_gemm_on_small_ragged_inputs(skm, orc, dg, max_tiles):
    """Tall products run on 256 x 256 tiles with the second operand split ahead.  The form is forced
    (skm_debug_gemm_config), so that ragged row and column tiles, several slabs and (with the tile limit lowered) the
    banding run on inputs the oracle finishes in seconds: exact assignment, rotation, a whole fit."""
    skm.debug_gemm_config(tile256=1, max_tiles=max_tiles)
    try:
        for (n, d, k) in ((3000, 64, 300), (1001, 96, 257), (700, 160, 5)):
            X = dg.mixture(n, d, 20, 2, "linear").numpy()
            Y = X[:k].copy() + np.float32(0.01)
            a, dist = skm.assign_exact(cuda(X), cuda(Y))
            ao, do = orc.assign_full(X.astype(np.float64), Y.astype(np.float64))
            same = a.cpu().numpy() == ao
            assert same.mean() > 0.999, (n, d, k, same.mean())
            assert np.abs(dist.cpu().numpy()[same] - do[same]).max() < 1e-5 * max(1.0, do.max())
            R = orc.random_rotation(d, 1)
            out = skm.rotate(cuda(X), cuda(R)).cpu().numpy()
            assert np.abs(out - orc.rotate(X, R)).max() < 2e-6 * max(1.0, np.abs(X).max())
        X = dg.mixture(4000, 128, 40, 11, "linear").numpy()   # a ragged last row tile
        R = orc.random_rotation(128, 7)
        idx = orc.sample_rows(7, 4000, 32)
        ref = orc.fit(X, 32, 4, 7, orc.FitParams(eps0=EPS0, adjust_dprime=False), R=R, init_idx=idx)
        got = skm.fit(cuda(X), 32, 4, 7, skm.FitOptions(R=cuda(R), adjust_dprime=False))
    finally:
        skm.debug_gemm_config()
    assert (got.assign.cpu().numpy() == ref.assign).mean() >= 0.999
    assert rel_l2(got.centroids.cpu().numpy(), ref.centroids) < 1e-3
    assert got.trace[-1]["objective"] == pytest.approx(ref.trace[-1]["objective"], rel=1e-4)


# ------------------------------------------------------------------ edge and degenerate cases
def test_single_cluster_and_one_point_per_cluster(skm, orc, dg):
    X = dg.mixture(700, 48, 5, 3, "linear").numpy()
    R = orc.random_rotation(48, 1)
    # k = 1: no challenger exists, nothing survives, the centroid is the global mean
    got = skm.fit(cuda(X), 1, 3, 5, skm.FitOptions(R=cuda(R)))
    assert (got.assign.cpu().numpy() == 0).all()
    assert np.abs(got.centroids.cpu().numpy()[0] - X.astype(np.float64).mean(0)).max() < 1e-6
    assert all(t["survivors"] == 0 and t["prune_frac"] == 0.0 for t in got.trace)
    # k = n: every point is its own centroid after iteration 1, all distances 0, nothing moves afterwards
    Xs = X[:130]
    got = skm.fit(cuda(Xs), 130, 3, 5, skm.FitOptions(R=cuda(R)))
    a = got.assign.cpu().numpy()
    assert sorted(a.tolist()) == list(range(130))
    assert rel_l2(got.centroids.cpu().numpy()[a], Xs) < 1e-6
    assert got.trace[-1]["objective"] < 1e-9 and got.trace[-1]["changed"] == 0


def test_smallest_shapes(skm, orc):
    rng = np.random.default_rng(0)
    X = rng.standard_normal((5, 16)).astype(np.float32)      # d = 16 is the smallest d, d' = d
    ref = orc.fit(X, 2, 3, 1, orc.FitParams(eps0=EPS0), R=None)
    got = skm.fit(cuda(X), 2, 3, 1, skm.FitOptions(rotate=False))
    assert (got.assign.cpu().numpy() == ref.assign).all()
    assert rel_l2(got.centroids.cpu().numpy(), ref.centroids) < 1e-5
    one = skm.fit(cuda(X[:1]), 1, 1, 1, skm.FitOptions(rotate=False))   # a single point
    assert one.assign.cpu().numpy().tolist() == [0] and np.allclose(one.centroids.cpu().numpy()[0], X[0])


def test_duplicate_points_tie_to_the_lowest_index(skm):
    X = np.zeros((300, 32), dtype=np.float32)
    X[:, 0] = 1.0
    X[150:, 1] = 1.0                                        # two distinct rows, 150 copies each
    Y = np.stack([X[0], X[0], X[200], X[200]])              # each row twice among the centroids
    a, dist = skm.assign_exact(cuda(X), cuda(Y))
    a = a.cpu().numpy()
    assert (a[:150] == 0).all() and (a[150:] == 2).all() and float(dist.abs().max()) < 1e-6
    # the pruned step keeps the incumbent on exact ties
    prev = np.where(np.arange(300) < 150, 1, 3).astype(np.int32)
    a2, _, _ = skm.assign(cuda(X), cuda(Y), cuda(prev), 16, skm.FitOptions(rotate=False))
    assert (a2.cpu().numpy() == prev).all()


def test_largest_dimension_and_many_blocks(skm, orc, dg):
    """d = 4096: 60 trailing blocks, more than the per-block counters of the trace hold."""
    X = dg.mixture(600, 4096, 10, 5, "embed").numpy()
    R = orc.random_rotation(4096, 2)
    Y = X[:40] + 0.01
    Xr, Yr = orc.rotate(X, R), orc.rotate(Y, R)
    prev = orc.assign_full(Xr, Yr)[0].astype(np.int32)
    prev[::3] = 7
    ref = orc.assign_pruned(Xr, Yr, prev, 512, EPS0, 0)
    for dense in (0.02, 1.0):
        a, dist, row = skm.assign(cuda(X), cuda(Y), cuda(prev), 512, skm.FitOptions(R=cuda(R), block_stats=True,
                                                                                     dense_frac=dense))
        check_assignment(a.cpu().numpy(), ref.assign, Xr, Yr)
        assert row["nblocks"] == 56 and row["enter"][0] == ref.enter[0]


# ------------------------------------------------------------------ sampled fit (Section 4.4)
@pytest.mark.parametrize("n,d,k,frac", [(20_000, 128, 64, 0.25), (6000, 100, 30, 0.5)])
def test_sampled_fit(skm, orc, dg, n, d, k, frac):
    X = dg.mixture(n, d, 80, 17, "linear").numpy()
    R = orc.random_rotation(d, 17)
    ref, idx = orc.fit_sampled(X, k, 6, 9, frac, orc.FitParams(eps0=EPS0), R=R)
    got = skm.fit(cuda(X), k, 6, 9, skm.FitOptions(R=cuda(R), sample_frac=frac))
    assert got.iters_run == 6 and len(got.trace) == 7
    assert [g["dprime"] for g in got.trace] == [r["dprime"] for r in ref.trace]
    assert rel_l2(got.centroids.cpu().numpy(), ref.centroids) < 1e-3
    check_assignment(got.assign.cpu().numpy(), ref.assign, orc.rotate(X, R), ref.centroids_rot,
                     own=(X, got.centroids.cpu().numpy()))
    assert got.trace[-1]["objective"] == pytest.approx(ref.trace[-1]["objective"], rel=1e-4)
    assert got.trace[0]["changed"] == len(idx)          # the loop ran on the sample only
    with pytest.raises(skm.SkmError):
        skm.fit(cuda(X), k, 2, 9, skm.FitOptions(R=cuda(R), sample_frac=frac, final_assign=False))


@pytest.mark.parametrize("n,d,k", [(20_000, 128, 64), (9000, 100, 30)])
def test_hierarchical_fit(skm, orc, dg, n, d, k):
    """Section 6: meso phase, shares of k, fine phase per meso-cluster, final assignment, against the oracle's
    composition of the same steps."""
    X = dg.mixture(n, d, 80, 21, "linear").numpy()
    R = orc.random_rotation(d, 21)
    ref = orc.fit_hierarchical(X, k, 13, 3, 5, orc.FitParams(eps0=EPS0), R=R)
    got, sizes, counts = skm.fit_hierarchical(cuda(X), k, 13, 3, 5, skm.FitOptions(R=cuda(R), eps0=EPS0))
    assert sizes == ref["meso_sizes"].tolist() and counts == ref["fine_counts"].tolist() and sum(counts) == k
    assert len(got.trace) == 3 + 2 and got.iters_run == 3
    for g, r in zip(got.trace[:4], ref["meso"].trace):
        assert g["objective"] == pytest.approx(r["objective"], rel=1e-4) and g["dprime"] == r["dprime"]
    a = got.assign.cpu().numpy()
    Y = got.centroids.cpu().numpy()
    check_assignment(a, ref["assign"], orc.rotate(X, R), ref["centroids_rot"], own=(X, Y))
    check_centroids(Y, ref["centroids"], a, ref["assign"])
    assert got.trace[-1]["objective"] == pytest.approx(ref["objective"], rel=1e-4)
    assert float(got.dist.sum()) == pytest.approx(ref["objective"], rel=1e-4)
    with pytest.raises(skm.SkmError):
        skm.fit_hierarchical(cuda(X), k, 13, 3, 5, skm.FitOptions(R=cuda(R), sample_frac=0.5))


@pytest.mark.parametrize("d,dp", [(144, 16), (208, 16), (272, 80)])
def test_pruned_step_counters_when_workgroups_take_many_tiles(skm, orc, dg, d, dp):
    """More row tiles than resident workgroups, so the persistent kernel walks several tiles per workgroup; the
    step counters (survivors, completed pairs, pairs entering each block) must still match the oracle exactly.
    The shapes give an even and an odd number of trailing blocks (a tile can end at either kind of checkpoint)."""
    n, k = 90_000, 24
    X = dg.mixture(n, d, 40, 31, "linear").numpy()
    R = orc.random_rotation(d, 31)
    Xr = orc.rotate(X, R)
    Y0 = Xr[orc.sample_rows(31, n, k)]
    a0, _ = orc.assign_full(Xr, Y0)
    Yr, _ = orc.update(Xr, a0, Y0)
    ref = orc.assign_pruned(Xr, Yr, a0, dp, EPS0)
    for dense in (0.02, 1.0):
        a, dist, row = skm.assign(cuda(Xr.astype(np.float32)), cuda(Yr.astype(np.float32)), cuda(a0.astype(np.int32)), dp,
                                  skm.FitOptions(rotate=False, eps0=EPS0, dense_frac=dense, block_stats=True))
        check_assignment(a.cpu().numpy(), ref.assign, Xr, Yr)
        surv_ref = n * (k - 1) - ref.pruned_first
        assert abs(row["survivors"] - surv_ref) <= max(2, 1e-3 * surv_ref)
        assert row["nblocks"] == len(ref.enter) - 1
        for m in range(row["nblocks"]):
            assert abs(row["enter"][m] - ref.enter[m]) <= max(2, 1e-3 * ref.enter[m])
        assert abs(row["completed"] - ref.enter[-1]) <= max(2, 1e-3 * ref.enter[-1])


def test_angular_fit(skm, orc, dg):
    """Angular metric: unit points, centroids renormalised after every update; against the oracle's option."""
    rng = np.random.default_rng(3)
    X = dg.mixture(15_000, 100, 60, 23, "linear").numpy() * rng.uniform(0.2, 5.0, (15_000, 1)).astype(np.float32)
    R = orc.random_rotation(100, 23)
    ref, got = fit_pair(skm, orc, X, 40, 6, 3, R, angular=True)
    Xu = orc.rotate(X, R)
    Xu /= np.linalg.norm(Xu, axis=1, keepdims=True)
    Y = got.centroids.cpu().numpy()
    assert np.abs(np.linalg.norm(Y, axis=1) - 1.0).max() < 1e-5
    Xo = X.astype(np.float64) / np.linalg.norm(X.astype(np.float64), axis=1, keepdims=True)
    check_assignment(got.assign.cpu().numpy(), ref.assign, Xu, ref.centroids_rot, own=(Xo, Y))
    check_centroids(Y, ref.centroids, got.assign.cpu().numpy(), ref.assign)
    for g, r in zip(got.trace, ref.trace):
        assert g["objective"] == pytest.approx(r["objective"], rel=1e-4) and g["dprime"] == r["dprime"]
    with pytest.raises(skm.SkmError):
        skm.fit(cuda(X), 40, 3, 3, skm.FitOptions(R=cuda(R), angular=True, sample_frac=0.5))
    with pytest.raises(skm.SkmError):
        skm.assign(cuda(X), cuda(Y), None, 0, skm.FitOptions(R=cuda(R), angular=True))


def test_incremental_update_matches_the_full_one(skm, orc, dg):
    """Once few points change cluster, the centroid update corrects the cluster sums of the previous update by the
    rows that joined and left.  The result must be that of recomputing every sum from all points (fp64 sums, so
    equal up to the last bit of the fp32 mean), and it must still match the oracle."""
    X = dg.mixture(40_000, 96, 50, 41, "linear").numpy()
    R = orc.random_rotation(96, 41)
    k, iters = 64, 9
    a = skm.fit(cuda(X), k, iters, 4, skm.FitOptions(R=cuda(R), eps0=EPS0))
    b = skm.fit(cuda(X), k, iters, 4, skm.FitOptions(R=cuda(R), eps0=EPS0, full_update=True))
    assert a.timing["inc_updates"] >= 3 and b.timing["inc_updates"] == 0
    assert [r["changed"] for r in a.trace] == [r["changed"] for r in b.trace]
    assert torch.equal(a.assign, b.assign)
    assert rel_l2(a.centroids.cpu().numpy(), b.centroids.cpu().numpy()) < 1e-6
    ref = orc.fit(X, k, iters, 4, orc.FitParams(eps0=EPS0), R=R)
    check_assignment(a.assign.cpu().numpy(), ref.assign, orc.rotate(X, R), ref.centroids_rot,
                     own=(X, a.centroids.cpu().numpy()))
    check_centroids(a.centroids.cpu().numpy(), ref.centroids, a.assign.cpu().numpy(), ref.assign)
    # an empty cluster that is re-seeded by a split must be handled by both paths alike
    idx = orc.sample_rows(2, len(X), k)
    idx[1] = idx[0]
    c = skm.fit(cuda(X), k, iters, 4, skm.FitOptions(R=cuda(R), eps0=EPS0, init_idx=list(idx)))
    d = skm.fit(cuda(X), k, iters, 4, skm.FitOptions(R=cuda(R), eps0=EPS0, init_idx=list(idx), full_update=True))
    assert c.trace[0]["nempty"] == 1 and torch.equal(c.assign, d.assign)
    assert rel_l2(c.centroids.cpu().numpy(), d.centroids.cpu().numpy()) < 1e-6


# ------------------------------------------------------------------ points that stay in host memory
@pytest.mark.parametrize("pinned", [True, False])
@pytest.mark.parametrize("n,d,k,batch", [(20_000, 128, 64, 4096),      # 5 batches, ragged last one (3616 rows)
                                         (5000, 100, 24, 1536),        # padded dims, 4 batches, tail of 392 rows
                                         (3000, 64, 16, 0),            # one batch holds everything
                                         (300_000, 32, 8, 262_144)])   # a large batch, then a tail an eighth its size
def test_host_resident_fit(skm, orc, dg, n, d, k, batch, pinned):
    """Section 7.1: the points stay in host memory and pass through the device in batches, every iteration.
    The result must be Algorithm 1's, i.e. the oracle's, and that of the device-resident fit."""
    X = dg.mixture(n, d, 40, 17, "linear").numpy()
    R = orc.random_rotation(d, 17)
    iters = 6
    Xh = torch.from_numpy(X)
    if pinned:
        Xh = Xh.pin_memory()
    opts = skm.FitOptions(R=cuda(R), eps0=EPS0, adjust_dprime=False, block_stats=True)
    got = skm.fit_host(Xh, k, iters, 3, batch_rows=batch, opts=opts)
    ref = orc.fit(X, k, iters, 3, orc.FitParams(eps0=EPS0, adjust_dprime=False), R=R)
    a = got.assign.numpy()
    check_assignment(a, ref.assign, orc.rotate(X, R), ref.centroids_rot, own=(X, got.centroids.cpu().numpy()))
    check_centroids(got.centroids.cpu().numpy(), ref.centroids, a, ref.assign)
    assert len(got.trace) == len(ref.trace) == iters + 1
    for g, r in zip(got.trace, ref.trace):
        assert g["objective"] == pytest.approx(r["objective"], rel=1e-4)
        assert g["dprime"] == r["dprime"] and g["nempty"] == r["nempty"]
        assert g["prune_frac"] == pytest.approx(r["prune_frac"], abs=1e-3)
    # the same fit with the points on the device, every cluster sum recomputed in every update
    dev = skm.fit(cuda(X), k, iters, 3, skm.FitOptions(R=cuda(R), eps0=EPS0, adjust_dprime=False, full_update=True))
    assert (dev.assign.cpu().numpy() == a).mean() >= 0.999
    # (the two fits visit the points in different orders and tile them differently: a near-tie may fall the other way,
    # which moves a point between two clusters; the clusters with the same members must agree)
    check_assignment(dev.assign.cpu().numpy(), ref.assign, orc.rotate(X, R), ref.centroids_rot,
                     own=(X, dev.centroids.cpu().numpy()))
    clean = check_centroids(got.centroids.cpu().numpy(), dev.centroids.cpu().numpy(), a, dev.assign.cpu().numpy())
    same = (dev.assign.cpu().numpy() == a) & np.isin(a, clean)          # clusters with the same members in both fits
    assert same.mean() > 0.97
    assert np.abs(got.dist.numpy()[same] - dev.dist.cpu().numpy()[same]).max() < 1e-5


def test_host_resident_fit_options(skm, orc, dg):
    """d' adjustment, no rotation, no final pass, empty clusters: the host-resident fit follows the same rules."""
    X = dg.mixture(12_000, 256, 64, 8, "embed").numpy()
    R = orc.random_rotation(256, 8)
    got = skm.fit_host(torch.from_numpy(X).pin_memory(), 64, 8, 5, batch_rows=5120,
                       opts=skm.FitOptions(R=cuda(R), eps0=EPS0))
    ref = orc.fit(X, 64, 8, 5, orc.FitParams(eps0=EPS0), R=R)
    assert [g["dprime"] for g in got.trace] == [r["dprime"] for r in ref.trace]
    assert got.trace[-1]["objective"] == pytest.approx(ref.trace[-1]["objective"], rel=1e-4)
    assert rel_l2(got.centroids.cpu().numpy(), ref.centroids) < 1e-3
    # repeated initial rows leave clusters empty after iteration 1; no rotation; labels of the last in-loop step
    X = dg.mixture(6000, 64, 24, 10, "linear").numpy()
    idx = orc.sample_rows(1, 6000, 12)
    idx[1] = idx[0]
    idx[2] = idx[0]
    got = skm.fit_host(torch.from_numpy(X), 12, 5, 1, batch_rows=2048,
                       opts=skm.FitOptions(rotate=False, eps0=EPS0, adjust_dprime=False, final_assign=False,
                                           init_idx=list(idx)))
    ref = orc.fit(X, 12, 5, 1, orc.FitParams(eps0=EPS0, adjust_dprime=False, final_assign=False), R=None, init_idx=idx)
    assert [g["nempty"] for g in got.trace] == [r["nempty"] for r in ref.trace] and ref.trace[0]["nempty"] == 2
    check_assignment(got.assign.numpy(), ref.assign, X, ref.centroids_rot, own=(X, got.centroids.cpu().numpy()))
    assert rel_l2(got.centroids.cpu().numpy(), ref.centroids) < 1e-3
    a = got.assign.numpy()
    S = np.zeros((12, 64))
    np.add.at(S, a, X.astype(np.float64))
    assert np.abs(got.centroids.cpu().numpy() - S / np.bincount(a, minlength=12)[:, None]).max() < 1e-6
    with pytest.raises(RuntimeError):
        skm.fit_host(torch.from_numpy(X), 12, 5, 1, opts=skm.FitOptions(angular=True))


# ------------------------------------------------------------------ whole fit in lock step: the strict contract
def _witness(orc, Xr, Yr, i, j, tau, d, dprime):
    """True if centroid j's partial distance to point i comes within fp32 rounding of the pruning threshold at some
    checkpoint (then the statistical test may fall either way in fp32 and in fp64)."""
    diff2 = (Xr[i] - Yr[j]) ** 2
    t = dprime
    while t < d:
        p = diff2[:t].sum()
        thr = orc.theta_ratio(d, t, EPS0) * tau
        if abs(p - thr) <= 2e-5 * max(thr, 1e-30):
            return True
        t = min(d, t + 64)
    return abs(diff2.sum() - tau) <= 2e-5 * max(tau, 1e-30)


def lockstep_fit(skm, orc, X, R, k, iters, seed, adjust, screen=0):
    """Algorithm 1 driven by the oracle; at every iteration the library's step calls (skm_assign_exact /
    skm_assign_ex, skm_update) get the oracle's state (centroids Y_t and labels a_t, rounded to fp32 once and used by
    both sides) and must meet the contract with no relaxation: >= 99.9 % of the labels equal, every other one a
    near-tie of <= 1e-4 (or a pair whose partial distance sits on the pruning threshold to fp32 rounding, counted and
    bounded), centroids of ALL clusters within 1e-3 relative L2, objective within 1e-4, survivor counters within
    0.1 %, the same d' decision."""
    n, d = X.shape
    Xr = orc.rotate(X, R).astype(np.float32)          # the rotated points both sides work on
    Xr64 = Xr.astype(np.float64)
    Xg = cuda(Xr)
    plain = dict(rotate=False, eps0=EPS0, block_stats=True, screen=screen)
    Y = Xr[orc.sample_rows(seed, n, k)].copy()         # fp32 centroids, the state handed from step to step
    rng_state = orc.rng_stream(seed, 1)
    dp = orc.dprime_init(d)
    prev = None
    on_threshold = 0
    for t in range(1, iters + 2):                       # iterations 1..iters, then the final assignment pass
        Y64 = Y.astype(np.float64)
        if t == 1:
            a_ref, d_ref = orc.assign_full(Xr64, Y64)
            a, dist = skm.assign_exact(Xg, cuda(Y))
            row = None
        else:
            ref = orc.assign_pruned(Xr64, Y64, prev, dp, EPS0, 0)
            a_ref, d_ref = ref.assign, ref.dist
            a, dist, row = skm.assign(Xg, cuda(Y), cuda(prev), dp, skm.FitOptions(**plain))
        a = a.cpu().numpy()
        diff = np.nonzero(a != a_ref)[0]
        assert len(diff) <= 1e-3 * n, (t, len(diff))
        far = 0
        for i in diff:
            dg = ((Xr64[i] - Y64[a[i]]) ** 2).sum()
            dr = ((Xr64[i] - Y64[a_ref[i]]) ** 2).sum()
            if abs(dg - dr) <= 1e-4 * min(dg, dr):
                continue
            # not a near-tie: only possible in a pruned step, when the statistical test of the better centroid sat on
            # its threshold (the side that pruned it keeps a farther centroid)
            assert t > 1, (t, i, dg, dr)
            tau = ((Xr64[i] - Y64[prev[i]]) ** 2).sum()
            loser = a_ref[i] if dr < dg else a[i]
            assert _witness(orc, Xr64, Y64, i, loser, tau, d, dp), (t, i, dg, dr)
            far += 1
        on_threshold += far
        say(f"lockstep t={t} d'={dp if t > 1 else d} disagreements {len(diff)} (on a threshold: {far})")
        same = a == a_ref
        assert np.abs(dist.cpu().numpy()[same] - d_ref[same]).max() < 2e-5 * max(1.0, d_ref.max())
        if row is not None:
            assert row["objective"] == pytest.approx(d_ref.sum(), rel=1e-4)
            surv_ref = n * (k - 1) - ref.pruned_first
            assert abs(row["survivors"] - surv_ref) <= max(2, 1e-3 * surv_ref)
            for m in range(min(row["nblocks"], 32)):
                assert abs(row["enter"][m] - ref.enter[m]) <= max(2, 1e-3 * ref.enter[m])
            assert abs(row["completed"] - ref.enter[-1]) <= max(2, 1e-3 * ref.enter[-1])
        if t == iters + 1:
            break
        # update on the oracle's labels, both sides; every cluster is compared
        Yn, cnt = orc.update(Xr64, a_ref, Y64)
        Yg = cuda(Y)
        cg = skm.update(Xg, cuda(a_ref), Yg).cpu().numpy()
        assert (cg == cnt).all()
        assert rel_l2(Yg.cpu().numpy(), Yn) < 1e-6 and np.abs(Yg.cpu().numpy() - Yn).max() < 1e-6
        if (cnt == 0).any():
            Yn, cnt, _, rng_state = orc.split_empty(Yn, cnt, rng_state)
        if t > 1 and adjust:
            f_ref = ref.pruned_first / (n * (k - 1))
            new_dp = orc.dprime_adjust(d, dp, f_ref)
            assert skm.dprime_adjust(d, dp, row["prune_frac"]) == new_dp
            dp = new_dp
        Y = Yn.astype(np.float32)
        prev = a_ref.astype(np.int32)
    return on_threshold


@pytest.mark.parametrize("screen", [-1, 1])
def test_lockstep_fit_c1(skm, orc, dg, screen):
    """Workload C1, all 10 iterations and the final pass, the strict contract at every step; without and with the
    low-precision first filter in front of every pruned step."""
    X = dg.config_data("C1").numpy()
    on_thr = lockstep_fit(skm, orc, X, orc.random_rotation(128, 42), 100, 10, 42, adjust=True, screen=screen)
    assert on_thr <= 2


@pytest.mark.parametrize("screen", [-1, 1])
def test_lockstep_fit_scaled_c2(skm, orc, dg, screen):
    """The first 131 072 rows of workload C2 (d = 1536, k = 1024), all 10 iterations and the final pass."""
    torch.cuda.empty_cache()
    X = dg.config_data("C2", device="cuda", n=131_072).cpu().numpy()
    on_thr = lockstep_fit(skm, orc, X, orc.random_rotation(1536, 42), 1024, 10, 42, adjust=True, screen=screen)
    assert on_thr <= 4
