"""Pins of the CPU oracle against things other than itself (CPU only).

Each test fixes one part of the oracle with a brute-force computation, a closed
form, an invariant or a published value, so that a dropped term, a wrong index
or a transposed operand in ``oracle/skm_oracle.c`` fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import scipy.stats

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def unit_rows(rng, n, d, m=8, spread=0.6):
    means = rng.standard_normal((m, d))
    x = means[rng.integers(0, m, n)] + spread * rng.standard_normal((n, d))
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    return x.astype(np.float32)


def brute_dist(Xr, Y):
    """All squared distances, fp64, by the plain definition."""
    diff = Xr[:, None, :].astype(np.float64) - Y[None, :, :].astype(np.float64)
    return np.einsum("ijk,ijk->ij", diff, diff)


# --------------------------------------------------------------- PRNG
def test_splitmix64_published_vectors(orc):
    want = [int(l, 16) for l in open(os.path.join(GOLD, "splitmix64_seed0.txt")) if l.strip()]
    got, _ = orc.rng_draws(0, len(want))
    assert got == want


def test_sample_rows_distinct_uniform(orc):
    idx = orc.sample_rows(7, 1000, 1000)
    assert sorted(idx.tolist()) == list(range(1000))          # a permutation when k = n
    a = orc.sample_rows(7, 10_000, 64)
    b = orc.sample_rows(7, 10_000, 64)
    c = orc.sample_rows(8, 10_000, 64)
    assert (a == b).all() and (a != c).any()
    assert len(set(a.tolist())) == 64 and a.min() >= 0 and a.max() < 10_000
    # every row is equally likely to be the first pick: chi-square over 20 bins
    firsts = np.array([orc.sample_rows(s, 20, 1)[0] for s in range(4000)])
    chi2 = ((np.bincount(firsts, minlength=20) - 200.0) ** 2 / 200.0).sum()
    assert chi2 < scipy.stats.chi2.ppf(0.9999, 19)
    # first draw is rng % n on stream 0 (partial Fisher-Yates, identity start)
    draws, _ = orc.rng_draws(orc.rng_stream(5, 0), 1)
    assert orc.sample_rows(5, 977, 3)[0] == draws[0] % 977


# --------------------------------------------------------------- theta
def test_theta_hand_values(orc):
    for line in open(os.path.join(GOLD, "theta_ratio.txt")):
        if line.startswith("#") or not line.strip():
            continue
        d, t, eps0, want = line.split()
        assert orc.theta_ratio(int(d), int(t), float(eps0)) == pytest.approx(float(want), rel=1e-12)


def test_theta_monotone_capped_and_limits(orc):
    for d in (128, 384, 768, 1536):
        r = [orc.theta_ratio(d, t, 2.1) for t in range(16, d + 1, 16)]
        assert all(b >= a for a, b in zip(r, r[1:]))
        assert max(r) == 1.0 and r[-1] == 1.0
        assert orc.theta_ratio(d, 16, 0.0) == pytest.approx(16 / d)          # eps0 = 0: plain scaling
        assert orc.theta_ratio(d, 16, float("inf")) == 1.0                     # test disabled -> exact bound only
        assert orc.theta_ratio(d, 16, 2.1) < orc.theta_ratio(d, 16, 3.0)


def test_theta_is_a_rare_event_bound_for_random_rotations(orc):
    """After a random rotation the share of a vector's squared norm that falls
    on t of d coordinates is Beta(t/2, (d-t)/2).  The ADSampling test must
    reject a borderline candidate (true distance == tau) only rarely, and must
    not be vacuous: the tail mass at the threshold is small but not zero."""
    for d, t in ((128, 16), (1536, 192), (768, 96), (384, 48), (1536, 704)):
        ratio = orc.theta_ratio(d, t, 2.1)
        if ratio >= 1.0:
            continue
        tail = scipy.stats.beta.sf(ratio, t / 2.0, (d - t) / 2.0)
        assert 1e-12 < tail < 5e-3, (d, t, tail)
        # a candidate 1.6x farther (in squared distance 2.56x) is cut with fair probability at d/8
        far = scipy.stats.beta.sf(ratio / 2.56, t / 2.0, (d - t) / 2.0)
        assert far > 0.5, (d, t, far)


def test_dprime_rules(orc):
    assert [orc.dprime_init(d) for d in (128, 1536, 768, 384)] == [16, 192, 96, 48]   # floor(d/8)
    assert orc.dprime_init(100) == 16 and orc.dprime_init(16) == 16
    assert orc.dprime_adjust(1536, 192, 0.98) == 160      # 192 - 38.4 = 153.6 -> 160
    assert orc.dprime_adjust(1536, 192, 0.90) == 224      # 230.4 -> 224
    assert orc.dprime_adjust(1536, 192, 0.96) == 192
    assert orc.dprime_adjust(1536, 192, 0.95) == 192 and orc.dprime_adjust(1536, 192, 0.97) == 192
    assert orc.dprime_adjust(256, 32, 0.90) == 48 and orc.dprime_adjust(256, 32, 0.99) == 16   # at least one step of 16
    assert orc.dprime_adjust(384, 48, 0.90) == 64 and orc.dprime_adjust(384, 48, 0.99) == 32
    assert orc.dprime_adjust(128, 16, 0.99) == 16         # lower clamp
    assert orc.dprime_adjust(128, 128, 0.5) == 128        # upper clamp
    assert orc.dprime_adjust(100, 96, 0.5) == 96          # upper clamp is the last multiple of 16


# --------------------------------------------------------------- rotation
def test_rotation_orthogonal_and_distance_preserving(orc):
    rng = np.random.default_rng(0)
    for d in (16, 80, 128):
        R = orc.random_rotation(d, 3)
        assert R.dtype == np.float32
        assert np.abs(R.astype(np.float64) @ R.astype(np.float64).T - np.eye(d)).max() < 1e-6
        X = unit_rows(rng, 200, d)
        Xr = orc.rotate(X, R)
        assert np.allclose(Xr, X.astype(np.float64) @ R.astype(np.float64), atol=1e-12)   # X*R, not X*R^T
        D0 = brute_dist(X, X)
        D1 = brute_dist(Xr, Xr)
        assert np.abs(D0 - D1).max() < 1e-5 * max(1.0, D0.max())
        back = orc.unrotate(Xr, R)                                  # (X R) R^T = X
        assert np.abs(back - X).max() < 1e-5
    # a rotation that is not symmetric tells X*R from X*R^T
    assert np.abs(R - R.T).max() > 0.1


def test_partial_plus_trailing_and_norm_expansion(orc):
    rng = np.random.default_rng(1)
    X = unit_rows(rng, 50, 96).astype(np.float64)
    Y = unit_rows(rng, 7, 96).astype(np.float64)
    full = brute_dist(X, Y)
    for dp in (16, 32, 80):
        front = brute_dist(X[:, :dp], Y[:, :dp])
        back = brute_dist(X[:, dp:], Y[:, dp:])
        assert np.allclose(front + back, full, rtol=1e-12)
        ident = (X[:, :dp] ** 2).sum(1)[:, None] + (Y[:, :dp] ** 2).sum(1)[None, :] - 2 * X[:, :dp] @ Y[:, :dp].T
        assert np.allclose(ident, front, rtol=1e-9, atol=1e-12)


# --------------------------------------------------------------- exact paths
SHAPES = [(300, 16, 5), (500, 80, 17), (400, 128, 64), (257, 200, 33), (64, 144, 64)]


@pytest.mark.parametrize("n,d,k", SHAPES)
def test_full_assignment_is_brute_force(orc, n, d, k):
    rng = np.random.default_rng(n + d + k)
    X = unit_rows(rng, n, d).astype(np.float64)
    Y = X[rng.choice(n, k, replace=False)].copy()
    a, dist = orc.assign_full(X, Y)
    D = brute_dist(X, Y)
    assert (a == D.argmin(1)).all()
    assert np.allclose(dist, D.min(1), rtol=1e-12, atol=1e-15)


def test_full_assignment_lowest_index_on_ties(orc):
    X = np.array([[0.0, 0.0] + [0.0] * 14], dtype=np.float64)
    Y = np.zeros((4, 16))
    Y[0, 0] = 2.0
    Y[1, 0] = 1.0
    Y[2, 1] = 1.0     # same distance as centroid 1
    Y[3, 0] = -1.0    # same again
    a, _ = orc.assign_full(X, Y)
    assert a[0] == 1


@pytest.mark.parametrize("n,d,k", SHAPES)
@pytest.mark.parametrize("G", [1, 7, 0])
def test_pruned_assignment_without_statistical_test_is_brute_force(orc, n, d, k, G):
    """eps0 = inf leaves only the always-valid bound p_t > tau, which cannot cut
    the true nearest centroid: the result must be the exact argmin, whatever the
    previous assignment and whatever d' (tail blocks, d' not a multiple of 64)."""
    rng = np.random.default_rng(n * 3 + d + k + G)
    X = unit_rows(rng, n, d).astype(np.float64)
    Y = unit_rows(rng, k, d).astype(np.float64)
    D = brute_dist(X, Y)
    prev = rng.integers(0, k, n).astype(np.int32)
    for dp in sorted(v for v in {16, 32, (d // 16) * 16, orc.dprime_init(d)} if v <= d):
        res = orc.assign_pruned(X, Y, prev, dp, eps0=float("inf"), G=G)
        dmin = D.min(1)
        assert np.allclose(res.dist, dmin, rtol=1e-12, atol=1e-15)
        # ties: the incumbent wins, else lowest index
        exp = np.where(D[np.arange(n), prev] <= dmin, prev, D.argmin(1))
        assert (res.assign == exp).all()


def test_incumbent_wins_ties_then_lowest_index(orc):
    d = 32
    X = np.zeros((1, d))
    Y = np.zeros((5, d))
    Y[0, 0] = 3.0
    Y[1, 20] = 1.0
    Y[2, 1] = 1.0
    Y[3, 2] = 1.0
    Y[4, 3] = 0.5
    for G in (1, 5):
        r = orc.assign_pruned(X, Y, np.array([3], np.int32), 16, eps0=float("inf"), G=G)
        assert r.assign[0] == 4                                   # strictly better challenger wins
        r = orc.assign_pruned(X, Y[:4], np.array([3], np.int32), 16, eps0=float("inf"), G=G)
        assert r.assign[0] == 3                                   # ties with the incumbent: incumbent stays
        r = orc.assign_pruned(X, Y[:4], np.array([0], np.int32), 16, eps0=float("inf"), G=G)
        assert r.assign[0] == 1                                   # ties among challengers: lowest index


# --------------------------------------------------------------- pruning proper
def checkpoints(d, dp):
    ts = []
    t = dp
    while t < d:
        t = min(d, t + 64)
        ts.append(t)
    return ts


def numpy_fates(X, Y, prev, dp, eps0, ratio):
    """Frozen-tau (G = k) fate of every pair, computed with cumulative sums."""
    n, d = X.shape
    k = Y.shape[0]
    sq = (X[:, None, :] - Y[None, :, :]) ** 2
    cum = np.cumsum(sq, axis=2)                     # cum[..., t-1] = distance on the first t dims
    tau = cum[np.arange(n), prev, d - 1]
    fate = np.full((n, k), d, dtype=np.int64)
    done = np.zeros((n, k), dtype=bool)
    for t in [dp] + checkpoints(d, dp)[:-1]:
        cut = (cum[:, :, t - 1] > tau[:, None] * ratio(d, t, eps0)) & ~done
        fate[cut] = t
        done |= cut
    if dp == d:   # no trailing block: the first test is the exact comparison
        pass
    fate[np.arange(n), prev] = 0
    return fate, cum, tau


@pytest.mark.parametrize("n,d,k,dp", [(200, 128, 20, 16), (150, 200, 33, 32), (120, 144, 16, 48), (100, 80, 9, 16)])
def test_fate_of_every_pair_matches_cumulative_sums(orc, n, d, k, dp):
    rng = np.random.default_rng(d + k)
    R = orc.random_rotation(d, 1)
    X = orc.rotate(unit_rows(rng, n, d), R)
    Y = X[rng.choice(n, k, replace=False)] + 0.05 * rng.standard_normal((k, d))
    prev = brute_dist(X, Y).argmin(1).astype(np.int32)
    prev[::3] = rng.integers(0, k, len(prev[::3]))          # a third of the points start from a poor incumbent
    res = orc.assign_pruned(X, Y, prev, dp, eps0=2.1, G=0, want_fate=True)
    fate, cum, tau = numpy_fates(X, Y, prev, dp, 2.1, orc.theta_ratio)
    assert (res.fate == fate).all()
    # counters follow from the fates
    assert res.pruned_first == int((fate == dp).sum()) - (0 if dp < d else 0)
    cps = checkpoints(d, dp)
    alive_before = [(fate > t).sum() for t in [dp] + cps[:-1]]
    assert res.enter[:-1].tolist() == [int(v) for v in alive_before]
    assert res.enter[-1] == int((fate == d).sum())
    # result = best completed challenger if strictly below tau, else the incumbent
    full = cum[:, :, d - 1]
    cand = np.where(fate == d, full, np.inf)
    bj = cand.argmin(1)
    bd = cand.min(1)
    win = bd < tau
    assert (res.assign == np.where(win, bj, prev)).all()
    assert np.allclose(res.dist, np.where(win, bd, tau), rtol=1e-12)


@pytest.mark.parametrize("G", [1, 4, 0])
def test_one_sided_and_every_false_prune_has_a_witness(orc, G):
    rng = np.random.default_rng(11)
    n, d, k, dp = 1500, 128, 48, 16
    R = orc.random_rotation(d, 2)
    X = orc.rotate(unit_rows(rng, n, d, m=30, spread=0.9), R)
    Y = X[rng.choice(n, k, replace=False)].copy()
    D = brute_dist(X, Y)
    prev = rng.integers(0, k, n).astype(np.int32)
    # a small eps0 makes false prunes frequent enough to be seen
    res = orc.assign_pruned(X, Y, prev, dp, eps0=0.3, G=G, want_fate=True)
    dmin = D.min(1)
    assert (res.dist >= dmin * (1 - 1e-12)).all()                       # never below the exact minimum
    assert (res.dist <= D[np.arange(n), prev] * (1 + 1e-12)).all()      # never worse than the incumbent
    assert np.allclose(res.dist, D[np.arange(n), res.assign], rtol=1e-12)  # the distance is that of the assignment
    wrong = np.nonzero(res.dist > dmin * (1 + 1e-12))[0]
    assert 0 < len(wrong) < n // 2
    cum = np.cumsum((X[:, None, :] - Y[None, :, :]) ** 2, axis=2)
    for i in wrong:
        js = D[i].argmin()
        t = res.fate[i, js]
        assert 0 < t < d                                                # the true best was cut early
        # ... by a threshold no larger than the initial one (tau only shrinks)
        assert cum[i, js, t - 1] > res.dist[i] * orc.theta_ratio(d, t, 0.3) * (1 - 1e-12)
    # with the paper-scale eps0 false prunes are rare
    res21 = orc.assign_pruned(X, Y, prev, dp, eps0=2.1, G=G)
    assert (res21.dist > dmin * (1 + 1e-12)).mean() < 0.01


def test_group_size_one_is_algorithm_one_to_the_letter(orc):
    """G = 1 against a direct Python transcription of the per-centroid loop."""
    rng = np.random.default_rng(5)
    n, d, k, dp, eps0 = 60, 144, 12, 16, 1.0
    X = orc.rotate(unit_rows(rng, n, d), orc.random_rotation(d, 9))
    Y = X[rng.choice(n, k, replace=False)] + 0.02 * rng.standard_normal((k, d))
    prev = rng.integers(0, k, n).astype(np.int32)
    res = orc.assign_pruned(X, Y, prev, dp, eps0=eps0, G=1)
    for i in range(n):
        tau = float(((X[i] - Y[prev[i]]) ** 2).sum())
        a = int(prev[i])
        for j in range(k):
            if j == prev[i]:
                continue
            t = dp
            p = float(((X[i, :dp] - Y[j, :dp]) ** 2).sum())
            if p > tau * min(1.0, t / d * (1 + eps0 / math.sqrt(t)) ** 2):
                continue
            alive = True
            while t < d:
                t1 = min(d, t + 64)
                p += float(((X[i, t:t1] - Y[j, t:t1]) ** 2).sum())
                t = t1
                if t < d and p > tau * min(1.0, t / d * (1 + eps0 / math.sqrt(t)) ** 2):
                    alive = False
                    break
            if alive and p < tau:
                tau = p
                a = j
        assert res.assign[i] == a
        assert res.dist[i] == pytest.approx(tau, rel=1e-12)


def test_no_prev_seeds_incumbent_from_partial_distances(orc):
    rng = np.random.default_rng(6)
    n, d, k, dp = 300, 128, 25, 16
    X = orc.rotate(unit_rows(rng, n, d), orc.random_rotation(d, 4))
    Y = X[rng.choice(n, k, replace=False)].copy()
    seed = brute_dist(X[:, :dp], Y[:, :dp]).argmin(1).astype(np.int32)
    a = orc.assign_pruned(X, Y, None, dp, eps0=2.1, G=0)
    b = orc.assign_pruned(X, Y, seed, dp, eps0=2.1, G=0)
    assert (a.assign == b.assign).all() and np.array_equal(a.dist, b.dist)


# --------------------------------------------------------------- update / split
def test_update_is_the_mean_of_assigned_points(orc):
    rng = np.random.default_rng(2)
    n, d, k = 3000, 48, 37
    X = unit_rows(rng, n, d).astype(np.float64)
    a = rng.integers(0, k - 2, n).astype(np.int32)       # clusters k-2, k-1 stay empty
    Y0 = rng.standard_normal((k, d))
    Y, counts = orc.update(X, a, Y0)
    S = np.zeros((k, d))
    np.add.at(S, a, X)
    cnt = np.bincount(a, minlength=k)
    assert (counts == cnt).all() and counts.sum() == n
    nz = cnt > 0
    assert np.allclose(Y[nz], S[nz] / cnt[nz, None], rtol=1e-12, atol=1e-15)
    assert np.array_equal(Y[~nz], Y0[~nz])               # empty clusters keep their centroid


def test_split_empty_rules(orc):
    rng = np.random.default_rng(3)
    k, d = 12, 10
    Y = rng.standard_normal((k, d))
    counts = np.array([5, 0, 1, 40, 0, 2, 0, 9, 1, 1, 30, 12], dtype=np.int64)
    st = orc.rng_stream(99, 1)
    Y2, c2, log, _ = orc.split_empty(Y, counts, st)
    assert [e for e, _ in log] == [1, 4, 6]               # increasing index
    assert c2.sum() == counts.sum() and (c2 > 0).all()
    Yw = Y.copy()
    cw = counts.copy()
    draws, _ = orc.rng_draws(st, 3)
    for (e, c), r in zip(log, draws):
        assert cw[c] >= 2                                  # donors hold at least two points
        elig = np.where(cw >= 2, cw, 0)
        assert c == int(np.searchsorted(np.cumsum(elig), int(r % int(elig.sum())), side="right"))
        s = np.where(np.arange(d) % 2 == 0, 1.0, -1.0)
        y = Yw[c].copy()
        Yw[e] = y * (1 + s / 1024)
        Yw[c] = y * (1 - s / 1024)
        cw[e] = cw[c] // 2
        cw[c] -= cw[e]
    assert np.allclose(Y2, Yw, rtol=1e-15) and (c2 == cw).all()
    one = np.array([3, 0, 7], dtype=np.int64)                          # a single split is symmetric around the donor
    Y3, c3, log3, _ = orc.split_empty(Y[:3], one, st)
    (e, c), = log3
    assert e == 1 and np.allclose((Y3[e] + Y3[c]) / 2, Y[c], rtol=1e-12) and not np.allclose(Y3[e], Y3[c])
    assert c3.tolist() in ([2, 1, 7], [3, 3, 4])


def test_split_donor_probability_grows_with_size(orc):
    counts = np.array([0, 10, 30, 60, 1], dtype=np.int64)
    Y = np.ones((5, 4))
    hits = np.zeros(5)
    st = orc.rng_stream(1, 1)
    for _ in range(3000):
        _, _, log, st = orc.split_empty(Y, counts, st)
        hits[log[0][1]] += 1
    assert hits[0] == 0 and hits[4] == 0
    exp = 3000 * np.array([10, 30, 60]) / 100.0
    assert (((hits[1:4] - exp) ** 2) / exp).sum() < scipy.stats.chi2.ppf(0.9999, 2)


# --------------------------------------------------------------- whole fit
def lloyd_numpy(X, Y, iters):
    X = X.astype(np.float64)
    Y = Y.astype(np.float64).copy()
    objs = []
    for _ in range(iters):
        D = brute_dist(X, Y)
        a = D.argmin(1)
        objs.append(D.min(1).sum())
        for c in range(len(Y)):
            if (a == c).any():
                Y[c] = X[a == c].mean(0)
    return Y, a, objs


def test_fit_without_rotation_and_test_is_textbook_lloyd(orc):
    rng = np.random.default_rng(4)
    n, d, k, iters = 1200, 64, 10, 6
    X = unit_rows(rng, n, d)
    idx = orc.sample_rows(42, n, k)
    p = orc.FitParams(eps0=float("inf"), adjust_dprime=False, final_assign=False)
    fr = orc.fit(X, k, iters, 42, p, R=None, init_idx=idx)
    Y, a, objs = lloyd_numpy(X, X[idx], iters)
    assert all(r["nempty"] == 0 for r in fr.trace)
    assert np.allclose(fr.centroids, Y, rtol=1e-10, atol=1e-12)
    assert (fr.assign == a).all()
    assert np.allclose([r["objective"] for r in fr.trace], objs, rtol=1e-10)


def test_convergence_stop_follows_textbook_label_changes(orc):
    """conv_tol (Section 3.3, second condition): with the statistical test off the fit is textbook Lloyd, so the
    iteration at which it stops is the first t >= 2 at which numpy's Lloyd changes at most conv_tol * n labels."""
    rng = np.random.default_rng(12)
    n, d, k, iters = 1500, 32, 6, 30
    X = unit_rows(rng, n, d)
    idx = orc.sample_rows(3, n, k)
    # label changes per iteration of the textbook algorithm
    Y = X[idx].astype(np.float64).copy()
    prev, changes = None, []
    for _ in range(iters):
        D = ((X[:, None, :].astype(np.float64) - Y[None, :, :]) ** 2).sum(2)
        a = D.argmin(1)
        changes.append(n if prev is None else int((a != prev).sum()))
        prev = a
        for c in range(k):
            if (a == c).any():
                Y[c] = X[a == c].mean(0)
    assert changes[-1] == 0 and changes[1] > 0.02 * n            # the run does converge, and not at once
    for tol in (0.02, 0.002, 1e-9, 1.0):
        want = next(t for t in range(2, iters + 1) if changes[t - 1] <= tol * n)
        p = orc.FitParams(eps0=float("inf"), adjust_dprime=False, final_assign=False, conv_tol=tol)
        fr = orc.fit(X, k, iters, 3, p, R=None, init_idx=idx)
        assert fr.iters_run == want, (tol, fr.iters_run, want)
    off = orc.fit(X, k, 8, 3, orc.FitParams(eps0=float("inf"), adjust_dprime=False, final_assign=False), R=None, init_idx=idx)
    assert off.iters_run == 8                                    # 0 = no convergence stop


def test_fit_rotation_invariance_and_unrotation(orc):
    rng = np.random.default_rng(8)
    n, d, k, iters = 800, 48, 8, 5
    X = unit_rows(rng, n, d)
    idx = orc.sample_rows(1, n, k)
    p = orc.FitParams(eps0=float("inf"), adjust_dprime=False)
    a = orc.fit(X, k, iters, 1, p, R=None, init_idx=idx)
    b = orc.fit(X, k, iters, 1, p, R=orc.random_rotation(d, 5), init_idx=idx)
    assert (a.assign == b.assign).mean() > 0.995
    assert np.abs(a.centroids - b.centroids).max() < 1e-4 or (a.assign == b.assign).all() is False
    same = (a.assign == b.assign).all()
    if same:
        assert np.abs(a.centroids - b.centroids).max() < 1e-5     # Y = Yr R^T is back in the original space
    assert a.trace[-1]["objective"] == pytest.approx(b.trace[-1]["objective"], rel=1e-4)


def test_fit_objective_never_increases_and_centroids_are_means(orc):
    from paper_2603_20009_amd import datagen
    X = datagen.mixture(4000, 128, 40, 77, "linear").numpy()
    k, iters = 32, 8
    R = orc.random_rotation(128, 77)
    for G, adjust in ((0, False), (1, True), (8, True)):
        p = orc.FitParams(tau_group=G, adjust_dprime=adjust, final_assign=True)
        fr = orc.fit(X, k, iters, 3, p, R=R)
        assert all(r["nempty"] == 0 for r in fr.trace)
        obj = [r["objective"] for r in fr.trace]
        assert all(b <= a * (1 + 1e-12) for a, b in zip(obj, obj[1:])), obj      # no-regress holds with pruning
        assert fr.trace[0]["prune_frac"] == 0.0 and fr.trace[0]["dprime"] == 128
        assert 0.3 < fr.trace[2]["prune_frac"] <= 1.0
        # centroids are the means of the last in-loop assignment: recompute it with one exact step from the
        # returned rotated centroids' predecessors is not possible here, so check through the final pass:
        Xr = orc.rotate(X, R)
        D = brute_dist(Xr, fr.centroids_rot)
        assert np.allclose(fr.dist, D[np.arange(len(X)), fr.assign], rtol=1e-10)
        # and the exact objective at these centroids is not above what the pruned pass reports by more than 0.1%
        assert D.min(1).sum() <= fr.dist.sum() <= D.min(1).sum() * 1.001
    # means: run without the final pass so that assign is the assignment the centroids were built from
    p = orc.FitParams(final_assign=False)
    fr = orc.fit(X, k, iters, 3, p, R=R)
    Xr = orc.rotate(X, R)
    S = np.zeros((k, 128))
    np.add.at(S, fr.assign, Xr)
    cnt = np.bincount(fr.assign, minlength=k)
    assert np.allclose(fr.centroids_rot, S / cnt[:, None], rtol=1e-12, atol=1e-15)
    assert np.allclose(fr.centroids, fr.centroids_rot @ R.astype(np.float64).T, rtol=1e-12, atol=1e-15)


def test_fit_is_deterministic_and_close_to_exact_kmeans(orc):
    from paper_2603_20009_amd import datagen
    X = datagen.mixture(3000, 128, 30, 5, "linear").numpy()
    R = orc.random_rotation(128, 5)
    a = orc.fit(X, 24, 6, 9, orc.FitParams(), R=R)
    b = orc.fit(X, 24, 6, 9, orc.FitParams(), R=R)
    assert (a.assign == b.assign).all() and np.array_equal(a.centroids, b.centroids)
    exact = orc.fit(X, 24, 6, 9, orc.FitParams(eps0=float("inf")), R=R)
    assert a.trace[-1]["objective"] == pytest.approx(exact.trace[-1]["objective"], rel=5e-3)


def test_fit_dprime_adjustment_follows_the_band(orc):
    from paper_2603_20009_amd import datagen
    X = datagen.mixture(3000, 256, 30, 6, "embed").numpy()
    fr = orc.fit(X, 40, 7, 2, orc.FitParams(adjust_dprime=True), R=orc.random_rotation(256, 6))
    tr = fr.trace
    assert tr[1]["dprime"] == 32
    for prev_row, row in zip(tr[1:], tr[2:]):
        assert row["dprime"] == orc.dprime_adjust(256, prev_row["dprime"], prev_row["prune_frac"])
        assert prev_row["prune_frac"] == prev_row["pruned_first"] / (3000 * 39)


def test_fit_splits_empty_clusters(orc):
    # 40 distinct points duplicated many times, k larger than the number of distinct points
    rng = np.random.default_rng(10)
    base = unit_rows(rng, 10, 32)
    X = np.repeat(base, 30, axis=0)
    fr = orc.fit(X, 16, 4, 1, orc.FitParams(eps0=float("inf"), final_assign=False), R=None)
    assert fr.trace[0]["nempty"] > 0
    cnt = np.bincount(fr.assign, minlength=16)
    assert cnt.sum() == 300


# --------------------------------------------------------------- ETR
def test_ground_truth_and_recall_closed_form(orc):
    rng = np.random.default_rng(12)
    n, d, k, nq, K = 900, 32, 30, 25, 10
    X = unit_rows(rng, n, d)
    Q = unit_rows(rng, nq, d)
    gt = orc.ground_truth(X, Q, K)
    D = brute_dist(Q, X)
    order = np.lexsort((np.arange(n)[None, :].repeat(nq, 0), D), axis=1)[:, :K]
    assert (gt == order).all()
    Y = X[rng.choice(n, k, replace=False)].astype(np.float64)
    a = brute_dist(X, Y).argmin(1).astype(np.int32)
    DQ = brute_dist(Q, Y)
    for nprobe in (1, 3, k):
        # explicit IVF search: scan every point of the probed clusters, keep the K nearest, intersect with gt
        hits = 0
        for q in range(nq):
            probed = np.argsort(DQ[q], kind="stable")[:nprobe]
            members = np.nonzero(np.isin(a, probed))[0]
            found = members[np.lexsort((members, D[q, members]))[:K]]
            hits += len(set(found.tolist()) & set(gt[q].tolist()))
        want = hits / (nq * K)
        got = orc.recall(Q.astype(np.float64), Y, nprobe, gt, a)
        assert got == pytest.approx(want, abs=1e-12)
    assert orc.recall(Q.astype(np.float64), Y, k, gt, a) == 1.0
    assert orc.nprobe(4096, 0.01) == 41 and orc.nprobe(10, 0.01) == 1 and orc.nprobe(1024, 0.01) == 10


def test_etr_stops_early_and_reports_recall(orc):
    from paper_2603_20009_amd import datagen
    X = datagen.mixture(3000, 64, 20, 3, "linear").numpy()
    Q = datagen.mixture(50, 64, 20, 4, "linear").numpy()
    p = orc.FitParams(etr=True, etr_tol=0.5, etr_patience=2, probe_frac=0.1)   # tol so large that nothing "improves"
    fr = orc.fit(X, 20, 10, 1, p, R=orc.random_rotation(64, 1), queries=Q)
    assert fr.iters_run == 3            # iteration 1 sets the mark, iterations 2 and 3 fail to beat it by tol
    assert all(0.0 <= r["recall"] <= 1.0 for r in fr.trace[:3])
    p2 = orc.FitParams(etr=True, etr_tol=-1.0, probe_frac=0.1)                   # any change counts as improvement
    assert orc.fit(X, 20, 5, 1, p2, R=None, queries=Q).iters_run == 5


def test_sampled_fit_composition(orc):
    from paper_2603_20009_amd import datagen
    X = datagen.mixture(3000, 64, 20, 3, "linear").numpy()
    R = orc.random_rotation(64, 3)
    fr, idx = orc.fit_sampled(X, 16, 5, 7, 0.3, orc.FitParams(), R=R)
    assert len(idx) == 900 and len(set(idx.tolist())) == 900 and (np.diff(idx) > 0).all()
    assert fr.assign.shape == (3000,) and fr.assign.max() < 16
    # the centroids are the means of the sample under its last in-loop assignment: one exact step from them
    # moves every centroid little, and the full assignment is one-sided against the exact nearest centroid
    Xr = orc.rotate(X, R)
    D = brute_dist(Xr, fr.centroids_rot)
    assert (fr.dist >= D.min(1) * (1 - 1e-12)).all() and (fr.dist > D.min(1) * (1 + 1e-9)).mean() < 0.01
    full = orc.fit(X, 16, 5, 7, orc.FitParams(), R=R)
    assert fr.trace[-1]["objective"] == pytest.approx(full.trace[-1]["objective"], rel=0.2)    # similar quality


# ---------------------------------------------------------------- hierarchical fit (Section 6)
def hamilton(sizes, k):
    """Largest-remainder apportionment written independently with exact rational comparisons where possible:
    one seat to every non-empty party, the rest by quota on sqrt(size)."""
    sizes = [int(s) for s in sizes]
    counts = [1 if s > 0 else 0 for s in sizes]
    r = k - sum(counts)
    w = [math.sqrt(s) for s in sizes]
    W = 0.0
    for v in w:
        W += v
    q = [r * v / W for v in w]
    for i, v in enumerate(q):
        counts[i] += min(int(math.floor(v)), sizes[i] - counts[i])
    order = sorted(range(len(sizes)), key=lambda i: (-(q[i] - math.floor(q[i])), i))
    left = k - sum(counts)
    while left > 0:
        moved = False
        for i in order:
            if left > 0 and counts[i] < sizes[i]:
                counts[i] += 1
                left -= 1
                moved = True
        if not moved:
            break
    return counts


def test_hier_counts_closed_forms(orc):
    assert [orc.hier_meso_count(k) for k in (1, 2, 3, 4, 10, 100, 1000, 1024, 16384, 32768)] == \
        [1, 1, 2, 2, 3, 10, 32, 32, 128, 181]
    # equal meso-clusters share k equally; sqrt weighting: sizes 400 : 100 : 25 weigh 4 : 2 : 1
    assert orc.hier_alloc([500] * 8, 64).tolist() == [8] * 8
    assert orc.hier_alloc([400, 100, 0, 25], 10).tolist() == [5, 3, 0, 2]
    # never more clusters than points; what a small meso-cluster cannot take goes to the others
    assert orc.hier_alloc([2, 1000, 3], 12).tolist() == [1, 9, 2]
    assert orc.hier_alloc([1, 1, 1, 97], 50).tolist() == [1, 1, 1, 47]
    assert orc.hier_alloc([5, 5], 10).tolist() == [5, 5]


def test_hier_alloc_against_independent_apportionment(orc):
    rng = np.random.default_rng(5)
    for _ in range(300):
        km = int(rng.integers(1, 40))
        sizes = rng.integers(0, 2000, km) * (rng.random(km) > 0.1)
        if sizes.sum() == 0:
            sizes[0] = 7
        k = int(rng.integers(max(km, 1), max(int(sizes.sum()), km) + 1))
        if k > sizes.sum():
            continue
        got = orc.hier_alloc(sizes, k)
        assert got.sum() == k and (got <= sizes).all() and ((got > 0) == (sizes > 0)).all()
        assert got.tolist() == hamilton(sizes, k)
        # more points never means fewer clusters
        o = np.argsort(sizes, kind="stable")
        assert (np.diff(got[o]) >= -1).all()


def test_hierarchical_fit_composition(orc):
    from paper_2603_20009_amd import datagen
    X = datagen.mixture(4000, 64, 30, 4, "linear").numpy()
    R = orc.random_rotation(64, 4)
    k = 36
    h = orc.fit_hierarchical(X, k, 9, 3, 5, orc.FitParams(eps0=float("inf")), R=R)
    Xr = orc.rotate(X, R)
    km = orc.hier_meso_count(k)
    assert km == 6 and h["meso_sizes"].sum() == 4000 and h["fine_counts"].sum() == k
    assert h["fine_counts"].tolist() == hamilton(h["meso_sizes"], k)
    # with exact Lloyd steps the final assignment is the nearest of all k centroids
    D = brute_dist(Xr, h["centroids_rot"])
    assert (h["assign"] == D.argmin(1)).mean() > 0.9999 and np.allclose(h["dist"], D.min(1), rtol=1e-9, atol=1e-12)
    # block c of the centroids belongs to meso-cluster c: every fine centroid is a mean of some of its points, so
    # it lies inside their bounding box, and the block's centroids, weighted by their member counts, average to the
    # mean of the meso-cluster (Lloyd's update keeps the total sum)
    off = 0
    for c in range(km):
        kc = int(h["fine_counts"][c])
        rows = np.nonzero(h["meso_assign"] == c)[0]
        P = Xr[rows]
        Yc = h["centroids_rot"][off:off + kc]
        assert (Yc >= P.min(0) - 1e-9).all() and (Yc <= P.max(0) + 1e-9).all()
        lab = brute_dist(P, Yc).argmin(1)        # members under the next exact step
        # one more exact step from Yc moves it little: Yc are fixed points up to the 5-iteration budget
        moved = np.stack([P[lab == j].mean(0) if (lab == j).any() else Yc[j] for j in range(kc)])
        assert np.linalg.norm(moved - Yc) / np.linalg.norm(Yc) < 0.2
        off += kc
    # k = 1: one meso-cluster, one fine cluster, the global mean
    one = orc.fit_hierarchical(X, 1, 9, 3, 5, orc.FitParams(), R=R)
    assert np.allclose(one["centroids_rot"][0], Xr.mean(0), atol=1e-9)
    # the unrotated centroids are the rotated ones times R^T
    assert np.allclose(h["centroids"], h["centroids_rot"] @ R.astype(np.float64).T, atol=1e-9)
    # quality: within a modest factor of the flat fit with the same k (the paper reports a small recall loss only)
    flat = orc.fit(X, k, 8, 9, orc.FitParams(), R=R)
    assert h["objective"] < 1.25 * flat.trace[-1]["objective"]


# ---------------------------------------------------------------- angular metric (spherical k-means)
def test_angular_fit_pins(orc):
    from paper_2603_20009_amd import datagen
    rng = np.random.default_rng(8)
    X = datagen.mixture(3000, 48, 25, 6, "linear").numpy() * rng.uniform(0.2, 5.0, (3000, 1)).astype(np.float32)
    R = orc.random_rotation(48, 6)
    k = 12
    fr = orc.fit(X, k, 6, 5, orc.FitParams(eps0=float("inf"), angular=True), R=R)
    U = orc.rotate(X, R)
    U /= np.linalg.norm(U, axis=1, keepdims=True)
    Y = fr.centroids_rot
    # centroids are unit vectors; with exact steps every point sits with the centroid of largest cosine
    assert np.allclose(np.linalg.norm(Y, axis=1), 1.0, atol=1e-12)
    cos = U @ Y.T
    assert (fr.assign == cos.argmax(1)).mean() > 0.9999
    assert np.allclose(fr.dist, 2.0 - 2.0 * cos.max(1), atol=1e-10)
    # a centroid is the direction of the mean of its (unit) members under the last in-loop assignment; after the
    # final pass the members changed little, so the direction of the new mean is close to it
    for c in range(k):
        m = U[fr.assign == c].mean(0)
        assert m @ Y[c] / np.linalg.norm(m) > 0.999
    # only directions matter: rescaling every point changes nothing
    fr2 = orc.fit(X * rng.uniform(0.5, 2.0, (3000, 1)).astype(np.float32), k, 6, 5,
                  orc.FitParams(eps0=float("inf"), angular=True), R=R)
    assert (fr2.assign == fr.assign).mean() > 0.999 and np.allclose(fr2.centroids_rot, Y, atol=1e-5)
    # and it is not the L2 clustering of the raw points
    l2 = orc.fit(X, k, 6, 5, orc.FitParams(eps0=float("inf")), R=R)
    assert (l2.assign != fr.assign).mean() > 0.05
    # pruning on: same trajectory up to the rare false prune
    pr = orc.fit(X, k, 6, 5, orc.FitParams(angular=True), R=R)
    assert (pr.assign == fr.assign).mean() > 0.995
