"""Acceptance rules shared by the GPU parity tests (comparison only, no method arithmetic)."""
import numpy as np

EPS0 = float(np.float32(2.1))   # the library stores eps0 as fp32; the oracle is given the same value


def sqdist(Xr, Y, idx):
    diff = np.asarray(Xr, dtype=np.float64) - np.asarray(Y, dtype=np.float64)[idx]
    return np.einsum("ij,ij->i", diff, diff)


def check_assignment(a_gpu, a_ref, Xr, Y, min_agree=0.999, gap=1e-4, own=None, max_far=None):
    """>= 99.9 % of the assignments agree, and wherever they differ the two centroids are a
    near-tie for that point: their fp64 distances differ by at most 1e-4 relative.

    For a fit of several iterations pass own = (X, Y_gpu), the library's input points and final centroids in
    one space.  A near-tie that falls the other way in some iteration is allowed, but it moves a point between
    two clusters, so the later centroids of the two runs differ slightly and a few points near a boundary may
    end on different sides without being near-ties under the reference centroids.  Such a point passes if the
    library's label is the nearest of the library's own centroids (to the same 1e-4): both runs are then
    valid Lloyd trajectories that split at a tie.  max_far bounds how many points may need that second rule
    (None: no bound); single steps never pass `own`, so for them every disagreement must be a near-tie."""
    a_gpu = np.asarray(a_gpu)
    a_ref = np.asarray(a_ref)
    assert a_gpu.shape == a_ref.shape
    diff = np.nonzero(a_gpu != a_ref)[0]
    agree = 1.0 - len(diff) / max(len(a_ref), 1)
    assert agree >= min_agree, f"agreement {agree:.6f} < {min_agree}"
    n_far = n_own = 0
    if len(diff):
        Xd = np.asarray(Xr, dtype=np.float64)[diff]
        dg = sqdist(Xd, Y, a_gpu[diff])
        dr = sqdist(Xd, Y, a_ref[diff])
        rel = np.abs(dg - dr) / np.maximum(np.minimum(dg, dr), 1e-300)
        bad = rel > gap
        n_far = int(bad.sum())
        if own is not None and bad.any():
            Xo = np.asarray(own[0], dtype=np.float64)[diff[bad]]
            Yo = np.asarray(own[1], dtype=np.float64)
            d_all = (Xo * Xo).sum(1)[:, None] - 2.0 * Xo @ Yo.T + (Yo * Yo).sum(1)[None, :]
            d_lab = sqdist(Xo, Yo, a_gpu[diff[bad]])
            valid = d_lab <= d_all.min(1) * (1.0 + gap) + 1e-12
            n_own = int(valid.sum())
            bad[np.nonzero(bad)[0][valid]] = False
        # what the run relied on: every fit prints how many of its disagreements needed the second rule
        print(f"parity: {len(a_ref)} points, {len(diff)} disagree, {n_far} of them no near-tie under the reference "
              f"centroids, {n_own} of those accepted as nearest under the library's own centroids", flush=True)
        assert not bad.any(), (f"disagreement that is no near-tie: rel gap {rel[bad].max():.3e} "
                               f"at point {diff[bad][rel[bad].argmax()]}")
        if max_far is not None:
            assert n_far <= max_far, f"{n_far} disagreements are no near-ties (at most {max_far} expected)"
    return agree


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def check_centroids(Yg, Yr, a_gpu, a_ref, tol=1e-3, min_clean=0.97):
    """Centroids agree to `tol` (relative L2).  If the two runs split at a near-tie (see check_assignment), the
    clusters that exchanged points have different members and therefore different means; the bound is then
    asserted over the clusters whose member sets are identical, which must be at least `min_clean` of all.
    Returns the indices of those clusters."""
    a_gpu = np.asarray(a_gpu)
    a_ref = np.asarray(a_ref)
    if (a_gpu == a_ref).all():
        assert rel_l2(Yg, Yr) < tol
        return np.arange(len(Yr))
    touched = np.union1d(a_gpu[a_gpu != a_ref], a_ref[a_gpu != a_ref])
    clean = np.setdiff1d(np.arange(len(Yr)), touched)
    print(f"parity: {len(touched)} of {len(Yr)} clusters exchanged points between the two runs; all centroids "
          f"rel L2 {rel_l2(Yg, Yr):.2e}, clusters with the same members {rel_l2(np.asarray(Yg)[clean], np.asarray(Yr)[clean]):.2e}",
          flush=True)
    # one split at a near-tie touches two clusters, and the two that pass a point on at the next boundary: a handful
    assert len(clean) >= min_clean * len(Yr) or len(touched) <= 4, \
        f"only {len(clean)} of {len(Yr)} clusters have the same members"
    assert rel_l2(np.asarray(Yg)[clean], np.asarray(Yr)[clean]) < tol
    return clean
