"""Parity metrics shared by the oracle pins and the GPU parity tests.

Nothing here is part of the method; it only measures how far two
decompositions are apart in a way that is well posed when singular values
repeat or cluster (then only the spanned subspace is unique).
"""
import numpy as np

EPS = {"f32": float(np.finfo(np.float32).eps), "f64": float(np.finfo(np.float64).eps)}
# spec tolerances
SV_RTOL = {"f32": 1e-3, "f64": 1e-5}
ANGLE_TOL = {"f32": 1e-2, "f64": 1e-4}
GAP_MIN = {"f32": 1e-2, "f64": 1e-4}


def orthonormal_basis(X):
    q, _ = np.linalg.qr(np.asarray(X, dtype=np.float64), mode="reduced")
    return q


def sin_theta(Ua, Ub):
    """Largest principal-angle sine between range(Ua) and range(Ub) (same dimension).

    Both are re-orthonormalised first so a slightly non-orthonormal input does
    not leak into the angle."""
    Qa, Qb = orthonormal_basis(Ua), orthonormal_basis(Ub)
    R = Qb - Qa @ (Qa.T @ Qb)
    return float(np.linalg.norm(R, 2))


def clusters(sig, gap_min, k):
    """Split the indices of `sig` (descending) into maximal runs of consecutive
    singular values whose relative gaps are below gap_min; return the runs that
    start before index k as (begin, end) pairs.  With `sig` holding all l
    values, a run that reaches past k is a cluster straddling the truncation."""
    sig = np.asarray(sig, dtype=np.float64)
    runs, start = [], 0
    for i in range(len(sig) - 1):
        gap = (sig[i] - sig[i + 1]) / sig[i] if sig[i] > 0 else 0.0
        if gap >= gap_min:
            runs.append((start, i + 1))
            start = i + 1
    runs.append((start, len(sig)))
    return [r for r in runs if r[0] < k]


ABS_C = 10.0     # a backward-stable SVD returns each singular value to within ~ABS_C * eps * sigma_1


def significant(sig, dtype, m=None, n=None):
    """Mask of singular values that can be held to the relative tolerance.

    Any SVD computed in precision eps delivers singular values with an ABSOLUTE
    error of order eps * sigma_1, so a relative error SV_RTOL is attainable only
    for sigma_i >= (ABS_C * eps / SV_RTOL) * sigma_1.  Values below that are
    compared absolutely, to ABS_C * eps * sigma_1 times sqrt(max(m, n)) (the
    growth of accumulated rounding in dot products of that length)."""
    sig = np.asarray(sig, dtype=np.float64)
    return sig > (ABS_C * EPS[dtype] / SV_RTOL[dtype]) * sig[0]


def jacobi_tol(l, dtype):
    """Frobenius-norm bound for orthogonality defects and residuals of vectors that
    went through the Jacobi SVD: every column is hit by about l rotations per sweep
    for a handful of sweeps, each adding one rounding error, so a single inner
    product drifts by ~sqrt(l * sweeps) * eps and the l x l Frobenius norm by l
    times that.  8 * l^1.5 * eps covers up to ~16 sweeps with a factor 2 to spare."""
    return 8.0 * float(l) ** 1.5 * EPS[dtype]


def orthonormality(Q):
    Q = np.asarray(Q, dtype=np.float64)
    return float(np.linalg.norm(Q.T @ Q - np.eye(Q.shape[1])))


def check_triplets(S_g, U_g, Vt_g, S_o, U_o, Vt_o, dtype, m, n,
                   S_all_o=None, U_all_o=None, Vt_all_o=None,
                   S_all_g=None, U_all_g=None, Vt_all_g=None):
    """Compare k triplets from the HIP path (g) with the oracle's (o).

    Returns a dict of measured quantities; raises AssertionError on a miss.
    When the untruncated l triplets of both sides are given, a cluster that
    straddles index k is compared over its full extent; otherwise such a
    trailing cluster is compared on singular values only.
    """
    k = len(S_o)
    S_g = np.asarray(S_g, dtype=np.float64)
    S_o = np.asarray(S_o, dtype=np.float64)
    sig_mask = significant(S_o, dtype, m, n)
    rel = np.abs(S_g - S_o)[sig_mask] / S_o[sig_mask]
    out = {"sv_rel_max": float(rel.max()) if rel.size else 0.0}
    assert out["sv_rel_max"] <= SV_RTOL[dtype], f"singular values off: {out['sv_rel_max']:.3e}"
    insig = ~sig_mask
    if insig.any():
        absd = np.abs(S_g - S_o)[insig].max()
        out["sv_abs_insig"] = float(absd)
        assert absd <= ABS_C * EPS[dtype] * S_o[0] * np.sqrt(max(m, n))

    have_all = S_all_o is not None and U_all_g is not None
    ref = S_all_o if have_all else S_o
    runs = clusters(ref, GAP_MIN[dtype], k)
    worst_u = worst_v = 0.0
    skipped = []
    for (a, b) in runs:
        if not significant(ref, dtype, m, n)[a:b].all():
            skipped.append((a, b, "below rank threshold"))
            continue
        if not have_all and b == k:
            skipped.append((a, b, "may straddle k (untruncated triplets not given)"))
            continue
        if b > k:
            Uo, Ug = U_all_o[:, a:b], U_all_g[:, a:b]
            Vo, Vg = Vt_all_o[a:b].T, Vt_all_g[a:b].T
        else:
            Uo, Ug = np.asarray(U_o)[:, a:b], np.asarray(U_g)[:, a:b]
            Vo, Vg = np.asarray(Vt_o)[a:b].T, np.asarray(Vt_g)[a:b].T
        worst_u = max(worst_u, sin_theta(Uo, Ug))
        worst_v = max(worst_v, sin_theta(Vo, Vg))
    out.update(sin_u=worst_u, sin_v=worst_v, clusters=len(runs), skipped=skipped)
    assert worst_u <= ANGLE_TOL[dtype], f"left vectors off: sin={worst_u:.3e}"
    assert worst_v <= ANGLE_TOL[dtype], f"right vectors off: sin={worst_v:.3e}"
    return out
