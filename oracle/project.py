"""CPU oracle for the two projections of a tentative perturbation onto the verifier's admissible
sets (Sec. 4.4) -- TEST INFRASTRUCTURE, numpy only, the steps in the paper's order.

(i)  theoretical bounds: element-wise clip to [-alpha tau, alpha tau];
(ii) empirical thresholds: sort |delta| increasingly, cap the k-th order statistic by the cap curve
     of Sec. 4.2 at the rank (k - 1/2)/n, after a running maximum over k, restore sign and shape.

Readings the paper leaves open (the GPU library documents the same ones):
  * the cap curve goes through (0, 0) and (p_j, alpha thr_j) for the 22 grid points (the last is
    p = 100); between knots, in binary64 and in this order,
        r = ((k - 0.5) / n) * 100,   j = first knot with r <= p_j,
        C = c_{j-1} + (c_j - c_{j-1}) * ((r - p_{j-1}) / (p_j - p_{j-1}));
  * equal magnitudes keep their index order (stable sort), so every element's rank is unique;
  * a clipped element takes the largest binary32 value not above its cap, so the result never
    leaves the admissible set through rounding; NaN elements sort last and stay NaN.
"""
import numpy as np

GRID_PERCENT = np.array([1] + [5 * g for g in range(1, 20)] + [99, 100], dtype=np.float64)


def _f32_not_above(c):
    """Largest binary32 value <= c, for binary64 c >= 0."""
    with np.errstate(over="ignore"):
        f = c.astype(np.float32)                             # beyond the binary32 range: inf, stepped down below
    over = f.astype(np.float64) > c
    return np.where(over, np.nextafter(f, np.float32(-np.inf), dtype=np.float32), f).astype(np.float32)


def project_clip(delta, tau, alpha=1.0):
    """Eq. of Sec. 4.4 (i): clip(delta, -alpha tau, alpha tau), the product alpha tau in binary64."""
    delta = np.ascontiguousarray(delta, dtype=np.float32)
    tau = np.ascontiguousarray(tau, dtype=np.float32)
    if delta.shape != tau.shape:
        raise ValueError("delta and tau differ in shape")
    if not (np.isfinite(alpha) and alpha >= 0):
        raise ValueError("alpha must be finite and non-negative")
    a = np.abs(delta)
    cap = tau.astype(np.float64) * np.float64(alpha)
    clipped = a.astype(np.float64) > cap                     # false for NaN: those stay
    out = np.where(clipped, _f32_not_above(cap), a)
    return np.copysign(out, delta).astype(np.float32)


def cap_curve(ranks, n, thr_abs, alpha=1.0):
    """C(r_k) for the 1-based ranks k (before the running maximum)."""
    c = np.concatenate([[0.0], np.asarray(thr_abs, dtype=np.float32).astype(np.float64) * np.float64(alpha)])
    p = np.concatenate([[0.0], GRID_PERCENT])
    k = np.asarray(ranks, dtype=np.float64)
    r = ((k - 0.5) / np.float64(n)) * 100.0
    j = np.searchsorted(p, r, side="left")                   # first knot with r <= p_j
    j = np.clip(j, 1, len(p) - 1)
    t = (r - p[j - 1]) / (p[j] - p[j - 1])
    return c[j - 1] + (c[j] - c[j - 1]) * t


def project_empirical(delta, thr_abs, alpha=1.0):
    """Sec. 4.4 (ii).  delta: any shape, binary32; thr_abs: the operator's 22 absolute-error
    thresholds (Sec. 3.2), finite and non-negative."""
    delta = np.ascontiguousarray(delta, dtype=np.float32)
    thr_abs = np.asarray(thr_abs, dtype=np.float32)
    if thr_abs.shape != (len(GRID_PERCENT),):
        raise ValueError("22 thresholds expected")
    if not (np.all(np.isfinite(thr_abs)) and np.all(thr_abs >= 0)):
        raise ValueError("thresholds must be finite and non-negative")
    if not (np.isfinite(alpha) and alpha >= 0):
        raise ValueError("alpha must be finite and non-negative")
    flat = delta.reshape(-1)
    n = flat.size
    if n == 0:
        return delta.copy()
    a = np.abs(flat)
    sigma = np.argsort(a, kind="stable")                     # NaN last
    caps = cap_curve(np.arange(1, n + 1), n, thr_abs, alpha)
    caps = np.maximum.accumulate(caps)                       # c_k <- max(c_k, c_{k-1})
    a_sorted = a[sigma]
    clipped = a_sorted.astype(np.float64) > caps
    star_sorted = np.where(clipped, _f32_not_above(caps), a_sorted)
    star = np.empty(n, dtype=np.float32)
    star[sigma] = star_sorted
    return np.copysign(star, flat).astype(np.float32).reshape(delta.shape)
