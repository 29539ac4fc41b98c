"""CPU checker for the partially-linear FFN hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what the method computes, written from
the paper (arXiv 2501.10054) so that a reader can check it against the text by
eye.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may
import this file; the GPU library never does, and this file imports nothing
from the GPU library.

Orientation.  The paper writes row vectors, FFN(x) = sigma(x W1) W2 with W1 of
size d x h (Sec. "Opportunity").  Here tokens are column vectors and the weight
arrays are the transposes, the layout a Linear layer stores:

    W1 : h x d   (row j  = neuron j's input weights,  paper W1[:, j])
    W2 : d x h   (col j  = neuron j's output weights, paper W2[j, :])
    FFN(x) = W2 . sigma(W1 x + b1) + b2

so the paper's folded matrix C is W'^T and its folded bias B is b'^T.  Paper
symbols (a, b) for slope and intercept are (a_j, c_j) here because b1/b2 name
the layer biases; the paper's range [l1, l2) is [lo_j, hi_j).

Every floating-point step is fp64 unless a comment says the value is rounded to
fp32 because the library interface carries it as fp32.

Pins (tests/test_oracle_pins.py): the paper's printed two-neuron example, its
2x2 folding example, the standard normal CDF table for GELU, closed forms for
the least-squares fit, a literal per-neuron rank-1 fold, brute-force integer
dot products, hand-worked 4-bit group codes, the reconstruction error bound of
both sketches, and the all-flagged / none-flagged identities.

parity unpinned: kde_centroid / range_search (the paper prints no worked
example of its range search and leaves the density estimate, the error
aggregation and the end of the growth loop open; they are pinned only by an
independent brute-force re-implementation and by invariants).  Nothing on the
gated path.  (The integer predictor below is a
reading of "a quantised copy of W1", Sec. "Predictor Generation"; the paper
prints no numbers for it, so it is pinned by brute force and by the printed
example's flag set, not by a published value.)
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
from scipy.special import erf as _erf

ACTS = ("gelu_erf", "gelu_tanh", "relu", "identity")


# ---------------------------------------------------------------------------
# activation  (Sec. "Opportunity": sigma between the two weight matrices)
# ---------------------------------------------------------------------------
def act(z, kind: str = "gelu_erf"):
    """sigma(z).  GELU is z * Phi(z) with Phi the standard normal CDF; the tanh
    form is the usual approximation of it; ReLU is max(z, 0)."""
    z = np.asarray(z, dtype=np.float64)
    if kind == "gelu_erf":
        return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))
    if kind == "gelu_tanh":
        return 0.5 * z * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z ** 3)))
    if kind == "relu":
        return np.maximum(z, 0.0)
    if kind == "identity":
        return z.copy()
    raise ValueError(kind)


def _f64(x):
    return None if x is None else np.asarray(x, dtype=np.float64)


def preact(W1, b1, X):
    """z = W1 x + b1 for every row x of X (n x d) -> n x h.  The activation
    input of each neuron (Sec. "Non-linear Function Approximation", step 1)."""
    Z = _f64(X) @ _f64(W1).T
    if b1 is not None:
        Z = Z + _f64(b1)[None, :]
    return Z


# ---------------------------------------------------------------------------
# dense FFN  (Sec. "Opportunity", FFN(x) = sigma(x W1) W2)
# ---------------------------------------------------------------------------
def dense(W1, b1, W2, b2, X, kind: str = "gelu_erf"):
    """Exact FFN for every row of X (n x d) -> n x d."""
    Y = act(preact(W1, b1, X), kind) @ _f64(W2).T
    if b2 is not None:
        Y = Y + _f64(b2)[None, :]
    return Y


# ---------------------------------------------------------------------------
# calibration  (Sec. "Insights" 2 and Sec. "Non-linear Function Approximation":
# a range holding a portion t of the calibration inputs, then a least-squares
# line through sigma on that range)
# ---------------------------------------------------------------------------
def quantile_linear(sorted_vals: np.ndarray, q: float) -> float:
    """Quantile by linear interpolation between order statistics at position
    q*(N-1)."""
    n = sorted_vals.shape[0]
    pos = q * (n - 1)
    i = int(math.floor(pos))
    i = min(max(i, 0), n - 1)
    g = pos - i
    i1 = min(i + 1, n - 1)
    return float(sorted_vals[i] + g * (sorted_vals[i1] - sorted_vals[i]))


def fit_line(z: np.ndarray, g: np.ndarray, fallback_point: float, kind: str):
    """Ordinary least squares of g on z: slope cov(z,g)/var(z), intercept
    mean(g) - slope*mean(z).  Degenerate sets (fewer than two samples, or all z
    equal) give slope 0 and the mean of g (sigma at the range's left end if
    there is no sample at all)."""
    n = z.shape[0]
    if n == 0:
        return 0.0, float(act(fallback_point, kind))
    zbar = z.mean()
    gbar = g.mean()
    var = ((z - zbar) ** 2).sum()
    if n < 2 or var <= 0.0:
        return 0.0, float(gbar)
    cov = ((z - zbar) * (g - gbar)).sum()
    a = cov / var
    return float(a), float(gbar - a * zbar)


def calibrate(W1, b1, X_cal, coverage, kind: str = "gelu_erf"):
    """Per neuron: [lo, hi) = central `coverage` quantile range of its
    calibration pre-activations, (a, c) = least-squares line through sigma over
    the calibration samples with lo <= z < hi.

    `coverage` is a scalar t or an array of h per-neuron values.  lo and hi are
    rounded to fp32 (the interface carries them as fp32) *before* the in-range
    test that selects the fit samples.  Returns four float32 arrays of length h.
    """
    Z = preact(W1, b1, X_cal)                      # n x h
    n, h = Z.shape
    t = np.broadcast_to(np.asarray(coverage, dtype=np.float64), (h,))
    lo = np.empty(h, np.float32)
    hi = np.empty(h, np.float32)
    a = np.empty(h, np.float32)
    c = np.empty(h, np.float32)
    for j in range(h):
        zj = Z[:, j]
        zs = np.sort(zj)
        lo[j] = np.float32(quantile_linear(zs, (1.0 - t[j]) / 2.0))
        hi[j] = np.float32(quantile_linear(zs, (1.0 + t[j]) / 2.0))
        sel = (zj >= np.float64(lo[j])) & (zj < np.float64(hi[j]))
        aj, cj = fit_line(zj[sel], act(zj[sel], kind), float(lo[j]), kind)
        a[j] = np.float32(aj)
        c[j] = np.float32(cj)
    return lo, hi, a, c


# ---------------------------------------------------------------------------
# range search  (Sec. "Non-linear Function Approximation", paragraph "Range
# Searching" and the inner loop of Algorithm 1: start at the centroid of the
# neuron's input distribution, grow the range by a step s to the left or to
# the right, whichever candidate is approximated with the smaller error, until
# the range holds the portion t of the calibration inputs)
# ---------------------------------------------------------------------------
KDE_GRID = 256            # points at which the density estimate is evaluated


def kde_centroid(zs: np.ndarray) -> float:
    """Mode of a Gaussian kernel density estimate of the samples `zs` (sorted).

    The paper names kernel density estimation and nothing more.  Reading:
    Gaussian kernel, bandwidth 1.06 * std * N^(-1/5) (std with N-1 in the
    denominator), density evaluated at KDE_GRID equally spaced points from the
    smallest to the largest sample (both included); the centroid is the grid
    point of largest density, the leftmost one among equals.  All samples equal
    (or one sample): that value.
    """
    n = zs.shape[0]
    zmin, zmax = float(zs[0]), float(zs[-1])
    if n < 2 or not zmax > zmin:
        return zmin
    mean = zs.sum() / n
    std = math.sqrt(((zs - mean) ** 2).sum() / (n - 1))
    bw = 1.06 * std * n ** (-0.2)
    grid = zmin + np.arange(KDE_GRID) * ((zmax - zmin) / (KDE_GRID - 1))
    u = (grid[:, None] - zs[None, :]) / bw
    dens = np.exp(-0.5 * u * u).sum(axis=1)
    return float(grid[int(np.argmax(dens))])       # argmax returns the first maximum


def approx_error(z_in: np.ndarray, kind: str) -> float:
    """Error of approximating sigma by its least-squares line over the samples
    `z_in` of a candidate range: the sum over the samples of |sigma(z) - (a z + c)|
    (the per-input L2 distance err_n(x) of one neuron's contribution, without the
    factor ||W2[:, n]|| that both candidates of a step share)."""
    if z_in.shape[0] == 0:
        return 0.0
    g = act(z_in, kind)
    a, c = fit_line(z_in, g, 0.0, kind)
    return float(np.abs(g - (a * z_in + c)).sum())


def range_search(z: np.ndarray, t: float, step: float, kind: str = "gelu_erf", centroid=None, trace=None):
    """Greedy range of one neuron.  Returns (lo, hi) in fp64.

    R = [centroid, centroid); while the portion of the samples with lo <= z < hi
    is below t: the two candidates are (lo - s, hi) and (lo, hi + s); the one
    with the smaller approx_error is taken, the right one when they are equal.
    Readings where the listing is silent or garbled: both candidates keep the
    other end of R; a side whose end already lies beyond every sample (lo <=
    min z, resp. hi > max z) is not offered again - the listing would otherwise
    keep choosing an extension that adds no sample and never end.  With that
    rule the loop ends by itself after at most (max z - min z) / s + 2 steps:
    there is no step limit.

    `centroid`: start there instead of at the density estimate's mode (for
    worked examples).  `trace`: a list that receives one tuple per growth step,
    (side taken 'L'/'R', e_l, e_r, gap) - the two candidates' errors (None when
    only one side was on offer) and the distance from the nearest sample to the
    nearest of the ends lo, hi, lo - s, hi + s that the step's tests compare
    samples with: a step whose errors nearly agree, or whose ends nearly touch a
    sample, is one that rounding of the inputs may decide the other way.
    """
    zs = np.sort(_f64(z))
    n = zs.shape[0]
    lo = hi = kde_centroid(zs) if centroid is None else float(centroid)
    zmin, zmax = float(zs[0]), float(zs[-1])
    while True:
        inside = (zs >= lo) & (zs < hi)
        if inside.sum() / n >= t:
            return lo, hi
        left_open, right_open = lo > zmin, not hi > zmax
        if not left_open and not right_open:
            return lo, hi
        e_l = e_r = None
        if left_open and right_open:
            e_l = approx_error(zs[(zs >= lo - step) & (zs < hi)], kind)
            e_r = approx_error(zs[(zs >= lo) & (zs < hi + step)], kind)
            go_left = e_l < e_r
        else:
            go_left = left_open
        if trace is not None:
            ends = np.array([lo, hi, lo - step, hi + step])
            trace.append(("L" if go_left else "R", e_l, e_r, float(np.abs(zs[:, None] - ends[None, :]).min())))
        if go_left:
            lo = lo - step
        else:
            hi = hi + step


def calibrate_search(W1, b1, X_cal, coverage, step, kind: str = "gelu_erf"):
    """As `calibrate`, with the range of every neuron found by `range_search`
    instead of central quantiles.  Returns four float32 arrays of length h."""
    Z = preact(W1, b1, X_cal)
    n, h = Z.shape
    t = np.broadcast_to(np.asarray(coverage, dtype=np.float64), (h,))
    lo = np.empty(h, np.float32)
    hi = np.empty(h, np.float32)
    a = np.empty(h, np.float32)
    c = np.empty(h, np.float32)
    for j in range(h):
        zj = Z[:, j]
        l, r = range_search(zj, float(t[j]), float(step), kind)
        lo[j] = np.float32(l)
        hi[j] = np.float32(r)
        sel = (zj >= np.float64(lo[j])) & (zj < np.float64(hi[j]))
        aj, cj = fit_line(zj[sel], act(zj[sel], kind), float(lo[j]), kind)
        a[j] = np.float32(aj)
        c[j] = np.float32(cj)
    return lo, hi, a, c


# ---------------------------------------------------------------------------
# adaptive thresholding  (Sec. "Non-linear Function Approximation", "Adaptive
# Thresholding"; the two error_aware_threshold calls and the two estimate_error
# calls of Algorithm 1)
# ---------------------------------------------------------------------------
def neuron_errors(W1, b1, W2, X_cal, lo, hi, a, c, kind: str = "gelu_erf"):
    """Empirical error of every neuron over the calibration inputs,
        E_n = sum_x err_n(x),
        err_n(x) = || sigma(z_n) W2[:, n] - phi_n(z_n) W2[:, n] ||_2
                 = |sigma(z_n) - (a_n z_n + c_n)| * ||W2[:, n]||_2   if lo_n <= z_n < hi_n, else 0
    (the per-neuron error metric of the section; phi_n equals sigma outside the
    range).  Returns fp64[h].  The layer's error is the sum over its neurons
    (err(x) = sum_n err_n(x))."""
    Z = preact(W1, b1, X_cal)
    lo = _f64(lo); hi = _f64(hi); a = _f64(a); c = _f64(c)
    inside = (Z >= lo[None, :]) & (Z < hi[None, :])
    resid = np.abs(act(Z, kind) - (Z * a[None, :] + c[None, :]))
    colnorm = np.sqrt((_f64(W2) ** 2).sum(axis=0))
    return (resid * inside).sum(axis=0) * colnorm


def error_aware_threshold(E, t: float, t_min: float, t_max: float):
    """Thresholds t_i for items (layers, or the neurons of a layer) with errors E_i:
        minimise sum_i E_i t_i   subject to   sum_i t_i = t * n,   t_min <= t_i <= t_max.
    The section prints the objective and the equality only; a linear objective
    under one equality has no minimum without bounds, so the caller supplies them
    (reading; 0 <= t_min <= t <= t_max <= 1).  The solution of this linear
    programme is the greedy one: the items with the largest errors sit at t_min,
    the others at t_max, and at most one item in between takes what is left of the
    budget.  Items of equal error are ordered by index (lower index first).
    Returns fp32[n]."""
    E = _f64(E)
    n = E.shape[0]
    t, t_min, t_max = float(t), float(t_min), float(t_max)
    if not (t_min <= t <= t_max):
        raise ValueError("need t_min <= t <= t_max")
    out = np.full(n, t_max, np.float64)
    if t_max > t_min:
        width = t_max - t_min
        excess = n * t_max - t * n                 # what has to be taken away from "everybody at t_max"
        k = int(math.floor(excess / width))
        k = min(k, n)
        order = sorted(range(n), key=lambda i: (-E[i], i))
        for r in range(k):
            out[order[r]] = t_min
        if k < n:
            out[order[k]] = t_max - (excess - k * width)
    return out.astype(np.float32)


# ---------------------------------------------------------------------------
# constant folding  (Sec. "Constant Folded Matrix Generation")
# ---------------------------------------------------------------------------
def fold(W1, b1, W2, b2, a, c):
    """W' = W2 diag(a) W1 (d x d),  b' = W2 (c + a*b1) + b2 (d).

    This is the sum over neurons of the per-neuron folded pair
    (a_n W1[:,n] W2[n,:], b_n W2[n,:]) in the paper's orientation, transposed,
    with the layer biases (which the paper sets to zero for presentation)
    carried through: a_j (W1[j].x + b1_j) + c_j = a_j W1[j].x + (c_j + a_j b1_j).
    """
    W1 = _f64(W1); W2 = _f64(W2); a = _f64(a); c = _f64(c)
    Wp = (W2 * a[None, :]) @ W1
    k = c if b1 is None else c + a * _f64(b1)
    bp = W2 @ k
    if b2 is not None:
        bp = bp + _f64(b2)
    return Wp, bp


# ---------------------------------------------------------------------------
# 8-bit floating-point storage of the folded matrix  (Sec. "Discussion": the
# method composes with weight compression; here the compressed thing is W')
# ---------------------------------------------------------------------------
def e4m3_values():
    """The 254 finite values of the 8-bit float with 4 exponent bits (bias 7) and 3
    mantissa bits, no infinities, one NaN pattern per sign (S.1111.111): byte b has
    sign b >> 7, exponent field e = (b >> 3) & 15, mantissa m = b & 7 and the value
    (-1)^s 2^(e-7) (1 + m/8) for e >= 1, (-1)^s 2^(-6) m/8 for e = 0.  Largest: 448.
    Returns fp64[256] indexed by the byte (NaN at 0x7F and 0xFF)."""
    out = np.empty(256)
    for b in range(256):
        sgn = -1.0 if b & 0x80 else 1.0
        e, m = (b >> 3) & 15, b & 7
        if e == 15 and m == 7:
            out[b] = np.nan
        elif e == 0:
            out[b] = sgn * 2.0 ** -6 * (m / 8.0)
        else:
            out[b] = sgn * 2.0 ** (e - 7) * (1.0 + m / 8.0)
    return out


def round_e4m3(x):
    """Nearest e4m3 value of every element (ties to the even mantissa), magnitudes
    above 448 saturate to 448.  Returns (codes uint8, values fp64)."""
    x = _f64(x)
    tab = e4m3_values()[:127]                      # non-negative finite values, ascending with the byte
    mag = np.minimum(np.abs(x), 448.0)
    hi = np.searchsorted(tab, mag, side="left").clip(1, 126)
    lo = hi - 1
    dlo, dhi = mag - tab[lo], tab[hi] - mag
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (hi % 2 == 0))      # even byte = even mantissa bit
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    code = np.where(mag == 0.0, 0, code).astype(np.uint8)
    neg = np.signbit(x) & (code != 0)
    val = np.where(neg, -tab[code], tab[code])
    return (code | (neg.astype(np.uint8) << 7)).astype(np.uint8), val


def fp8_rows(Wp):
    """W' as stored with 8-bit floats: every row i gets a power-of-two scale 2^e_i, the
    smallest with max_k |W'_ik| / 2^e_i <= 448, and its elements are rounded to
    e4m3 in that scale.  A power of two, so that the stored value code * 2^e_i is
    also a bfloat16 number and every path of the library multiplies the same
    matrix.  Returns (values fp64 d x d, codes uint8 d x d, exponents int d)."""
    Wp = _f64(Wp)
    mx = np.abs(Wp).max(axis=1)
    e = np.zeros(Wp.shape[0], np.int64)
    nz = mx > 0.0
    e[nz] = np.ceil(np.log2(mx[nz] / 448.0)).astype(np.int64)
    # log2 may land a hair on the wrong side of an exact power of two: fix up by the definition
    for i in np.flatnonzero(nz):
        while mx[i] / 2.0 ** e[i] > 448.0:
            e[i] += 1
        while mx[i] / 2.0 ** (e[i] - 1) <= 448.0:
            e[i] -= 1
    scale = 2.0 ** e.astype(np.float64)
    code, val = round_e4m3(Wp / scale[:, None])
    return val * scale[:, None], code, e


# ---------------------------------------------------------------------------
# predictor  (Sec. "Predictor Generation": a quantised copy of W1 that is just
# good enough to tell which neurons leave their range)
# ---------------------------------------------------------------------------
@dataclass
class Sketch:
    Q: np.ndarray      # h x d int8 codes of W1: W1[j] ~ s[j] * Q[j]
    s: np.ndarray      # h fp64 row scales
    tlo: np.ndarray    # h fp32, (lo - b1) / s
    thi: np.ndarray    # h fp32, (hi - b1) / s
    bits: int = 8
    group: int = 0     # columns per group (4-bit sketch), 0 for the ungrouped 8-bit sketch
    m: np.ndarray | None = None   # h x ceil(d/group) uint8 group multipliers (4-bit sketch)
    q4: np.ndarray | None = None  # h x d int8 low-bit codes (in [-7, 7] for 4 bits); Q = m (per group) * q4


SKETCH_MMAX = 15       # largest group multiplier (4 bits, 1..15)
SKETCH_GROUP = 32      # consecutive columns that share one multiplier


def _thresholds(lo, hi, b, s):
    """Range bounds in sketch units, rounded once to fp32.  A neuron whose weights
    are all zero (s = 0) has z = b1_j for every token: it is never flagged if
    b1_j lies in its range and always otherwise."""
    h = s.shape[0]
    tlo = np.empty(h, np.float32)
    thi = np.empty(h, np.float32)
    for j in range(h):
        if s[j] > 0.0:
            tlo[j] = np.float32((lo[j] - b[j]) / s[j])
            thi[j] = np.float32((hi[j] - b[j]) / s[j])
        elif lo[j] <= b[j] < hi[j]:
            tlo[j] = -np.inf
            thi[j] = np.inf
        else:                       # empty interval: the neuron is always flagged
            tlo[j] = np.inf
            thi[j] = np.inf
    return tlo, thi


def sketch(W1, b1, lo, hi, bits: int = 8, margin: float = 0.0) -> Sketch:
    """Integer sketch of W1 (the "quantised copy of W1" of Sec. "Predictor
    Generation", round-to-nearest) and the range bounds in sketch units.

    bits = 8:  s_j = max_k |W1[j,k]| / 127 ; q_jk = rint(W1[j,k] / s_j) (ties to
    even), clamped to [-127, 127].

    bits = 4:  the row is cut into groups of 32 consecutive columns (the last one
    may be shorter).  With g_jG = max_{k in G} |W1[j,k]| and r_j = max_G g_jG,
        s_j  = r_j / (7 * 15)
        m_jG = ceil(g_jG / (7 s_j))  clamped to [1, 15]        (4-bit multiplier)
        q_jk = rint(W1[j,k] / (m_jG s_j))  clamped to [-7, 7]  (4-bit code)
    and the code the predictor multiplies with is the integer Q_jk = m_jG q_jk
    (|Q_jk| <= 105), so that W1[j,k] ~ s_j Q_jk exactly as in the 8-bit case and
    the dot product stays one exact integer sum.  Storage: 4 bits per weight plus
    4 bits per group of 32.

    bits = 3, 2 (the predictor-width study of Sec. "Predictor Size"): the same
    grouped form with the largest code 2^(bits-1) - 1 in place of 7.

    margin (0 <= margin < 0.5; not in the paper, which only names a quantised
    W1): the predictor tests against the range narrowed by that fraction of its
    width at either end, [lo + margin (hi - lo), hi - margin (hi - lo)): more
    neurons are flagged - and then repaired exactly - so fewer out-of-range
    neurons slip through a coarse sketch.

    Either way the test lo <= s_j*(Q_j . x) + b1_j < hi becomes
    tlo_j <= Q_j . x < thi_j with tlo = (lo-b1)/s, thi = (hi-b1)/s.
    """
    W1 = _f64(W1)
    h, d = W1.shape
    lo = _f64(lo); hi = _f64(hi)
    if margin > 0.0:
        w = hi - lo
        ok = (w > 0.0) & np.isfinite(w)
        mu = float(np.float32(margin))             # the interface carries fp32
        w_ok = np.where(ok, w, 0.0)                # (an empty or unbounded range is left as it is)
        lo, hi = np.where(ok, lo + mu * w_ok, lo), np.where(ok, hi - mu * w_ok, hi)
    b = np.zeros(h) if b1 is None else _f64(b1)
    if bits == 8:
        Q = np.zeros((h, d), np.int8)
        s = np.abs(W1).max(axis=1) / 127.0
        for j in range(h):
            if s[j] > 0.0:
                Q[j] = np.clip(np.rint(W1[j] / s[j]), -127, 127).astype(np.int8)
        tlo, thi = _thresholds(lo, hi, b, s)
        return Sketch(Q=Q, s=s, tlo=tlo, thi=thi)
    if bits not in (4, 3, 2):
        raise ValueError("sketch bits must be 8, 4, 3 or 2")
    qmax = 2 ** (bits - 1) - 1
    G = SKETCH_GROUP
    ng = (d + G - 1) // G
    Wg = np.zeros((h, ng * G))                     # zero padding changes no maximum and no code
    Wg[:, :d] = W1
    Wg = Wg.reshape(h, ng, G)
    gmax = np.abs(Wg).max(axis=2)                  # h x ng
    s = gmax.max(axis=1) / float(qmax * SKETCH_MMAX)
    live = s > 0.0
    s_safe = np.where(live, s, 1.0)
    m = np.clip(np.ceil(gmax / (qmax * s_safe)[:, None]), 1, SKETCH_MMAX)
    m = np.where(live[:, None], m, 1.0)
    q = np.clip(np.rint(Wg / (m * s_safe[:, None])[:, :, None]), -qmax, qmax)
    q = np.where(live[:, None, None], q, 0.0)
    q4 = q.reshape(h, ng * G)[:, :d].astype(np.int8)
    Q = (m[:, :, None] * q).reshape(h, ng * G)[:, :d].astype(np.int8)
    m = m.astype(np.uint8)
    tlo, thi = _thresholds(lo, hi, b, s)
    return Sketch(Q=Q, s=s, tlo=tlo, thi=thi, bits=bits, group=G, m=m, q4=q4)


def quantize_token(x):
    """int8 code of one token with a power-of-two scale.

    m = max|x_k|; e = floor(log2 m) - 6, so |x_k| / 2^e < 128;
    xq_k = rint(x_k / 2^e) clamped to [-127, 127].  A zero token has e = 0 and
    xq = 0.  Returns (xq int8[d], e int).
    """
    x = _f64(x)
    m = float(np.abs(x).max()) if x.size else 0.0
    if m == 0.0:
        return np.zeros(x.shape, np.int8), 0
    e = math.frexp(m)[1] - 1 - 6          # frexp: m = f * 2^k with 0.5 <= f < 1
    xq = np.clip(np.rint(np.ldexp(x, -e)), -127, 127).astype(np.int8)
    return xq, e


def predict(sk: Sketch, x):
    """Flags of one token: neuron j is flagged unless tlo_j <= v_j < thi_j with
    v_j = fp32(acc_j) * 2^e and acc_j = sum_k Q[j,k] * xq[k] (an exact integer).
    A NaN bound or value flags the neuron (the test is a negated AND)."""
    xq, e = quantize_token(x)
    # every partial sum is an integer below 2^53, so the fp64 product is exact
    acc = sk.Q.astype(np.float64) @ xq.astype(np.float64)
    acc = acc.astype(np.int64)
    v = np.ldexp(acc.astype(np.float32), e).astype(np.float32)
    with np.errstate(invalid="ignore"):
        inside = (v >= sk.tlo) & (v < sk.thi)
    return ~inside


# ---------------------------------------------------------------------------
# online forward  (Sec. "Inference Runtime": speculative approximation, then
# result fixing for the neurons the predictor names)
# ---------------------------------------------------------------------------
@dataclass
class Folded:
    d: int
    h: int
    kind: str
    W1: np.ndarray
    b1: np.ndarray | None
    W2: np.ndarray
    a: np.ndarray
    c: np.ndarray
    Wp: np.ndarray
    bp: np.ndarray
    sk: Sketch


def build(W1, b1, W2, b2, lo, hi, a, c, kind: str = "gelu_erf", wp_round=None, sketch_bits: int = 8,
          margin: float = 0.0) -> Folded:
    """Everything the online path needs.  `wp_round`, if given, is applied to W'
    once (e.g. rounding to the storage dtype) for the storage-matched variant."""
    Wp, bp = fold(W1, b1, W2, b2, a, c)
    if wp_round is not None:
        Wp = np.asarray(wp_round(Wp), dtype=np.float64)
    h, d = np.shape(W1)
    return Folded(d=d, h=h, kind=kind, W1=_f64(W1), b1=_f64(b1), W2=_f64(W2),
                  a=_f64(a), c=_f64(c), Wp=Wp, bp=bp, sk=sketch(W1, b1, lo, hi, sketch_bits, margin))


def fix_terms(F: Folded, x, flags):
    """delta_j = sigma(z_j) - (a_j z_j + c_j) for the flagged neurons (exact
    weights): remove the speculative linear result, add the true one."""
    idx = np.flatnonzero(flags)
    z = F.W1[idx] @ _f64(x)
    if F.b1 is not None:
        z = z + F.b1[idx]
    return idx, act(z, F.kind) - (F.a[idx] * z + F.c[idx])


def forward_token(F: Folded, x, flags=None):
    """y = W'x + b' + sum_{j flagged} delta_j W2[:, j].  Every flagged neuron is
    fixed whether or not its exact z turns out to be in range.  Returns
    (y fp64[d], flags bool[h])."""
    x = _f64(x)
    if flags is None:
        flags = predict(F.sk, x)
    y = F.Wp @ x + F.bp
    idx, delta = fix_terms(F, x, flags)
    y = y + F.W2[:, idx] @ delta
    return y, flags


def forward(F: Folded, X, flags=None):
    """Batched forward, strictly per token (a token is fixed only for the
    neurons its own predictor pass flagged).  X: n x d -> (Y n x d, flags n x h)."""
    X = _f64(X)
    n = X.shape[0]
    Y = np.empty((n, F.d))
    FL = np.empty((n, F.h), bool)
    for t in range(n):
        Y[t], FL[t] = forward_token(F, X[t], None if flags is None else flags[t])
    return Y, FL


# ---------------------------------------------------------------------------
# helpers used by the tests of the stacked configuration and of bf16 storage
# ---------------------------------------------------------------------------
def rmsnorm(Y, eps: float = 1e-6):
    """x = y / sqrt(mean(y^2) + eps), unit gain, per token (row)."""
    Y = _f64(Y)
    return Y / np.sqrt((Y * Y).mean(axis=-1, keepdims=True) + eps)


def to_bf16(x):
    """Nearest bfloat16 (ties to even) of fp64/fp32 values, returned as fp64.
    Goes through fp32 first, as a conversion from an fp32 accumulator does."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
    return r.view(np.float32).astype(np.float64).reshape(np.shape(x))


def pack_mask(flags):
    """bool n x h -> uint32 n x ceil(h/32); bit (j % 32) of word j // 32."""
    flags = np.atleast_2d(np.asarray(flags, bool))
    n, h = flags.shape
    w = (h + 31) // 32
    pad = np.zeros((n, w * 32), bool)
    pad[:, :h] = flags
    bits = pad.reshape(n, w, 32).astype(np.uint32)
    return (bits << np.arange(32, dtype=np.uint32)[None, None, :]).sum(axis=2, dtype=np.uint64).astype(np.uint32)
