"""CPU oracle for the vector-quantised KAN forward pass (SHARe-KAN / LUTHAM).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, float64
numpy/Python statement of what the layer computes, written from the paper.
Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
import it.  It shares no code, table or constant with the HIP path and never
imports the package that binds the HIP library.

What it follows
---------------
* KAN layer: every edge (i, j) carries a univariate spline, the layer output is
  the sum of the edge contributions, y_j = sum_i phi_ij(x_i)          (paper §3).
* Spline family: cubic B-splines (k = 3), G = 10 coefficients per edge on the
  range [-1, 1] with normalised inputs                           (paper App. A.1).
  G = 7 uniform intervals + degree 3, so the knot vector has G + k + 1 = 14
  knots, three of them beyond each end of [-1, 1].
* Gain-Shape-Bias decomposition, Eq. (1): phi_ij(x) = g_ij * C[k_ij](x) + b_ij
  with one K x G codebook C per layer; the reconstructed coefficient vector is
  c_ij = g_ij * C[k_ij] + b_ij                                    (paper §4.2).
  On [-1, 1] the two statements agree because the bases sum to one.
* Int8 codebooks store one byte per coefficient (paper §4.3, §5.4); the value
  is scale * q with one fp32 scale per layer (a reading: the paper gives the
  byte count but not the mapping).
* Block-floating-point codebooks (the BFP8 row of the paper's Table 1): one shared
  exponent byte per codeword row and ten signed mantissa bytes (a reading: the
  paper names the precision only; PARITY WITH THE PAPER'S OWN ENCODING IS UNPINNED,
  the decoder is pinned against what fixes this reading's meaning).
* Heads: tanh between layers, none after the last (benchmark configuration).

* The runtime operator's own rule (paper §4.1, §4.3), selectable with
  rule="pli": the G entries of a codeword are samples at G uniform nodes over
  [-1, 1], the lookup index is floor((x + 1) / dx), dx = 2 / (G - 1), and the
  value is the linear interpolation between the two neighbouring entries; the
  last interval is closed at x = +1 (a reading: the paper gives the index
  expression and names two codebook entries, not dx or the end rule).

Bases are evaluated by the Cox-de Boor recursion, exactly as the textbook
definition states it; nothing here uses the closed-form uniform cubic weights
that the GPU kernels use.  The piecewise-linear rule is written out from its
definition (locate the interval by search over the nodes, interpolate).

Pins (see tests/test_oracle_pins.py): partition of unity, exactly four nonzero
bases at span..span+3, constant codeword => gain*v+bias, VQ == dense on
reconstructed coefficients, basis integrals == h, knot/mid-interval closed-form
weights, linear and quadratic precision (Greville / Marsden coefficients),
scipy.interpolate.BSpline, scalar brute force vs vectorised form, permutation
invariance, linearity in gain / additivity in bias, Int8 == fp32 twin; for the
piecewise-linear rule: numpy.interp, reproduction of the node values and of
every linear function, hat-function integrals, index against brute force; for
byte-coded gain/bias: exact powers of two at integer exponents, zero code,
monotonicity, round trip through the encoder within half a step; for the
assignment step: brute-force loops, scipy's k-d tree, exact recovery of a layer built
from the codebook (R^2 = 1), invariance under affine changes of a grid; for the error
scale A = sum_i |phi_ij|: the scalar definition summed edge by edge, constant and linear
codewords (closed forms), in both vectorised forms; for block-floating-point codebooks:
rows of exact powers of two, negative exponents, the ignored twelfth byte, round trip
through the generator's encoder within half a mantissa step, equality with the layer built
from the decoded fp64 rows.
"""
from __future__ import annotations

import math

import numpy as np

DEGREE = 3           # cubic                                    (paper App. A.1)
G = 10               # coefficients per edge                    (paper App. A.1)
N_INTERVALS = G - DEGREE          # 7 uniform intervals on [-1, 1]
N_KNOTS = G + DEGREE + 1          # 14
X_LO, X_HI = -1.0, 1.0            # grid range                  (paper App. A.1)


def knots() -> np.ndarray:
    """Uniform knot vector t_0..t_13, t_3 = -1, t_10 = +1, spacing 2/7.

    Written as a single division so that both ends of [-1, 1] are exact.
    """
    return np.array([(2.0 * (m - DEGREE) - N_INTERVALS) / N_INTERVALS
                     for m in range(N_KNOTS)], dtype=np.float64)


def clamp_input(x):
    """Inputs are normalised to [-1, 1] (paper App. A.1); values outside are clamped."""
    return np.minimum(np.maximum(np.asarray(x, dtype=np.float64), X_LO), X_HI)


# --------------------------------------------------------------------------
# Scalar definition (pure Python; tiny inputs only)
# --------------------------------------------------------------------------

def basis_scalar(m: int, p: int, x: float, t=None, close_right: bool = True) -> float:
    """B_{m,p}(x) by the Cox-de Boor recursion.

    B_{m,0}(x) = 1 on the half-open interval [t_m, t_{m+1}), else 0.
    With close_right the point x = t_10 = +1 belongs to the last interior
    interval [t_9, t_10] (and therefore not to [t_10, t_11)).
    """
    if t is None:
        t = knots()
    if p == 0:
        if close_right and x == t[G]:
            return 1.0 if m == G - 1 else 0.0
        return 1.0 if (t[m] <= x < t[m + 1]) else 0.0
    left = (x - t[m]) / (t[m + p] - t[m]) * basis_scalar(m, p - 1, x, t, close_right)
    right = ((t[m + p + 1] - x) / (t[m + p + 1] - t[m + 1])
             * basis_scalar(m + 1, p - 1, x, t, close_right))
    return left + right


def span_scalar(x: float) -> int:
    """Index l in 0..6 of the interior interval [t_{l+3}, t_{l+4}) that holds the
    clamped x; x = +1 belongs to the last one (l = 6).  Found by search."""
    t = knots()
    x = min(max(float(x), X_LO), X_HI)
    if x == t[G]:
        return N_INTERVALS - 1
    for l in range(N_INTERVALS):
        if t[l + DEGREE] <= x < t[l + DEGREE + 1]:
            return l
    raise ValueError("x is NaN or outside the knot range")


def edge_phi_scalar(coef, x: float) -> float:
    """phi(x) = sum_m B_{m,3}(x) * c_m for one edge, x clamped to [-1, 1]."""
    x = min(max(float(x), X_LO), X_HI)
    t = knots()
    return math.fsum(basis_scalar(m, DEGREE, x, t) * float(coef[m]) for m in range(G))


def reconstruct_scalar(codebook, scale: float, idx, gain, bias, i: int, j: int):
    """c_ij = g_ij * (scale * C[k_ij]) + b_ij  (paper §4.2, reconstructed grid)."""
    k = int(idx[i][j])
    return [float(gain[i][j]) * (float(scale) * float(codebook[k][m])) + float(bias[i][j])
            for m in range(G)]


def vq_layer_forward_scalar(x, codebook, scale, idx, gain, bias):
    """Definition of the layer, three nested Python loops.  x: [B][in]."""
    B, n_in = len(x), len(x[0])
    n_out = len(idx[0])
    y = [[0.0] * n_out for _ in range(B)]
    for b in range(B):
        for j in range(n_out):
            terms = []
            for i in range(n_in):
                c = reconstruct_scalar(codebook, scale, idx, gain, bias, i, j)
                terms.append(edge_phi_scalar(c, x[b][i]))
            y[b][j] = math.fsum(terms)
    return np.array(y, dtype=np.float64)


# --------------------------------------------------------------------------
# Vectorised float64 form (used for the configurations and as CPU baseline)
# --------------------------------------------------------------------------

def basis_matrix(x, clamp: bool = True, close_right: bool = True) -> np.ndarray:
    """All G cubic bases at every x: returns [..., G] float64.

    The recursion is carried out level by level on arrays: level 0 holds the 13
    interval indicators, level p the 13 - p bases of degree p.
    With clamp=False and close_right=False the bases are those of the plain
    half-open definition on the whole knot range (used to integrate a basis
    over its full support).
    """
    t = knots()
    x = np.asarray(x, dtype=np.float64)
    shape = x.shape
    x = x.reshape(-1)
    if clamp:
        x = clamp_input(x)
    xs = x[:, None]
    lvl = ((t[:-1] <= xs) & (xs < t[1:])).astype(np.float64)      # [..., 13]
    if close_right:
        at_end = (x == t[G])
        lvl[at_end, :] = 0.0
        lvl[at_end, G - 1] = 1.0
    for p in range(1, DEGREE + 1):
        n = N_KNOTS - 1 - p
        m = np.arange(n)
        left = (xs - t[m]) / (t[m + p] - t[m])
        right = (t[m + p + 1] - xs) / (t[m + p + 1] - t[m + 1])
        lvl = left * lvl[:, :n] + right * lvl[:, 1:n + 1]
    return lvl.reshape(shape + (G,))                             # [..., 10]


# --------------------------------------------------------------------------
# The runtime operator's two-tap rule (paper §4.1: the cell index is x / dx rounded down,
# and the value is interpolated linearly between the two codebook entries at that cell's
# ends; §4.3 writes it as LinearInterp(C[k], x))
# --------------------------------------------------------------------------

def pli_nodes() -> np.ndarray:
    """The G uniform nodes n_0 = -1 .. n_{G-1} = +1 at which a codeword's entries sit."""
    return np.array([(2.0 * k - (G - 1)) / (G - 1) for k in range(G)], dtype=np.float64)


def pli_index(x) -> np.ndarray:
    """Lookup index k in 0..G-2 of every (clamped) x: the interval [n_k, n_{k+1}) that holds
    it, found by search over the interior nodes; x = +1 belongs to the last interval."""
    n = pli_nodes()
    return np.searchsorted(n[1:G - 1], clamp_input(x), side="right").astype(np.uint8)


def pli_scalar(row, x: float) -> float:
    """LinearInterp(row, x) for one codeword row (any sequence of G numbers) and one x."""
    n = pli_nodes()
    xc = min(max(float(x), X_LO), X_HI)
    k = 0
    while k < G - 2 and xc >= n[k + 1]:
        k += 1
    u = (xc - n[k]) / (n[k + 1] - n[k])
    return (1.0 - u) * float(row[k]) + u * float(row[k + 1])


def pli_matrix(x) -> np.ndarray:
    """[..., G] weights of the G entries at every x: (1 - u) on entry k, u on entry k + 1."""
    n = pli_nodes()
    x = np.asarray(x, dtype=np.float64)
    xc = clamp_input(x).reshape(-1)
    k = pli_index(xc).astype(np.int64)
    u = (xc - n[k]) / (n[k + 1] - n[k])
    W = np.zeros((xc.size, G), dtype=np.float64)
    r = np.arange(xc.size)
    W[r, k] = 1.0 - u
    W[r, k + 1] = u
    return W.reshape(x.shape + (G,))


def design_matrix(x, rule: str = "bspline") -> np.ndarray:
    """Weights of a codeword's G entries at every x under the chosen edge rule."""
    if rule == "bspline":
        return basis_matrix(x)
    if rule == "pli":
        return pli_matrix(x)
    raise ValueError(rule)


def span_index(x) -> np.ndarray:
    """Interval index l in 0..6 for every (clamped) x, by search over the float64
    interior knots: l = number of interior knots t_4..t_9 that are <= x."""
    t = knots()
    xc = clamp_input(x)
    return np.searchsorted(t[DEGREE + 1:G], xc, side="right").astype(np.uint8)


BFP8_ROW_BYTES = G + 2       # ten mantissa bytes, the row's exponent byte, one zero byte


def dequantise_codebook(codebook, scale=1.0) -> np.ndarray:
    """Codebook as float64 [K][G].  Int8 codebooks [K][G]: value = scale * q; floating
    codebooks are taken as they are (scale ignored).

    Block floating point with 8-bit mantissas (the BFP8 row of the paper's Table 1; the paper
    names the precision, not the format - this reading: one block per codeword row): an int8
    array [K][12] whose row k holds ten signed mantissas q[k][0..9], then the signed exponent
    e[k] shared by the row, then a zero byte; entry m is q[k][m] * 2 ** e[k] (scale ignored)."""
    cb = np.asarray(codebook)
    if cb.dtype == np.int8 and cb.shape[-1] == BFP8_ROW_BYTES:
        q = cb[..., :G].astype(np.float64)
        e = cb[..., G].astype(np.float64)
        return q * np.exp2(e)[..., None]
    if cb.dtype == np.int8:
        return np.float64(np.float32(scale)) * cb.astype(np.float64)
    return cb.astype(np.float64)


def dequantise_gain_bias(gain, bias, gb_params=None):
    """Per-edge gain and bias as float64.

    Floating arrays are taken as they are.  With gb_params = (gain_log2_lo, gain_log2_step,
    bias_scale) the arrays hold one byte per value (paper §4.2: gains on a logarithmic Int8
    grid, biases on a linear Int8 grid; the paper prints no formula, this is a reading):
    gain code 0 is a zero gain, code c = 1..255 means 2 ** (lo + step * c); bias code c
    (signed) means bias_scale * c.
    """
    if gb_params is None:
        return np.asarray(gain).astype(np.float64), np.asarray(bias).astype(np.float64)
    lo, step, bscale = (np.float64(np.float32(v)) for v in gb_params)
    qg = np.asarray(gain)
    qb = np.asarray(bias)
    assert qg.dtype == np.uint8 and qb.dtype == np.int8
    c = qg.astype(np.float64)
    g = np.where(qg == 0, 0.0, np.exp2(lo + step * c))
    return g, bscale * qb.astype(np.float64)


def reconstruct_coefficients(codebook, scale, idx, gain, bias, gb_params=None) -> np.ndarray:
    """Dense coefficients c[i][j][m] = g_ij * C[k_ij][m] + b_ij  (paper §4.2)."""
    cb = dequantise_codebook(codebook, scale)
    idx = np.asarray(idx).astype(np.int64)
    g, b = dequantise_gain_bias(gain, bias, gb_params)
    return g[..., None] * cb[idx] + b[..., None]


def dense_layer_forward(coef, x, return_abs: bool = False, rule: str = "bspline"):
    """y[b][j] = sum_i sum_m B_{m,3}(x_bi) * coef[i][j][m]      (paper §3); with rule="pli"
    the weights B are those of the two-tap interpolation instead.

    return_abs additionally gives A[b][j] = sum_i |phi_ij(x_bi)|, the scale
    against which a per-element error is judged.
    """
    coef = np.asarray(coef, dtype=np.float64)
    n_in, n_out, g = coef.shape
    assert g == G
    x = np.asarray(x, dtype=np.float64)
    assert x.ndim == 2 and x.shape[1] == n_in
    Bm = design_matrix(x, rule)                                  # [B][in][G]
    Phi = Bm.reshape(x.shape[0], n_in * G)
    Chat = coef.transpose(0, 2, 1).reshape(n_in * G, n_out)
    y = Phi @ Chat
    if not return_abs:
        return y
    A = np.empty_like(y)
    for b in range(x.shape[0]):
        phi = np.einsum("im,ijm->ij", Bm[b], coef)
        A[b] = np.abs(phi).sum(axis=0)
    return y, A


def vq_layer_forward(x, codebook, scale, idx, gain, bias, return_abs: bool = False, rule: str = "bspline",
                     gb_params=None):
    """Forward pass of one VQ-KAN layer: reconstruct, evaluate, sum over inputs."""
    coef = reconstruct_coefficients(codebook, scale, idx, gain, bias, gb_params)
    return dense_layer_forward(coef, x, return_abs=return_abs, rule=rule)


def vq_layer_outputs_at(x, codebook, scale, idx, gain, bias, bs, js, return_abs=False, rule: str = "bspline",
                        gb_params=None):
    """y[b][j] for listed (b, j) pairs only; O(in) work each.  For parity checks
    at sizes where the whole layer is too slow on the CPU."""
    cb = dequantise_codebook(codebook, scale)
    idx = np.asarray(idx)
    gain, bias = dequantise_gain_bias(gain, bias, gb_params)
    x = np.asarray(x, dtype=np.float64)
    out = np.empty(len(bs), dtype=np.float64)
    ab = np.empty(len(bs), dtype=np.float64)
    for n, (b, j) in enumerate(zip(bs, js)):
        Bm = design_matrix(x[b], rule)                           # [in][G]
        c = (gain[:, j].astype(np.float64)[:, None] * cb[idx[:, j].astype(np.int64)]
             + bias[:, j].astype(np.float64)[:, None])           # [in][G]
        phi = (Bm * c).sum(axis=1)
        out[n] = phi.sum()
        ab[n] = np.abs(phi).sum()
    return (out, ab) if return_abs else out


def vq_head_forward(x, layers, return_hidden: bool = False, rule: str = "bspline"):
    """Multi-layer head: tanh between layers, none after the last.

    layers: sequence of dicts with keys codebook, scale, idx, gain, bias.
    """
    a = np.asarray(x, dtype=np.float64)
    hidden = []
    for n, L in enumerate(layers):
        y = vq_layer_forward(a, L["codebook"], L["scale"], L["idx"], L["gain"], L["bias"], rule=rule,
                             gb_params=L.get("gb_params"))
        if n + 1 < len(layers):
            a = np.tanh(y)
            hidden.append(a)
        else:
            a = y
    return (a, hidden) if return_hidden else a


# --------------------------------------------------------------------------
# Compression side: normalise every grid, assign it to the nearest codebook shape
# (paper §4.2, steps (1) and (3) of the post-training procedure; R^2 of the reconstruction)
# --------------------------------------------------------------------------

def normalise_grids(coef):
    """coef [..., G] -> (shape [..., G], gain [...], bias [...]): bias is the mean of the grid,
    gain the Euclidean norm of the centred grid, shape = centred / gain (zeros where gain is 0).
    The paper normalises to zero mean and unit variance; the benchmark's codebooks hold
    zero-mean unit-NORM shapes, so the norm is used here: the same shapes, gains differ by
    sqrt(G)."""
    c = np.asarray(coef, dtype=np.float64)
    bias = c.mean(axis=-1)
    centred = c - bias[..., None]
    gain = np.sqrt((centred * centred).sum(axis=-1))
    safe = np.where(gain > 0, gain, 1.0)
    return centred / safe[..., None], gain, bias


def squared_distances(shapes, codebook):
    """d2[e][k] = sum_m (shapes[e][m] - codebook[k][m])^2, written out as the definition
    (memory E*K*G doubles: small inputs only)."""
    n = np.asarray(shapes, dtype=np.float64).reshape(-1, G)
    C = np.asarray(codebook, dtype=np.float64)
    diff = n[:, None, :] - C[None, :, :]
    return (diff * diff).sum(axis=-1)


def assign_edges(coef, codebook, chunk: int = 64):
    """(idx, gain, bias, d2_min) for a dense layer coef [in][out][G]: idx[i][j] is the first
    codebook row at the smallest squared distance from the normalised grid of edge (i, j)."""
    c = np.asarray(coef, dtype=np.float64)
    n, gain, bias = normalise_grids(c)
    flat = n.reshape(-1, G)
    idx = np.empty(flat.shape[0], dtype=np.int64)
    dmin = np.empty(flat.shape[0], dtype=np.float64)
    for s in range(0, flat.shape[0], chunk):
        d2 = squared_distances(flat[s:s + chunk], codebook)
        idx[s:s + chunk] = d2.argmin(axis=1)
        dmin[s:s + chunk] = d2.min(axis=1)
    return idx.reshape(c.shape[:-1]), gain, bias, dmin.reshape(c.shape[:-1])


def r_squared(coef, codebook, idx, gain, bias) -> float:
    """R^2 between the original grids and the reconstruction gain * C[idx] + bias (paper §4.2):
    1 - SS_res / SS_tot over all coefficients, SS_tot about their overall mean."""
    c = np.asarray(coef, dtype=np.float64)
    rec = reconstruct_coefficients(np.asarray(codebook, dtype=np.float64), 1.0, idx, gain, bias)
    ss_res = ((c - rec) ** 2).sum()
    ss_tot = ((c - c.mean()) ** 2).sum()
    return float(1.0 - ss_res / ss_tot)


def error_report(y_test, y_ref, A_ref=None) -> dict:
    """Error figures used by the parity tests.

    headline : max|dy| / max|y_ref|  over the tensor
    strict   : max over elements of |dy| / A_ref, A_ref[b][j] = sum_i |phi_ij|
               (a sum of thousands of mixed-sign terms can cancel to ~0, so a
               plain per-element |dy|/|y| is ill-conditioned and is not a gate)
    """
    y_test = np.asarray(y_test, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    d = np.abs(y_test - y_ref)
    rep = {"headline": float(d.max() / max(np.abs(y_ref).max(), 1e-300)),
           "max_abs": float(d.max())}
    if A_ref is not None:
        rep["strict"] = float((d / np.maximum(np.asarray(A_ref, dtype=np.float64), 1e-300)).max())
    return rep
