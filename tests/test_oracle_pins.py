"""Pins for the CPU oracle: facts fixed by the paper and by the mathematics of
B-splines, none of which re-type the oracle's own formula.

Each pin names the part of the oracle it would catch a mistake in.
"""
import math
import os

import numpy as np
import pytest
from scipy.interpolate import BSpline

from oracle import kan_oracle as ko
from paper_2512_15742_amd import synth

H = 2.0 / 7.0


def _probe_points():
    """[-1, 1] densely, both ends, every knot and its float32/float64 neighbours."""
    t = ko.knots()
    pts = [np.linspace(-1.0, 1.0, 2001)]
    for k in t[3:11]:
        f = np.float32(k)
        pts.append(np.array([k, np.nextafter(k, -2), np.nextafter(k, 2), float(f),
                             float(np.nextafter(f, np.float32(-2))),
                             float(np.nextafter(f, np.float32(2)))]))
    x = np.concatenate(pts)
    return x[(x >= -1.0) & (x <= 1.0)]


def _golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")
    out = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = int(v)
    return out


# ---- constants the paper prints ------------------------------------------------

def test_paper_constants():
    g = _golden()
    assert ko.DEGREE == g["spline_degree"]
    assert ko.G == g["grid_size_G"]
    assert (ko.X_LO, ko.X_HI) == (g["range_lo"], g["range_hi"])
    t = ko.knots()
    assert len(t) == ko.G + ko.DEGREE + 1
    assert t[3] == -1.0 and t[10] == 1.0
    assert np.allclose(np.diff(t), H, rtol=0, atol=1e-15)
    # storage arithmetic of the Int8 codebook and of a dense edge
    L = synth.make_layer(7, 4, 4, g["codebook_entries_K"], cb_dtype="i8", gb_dtype="f16")
    assert L.codebook.nbytes == g["int8_codebook_bytes"]
    assert L.idx.dtype.itemsize * 8 == g["index_bits_at_K"]
    assert ko.G * 4 == g["dense_bytes_per_edge"]


# ---- P1: partition of unity, four nonzero bases at span..span+3 ----------------

def test_partition_of_unity_and_support():
    x = _probe_points()
    Bm = ko.basis_matrix(x)
    assert Bm.shape == (x.size, 10)
    assert np.abs(Bm.sum(axis=1) - 1.0).max() < 1e-14
    assert (Bm >= 0).all()
    sp = ko.span_index(x).astype(int)
    assert sp.min() == 0 and sp.max() == 6
    m = np.arange(10)[None, :]
    outside = (m < sp[:, None]) | (m > sp[:, None] + 3)
    assert (Bm[outside] == 0.0).all()
    # strictly inside an interval all four are positive
    t = ko.knots()
    xin = (t[3:10] + 0.37 * H)
    Bin = ko.basis_matrix(xin)
    for r, l in enumerate(range(7)):
        assert (Bin[r, l:l + 4] > 0).all()


def test_span_matches_scalar_search_and_ends():
    x = _probe_points()
    sp = ko.span_index(x)
    for xv, s in zip(x[::7], sp[::7]):
        assert ko.span_scalar(xv) == s
    assert ko.span_index(np.array([-1.0]))[0] == 0
    assert ko.span_index(np.array([1.0]))[0] == 6
    assert ko.span_index(np.array([-3.0, 5.0])).tolist() == [0, 6]      # clamped
    # an x just below / at / above the float32 neighbours of an interior knot
    t = ko.knots()
    for l in range(1, 7):
        k = t[l + 3]
        f = np.float32(k)
        lo, hi = (f, np.nextafter(f, np.float32(2))) if float(f) < k else (np.nextafter(f, np.float32(-2)), f)
        assert float(lo) < k <= float(hi)
        assert ko.span_index(np.array([float(lo)]))[0] == l - 1
        assert ko.span_index(np.array([float(hi)]))[0] == l


# ---- P5: closed-form values at knots and mid-interval --------------------------

def test_closed_form_weights_at_knot_and_midpoint():
    t = ko.knots()
    for l in range(7):
        Bk = ko.basis_matrix(np.array([t[l + 3]]))[0]
        np.testing.assert_allclose(Bk[l:l + 4], [1 / 6, 2 / 3, 1 / 6, 0.0], atol=1e-15)
        Bmid = ko.basis_matrix(np.array([t[l + 3] + H / 2]))[0]
        np.testing.assert_allclose(Bmid[l:l + 4], [1 / 48, 23 / 48, 23 / 48, 1 / 48], atol=1e-15)
    # right end is closed: x = +1 uses coefficients 6..9 with (0, 1/6, 2/3, 1/6)
    Bend = ko.basis_matrix(np.array([1.0]))[0]
    np.testing.assert_allclose(Bend[6:10], [0.0, 1 / 6, 2 / 3, 1 / 6], atol=1e-15)
    assert (Bend[:6] == 0).all()
    # scalar definition agrees at the same points
    for m in range(10):
        assert abs(ko.basis_scalar(m, 3, 1.0) - Bend[m]) < 1e-15


# ---- P4: integral of a single basis over its support equals h ------------------

def test_basis_integrals():
    t = ko.knots()
    n = 200001
    xs = np.linspace(t[0], t[-1], n)
    Bm = ko.basis_matrix(xs, clamp=False, close_right=False)
    dx = xs[1] - xs[0]
    integ = (Bm[:-1] + Bm[1:]).sum(axis=0) * dx / 2            # trapezoid, brute force
    np.testing.assert_allclose(integ, np.full(10, H), rtol=1e-8)
    # restricted to [-1, 1] the end bases lose part of their support
    inside = (xs >= -1) & (xs <= 1)
    Bi = Bm[inside]
    integ_in = (Bi[:-1] + Bi[1:]).sum(axis=0) * dx / 2
    expect = np.array([1 / 24, 1 / 2, 23 / 24, 1, 1, 1, 1, 23 / 24, 1 / 2, 1 / 24]) * H
    np.testing.assert_allclose(integ_in, expect, rtol=2e-4)
    assert abs(integ_in.sum() - 2.0) < 1e-4


# ---- P6 / P7: linear and quadratic precision -----------------------------------

def test_linear_precision_greville():
    t = ko.knots()
    c = np.array([(t[m + 1] + t[m + 2] + t[m + 3]) / 3 for m in range(10)])
    x = _probe_points()
    phi = ko.basis_matrix(x) @ c
    assert np.abs(phi - x).max() < 1e-15 * 4
    for xv in (-1.0, -0.3, 0.0, 0.99, 1.0):
        assert abs(ko.edge_phi_scalar(c, xv) - xv) < 1e-15


def test_quadratic_precision_marsden():
    t = ko.knots()
    c = np.array([(t[m + 1] * t[m + 2] + t[m + 1] * t[m + 3] + t[m + 2] * t[m + 3]) / 3
                  for m in range(10)])
    x = _probe_points()
    phi = ko.basis_matrix(x) @ c
    assert np.abs(phi - x * x).max() < 1e-15 * 4


def test_layer_closed_form_linear_shapes():
    """A codebook whose rows are multiples of the Greville vector makes every
    edge linear: y_j = sum_i (g_ij * a_k * x_i + b_ij), a plain mat-vec."""
    rng = np.random.default_rng(11)
    t = ko.knots()
    grev = np.array([(t[m + 1] + t[m + 2] + t[m + 3]) / 3 for m in range(10)])
    K, n_in, n_out, B = 7, 9, 5, 6
    a = rng.normal(size=K)
    cb = (a[:, None] * grev[None, :])
    idx = rng.integers(0, K, size=(n_in, n_out)).astype(np.uint16)
    gain = rng.normal(size=(n_in, n_out))
    bias = rng.normal(size=(n_in, n_out))
    x = rng.uniform(-1, 1, size=(B, n_in))
    y = ko.vq_layer_forward(x, cb, 1.0, idx, gain, bias)
    W = gain * a[idx]
    expect = x @ W + bias.sum(axis=0)[None, :]
    np.testing.assert_allclose(y, expect, atol=1e-13)
    # a transposed idx/gain layout or a swapped (i, j) would break this
    assert n_in != n_out


# ---- P2: constant codeword => gain * v + bias ----------------------------------

def test_constant_codeword():
    rng = np.random.default_rng(5)
    K, n_in, n_out, B = 4, 6, 3, 8
    v = rng.normal(size=K)
    cb = np.repeat(v[:, None], 10, axis=1)
    idx = rng.integers(0, K, size=(n_in, n_out)).astype(np.uint16)
    gain = rng.normal(size=(n_in, n_out))
    bias = rng.normal(size=(n_in, n_out))
    x = rng.uniform(-1.5, 1.5, size=(B, n_in))                  # includes clamped values
    y = ko.vq_layer_forward(x, cb, 1.0, idx, gain, bias)
    expect = (gain * v[idx] + bias).sum(axis=0)
    np.testing.assert_allclose(y, np.broadcast_to(expect, (B, n_out)), atol=1e-13)


# ---- P8: scipy's B-spline routines ---------------------------------------------

def test_against_scipy_bspline():
    t = ko.knots()
    rng = np.random.default_rng(3)
    x = _probe_points()
    for _ in range(5):
        c = rng.normal(size=10)
        ref = BSpline(t, c, 3, extrapolate=False)(x)
        got = ko.basis_matrix(x) @ c
        np.testing.assert_allclose(got, ref, atol=1e-14)
    dm = BSpline.design_matrix(x, t, 3).toarray()
    np.testing.assert_allclose(ko.basis_matrix(x), dm, atol=1e-14)


# ---- P9: brute force on tiny inputs, invariances --------------------------------

def _tiny(seed=0, n_in=3, n_out=2, B=4, K=5, int8=False):
    rng = np.random.default_rng(seed)
    shapes = synth.make_shapes(rng, K)
    if int8:
        cb, scale = synth.quantise_shapes(shapes)
    else:
        cb, scale = shapes, np.float32(1.0)
    idx = rng.integers(0, K, size=(n_in, n_out)).astype(np.uint16)
    gain = np.abs(rng.normal(0, 0.1, size=(n_in, n_out))).astype(np.float32)
    bias = rng.normal(0, 0.01, size=(n_in, n_out)).astype(np.float32)
    x = rng.uniform(-1, 1, size=(B, n_in)).astype(np.float32)
    x[0, 0], x[1, 0] = -1.0, 1.0
    return x, cb, scale, idx, gain, bias


@pytest.mark.parametrize("int8", [False, True])
def test_scalar_definition_vs_vectorised(int8):
    x, cb, scale, idx, gain, bias = _tiny(int8=int8)
    y_def = ko.vq_layer_forward_scalar(x.tolist(), cb.tolist(), float(scale), idx.tolist(),
                                       gain.tolist(), bias.tolist())
    y_vec, A = ko.vq_layer_forward(x, cb, scale, idx, gain, bias, return_abs=True)
    np.testing.assert_allclose(y_vec, y_def, atol=1e-15)
    assert (A >= np.abs(y_vec) - 1e-15).all()
    bs, js = [0, 3, 2], [1, 0, 1]
    ys, As = ko.vq_layer_outputs_at(x, cb, scale, idx, gain, bias, bs, js, return_abs=True)
    np.testing.assert_allclose(ys, y_vec[bs, js], atol=1e-15)
    np.testing.assert_allclose(As, A[bs, js], atol=1e-15)


def test_vq_equals_dense_on_reconstructed():          # P3
    x, cb, scale, idx, gain, bias = _tiny(seed=2, n_in=7, n_out=5, B=6, K=9)
    coef = ko.reconstruct_coefficients(cb, scale, idx, gain, bias)
    assert coef.shape == (7, 5, 10)
    # each reconstructed row is gain * shape + bias of the indexed codeword
    i, j = 4, 3
    np.testing.assert_allclose(coef[i, j], float(gain[i, j]) * cb[idx[i, j]].astype(np.float64)
                               + float(bias[i, j]), atol=0)
    assert np.array_equal(ko.vq_layer_forward(x, cb, scale, idx, gain, bias),
                          ko.dense_layer_forward(coef, x))


def test_permutation_linearity_additivity():
    x, cb, scale, idx, gain, bias = _tiny(seed=4, n_in=8, n_out=3, B=5, K=6)
    y = ko.vq_layer_forward(x, cb, scale, idx, gain, bias)
    perm = np.random.default_rng(1).permutation(8)
    yp = ko.vq_layer_forward(x[:, perm], cb, scale, idx[perm], gain[perm], bias[perm])
    np.testing.assert_allclose(yp, y, atol=1e-15)
    y0 = ko.vq_layer_forward(x, cb, scale, idx, gain * 0, bias)
    np.testing.assert_allclose(y0, np.broadcast_to(bias.astype(np.float64).sum(0), y.shape), atol=1e-15)
    y2 = ko.vq_layer_forward(x, cb, scale, idx, 2 * gain, bias)
    np.testing.assert_allclose(y2 - y0, 2 * (y - y0), atol=1e-14)
    db = np.random.default_rng(2).normal(size=bias.shape).astype(np.float32)
    yb = ko.vq_layer_forward(x, cb, scale, idx, gain, bias.astype(np.float64) + db)
    np.testing.assert_allclose(yb - y, np.broadcast_to(db.astype(np.float64).sum(0), y.shape), atol=1e-13)


# ---- P10: Int8 layer equals its fp32 twin --------------------------------------

def test_int8_equals_fp32_twin():
    x, q, scale, idx, gain, bias = _tiny(seed=6, n_in=5, n_out=4, B=3, K=8, int8=True)
    assert q.dtype == np.int8 and np.abs(q).max() <= 127
    twin = (np.float64(scale) * q.astype(np.float64))
    y_q = ko.vq_layer_forward(x, q, scale, idx, gain.astype(np.float16), bias.astype(np.float16))
    y_t = ko.vq_layer_forward(x, twin, 1.0, idx, gain.astype(np.float16).astype(np.float64),
                              bias.astype(np.float16).astype(np.float64))
    assert np.array_equal(y_q, y_t)
    # scale is ignored for floating codebooks
    y_f = ko.vq_layer_forward(x, twin, 123.0, idx, gain, bias)
    y_g = ko.vq_layer_forward(x, twin, 1.0, idx, gain, bias)
    assert np.array_equal(y_f, y_g)


def test_fp16_codebook_equals_its_fp32_twin():
    """An fp16 codebook (Table 1) holds numbers that fp32 and float64 represent exactly: the
    layer equals, bit for bit, the one built from the converted rows, whatever scale says,
    and differs from the unrounded fp32 codebook by at most half an fp16 ulp per entry."""
    P = synth.make_layer(31, 6, 5, 40, cb_dtype="f16", gb_dtype="f16")
    assert P.codebook.dtype == np.float16 and float(P.scale) == 1.0
    x = synth.make_x(4, 7, 6)
    y_h = ko.vq_layer_forward(x, **P.as_dict())
    y_t = ko.vq_layer_forward(x, P.codebook.astype(np.float32), 77.0, P.idx, P.gain, P.bias)
    assert np.array_equal(y_h, y_t)
    y_s = np.array(ko.vq_layer_forward_scalar(x.tolist(), P.codebook.tolist(), 1.0, P.idx.tolist(),
                                              P.gain.astype(np.float64).tolist(), P.bias.astype(np.float64).tolist()))
    np.testing.assert_allclose(y_h, y_s, atol=1e-14)
    F = synth.make_layer(31, 6, 5, 40, cb_dtype="f32", gb_dtype="f16")      # same draws, unrounded rows
    assert np.array_equal(F.idx, P.idx) and np.array_equal(F.gain, P.gain)
    err = np.abs(F.codebook.astype(np.float64) - P.codebook.astype(np.float64))
    assert 0 < err.max() <= 2.0 ** -12                   # |entries| < 1: half an ulp of fp16 is at most 2^-12
    y_f = ko.vq_layer_forward(x, **F.as_dict())
    bound = 2.0 ** -12 * np.abs(P.gain.astype(np.float64)).sum(axis=0)      # the basis weights sum to 1
    assert (np.abs(y_f - y_h) <= bound[None, :] + 1e-15).all()


# ---- heads ---------------------------------------------------------------------

def test_head_is_layers_with_tanh_between():
    rng = np.random.default_rng(9)
    L1 = synth.make_layer(21, 6, 5, 16, cb_dtype="i8", gb_dtype="f16")
    L2 = synth.make_layer(22, 5, 3, 16, cb_dtype="i8", gb_dtype="f16")
    x = rng.uniform(-1, 1, size=(4, 6)).astype(np.float32)
    y, hidden = ko.vq_head_forward(x, [L1.as_dict(), L2.as_dict()], return_hidden=True)
    y1 = ko.vq_layer_forward(x, **L1.as_dict())
    a = np.array([[math.tanh(v) for v in row] for row in y1])
    np.testing.assert_allclose(hidden[0], a, atol=1e-15)
    y2 = ko.vq_layer_forward(a, **L2.as_dict())
    np.testing.assert_allclose(y, y2, atol=1e-15)
    assert np.abs(y).max() > 1e-3          # no tanh after the last layer would not bound it; sanity only


def test_error_report():
    y = np.array([[1.0, -2.0], [0.0, 4.0]])
    rep = ko.error_report(y + 1e-3, y, np.full_like(y, 10.0))
    assert abs(rep["headline"] - 1e-3 / 4) < 1e-12
    assert abs(rep["strict"] - 1e-4) < 1e-12


# ---- the runtime operator's two-tap rule (paper §4.1, §4.3) ---------------------------

def _pli_probe():
    n = ko.pli_nodes()
    pts = [np.linspace(-1.0, 1.0, 1801)]
    for k in n:
        f = np.float32(k)
        pts.append(np.array([k, np.nextafter(k, -2), np.nextafter(k, 2), float(f),
                             float(np.nextafter(f, np.float32(-2))), float(np.nextafter(f, np.float32(2)))]))
    x = np.concatenate(pts)
    return x[(x >= -1.0) & (x <= 1.0)]


def test_pli_nodes_and_index():
    """Nodes: G of them, uniform, ends exact.  Index: the interval that holds x, by brute
    force over all intervals; the last one closed on the right."""
    n = ko.pli_nodes()
    assert len(n) == ko.G and n[0] == -1.0 and n[-1] == 1.0
    assert np.allclose(np.diff(n), 2.0 / 9.0, rtol=0, atol=1e-15)
    x = _pli_probe()
    k = ko.pli_index(x)
    for xv, kv in zip(x, k):
        inside = [m for m in range(ko.G - 1) if n[m] <= xv < n[m + 1]]
        assert kv == (inside[0] if inside else ko.G - 2)
    assert ko.pli_index(np.array([-1.0, 1.0, -5.0, 7.0])).tolist() == [0, 8, 0, 8]


def test_pli_is_linear_interpolation_numpy_interp():
    """The library routine for exactly this operation."""
    rng = np.random.default_rng(3)
    x = np.concatenate([_pli_probe(), [-3.0, 2.5]])
    n = ko.pli_nodes()
    for _ in range(5):
        row = rng.standard_normal(ko.G)
        ref = np.interp(np.clip(x, -1, 1), n, row)
        got = ko.pli_matrix(x) @ row
        assert np.abs(got - ref).max() < 1e-14
        assert abs(ko.pli_scalar(row, 0.3337) - np.interp(0.3337, n, row)) < 1e-15


def test_pli_reproduces_node_values_linear_functions_and_unity():
    n = ko.pli_nodes()
    W = ko.pli_matrix(_pli_probe())
    assert np.abs(W.sum(axis=-1) - 1).max() < 1e-15                  # weights sum to 1
    assert (W >= 0).all() and ((W > 0).sum(axis=-1) <= 2).all()      # at most two taps
    assert np.abs(ko.pli_matrix(n) - np.eye(ko.G)).max() < 1e-15     # entry k is the value at node k
    row = 0.75 * n - 0.2                                             # samples of a linear function
    x = _pli_probe()
    assert np.abs(W @ row - (0.75 * x - 0.2)).max() < 1e-15
    # hat functions: integral of an interior one is dx, of an end one dx / 2 (brute force)
    xs = np.linspace(-1, 1, 180001)
    area = np.trapezoid(ko.pli_matrix(xs), xs, axis=0) if hasattr(np, "trapezoid") else np.trapz(ko.pli_matrix(xs), xs, axis=0)
    assert np.abs(area[1:-1] - 2.0 / 9.0).max() < 1e-9
    assert abs(area[0] - 1.0 / 9.0) < 1e-9 and abs(area[-1] - 1.0 / 9.0) < 1e-9


def test_pli_layer_closed_forms_and_scalar_definition():
    """Layer level: constant codeword => gain*v + bias; linear codeword => a matrix-vector
    product; vectorised form == scalar definition summed edge by edge."""
    rng = np.random.default_rng(11)
    n_in, n_out, K, B = 5, 4, 6, 7
    cb = rng.standard_normal((K, ko.G))
    cb[2] = 0.37                                                     # constant codeword
    cb[4] = ko.pli_nodes()                                           # C[4](x) = x
    idx = rng.integers(0, K, size=(n_in, n_out))
    gain = np.abs(rng.normal(0, 0.1, size=(n_in, n_out)))
    bias = rng.normal(0, 0.01, size=(n_in, n_out))
    x = rng.uniform(-1.2, 1.2, size=(B, n_in))
    y = ko.vq_layer_forward(x, cb, 1.0, idx, gain, bias, rule="pli")
    ref = np.zeros((B, n_out))
    for b in range(B):
        for i in range(n_in):
            for j in range(n_out):
                ref[b, j] += gain[i, j] * ko.pli_scalar(cb[idx[i, j]], x[b, i]) + bias[i, j]      # Eq. (1)
    assert np.abs(y - ref).max() < 1e-13
    idx2 = np.full((n_in, n_out), 2)
    y2 = ko.vq_layer_forward(x, cb, 1.0, idx2, gain, bias, rule="pli")
    assert np.abs(y2 - (0.37 * gain + bias).sum(axis=0)[None, :]).max() < 1e-14
    idx4 = np.full((n_in, n_out), 4)
    y4 = ko.vq_layer_forward(x, cb, 1.0, idx4, gain, bias, rule="pli")
    assert np.abs(y4 - (np.clip(x, -1, 1) @ gain + bias.sum(axis=0)[None, :])).max() < 1e-14
    # the two rules are different functions of the same ten numbers
    assert np.abs(y - ko.vq_layer_forward(x, cb, 1.0, idx, gain, bias)).max() > 1e-3
    # sampled form and head chaining use the same rule
    bs, js = np.array([0, 3, 6]), np.array([1, 0, 3])
    assert np.abs(ko.vq_layer_outputs_at(x, cb, 1.0, idx, gain, bias, bs, js, rule="pli") - y[bs, js]).max() < 1e-14


# ---- the error scale A = sum_i |phi_ij| (the denominator of every strict per-element gate) ----

def test_abs_sum_A_against_the_scalar_definition_and_closed_forms():
    """A[b][j] = sum_i |phi_ij(x_bi)| from both vectorised forms against (a) the scalar Cox-de Boor
    definition summed edge by edge, (b) a constant codeword, where every edge is the constant
    gain * v + bias, and (c) a Greville (linear) codeword, where phi_ij(x) = gain * a * x + bias.
    A mistake such as sum_i sum_m |B_m c_m| (larger: it would loosen every strict gate) fails all three."""
    for int8 in (False, True):
        x, cb, scale, idx, gain, bias = _tiny(seed=12, n_in=6, n_out=4, B=5, K=7, int8=int8)
        A_def = np.zeros((x.shape[0], idx.shape[1]))
        for b in range(x.shape[0]):
            for j in range(idx.shape[1]):
                A_def[b, j] = math.fsum(
                    abs(ko.edge_phi_scalar(ko.reconstruct_scalar(cb.tolist(), float(scale), idx.tolist(), gain.tolist(),
                                                                 bias.tolist(), i, j), float(x[b, i])))
                    for i in range(x.shape[1]))
        _, A = ko.vq_layer_forward(x, cb, scale, idx, gain, bias, return_abs=True)
        np.testing.assert_allclose(A, A_def, rtol=0, atol=1e-15)
        bs, js = [0, 4, 2, 1], [3, 0, 1, 2]
        _, As = ko.vq_layer_outputs_at(x, cb, scale, idx, gain, bias, bs, js, return_abs=True)
        np.testing.assert_allclose(As, A_def[bs, js], rtol=0, atol=1e-15)
    rng = np.random.default_rng(13)
    K, n_in, n_out, B = 5, 7, 3, 6
    idx = rng.integers(0, K, size=(n_in, n_out)).astype(np.uint16)
    gain = rng.normal(size=(n_in, n_out))               # mixed signs: |sum| and sum of |.| differ
    bias = rng.normal(size=(n_in, n_out))
    x = rng.uniform(-1.3, 1.3, size=(B, n_in))
    # (b) constant codewords
    v = rng.normal(size=K)
    cb = np.repeat(v[:, None], 10, axis=1)
    y, A = ko.vq_layer_forward(x, cb, 1.0, idx, gain, bias, return_abs=True)
    expect = np.abs(gain * v[idx] + bias).sum(axis=0)
    np.testing.assert_allclose(A, np.broadcast_to(expect, (B, n_out)), atol=1e-13)
    assert (A > np.abs(y) + 1e-3).any()                 # the case tells A from |y|
    _, As = ko.vq_layer_outputs_at(x, cb, 1.0, idx, gain, bias, [1, 5], [2, 0], return_abs=True)
    np.testing.assert_allclose(As, expect[[2, 0]], atol=1e-13)
    # (c) linear codewords: rows a_k * (Greville abscissae)
    t = ko.knots()
    grev = np.array([(t[m + 1] + t[m + 2] + t[m + 3]) / 3 for m in range(10)])
    a = rng.normal(size=K)
    cbl = a[:, None] * grev[None, :]
    xc = np.clip(x, -1, 1)
    expect = np.abs(gain[None] * a[idx][None] * xc[:, :, None] + bias[None]).sum(axis=1)       # [B][out]
    for rule_cb, rule in ((cbl, "bspline"), (a[:, None] * ko.pli_nodes()[None, :], "pli")):
        _, A = ko.vq_layer_forward(x, rule_cb, 1.0, idx, gain, bias, return_abs=True, rule=rule)
        np.testing.assert_allclose(A, expect, atol=1e-13)
        _, As = ko.vq_layer_outputs_at(x, rule_cb, 1.0, idx, gain, bias, [0, 3], [1, 2], return_abs=True, rule=rule)
        np.testing.assert_allclose(As, expect[[0, 3], [1, 2]], atol=1e-13)
    # dense form on its own (the dense baseline's gate)
    coef = rng.normal(size=(n_in, n_out, 10))
    _, Ad = ko.dense_layer_forward(coef, x, return_abs=True)
    ref = np.array([[math.fsum(abs(ko.edge_phi_scalar(coef[i, j], x[b, i])) for i in range(n_in))
                     for j in range(n_out)] for b in range(B)])
    np.testing.assert_allclose(Ad, ref, atol=1e-14)


# ---- block-floating-point codebooks (the BFP8 row of Table 1; the format is a reading) ----------

def test_bfp8_codebook_meaning_and_round_trip():
    """What the twelve bytes of a row mean, by values that need no formula of the oracle's:
    mantissa 1 with exponent e is exactly 2**e (negative exponents included: the byte is signed),
    mantissas scale linearly, the twelfth byte is ignored, `scale` is ignored; decoded rows of the
    generator's encoder lie within half a mantissa step of the shapes they encode; a layer over a
    block-floating-point codebook equals the layer over its decoded rows."""
    rows = np.zeros((6, 12), dtype=np.int8)
    rows[0, :10], rows[0, 10] = 1, 0                       # all ones
    rows[1, :10], rows[1, 10] = np.arange(-5, 5), -3       # q / 8
    rows[2, :10], rows[2, 10] = 127, -126                  # smallest exponent
    rows[3, :10], rows[3, 10] = -127, 5                    # -127 * 32
    rows[4, :10], rows[4, 10], rows[4, 11] = 64, -7, 99    # the last byte carries nothing
    rows[5, 10] = 17                                       # zero mantissas
    C = ko.dequantise_codebook(rows, 123.0)
    assert C.shape == (6, 10) and C.dtype == np.float64
    assert (C[0] == 1.0).all()
    assert np.array_equal(C[1], np.arange(-5, 5) / 8.0)
    assert (C[2] == 127.0 * 2.0 ** -126).all()
    assert (C[3] == -127.0 * 32.0).all()
    assert (C[4] == 0.5).all() and (C[5] == 0.0).all()
    # an Int8 codebook [K][10] keeps its own meaning
    q = np.arange(-5, 5, dtype=np.int8)[None, :]
    assert np.array_equal(ko.dequantise_codebook(q, 0.5), 0.5 * q.astype(np.float64))
    # round trip through the encoder
    rng = np.random.default_rng(17)
    shapes = synth.make_shapes(rng, 400)
    shapes[7] *= 1e-3                                      # a row far smaller than the others keeps its own exponent
    shapes[9] = 0.0
    enc = synth.quantise_shapes_bfp8(shapes)
    assert enc.dtype == np.int8 and enc.shape == (400, 12) and (enc[:, 11] == 0).all()
    dec = ko.dequantise_codebook(enc)
    step = np.exp2(enc[:, 10].astype(np.float64))
    assert (np.abs(dec - shapes.astype(np.float64)) <= 0.5 * step[:, None] * (1 + 1e-12)).all()
    assert (dec[9] == 0).all() and np.abs(dec[7]).max() < 2e-3 and np.abs(dec[7] - shapes[7]).max() < 1e-5
    assert np.abs(enc[:, :10]).max(axis=1).min() >= 0 and (np.abs(enc[np.abs(shapes).max(axis=1) > 0, :10]).max(axis=1) >= 64).all()
    # layer level: equal to the layer over the decoded rows, whatever `scale` says
    P = synth.make_layer(51, 9, 6, 30, cb_dtype="bfp8", gb_dtype="f16")
    assert P.codebook.shape == (30, 12)
    x = synth.make_x(5, 7, 9)
    y_b = ko.vq_layer_forward(x, P.codebook, 55.0, P.idx, P.gain, P.bias)
    y_d = ko.vq_layer_forward(x, ko.dequantise_codebook(P.codebook), 1.0, P.idx, P.gain, P.bias)
    assert np.array_equal(y_b, y_d)
    y_s = ko.vq_layer_forward_scalar(x.tolist(), ko.dequantise_codebook(P.codebook).tolist(), 1.0, P.idx.tolist(),
                                     P.gain.astype(np.float64).tolist(), P.bias.astype(np.float64).tolist())
    np.testing.assert_allclose(y_b, y_s, atol=1e-14)
    # and close to the fp32 layer it was encoded from: |dC| <= step / 2 per entry, weights sum to 1
    F = synth.make_layer(51, 9, 6, 30, cb_dtype="f32", gb_dtype="f16")
    y_f = ko.vq_layer_forward(x, **F.as_dict())
    stepP = np.exp2(P.codebook[:, 10].astype(np.float64))
    bound = (np.abs(P.gain.astype(np.float64)) * 0.5 * stepP[P.idx.astype(np.int64)]).sum(axis=0)
    assert (np.abs(y_b - y_f) <= bound[None, :] + 1e-12).all() and np.abs(y_b - y_f).max() > 0


# ---- the pins bite: a planted mistake in the oracle fails at least one of them ----------

def _pin_suite():
    """The pins that exercise the oracle's arithmetic, as callables."""
    return [test_partition_of_unity_and_support, test_span_matches_scalar_search_and_ends,
            test_closed_form_weights_at_knot_and_midpoint, test_basis_integrals, test_linear_precision_greville,
            test_quadratic_precision_marsden, test_layer_closed_form_linear_shapes, test_constant_codeword,
            test_against_scipy_bspline, test_vq_equals_dense_on_reconstructed,
            test_permutation_linearity_additivity, test_int8_equals_fp32_twin,
            test_head_is_layers_with_tanh_between, test_pli_nodes_and_index,
            test_pli_is_linear_interpolation_numpy_interp,
            test_pli_reproduces_node_values_linear_functions_and_unity,
            test_pli_layer_closed_forms_and_scalar_definition, test_q8_gain_bias_meaning,
            test_q8_round_trip_through_the_encoder, test_assignment_brute_force_and_kdtree,
            test_assignment_recovers_a_layer_built_from_the_codebook,
            test_abs_sum_A_against_the_scalar_definition_and_closed_forms,
            test_bfp8_codebook_meaning_and_round_trip,
            lambda: test_scalar_definition_vs_vectorised(False), lambda: test_scalar_definition_vs_vectorised(True)]


def _fails_some_pin():
    for pin in _pin_suite():
        try:
            pin()
        except AssertionError:
            return True
        except Exception:
            return True
    return False


def _mutations():
    """(name, attribute of the oracle module, replacement) - each a plausible slip."""
    real = {k: getattr(ko, k) for k in ("knots", "basis_matrix", "reconstruct_coefficients", "dequantise_codebook",
                                        "dense_layer_forward", "pli_matrix", "pli_nodes", "clamp_input",
                                        "vq_head_forward", "dequantise_gain_bias", "normalise_grids",
                                        "squared_distances", "vq_layer_outputs_at")}

    def knots_shifted():                       # knot vector off by one interval
        return real["knots"]() + 2.0 / 7.0

    def knots_wrong_spacing():                 # 8 intervals instead of 7
        return np.array([(2.0 * (m - 3) - 8) / 8 for m in range(14)])

    def basis_reversed(x, *a, **k):            # coefficient order reversed
        return real["basis_matrix"](x, *a, **k)[..., ::-1]

    def basis_dropped_term(x, *a, **k):        # last basis lost
        Bm = real["basis_matrix"](x, *a, **k).copy()
        Bm[..., -1] = 0.0
        return Bm

    def recon_no_bias(cb, scale, idx, gain, bias, gb_params=None):
        g, b = real["dequantise_gain_bias"](gain, bias, gb_params)
        return real["reconstruct_coefficients"](cb, scale, idx, g, np.zeros_like(b))

    def recon_transposed_idx(cb, scale, idx, gain, bias, gb_params=None):
        idx = np.asarray(idx)
        if idx.shape[0] == idx.shape[1]:
            idx = idx.T
        else:
            idx = idx[::-1]
        return real["reconstruct_coefficients"](cb, scale, idx, gain, bias, gb_params)

    def recon_gain_on_bias(cb, scale, idx, gain, bias, gb_params=None):     # g * (C + b) instead of g * C + b
        c = real["dequantise_codebook"](cb, scale)
        g, b = real["dequantise_gain_bias"](gain, bias, gb_params)
        return g[..., None] * (c[np.asarray(idx).astype(np.int64)] + b[..., None])

    def q8_zero_code_is_smallest_gain(gain, bias, gb_params=None):       # code 0 not treated as zero
        if gb_params is None:
            return real["dequantise_gain_bias"](gain, bias, gb_params)
        lo, step, bscale = (float(v) for v in gb_params)
        return np.exp2(lo + step * np.asarray(gain).astype(np.float64)), bscale * np.asarray(bias).astype(np.float64)

    def q8_bias_unsigned(gain, bias, gb_params=None):                    # bias byte read as unsigned
        if gb_params is None:
            return real["dequantise_gain_bias"](gain, bias, gb_params)
        g, _ = real["dequantise_gain_bias"](gain, bias, gb_params)
        return g, float(gb_params[2]) * np.asarray(bias).view(np.uint8).astype(np.float64)

    def q8_natural_log(gain, bias, gb_params=None):                      # e ** instead of 2 **
        if gb_params is None:
            return real["dequantise_gain_bias"](gain, bias, gb_params)
        g, b = real["dequantise_gain_bias"](gain, bias, gb_params)
        lo, step = float(gb_params[0]), float(gb_params[1])
        c = np.asarray(gain).astype(np.float64)
        return np.where(np.asarray(gain) == 0, 0.0, np.exp(lo + step * c)), b

    def dequant_ignores_scale(cb, scale=1.0):
        return np.asarray(cb).astype(np.float64)

    def dequant_unsigned(cb, scale=1.0):        # int8 read as uint8
        cb = np.asarray(cb)
        if cb.dtype == np.int8:
            return np.float64(np.float32(scale)) * cb.view(np.uint8).astype(np.float64)
        return cb.astype(np.float64)

    def dense_sums_wrong_axis(coef, x, return_abs=False, rule="bspline"):
        coef = np.asarray(coef, dtype=np.float64)
        y = real["dense_layer_forward"](np.ascontiguousarray(coef[:, ::-1, :]), x, rule=rule)     # outputs reversed
        return (y, np.abs(y)) if return_abs else y

    def dense_abs_per_coefficient(coef, x, return_abs=False, rule="bspline"):       # A = sum_i sum_m |B_m c_m|: too large
        y = real["dense_layer_forward"](coef, x, rule=rule)
        if not return_abs:
            return y
        Bm = ko.design_matrix(np.asarray(x, dtype=np.float64), rule)
        return y, np.einsum("bim,ijm->bj", np.abs(Bm), np.abs(np.asarray(coef, dtype=np.float64)))

    def outputs_at_abs_of_the_sum(x, cb, scale, idx, gain, bias, bs, js, return_abs=False, rule="bspline", gb_params=None):
        out = real["vq_layer_outputs_at"](x, cb, scale, idx, gain, bias, bs, js, rule=rule, gb_params=gb_params)
        return (out, np.abs(out)) if return_abs else out      # A = |sum_i phi|: too small

    def outputs_at_abs_per_coefficient(x, cb, scale, idx, gain, bias, bs, js, return_abs=False, rule="bspline", gb_params=None):
        out = real["vq_layer_outputs_at"](x, cb, scale, idx, gain, bias, bs, js, rule=rule, gb_params=gb_params)
        if not return_abs:
            return out
        coef = real["reconstruct_coefficients"](cb, scale, idx, gain, bias, gb_params)
        Bm = ko.design_matrix(np.asarray(x, dtype=np.float64), rule)
        return out, np.array([(np.abs(Bm[b]) * np.abs(coef[:, j])).sum() for b, j in zip(bs, js)])

    def bfp8_exponent_unsigned(cb, scale=1.0):           # exponent byte read as unsigned
        cb = np.asarray(cb)
        if cb.dtype == np.int8 and cb.shape[-1] == 12:
            return cb[..., :10].astype(np.float64) * np.exp2(cb[..., 10].view(np.uint8).astype(np.float64))[..., None]
        return real["dequantise_codebook"](cb, scale)

    def bfp8_exponent_negated(cb, scale=1.0):            # q / 2**e instead of q * 2**e
        cb = np.asarray(cb)
        if cb.dtype == np.int8 and cb.shape[-1] == 12:
            return cb[..., :10].astype(np.float64) * np.exp2(-cb[..., 10].astype(np.float64))[..., None]
        return real["dequantise_codebook"](cb, scale)

    def bfp8_scale_applied(cb, scale=1.0):               # the layer scale wrongly applied on top
        cb = np.asarray(cb)
        out = real["dequantise_codebook"](cb, scale)
        return out * float(scale) if (cb.dtype == np.int8 and cb.shape[-1] == 12) else out

    def bfp8_exponent_from_last_byte(cb, scale=1.0):     # exponent taken from byte 11 instead of byte 10
        cb = np.asarray(cb)
        if cb.dtype == np.int8 and cb.shape[-1] == 12:
            return cb[..., :10].astype(np.float64) * np.exp2(cb[..., 11].astype(np.float64))[..., None]
        return real["dequantise_codebook"](cb, scale)

    def pli_swapped_taps(x):                   # u and 1-u exchanged
        W = real["pli_matrix"](x)
        k = ko.pli_index(np.asarray(x, dtype=np.float64).reshape(-1)).astype(np.int64)
        flat = W.reshape(-1, ko.G)
        o = np.zeros_like(flat)
        r = np.arange(flat.shape[0])
        o[r, k] = flat[r, k + 1]
        o[r, k + 1] = flat[r, k]
        return o.reshape(W.shape)

    def pli_nodes_ten_intervals():             # dx = 2/G instead of 2/(G-1)
        return np.array([-1.0 + 2.0 * k / ko.G for k in range(ko.G)])

    def no_clamp(x):
        return np.asarray(x, dtype=np.float64)

    def head_tanh_after_last(x, layers, return_hidden=False, rule="bspline"):
        out = real["vq_head_forward"](x, layers, return_hidden=return_hidden, rule=rule)
        if return_hidden:
            return np.tanh(out[0]), out[1]
        return np.tanh(out)

    def normalise_by_std(coef):                                         # unit variance instead of unit norm
        n, g, b = real["normalise_grids"](coef)
        return n * math.sqrt(ko.G), g / math.sqrt(ko.G), b

    def normalise_without_centring(coef):
        c = np.asarray(coef, dtype=np.float64)
        g = np.sqrt((c * c).sum(axis=-1))
        return c / np.where(g > 0, g, 1.0)[..., None], g, np.zeros(c.shape[:-1])

    def distances_as_dot_products(shapes, codebook):                     # similarity mistaken for distance
        return np.asarray(shapes, dtype=np.float64).reshape(-1, ko.G) @ np.asarray(codebook, dtype=np.float64).T

    return [("knots shifted", "knots", knots_shifted), ("8 intervals", "knots", knots_wrong_spacing),
            ("bases reversed", "basis_matrix", basis_reversed), ("basis dropped", "basis_matrix", basis_dropped_term),
            ("bias dropped", "reconstruct_coefficients", recon_no_bias),
            ("idx transposed", "reconstruct_coefficients", recon_transposed_idx),
            ("gain applied to bias", "reconstruct_coefficients", recon_gain_on_bias),
            ("scale ignored", "dequantise_codebook", dequant_ignores_scale),
            ("int8 read unsigned", "dequantise_codebook", dequant_unsigned),
            ("outputs reversed", "dense_layer_forward", dense_sums_wrong_axis),
            ("taps swapped", "pli_matrix", pli_swapped_taps), ("dx = 2/G", "pli_nodes", pli_nodes_ten_intervals),
            ("no clamp", "clamp_input", no_clamp), ("tanh after last layer", "vq_head_forward", head_tanh_after_last),
            ("gain code 0 not zero", "dequantise_gain_bias", q8_zero_code_is_smallest_gain),
            ("bias byte unsigned", "dequantise_gain_bias", q8_bias_unsigned),
            ("natural instead of binary log", "dequantise_gain_bias", q8_natural_log),
            ("unit variance instead of unit norm", "normalise_grids", normalise_by_std),
            ("grids not centred", "normalise_grids", normalise_without_centring),
            ("dot product used as a distance", "squared_distances", distances_as_dot_products),
            ("block exponent read unsigned", "dequantise_codebook", bfp8_exponent_unsigned),
            ("block exponent negated", "dequantise_codebook", bfp8_exponent_negated),
            ("layer scale applied to a block codebook", "dequantise_codebook", bfp8_scale_applied),
            ("block exponent taken from the wrong byte", "dequantise_codebook", bfp8_exponent_from_last_byte),
            ("A summed per coefficient (dense form)", "dense_layer_forward", dense_abs_per_coefficient),
            ("A taken as |sum| (sampled form)", "vq_layer_outputs_at", outputs_at_abs_of_the_sum),
            ("A summed per coefficient (sampled form)", "vq_layer_outputs_at", outputs_at_abs_per_coefficient)]


def test_pins_pass_unmutated():
    assert not _fails_some_pin()


@pytest.mark.parametrize("name,attr,repl", _mutations(), ids=[m[0] for m in _mutations()])
def test_planted_mistake_fails_a_pin(monkeypatch, name, attr, repl):
    monkeypatch.setattr(ko, attr, repl)
    assert _fails_some_pin(), f"no pin notices: {name}"


# ---- byte-coded gain / bias (paper §4.2: logarithmic Int8 gain, linear Int8 bias) --------

def test_q8_gain_bias_meaning():
    """What the codes mean, pinned by values that need no formula of the oracle's: with
    lo = -8 and step = 1/16 every 16th code is an exact power of two; code 0 is zero; the
    grid is strictly increasing; bias codes are a plain multiple."""
    qg = np.arange(256, dtype=np.uint8)
    qb = np.arange(-128, 128).astype(np.int8)
    g, b = ko.dequantise_gain_bias(qg, qb, (np.float32(-8.0), np.float32(1.0 / 16.0), np.float32(0.25)))
    assert g[0] == 0.0
    for c in range(16, 256, 16):
        assert g[c] == 2.0 ** (-8 + c // 16)
    assert (np.diff(g[1:]) > 0).all()
    assert np.allclose(g[2:] / g[1:-1], 2.0 ** (1.0 / 16.0), rtol=1e-15)
    assert np.array_equal(b, 0.25 * np.arange(-128, 128))
    # floating arrays pass through untouched
    gf, bf = ko.dequantise_gain_bias(np.float16([0.5, 0.25]), np.float32([1.5, -2.0]))
    assert gf.tolist() == [0.5, 0.25] and bf.tolist() == [1.5, -2.0]


def test_q8_round_trip_through_the_encoder():
    """Encoder (generator side) and meaning (oracle) fit together: decoded gains are within
    half a logarithmic step of the originals, biases within half a linear step, zeros stay zero."""
    rng = np.random.default_rng(4)
    gain = np.abs(rng.normal(0, 0.1, size=(40, 30)))
    gain[3, 4] = 0.0
    bias = rng.normal(0, 0.01, size=(40, 30))
    qg, qb, params = synth.encode_gain_bias_q8(gain, bias)
    g, b = ko.dequantise_gain_bias(qg, qb, params)
    assert g[3, 4] == 0.0 and qg[3, 4] == 0
    pos = gain > 0
    assert np.abs(np.log2(g[pos]) - np.log2(gain[pos])).max() <= 0.5 * float(params[1]) * (1 + 1e-6)
    assert np.abs(b - bias).max() <= 0.5 * float(params[2]) * (1 + 1e-6)
    # a layer in the byte-coded format equals the floating layer built from the decoded values
    P = synth.make_layer(9, 12, 7, 50, cb_dtype="i8", gb_dtype="q8")
    x = synth.make_x(2, 5, 12)
    gd, bd = ko.dequantise_gain_bias(P.gain, P.bias, P.gb_params)
    y_codes = ko.vq_layer_forward(x, **P.as_dict())
    y_float = ko.vq_layer_forward(x, P.codebook, P.scale, P.idx, gd, bd)
    assert np.array_equal(y_codes, y_float)
    assert P.metadata_bytes == 4 * P.edges                 # 32 bits per edge at K <= 2^16 (§4.2)


# ---- compression side: normalise + nearest codebook shape (paper §4.2 steps 1 and 3) ---------

def test_assignment_brute_force_and_kdtree():
    from scipy.spatial import cKDTree
    rng = np.random.default_rng(8)
    coef = rng.standard_normal((6, 5, ko.G)) * rng.uniform(0.1, 3.0, size=(6, 5, 1)) + rng.normal(size=(6, 5, 1))
    cb = synth.make_shapes(rng, 300).astype(np.float64)
    idx, gain, bias, dmin = ko.assign_edges(coef, cb)
    for i in range(6):
        for j in range(5):
            grid = coef[i, j]
            b = sum(grid) / ko.G
            cen = [v - b for v in grid]
            g = math.sqrt(sum(v * v for v in cen))
            shape = [v / g for v in cen]
            d = [sum((shape[m] - cb[k][m]) ** 2 for m in range(ko.G)) for k in range(300)]
            k_best = min(range(300), key=lambda k: d[k])
            assert idx[i, j] == k_best and abs(dmin[i, j] - d[k_best]) < 1e-12
            assert abs(gain[i, j] - g) < 1e-12 and abs(bias[i, j] - b) < 1e-12
    shapes, _, _ = ko.normalise_grids(coef)
    assert np.abs(shapes.sum(axis=-1)).max() < 1e-12 and np.abs((shapes ** 2).sum(axis=-1) - 1).max() < 1e-12
    dist, nn = cKDTree(cb).query(shapes.reshape(-1, ko.G), k=1)            # library nearest-neighbour search
    assert np.array_equal(nn, idx.reshape(-1)) and np.abs(dist ** 2 - dmin.reshape(-1)).max() < 1e-12


def test_assignment_recovers_a_layer_built_from_the_codebook():
    """c = g * C[k] + b with zero-mean unit-norm shapes: the assignment returns k, g, b and R^2 = 1;
    an affine change of a grid changes gain and bias but not its index; a constant grid has gain 0."""
    rng = np.random.default_rng(9)
    cb = synth.make_shapes(rng, 500).astype(np.float64)
    cb -= cb.mean(axis=1, keepdims=True)                  # zero mean and unit norm to float64 accuracy
    cb /= np.linalg.norm(cb, axis=1, keepdims=True)
    k = rng.integers(0, 500, size=(7, 9))
    g = rng.uniform(0.05, 2.0, size=(7, 9))
    b = rng.normal(size=(7, 9))
    coef = g[..., None] * cb[k] + b[..., None]
    idx, gain, bias, dmin = ko.assign_edges(coef, cb)
    assert np.array_equal(idx, k) and np.abs(gain - g).max() < 1e-12 and np.abs(bias - b).max() < 1e-12
    assert dmin.max() < 1e-24
    assert abs(ko.r_squared(coef, cb, idx, gain, bias) - 1.0) < 1e-12
    noisy = coef + 0.05 * rng.standard_normal(coef.shape)
    i1, g1, b1, _ = ko.assign_edges(noisy, cb)
    i2, g2, b2, _ = ko.assign_edges(3.0 * noisy - 1.5, cb)
    assert np.array_equal(i1, i2) and np.abs(g2 - 3.0 * g1).max() < 1e-12 and np.abs(b2 - (3.0 * b1 - 1.5)).max() < 1e-12
    r2 = ko.r_squared(noisy, cb, i1, g1, b1)
    assert 0.5 < r2 < 1.0
    # R^2 against its definition written with numpy's variance
    rec = g1[..., None] * cb[i1] + b1[..., None]
    assert abs(r2 - (1 - ((noisy - rec) ** 2).mean() / noisy.var())) < 1e-12
    flat = np.full((1, 1, ko.G), 0.7)
    i0, g0, b0, _ = ko.assign_edges(flat, cb)
    assert g0[0, 0] == 0.0 and abs(b0[0, 0] - 0.7) < 1e-15


@pytest.mark.parametrize("rule", ["bspline", "pli"])
def test_support_never_holds_both_entries_m_and_m_plus_5(rule):
    """The streaming matrix-core kernel orders a codeword's ten entries in pairs (m, m + 5) and
    relies on at most one entry of a pair carrying weight, whatever x: the four nonzero cubic
    bases (and the two taps of the interpolation rule) are consecutive.  Checked on the
    oracle's own weights, at random points, at the knots and at both ends."""
    rng = np.random.default_rng(11)
    x = np.concatenate([rng.uniform(-1.0, 1.0, 20000), ko.knots()[3:11], ko.pli_nodes(), [-1.0, 1.0, -1.5, 1.5]])
    W = ko.design_matrix(x, rule)                       # [n][10]
    assert W.shape == (x.size, 10)
    nz = W != 0.0
    assert not (nz[:, :5] & nz[:, 5:]).any()
    # and the nonzero entries are consecutive: last - first + 1 <= 4
    first = np.argmax(nz, axis=1)
    last = 9 - np.argmax(nz[:, ::-1], axis=1)
    assert (last - first <= 3).all() and (nz.sum(axis=1) >= 1).all()
