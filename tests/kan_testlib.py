"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np

from oracle import kan_oracle as ko

TOL_FP32 = 1e-5     # gather path: relative bound stated for the fp32 kernels
TOL_MFMA = 2e-2     # matrix-core path with fp16 operands (the bound stated for 16-bit operands)


def gpu_layers(param_list):
    from paper_2512_15742_amd import binding as kb
    return [kb.VQLayer(p) for p in param_list]


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_layer_output(y_gpu, x, P, tol, n_samples=48, seed=0, full=True):
    """Compare y_gpu [B][out] (numpy) with the oracle for layer params P.

    full=True: the whole tensor against the headline metric max|dy|/max|y|, and
    per-element |dy| <= tol * A on sampled (b, j) with A = sum_i |phi_ij|.
    full=False: only the sampled outputs (sizes the oracle cannot cover whole);
    the headline scale is then the largest |y| among the samples.
    """
    B, n_out = y_gpu.shape
    rng = np.random.default_rng(seed)
    bs = rng.integers(0, B, size=n_samples)
    js = rng.integers(0, n_out, size=n_samples)
    bs[0], js[0] = 0, 0
    bs[1], js[1] = B - 1, n_out - 1
    ys, As = ko.vq_layer_outputs_at(x, P.codebook, P.scale, P.idx, P.gain, P.bias, bs, js, return_abs=True)
    d = np.abs(y_gpu[bs, js].astype(np.float64) - ys)
    strict = float((d / As).max())
    assert strict <= tol, f"strict per-element error {strict:.3e} > {tol}"
    if full:
        y_ref = ko.vq_layer_forward(x, P.codebook, P.scale, P.idx, P.gain, P.bias)
        rep = ko.error_report(y_gpu, y_ref)
    else:
        rep = {"headline": float(d.max() / np.abs(ys).max())}
    assert rep["headline"] <= tol, f"headline error {rep['headline']:.3e} > {tol}"
    rep["strict"] = strict
    return rep


def check_dense_output(y_gpu, x, coef, tol):
    y_ref, A = ko.dense_layer_forward(coef, x, return_abs=True)
    rep = ko.error_report(y_gpu, y_ref, A)
    assert rep["headline"] <= tol and rep["strict"] <= tol, rep
    return rep


def check_head_layer_by_layer(kb, Ls, Ps, x, path, tol, rows=None, rule="bspline"):
    """Every layer of a head at `tol` on identical fp32 inputs: layer l runs through the single-layer
    entry point on the activation the GPU itself produced for layers 1..l-1 (tanh of its own fp32
    output), and the oracle evaluates layer l on exactly those fp32 numbers.  Errors of earlier
    layers therefore do not enter a later layer's figure and no factor for depth is needed.
    Returns the GPU's final output [B][out] (numpy) of that chain and the worst figure."""
    import torch
    a = to_dev(x)
    worst = 0.0
    y = None
    for l, (L, P) in enumerate(zip(Ls, Ps)):
        y_t = kb.kan_vq_layer_forward(L, a, path=path)
        y = y_t.cpu().numpy()
        a_np = a.cpu().numpy()
        sel = np.arange(a_np.shape[0]) if rows is None else rows
        y_ref = ko.vq_layer_forward(a_np[sel], **P.as_dict(), rule=rule)
        rep = ko.error_report(y[sel], y_ref)
        assert np.isfinite(y).all() and rep["headline"] <= tol, (l, rep)
        worst = max(worst, rep["headline"])
        a = torch.tanh(y_t)
    return y, worst
