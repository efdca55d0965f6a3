"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np

from oracle import kan_oracle as ko

TOL_FP32 = 1e-5     # gather path: relative bound stated for the fp32 kernels
TOL_MFMA = 2e-2     # bf16 matrix-core path


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
