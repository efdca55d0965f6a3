"""GPU parity for the precise path at large batch: the streaming matrix-core kernels run on
operands split into high and low fp16 parts (hi*hi + hi*lo + lo*hi), which must hold the fp32
bound of the precise path (1e-5), not the fp16 path's.  Shapes, dtypes, both edge rules,
multi-layer hand-overs, several heads, and coefficients small enough to be fp16 subnormals."""
import dataclasses

import numpy as np
import pytest

from oracle import kan_oracle as ko
from paper_2512_15742_amd import synth

from kan_testlib import TOL_FP32, check_layer_output, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def kb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2512_15742_amd import binding
    binding.lib()
    return binding


def test_split_takes_over_the_precise_path_at_large_batch(kb):
    P = synth.make_layer(1, 256, 128, 4096, cb_dtype="i8", gb_dtype="f16")
    L = kb.VQLayer(P)
    assert kb.kan_vq_planned_kernel(L, 64, 1, kb.KAN_PATH_GATHER) == "kan_fused_f32"
    assert kb.kan_vq_planned_kernel(L, 65, 1, kb.KAN_PATH_GATHER) == "kan_mfma_split"
    assert kb.kan_vq_planned_kernel(L, 4096, 1, kb.KAN_PATH_GATHER) == "kan_mfma_split"
    assert kb.kan_vq_planned_kernel(L, 4096, 1, kb.KAN_PATH_MFMA) == "kan_mfma"
    assert kb.kan_vq_planned_kernel(L, 4096, 1, kb.KAN_PATH_AUTO) == "kan_mfma"


@pytest.mark.parametrize("n_in,n_out,B,cb,gb,idx", [
    (8, 32, 129, "f32", "f32", "u16"), (130, 67, 200, "i8", "f16", "u16"), (257, 130, 150, "f16", "f16", "u32"),
    (64, 520, 133, "i8", "q8", "u16"), (1000, 264, 300, "f32", "f32", "u16"), (2052, 300, 200, "i8", "f32", "u32"),
    (2048, 8, 129, "f32", "f16", "u16"), (70, 1900, 2100, "i8", "f16", "u16"),
    (100, 1000, 1100, "i8", "f16", "u16"), (16, 2048, 1030, "f32", "f32", "u32")])    # eight-wave tiles: 21 and 3 passes' steps
def test_split_shapes_and_dtypes(kb, n_in, n_out, B, cb, gb, idx):
    P = synth.make_layer(n_in * 7 + n_out, n_in, n_out, 1000, cb_dtype=cb, gb_dtype=gb, idx_dtype=idx)
    x = synth.make_x(B, B, n_in)
    x[0, 0] = 1.0
    x[-1, -1] = -1.0
    L = kb.VQLayer(P)
    assert kb.kan_vq_planned_kernel(L, B, 1, kb.KAN_PATH_GATHER) == "kan_mfma_split"
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    if B * n_in * n_out <= 1.5e8:
        y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
        rep = ko.error_report(y, y_ref, A)
        assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, rep
    else:
        check_layer_output(y, x, P, TOL_FP32, n_samples=96, full=False, seed=B)
        rows = np.array([0, 63, 64, 127, 128, B // 2, B - 129, B - 1])
        y_ref, A = ko.vq_layer_forward(x[rows], **P.as_dict(), return_abs=True)
        rep = ko.error_report(y[rows], y_ref, A)
        assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, rep


def test_split_keeps_coefficients_and_weights_below_the_fp16_normal_range(kb):
    """An fp32 codebook whose entries span six decades, gains down to 1e-6 and inputs a hair
    from the knots: high parts that fp16 can only hold as subnormals (or not at all) must be
    made up for by the low parts."""
    n_in, n_out, B = 300, 130, 160
    P = synth.make_layer(41, n_in, n_out, 500, cb_dtype="f32", gb_dtype="f32")
    rng = np.random.default_rng(3)
    cb = (P.codebook * 10.0 ** rng.uniform(-6, 0, size=P.codebook.shape)).astype(np.float32)
    gain = (P.gain * 10.0 ** rng.uniform(-4, 0, size=P.gain.shape)).astype(np.float32)
    P2 = dataclasses.replace(P, codebook=cb, gain=gain)
    x = synth.make_x(7, B, n_in)
    knots = ko.knots()[3:11].astype(np.float32)
    x[:, ::3] = (knots[rng.integers(0, 8, size=x[:, ::3].shape)] + rng.uniform(-1e-3, 1e-3, size=x[:, ::3].shape)).astype(np.float32)
    L = kb.VQLayer(P2)
    assert kb.kan_vq_planned_kernel(L, B, 1, kb.KAN_PATH_GATHER) == "kan_mfma_split"
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    y_ref, A = ko.vq_layer_forward(x, **P2.as_dict(), return_abs=True)
    rep = ko.error_report(y, y_ref, A)
    assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, rep


def test_large_gains_up_to_the_fp16_range_and_the_range_report(kb):
    """The coefficient operand of the matrix-core kernels is gain * q in fp16: gains of a few
    hundred with Int8 codes reach the tens of thousands, still below 65504.  kan_vq_coef_range
    reports the smallest nonzero and the largest such product bit for bit; inside the supported
    range the split form keeps the fp32 bound and the one-pass form the fp16 bound."""
    n_in, n_out, B = 200, 130, 150
    P = synth.make_layer(43, n_in, n_out, 700, cb_dtype="i8", gb_dtype="f32")
    rng = np.random.default_rng(5)
    gain = (400.0 * rng.uniform(0.01, 1.0, size=P.gain.shape)).astype(np.float32)
    gain[3, 5] = 0.0
    P2 = dataclasses.replace(P, gain=gain)
    L = kb.VQLayer(P2)
    lo, hi = kb.kan_vq_coef_range(L)
    prod = np.abs(gain.astype(np.float32)[:, :, None] * P2.codebook[P2.idx.astype(np.int64)].astype(np.float32))
    assert hi == float(prod.max()) and lo == float(prod[prod > 0].min())
    assert 6.1e-5 <= lo and hi < 65504 and hi > 4e4
    x = synth.make_x(9, B, n_in)
    y_ref, A = ko.vq_layer_forward(x, **P2.as_dict(), return_abs=True)
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    rep = ko.error_report(y, y_ref, A)
    assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, rep
    y16 = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_MFMA).cpu().numpy()
    rep16 = ko.error_report(y16, y_ref, A)
    assert rep16["headline"] <= 2e-2 and rep16["strict"] <= 2e-2, rep16
    # all-zero gains: nothing nonzero to report
    Z = kb.VQLayer(dataclasses.replace(P, gain=np.zeros_like(P.gain)))
    lo0, hi0 = kb.kan_vq_coef_range(Z)
    assert lo0 == float("inf") and hi0 == 0.0


@pytest.mark.parametrize("B", [130, 700])
def test_split_pli_rule(kb, B):
    P = synth.make_layer(63, 130, 70, 4000, cb_dtype="f16", gb_dtype="f16")
    x = synth.make_x(B + 3, B, 130)
    L = kb.VQLayer(P, rule=kb.KAN_RULE_PLI2)
    assert kb.kan_vq_planned_kernel(L, B, 1, kb.KAN_PATH_GATHER) == "kan_mfma_split"
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True, rule="pli")
    rep = ko.error_report(y, y_ref, A)
    assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, rep


@pytest.mark.parametrize("B,n_heads", [(150, 1), (120, 3), (4200, 1)])
def test_split_three_layer_head(kb, B, n_heads):
    """Hand-overs: few slices (the next layer's basis preparation adds them) and many (the
    reduction pass writes the hidden activation); a second call gives the same bits."""
    dims = [(520, 264), (264, 130), (130, 21)]
    heads_p = [[synth.make_layer(900 + 10 * h + l, i, o, 20000, cb_dtype="i8", gb_dtype="f16")
                for l, (i, o) in enumerate(dims)] for h in range(n_heads)]
    heads = [[kb.VQLayer(p) for p in ps] for ps in heads_p]
    x = synth.make_x(B + n_heads, B, 520)
    xd = to_dev(x)
    y = kb.kan_vq_head_forward(heads, xd, path=kb.KAN_PATH_GATHER)
    y2 = kb.kan_vq_head_forward(heads, xd, path=kb.KAN_PATH_GATHER)
    assert torch.equal(y, y2)
    y = y.cpu().numpy()
    rows = np.arange(B) if B <= 200 else np.sort(np.random.default_rng(B).choice(B, 64, replace=False))
    for h in range(n_heads):
        y_ref = ko.vq_head_forward(x[rows], [p.as_dict() for p in heads_p[h]])
        assert ko.error_report(y[h][rows], y_ref)["headline"] <= TOL_FP32, h


@pytest.mark.parametrize("B", [256, 1024])
def test_split_config2_and_config3(kb, B):
    (P,), x = synth.config2(B)
    L = kb.VQLayer(P)
    assert kb.kan_vq_planned_kernel(L, B, 1, kb.KAN_PATH_GATHER) == "kan_mfma_split"
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    check_layer_output(y, x, P, TOL_FP32, n_samples=96, full=False, seed=B)
    Ps, x3 = synth.config3(B)
    Ls = [kb.VQLayer(p) for p in Ps]
    y3 = kb.kan_vq_head_forward([Ls], to_dev(x3), path=kb.KAN_PATH_GATHER)[0].cpu().numpy()
    rows = np.unique(np.concatenate([np.arange(0, B, 64), np.random.default_rng(B).choice(B, 16, replace=False)]))
    y_ref = ko.vq_head_forward(x3[rows], [p.as_dict() for p in Ps])
    assert ko.error_report(y3[rows], y_ref)["headline"] <= TOL_FP32


# ---- the dense baseline on the same split operands -----------------------------------

@pytest.mark.parametrize("n_in,n_out,B", [(8, 32, 129), (130, 67, 200), (257, 130, 150), (64, 520, 133),
                                          (1000, 264, 300), (2052, 70, 112), (33, 1, 500), (300, 40, 17)])
def test_dense_baseline_split_form(kb, n_in, n_out, B):
    """The dense layer at batch >= 17 runs the same three-pass contraction on coefficients it
    splits itself; below that it stays on the fp32 FMA kernel.  Both against the oracle's
    dense layer, and against each other across the switch (the first 16 rows again)."""
    rng = np.random.default_rng(n_in * 13 + n_out)
    coef = (rng.standard_normal((n_in, n_out, 10)) * rng.uniform(1e-3, 2.0, (n_in, n_out, 1))).astype(np.float32)
    coef[0, 0, :] = 1e-6                      # below fp16's normal range
    x = synth.make_x(B + 5, B, n_in)
    x[0, 0] = 1.0
    x[-1, -1] = -1.0
    cd = to_dev(coef)
    y = kb.kan_dense_layer_forward(cd, to_dev(x)).cpu().numpy()
    y_ref, A = ko.dense_layer_forward(coef, x, return_abs=True)
    rep = ko.error_report(y, y_ref, A)
    assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, rep
    y_small = kb.kan_dense_layer_forward(cd, to_dev(x[:16])).cpu().numpy()
    assert np.abs(y_small - y[:16]).max() <= 2 * TOL_FP32 * np.abs(y_ref).max()


def test_dense_baseline_split_config2_twin(kb):
    (P,), x = synth.config2(256)
    coef = ko.reconstruct_coefficients(**P.as_dict()).astype(np.float32)
    xd = to_dev(x)
    yd = kb.kan_dense_layer_forward(to_dev(coef), xd).cpu().numpy()
    y = kb.kan_vq_layer_forward(kb.VQLayer(P), xd, path=kb.KAN_PATH_GATHER).cpu().numpy()
    y_ref = ko.dense_layer_forward(coef, x)
    assert ko.error_report(yd, y_ref)["headline"] <= TOL_FP32
    assert np.abs(yd - y).max() <= 2 * TOL_FP32 * np.abs(y_ref).max()


def test_dense_planned_kernel(kb):
    assert kb.kan_dense_planned_kernel(2048, 512, 16) == "kan_dense"
    assert kb.kan_dense_planned_kernel(2048, 512, 17) == "kan_dense_split"
    assert kb.kan_dense_planned_kernel(0, 512, 112) == "invalid"


def test_split_config5_sampled(kb):
    """The largest configured layer (4096 -> 4096, K = 262,144, batch 8192) through the
    three-pass form: sampled outputs and whole rows against the oracle at the fp32 bound."""
    (P,), x = synth.config5("i8")
    L = kb.VQLayer(P)
    assert kb.kan_vq_planned_kernel(L, x.shape[0], 1, kb.KAN_PATH_GATHER) == "kan_mfma_split"
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    assert np.isfinite(y).all()
    rep = check_layer_output(y, x, P, TOL_FP32, n_samples=64, full=False, seed=55)
    rows = np.array([0, 127, 128, 4095, 8191])
    y_ref, A = ko.vq_layer_forward(x[rows], **P.as_dict(), return_abs=True)
    rep_rows = ko.error_report(y[rows], y_ref, A)
    print("config5 precise", rep, rep_rows)
    assert rep_rows["headline"] <= TOL_FP32 and rep_rows["strict"] <= TOL_FP32, rep_rows
