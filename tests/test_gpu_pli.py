"""GPU parity of the runtime operator's two-tap rule (linear interpolation between two
codeword entries, paper sections 4.1 and 4.3) through every kernel family: the lookup index
is compared bit for bit, outputs under the same bounds as the cubic rule."""
import numpy as np
import pytest

from oracle import kan_oracle as ko
from paper_2512_15742_amd import synth

from kan_testlib import TOL_FP32, TOL_MFMA, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def kb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2512_15742_amd import binding
    binding.lib()
    return binding


def _probe():
    n = ko.pli_nodes()
    pts = [np.linspace(-1, 1, 4099, dtype=np.float64).astype(np.float32),
           np.random.default_rng(0).uniform(-1, 1, 200000).astype(np.float32),
           np.array([-1.0, 1.0, -0.0, 0.0, -1.5, 3.0, -np.inf, np.inf, 1e-45, -1e-45], dtype=np.float32)]
    for k in n:
        f = np.float32(k)
        nb = [f]
        lo = hi = f
        for _ in range(4):
            lo = np.nextafter(lo, np.float32(-4))
            hi = np.nextafter(hi, np.float32(4))
            nb += [lo, hi]
        pts.append(np.array(nb, dtype=np.float32))
    return np.concatenate(pts)


def test_pli_index_bit_exact_and_weights(kb):
    x = _probe()
    index, w = kb.kan_pli_basis(to_dev(x))
    index, w = index.cpu().numpy(), w.cpu().numpy()
    ref_k = ko.pli_index(x.astype(np.float64))
    assert np.array_equal(index, ref_k)
    W = ko.pli_matrix(x.astype(np.float64))
    ref_w = np.take_along_axis(W, ref_k[:, None].astype(np.int64) + np.arange(2)[None, :], axis=1)
    assert np.abs(w.astype(np.float64) - ref_w).max() <= 6e-8
    e, w2 = kb.kan_pli_basis(torch.empty(0, dtype=torch.float32, device="cuda"))
    assert e.numel() == 0 and w2.shape == (0, 2)


@pytest.mark.parametrize("variant", [0, 1])
def test_pli_window_routines_index_bit_exact(kb, variant):
    """The two-tap rule as the kernels carry it - a window of four entries starting at min(k, 6)
    with the taps 1 - u, u at offset k - start - from both device routines (variant 1: the one of
    the fused kernel and of the basis preparation), index bit for bit against the oracle's search."""
    x = _probe()
    start, w = kb.kan_basis_window(to_dev(x), rule=kb.KAN_RULE_PLI2, variant=variant)
    start, w = start.cpu().numpy().astype(np.int64), w.cpu().numpy().astype(np.float64)
    ref_k = ko.pli_index(x.astype(np.float64)).astype(np.int64)
    assert np.array_equal(start, np.minimum(ref_k, 6))
    W = ko.pli_matrix(x.astype(np.float64))                    # [n][10]: weights of all ten entries
    ref_w = np.take_along_axis(W, start[:, None] + np.arange(4)[None, :], axis=1)
    assert np.abs(w - ref_w).max() <= (6e-8 if variant == 0 else 1.2e-7)
    # exactly the two taps are set: the weights outside offsets k - start, k - start + 1 are zero
    off = ref_k - start
    mask = (np.arange(4)[None, :] == off[:, None]) | (np.arange(4)[None, :] == off[:, None] + 1)
    assert (w[~mask] == 0).all()


def _check(kb, P, x, path, tol, prepared=False):
    L = kb.VQLayer(P, rule=kb.KAN_RULE_PLI2)
    if prepared:
        L.prepare()
        L.keep_on_bucket_kernel(prepared is True)       # prepared == "column": the small-layer kernel
    kern = kb.kan_vq_planned_kernel(L, x.shape[0], 1, path)
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=path).cpu().numpy()
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True, rule="pli")
    rep = ko.error_report(y, y_ref, A)
    assert rep["headline"] <= tol and rep["strict"] <= tol, (kern, rep)
    # and it is not the cubic rule's answer
    y_cubic = ko.vq_layer_forward(x, **P.as_dict())
    assert np.abs(y_ref - y_cubic).max() > 10 * tol * np.abs(y_ref).max()
    return kern


@pytest.mark.parametrize("cb,gb", [("i8", "f16"), ("f32", "f32")])
def test_pli_every_kernel_family(kb, cb, gb):
    P = synth.make_layer(21, 300, 200, 20000, cb_dtype=cb, gb_dtype=gb)
    rng = np.random.default_rng(5)
    seen = set()
    for B, path, tol, prepared in [(1, kb.KAN_PATH_GATHER, TOL_FP32, False), (1, kb.KAN_PATH_GATHER, TOL_FP32, True),
                                   (3, kb.KAN_PATH_GATHER, TOL_FP32, True), (2, kb.KAN_PATH_GATHER, TOL_FP32, "column"),
                                   (9, kb.KAN_PATH_GATHER, TOL_FP32, False),
                                   (50, kb.KAN_PATH_GATHER, TOL_FP32, False), (70, kb.KAN_PATH_GATHER, TOL_FP32, False),
                                   (20, kb.KAN_PATH_MFMA, TOL_MFMA, False),
                                   (150, kb.KAN_PATH_MFMA, TOL_MFMA, False)]:
        x = rng.uniform(-1.1, 1.1, size=(B, 300)).astype(np.float32)
        x[0, :4] = [1.0, -1.0, np.float32(7.0 / 9.0), np.float32(-1.0 / 9.0)]
        seen.add(_check(kb, P, x, path, tol, prepared))
    assert seen == {"kan_gather_bt1", "kan_bucket", "kan_column", "kan_fused_f32", "kan_mfma_split", "kan_fused_f16", "kan_mfma"}


@pytest.mark.parametrize("B,path,prepared", [(1, "gather", True), (1, "gather", False), (16, "gather", False),
                                             (16, "mfma", False), (1024, "mfma", False)])
def test_pli_config3_head(kb, B, path, prepared):
    Ps, x = synth.config3(B)
    Ls = [kb.VQLayer(p, rule=kb.KAN_RULE_PLI2) for p in Ps]
    if prepared:
        for L in Ls:
            L.prepare()
    pth, tol = (kb.KAN_PATH_GATHER, TOL_FP32) if path == "gather" else (kb.KAN_PATH_MFMA, TOL_MFMA)
    y = kb.kan_vq_head_forward([Ls], to_dev(x), path=pth)[0].cpu().numpy()
    rows = np.arange(B) if B <= 64 else np.sort(np.random.default_rng(B).choice(B, 48, replace=False))
    y_ref = ko.vq_head_forward(x[rows], [p.as_dict() for p in Ps], rule="pli")
    assert ko.error_report(y[rows], y_ref)["headline"] <= tol


def test_rules_do_not_mix_in_a_group(kb):
    P = synth.make_layer(2, 16, 8, 50)
    a, b = kb.VQLayer(P), kb.VQLayer(P, rule=kb.KAN_RULE_PLI2)
    with pytest.raises(kb.KanError) as e:
        kb.kan_vq_head_forward([[a], [b]], torch.zeros((2, 16), device="cuda"))
    assert e.value.status == kb.KAN_ERR_UNSUPPORTED
