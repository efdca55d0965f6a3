"""GPU parity under skewed assignment histograms (a trained layer's histogram is unknown;
the configurations draw the uniform worst case).  A Zipfian histogram makes the codebook
buckets of the prepared layout very unequal (most edges in one bucket when the popular
codewords have the low ids) and makes many lanes of a wave gather the same row."""
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


@pytest.mark.parametrize("dist,zipf_s", [("zipf", 1.0), ("zipf-sorted", 1.0), ("zipf-sorted", 2.5)])
@pytest.mark.parametrize("n_in,n_out,K", [(300, 200, 20000), (2100, 130, 65536)])
def test_skewed_histograms_every_kernel_family(kb, dist, zipf_s, n_in, n_out, K):
    P = synth.make_layer(71, n_in, n_out, K, cb_dtype="i8", gb_dtype="f16", idx_dist=dist, zipf_s=zipf_s)
    counts = np.bincount(P.idx.reshape(-1).astype(np.int64), minlength=K)
    assert counts.max() > 20 * counts.mean()                   # really skewed
    rng = np.random.default_rng(9)
    for B, path, tol, prepared in [(1, kb.KAN_PATH_GATHER, TOL_FP32, False), (1, kb.KAN_PATH_GATHER, TOL_FP32, True),
                                   (3, kb.KAN_PATH_GATHER, TOL_FP32, True), (2, kb.KAN_PATH_GATHER, TOL_FP32, "column"),
                                   (9, kb.KAN_PATH_GATHER, TOL_FP32, False),
                                   (20, kb.KAN_PATH_MFMA, TOL_MFMA, False), (150, kb.KAN_PATH_MFMA, TOL_MFMA, False)]:
        x = rng.uniform(-1.0, 1.0, size=(B, n_in)).astype(np.float32)
        L = kb.VQLayer(P)
        if prepared:
            L.prepare()
            L.keep_on_bucket_kernel(prepared is True)
            small = prepared == "column"
            assert kb.kan_vq_planned_kernel(L, B, 1, path) == ("kan_column" if small else "kan_bucket")
        y = kb.kan_vq_layer_forward(L, to_dev(x), path=path).cpu().numpy()
        y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
        rep = ko.error_report(y, y_ref, A)
        assert rep["headline"] <= tol and rep["strict"] <= tol, (B, path, prepared, rep)


def test_one_codeword_for_every_edge(kb):
    """The degenerate histogram: a single codeword (all lanes gather one row; one bucket holds all)."""
    P = synth.make_layer(72, 257, 67, 9000, cb_dtype="i8", gb_dtype="f16")
    P.idx[...] = 8999
    x = synth.make_x(5, 4, 257)
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
    for prepared in (False, True):
        L = kb.VQLayer(P)
        if prepared:
            L.prepare()
        y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
        rep = ko.error_report(y, y_ref, A)
        assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, (prepared, rep)
