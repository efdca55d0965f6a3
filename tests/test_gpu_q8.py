"""GPU parity of the fully quantised 4-bytes-per-edge format (paper section 4.2: 16-bit index,
logarithmic one-byte gain, linear one-byte bias; one-byte codebook entries) through every
kernel family.  The oracle decodes the same codes in float64."""
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


def _q8_config3_layers():
    return synth.config3_layers("q8")


def test_q8_every_kernel_family(kb):
    P = synth.make_layer(61, 300, 200, 20000, cb_dtype="i8", gb_dtype="q8")
    P.gain[5, :7] = 0                                     # zero code: exact zero gain
    assert P.metadata_bytes == 4 * P.edges
    rng = np.random.default_rng(6)
    seen = set()
    for B, path, tol, prepared in [(1, kb.KAN_PATH_GATHER, TOL_FP32, False), (1, kb.KAN_PATH_GATHER, TOL_FP32, True),
                                   (3, kb.KAN_PATH_GATHER, TOL_FP32, True), (2, kb.KAN_PATH_GATHER, TOL_FP32, "column"),
                                   (9, kb.KAN_PATH_GATHER, TOL_FP32, False),
                                   (50, kb.KAN_PATH_GATHER, TOL_FP32, False), (70, kb.KAN_PATH_GATHER, TOL_FP32, False),
                                   (20, kb.KAN_PATH_MFMA, TOL_MFMA, False),
                                   (150, kb.KAN_PATH_MFMA, TOL_MFMA, False)]:
        x = rng.uniform(-1.1, 1.1, size=(B, 300)).astype(np.float32)
        L = kb.VQLayer(P)
        if prepared:
            L.prepare()
            L.keep_on_bucket_kernel(prepared is True)       # prepared == "column": the small-layer kernel
        seen.add(kb.kan_vq_planned_kernel(L, B, 1, path))
        y = kb.kan_vq_layer_forward(L, to_dev(x), path=path).cpu().numpy()
        y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
        rep = ko.error_report(y, y_ref, A)
        assert rep["headline"] <= tol and rep["strict"] <= tol, (B, path, prepared, rep)
    assert seen == {"kan_gather_bt1", "kan_bucket", "kan_column", "kan_fused_f32", "kan_mfma_split", "kan_fused_f16", "kan_mfma"}


@pytest.mark.parametrize("n_in,n_out,K,B", [(1, 1, 2, 1), (3, 21, 5, 2), (130, 67, 9000, 5), (257, 530, 20000, 1),
                                            (64, 520, 300, 33), (2100, 9, 30000, 1)])
def test_q8_ragged_shapes(kb, n_in, n_out, K, B):
    P = synth.make_layer(n_in * 3 + n_out, n_in, n_out, K, cb_dtype="i8", gb_dtype="q8")
    x = synth.make_x(B + 1, B, n_in)
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
    for prepared in (False, True):
        L = kb.VQLayer(P)
        if prepared:
            L.prepare()
        y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
        rep = ko.error_report(y, y_ref, A)
        assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, (prepared, rep)


def test_q8_prepared_layout_and_bias_sums(kb):
    """Records keep the one-byte gain code; the bias sums are those of the decoded biases."""
    P = synth.make_layer(77, 130, 40, 20000, cb_dtype="i8", gb_dtype="q8")
    L = kb.VQLayer(P).prepare()
    E = 130 * 40
    up = lambda v: (v + 32 + 255) // 256 * 256
    nb = 3
    raw = L.prepared.cpu().numpy()
    o = up((nb * 40 + 1) * 4)
    bias_sum = raw[o:o + 40 * 4].view(np.float32); o += up(40 * 4)
    pi = raw[o:o + 2 * E].view(np.uint16); o += up(2 * E)
    pq = raw[o:o + 2 * E].view(np.uint16); o += up(2 * E)
    pg = raw[o:o + E]; o += up(E)
    tab_w = [max(256 // (t + 1), nb) for t in range(4)] + [nb]          # block tables, then per-bucket block counts
    o += up(sum(tab_w) * 32) + up(5 * (nb + 1) * 4)
    o += up(1 * nb * 40 * 2) + up(1 * 40 * 8)          # the preparation's scratch: counts and bias sums per block of 256 inputs
    ti = raw[o:o + 4 * E].view(np.uint32).reshape(40, 130); o += up(4 * E)      # small layer: ids and gain codes transposed
    tgc = raw[o:o + E].reshape(40, 130); o += up(E)
    assert o == raw.size
    assert np.array_equal(ti, P.idx.T.astype(np.uint32)) and np.array_equal(tgc, P.gain.T)
    bucket = P.idx.astype(np.int64) // 8192
    ii, jj = np.meshgrid(np.arange(130), np.arange(40), indexing="ij")
    order = np.lexsort((ii.ravel(), jj.ravel(), bucket.ravel()))
    assert np.array_equal(pi, ii.ravel()[order].astype(np.uint16))
    assert np.array_equal(pq, (P.idx.astype(np.int64).ravel()[order] % 8192).astype(np.uint16))
    assert np.array_equal(pg, P.gain.ravel()[order])
    _, b = ko.dequantise_gain_bias(P.gain, P.bias, P.gb_params)
    assert np.abs(bias_sum - b.sum(axis=0)).max() <= 1e-6 * np.abs(b).sum(axis=0).max()


@pytest.mark.parametrize("B,path,prepared", [(1, "gather", True), (1, "gather", False), (16, "gather", False),
                                             (16, "mfma", False), (1024, "mfma", False)])
def test_q8_config3_shaped_head(kb, B, path, prepared):
    Ps = _q8_config3_layers()
    x = synth.make_x(3900 + B, B, 2048)
    Ls = [kb.VQLayer(p) for p in Ps]
    if prepared:
        for L in Ls:
            L.prepare()
    pth, tol = (kb.KAN_PATH_GATHER, TOL_FP32) if path == "gather" else (kb.KAN_PATH_MFMA, TOL_MFMA)
    y = kb.kan_vq_head_forward([Ls], to_dev(x), path=pth)[0].cpu().numpy()
    rows = np.arange(B) if B <= 64 else np.sort(np.random.default_rng(B).choice(B, 48, replace=False))
    y_ref = ko.vq_head_forward(x[rows], [p.as_dict() for p in Ps])
    assert ko.error_report(y[rows], y_ref)["headline"] <= tol


def test_q8_needs_int8_codebook(kb):
    P = synth.make_layer(2, 16, 8, 50, cb_dtype="i8", gb_dtype="q8")
    L = kb.VQLayer(P)
    L.desc.cb_dtype = kb.KAN_F32
    with pytest.raises(kb.KanError) as e:
        kb.kan_vq_layer_forward(L, torch.zeros((2, 16), device="cuda"))
    assert e.value.status == kb.KAN_ERR_UNSUPPORTED
