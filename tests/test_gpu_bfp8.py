"""GPU parity for block-floating-point codebooks (8-bit mantissas, one exponent byte per codeword
row: the BFP8 row of the paper's Table 1 in this repository's reading of it - the paper defines no
format, so parity with the paper's own encoding is unpinned): dequantised rows and gathered ids bit
for bit, outputs of every kernel family that serves the format within the bounds of its path."""
import numpy as np
import pytest

from oracle import kan_oracle as ko
from paper_2512_15742_amd import synth

from kan_testlib import TOL_FP32, TOL_MFMA, check_layer_output, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def kb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2512_15742_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("idx_dtype,K", [("u16", 65536), ("u32", 70000)])
def test_bfp8_rows_and_ids_bit_exact(kb, idx_dtype, K):
    P = synth.make_layer(61, 37, 29, K, cb_dtype="bfp8", gb_dtype="f16", idx_dtype=idx_dtype)
    special = [0, 32767, 32768, 65535, K - 1, K - 2, 1]
    P.idx.reshape(-1)[:len(special)] = special
    # rows with the extreme exponents and mantissas
    P.codebook[0, :10], P.codebook[0, 10] = 127, -126
    P.codebook[1, :10], P.codebook[1, 10] = -127, 100
    P.codebook[K - 1, :10], P.codebook[K - 1, 10] = np.arange(-5, 5), 0
    L = kb.VQLayer(P)
    assert L.desc.cb_dtype == kb.KAN_BFP8
    ids, rows = kb.kan_vq_debug_gather(L)
    assert np.array_equal(ids.cpu().numpy().view(np.uint32), P.idx.reshape(-1).astype(np.uint32))
    ref = ko.dequantise_codebook(P.codebook)[P.idx.reshape(-1).astype(np.int64)].astype(np.float32)
    assert np.array_equal(rows.cpu().numpy(), ref)
    assert kb.kan_vq_count_bad_indices(L) == 0
    assert kb.kan_vq_prepared_bytes(L) > 0                   # buckets of 4096 twelve-byte rows


@pytest.mark.parametrize("gb", ["f16", "f32"])
@pytest.mark.parametrize("n_in,n_out,B", [(130, 67, 1), (257, 130, 5), (520, 264, 33), (300, 140, 64), (1000, 264, 300)])
def test_bfp8_every_kernel_family(kb, gb, n_in, n_out, B):
    """Batch 1: vector-ALU kernel; 2..64: fused kernel (fp32 and fp16 operands); above: streaming
    contraction (fp16 operands, and the split form on the precise path)."""
    P = synth.make_layer(7 * n_in + n_out, n_in, n_out, 5000, cb_dtype="bfp8", gb_dtype=gb)
    x = synth.make_x(B + 3, B, n_in)
    x[0, 0], x[-1, -1] = 1.0, -1.0
    L = kb.VQLayer(P)
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
    for path, tol in ((kb.KAN_PATH_GATHER, TOL_FP32), (kb.KAN_PATH_MFMA, TOL_MFMA)):
        y = kb.kan_vq_layer_forward(L, to_dev(x), path=path).cpu().numpy()
        rep = ko.error_report(y, y_ref, A)
        assert rep["headline"] <= tol and rep["strict"] <= tol, (path, kb.kan_vq_planned_kernel(L, B, 1, path), rep)
    expect = {1: "kan_gather_bt1", 5: "kan_fused_f32", 33: "kan_fused_f32", 64: "kan_fused_f32", 300: "kan_mfma_split"}[B]
    assert kb.kan_vq_planned_kernel(L, B, 1, kb.KAN_PATH_GATHER) == expect


def test_bfp8_rows_with_their_own_exponents(kb):
    """Rows six decades apart in size: every row keeps its own exponent (the point of the format),
    which an Int8 codebook with one scale per layer cannot do."""
    n_in, n_out, B = 200, 96, 40
    P = synth.make_layer(71, n_in, n_out, 300, cb_dtype="f32", gb_dtype="f32")
    rng = np.random.default_rng(2)
    shapes = (P.codebook * 10.0 ** rng.uniform(-6, 0, size=(300, 1))).astype(np.float32)
    import dataclasses
    Pb = dataclasses.replace(P, codebook=synth.quantise_shapes_bfp8(shapes))
    x = synth.make_x(8, B, n_in)
    L = kb.VQLayer(Pb)
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    y_ref, A = ko.vq_layer_forward(x, **Pb.as_dict(), return_abs=True)
    rep = ko.error_report(y, y_ref, A)
    assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, rep
    # the same shapes under one Int8 scale lose the small rows altogether; in block floating point they survive
    small = np.abs(shapes).max(axis=1) < 1e-4
    assert small.any() and np.abs(ko.dequantise_codebook(Pb.codebook)[small]).max() > 0
    q, scale = synth.quantise_shapes(shapes)
    assert (q[small] == 0).all()


@pytest.mark.parametrize("B,path_name", [(1, "gather"), (16, "gather"), (16, "mfma"), (256, "mfma"), (256, "gather")])
def test_bfp8_config3_shape_head(kb, B, path_name):
    Ps = synth.config3_layers("f16", cb_dtype="bfp8")
    Ls = [kb.VQLayer(p) for p in Ps]
    x = synth.make_x(3990 + B, B, 2048)
    path, tol = (kb.KAN_PATH_GATHER, TOL_FP32) if path_name == "gather" else (kb.KAN_PATH_MFMA, TOL_MFMA)
    y = kb.kan_vq_head_forward([Ls], to_dev(x), path=path)[0].cpu().numpy()
    rows = np.arange(B) if B <= 16 else np.sort(np.random.default_rng(B).choice(B, 16, replace=False))
    y_ref = ko.vq_head_forward(x[rows], [p.as_dict() for p in Ps])
    assert np.isfinite(y).all() and ko.error_report(y[rows], y_ref)["headline"] <= tol


def test_bfp8_descriptor_rules(kb):
    P = synth.make_layer(3, 16, 16, 100, cb_dtype="bfp8", gb_dtype="f16")
    L = kb.VQLayer(P)
    L.desc.codebook = L.codebook.data_ptr() + 2              # rows must be 4-byte aligned
    with pytest.raises(kb.KanError) as e:
        kb.kan_vq_layer_forward(L, torch.zeros((2, 16), device="cuda"))
    assert e.value.status == kb.KAN_ERR_SHAPE


@pytest.mark.parametrize("gb", ["f16", "f32"])
@pytest.mark.parametrize("n_in,n_out,K,B", [(130, 67, 5000, 1), (257, 130, 4097, 3), (520, 264, 9000, 4), (2100, 96, 2049, 2),
                                             (1000, 600, 20001, 1), (64, 24, 1, 4)])
def test_bfp8_prepared_layout(kb, gb, n_in, n_out, K, B):
    """Prepared block-floating-point layers: buckets of 4096 twelve-byte rows (2048 for more than 2048 inputs) in
    LDS, the row's exponent read beside its window; small layers on the column kernel, the others on the bucket
    kernel (also forced there).  Against the oracle and against the same layer unprepared."""
    P = synth.make_layer(11 * n_in + n_out + K, n_in, n_out, K, cb_dtype="bfp8", gb_dtype=gb)
    P.idx.reshape(-1)[:4] = [0, K - 1, min(K - 1, 4095), min(K - 1, 4096)]       # both sides of a bucket boundary
    x = synth.make_x(B + 5, B, n_in)
    x[0, 0], x[-1, -1] = 1.0, -1.0
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
    plain = kb.kan_vq_layer_forward(kb.VQLayer(P), to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    for flags in (0, kb.KAN_LAYER_NO_COLUMN):
        L = kb.VQLayer(P)
        L.desc.flags = flags
        L.prepare()
        name = kb.kan_vq_planned_kernel(L, B, 1, kb.KAN_PATH_GATHER)
        assert name in ("kan_bucket", "kan_column") and (flags == 0 or name == "kan_bucket")
        y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
        rep = ko.error_report(y, y_ref, A)
        assert np.isfinite(y).all() and rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, (name, rep)
        assert (np.abs(y - plain) <= 2 * TOL_FP32 * A).all()


def test_bfp8_prepared_config3_shape_head(kb):
    """Config 3's shapes with block-floating-point codebooks, both layers prepared: bucket kernel on the first,
    column kernel on the second, partial sums handed over between them."""
    Ps = synth.config3_layers("f16", cb_dtype="bfp8")
    Ls = [kb.VQLayer(p).prepare() for p in Ps]
    for B in (1, 4):
        x = synth.make_x(4100 + B, B, 2048)
        y = kb.kan_vq_head_forward([Ls], to_dev(x), path=kb.KAN_PATH_GATHER)[0].cpu().numpy()
        y_ref = ko.vq_head_forward(x, [p.as_dict() for p in Ps])
        assert kb.kan_vq_planned_kernel(Ls[0], B, 1, kb.KAN_PATH_GATHER) == "kan_bucket"
        assert np.isfinite(y).all() and ko.error_report(y, y_ref)["headline"] <= TOL_FP32
