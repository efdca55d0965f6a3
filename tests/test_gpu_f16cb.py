"""GPU parity for fp16 codebooks (Table 1 lists FP32, FP16 and Int8 codebook precisions):
every kernel family against the float64 oracle, gathered rows bit-exact, ragged shapes,
both edge rules, a two-layer head, the prepared (bucket) layout."""
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


def test_f16cb_gathered_rows_bit_exact(kb):
    for idx_dtype, K in (("u16", 3000), ("u32", 70000)):
        P = synth.make_layer(7, 37, 53, K, cb_dtype="f16", gb_dtype="f16", idx_dtype=idx_dtype)
        L = kb.VQLayer(P)
        ids, rows = kb.kan_vq_debug_gather(L)
        idx = P.idx.reshape(-1).astype(np.int64)
        assert np.array_equal(ids.cpu().numpy().astype(np.int64), idx)
        want = P.codebook[idx].astype(np.float32)              # every half is exactly a float
        assert np.array_equal(rows.cpu().numpy(), want)


@pytest.mark.parametrize("gb_dtype", ["f32", "f16"])
def test_f16cb_every_kernel_family(kb, gb_dtype):
    P = synth.make_layer(62, 300, 200, 20000, cb_dtype="f16", gb_dtype=gb_dtype)
    rng = np.random.default_rng(8)
    seen = set()
    for B, path, tol in [(1, kb.KAN_PATH_GATHER, TOL_FP32), (9, kb.KAN_PATH_GATHER, TOL_FP32),
                         (50, kb.KAN_PATH_GATHER, TOL_FP32), (70, kb.KAN_PATH_GATHER, TOL_FP32),
                             (20, kb.KAN_PATH_MFMA, TOL_MFMA),
                         (150, kb.KAN_PATH_MFMA, TOL_MFMA)]:
        x = rng.uniform(-1.1, 1.1, size=(B, 300)).astype(np.float32)
        L = kb.VQLayer(P)
        seen.add(kb.kan_vq_planned_kernel(L, B, 1, path))
        y = kb.kan_vq_layer_forward(L, to_dev(x), path=path).cpu().numpy()
        y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
        rep = ko.error_report(y, y_ref, A)
        assert rep["headline"] <= tol and rep["strict"] <= tol, (B, path, rep)
    assert seen == {"kan_gather_bt1", "kan_fused_f32", "kan_mfma_split", "kan_fused_f16", "kan_mfma"}


@pytest.mark.parametrize("n_in,n_out,K,B", [(1, 1, 2, 1), (3, 21, 5, 2), (130, 67, 9000, 5), (257, 530, 20000, 1),
                                            (64, 520, 300, 33), (2100, 9, 70000, 1), (520, 264, 1000, 150)])
def test_f16cb_ragged_shapes(kb, n_in, n_out, K, B):
    P = synth.make_layer(n_in * 5 + n_out, n_in, n_out, K, cb_dtype="f16", gb_dtype="f16")
    x = synth.make_x(B + 2, B, n_in)
    x[0, 0] = 1.0
    x[-1, -1] = -1.0
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
    L = kb.VQLayer(P)
    for path, tol in ((kb.KAN_PATH_GATHER, TOL_FP32), (kb.KAN_PATH_MFMA, TOL_MFMA)):
        y = kb.kan_vq_layer_forward(L, to_dev(x), path=path).cpu().numpy()
        rep = ko.error_report(y, y_ref, A)
        assert rep["headline"] <= tol and rep["strict"] <= tol, (path, rep)


@pytest.mark.parametrize("B,path", [(1, "gather"), (16, "gather"), (16, "mfma"), (300, "mfma")])
def test_f16cb_pli_rule(kb, B, path):
    P = synth.make_layer(63, 130, 70, 4000, cb_dtype="f16", gb_dtype="f16")
    x = synth.make_x(B + 3, B, 130)
    L = kb.VQLayer(P, rule=kb.KAN_RULE_PLI2)
    pth, tol = (kb.KAN_PATH_GATHER, TOL_FP32) if path == "gather" else (kb.KAN_PATH_MFMA, TOL_MFMA)
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=pth).cpu().numpy()
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True, rule="pli")
    rep = ko.error_report(y, y_ref, A)
    assert rep["headline"] <= tol and rep["strict"] <= tol, rep


@pytest.mark.parametrize("B,path", [(1, "gather"), (16, "gather"), (256, "mfma")])
def test_f16cb_config3_shaped_head(kb, B, path):
    Ps = [synth.make_layer(3100, 2048, 1024, 65536, cb_dtype="f16", gb_dtype="f16"),
          synth.make_layer(3101, 1024, 256, 65536, cb_dtype="f16", gb_dtype="f16")]
    x = synth.make_x(3, B, 2048)
    Ls = [kb.VQLayer(p) for p in Ps]
    pth, tol = (kb.KAN_PATH_GATHER, TOL_FP32) if path == "gather" else (kb.KAN_PATH_MFMA, TOL_MFMA)
    y = kb.kan_vq_head_forward([Ls], to_dev(x), path=pth)[0].cpu().numpy()
    rows = np.arange(B) if B <= 64 else np.sort(np.random.default_rng(B).choice(B, 48, replace=False))
    y_ref = ko.vq_head_forward(x[rows], [p.as_dict() for p in Ps])
    assert ko.error_report(y[rows], y_ref)["headline"] <= tol


@pytest.mark.parametrize("gb_dtype", ["f32", "f16"])
@pytest.mark.parametrize("rule", ["bspline", "pli"])
def test_f16cb_prepared_layer(kb, gb_dtype, rule):
    """Buckets of 4096 fp16 rows: 5 buckets, odd and even row offsets inside a dword, batch 1..4."""
    P = synth.make_layer(66, 300, 200, 20000, cb_dtype="f16", gb_dtype=gb_dtype)
    P.idx.reshape(-1)[:6] = [0, 1, 4095, 4096, 19999, 8191]
    L = kb.VQLayer(P, rule=kb.KAN_RULE_PLI2 if rule == "pli" else kb.KAN_RULE_BSPLINE3).prepare()
    L.keep_on_bucket_kernel()                    # (this small layer would take the column kernel otherwise)
    assert kb.kan_vq_prepared_bytes(L) == L.prepared.numel() > 0
    plain = kb.VQLayer(P, rule=kb.KAN_RULE_PLI2 if rule == "pli" else kb.KAN_RULE_BSPLINE3)
    for B in (1, 3, 4):
        x = synth.make_x(B + 40, B, 300)
        x[0, 0], x[-1, -1] = 1.0, -1.0
        assert kb.kan_vq_planned_kernel(L, B, 1, kb.KAN_PATH_AUTO) == "kan_bucket"
        y = kb.kan_vq_layer_forward(L, to_dev(x)).cpu().numpy()
        y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True, rule=rule)
        rep = ko.error_report(y, y_ref, A)
        assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, (B, rep)
        y_plain = kb.kan_vq_layer_forward(plain, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
        assert np.abs(y - y_plain).max() <= 2 * TOL_FP32 * np.abs(y_ref).max()


@pytest.mark.parametrize("B", [1, 2, 4])
def test_f16cb_config3_shaped_head_prepared(kb, B):
    Ps = synth.config3_layers(gb_dtype="f16", cb_dtype="f16")
    x = synth.make_x(B + 11, B, Ps[0].idx.shape[0])
    Ls = [kb.VQLayer(P).prepare() for P in Ps]
    assert kb.kan_vq_planned_kernel(Ls[0], B, 1, kb.KAN_PATH_AUTO) == "kan_bucket"
    y = kb.kan_vq_head_forward([Ls], to_dev(x))[0].cpu().numpy()
    y_ref = ko.vq_head_forward(x, [p.as_dict() for p in Ps])
    assert ko.error_report(y, y_ref)["headline"] <= TOL_FP32


def test_f16cb_takes_no_byte_coded_gains(kb):
    Q = synth.make_layer(65, 16, 8, 50, cb_dtype="i8", gb_dtype="q8")
    Lq = kb.VQLayer(Q)
    Lq.desc.cb_dtype = kb.KAN_F16
    with pytest.raises(kb.KanError) as e:
        kb.kan_vq_layer_forward(Lq, torch.zeros((2, 16), device="cuda"))
    assert e.value.status == kb.KAN_ERR_UNSUPPORTED
