"""GPU parity of the column kernel: small prepared layers served by one workgroup per
(output, sample), which reads the output's ids and gains from the transposed copy in the prepared
buffer, gathers the codeword windows from L2 and writes the finished output.  Every result is compared with the float64
oracle under the 1e-5 bound of the fp32 kernels (whole tensor: headline and strict
per-element criteria), and with the bucket kernel's result on the same buffer."""
import numpy as np
import pytest

from oracle import kan_oracle as ko
from paper_2512_15742_amd import synth

from kan_testlib import TOL_FP32, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def kb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2512_15742_amd import binding
    binding.lib()
    return binding


def _check(kb, P, x, rule="bspline"):
    """Column kernel against the oracle (all outputs), and against the bucket kernel."""
    B = x.shape[0]
    L = kb.VQLayer(P, rule=kb.KAN_RULE_PLI2 if rule == "pli" else kb.KAN_RULE_BSPLINE3).prepare()
    assert kb.kan_vq_planned_kernel(L, B, 1, kb.KAN_PATH_GATHER) == "kan_column"
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True, rule=rule)
    rep = ko.error_report(y, y_ref, A)
    assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, rep
    L.keep_on_bucket_kernel()
    assert kb.kan_vq_planned_kernel(L, B, 1, kb.KAN_PATH_GATHER) == "kan_bucket"
    yb = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    assert np.abs(y - yb).max() <= TOL_FP32 * np.abs(y_ref).max()
    return rep


@pytest.mark.parametrize("cb_dtype,gb_dtype", [("i8", "f16"), ("i8", "f32"), ("i8", "q8"), ("f16", "f16"),
                                               ("f16", "f32"), ("f32", "f16"), ("f32", "f32")])
@pytest.mark.parametrize("B", [1, 3])
def test_column_storage_types(kb, cb_dtype, gb_dtype, B):
    P = synth.make_layer(410 + B, 600, 200, 30000, cb_dtype=cb_dtype, gb_dtype=gb_dtype)
    x = synth.make_x(411, B, 600, "uniform")
    _check(kb, P, x)


def test_column_config3_second_layer_shape(kb):
    """1024 -> 256 with K = 65,536 Int8 rows (eight buckets), the layer the kernel was made for."""
    P = synth.config3_layers()[1]
    for B in (1, 4):
        x = synth.make_x(420 + B, B, 1024, "normal")
        _check(kb, P, x)


@pytest.mark.parametrize("n_in,n_out,K,cb", [(1, 1, 1, "i8"), (1, 5, 3, "f32"), (7, 1, 100, "f16"), (255, 3, 9000, "i8"),
                                              (257, 70, 5000, "i8"), (2048, 256, 65536, "i8"), (2047, 11, 131072, "f32"),
                                              (2049, 8, 1000, "i8"), (4096, 100, 70000, "i8"), (512, 1024, 600000, "i8")])
def test_column_shapes(kb, n_in, n_out, K, cb):
    """Ragged and extreme shapes: a single edge, partly filled rounds of the thread loop, exactly one round
    (2048 inputs), one input more, two rounds (4096 inputs, the most a prepared layer may have), 32-bit
    ids, 2^19 edges at batch 2 (edges x samples = 2^20, the most the kernel takes)."""
    P = synth.make_layer(n_in + 3 * n_out, n_in, n_out, K, cb_dtype=cb, gb_dtype="f16" if cb != "f32" else "f32")
    x = synth.make_x(430, 2, n_in, "uniform")
    _check(kb, P, x)


def test_column_limits_fall_back_to_bucket(kb):
    """The kernel takes a layer while edges x samples stay within 2^20."""
    for n_in, n_out, expect in [(1024, 1024, ["kan_column", "kan_bucket", "kan_bucket", "kan_bucket"]),
                                (1024, 1025, ["kan_bucket"] * 4),
                                (4096, 129, ["kan_column", "kan_bucket", "kan_bucket", "kan_bucket"]),
                                (1024, 256, ["kan_column"] * 4), (1024, 257, ["kan_column"] * 3 + ["kan_bucket"])]:
        P = synth.make_layer(5, n_in, n_out, 1000, cb_dtype="i8", gb_dtype="f16")
        L = kb.VQLayer(P).prepare()
        assert [kb.kan_vq_planned_kernel(L, B, 1, kb.KAN_PATH_GATHER) for B in (1, 2, 3, 4)] == expect, (n_in, n_out)
    L = kb.VQLayer(synth.make_layer(5, 64, 64, 1000, cb_dtype="i8", gb_dtype="f16")).prepare()
    assert kb.kan_vq_planned_kernel(L, 5, 1, kb.KAN_PATH_GATHER) == "kan_fused_f32"


@pytest.mark.parametrize("dist", ["zipf", "zipf-sorted"])
def test_column_skewed_histograms(kb, dist):
    """Runs of very different lengths: most edges of an output in the first bucket, empty runs elsewhere."""
    P = synth.make_layer(440, 700, 90, 65536, cb_dtype="i8", gb_dtype="f16", idx_dist=dist, zipf_s=1.3)
    x = synth.make_x(441, 2, 700, "normal")
    _check(kb, P, x)


def test_column_knots_and_clamped_inputs(kb):
    P = synth.make_layer(450, 64, 40, 3000, cb_dtype="i8", gb_dtype="f16")
    knots = np.array([-1 + 2 * k / 7 for k in range(8)], dtype=np.float32)
    xs = np.concatenate([knots, np.nextafter(knots, np.float32(2)), np.nextafter(knots, np.float32(-2)),
                         np.array([-3.0, 3.0, 0.0, 1e-30, -1e-30], dtype=np.float32)])
    x = np.resize(xs, (2, 64)).astype(np.float32)
    _check(kb, P, x)


def test_column_two_tap_rule(kb):
    P = synth.make_layer(460, 300, 64, 20000, cb_dtype="i8", gb_dtype="f16")
    x = synth.make_x(461, 2, 300, "uniform")
    _check(kb, P, x, rule="pli")


@pytest.mark.parametrize("B", [1, 2, 4])
def test_column_after_bucket_layer_in_a_head(kb, B):
    """Config 3, both layers prepared: the first layer's per-bucket sums go straight into the column
    kernel of the second (no reduction launch, no hidden tensor); three launches become two."""
    Ps, x = synth.config3(B)
    Ls = [kb.VQLayer(p).prepare() for p in Ps]
    assert kb.kan_vq_planned_kernel(Ls[0], B, 1, kb.KAN_PATH_GATHER) == "kan_bucket"
    assert kb.kan_vq_planned_kernel(Ls[1], B, 1, kb.KAN_PATH_GATHER) == "kan_column"
    xd = to_dev(x)
    kb.kan_prof_begin(16)
    y = kb.kan_vq_head_forward([Ls], xd, path=kb.KAN_PATH_GATHER)[0].cpu().numpy()
    rec = kb.kan_prof_end()
    assert sorted(rec) == ["kan_bucket@L1", "kan_column@L2"], rec
    y_ref = ko.vq_head_forward(x, [p.as_dict() for p in Ps])
    assert ko.error_report(y, y_ref)["headline"] <= TOL_FP32
    # layer 2 alone on the GPU's own hidden activation against the oracle on the same fp32 numbers
    hid = torch.tanh(kb.kan_vq_layer_forward(Ls[0], xd, path=kb.KAN_PATH_GATHER))
    y2 = kb.kan_vq_layer_forward(Ls[1], hid, path=kb.KAN_PATH_GATHER).cpu().numpy()
    y2_ref, A = ko.vq_layer_forward(hid.cpu().numpy(), **Ps[1].as_dict(), return_abs=True)
    rep = ko.error_report(y2, y2_ref, A)
    assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, rep


def test_column_heads_in_a_group_and_hidden_layers(kb):
    """Five heads of three small layers each (column kernel on every layer, tanh between them) on one input."""
    B, shapes = 2, [(96, 80), (80, 48), (48, 9)]
    heads_p = [[synth.make_layer(470 + 10 * h + l, i, o, 12000, cb_dtype="i8", gb_dtype="f16")
                for l, (i, o) in enumerate(shapes)] for h in range(5)]
    heads = [[kb.VQLayer(p).prepare() for p in ps] for ps in heads_p]
    for l in range(3):
        assert kb.kan_vq_planned_kernel(heads[0][l], B, 5, kb.KAN_PATH_GATHER) == "kan_column"
    x = synth.make_x(479, B, 96, "uniform")
    y = kb.kan_vq_head_forward(heads, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    for h in range(5):
        y_ref = ko.vq_head_forward(x, [p.as_dict() for p in heads_p[h]])
        assert ko.error_report(y[h], y_ref)["headline"] <= TOL_FP32, h


def test_column_flags_must_be_known(kb):
    P = synth.make_layer(480, 16, 8, 50, cb_dtype="i8", gb_dtype="f16")
    L = kb.VQLayer(P)
    L.desc.flags = 2
    with pytest.raises(kb.KanError):
        kb.kan_vq_layer_forward(L, to_dev(synth.make_x(1, 1, 16, "uniform")), path=kb.KAN_PATH_GATHER)
