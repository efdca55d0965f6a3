"""Heads of several layers at batch 2..32 on the fused kernel (and at batch 1 on the vector-ALU kernel): a layer that cut its inputs into chunks
hands its partial sums straight to the next layer's fused kernel, which adds the slices of its own chunk
of inputs (fixed order), squashes them and keeps them in LDS; no reduction launch in between.  Checked:
the launches that ran (no reduction after a chained layer; one where the hand-over does not apply), the
head's output against the float64 head of the oracle and against the layer-by-layer chain of single-layer
calls, bit-reproducibility, groups of heads, ragged shapes, every storage type."""
import numpy as np
import pytest

from oracle import kan_oracle as ko
from paper_2512_15742_amd import synth

from kan_testlib import TOL_FP32, TOL_MFMA, check_head_layer_by_layer, gpu_layers, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def kb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2512_15742_amd import binding
    binding.lib()
    return binding


def _launches(kb, heads, xd, path):
    kb.kan_vq_head_forward(heads, xd, path=path)
    torch.cuda.synchronize()
    kb.kan_prof_begin(64)
    kb.kan_vq_head_forward(heads, xd, path=path)
    return set(kb.kan_prof_end())


def _head(seed, dims, K, cb="i8", gb="f16", idx="u16"):
    return [synth.make_layer(seed + l, dims[l], dims[l + 1], K, cb_dtype=cb, gb_dtype=gb, idx_dtype=idx)
            for l in range(len(dims) - 1)]


def _check(kb, Ps, x, path, tol, expect_reduce_after_first):
    Ls = gpu_layers(Ps)
    xd = to_dev(x)
    B = x.shape[0]
    name = "kan_fused_f32" if path == kb.KAN_PATH_GATHER else "kan_fused_f16"
    if B == 1 and path == kb.KAN_PATH_GATHER:
        name = "kan_gather_bt1"
    for L in Ls:
        assert kb.kan_vq_planned_kernel(L, B, 1, path) == name
    rec = _launches(kb, [Ls], xd, path)
    assert ("kan_reduce@L1" in rec) == expect_reduce_after_first, rec
    assert f"{name}@L{len(Ps)}" in rec, rec
    y_dev = torch.full((1, B, Ps[-1].n_out), float("nan"), device="cuda")       # an output left unwritten would show
    ws = torch.empty(kb.kan_vq_workspace_bytes([Ls], B, path), dtype=torch.uint8, device="cuda")
    y = kb.kan_vq_head_forward([Ls], xd, path=path, ws=ws, y=y_dev)[0].cpu().numpy()
    assert np.isfinite(y).all()
    y_ref = ko.vq_head_forward(x, [p.as_dict() for p in Ps])
    rep = ko.error_report(y, y_ref)
    assert rep["headline"] <= tol, rep
    # every layer on identical fp32 inputs, and the head call against that chain: two GPU evaluations of
    # the same hidden activations, which differ in the last bits (summation order)
    y_chain, worst = check_head_layer_by_layer(kb, Ls, Ps, x, path, tol)
    assert np.abs(y - y_chain).max() <= 2 * tol * np.abs(y_chain).max(), (worst, rep)
    # bit-reproducible
    y_again = kb.kan_vq_head_forward([Ls], xd, path=path, ws=ws)[0].cpu().numpy()
    assert np.array_equal(y, y_again)
    return y


@pytest.mark.parametrize("B", [2, 5, 16, 17, 32])
@pytest.mark.parametrize("path_name", ["precise", "fp16"])
def test_config3_shapes(kb, B, path_name):
    path, tol = (kb.KAN_PATH_GATHER, TOL_FP32) if path_name == "precise" else (kb.KAN_PATH_MFMA, TOL_MFMA)
    Ps, x = synth.config3(B)
    _check(kb, Ps, x, path, tol, expect_reduce_after_first=False)


@pytest.mark.parametrize("dims", [(256, 128, 32), (100, 60, 20), (512, 256, 128, 16), (72, 36, 130), (1000, 200, 300, 7)],
                         ids=lambda d: "-".join(map(str, d)))
@pytest.mark.parametrize("B", [3, 16, 29])
def test_ragged_heads(kb, dims, B):
    Ps = _head(8100 + B, dims, 5003)
    x = synth.make_x(8200 + B, B, dims[0])
    x[0, 0], x[-1, -1] = -1.0, 1.0
    for path, tol in ((kb.KAN_PATH_GATHER, TOL_FP32), (kb.KAN_PATH_MFMA, TOL_MFMA)):
        Ls = gpu_layers(Ps)
        rec = _launches(kb, [Ls], to_dev(x), path)
        _check(kb, Ps, x, path, tol, expect_reduce_after_first="kan_reduce@L1" in rec)
    # (whether a layer is cut into chunks at all depends on its size: the shapes above cover both)


def test_hidden_width_not_in_fours_keeps_the_reduction(kb):
    """The hand-over needs the consumer's inputs in groups of four (16-byte loads of the slices)."""
    Ps = _head(8300, (512, 130, 40), 4099)
    x = synth.make_x(8301, 16, 512)
    for path, tol in ((kb.KAN_PATH_GATHER, TOL_FP32), (kb.KAN_PATH_MFMA, TOL_MFMA)):
        _check(kb, Ps, x, path, tol, expect_reduce_after_first=True)


@pytest.mark.parametrize("cb,gb,idx,K", [("f32", "f32", "u32", 70001), ("f16", "f16", "u16", 300), ("i8", "q8", "u16", 65536),
                                         ("bfp8", "f16", "u16", 1000), ("f16", "f32", "u16", 2000)])
def test_storage_types(kb, cb, gb, idx, K):
    Ps = _head(8400, (768, 256, 64), K, cb=cb, gb=gb, idx=idx)
    for B in (4, 16, 24):
        x = synth.make_x(8401 + B, B, 768)
        for path, tol in ((kb.KAN_PATH_GATHER, TOL_FP32), (kb.KAN_PATH_MFMA, TOL_MFMA)):
            _check(kb, Ps, x, path, tol, expect_reduce_after_first=False)


def test_group_of_heads(kb):
    """Three heads in one grouped call: each one's slices are its own."""
    B = 12
    heads_P = [_head(8500 + 10 * h, (1024, 256, 48), 4096) for h in range(3)]
    x = synth.make_x(8501, B, 1024)
    heads_L = [gpu_layers(Ps) for Ps in heads_P]
    for path, tol in ((kb.KAN_PATH_GATHER, TOL_FP32), (kb.KAN_PATH_MFMA, TOL_MFMA)):
        rec = _launches(kb, heads_L, to_dev(x), path)
        assert "kan_reduce@L1" not in rec, rec
        y = kb.kan_vq_head_forward(heads_L, to_dev(x), path=path).cpu().numpy()
        for h, Ps in enumerate(heads_P):
            y_ref = ko.vq_head_forward(x, [p.as_dict() for p in Ps])
            rep = ko.error_report(y[h], y_ref)
            assert np.isfinite(y[h]).all() and rep["headline"] <= tol, (h, rep)
            y_one = kb.kan_vq_head_forward([heads_L[h]], to_dev(x), path=path)[0].cpu().numpy()
            assert np.abs(y[h] - y_one).max() <= 2 * tol * np.abs(y_ref).max()


@pytest.mark.parametrize("dims", [(2048, 1024, 256), (256, 128, 32), (100, 61, 20), (520, 300, 129, 16), (1000, 200, 7)],
                         ids=lambda d: "-".join(map(str, d)))
def test_batch1_vector_alu_kernel(kb, dims):
    """Batch 1 on layers as given: the vector-ALU kernel of the next layer adds the slices itself (the threads
    that share a row of its basis table split them), whatever the hidden width."""
    Ps = _head(8600, dims, 5003)
    x = synth.make_x(8601, 1, dims[0])
    Ls = gpu_layers(Ps)
    rec = _launches(kb, [Ls], to_dev(x), kb.KAN_PATH_GATHER)
    # a layer that was cut into chunks is followed by no reduction unless it is the last one
    for l in range(1, len(Ps)):
        assert f"kan_reduce@L{l}" not in rec, rec
    _check(kb, Ps, x, kb.KAN_PATH_GATHER, TOL_FP32, expect_reduce_after_first=False)


@pytest.mark.parametrize("cb,gb,idx,K", [("f32", "f32", "u32", 70001), ("f16", "f16", "u16", 300), ("i8", "q8", "u16", 65536),
                                         ("bfp8", "f16", "u16", 1000)])
def test_batch1_storage_types(kb, cb, gb, idx, K):
    Ps = _head(8700, (768, 256, 64), K, cb=cb, gb=gb, idx=idx)
    x = synth.make_x(8701, 1, 768)
    _check(kb, Ps, x, kb.KAN_PATH_GATHER, TOL_FP32, expect_reduce_after_first=False)


def test_batch1_group_of_heads(kb):
    heads_P = [_head(8800 + 10 * h, (1024, 256, 48), 4096) for h in range(3)]
    x = synth.make_x(8801, 1, 1024)
    heads_L = [gpu_layers(Ps) for Ps in heads_P]
    rec = _launches(kb, heads_L, to_dev(x), kb.KAN_PATH_GATHER)
    assert "kan_reduce@L1" not in rec and "kan_gather_bt1@L2" in rec, rec
    y = kb.kan_vq_head_forward(heads_L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    for h, Ps in enumerate(heads_P):
        y_ref = ko.vq_head_forward(x, [p.as_dict() for p in Ps])
        rep = ko.error_report(y[h], y_ref)
        assert np.isfinite(y[h]).all() and rep["headline"] <= TOL_FP32, (h, rep)


@pytest.mark.parametrize("B", [1, 7, 16, 24])
def test_two_tap_rule_with_handed_over_sums(kb, B):
    """The two-tap rule (linear interpolation between two grid points) through the same hand-over."""
    Ps, x = synth.config3(B)
    Ls = [kb.VQLayer(p, rule=kb.KAN_RULE_PLI2) for p in Ps]
    xd = to_dev(x)
    for path, tol in ((kb.KAN_PATH_GATHER, TOL_FP32), (kb.KAN_PATH_MFMA, TOL_MFMA)):
        rec = _launches(kb, [Ls], xd, path)
        assert "kan_reduce@L1" not in rec, rec
        y_dev = torch.full((1, B, Ps[-1].n_out), float("nan"), device="cuda")
        y = kb.kan_vq_head_forward([Ls], xd, path=path, y=y_dev)[0].cpu().numpy()
        y_ref = ko.vq_head_forward(x, [p.as_dict() for p in Ps], rule="pli")
        rep = ko.error_report(y, y_ref)
        assert np.isfinite(y).all() and rep["headline"] <= tol, (path, rep)
        y_chain, _ = check_head_layer_by_layer(kb, Ls, Ps, x, path, tol, rule="pli")
        assert np.abs(y - y_chain).max() <= 2 * tol * np.abs(y_chain).max()


def _random_heads(n, seed):
    rng = np.random.default_rng(seed)
    kinds = [("i8", "f16", "u16"), ("i8", "q8", "u16"), ("f16", "f16", "u16"), ("bfp8", "f16", "u16"), ("f32", "f32", "u32"),
             ("i8", "f32", "u32"), ("f16", "f32", "u16")]
    out = []
    for c in range(n):
        depth = int(rng.integers(2, 5))
        dims = [int(rng.choice([int(rng.integers(8, 1500)), 4 * int(rng.integers(2, 375)), 16 * int(rng.integers(1, 90))]))
                for _ in range(depth + 1)]
        cb, gb, idx = kinds[int(rng.integers(len(kinds)))]
        K = int(rng.integers(2, 66000 if idx == "u32" else 60000))
        B = int(rng.choice([1, 1, 2, 3, 8, 13, 16, 17, 25, 32]))
        out.append(pytest.param(dims, cb, gb, idx, K, B, 9000 + 17 * c, id=f"{c}-{'x'.join(map(str, dims))}-{cb}-{gb}-B{B}"))
    return out


@pytest.mark.parametrize("dims,cb,gb,idx,K,B,seed", _random_heads(24, 20251129))
def test_random_heads(kb, dims, cb, gb, idx, K, B, seed):
    """Seeded random heads (depth 2..4, widths with and without a factor of four, every storage type, batch
    1..32): whichever layers hand their partial sums on, the head matches the float64 head and the chain of
    single-layer calls, and leaves no output unwritten."""
    Ps = _head(seed, dims, K, cb=cb, gb=gb, idx=idx)
    x = synth.make_x(seed + 7, B, dims[0])
    Ls = gpu_layers(Ps)
    xd = to_dev(x)
    for path, tol in ((kb.KAN_PATH_GATHER, TOL_FP32), (kb.KAN_PATH_MFMA, TOL_MFMA)):
        y_dev = torch.full((1, B, dims[-1]), float("nan"), device="cuda")
        y = kb.kan_vq_head_forward([Ls], xd, path=path, y=y_dev)[0].cpu().numpy()
        assert np.isfinite(y).all()
        y_ref = ko.vq_head_forward(x, [p.as_dict() for p in Ps])
        rep = ko.error_report(y, y_ref)
        assert rep["headline"] <= tol, (path, rep)
        y_chain, _ = check_head_layer_by_layer(kb, Ls, Ps, x, path, tol)
        assert np.abs(y - y_chain).max() <= 2 * tol * max(np.abs(y_chain).max(), 1e-30)
        assert np.array_equal(y, kb.kan_vq_head_forward([Ls], xd, path=path)[0].cpu().numpy())
