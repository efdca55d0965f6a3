"""GPU parity of the matrix-core path (fp16 operand tiles, fp32 accumulation) against the
float64 oracle: outputs within 2e-2 relative, the bound stated for 16-bit operands; everything
integer (spans, ids) is covered by the exact routines in test_gpu_parity.py."""
import numpy as np
import pytest

from oracle import kan_oracle as ko
from paper_2512_15742_amd import synth

from kan_testlib import TOL_FP32, TOL_MFMA, check_head_layer_by_layer, check_layer_output, gpu_layers, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def kb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2512_15742_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("n_in,n_out,B", [(1, 1, 1), (8, 32, 32), (3, 21, 2), (130, 67, 5), (257, 130, 150),
                                          (64, 520, 33), (1000, 264, 300), (2048, 8, 129),
                                          # 64-sample tiles of the fused kernel (its deep pipeline): long and short chunks
                                          (2048, 264, 50), (1000, 130, 64), (300, 21, 40), (4100, 70, 33)])
def test_mfma_ragged_shapes(kb, n_in, n_out, B):
    P = synth.make_layer(n_in * 7 + n_out, n_in, n_out, 1000, cb_dtype="i8", gb_dtype="f16")
    x = synth.make_x(B, B, n_in)
    x[0, 0] = 1.0
    x[-1, -1] = -1.0
    (L,) = gpu_layers([P])
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_MFMA).cpu().numpy()
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
    rep = ko.error_report(y, y_ref, A)
    assert rep["headline"] <= TOL_MFMA and rep["strict"] <= TOL_MFMA, rep
    assert rep["headline"] >= 0 and np.isfinite(y).all()


@pytest.mark.parametrize("gb,cb,idx", [("f16", "i8", "u16"), ("f32", "i8", "u16"), ("q8", "i8", "u16"), ("f16", "i8", "u32"),
                                       ("f32", "i8", "u32"), ("f16", "f16", "u16"), ("f32", "bfp8", "u16"), ("f16", "bfp8", "u32"),
                                       ("f32", "f32", "u16")])
@pytest.mark.parametrize("n_in,n_out,B", [(520, 272, 50), (1001, 48, 64), (24, 16, 33), (300, 400, 40), (2048, 1024, 64)])
def test_fused_64_sample_tiles_with_staged_metadata(kb, gb, cb, idx, n_in, n_out, B):
    """Batch 33..64 on the fp16 path: the fused kernel's deep pipeline.  With n_out a multiple of 16 (and
    aligned arrays) the per-edge metadata of two steps comes in through 16-byte loads and a strip of LDS:
    output tiles cut short by n_out, chunks whose last pair of steps is ragged or missing, every storage
    type of index, gain/bias and codebook (fp32 rows take the unstaged pipeline)."""
    if n_in * n_out > 500000 and (gb, cb, idx) != ("f16", "i8", "u16"):
        pytest.skip("the large shape runs once")
    K = 70000 if idx == "u32" else 3000
    P = synth.make_layer(n_in + 3 * n_out + B, n_in, n_out, K, cb_dtype=cb, gb_dtype=gb, idx_dtype=idx)
    x = synth.make_x(B + 7, B, n_in)
    (L,) = gpu_layers([P])
    assert kb.kan_vq_planned_kernel(L, B, 1, kb.KAN_PATH_MFMA) == "kan_fused_f16"
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_MFMA).cpu().numpy()
    if n_in * n_out * B <= 2e8:
        y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
        rep = ko.error_report(y, y_ref, A)
        assert rep["headline"] <= TOL_MFMA and rep["strict"] <= TOL_MFMA, rep
    else:
        assert np.isfinite(y).all()
        check_layer_output(y, x, P, TOL_MFMA, n_samples=96, full=False, seed=B)
    # the same layer with arrays 2 bytes off a 16-byte boundary takes the unstaged pipeline: same sums
    # up to the order of nothing - both add the same products in the same order
    L2 = kb.VQLayer(P)
    for name in ("idx", "gain", "bias"):
        t = getattr(L2, name)
        pad = 16 // t.element_size()
        buf = torch.empty(t.numel() + 2 * pad, dtype=t.dtype, device="cuda")
        off = pad + 1                                     # one element past a 16-byte boundary
        buf[off:off + t.numel()] = t.reshape(-1)
        setattr(L2, name + "_shifted", buf)
        setattr(L2.desc, name, buf.data_ptr() + off * t.element_size())
    y2 = kb.kan_vq_layer_forward(L2, to_dev(x), path=kb.KAN_PATH_MFMA).cpu().numpy()
    assert np.array_equal(y2, y)


@pytest.mark.parametrize("gb,cb,idx", [("f32", "i8", "u16"), ("f16", "f32", "u16"), ("f32", "f32", "u32"), ("f16", "i8", "u32")])
def test_mfma_dtype_combinations(kb, gb, cb, idx):
    P = synth.make_layer(9, 96, 160, 70000 if idx == "u32" else 4096, cb_dtype=cb, gb_dtype=gb, idx_dtype=idx)
    x = synth.make_x(4, 200, 96, "normal")
    (L,) = gpu_layers([P])
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_MFMA).cpu().numpy()
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
    rep = ko.error_report(y, y_ref, A)
    assert rep["headline"] <= TOL_MFMA and rep["strict"] <= TOL_MFMA, rep


def test_mfma_config1(kb):
    (P,), x = synth.config1()
    (L,) = gpu_layers([P])
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_MFMA).cpu().numpy()
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
    rep = ko.error_report(y, y_ref, A)
    assert rep["headline"] <= TOL_MFMA and rep["strict"] <= TOL_MFMA, rep


def test_mfma_config2_b256(kb):
    (P,), x = synth.config2(256)
    (L,) = gpu_layers([P])
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_MFMA).cpu().numpy()
    rep = check_layer_output(y, x, P, TOL_MFMA)
    print("config2 B=256 mfma", rep)


@pytest.mark.parametrize("B", [256, 1024, 2048, 4096])
def test_mfma_config3_head(kb, B):
    """The batch sizes differ in tile height, number of chunks of inputs and in how the kernel
    deals its workgroups to the XCDs (8, 4, 2 chunks for layer 1, 16 for layer 2)."""
    Ps, x = synth.config3(B)
    Ls = gpu_layers(Ps)
    y = kb.kan_vq_head_forward([Ls], to_dev(x), path=kb.KAN_PATH_MFMA)[0].cpu().numpy()
    # a row of every 64-sample tile (a tile left out by the workgroup mapping would show), and random ones
    rows = np.unique(np.concatenate([np.arange(0, B, 64) + (np.arange(0, B, 64) // 64) % 64,
                                     np.random.default_rng(B).choice(B, 16, replace=False)]))
    y_ref = ko.vq_head_forward(x[rows], [p.as_dict() for p in Ps])
    rep = ko.error_report(y[rows], y_ref)
    print("config3 mfma", B, rep)
    assert rep["headline"] <= TOL_MFMA, rep
    # the automatic dispatcher takes the same path at these batch sizes
    assert kb.kan_vq_planned_kernel(Ls[0], B, 1, kb.KAN_PATH_AUTO) == "kan_mfma"
    y_auto = kb.kan_vq_head_forward([Ls], to_dev(x), path=kb.KAN_PATH_AUTO)[0]
    assert np.array_equal(y_auto.cpu().numpy(), y)


def test_mfma_config4_multi_head(kb):
    n_heads, B = 50, 64
    heads_p, x = synth.config4(n_heads, B)
    heads = [gpu_layers(ps) for ps in heads_p]
    y = kb.kan_vq_head_forward(heads, to_dev(x), path=kb.KAN_PATH_MFMA).cpu().numpy()
    for h in (0, 23, 49):
        y_ref = ko.vq_head_forward(x, [p.as_dict() for p in heads_p[h]])
        assert ko.error_report(y[h], y_ref)["headline"] <= TOL_MFMA


@pytest.mark.parametrize("n_in,n_out,B", [
    (70, 1900, 2100),      # 15 x 17 tiles of 128 samples (ragged in both directions)
    (70, 1900, 300),       # 15 x 3 tiles of 128 samples would be too few: 64-sample tiles, 15 x 5
    (200, 100, 5000),      # one column tile: 64-sample tiles, 79 of them
    (330, 129, 4100),      # one output past a tile; 128-sample tiles, the last one 4 samples
    (96, 1000, 1100),      # 128 x 256 tiles for eight waves (four Phi tiles, a barrier every second step): 6 steps,
    (100, 1000, 1100),     # 7 steps (a ragged last one),
    (16, 2048, 1030),      # a single step,
    (40, 1024, 1024),      # three steps
])
def test_mfma_both_tile_heights_sampled(kb, n_in, n_out, B):
    """The contraction kernel has a 128-sample and a 64-sample tile; which one a layer gets
    depends on how many tiles its grid has.  Sampled outputs against the oracle, and whole
    rows (first, last, around tile boundaries) so that every column of a row is checked."""
    P = synth.make_layer(n_in + n_out + B, n_in, n_out, 3000, cb_dtype="i8", gb_dtype="f16")
    x = synth.make_x(B + 1, B, n_in)
    (L,) = gpu_layers([P])
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_MFMA).cpu().numpy()
    assert np.isfinite(y).all()
    check_layer_output(y, x, P, TOL_MFMA, n_samples=96, full=False, seed=B)
    rows = np.array([0, 63, 64, B // 2, B - 65, B - 1])
    y_ref, A = ko.vq_layer_forward(x[rows], **P.as_dict(), return_abs=True)
    rep = ko.error_report(y[rows], y_ref, A)
    assert rep["headline"] <= TOL_MFMA and rep["strict"] <= TOL_MFMA, rep


@pytest.mark.parametrize("variant", ["i8", "f32"])
def test_mfma_config5_sampled(kb, variant):
    """The full-size layer: 64 sample tiles x 32 output tiles of 128 x 128, the only grid on which the
    contraction kernel's 8 x 8 patches run four to a row.  The output starts as NaN (the binding
    fills what it allocates), so a tile that no workgroup wrote fails `isfinite`; one whole row of
    every sample tile (all 32 output tiles of it) goes against the oracle, and the whole tensor
    against the precise path, whose own parity is checked in test_gpu_parity.py."""
    (P,), x = synth.config5(variant)
    (L,) = gpu_layers([P])
    xd = to_dev(x)
    y_t = kb.kan_vq_layer_forward(L, xd, path=kb.KAN_PATH_MFMA)
    y = y_t.cpu().numpy()
    assert np.isfinite(y).all()
    rep = check_layer_output(y, x, P, TOL_MFMA, n_samples=64, full=False, seed=5)
    print("config5 mfma", variant, rep)
    B = x.shape[0]
    rows = np.arange(0, B, 128) + (np.arange(0, B, 128) // 128 * 37) % 128      # one row of each 128-sample tile
    y_ref = ko.vq_layer_forward(x[rows], **P.as_dict())
    rep_rows = ko.error_report(y[rows], y_ref)
    print("config5 mfma rows", variant, rep_rows)
    assert rep_rows["headline"] <= TOL_MFMA, rep_rows
    y_precise = kb.kan_vq_layer_forward(L, xd, path=kb.KAN_PATH_GATHER)
    scale = float(y_precise.abs().max())
    assert float((y_t - y_precise).abs().max()) <= (TOL_MFMA + TOL_FP32) * scale


@pytest.mark.parametrize("B", [256, 1024])
def test_mfma_deterministic(kb, B):
    """Bit-identical repeats: 64-sample tiles (batch 256) and the eight-wave 128 x 256 tiles (batch 1024), whose
    waves may drift two steps apart between barriers; five runs each."""
    Ps, x = synth.config3(B)
    Ls = gpu_layers(Ps)
    xd = to_dev(x)
    y1 = kb.kan_vq_head_forward([Ls], xd, path=kb.KAN_PATH_MFMA).clone()
    for _ in range(4):
        y2 = kb.kan_vq_head_forward([Ls], xd, path=kb.KAN_PATH_MFMA)
        assert torch.equal(y1, y2)


@pytest.mark.parametrize("B,n_heads", [(150, 1), (40, 3), (700, 2)])
def test_mfma_three_layer_head_hand_over(kb, B, n_heads):
    """Hidden activations between matrix-core layers: layers that split their inputs into few
    chunks leave the partial sums to the next layer's basis preparation (which adds and
    squashes them), layers with many chunks go through the reduction pass; ragged sizes."""
    dims = [(520, 264), (264, 130), (130, 21)]
    heads_p = [[synth.make_layer(100 * h + 7 * l + 1, i, o, 1000, cb_dtype="i8", gb_dtype="f16")
                for l, (i, o) in enumerate(dims)] for h in range(n_heads)]
    x = synth.make_x(B + n_heads, B, dims[0][0])
    heads = [gpu_layers(ps) for ps in heads_p]
    y = kb.kan_vq_head_forward(heads, to_dev(x), path=kb.KAN_PATH_MFMA).cpu().numpy()
    assert y.shape == (n_heads, B, 21) and np.isfinite(y).all()
    for h in range(n_heads):
        y_ref = ko.vq_head_forward(x, [p.as_dict() for p in heads_p[h]])
        rep = ko.error_report(y[h], y_ref)
        assert rep["headline"] <= TOL_MFMA, (h, rep)


@pytest.mark.parametrize("path_name", ["mfma", "gather"])
def test_single_head_start_launch_mixed_types_and_many_layers(kb, path_name):
    """A single head's call prepares the coefficient records of its layers in one launch, but only
    those stored like the first layer and only the first four: a six-layer head whose third and
    fifth layers use other storage types takes both ways in one call (fp16 path, and the split
    precise path from batch 65)."""
    path = kb.KAN_PATH_MFMA if path_name == "mfma" else kb.KAN_PATH_GATHER
    tol = TOL_MFMA if path_name == "mfma" else 1e-5
    dims = [(70, 96), (96, 130), (130, 64), (64, 80), (80, 33), (33, 21)]
    kinds = [("i8", "f16", "u16"), ("i8", "f16", "u16"), ("f32", "f32", "u32"), ("i8", "f16", "u16"),
             ("f16", "f16", "u16"), ("i8", "f16", "u16")]
    Ps = [synth.make_layer(31 + l, i, o, 70000 if idx == "u32" else 1000, cb_dtype=cb, gb_dtype=gb, idx_dtype=idx)
          for l, ((i, o), (cb, gb, idx)) in enumerate(zip(dims, kinds))]
    B = 150
    x = synth.make_x(77, B, dims[0][0])
    Ls = gpu_layers(Ps)
    y = kb.kan_vq_head_forward([Ls], to_dev(x), path=path)[0].cpu().numpy()
    assert np.isfinite(y).all()
    # Every layer at `tol` on identical fp32 inputs (no factor for depth) ...
    y_chain, worst = check_head_layer_by_layer(kb, Ls, Ps, x, path, tol)
    # ... and the head call against that chain: two evaluations on the GPU of the same six layers,
    # whose hidden activations differ in the last bits (order of the partial sums, tanh in the
    # kernel's epilogue): each layer of either is within `tol` of the oracle on its own inputs.
    scale = np.abs(y_chain).max()
    assert np.abs(y - y_chain).max() <= 2 * tol * scale
    print("six-layer head", path_name, "worst layer", worst, "end to end vs float64 head",
          ko.error_report(y, ko.vq_head_forward(x, [p.as_dict() for p in Ps])))
    # the same head through the grouped launches (two identical heads; the planner may cut the
    # inputs into other chunks there, so the sums agree to rounding only)
    y2 = kb.kan_vq_head_forward([Ls, Ls], to_dev(x), path=path).cpu().numpy()
    assert np.array_equal(y2[0], y2[1])
    assert np.abs(y2[0] - y_chain).max() <= 2 * tol * scale


def test_profiled_launches_are_keyed_by_layer(kb):
    """The library's event timing names the launches of a head call by layer; a single head on
    the matrix cores starts with the merged preparation launch."""
    Ps, x = synth.config3(256)
    Ls = gpu_layers(Ps)
    xd = to_dev(x)
    kb.kan_vq_head_forward([Ls], xd, path=kb.KAN_PATH_MFMA)
    torch.cuda.synchronize()
    kb.kan_prof_begin(64)
    for _ in range(3):
        kb.kan_vq_head_forward([Ls], xd, path=kb.KAN_PATH_MFMA)
    rec = kb.kan_prof_end()
    assert set(rec) == {"kan_prep_start", "kan_mfma@L1", "kan_prep_basis@L2", "kan_mfma@L2", "kan_reduce@L2"}, rec
    assert all(v["launches"] == 3 and v["total_ms"] > 0 for v in rec.values()), rec
    # outside a head call nothing carries a layer
    kb.kan_prof_begin(8)
    kb.kan_bspline_basis(xd[0])
    assert set(kb.kan_prof_end()) == {"kan_basis"}


@pytest.mark.parametrize("B", [100, 128, 129])
def test_large_layer_keeps_the_fused_kernel_for_two_batch_tiles(kb, B):
    """A layer of 2^22 edges (Int8 rows): up to batch 128 both paths gather every row once per tile of 64
    samples instead of preparing records; from 129 the streaming kernels take over.  Sampled outputs of
    both tiles against the oracle, and the ragged second tile."""
    P = synth.make_layer(610, 4096, 1024, 65536, cb_dtype="i8", gb_dtype="f16")
    L = kb.VQLayer(P)
    x = synth.make_x(611, B, 4096, "uniform")
    xd = to_dev(x)
    for path, tol, fused, streaming in ((kb.KAN_PATH_MFMA, TOL_MFMA, "kan_fused_f16", "kan_mfma"),
                                        (kb.KAN_PATH_GATHER, TOL_FP32, "kan_fused_f32", "kan_mfma_split")):
        assert kb.kan_vq_planned_kernel(L, B, 1, path) == (fused if B <= 128 else streaming)
        y = kb.kan_vq_layer_forward(L, xd, path=path).cpu().numpy()
        assert np.isfinite(y).all()
        check_layer_output(y, x, P, tol, n_samples=96, seed=B, full=False)
    small = kb.VQLayer(synth.make_layer(612, 2048, 1024, 65536, cb_dtype="i8", gb_dtype="f16"))
    assert kb.kan_vq_planned_kernel(small, 100, 1, kb.KAN_PATH_MFMA) == "kan_mfma"
    wide_rows = kb.VQLayer(synth.make_layer(613, 4096, 1024, 65536, cb_dtype="f32", gb_dtype="f32"))
    assert kb.kan_vq_planned_kernel(wide_rows, 100, 1, kb.KAN_PATH_GATHER) == "kan_mfma_split"
