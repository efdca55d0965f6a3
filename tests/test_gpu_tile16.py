"""The precise path at batch 2..16 runs the fused kernel on 16-sample tiles (two blocks of 16 columns per
wave on the 16 x 16 x 4 fp32 matrix instruction).  Cases around that tile: batches that fill 1..4 of its
row groups or leave a ragged one, outputs that end inside either column block of a wave, inputs that end
inside a step and inside the pair of inputs a lane group serves; every storage type of ids, gains and rows
(the 16-byte metadata loads need outputs in multiples of 16, the others take the narrow loads)."""
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


SHAPES = [(9, 17), (70, 48), (33, 130), (257, 16), (64, 15), (16, 161)]


@pytest.mark.parametrize("B", [2, 6, 11, 15, 16, 17])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: f"{s[0]}x{s[1]}")
def test_tile16_ragged(kb, B, shape):
    n_in, n_out = shape
    for n, (cb, gb, idx, K) in enumerate((("i8", "f16", "u16", 4099), ("f32", "f32", "u32", 70001), ("f16", "f16", "u16", 300),
                                          ("i8", "q8", "u16", 65536), ("bfp8", "f16", "u16", 1000))):
        P = synth.make_layer(7100 + 10 * B + n, n_in, n_out, K, cb_dtype=cb, gb_dtype=gb, idx_dtype=idx)
        x = np.random.default_rng(B * 131 + n_in).uniform(-1.1, 1.1, size=(B, n_in)).astype(np.float32)
        x[0, 0], x[-1, -1] = -1.0, 1.0
        L = kb.VQLayer(P)
        assert kb.kan_vq_planned_kernel(L, B, 1, kb.KAN_PATH_GATHER) == "kan_fused_f32"
        y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
        y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
        rep = ko.error_report(y, y_ref, A)
        assert np.isfinite(y).all() and rep["headline"] <= TOL_FP32, (cb, gb, idx, rep)
        if n_in >= 8:
            assert rep["strict"] <= TOL_FP32, (cb, gb, idx, rep)


def test_tile16_matches_32_row_tile(kb):
    """The same rows through the 16-sample tile (batch 16) and the 32-sample tile (batch 17, one more row):
    two matrix instructions, the same sums to fp32 rounding."""
    P = synth.make_layer(7300, 300, 200, 20001, cb_dtype="i8", gb_dtype="f16")
    x = synth.make_x(7301, 17, 300)
    L = kb.VQLayer(P)
    y16 = kb.kan_vq_layer_forward(L, to_dev(x[:16]), path=kb.KAN_PATH_GATHER).cpu().numpy()
    y17 = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    _, A = ko.vq_layer_forward(x[:16], **P.as_dict(), return_abs=True)
    assert (np.abs(y16 - y17[:16]) <= 2 * TOL_FP32 * A).all()
