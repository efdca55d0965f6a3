"""GPU parity of the compression-side assignment step (normalise every grid, nearest codebook
shape; paper section 4.2) against the float64 oracle.

The index is an arg-min decided by floating-point scores.  The kernel's scores are fp32-grade
(split fp16 operands, fp32 accumulation, 4 mantissa bits given to the arg-max bookkeeping), so
the comparison is: the index must equal the oracle's wherever the oracle's best and second-best
squared distances differ by more than GAP, and everywhere the distance of the chosen row must be
within GAP of the smallest one (a different but equally near row is a valid answer)."""
import numpy as np
import pytest

from oracle import kan_oracle as ko
from paper_2512_15742_amd import synth

from kan_testlib import to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

GAP = 2e-5          # squared distances are O(1): shapes and rows have unit norm


@pytest.fixture(scope="module")
def kb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2512_15742_amd import binding
    binding.lib()
    return binding


def _idx_np(idx):
    a = idx.cpu().numpy()
    return a.view(np.uint16 if a.dtype == np.int16 else np.uint32).astype(np.int64)


def _check_assignment(kb, coef, cb):
    idx, gain, bias = kb.kan_vq_assign(to_dev(coef), to_dev(cb))
    idx, gain, bias = _idx_np(idx), gain.cpu().numpy(), bias.cpu().numpy()
    shapes, g_ref, b_ref = ko.normalise_grids(coef)
    assert np.abs(gain - g_ref).max() <= 2e-6 * g_ref.max()
    assert np.abs(bias - b_ref).max() <= 2e-6 * max(np.abs(b_ref).max(), np.abs(coef).max())
    flat = shapes.reshape(-1, ko.G)
    n_bad_far, n_diff = 0, 0
    step = 256 if cb.shape[0] <= 4096 else 32            # the oracle materialises E x K x 10 doubles
    for s in range(0, flat.shape[0], step):
        d2 = ko.squared_distances(flat[s:s + step], cb)
        chosen = idx.reshape(-1)[s:s + step]
        assert (chosen >= 0).all() and (chosen < cb.shape[0]).all()
        d_chosen = d2[np.arange(d2.shape[0]), chosen]
        if d2.shape[1] > 1:
            part = np.partition(d2, 1, axis=1)
            best, second = part[:, 0], part[:, 1]
        else:
            best, second = d2[:, 0], np.full(d2.shape[0], np.inf)
        assert (d_chosen <= best + GAP).all(), float((d_chosen - best).max())
        clear = second - best > GAP
        n_bad_far += int((chosen[clear] != d2.argmin(axis=1)[clear]).sum())
        n_diff += int((chosen != d2.argmin(axis=1)).sum())
    assert n_bad_far == 0
    return idx, gain, bias, n_diff


@pytest.mark.parametrize("n_in,n_out,K", [(64, 32, 256), (37, 29, 1000), (96, 128, 65536), (5, 3, 7), (1, 1, 1),
                                          (200, 13, 70000)])
def test_assignment_matches_oracle(kb, n_in, n_out, K):
    coef, cb, k_true = synth.make_dense_grids(n_in + K, n_in, n_out, K)
    idx, gain, bias, n_diff = _check_assignment(kb, coef, cb)
    assert n_diff <= max(2, idx.size // 1000)              # near-ties are rare
    if K >= 256:
        # the layer was built from these shapes with 5 % noise: most edges find their own shape again
        assert (idx == k_true).mean() > 0.5


def test_assignment_exact_recovery_special_grids_and_r2(kb):
    rng = np.random.default_rng(3)
    cb = synth.make_shapes(rng, 4096)
    k = rng.integers(0, 4096, size=(40, 50))
    g = rng.uniform(0.05, 2.0, size=(40, 50))
    b = rng.normal(size=(40, 50))
    coef = (g[..., None] * cb[k].astype(np.float64) + b[..., None]).astype(np.float32)
    coef[0, 0] = 0.25                                     # constant grid: gain 0
    coef[0, 1] = 0.0
    idx, gain, bias = kb.kan_vq_assign(to_dev(coef), to_dev(cb))
    idx_np = _idx_np(idx)
    mask = np.ones((40, 50), dtype=bool)
    mask[0, :2] = False
    assert np.array_equal(idx_np[mask], k[mask])
    assert np.abs(gain.cpu().numpy()[mask] - g[mask]).max() < 1e-5 and gain[0, 0].item() == 0.0
    assert abs(bias[0, 0].item() - 0.25) < 1e-7
    # constant grids go to the row of smallest norm (all rows have unit norm here: any valid row)
    assert 0 <= idx_np[0, 0] < 4096
    r2 = kb.kan_vq_reconstruction_r2(to_dev(coef), to_dev(cb), idx, gain, bias)
    r2_ref = ko.r_squared(coef, cb, idx_np, gain.cpu().numpy(), bias.cpu().numpy())
    assert abs(r2 - r2_ref) < 1e-9 and r2 > 1 - 1e-6
    noisy, cb2, _ = synth.make_dense_grids(11, 64, 48, 2048, noise=0.2)
    i2, g2, b2 = kb.kan_vq_assign(to_dev(noisy), to_dev(cb2))
    r2 = kb.kan_vq_reconstruction_r2(to_dev(noisy), to_dev(cb2), i2, g2, b2)
    r2_ref = ko.r_squared(noisy, cb2, _idx_np(i2), g2.cpu().numpy(), b2.cpu().numpy())
    assert abs(r2 - r2_ref) < 1e-9 and 0.3 < r2 < 1.0


def test_assigned_layer_runs_through_the_forward_pass(kb):
    """Compress a dense layer, run the compressed layer, compare with the oracle run on the same
    compressed parameters and with the dense layer itself (close, since R^2 is high)."""
    coef, cb, _ = synth.make_dense_grids(21, 128, 96, 8192, noise=0.02)
    idx, gain, bias = kb.kan_vq_assign(to_dev(coef), to_dev(cb))
    P = synth.VQLayerParams(128, 96, 8192, cb, np.float32(1.0), _idx_np(idx).astype(np.uint16),
                            gain.cpu().numpy(), bias.cpu().numpy())
    x = synth.make_x(5, 7, 128)
    y = kb.kan_vq_layer_forward(kb.VQLayer(P), to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    y_ref = ko.vq_layer_forward(x, **P.as_dict())
    assert ko.error_report(y, y_ref)["headline"] <= 1e-5
    y_dense = ko.dense_layer_forward(coef, x)
    assert ko.error_report(y, y_dense)["headline"] < 0.15          # 2 % noise per coefficient, summed over 128 inputs
