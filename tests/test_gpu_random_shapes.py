"""Seeded random sweep over shapes, dtypes, rules, batch sizes and paths: every case through the
C-ABI against the float64 oracle.  The cases are drawn once from a fixed seed (the list is the
same on every run), small enough for the oracle, and lean towards the awkward: sizes of 1,
sizes just past a tile or bucket boundary, K = 1, odd K, batch sizes around the dispatcher's
thresholds."""
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


def _cases(n=120, seed=20251127):
    rng = np.random.default_rng(seed)
    dims = [1, 2, 3, 7, 8, 9, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 257, 300, 513, 600]
    ks = [1, 2, 3, 5, 255, 256, 2047, 2048, 2049, 8191, 8192, 8193, 20001, 65536, 70001]
    bs = [1, 2, 3, 4, 5, 16, 31, 32, 33, 63, 64, 65, 100, 129, 300]
    out = []
    for c in range(n):
        n_in, n_out = int(rng.choice(dims)), int(rng.choice(dims))
        K = int(rng.choice(ks))
        cb = str(rng.choice(["i8", "f32", "f16"]))
        gb = str(rng.choice(["f32", "f16"] + (["q8"] if cb == "i8" else [])))
        idx = "u32" if K > 65536 else str(rng.choice(["u16", "u32"]))
        out.append(dict(seed=1000 + c, n_in=n_in, n_out=n_out, K=K, cb=cb, gb=gb, idx=idx, B=int(rng.choice(bs)),
                        rule=str(rng.choice(["bspline", "pli"])), dist=str(rng.choice(["uniform", "zipf", "zipf-sorted"])),
                        prepared=bool(rng.integers(0, 2))))
    return out


def _cases_bfp8(n=24, seed=20251128):
    """A second list for block-floating-point codebooks (drawn apart, so that the list above stays as it was)."""
    rng = np.random.default_rng(seed)
    dims = [1, 3, 8, 33, 64, 129, 257, 600, 2100]
    out = []
    for c in range(n):
        out.append(dict(seed=3000 + c, n_in=int(rng.choice(dims)), n_out=int(rng.choice(dims[:-1])),
                        K=int(rng.choice([1, 5, 2047, 2048, 2049, 4096, 4097, 20001])), cb="bfp8",
                        gb=str(rng.choice(["f32", "f16"])), idx=str(rng.choice(["u16", "u32"])),
                        B=int(rng.choice([1, 2, 3, 4, 5, 16, 33, 64, 65, 130])),
                        rule=str(rng.choice(["bspline", "pli"])), dist=str(rng.choice(["uniform", "zipf", "zipf-sorted"])),
                        prepared=bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("case", _cases() + _cases_bfp8(), ids=lambda c: "-".join(str(v) for v in c.values()))
def test_random_case(kb, case):
    P = synth.make_layer(case["seed"], case["n_in"], case["n_out"], case["K"], cb_dtype=case["cb"],
                         gb_dtype=case["gb"], idx_dtype=case["idx"], idx_dist=case["dist"], zipf_s=1.3)
    B = case["B"]
    x = np.random.default_rng(case["seed"] + 7).uniform(-1.2, 1.2, size=(B, case["n_in"])).astype(np.float32)
    x[0, 0], x[-1, -1] = 1.0, -1.0
    rule = kb.KAN_RULE_PLI2 if case["rule"] == "pli" else kb.KAN_RULE_BSPLINE3
    L = kb.VQLayer(P, rule=rule)
    if case["prepared"]:
        L.prepare()
    assert kb.kan_vq_count_bad_indices(L) == 0
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True, rule=case["rule"])
    for path, tol in ((kb.KAN_PATH_GATHER, TOL_FP32), (kb.KAN_PATH_MFMA, TOL_MFMA), (kb.KAN_PATH_AUTO, TOL_MFMA)):
        y = kb.kan_vq_layer_forward(L, to_dev(x), path=path).cpu().numpy()
        assert np.isfinite(y).all()
        rep = ko.error_report(y, y_ref, A)
        assert rep["headline"] <= tol, (path, kb.kan_vq_planned_kernel(L, B, 1, path), rep)
        # The per-element bound |dy| <= tol * sum_i |phi_ij| presumes that the sum over inputs is where
        # magnitudes add up; with a handful of inputs an edge's own gain * C(x) + bias can cancel to
        # far below its two terms, and rounding relative to those terms is then large relative to phi.
        if case["n_in"] >= 8:
            assert rep["strict"] <= tol, (path, kb.kan_vq_planned_kernel(L, B, 1, path), rep)


def _head_cases(n=30, seed=771):
    rng = np.random.default_rng(seed)
    widths = [5, 21, 64, 130, 264, 520]
    out = []
    for c in range(n):
        n_layers = int(rng.integers(2, 5))
        dims = [int(rng.choice(widths)) for _ in range(n_layers + 1)]
        out.append(dict(seed=5000 + 10 * c, dims=tuple(dims), heads=int(rng.choice([1, 1, 2, 3])),
                        B=int(rng.choice([1, 2, 4, 5, 33, 70, 200])), K=int(rng.choice([300, 9000, 20001])),
                        prep=tuple(bool(v) for v in rng.integers(0, 2, size=n_layers)),
                        gb=str(rng.choice(["f16", "f32", "q8"]))))
    return out


@pytest.mark.parametrize("case", _head_cases(), ids=lambda c: "-".join(str(v) for v in c.values()))
def test_random_head(kb, case):
    """Several layers and heads: hand-overs of partial sums between kernels of every kind (bucket to
    bucket, split layers to the basis preparation, reductions where neither applies), with
    prepared and unprepared layers mixed at random."""
    dims, B = case["dims"], case["B"]
    heads_p = [[synth.make_layer(case["seed"] + 100 * h + l, dims[l], dims[l + 1], case["K"], cb_dtype="i8",
                                 gb_dtype=case["gb"]) for l in range(len(dims) - 1)] for h in range(case["heads"])]
    heads = [[kb.VQLayer(p) for p in ps] for ps in heads_p]
    for ls in heads:
        for L, pr in zip(ls, case["prep"]):
            if pr:
                L.prepare()
    x = synth.make_x(case["seed"] + 3, B, dims[0])
    for path, tol in ((kb.KAN_PATH_GATHER, TOL_FP32), (kb.KAN_PATH_MFMA, TOL_MFMA)):
        y = kb.kan_vq_head_forward(heads, to_dev(x), path=path).cpu().numpy()
        assert y.shape == (case["heads"], B, dims[-1]) and np.isfinite(y).all()
        for h in range(case["heads"]):
            y_ref = ko.vq_head_forward(x, [p.as_dict() for p in heads_p[h]])
            assert ko.error_report(y[h], y_ref)["headline"] <= tol, (path, h)
