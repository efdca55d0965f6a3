"""The entry point that allocates nothing, kan_vq_head_forward_static, through the C-ABI: same
results as kan_vq_head_forward (bit for bit: same plan, same kernels, the scratch regions merely
live in the library's fixed per-GPU array) and within the bounds of the oracle, on two calls in a
row - the second with a smaller input, which finds the array full of the first call's data - on
both paths, for several heads, and the rejection of a call whose scratch need exceeds the array."""
import ctypes as C

import numpy as np
import pytest

from oracle import kan_oracle as ko
from paper_2512_15742_amd import synth

from kan_testlib import TOL_FP32, TOL_MFMA, gpu_layers, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def kb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2512_15742_amd import binding
    binding.lib()
    return binding


def _heads(n_heads, dims, seed):
    return [[synth.make_layer(seed + 100 * h + l, i, o, 3000, cb_dtype="i8", gb_dtype="f16")
             for l, (i, o) in enumerate(dims)] for h in range(n_heads)]


@pytest.mark.parametrize("path_name", ["gather", "mfma"])
def test_static_scratch_matches_workspace_entry_point_two_calls_in_a_row(kb, path_name):
    path = kb.KAN_PATH_GATHER if path_name == "gather" else kb.KAN_PATH_MFMA
    tol = TOL_FP32 if path_name == "gather" else TOL_MFMA
    dims = [(520, 264), (264, 130), (130, 21)]
    heads_p = _heads(3, dims, 7)
    heads = [gpu_layers(ps) for ps in heads_p]
    # first a large call (several chunks of inputs, hidden activations, matrix-core records on the fp16
    # path), then a smaller one that reuses the array as the first left it
    for B, seed in ((200, 1), (5, 2)):
        x = synth.make_x(seed, B, dims[0][0])
        xd = to_dev(x)
        need = kb.kan_vq_workspace_bytes(heads, B, path)
        assert 0 < need <= kb.KAN_STATIC_SCRATCH_BYTES
        y_ws = kb.kan_vq_head_forward(heads, xd, path=path)
        y_st = torch.full_like(y_ws, float("nan"))
        arr, n_layers, n_heads = kb._desc_array(heads)
        st = kb.lib().kan_vq_head_forward_static(arr, n_layers, n_heads, C.c_void_p(xd.data_ptr()), B,
                                                 C.c_void_p(y_st.data_ptr()), int(path),
                                                 C.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert st == kb.KAN_OK
        torch.cuda.synchronize()
        assert torch.equal(y_st, y_ws)
        y = y_st.cpu().numpy()
        for h in range(n_heads):
            y_ref = ko.vq_head_forward(x, [p.as_dict() for p in heads_p[h]])
            rep = ko.error_report(y[h], y_ref)
            assert rep["headline"] <= tol, (B, h, rep)


def test_static_scratch_prepared_layers_and_single_layer(kb):
    """Batch 1 over prepared layers (bucket kernel: per-bucket sums in the scratch array) and a
    single layer that needs no scratch at all."""
    Ps = [synth.make_layer(1, 256, 128, 4096, cb_dtype="i8", gb_dtype="f16"),
          synth.make_layer(2, 128, 32, 4096, cb_dtype="i8", gb_dtype="f16")]
    Ls = [kb.VQLayer(p).prepare() for p in Ps]
    Ls[0].keep_on_bucket_kernel()                 # (small layers: the first stays on the bucket kernel, the second takes the column kernel)
    x = synth.make_x(3, 1, 256)
    xd = to_dev(x)
    assert kb.kan_vq_planned_kernel(Ls[0], 1, 1, kb.KAN_PATH_GATHER) == "kan_bucket"
    assert kb.kan_vq_planned_kernel(Ls[1], 1, 1, kb.KAN_PATH_GATHER) == "kan_column"
    y_st = kb.kan_vq_head_forward_static([Ls], xd, path=kb.KAN_PATH_GATHER)
    y_ws = kb.kan_vq_head_forward([Ls], xd, path=kb.KAN_PATH_GATHER)
    assert torch.equal(y_st, y_ws)
    y_ref = ko.vq_head_forward(x, [p.as_dict() for p in Ps])
    assert ko.error_report(y_st[0].cpu().numpy(), y_ref)["headline"] <= TOL_FP32
    P = synth.make_layer(5, 8, 32, 100)
    (L,) = gpu_layers([P])
    x1 = synth.make_x(4, 1, 8)
    y1 = kb.kan_vq_head_forward_static([[L]], to_dev(x1), path=kb.KAN_PATH_GATHER)[0].cpu().numpy()
    assert ko.error_report(y1, ko.vq_layer_forward(x1, **P.as_dict()))["headline"] <= TOL_FP32


def test_static_scratch_rejects_what_does_not_fit(kb):
    Ps, x = synth.config3(1024)
    Ls = gpu_layers(Ps)
    assert kb.kan_vq_workspace_bytes([Ls], 1024, kb.KAN_PATH_MFMA) > kb.KAN_STATIC_SCRATCH_BYTES
    y = torch.zeros((1, 1024, 256), dtype=torch.float32, device="cuda")
    with pytest.raises(kb.KanError) as e:
        kb.kan_vq_head_forward_static([Ls], to_dev(x), path=kb.KAN_PATH_MFMA, y=y)
    assert e.value.status == kb.KAN_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert float(y.abs().max()) == 0.0          # nothing was enqueued
    # the same head at batch 64 fits on either path
    for path in (kb.KAN_PATH_GATHER, kb.KAN_PATH_MFMA):
        assert kb.kan_vq_workspace_bytes([Ls], 64, path) <= kb.KAN_STATIC_SCRATCH_BYTES
