"""The forward calls only enqueue kernels on the caller's stream (no allocation, no memset, no
synchronisation), so a call can be captured into a HIP graph.  Every replay - with the
program's own eager work and synchronisations in between - must give the bits of the eager call."""
import numpy as np
import pytest

from paper_2512_15742_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def kb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2512_15742_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("B,path,prepared,kernel", [
    (1, "gather", True, "kan_bucket"), (1, "gather", False, "kan_gather_bt1"), (3, "gather", True, "kan_bucket"),
    (2, "gather", True, "kan_column"),
    (16, "gather", False, "kan_fused_f32"), (48, "mfma", False, "kan_fused_f16"), (300, "mfma", False, "kan_mfma")])
def test_head_forward_replays_from_a_graph(kb, B, path, prepared, kernel):
    dims = [(520, 264), (264, 130), (130, 21)]
    Ps = [synth.make_layer(40 + l, i, o, 20000, cb_dtype="i8", gb_dtype="f16") for l, (i, o) in enumerate(dims)]
    Ls = [kb.VQLayer(p) for p in Ps]
    if prepared:
        for L in Ls:
            L.prepare()
            L.keep_on_bucket_kernel(kernel == "kan_bucket")     # (small layers: the column kernel otherwise)
    pth = kb.KAN_PATH_GATHER if path == "gather" else kb.KAN_PATH_MFMA
    assert kb.kan_vq_planned_kernel(Ls[0], B, 1, pth) == kernel
    xs = [torch.from_numpy(synth.make_x(70 + r, B, 520)).cuda() for r in range(4)]
    ws = torch.empty(max(kb.kan_vq_workspace_bytes([Ls], B, pth), 256), dtype=torch.uint8, device="cuda")
    eager = []
    for x in xs:
        y = torch.empty((1, B, 21), dtype=torch.float32, device="cuda")
        kb.kan_vq_head_forward([Ls], x, path=pth, ws=ws, y=y)
        eager.append(y.clone())
    torch.cuda.synchronize()

    x_static = xs[0].clone()
    y_static = torch.empty((1, B, 21), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up on the capture stream, as torch asks
        kb.kan_vq_head_forward([Ls], x_static, path=pth, ws=ws, y=y_static)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        kb.kan_vq_head_forward([Ls], x_static, path=pth, ws=ws, y=y_static)
    for r in (1, 2, 3, 0, 2):
        x_static.copy_(xs[r])
        ws.fill_(0xA5)                                  # eager work between replays: scratch contents must not matter
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_static, eager[r]), (r, float((y_static - eager[r]).abs().max()))
