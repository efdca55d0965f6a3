"""Calls on different streams are independent when each has its own workspace and output: the forward
calls keep no state on the device between calls.  Two requests in flight on two streams (default
priority) must give the bits of the same calls made one after the other."""
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


@pytest.mark.parametrize("B,path,prepared", [(3, "gather", True), (16, "gather", False), (40, "mfma", False),
                                              (300, "mfma", False), (300, "gather", False)])
def test_two_streams_give_the_serial_bits(kb, B, path, prepared):
    dims = [(520, 264), (264, 130), (130, 21)]
    Ps = [synth.make_layer(140 + l, i, o, 20000, cb_dtype="i8", gb_dtype="f16") for l, (i, o) in enumerate(dims)]
    Ls = [kb.VQLayer(p) for p in Ps]
    if prepared:
        for L in Ls:
            L.prepare()
    pth = kb.KAN_PATH_GATHER if path == "gather" else kb.KAN_PATH_MFMA
    xs = [torch.from_numpy(synth.make_x(170 + r, B, 520)).cuda() for r in range(2)]
    nbytes = max(kb.kan_vq_workspace_bytes([Ls], B, pth), 256)
    wss = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
    serial = []
    for r in range(2):
        y = torch.empty((1, B, 21), dtype=torch.float32, device="cuda")
        kb.kan_vq_head_forward([Ls], xs[r], path=pth, ws=wss[r], y=y)
        serial.append(y)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(2)]
    ys = [torch.full((1, B, 21), float("nan"), dtype=torch.float32, device="cuda") for _ in range(2)]
    torch.cuda.synchronize()
    for rep in range(6):                               # the two requests overlap on the device
        for r in range(2):
            with torch.cuda.stream(streams[r]):
                kb.kan_vq_head_forward([Ls], xs[r], path=pth, ws=wss[r], y=ys[r])
    torch.cuda.synchronize()
    for r in range(2):
        assert torch.equal(ys[r], serial[r]), r


def test_two_host_threads_give_the_serial_bits(kb):
    """The same from two host threads (ctypes releases the interpreter lock during a call)."""
    import threading
    dims = [(520, 264), (264, 21)]
    Ps = [synth.make_layer(240 + l, i, o, 20000, cb_dtype="i8", gb_dtype="f16") for l, (i, o) in enumerate(dims)]
    Ls = [kb.VQLayer(p) for p in Ps]
    cases = [(16, kb.KAN_PATH_GATHER), (200, kb.KAN_PATH_MFMA)]
    xs = [torch.from_numpy(synth.make_x(270 + r, B, 520)).cuda() for r, (B, _) in enumerate(cases)]
    wss = [torch.empty(max(kb.kan_vq_workspace_bytes([Ls], B, p), 256), dtype=torch.uint8, device="cuda") for B, p in cases]
    serial = []
    for r, (B, p) in enumerate(cases):
        y = torch.empty((1, B, 21), dtype=torch.float32, device="cuda")
        kb.kan_vq_head_forward([Ls], xs[r], path=p, ws=wss[r], y=y)
        serial.append(y)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in cases]
    ys = [torch.full((1, B, 21), float("nan"), dtype=torch.float32, device="cuda") for B, _ in cases]
    torch.cuda.synchronize()
    errors = []

    def work(r):
        try:
            B, p = cases[r]
            with torch.cuda.stream(streams[r]):
                for _ in range(20):
                    kb.kan_vq_head_forward([Ls], xs[r], path=p, ws=wss[r], y=ys[r])
        except Exception as e:           # pragma: no cover
            errors.append(e)

    threads = [threading.Thread(target=work, args=(r,)) for r in range(len(cases))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for r in range(len(cases)):
        assert torch.equal(ys[r], serial[r]), r
