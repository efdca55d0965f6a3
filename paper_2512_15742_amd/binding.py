"""ctypes binding of libkan_mi355x.so (declared in include/kan.h).

Argument marshalling only: every step of the forward pass runs in the HIP
kernels behind the C-ABI.  PyTorch supplies device memory and the stream.
There is no CPU fallback: if the library has not been built, importing a symbol
from it raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkan_mi355x.so")

KAN_OK = 0
KAN_ERR_NULL, KAN_ERR_SHAPE, KAN_ERR_DTYPE, KAN_ERR_WORKSPACE, KAN_ERR_UNSUPPORTED, KAN_ERR_LAUNCH = 1, 2, 3, 4, 5, 6
KAN_F32, KAN_F16, KAN_I8, KAN_U16, KAN_U32, KAN_Q8, KAN_BFP8 = 0, 1, 2, 3, 4, 5, 6
KAN_PATH_AUTO, KAN_PATH_GATHER, KAN_PATH_MFMA = 0, 1, 2
KAN_RULE_BSPLINE3, KAN_RULE_PLI2 = 0, 1

EXPORTS = [
    "kan_bspline_basis", "kan_vq_workspace_bytes", "kan_vq_layer_forward",
    "kan_dense_workspace_bytes", "kan_dense_layer_forward", "kan_vq_head_forward",
    "kan_vq_debug_gather", "kan_vq_count_bad_indices", "kan_prof_begin", "kan_prof_end",
    "kan_status_string", "kan_vq_planned_kernel", "kan_dense_planned_kernel", "kan_vq_prepared_bytes", "kan_vq_prepare", "kan_pli_basis",
    "kan_vq_assign_workspace_bytes", "kan_vq_assign", "kan_vq_reconstruction_workspace_bytes",
    "kan_vq_reconstruction_sums", "kan_basis_window", "kan_vq_coef_range", "kan_vq_head_forward_static",
]
KAN_LAYER_NO_COLUMN = 1
KAN_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024


class kan_vq_layer(C.Structure):
    _fields_ = [
        ("n_in", C.c_int32), ("n_out", C.c_int32), ("G", C.c_int32), ("degree", C.c_int32),
        ("K", C.c_int32), ("idx_dtype", C.c_int32), ("gb_dtype", C.c_int32), ("cb_dtype", C.c_int32),
        ("idx", C.c_void_p), ("gain", C.c_void_p), ("bias", C.c_void_p), ("codebook", C.c_void_p),
        ("scale", C.c_float), ("rule", C.c_int32), ("prepared", C.c_void_p),
        ("gain_log2_lo", C.c_float), ("gain_log2_step", C.c_float), ("bias_scale", C.c_float), ("flags", C.c_int32),
    ]


class kan_prof_record(C.Structure):
    _fields_ = [("name", C.c_char * 56), ("launches", C.c_int32), ("total_ms", C.c_float)]


class KanError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


_lib = None


def lib():
    """The loaded shared library (loads on first use; raises if it is not built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2512_15742_amd.build`")
        L = C.CDLL(LIB_PATH)
        P, I32, I64, SZ = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        LP = C.POINTER(kan_vq_layer)
        L.kan_bspline_basis.argtypes = [P, I64, P, P, P]
        L.kan_bspline_basis.restype = I32
        L.kan_pli_basis.argtypes = [P, I64, P, P, P]
        L.kan_pli_basis.restype = I32
        L.kan_basis_window.argtypes = [P, I64, I32, I32, P, P, P]
        L.kan_basis_window.restype = I32
        L.kan_vq_workspace_bytes.argtypes = [LP, I32, I32, I64, I32]
        L.kan_vq_workspace_bytes.restype = SZ
        L.kan_vq_layer_forward.argtypes = [LP, P, I64, P, P, SZ, I32, P]
        L.kan_vq_layer_forward.restype = I32
        L.kan_dense_workspace_bytes.argtypes = [I32, I32, I64]
        L.kan_dense_workspace_bytes.restype = SZ
        L.kan_dense_layer_forward.argtypes = [P, I32, I32, I32, P, I64, P, P, SZ, P]
        L.kan_dense_layer_forward.restype = I32
        L.kan_vq_head_forward.argtypes = [LP, I32, I32, P, I64, P, P, SZ, I32, P]
        L.kan_vq_head_forward.restype = I32
        L.kan_vq_head_forward_static.argtypes = [LP, I32, I32, P, I64, P, I32, P]
        L.kan_vq_head_forward_static.restype = I32
        L.kan_vq_debug_gather.argtypes = [LP, P, P, P]
        L.kan_vq_debug_gather.restype = I32
        L.kan_vq_count_bad_indices.argtypes = [LP, P, P]
        L.kan_vq_count_bad_indices.restype = I32
        L.kan_vq_coef_range.argtypes = [LP, P, P]
        L.kan_vq_coef_range.restype = I32
        L.kan_prof_begin.argtypes = [I32]
        L.kan_prof_begin.restype = I32
        L.kan_prof_end.argtypes = [C.POINTER(kan_prof_record), I32, C.POINTER(I32)]
        L.kan_prof_end.restype = I32
        L.kan_status_string.argtypes = [I32]
        L.kan_status_string.restype = C.c_char_p
        L.kan_vq_planned_kernel.argtypes = [LP, I64, I32, I32]
        L.kan_vq_planned_kernel.restype = C.c_char_p
        L.kan_dense_planned_kernel.argtypes = [I32, I32, I64]
        L.kan_dense_planned_kernel.restype = C.c_char_p
        L.kan_vq_prepared_bytes.argtypes = [LP]
        L.kan_vq_prepared_bytes.restype = SZ
        L.kan_vq_prepare.argtypes = [LP, P, SZ, P]
        L.kan_vq_prepare.restype = I32
        L.kan_vq_assign_workspace_bytes.argtypes = [I32]
        L.kan_vq_assign_workspace_bytes.restype = SZ
        L.kan_vq_assign.argtypes = [P, I32, I32, P, I32, I32, P, P, P, P, SZ, P]
        L.kan_vq_assign.restype = I32
        L.kan_vq_reconstruction_workspace_bytes.argtypes = [I32, I32]
        L.kan_vq_reconstruction_workspace_bytes.restype = SZ
        L.kan_vq_reconstruction_sums.argtypes = [P, I32, I32, P, I32, I32, P, P, P, P, P, SZ, P]
        L.kan_vq_reconstruction_sums.restype = I32
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().kan_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != KAN_OK:
        raise KanError(status, where)


SIZE_INVALID = C.c_size_t(-1).value


def _torch():
    import torch
    return torch


def _stream_ptr():
    return C.c_void_p(_torch().cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


class VQLayer:
    """Device-resident parameters of one VQ layer plus its C descriptor."""

    def __init__(self, params, device="cuda", rule=KAN_RULE_BSPLINE3):
        torch = _torch()
        self.n_in, self.n_out, self.K = int(params.n_in), int(params.n_out), int(params.K)
        idx = np.ascontiguousarray(params.idx)
        # torch has no uint16/uint32 arithmetic; the bytes are carried in same-width ints
        view = {np.dtype(np.uint16): np.int16, np.dtype(np.uint32): np.int32}[idx.dtype]
        self.idx = torch.from_numpy(idx.view(view)).to(device)
        self.gain = torch.from_numpy(np.ascontiguousarray(params.gain)).to(device)
        self.bias = torch.from_numpy(np.ascontiguousarray(params.bias)).to(device)
        q8 = params.gain.dtype == np.uint8          # byte-coded gain (uint8) and bias (int8)
        gb = KAN_Q8 if q8 else (KAN_F16 if params.gain.dtype == np.float16 else KAN_F32)
        gbp = tuple(float(v) for v in params.gb_params) if q8 else (0.0, 0.0, 0.0)
        self.codebook = torch.from_numpy(np.ascontiguousarray(params.codebook)).to(device)
        self.scale = float(params.scale)
        self.desc = kan_vq_layer(
            self.n_in, self.n_out, 10, 3, self.K,
            KAN_U16 if idx.dtype == np.uint16 else KAN_U32,
            gb,
            # (an int8 array of 12-byte rows is a block-floating-point codebook: 10 mantissas, exponent, zero)
            KAN_BFP8 if (params.codebook.dtype == np.int8 and params.codebook.shape[1] == 12) else
            {np.dtype(np.int8): KAN_I8, np.dtype(np.float16): KAN_F16,
             np.dtype(np.float32): KAN_F32}[params.codebook.dtype],
            self.idx.data_ptr(), self.gain.data_ptr(), self.bias.data_ptr(), self.codebook.data_ptr(),
            self.scale, int(rule), None, gbp[0], gbp[1], gbp[2], 0)
        self.prepared = None

    def prepare(self):
        """Builds the small-batch layout (kan_vq_prepare) and attaches it to the descriptor."""
        self.prepared = kan_vq_prepare(self)
        self.desc.prepared = self.prepared.data_ptr()
        return self

    def unprepare(self):
        self.prepared = None
        self.desc.prepared = None
        return self

    def keep_on_bucket_kernel(self, on: bool = True):
        """KAN_LAYER_NO_COLUMN: a small prepared layer stays on the bucket kernel."""
        self.desc.flags = KAN_LAYER_NO_COLUMN if on else 0

    def use_prepared(self, on: bool):
        """Shows or hides an existing prepared buffer to the forward calls."""
        self.desc.prepared = self.prepared.data_ptr() if (on and self.prepared is not None) else None
        return self

    @property
    def metadata_bytes(self):
        return self.idx.numel() * self.idx.element_size() + 2 * self.gain.numel() * self.gain.element_size()


def _desc_array(heads):
    """heads: list (heads) of lists (layers) of VQLayer -> C array [n_heads][n_layers]."""
    n_heads, n_layers = len(heads), len(heads[0])
    arr = (kan_vq_layer * (n_heads * n_layers))()
    for h, layers in enumerate(heads):
        assert len(layers) == n_layers
        for l, L in enumerate(layers):
            arr[h * n_layers + l] = L.desc
    return arr, n_layers, n_heads


def _new_output(shape, device):
    """An output tensor the binding allocates itself starts as NaN, so that an element no kernel
    wrote cannot pass for a result (callers that time a call pass their own y)."""
    torch = _torch()
    return torch.full(shape, float("nan"), dtype=torch.float32, device=device)


def _workspace(nbytes, device):
    torch = _torch()
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def kan_bspline_basis(x):
    """x: float32 CUDA tensor (any shape) -> (span uint8 same shape, w float32 [..., 4])."""
    torch = _torch()
    x = x.contiguous()
    span = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    w = torch.empty(tuple(x.shape) + (4,), dtype=torch.float32, device=x.device)
    _check(lib().kan_bspline_basis(_ptr(x), x.numel(), _ptr(span), _ptr(w), _stream_ptr()), "kan_bspline_basis")
    return span, w


def kan_pli_basis(x):
    """x: float32 CUDA tensor (any shape) -> (index uint8 same shape, w float32 [..., 2])."""
    torch = _torch()
    x = x.contiguous()
    index = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    w = torch.empty(tuple(x.shape) + (2,), dtype=torch.float32, device=x.device)
    _check(lib().kan_pli_basis(_ptr(x), x.numel(), _ptr(index), _ptr(w), _stream_ptr()), "kan_pli_basis")
    return index, w


def kan_basis_window(x, rule=KAN_RULE_BSPLINE3, variant=0):
    """x: float32 CUDA tensor -> (start uint8 same shape, w float32 [..., 4]): the four-entry window
    of either rule as the kernels form it (variant 1: the routine of the matrix-core kernels)."""
    torch = _torch()
    x = x.contiguous()
    start = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    w = torch.empty(tuple(x.shape) + (4,), dtype=torch.float32, device=x.device)
    _check(lib().kan_basis_window(_ptr(x), x.numel(), int(rule), int(variant), _ptr(start), _ptr(w), _stream_ptr()),
           "kan_basis_window")
    return start, w


def kan_vq_workspace_bytes(heads, B, path=KAN_PATH_AUTO, strict=True) -> int:
    arr, n_layers, n_heads = _desc_array(heads)
    n = lib().kan_vq_workspace_bytes(arr, n_layers, n_heads, int(B), int(path))
    if n == SIZE_INVALID:
        if strict:
            raise KanError(KAN_ERR_SHAPE, "kan_vq_workspace_bytes")
        return 0        # the forward call that follows reports the precise status
    return n


def kan_vq_layer_forward(layer: VQLayer, x, path=KAN_PATH_AUTO, ws=None, y=None):
    torch = _torch()
    assert x.dtype == torch.float32 and x.is_contiguous() and x.shape[1] == layer.n_in
    B = x.shape[0]
    if ws is None:
        ws = _workspace(kan_vq_workspace_bytes([[layer]], B, path, strict=False), x.device)
    if y is None:
        y = _new_output((B, layer.n_out), x.device)
    st = lib().kan_vq_layer_forward(C.byref(layer.desc), _ptr(x), B, _ptr(y), _ptr(ws),
                                    0 if ws is None else ws.numel(), int(path), _stream_ptr())
    _check(st, "kan_vq_layer_forward")
    return y


def kan_vq_head_forward(heads, x, path=KAN_PATH_AUTO, ws=None, y=None):
    """heads: list of heads, each a list of VQLayer; x [B][in0] shared -> y [n_heads][B][out_last]."""
    torch = _torch()
    assert x.dtype == torch.float32 and x.is_contiguous()
    arr, n_layers, n_heads = _desc_array(heads)
    B = x.shape[0]
    if ws is None:
        ws = _workspace(kan_vq_workspace_bytes(heads, B, path, strict=False), x.device)
    if y is None:
        y = _new_output((n_heads, B, heads[0][-1].n_out), x.device)
    st = lib().kan_vq_head_forward(arr, n_layers, n_heads, _ptr(x), B, _ptr(y), _ptr(ws),
                                   0 if ws is None else ws.numel(), int(path), _stream_ptr())
    _check(st, "kan_vq_head_forward")
    return y


def kan_vq_head_forward_static(heads, x, path=KAN_PATH_AUTO, y=None):
    """kan_vq_head_forward on the library's own fixed scratch array: no workspace argument, and the
    call itself allocates nothing when y is given."""
    torch = _torch()
    assert x.dtype == torch.float32 and x.is_contiguous()
    arr, n_layers, n_heads = _desc_array(heads)
    B = x.shape[0]
    if y is None:
        y = _new_output((n_heads, B, heads[0][-1].n_out), x.device)
    st = lib().kan_vq_head_forward_static(arr, n_layers, n_heads, _ptr(x), B, _ptr(y), int(path), _stream_ptr())
    _check(st, "kan_vq_head_forward_static")
    return y


def kan_dense_workspace_bytes(n_in, n_out, B) -> int:
    n = lib().kan_dense_workspace_bytes(int(n_in), int(n_out), int(B))
    if n == SIZE_INVALID:
        raise KanError(KAN_ERR_SHAPE, "kan_dense_workspace_bytes")
    return n


def kan_dense_layer_forward(coef, x, ws=None, y=None):
    """coef [in][out][10] float32, x [B][in] float32 -> y [B][out]."""
    torch = _torch()
    assert coef.dtype == torch.float32 and coef.is_contiguous() and x.is_contiguous()
    n_in, n_out, g = coef.shape
    B = x.shape[0]
    if ws is None:
        ws = _workspace(kan_dense_workspace_bytes(n_in, n_out, B), x.device)
    if y is None:
        y = _new_output((B, n_out), x.device)
    st = lib().kan_dense_layer_forward(_ptr(coef), n_in, n_out, g, _ptr(x), B, _ptr(y), _ptr(ws),
                                       0 if ws is None else ws.numel(), _stream_ptr())
    _check(st, "kan_dense_layer_forward")
    return y


def kan_vq_debug_gather(layer: VQLayer, want_rows=True):
    torch = _torch()
    E = layer.n_in * layer.n_out
    dev = layer.idx.device
    ids = torch.empty(E, dtype=torch.int32, device=dev)
    rows = torch.empty((E, 10), dtype=torch.float32, device=dev) if want_rows else None
    _check(lib().kan_vq_debug_gather(C.byref(layer.desc), _ptr(ids), _ptr(rows), _stream_ptr()), "kan_vq_debug_gather")
    return ids, rows


def kan_vq_count_bad_indices(layer: VQLayer) -> int:
    torch = _torch()
    cnt = torch.zeros(1, dtype=torch.int32, device=layer.idx.device)
    _check(lib().kan_vq_count_bad_indices(C.byref(layer.desc), _ptr(cnt), _stream_ptr()), "kan_vq_count_bad_indices")
    return int(cnt.item())


def kan_vq_coef_range(layer: VQLayer):
    """(smallest nonzero, largest) magnitude of the fp16 coefficient operand gain * q / gain * C."""
    torch = _torch()
    r = torch.empty(2, dtype=torch.float32, device=layer.idx.device)
    _check(lib().kan_vq_coef_range(C.byref(layer.desc), _ptr(r), _stream_ptr()), "kan_vq_coef_range")
    lo, hi = (float(v) for v in r.cpu())
    return lo, hi


def kan_vq_prepared_bytes(layer: VQLayer) -> int:
    n = lib().kan_vq_prepared_bytes(C.byref(layer.desc))
    if n == SIZE_INVALID:
        raise KanError(KAN_ERR_SHAPE, "kan_vq_prepared_bytes")
    return n


def kan_vq_prepare(layer: VQLayer, out=None):
    """Returns the uint8 CUDA tensor holding the regrouped layer (caller keeps it alive)."""
    torch = _torch()
    n = kan_vq_prepared_bytes(layer)
    if out is None:
        out = torch.empty(max(n, 1), dtype=torch.uint8, device=layer.idx.device)
    _check(lib().kan_vq_prepare(C.byref(layer.desc), _ptr(out), out.numel(), _stream_ptr()), "kan_vq_prepare")
    return out


def kan_vq_assign(coef, codebook, ws=None):
    """coef [in][out][10] float32, codebook [K][10] float32 (CUDA tensors) ->
    (idx int16/int32 carrying uint16/uint32 bits [in][out], gain float32 [in][out], bias float32 [in][out])."""
    torch = _torch()
    assert coef.dtype == torch.float32 and coef.is_contiguous() and coef.shape[2] == 10
    assert codebook.dtype == torch.float32 and codebook.is_contiguous() and codebook.shape[1] == 10
    n_in, n_out, _ = coef.shape
    K = codebook.shape[0]
    u16 = K <= 65536
    idx = torch.empty((n_in, n_out), dtype=torch.int16 if u16 else torch.int32, device=coef.device)
    gain = torch.empty((n_in, n_out), dtype=torch.float32, device=coef.device)
    bias = torch.empty((n_in, n_out), dtype=torch.float32, device=coef.device)
    if ws is None:
        ws = _workspace(lib().kan_vq_assign_workspace_bytes(K), coef.device)
    st = lib().kan_vq_assign(_ptr(coef), n_in, n_out, _ptr(codebook), K, KAN_U16 if u16 else KAN_U32, _ptr(idx),
                             _ptr(gain), _ptr(bias), _ptr(ws), ws.numel(), _stream_ptr())
    _check(st, "kan_vq_assign")
    return idx, gain, bias


def kan_vq_reconstruction_r2(coef, codebook, idx, gain, bias) -> float:
    """R^2 between the dense grids and gain * C[idx] + bias, as the library computes it (fp64)."""
    torch = _torch()
    n_in, n_out, _ = coef.shape
    K = codebook.shape[0]
    ws = _workspace(lib().kan_vq_reconstruction_workspace_bytes(n_in, n_out), coef.device)
    sums = torch.empty(4, dtype=torch.float64, device=coef.device)
    st = lib().kan_vq_reconstruction_sums(_ptr(coef), n_in, n_out, _ptr(codebook), K,
                                          KAN_U16 if idx.dtype == torch.int16 else KAN_U32, _ptr(idx), _ptr(gain),
                                          _ptr(bias), _ptr(sums), _ptr(ws), ws.numel(), _stream_ptr())
    _check(st, "kan_vq_reconstruction_sums")
    return float(sums[3].item())


def kan_vq_planned_kernel(layer: VQLayer, B, n_heads=1, path=KAN_PATH_AUTO) -> str:
    return lib().kan_vq_planned_kernel(C.byref(layer.desc), int(B), int(n_heads), int(path)).decode()


def kan_dense_planned_kernel(n_in, n_out, B) -> str:
    return lib().kan_dense_planned_kernel(int(n_in), int(n_out), int(B)).decode()


def kan_prof_begin(max_launches=4096):
    _check(lib().kan_prof_begin(int(max_launches)), "kan_prof_begin")


def kan_prof_end(cap=64) -> dict:
    recs = (kan_prof_record * cap)()
    n = C.c_int32(0)
    _check(lib().kan_prof_end(recs, cap, C.byref(n)), "kan_prof_end")
    return {recs[i].name.decode(): {"launches": recs[i].launches, "total_ms": recs[i].total_ms}
            for i in range(n.value)}
