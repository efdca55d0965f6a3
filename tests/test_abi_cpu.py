"""Host-side checks of the C-ABI that need no GPU: the library loads, exports
every function include/kan.h declares, rejects invalid arguments before any
launch, and plans workspaces consistently.  No compute call is made here."""
import ctypes as C
import os
import re

import pytest

from paper_2512_15742_amd import binding as kb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.skipif(not os.path.exists(kb.LIB_PATH), reason="library not built")


def _declared():
    text = open(os.path.join(ROOT, "include", "kan.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kan_[a-z0-9_]+)\s*\(", text)))


def test_exports_match_header():
    names = _declared()
    assert set(names) == set(kb.EXPORTS)
    L = kb.lib()
    for n in names:
        assert hasattr(L, n), n


def test_struct_layout_matches_header():
    # 8 int32, 4 pointers, float, int32, pointer, 3 floats, int32 -> 96 bytes on LP64;
    # profile record 56 + 4 + 4
    assert C.sizeof(kb.kan_vq_layer) == 96
    assert kb.kan_vq_layer.prepared.offset == 72
    assert kb.kan_vq_layer.gain_log2_lo.offset == 80 and kb.kan_vq_layer.bias_scale.offset == 88
    assert C.sizeof(kb.kan_prof_record) == 64


def test_status_strings():
    seen = {kb.status_string(s) for s in range(7)}
    assert len(seen) == 7
    assert kb.status_string(99) == "unknown status"


def _desc(**kw):
    base = dict(n_in=8, n_out=8, G=10, degree=3, K=16, idx_dtype=kb.KAN_U16, gb_dtype=kb.KAN_F32,
                cb_dtype=kb.KAN_F32, idx=0x1000, gain=0x2000, bias=0x3000, codebook=0x4000,
                scale=1.0, rule=0, prepared=None, gain_log2_lo=0.0, gain_log2_step=0.0,
                bias_scale=0.0, flags=0)
    base.update(kw)
    return kb.kan_vq_layer(**base)


FAKE = C.c_void_p(0x10000)


@pytest.mark.parametrize("kw,status", [
    (dict(G=8), kb.KAN_ERR_UNSUPPORTED),
    (dict(degree=2), kb.KAN_ERR_UNSUPPORTED),
    (dict(rule=2), kb.KAN_ERR_UNSUPPORTED),
    (dict(n_in=0), kb.KAN_ERR_SHAPE),
    (dict(n_out=-3), kb.KAN_ERR_SHAPE),
    (dict(K=0), kb.KAN_ERR_SHAPE),
    (dict(K=65537), kb.KAN_ERR_SHAPE),                       # does not fit a 16-bit index
    (dict(idx_dtype=kb.KAN_F32), kb.KAN_ERR_DTYPE),
    (dict(gb_dtype=kb.KAN_I8), kb.KAN_ERR_DTYPE),
    (dict(gb_dtype=kb.KAN_Q8), kb.KAN_ERR_UNSUPPORTED),       # byte-coded gain/bias need an Int8 codebook
    (dict(cb_dtype=kb.KAN_U16), kb.KAN_ERR_DTYPE),
    (dict(cb_dtype=kb.KAN_F16, codebook=0x4002), kb.KAN_ERR_SHAPE),   # fp16 rows are read in pairs: 4-byte alignment
    (dict(cb_dtype=kb.KAN_F16, gb_dtype=kb.KAN_Q8), kb.KAN_ERR_UNSUPPORTED),
    (dict(idx=0), kb.KAN_ERR_NULL),
    (dict(codebook=0), kb.KAN_ERR_NULL),
    (dict(gain=0x2001), kb.KAN_ERR_SHAPE),                   # misaligned fp32
    (dict(codebook=0x4004), kb.KAN_ERR_SHAPE),               # fp32 rows need 8-byte alignment
])
def test_layer_validation_rejects_before_launch(kw, status):
    d = _desc(**kw)
    st = kb.lib().kan_vq_layer_forward(C.byref(d), FAKE, 4, FAKE, FAKE, 1 << 20, kb.KAN_PATH_AUTO, None)
    assert st == status
    assert kb.lib().kan_vq_workspace_bytes(C.byref(d), 1, 1, 4, kb.KAN_PATH_AUTO) == kb.SIZE_INVALID
    assert kb.lib().kan_vq_debug_gather(C.byref(d), FAKE, FAKE, None) == status
    assert kb.lib().kan_vq_count_bad_indices(C.byref(d), FAKE, None) == status


def test_forward_argument_errors():
    L = kb.lib()
    d = _desc()
    assert L.kan_vq_layer_forward(None, FAKE, 4, FAKE, FAKE, 1 << 20, 0, None) == kb.KAN_ERR_NULL
    assert L.kan_vq_layer_forward(C.byref(d), None, 4, FAKE, FAKE, 1 << 20, 0, None) == kb.KAN_ERR_NULL
    assert L.kan_vq_layer_forward(C.byref(d), FAKE, 4, None, FAKE, 1 << 20, 0, None) == kb.KAN_ERR_NULL
    assert L.kan_vq_layer_forward(C.byref(d), FAKE, -1, FAKE, FAKE, 1 << 20, 0, None) == kb.KAN_ERR_SHAPE
    assert L.kan_vq_layer_forward(C.byref(d), FAKE, 4, FAKE, FAKE, 1 << 20, 17, None) == kb.KAN_ERR_UNSUPPORTED
    # B == 0 is a no-op
    assert L.kan_vq_layer_forward(C.byref(d), None, 0, None, None, 0, 0, None) == kb.KAN_OK
    assert L.kan_bspline_basis(None, 0, None, None, None) == kb.KAN_OK
    assert L.kan_bspline_basis(None, 5, FAKE, FAKE, None) == kb.KAN_ERR_NULL
    assert L.kan_bspline_basis(FAKE, -1, FAKE, FAKE, None) == kb.KAN_ERR_SHAPE
    assert L.kan_pli_basis(None, 0, None, None, None) == kb.KAN_OK
    assert L.kan_pli_basis(FAKE, 5, None, FAKE, None) == kb.KAN_ERR_NULL
    assert L.kan_pli_basis(FAKE, -1, FAKE, FAKE, None) == kb.KAN_ERR_SHAPE
    assert L.kan_dense_layer_forward(FAKE, 8, 8, 9, FAKE, 4, FAKE, None, 0, None) == kb.KAN_ERR_UNSUPPORTED
    assert L.kan_dense_layer_forward(FAKE, 0, 8, 10, FAKE, 4, FAKE, None, 0, None) == kb.KAN_ERR_SHAPE
    assert L.kan_dense_layer_forward(None, 8, 8, 10, FAKE, 4, FAKE, None, 0, None) == kb.KAN_ERR_NULL
    assert L.kan_dense_layer_forward(None, 8, 8, 10, None, 0, None, None, 0, None) == kb.KAN_OK


def test_workspace_required_and_checked():
    L = kb.lib()
    # a layer wide enough that i is split into chunks needs room for partial sums
    d = _desc(n_in=2048, n_out=1024, K=65536, cb_dtype=kb.KAN_I8, gb_dtype=kb.KAN_F16)
    need = L.kan_vq_workspace_bytes(C.byref(d), 1, 1, 1, kb.KAN_PATH_GATHER)
    assert 0 < need < (64 << 20) and need % 256 == 0
    assert L.kan_vq_layer_forward(C.byref(d), FAKE, 1, FAKE, None, 0, kb.KAN_PATH_GATHER, None) == kb.KAN_ERR_WORKSPACE
    assert L.kan_vq_layer_forward(C.byref(d), FAKE, 1, FAKE, FAKE, need - 1, kb.KAN_PATH_GATHER, None) == kb.KAN_ERR_WORKSPACE
    assert L.kan_vq_layer_forward(C.byref(d), FAKE, 1, FAKE, C.c_void_p(0x10010), need, kb.KAN_PATH_GATHER, None) == kb.KAN_ERR_WORKSPACE
    assert L.kan_vq_workspace_bytes(C.byref(d), 1, 1, 0, kb.KAN_PATH_AUTO) == 0
    assert L.kan_dense_workspace_bytes(2048, 512, 1) > 0
    assert L.kan_dense_workspace_bytes(0, 512, 1) == kb.SIZE_INVALID


def test_prepare_arguments_and_planning():
    L = kb.lib()
    d = _desc(n_in=2048, n_out=1024, K=65536, cb_dtype=kb.KAN_I8, gb_dtype=kb.KAN_F16)
    need = L.kan_vq_prepared_bytes(C.byref(d))
    # segment table + bias sums + 6 bytes per edge (u16 input, u16 local id, fp16 gain)
    E = 2048 * 1024
    # (+ the preparation's scratch: a u16 count per (block of 256 inputs, bucket, output), a bias sum per (block, output))
    scratch = 8 * 8 * 1024 * 2 + 8 * 1024 * 8
    assert need % 256 == 0 and 6 * E + scratch < need < 6 * E + scratch + (1 << 17)
    assert L.kan_vq_prepare(C.byref(d), None, need, None) == kb.KAN_ERR_WORKSPACE
    assert L.kan_vq_prepare(C.byref(d), FAKE, need - 1, None) == kb.KAN_ERR_WORKSPACE
    assert L.kan_vq_prepare(C.byref(d), C.c_void_p(0x10010), need, None) == kb.KAN_ERR_WORKSPACE
    assert L.kan_vq_prepare(None, FAKE, need, None) == kb.KAN_ERR_NULL
    wide = _desc(n_in=4097, n_out=8)
    assert L.kan_vq_prepared_bytes(C.byref(wide)) == 0
    assert L.kan_vq_prepare(C.byref(wide), FAKE, 1 << 30, None) == kb.KAN_ERR_UNSUPPORTED
    assert L.kan_vq_prepared_bytes(C.byref(_desc(G=8))) == kb.SIZE_INVALID
    # planning: a prepared layer takes the bucket kernel on the precise path up to batch 4
    assert L.kan_vq_planned_kernel(C.byref(d), 1, 1, kb.KAN_PATH_GATHER) == b"kan_gather_bt1"
    d.prepared = 0x100000
    assert L.kan_vq_planned_kernel(C.byref(d), 1, 1, kb.KAN_PATH_GATHER) == b"kan_bucket"
    assert L.kan_vq_planned_kernel(C.byref(d), 4, 1, kb.KAN_PATH_AUTO) == b"kan_bucket"
    assert L.kan_vq_planned_kernel(C.byref(d), 5, 1, kb.KAN_PATH_GATHER) == b"kan_fused_f32"
    assert L.kan_vq_planned_kernel(C.byref(d), 1, 1, kb.KAN_PATH_MFMA) == b"kan_fused_f16"
    # per-bucket partial sums: 8 buckets x out floats
    assert L.kan_vq_workspace_bytes(C.byref(d), 1, 1, 1, kb.KAN_PATH_GATHER) == 8 * 1024 * 4
    d.codebook = 0x4008                                  # bucket copies need 16-byte alignment
    assert L.kan_vq_planned_kernel(C.byref(d), 1, 1, kb.KAN_PATH_GATHER) == b"kan_gather_bt1"


def test_byte_coded_layers_plan_and_prepare():
    L = kb.lib()
    d = _desc(n_in=2048, n_out=1024, K=65536, cb_dtype=kb.KAN_I8, gb_dtype=kb.KAN_Q8, gain=0x2001, bias=0x3003,
              gain_log2_lo=-12.0, gain_log2_step=0.04, bias_scale=1e-4)
    assert L.kan_vq_workspace_bytes(C.byref(d), 1, 1, 16, kb.KAN_PATH_AUTO) != kb.SIZE_INVALID   # bytes need no alignment
    need = L.kan_vq_prepared_bytes(C.byref(d))
    E = 2048 * 1024
    scratch = 8 * 8 * 1024 * 2 + 8 * 1024 * 8            # the preparation's scratch (counts per row block, bias sums)
    assert 5 * E + scratch < need < 5 * E + scratch + (1 << 17)      # u16 input + u16 local id + 1-byte gain code


def test_fp16_codebook_layers_plan_and_prepare():
    L = kb.lib()
    d = _desc(n_in=2048, n_out=1024, K=65536, cb_dtype=kb.KAN_F16, gb_dtype=kb.KAN_F16, codebook=0x4004)
    for B, path, name in ((1, kb.KAN_PATH_GATHER, b"kan_gather_bt1"), (16, kb.KAN_PATH_GATHER, b"kan_fused_f32"),
                          (16, kb.KAN_PATH_MFMA, b"kan_fused_f16"), (1024, kb.KAN_PATH_AUTO, b"kan_mfma")):
        assert L.kan_vq_planned_kernel(C.byref(d), B, 1, path) == name
        assert L.kan_vq_workspace_bytes(C.byref(d), 1, 1, B, path) != kb.SIZE_INVALID
    E = 2048 * 1024
    need = L.kan_vq_prepared_bytes(C.byref(d))
    scratch = 8 * 16 * 1024 * 2 + 8 * 1024 * 8                    # the preparation's scratch (counts per row block, bias sums)
    assert 6 * E + scratch < need < 6 * E + scratch + 16 * 1024 * 4 * 2 + (1 << 17)   # 16 buckets of 4096 fp16 rows: 16 segment tables
    assert L.kan_vq_prepare(C.byref(d), FAKE, need - 1, None) == kb.KAN_ERR_WORKSPACE
    d.prepared = 0x100000
    assert L.kan_vq_planned_kernel(C.byref(d), 1, 1, kb.KAN_PATH_GATHER) == b"kan_gather_bt1"   # codebook not 16-byte aligned
    d.codebook = 0x4000
    assert L.kan_vq_planned_kernel(C.byref(d), 1, 1, kb.KAN_PATH_GATHER) == b"kan_bucket"
    assert L.kan_vq_planned_kernel(C.byref(d), 4, 1, kb.KAN_PATH_AUTO) == b"kan_bucket"
    assert L.kan_vq_planned_kernel(C.byref(d), 8, 1, kb.KAN_PATH_GATHER) == b"kan_fused_f32"
    # the largest layers leave the bucket kernel one sample earlier (2^23 edges or more)
    n_in0, n_out0 = d.n_in, d.n_out
    d.n_in, d.n_out = 4096, 2048
    assert L.kan_vq_planned_kernel(C.byref(d), 3, 1, kb.KAN_PATH_GATHER) == b"kan_bucket"
    assert L.kan_vq_planned_kernel(C.byref(d), 4, 1, kb.KAN_PATH_GATHER) == b"kan_fused_f32"
    d.n_in, d.n_out = n_in0, n_out0


def test_precise_path_switches_and_workspace_sizes():
    """Host logic only: where the precise path and the dense baseline change kernels, and that
    the workspace of the split form holds both parts of both operands and one set of partial
    sums (its three products are passes of one launch)."""
    L = kb.lib()
    d = _desc(n_in=2048, n_out=1024, K=65536)
    assert L.kan_vq_planned_kernel(C.byref(d), 64, 1, kb.KAN_PATH_GATHER) == b"kan_fused_f32"
    assert L.kan_vq_planned_kernel(C.byref(d), 65, 1, kb.KAN_PATH_GATHER) == b"kan_mfma_split"
    assert L.kan_vq_planned_kernel(C.byref(d), 65, 1, kb.KAN_PATH_MFMA) == b"kan_mfma"
    assert L.kan_dense_planned_kernel(2048, 1024, 16) == b"kan_dense"
    assert L.kan_dense_planned_kernel(2048, 1024, 17) == b"kan_dense_split"
    assert L.kan_dense_planned_kernel(2048, 1024, 0) == b"invalid"
    B = 1024
    one = L.kan_vq_workspace_bytes(C.byref(d), 1, 1, B, kb.KAN_PATH_MFMA)
    three = L.kan_vq_workspace_bytes(C.byref(d), 1, 1, B, kb.KAN_PATH_GATHER)
    records = (2048 // 16) * 20 * 1024 * 16              # coefficient records of one part
    words = 2048 * B * 8                                 # basis words of one part
    assert three - one == records + words, (one, three)  # same chunks, same partial sums
    dense = L.kan_dense_workspace_bytes(2048, 1024, B)
    assert dense >= 2 * (records + words) and dense < three


def test_assign_argument_errors():
    L = kb.lib()
    F = FAKE
    need = L.kan_vq_assign_workspace_bytes(65536)
    assert need == 65536 * 64
    assert L.kan_vq_assign(F, 8, 8, F, 65537, kb.KAN_U16, F, F, F, F, 1 << 30, None) == kb.KAN_ERR_SHAPE
    assert L.kan_vq_assign(F, 8, 8, F, 100, kb.KAN_F32, F, F, F, F, 1 << 30, None) == kb.KAN_ERR_DTYPE
    assert L.kan_vq_assign(None, 8, 8, F, 100, kb.KAN_U16, F, F, F, F, 1 << 30, None) == kb.KAN_ERR_NULL
    assert L.kan_vq_assign(F, 8, 8, F, 100, kb.KAN_U16, F, F, F, F, 100, None) == kb.KAN_ERR_WORKSPACE
    assert L.kan_vq_assign(F, 0, 8, F, 100, kb.KAN_U16, F, F, F, F, 1 << 30, None) == kb.KAN_ERR_SHAPE
    assert L.kan_vq_reconstruction_sums(F, 8, 8, F, 100, kb.KAN_U16, F, F, F, None, F, 1 << 20, None) == kb.KAN_ERR_NULL


def test_head_table_consistency():
    L = kb.lib()
    arr = (kb.kan_vq_layer * 4)()
    arr[0] = _desc(n_in=32, n_out=16)
    arr[1] = _desc(n_in=16, n_out=4)
    arr[2] = _desc(n_in=32, n_out=16)
    arr[3] = _desc(n_in=16, n_out=4)
    assert L.kan_vq_workspace_bytes(arr, 2, 2, 8, 0) != kb.SIZE_INVALID
    arr[2] = _desc(n_in=32, n_out=16, rule=kb.KAN_RULE_PLI2)       # heads must share the edge rule
    assert L.kan_vq_head_forward(arr, 2, 2, FAKE, 8, FAKE, FAKE, 1 << 24, 0, None) == kb.KAN_ERR_UNSUPPORTED
    arr[2] = _desc(n_in=32, n_out=16)
    arr[3] = _desc(n_in=16, n_out=5)            # heads must share layer shapes
    assert L.kan_vq_head_forward(arr, 2, 2, FAKE, 8, FAKE, FAKE, 1 << 24, 0, None) == kb.KAN_ERR_UNSUPPORTED
    arr[1] = _desc(n_in=15, n_out=4)            # layer chain broken: 16 -> 15
    arr[3] = _desc(n_in=15, n_out=4)
    assert L.kan_vq_head_forward(arr, 2, 2, FAKE, 8, FAKE, FAKE, 1 << 24, 0, None) == kb.KAN_ERR_SHAPE
    assert L.kan_vq_head_forward(arr, 0, 2, FAKE, 8, FAKE, FAKE, 1 << 24, 0, None) == kb.KAN_ERR_SHAPE
    assert L.kan_vq_head_forward(None, 2, 2, FAKE, 8, FAKE, FAKE, 1 << 24, 0, None) == kb.KAN_ERR_NULL


def test_prof_state_machine_without_gpu_work():
    L = kb.lib()
    n = C.c_int32(-1)
    assert L.kan_prof_end(None, 0, C.byref(n)) == kb.KAN_ERR_UNSUPPORTED      # not begun
    assert L.kan_prof_begin(0) == kb.KAN_ERR_SHAPE


def test_planner_accepts_every_shape_and_names_a_known_kernel():
    """Host logic over a seeded sweep of shapes, batches, head counts, storage types and paths:
    the workspace query succeeds, is a multiple of 256 bytes, and the kernel the dispatcher
    names is one of the families the library has."""
    import numpy as np
    L = kb.lib()
    rng = np.random.default_rng(20251127)
    known = {b"kan_gather_bt1", b"kan_gather_bt4", b"kan_gather_bt16", b"kan_fused_f32", b"kan_fused_f16",
             b"kan_mfma", b"kan_mfma_split", b"kan_bucket"}
    kinds = [(kb.KAN_F32, kb.KAN_F32), (kb.KAN_I8, kb.KAN_F16), (kb.KAN_I8, kb.KAN_F32), (kb.KAN_F16, kb.KAN_F16),
             (kb.KAN_I8, kb.KAN_Q8)]
    seen = set()
    for _ in range(400):
        n_in = int(rng.choice([1, 3, 8, 64, 130, 1000, 2048, 4100, 8192]))
        n_out = int(rng.choice([1, 8, 21, 128, 264, 1024, 4096]))
        B = int(rng.choice([1, 2, 4, 5, 16, 33, 64, 65, 111, 200, 1024, 5000]))
        heads = int(rng.choice([1, 1, 2, 50, 70]))
        cb, gb = kinds[int(rng.integers(len(kinds)))]
        u32 = bool(rng.integers(2))
        d = _desc(n_in=n_in, n_out=n_out, K=70000 if u32 else 4096, cb_dtype=cb, gb_dtype=gb,
                  idx_dtype=kb.KAN_U32 if u32 else kb.KAN_U16, scale=0.01, gain_log2_lo=-8.0, gain_log2_step=0.05,
                  bias_scale=1e-3)
        for path in (kb.KAN_PATH_AUTO, kb.KAN_PATH_GATHER, kb.KAN_PATH_MFMA):
            name = L.kan_vq_planned_kernel(C.byref(d), B, heads, path)
            assert name in known, (n_in, n_out, B, heads, cb, gb, path, name)
            seen.add(name)
            arr = (kb.kan_vq_layer * heads)(*([d] * heads))
            ws = L.kan_vq_workspace_bytes(arr, 1, heads, B, path)
            assert ws != kb.SIZE_INVALID and ws % 256 == 0, (n_in, n_out, B, heads, path, ws)
    assert {b"kan_gather_bt1", b"kan_fused_f32", b"kan_fused_f16", b"kan_mfma", b"kan_mfma_split"} <= seen
