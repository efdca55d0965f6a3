"""GPU parity of the small-batch path over prepared layers (codebook buckets in LDS).

The regrouped layout is integer work and must be bit-exact: the expected layout is built
here with numpy straight from the layer's idx/gain/bias.  The forward results are compared
with the float64 oracle under the same 1e-5 bound as the other fp32 kernels."""
import dataclasses

import numpy as np
import pytest

from oracle import kan_oracle as ko
from paper_2512_15742_amd import synth

from kan_testlib import TOL_FP32, check_layer_output, gpu_layers, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def kb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2512_15742_amd import binding
    binding.lib()
    return binding


def _bucket_rows(P):
    """Codewords per bucket: 80 KB of rows, 40 KB for layers with more than 2048 inputs."""
    rows = {np.dtype(np.int8): 8192, np.dtype(np.float16): 4096}.get(P.codebook.dtype, 2048)
    return rows // 2 if P.idx.shape[0] > 2048 else rows


def _bias_f64(P):
    """Per-edge biases as float64 (the prepared layout is not used with byte-coded biases here)."""
    return P.bias.astype(np.float64)


def _expected_layout(P):
    """(seg_off, bias_sum, i, q, gain) of the regrouped layer: bucket-major, then j, then i."""
    n_in, n_out = P.idx.shape
    rows = _bucket_rows(P)
    nb = (P.K + rows - 1) // rows
    idx = P.idx.astype(np.int64)
    bucket = idx // rows
    ii, jj = np.meshgrid(np.arange(n_in), np.arange(n_out), indexing="ij")
    order = np.lexsort((ii.ravel(), jj.ravel(), bucket.ravel()))          # last key is primary
    counts = np.zeros(nb * n_out, dtype=np.int64)
    np.add.at(counts, (bucket * n_out + jj).ravel(), 1)
    seg = np.concatenate([[0], np.cumsum(counts)]).astype(np.uint32)
    # same order as the kernel: fp64 sums over quarters of 64 inputs, ((q0 + q1) + q2) + q3 per block of
    # 256 inputs, the blocks added in order, rounded once to fp32
    bias_sum = np.zeros(n_out, dtype=np.float64)
    b64 = _bias_f64(P)
    for r0 in range(0, n_in, 256):
        quarters = []
        for q0 in range(r0, r0 + 256, 64):
            acc = np.zeros(n_out, dtype=np.float64)
            for i in range(q0, min(q0 + 64, n_in)):
                acc += b64[i]
            quarters.append(acc)
        bias_sum += ((quarters[0] + quarters[1]) + quarters[2]) + quarters[3]
    return (seg, bias_sum.astype(np.float32), ii.ravel()[order].astype(np.uint16),
            (idx.ravel()[order] % rows).astype(np.uint16), P.gain.ravel()[order])


def _read_layout(buf, P):
    up = lambda v: (v + 32 + 255) // 256 * 256       # every array is followed by >= 32 bytes of slack
    n_in, n_out = P.idx.shape
    rows = _bucket_rows(P)
    nb = (P.K + rows - 1) // rows
    E = n_in * n_out
    raw = buf.cpu().numpy()
    o = 0
    seg = raw[o:o + (nb * n_out + 1) * 4].view(np.uint32); o += up((nb * n_out + 1) * 4)
    bias = raw[o:o + n_out * 4].view(np.float32); o += up(n_out * 4)
    pi = raw[o:o + 2 * E].view(np.uint16); o += up(2 * E)
    pq = raw[o:o + 2 * E].view(np.uint16); o += up(2 * E)
    gsz = P.gain.dtype.itemsize
    pg = raw[o:o + gsz * E].view(P.gain.dtype); o += up(gsz * E)
    # block tables (five, for 1, 2, 3, 4 and more samples x heads) and the per-bucket block counts
    w_min = nb * ((n_out + 1023) // 1024)
    tab_w = [max(256 // (t + 1), w_min) for t in range(4)] + [w_min]
    tables = []
    for w in tab_w:
        tables.append(raw[o:o + w * 32].view(np.uint32).reshape(w, 8))
        o += w * 32
    o = (o + 32 + 255) // 256 * 256
    o += up(5 * (nb + 1) * 4)
    # scratch of the preparation: edges per (row block of 256 inputs, bucket, output) as u16, bias sums per row block as fp64
    n_rb = (n_in + 255) // 256
    o += up(n_rb * nb * n_out * 2) + up(n_rb * n_out * 8)
    if E <= 2 ** 20:
        # small layers: ids (as u32) and gains once more, transposed (the inputs of an output side by side)
        ti = raw[o:o + 4 * E].view(np.uint32).reshape(n_out, n_in); o += up(4 * E)
        tgn = raw[o:o + gsz * E].view(P.gain.dtype).reshape(n_out, n_in); o += up(gsz * E)
        assert np.array_equal(ti, P.idx.T.astype(np.uint32))
        assert np.array_equal(tgn.view(np.uint8), np.ascontiguousarray(P.gain.T).view(np.uint8))
    assert o == raw.size
    _read_layout.tables = tables
    return seg, bias, pi, pq, pg


def _table_position(s, W):
    """Position of the s-th block of the bucket-sorted list: the list is dealt out in 8 contiguous
    runs, run x taking positions x, x + 8, ... (workgroups go to the 8 XCDs in turn)."""
    base, rem = W >> 3, W & 7
    x = start = 0
    while x < 7:
        c = base + (1 if x < rem else 0)
        if s < start + c:
            break
        start += c
        x += 1
    return (s - start) * 8 + x


def _check_tables(tables, seg, nb, n_in, n_out):
    """Every table cuts every bucket's outputs into consecutive blocks of at most 1024 outputs,
    carries the matching edge bounds, and gives the buckets blocks in proportion to their edges."""
    E = int(seg[-1])
    m = (n_out + 1023) // 1024
    for T in tables:
        W = len(T)
        T = T[[_table_position(q, W) for q in range(W)]]          # back to bucket order
        assert (T[:, 5:] == 0).all()
        buckets = T[:, 0].astype(np.int64)
        assert (np.diff(buckets) >= 0).all() and set(buckets.tolist()) == set(range(nb))
        for b in range(nb):
            rows = T[buckets == b]
            assert len(rows) >= m
            assert rows[0, 1] == 0 and rows[-1, 2] == n_out
            assert (rows[1:, 1] == rows[:-1, 2]).all()
            assert ((rows[:, 2].astype(np.int64) - rows[:, 1]) <= 1024).all() and (rows[:, 2] >= rows[:, 1]).all()
            assert np.array_equal(rows[:, 3], seg[b * n_out + rows[:, 1].astype(np.int64)])
            assert np.array_equal(rows[:, 4], seg[b * n_out + rows[:, 2].astype(np.int64)])
            e_b = int(seg[(b + 1) * n_out]) - int(seg[b * n_out])
            spare = W - nb * m
            assert abs(len(rows) - m - spare * e_b / max(E, 1)) <= 1.0 + 1e-9
        edges = T[:, 4].astype(np.int64) - T[:, 3]
        assert edges.sum() == E
        if n_out <= 1024 and W >= 8 * nb * m:      # enough blocks to share out, no output-count limit in the way
            assert edges.max() <= 2 * (E / W) + 2 * n_in


@pytest.mark.parametrize("n_in,n_out,K,cb,gb,idxd", [
    (37, 29, 20000, "i8", "f16", "u16"),       # 3 buckets, the last one partial
    (64, 32, 256, "f32", "f32", "u16"),        # one bucket
    (130, 300, 70000, "f32", "f16", "u32"),    # 35 fp32 buckets
    (77, 130, 9000, "f16", "f16", "u16"),      # 3 fp16 buckets of 4096 rows, the last one partial
    (2050, 11, 4100, "f16", "f32", "u16"),     # more than 2048 inputs: fp16 buckets of 2048 rows
    (2048, 64, 65536, "i8", "f16", "u16"),
    (2100, 9, 30000, "i8", "f32", "u16"),      # more than 2048 inputs: buckets of 4096 rows
])
def test_prepared_layout_bit_exact(kb, n_in, n_out, K, cb, gb, idxd):
    P = synth.make_layer(n_in + K, n_in, n_out, K, cb_dtype=cb, gb_dtype=gb, idx_dtype=idxd)
    P.idx.reshape(-1)[:4] = [0, K - 1, min(K - 1, 8191), min(K - 1, 8192)]
    L = kb.VQLayer(P).prepare()
    assert L.prepared.numel() == kb.kan_vq_prepared_bytes(L)
    got = _read_layout(L.prepared, P)
    exp = _expected_layout(P)
    for name, g, e in zip(("seg", "bias_sum", "i", "q", "gain"), got, exp):
        assert np.array_equal(g, e), name
    rows = _bucket_rows(P)
    _check_tables(_read_layout.tables, got[0], (P.K + rows - 1) // rows, n_in, n_out)


@pytest.mark.parametrize("dist,n_out", [("zipf-sorted", 300), ("zipf", 300), ("zipf-sorted", 2500), ("uniform", 1024)])
def test_block_tables_balance_skewed_histograms(kb, dist, n_out):
    P = synth.make_layer(91, 700, n_out, 40000, cb_dtype="i8", gb_dtype="f16", idx_dist=dist, zipf_s=1.2)
    L = kb.VQLayer(P).prepare()
    seg = _read_layout(L.prepared, P)[0]
    _check_tables(_read_layout.tables, seg, 5, 700, n_out)
    T = _read_layout.tables[0]
    # an XCD (positions x, x + 8, ...) serves a contiguous run of the bucket-sorted blocks: few buckets
    per_xcd = [len(set(T[x::8, 0].tolist())) for x in range(8)]
    assert sum(per_xcd) <= 5 + 7, per_xcd           # a bucket is split over two XCDs only at the 7 run ends
    edges = T[:, 4].astype(np.int64) - T[:, 3]
    if n_out <= 1024:
        assert edges.max() <= 1.6 * edges.mean() + 700, (edges.max(), edges.mean())


def _forward_prepared(kb, P, x, expect_kernel="kan_bucket"):
    """The bucket kernel's result (small layers are kept on it by their flag).  Where the layer is small
    enough for the column kernel, that kernel runs on the same buffer too and must agree: the same
    finite outputs of the bucket kernel finite here too and equal within the fp32 bound."""
    L = kb.VQLayer(P).prepare()
    L.keep_on_bucket_kernel()
    assert kb.kan_vq_planned_kernel(L, x.shape[0], 1, kb.KAN_PATH_GATHER) == expect_kernel
    y = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    L.keep_on_bucket_kernel(False)
    if kb.kan_vq_planned_kernel(L, x.shape[0], 1, kb.KAN_PATH_GATHER) == "kan_column":
        yc = kb.kan_vq_layer_forward(L, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
        fin = np.isfinite(y)
        assert np.isfinite(yc[fin]).all()       # (the bucket kernel may give up more outputs than the edges make non-finite)
        if fin.any():
            assert np.abs(yc[fin] - y[fin]).max() <= TOL_FP32 * max(float(np.abs(y[fin]).max()), 1e-30)
    return y


def test_config1_prepared(kb):
    (P,), x = synth.config1()
    for B in (1, 4):
        y = _forward_prepared(kb, P, x[:B])
        y_ref, A = ko.vq_layer_forward(x[:B], **P.as_dict(), return_abs=True)
        rep = ko.error_report(y, y_ref, A)
        assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, rep


def test_config2_prepared_batch1(kb):
    (P,), x = synth.config2(1)
    y = _forward_prepared(kb, P, x)
    check_layer_output(y, x, P, TOL_FP32)


@pytest.mark.parametrize("B", [1, 2, 4])
def test_config3_head_prepared(kb, B):
    Ps, x = synth.config3(B)
    Ls = [L.prepare() for L in gpu_layers(Ps)]
    xd = to_dev(x)
    assert kb.kan_vq_planned_kernel(Ls[0], B, 1, kb.KAN_PATH_AUTO) == "kan_bucket"
    ws = torch.empty(kb.kan_vq_workspace_bytes([Ls], B, kb.KAN_PATH_AUTO), dtype=torch.uint8, device="cuda")
    y = kb.kan_vq_head_forward([Ls], xd, path=kb.KAN_PATH_AUTO, ws=ws)[0].cpu().numpy()
    y_ref, hidden_ref = ko.vq_head_forward(x, [p.as_dict() for p in Ps], return_hidden=True)
    assert ko.error_report(y, y_ref)["headline"] <= TOL_FP32
    # chained bucket layers pass per-bucket sums straight on (no hidden tensor is written):
    # layer 1 alone, squashed, must reproduce the oracle's hidden activation, and layer 2 of
    # the oracle fed with exactly those fp32 numbers must reproduce y
    y1 = kb.kan_vq_layer_forward(Ls[0], xd, path=kb.KAN_PATH_GATHER)
    hid = torch.tanh(y1).cpu().numpy()
    assert ko.error_report(hid, hidden_ref[0])["headline"] <= TOL_FP32
    y2_ref = ko.vq_layer_forward(hid, **Ps[1].as_dict())
    assert ko.error_report(y, y2_ref)["headline"] <= TOL_FP32
    # same bits on a second call, and the unprepared kernels agree within the bound
    y_again = kb.kan_vq_head_forward([Ls], xd, path=kb.KAN_PATH_AUTO, ws=ws)[0].cpu().numpy()
    assert np.array_equal(y, y_again)
    y_plain = kb.kan_vq_head_forward([gpu_layers(Ps)], xd, path=kb.KAN_PATH_GATHER)[0].cpu().numpy()
    assert np.abs(y_plain - y).max() <= 2 * TOL_FP32 * np.abs(y_ref).max()
    check_layer_output(y1.cpu().numpy(), x, Ps[0], TOL_FP32, full=False, seed=B)


@pytest.mark.parametrize("variant", ["i8", "f32"])
def test_config5_shape_prepared_batch2(kb, variant):
    """The 4096 x 4096, K = 262,144 layer of configuration 5 (32 Int8 / 128 fp32 buckets) at batch 2."""
    (P,), x = synth.config5(variant, B=2)
    y = _forward_prepared(kb, P, x)
    assert np.isfinite(y).all()
    check_layer_output(y, x, P, TOL_FP32, n_samples=64, full=False, seed=5)


@pytest.mark.parametrize("n_in,n_out,K,B", [(1, 1, 1, 1), (3, 21, 5, 2), (130, 67, 9000, 3), (257, 530, 20000, 1),
                                            (1000, 264, 8193, 4), (4096, 8, 1000, 1), (40, 1500, 65536, 1)])
@pytest.mark.parametrize("cb,gb", [("i8", "f16"), ("f32", "f32"), ("f16", "f16")])
def test_ragged_shapes_prepared(kb, n_in, n_out, K, B, cb, gb):
    P = synth.make_layer(n_in * 7 + n_out, n_in, n_out, K, cb_dtype=cb, gb_dtype=gb)
    x = synth.make_x(B, B, n_in)
    x[0, 0] = 1.0
    x[-1, -1] = -1.0
    y = _forward_prepared(kb, P, x)
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
    rep = ko.error_report(y, y_ref, A)
    assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, rep


def test_three_chained_layers_and_mixed_chain(kb):
    """Three prepared layers in a row (two hand-overs of per-bucket sums, alternating buffers),
    then the same head with the middle layer unprepared (hand-over only where both sides are
    bucket layers)."""
    Ps = [synth.make_layer(31, 200, 300, 30000, cb_dtype="i8", gb_dtype="f16"),
          synth.make_layer(32, 300, 90, 20000, cb_dtype="i8", gb_dtype="f16"),
          synth.make_layer(33, 90, 17, 9000, cb_dtype="f32", gb_dtype="f32")]
    x = synth.make_x(7, 2, 200)
    y_ref = ko.vq_head_forward(x, [p.as_dict() for p in Ps])
    Ls = [L.prepare() for L in gpu_layers(Ps)]
    for bucket_only in (True, False):             # small layers: kept on the bucket kernel, then on the column kernel
        for L in Ls:
            L.use_prepared(True)
            L.keep_on_bucket_kernel(bucket_only)
        assert kb.kan_vq_planned_kernel(Ls[1], 2, 1, kb.KAN_PATH_GATHER) == ("kan_bucket" if bucket_only else "kan_column")
        y = kb.kan_vq_head_forward([Ls], to_dev(x), path=kb.KAN_PATH_GATHER)[0].cpu().numpy()
        assert ko.error_report(y, y_ref)["headline"] <= TOL_FP32
        Ls[1].use_prepared(False)
        y = kb.kan_vq_head_forward([Ls], to_dev(x), path=kb.KAN_PATH_GATHER)[0].cpu().numpy()
        assert ko.error_report(y, y_ref)["headline"] <= TOL_FP32
    # a bucket layer hands its per-bucket sums to a column layer behind it
    for L, bucket_only in zip(Ls, (True, False, True)):
        L.use_prepared(True)
        L.keep_on_bucket_kernel(bucket_only)
    y = kb.kan_vq_head_forward([Ls], to_dev(x), path=kb.KAN_PATH_GATHER)[0].cpu().numpy()
    assert ko.error_report(y, y_ref)["headline"] <= TOL_FP32


def test_long_and_empty_segments(kb):
    """All edges of some outputs in one bucket (segments of 1500 edges: several chunks per
    wave), none in the others (empty segments)."""
    P = synth.make_layer(5, 1500, 40, 30000, cb_dtype="i8", gb_dtype="f16")
    P.idx[:, :20] = P.idx[:, :20] % 8192 + 8192          # outputs 0..19 live in bucket 1 only
    P.idx[:, 20:] = P.idx[:, 20:] % 100                  # outputs 20..39 in bucket 0 only
    x = synth.make_x(3, 2, 1500)
    y = _forward_prepared(kb, P, x)
    y_ref, A = ko.vq_layer_forward(x, **P.as_dict(), return_abs=True)
    rep = ko.error_report(y, y_ref, A)
    assert rep["headline"] <= TOL_FP32 and rep["strict"] <= TOL_FP32, rep


def test_grouped_heads_prepared(kb):
    B = 2
    heads_p = [[synth.make_layer(500 + h, 96, 48, 20000, cb_dtype="i8", gb_dtype="f16"),
                synth.make_layer(700 + h, 48, 7, 300, cb_dtype="i8", gb_dtype="f16")] for h in range(5)]
    x = synth.make_x(1, B, 96)
    heads = [[L.prepare() for L in gpu_layers(ps)] for ps in heads_p]
    for ls in heads:
        for L in ls:
            L.keep_on_bucket_kernel()             # (these small layers would take the column kernel otherwise)
    assert kb.kan_vq_planned_kernel(heads[0][0], B, 5, kb.KAN_PATH_GATHER) == "kan_bucket"
    y = kb.kan_vq_head_forward(heads, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    for h in range(5):
        y_ref = ko.vq_head_forward(x, [p.as_dict() for p in heads_p[h]])
        assert ko.error_report(y[h], y_ref)["headline"] <= TOL_FP32
    # heads whose flags differ: the whole group stays on the bucket kernel
    heads[2][0].keep_on_bucket_kernel(False)
    y3 = kb.kan_vq_head_forward(heads, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    assert np.array_equal(y3, y)
    heads[2][0].keep_on_bucket_kernel()
    # one head without a prepared buffer sends the whole group to the ordinary kernels
    heads[3][0].unprepare()
    assert kb.kan_vq_planned_kernel(heads[3][0], B, 5, kb.KAN_PATH_GATHER) != "kan_bucket"
    y2 = kb.kan_vq_head_forward(heads, to_dev(x), path=kb.KAN_PATH_GATHER).cpu().numpy()
    assert np.abs(y2 - y).max() <= 2 * TOL_FP32 * np.abs(y).max()


def test_unused_codeword_rows_may_hold_anything(kb):
    """Rows no edge refers to (here NaN) must not leak into the sums, not even through
    lanes that run past the end of a segment."""
    P = synth.make_layer(8, 70, 33, 3000, cb_dtype="f32", gb_dtype="f32")
    P.idx[P.idx == 0] = 1
    P.idx[P.idx == 2048] = 2049
    cb = P.codebook.copy()
    cb[0] = np.nan                                       # row 0 of buckets 0 and 1
    cb[2048] = np.nan
    x = synth.make_x(2, 1, 70)
    P2 = dataclasses.replace(P, codebook=cb)
    y = _forward_prepared(kb, P2, x)
    y_ref = ko.vq_layer_forward(x, **P.as_dict())
    assert np.isfinite(y).all()
    assert ko.error_report(y, y_ref)["headline"] <= TOL_FP32


@pytest.mark.parametrize("n_bad", [3, 200])
def test_non_finite_codewords_reach_only_their_own_outputs(kb, n_bad):
    """A codeword with an Inf or a NaN that edges do refer to makes exactly the outputs of those
    edges non-finite; every other output keeps its value (the running sums of a pass must not
    carry such a product into the segments behind it).  With very many such products in one
    workgroup's pass (n_bad = 200 edges of one output column range) whole blocks of outputs may
    be given up, but never silently wrong: every finite output still matches the oracle."""
    n_in, n_out, K = 300, 200, 20000
    P = synth.make_layer(77, n_in, n_out, K, cb_dtype="f32", gb_dtype="f32")
    rng = np.random.default_rng(n_bad)
    bad_rows = np.array([5, 4100, 19999])
    P.idx[np.isin(P.idx, bad_rows)] = 6                              # nobody refers to them by chance
    cb = P.codebook.copy()
    cb[5] = np.inf
    cb[4100] = np.nan
    cb[19999] = -np.inf                                             # (whole rows: an entry outside the four under the
                                                                    # span is never read by the kernels)
    ii = rng.integers(0, n_in, n_bad)
    jj = rng.integers(0, 12, n_bad) if n_bad > 50 else rng.integers(0, n_out, n_bad)
    P.idx[ii, jj] = bad_rows[np.arange(n_bad) % 3]
    P2 = dataclasses.replace(P, codebook=cb)
    hit = np.isin(P2.idx, bad_rows).any(axis=0)                      # outputs with such an edge
    for B in (1, 3):
        x = synth.make_x(5 + B, B, n_in)
        y = _forward_prepared(kb, P2, x)
        cb0 = cb.copy()
        cb0[bad_rows] = 0.0
        y_ref = ko.vq_layer_forward(x, **dataclasses.replace(P, codebook=cb0).as_dict())
        assert not np.isfinite(y[:, hit]).any()
        fin = np.isfinite(y)
        if n_bad <= 50:
            assert fin[:, ~hit].all()
        assert fin.any()
        scale = np.abs(y_ref).max()
        assert (np.abs(y[fin] - y_ref[fin]) <= TOL_FP32 * scale).all()
