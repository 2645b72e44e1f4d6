"""Parity of the HIP path (through the C ABI) with the CPU oracle.  Needs an MI355X.

Bars: pi, group boundaries, packed bytes and integer-valued v: bit-exact.
float32 / bf16 v: |gpu - oracle| <= 1e-4 * |scale| * sum_j |v_j| per output
(the oracle accumulates the same, already rounded, inputs in float64).
"""
import numpy as np
import pytest

import oracle
import rsr_inputs as gen

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
rsr = pytest.importorskip("paper_2603_27462_amd")

KINDS = {rsr.RSR_BINARY: oracle.BINARY, rsr.RSR_TERNARY_2PASS: oracle.TERNARY_2PASS,
         rsr.RSR_TERNARY_FUSED: oracle.TERNARY_FUSED}
DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _bf16_dev(bits):
    return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)


def _matrix(kind, rows, cols, seed, p=0.35):
    if kind == rsr.RSR_BINARY:
        return gen.binary_matrix(rows, cols, p, seed)
    return gen.ternary_matrix(rows, cols, p, seed)


def _check_artifacts(h, art):
    assert rsr.rsr_num_passes(h) == len(art.passes)
    for n, p in enumerate(art.passes):
        assert np.array_equal(rsr.rsr_get_perm(h, n), p.pi), "pi differs (pass %d)" % n
        assert np.array_equal(rsr.rsr_get_offsets(h, n), p.off), "offsets differ (pass %d)" % n


def _tol(v, scale=1.0):
    return 1e-4 * abs(scale) * float(np.abs(v.astype(np.float64)).sum())


def _check_matvec(h, M, cols, seed, scale=0.5):
    # integer-valued v: exact
    vi = gen.integer_f32(cols, seed=seed)
    want = oracle.dense_matvec(M, vi.astype(np.float64))
    got = rsr.rsr_matvec(h, _dev(vi)).cpu().numpy()
    assert np.array_equal(got.astype(np.float64), want), "integer v not exact"
    # float32 v, scaled
    vf = gen.normal_f32(cols, seed=seed + 1)
    want = oracle.dense_matvec(M, vf.astype(np.float64), scale)
    got = rsr.rsr_matvec_ex(h, _dev(vf), scale=scale).cpu().numpy()
    assert np.max(np.abs(got - want)) <= _tol(vf, scale)
    # bf16 v
    bits, vals = gen.normal_bf16(cols, seed=seed + 2)
    want = oracle.dense_matvec(M, vals.astype(np.float64), scale)
    got = rsr.rsr_matvec_ex(h, _bf16_dev(bits), scale=scale).cpu().numpy()
    assert np.max(np.abs(got - want)) <= _tol(vals, scale)
    # determinism: the kernel uses no atomics
    again = rsr.rsr_matvec_ex(h, _bf16_dev(bits), scale=scale).cpu().numpy()
    assert np.array_equal(got, again)


# shapes span several waves/iterations, ragged column counts and ragged last blocks
CASES = [
    # kind, rows, cols, k
    (rsr.RSR_BINARY, 1024, 1024, 8),          # config 1
    (rsr.RSR_BINARY, 37, 200, 5),
    (rsr.RSR_BINARY, 100, 4099, 10),
    (rsr.RSR_BINARY, 9, 77, 1),
    (rsr.RSR_BINARY, 33, 9000, 3),            # long groups, several waves
    (rsr.RSR_BINARY, 64, 513, 12),
    (rsr.RSR_TERNARY_2PASS, 130, 4096, 4),
    (rsr.RSR_TERNARY_2PASS, 130, 4096, 6),
    (rsr.RSR_TERNARY_2PASS, 130, 4096, 8),
    (rsr.RSR_TERNARY_2PASS, 130, 4096, 10),
    (rsr.RSR_TERNARY_2PASS, 50, 333, 7),
    (rsr.RSR_TERNARY_FUSED, 130, 4096, 4),
    (rsr.RSR_TERNARY_FUSED, 130, 4096, 6),
    (rsr.RSR_TERNARY_FUSED, 130, 4096, 8),
    (rsr.RSR_TERNARY_FUSED, 50, 333, 5),
    (rsr.RSR_TERNARY_FUSED, 22, 14336, 8),    # metric column count
    (rsr.RSR_TERNARY_FUSED, 20, 2560, 9),
    (rsr.RSR_TERNARY_FUSED, 7, 31, 2),
    (rsr.RSR_TERNARY_FUSED, 5, 20001, 7),     # more than eight waves per block
    # pattern spaces far larger than the column count: E indexed by group rank
    (rsr.RSR_TERNARY_FUSED, 130, 4096, 10),
    (rsr.RSR_TERNARY_FUSED, 33, 700, 10),
    (rsr.RSR_BINARY, 40, 4096, 15),
    (rsr.RSR_BINARY, 30, 3000, 13),
    (rsr.RSR_BINARY, 30, 3000, 14),
    (rsr.RSR_TERNARY_2PASS, 20, 2048, 15),
    (rsr.RSR_TERNARY_2PASS, 45, 30000, 11),
    # at most 256 columns: one wave per block, 8-bit entries
    (rsr.RSR_BINARY, 300, 256, 8),
    (rsr.RSR_BINARY, 1000, 255, 4),
    (rsr.RSR_BINARY, 40, 100, 15),
    (rsr.RSR_BINARY, 50, 1, 3),
    (rsr.RSR_TERNARY_FUSED, 100, 256, 5),
    (rsr.RSR_TERNARY_FUSED, 33, 255, 8),
    (rsr.RSR_TERNARY_FUSED, 45, 100, 10),
    (rsr.RSR_TERNARY_2PASS, 64, 129, 8),
]


@pytest.mark.parametrize("kind,rows,cols,k", CASES)
def test_rsr_parity(kind, rows, cols, k):
    seed = 1000 + rows + cols + k
    M = _matrix(kind, rows, cols, seed)
    h = rsr.rsr_preprocess(_dev(M), k, kind)
    art = oracle.preprocess(M, k, KINDS[kind])
    _check_artifacts(h, art)
    _check_matvec(h, M, cols, seed)
    rsr.rsr_destroy(h)


@pytest.mark.parametrize("kind", [rsr.RSR_BINARY, rsr.RSR_TERNARY_2PASS, rsr.RSR_TERNARY_FUSED])
def test_degenerate_matrices(kind):
    rows, cols, k = 21, 1500, 4
    for name, M in [("zeros", np.zeros((rows, cols), np.int8)),
                    ("ones", np.ones((rows, cols), np.int8)),
                    ("minus_ones", -np.ones((rows, cols), np.int8)),
                    ("one_column", np.zeros((rows, 1), np.int8) + 1),
                    ("one_row", _matrix(kind, 1, cols, 3))]:
        if kind == rsr.RSR_BINARY and name == "minus_ones":
            continue
        h = rsr.rsr_preprocess(_dev(M), k, kind)
        _check_artifacts(h, oracle.preprocess(M, k, KINDS[kind]))
        _check_matvec(h, M, M.shape[1], 7)


def test_all_columns_equal_wide():
    """One group holding every column, at the widest strips: 30000 equal columns."""
    M = np.ones((26, 30000), np.int8)
    M[::3] = 0
    for kind, k in ((rsr.RSR_BINARY, 13), (rsr.RSR_TERNARY_FUSED, 8)):
        h = rsr.rsr_preprocess(_dev(M), k, kind)
        _check_artifacts(h, oracle.preprocess(M, k, KINDS[kind]))
        _check_matvec(h, M, 30000, 19)
        rsr.rsr_destroy(h)


def test_stream_longer_than_one_round_of_slabs():
    """A code-indexed stream of more than 64 slabs per block: eight waves, each working
    through several groups of four slabs, the first group short at its front.  30000 columns
    drawn from 1000 patterns per block of 12 rows: 30000 entries + about 3100 placeholders."""
    rows, cols, k = 30, 30000, 12
    M = gen.dictionary_binary_matrix(rows, cols, k, 1000, 17)
    h = rsr.rsr_preprocess(_dev(M), k, rsr.RSR_BINARY)
    assert rsr.rsr_algorithmic_bytes(h, rsr.RSR_F32, 1) > 3 * 65 * 1024   # > 64 slabs per block
    _check_artifacts(h, oracle.preprocess(M, k, oracle.BINARY))
    _check_matvec(h, M, cols, 23)
    rsr.rsr_destroy(h)


def test_block_height_exceeds_rows():
    M = _matrix(rsr.RSR_TERNARY_FUSED, 3, 700, 9)
    h = rsr.rsr_preprocess(_dev(M), 8, rsr.RSR_TERNARY_FUSED)
    _check_artifacts(h, oracle.preprocess(M, 8, oracle.TERNARY_FUSED))
    _check_matvec(h, M, 700, 11)


def test_widest_supported_vector():
    cols = 32766
    M = _matrix(rsr.RSR_TERNARY_2PASS, 12, cols, 21)
    h = rsr.rsr_preprocess(_dev(M), 6, rsr.RSR_TERNARY_2PASS)
    _check_artifacts(h, oracle.preprocess(M, 6, oracle.TERNARY_2PASS))
    _check_matvec(h, M, cols, 13)


def test_batch_and_strides():
    rows, cols, k = 96, 4096, 8
    M = _matrix(rsr.RSR_TERNARY_FUSED, rows, cols, 31)
    h = rsr.rsr_preprocess(_dev(M), k, rsr.RSR_TERNARY_FUSED)
    vs = np.stack([gen.to_bf16(gen.normal_f32(cols, seed=50 + i))[0] for i in range(4)])
    vals = (vs.astype(np.uint32) << 16).view(np.float32)
    vbuf = torch.zeros((4, cols + 64), dtype=torch.bfloat16, device=DEV)     # ldv > cols
    vbuf[:, :cols] = _bf16_dev(vs)
    out = torch.full((4, rows + 8), 777.0, dtype=torch.float32, device=DEV)  # ldo > rows
    rsr.rsr_matvec_ex(h, vbuf[:, :cols], scale=2.0, out=out[:, :rows])
    got = out.cpu().numpy()
    assert np.all(got[:, rows:] == 777.0)                                     # nothing past rows
    for i in range(4):
        want = oracle.dense_matvec(M, vals[i].astype(np.float64), 2.0)
        assert np.max(np.abs(got[i, :rows] - want)) <= _tol(vals[i], 2.0)


@pytest.mark.parametrize("kind,bf16,pad,batch", [
    (rsr.RSR_TERNARY_FUSED, True, 0, 5), (rsr.RSR_TERNARY_FUSED, True, 3, 7),
    (rsr.RSR_BINARY, False, 0, 6), (rsr.RSR_BINARY, False, 1, 5),
    (rsr.RSR_TERNARY_2PASS, True, 8, 5), (rsr.RSR_DENSE_TERNARY_P2, True, 0, 5),
    (rsr.RSR_DENSE_TERNARY_P2, True, 5, 19), (rsr.RSR_DENSE_TERNARY_P2, False, 2, 6)])
def test_batch_many_blocks(kind, bf16, pad, batch):
    """Many blocks and several vectors in one call; aligned and unaligned vector strides;
    integer-valued vectors, so every output is exact.  264 columns take the general kernel,
    200 columns the one for narrow matrices."""
    for cols in (264, 200):
        _batch_many_blocks(kind, bf16, pad, batch, cols)


def _batch_many_blocks(kind, bf16, pad, batch, cols):
    rows, k = 2100, 2
    M = _matrix(kind, rows, cols, 77)
    h = rsr.rsr_preprocess(_dev(M), k, kind)
    vi = np.stack([gen.integer_f32(cols, seed=900 + i) for i in range(batch)])
    vbuf = torch.zeros((batch, cols + pad), dtype=torch.bfloat16 if bf16 else torch.float32, device=DEV)
    vbuf[:, :cols] = _dev(vi).to(vbuf.dtype)
    out = torch.full((batch, rows + 3), -5.0, dtype=torch.float32, device=DEV)
    rsr.rsr_matvec_ex(h, vbuf[:, :cols], scale=3.0, out=out[:, :rows])
    got = out.cpu().numpy()
    assert np.all(got[:, rows:] == -5.0)
    for i in range(batch):
        want = oracle.dense_matvec(M, vi[i].astype(np.float64), 3.0)
        assert np.array_equal(got[i, :rows].astype(np.float64), want), "vector %d" % i


@pytest.mark.parametrize("kind,rows,cols,k,batch,bf16,pad", [
    (rsr.RSR_TERNARY_FUSED, 2600, 300, 10, 3, True, 0),     # E by rank
    (rsr.RSR_TERNARY_2PASS, 2600, 1500, 5, 4, False, 1),    # two passes per vector, unaligned vectors
    (rsr.RSR_BINARY, 1024, 1024, 8, 7, False, 0),           # 128 blocks, five of eight waves without a slab
    (rsr.RSR_BINARY, 3120, 30000, 12, 3, True, 0),          # several groups of slabs per wave
    (rsr.RSR_TERNARY_FUSED, 4096, 1000, 8, 4, True, 4),     # the common class count, short stream
    (rsr.RSR_BINARY, 3100, 2000, 2, 5, True, 0)])           # four waves per block
def test_batch_shapes(kind, rows, cols, k, batch, bf16, pad):
    """Batches over the launch shapes of the multiply kernel: integer-valued vectors, so
    every output of every vector is exact; rows past the matrix stay untouched."""
    if cols >= 30000:
        M = gen.dictionary_binary_matrix(rows, cols, k, 1000, 5)   # 30000 entries + 3100 placeholders
    else:
        M = _matrix(kind, rows, cols, 78)
    h = rsr.rsr_preprocess(_dev(M), k, kind)
    vi = np.stack([gen.integer_f32(cols, seed=300 + i) for i in range(batch)])
    vbuf = torch.zeros((batch, cols + pad), dtype=torch.bfloat16 if bf16 else torch.float32, device=DEV)
    vbuf[:, :cols] = _dev(vi).to(vbuf.dtype)
    out = torch.full((batch, rows + 5), -7.0, dtype=torch.float32, device=DEV)
    rsr.rsr_matvec_ex(h, vbuf[:, :cols], scale=-2.0, out=out[:, :rows])
    got = out.cpu().numpy()
    assert np.all(got[:, rows:] == -7.0)
    for i in range(batch):
        want = oracle.dense_matvec(M, vi[i].astype(np.float64), -2.0)
        assert np.array_equal(got[i, :rows].astype(np.float64), want), "vector %d" % i
    # and one vector alone gives the same bits as it did inside the batch
    alone = rsr.rsr_matvec_ex(h, vbuf[1, :cols], scale=-2.0).cpu().numpy()
    assert np.array_equal(alone, got[1, :rows])


@pytest.mark.parametrize("kind,k", [(rsr.RSR_TERNARY_FUSED, 6), (rsr.RSR_TERNARY_2PASS, 5),
                                    (rsr.RSR_BINARY, 8), (rsr.RSR_DENSE_TERNARY_P2, 0)])
def test_serialize_round_trip(kind, k):
    rows, cols = 203, 1500
    M = _matrix(kind, rows, cols, 55)
    h = rsr.rsr_preprocess(_dev(M), k, kind)
    blob = rsr.rsr_serialize(h)
    h2 = rsr.rsr_deserialize(blob.tobytes())
    assert (h2.rows, h2.cols, h2.k, h2.kind) == (rows, cols, k, kind)
    assert np.array_equal(rsr.rsr_serialize(h2), blob)
    if kind == rsr.RSR_DENSE_TERNARY_P2:
        assert np.array_equal(rsr.rsr_get_packed(h2), oracle.pack2(M))
    else:
        _check_artifacts(h2, oracle.preprocess(M, k, KINDS[kind]))
    v = _dev(gen.normal_f32(cols, seed=8))
    assert torch.equal(rsr.rsr_matvec(h, v), rsr.rsr_matvec(h2, v))      # same stream, same bits
    rsr.rsr_destroy(h)
    _check_matvec(h2, M, cols, 9)                                          # and it outlives h
    bad = blob.copy()
    bad[8] ^= 0xFF                                                         # kind field
    with pytest.raises(rsr.RsrError):
        rsr.rsr_deserialize(bad)
    with pytest.raises(rsr.RsrError):
        rsr.rsr_deserialize(blob[:-7])


@pytest.mark.parametrize("kind,k", [(rsr.RSR_TERNARY_FUSED, 5), (rsr.RSR_BINARY, 7),
                                    (rsr.RSR_DENSE_TERNARY_P2, 0)])
def test_transposed_handle(kind, k):
    # the row-vector product v^T M: the handle of M^T against the oracle on M^T
    rows, cols = 300, 130
    M = _matrix(kind, rows, cols, 66)
    h = rsr.rsr_preprocess_transposed(_dev(M), k, kind)
    assert (h.rows, h.cols) == (cols, rows)
    Mt = np.ascontiguousarray(M.T)
    if kind == rsr.RSR_DENSE_TERNARY_P2:
        assert np.array_equal(rsr.rsr_get_packed(h), oracle.pack2(Mt))
    else:
        _check_artifacts(h, oracle.preprocess(Mt, k, KINDS[kind]))
    _check_matvec(h, Mt, rows, 12)


@pytest.mark.parametrize("kind,k", [(rsr.RSR_TERNARY_FUSED, 6), (rsr.RSR_TERNARY_FUSED, 0),
                                    (rsr.RSR_TERNARY_2PASS, 5), (rsr.RSR_BINARY, 8),
                                    (rsr.RSR_TERNARY_FUSED, 10), (rsr.RSR_DENSE_TERNARY_P2, 0)])
def test_stacked_sibling_layers(kind, k):
    """Layers that share their input in one handle and one launch: per layer the artifacts are
    those of the layer alone, block for block, and the outputs (own scale, own vector) are the
    dense products; nothing is written behind a layer's rows."""
    cols, rows = 640, [96, 41, 33]
    Ms = [_matrix(kind, r, cols, 400 + r) for r in rows]
    h = rsr.rsr_preprocess_stacked([_dev(M) for M in Ms], k, kind)
    kk = h.k
    if kind != rsr.RSR_DENSE_TERNARY_P2:
        arts = [oracle.preprocess(M, kk, KINDS[kind]) for M in Ms]
        for ps in range(rsr.rsr_num_passes(h)):
            pi, off = rsr.rsr_get_perm(h, ps), rsr.rsr_get_offsets(h, ps)
            b0 = 0
            for art in arts:
                nb = art.passes[ps].pi.shape[0]
                assert np.array_equal(pi[b0:b0 + nb], art.passes[ps].pi)
                assert np.array_equal(off[b0:b0 + nb], art.passes[ps].off)
                b0 += nb
            assert b0 == pi.shape[0]
    scales = [0.5, 2.0, -1.25]
    vi = gen.integer_f32(cols, seed=77)
    outs = [torch.full((r + 5,), 9.0, dtype=torch.float32, device=DEV) for r in rows]
    rsr.rsr_matvec_stacked(h, _dev(vi), scales, [o[:r] for o, r in zip(outs, rows)])
    for M, sc, o, r in zip(Ms, scales, outs, rows):
        got = o.cpu().numpy()
        assert np.all(got[r:] == 9.0)
        assert np.array_equal(got[:r].astype(np.float64), oracle.dense_matvec(M, vi.astype(np.float64), sc))
    bits, vals = gen.normal_bf16(cols, seed=78)
    got = rsr.rsr_matvec_stacked(h, _bf16_dev(bits), scales)
    for M, sc, o in zip(Ms, scales, got):
        want = oracle.dense_matvec(M, vals.astype(np.float64), sc)
        assert np.max(np.abs(o.cpu().numpy() - want)) <= _tol(vals, sc)
    with pytest.raises(rsr.RsrError):
        rsr.rsr_matvec(h, _dev(vi))            # a stacked handle has no single output vector
    rsr.rsr_destroy(h)


def test_linear_module():
    from paper_2603_27462_amd.linear import RsrLinear
    rows, cols = 96, 640
    M = gen.ternary_matrix(rows, cols, 0.4, 91)
    layer = RsrLinear(_dev(M), scale=0.25)                     # k chosen by the library
    xi = np.stack([gen.integer_f32(cols, seed=700 + i) for i in range(6)]).reshape(2, 3, cols)
    y = layer(_dev(xi).to(torch.bfloat16)).cpu().numpy()
    assert y.shape == (2, 3, rows)
    for a in range(2):
        for b in range(3):
            want = oracle.dense_matvec(M, xi[a, b].astype(np.float64), 0.25)
            assert np.array_equal(y[a, b].astype(np.float64), want)
    y1 = layer(_dev(xi[0, 0])).cpu().numpy()                   # a single float32 vector
    assert np.array_equal(y1.astype(np.float64), oracle.dense_matvec(M, xi[0, 0].astype(np.float64), 0.25))


def test_second_stream():
    rows, cols = 64, 2048
    M = _matrix(rsr.RSR_BINARY, rows, cols, 41)
    h = rsr.rsr_preprocess(_dev(M), 8, rsr.RSR_BINARY)
    vi = gen.integer_f32(cols, seed=5)
    v = _dev(vi)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    out = rsr.rsr_matvec(h, v, stream=s)
    s.synchronize()
    assert np.array_equal(out.cpu().numpy().astype(np.float64),
                          oracle.dense_matvec(M, vi.astype(np.float64)))


# ------------------------------------------------------------ dense comparison kernel
@pytest.mark.parametrize("rows,cols", [(64, 1024), (37, 333), (130, 4096), (9, 2561), (22, 14336)])
def test_dense_packed_parity(rows, cols):
    M = gen.ternary_matrix(rows, cols, 0.35, rows + cols)
    h = rsr.rsr_preprocess(_dev(M), 0, rsr.RSR_DENSE_TERNARY_P2)
    assert np.array_equal(rsr.rsr_get_packed(h), oracle.pack2(M))
    _check_matvec(h, M, cols, rows)


# ------------------------------------------------------------------- error behaviour
@pytest.mark.parametrize("kind,rows,cols", [(rsr.RSR_TERNARY_FUSED, 320, 1024),
                                            (rsr.RSR_BINARY, 257, 700),
                                            (rsr.RSR_TERNARY_2PASS, 96, 2048)])
def test_library_chosen_block_height(kind, rows, cols):
    """k = 0: the library picks the height by timing; whatever it picks, the artifacts are
    the oracle's for that k and the product is the dense one."""
    M = _matrix(kind, rows, cols, 123)
    h = rsr.rsr_preprocess(_dev(M), 0, kind)
    k = rsr.rsr_block_height(h)
    assert k in ((4, 5, 6, 7, 8) if kind == rsr.RSR_TERNARY_FUSED else (4, 6, 8, 10, 12))
    assert h.k == k and rsr.rsr_num_blocks(h) == -(-rows // k)
    _check_artifacts(h, oracle.preprocess(M, k, KINDS[kind]))
    _check_matvec(h, M, cols, 17)


def test_errors():
    M = _dev(gen.ternary_matrix(16, 64, 0.3, 1))
    with pytest.raises(rsr.RsrError) as e:
        rsr.rsr_preprocess(M, 4, rsr.RSR_BINARY)          # -1 entries in a binary matrix
    assert e.value.code == 2
    with pytest.raises(rsr.RsrError) as e:
        rsr.rsr_preprocess(M, 11, rsr.RSR_TERNARY_FUSED)  # k beyond the fused limit
    assert e.value.code == 3
    with pytest.raises(rsr.RsrError) as e:
        rsr.rsr_preprocess(M, -2, rsr.RSR_TERNARY_2PASS)
    assert e.value.code == 1
    with pytest.raises(rsr.RsrError) as e:
        rsr.rsr_preprocess(M, 4, 9)
    assert e.value.code == 1
    bad = _dev(np.full((4, 8), 2, np.int8))
    with pytest.raises(rsr.RsrError) as e:
        rsr.rsr_preprocess(bad, 0, rsr.RSR_DENSE_TERNARY_P2)
    assert e.value.code == 2
    wide = torch.zeros((2, 32767), dtype=torch.int8, device=DEV)
    with pytest.raises(rsr.RsrError) as e:
        rsr.rsr_preprocess(wide, 4, rsr.RSR_BINARY)
    assert e.value.code == 3
    h = rsr.rsr_preprocess(M, 4, rsr.RSR_TERNARY_FUSED)
    with pytest.raises(rsr.RsrError):
        rsr.rsr_get_packed(h)
    with pytest.raises(rsr.RsrError):
        rsr.rsr_get_perm(h, 1)
    # the library keeps working after errors
    _check_matvec(h, M.cpu().numpy(), 64, 3)
