"""Pins for the CPU oracle (no GPU).

Each oracle function is tied to something other than itself: hand-worked
examples (tests/golden/hand_examples.json), numpy library routines (integer
matmul, stable argsort, bincount, base_repr), closed forms, and exhaustive
enumeration of every small matrix.  The vectors used in exact checks are
distinct powers of two, so any column sent to a wrong group or any group sent
to a wrong output row changes the result.
"""
import itertools
import json
import os

import numpy as np
import pytest

import oracle
import rsr_inputs as gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_examples.json")
KINDS = {"binary": oracle.BINARY, "ternary_2pass": oracle.TERNARY_2PASS,
         "ternary_fused": oracle.TERNARY_FUSED}


def _golden():
    with open(GOLDEN) as f:
        return json.load(f)


# ------------------------------------------------------------ hand examples
def test_hand_example_binary():
    g = _golden()["binary_3x4_k2"]
    M = np.array(g["M"], dtype=np.int8)
    v = np.array(g["v"], dtype=np.float64)
    code = oracle.encode(M, g["k"], oracle.MODE_BINARY)
    assert code.tolist() == g["code"]
    art = oracle.preprocess(M, g["k"], oracle.BINARY)
    assert art.passes[0].pi.tolist() == g["pi"]
    assert art.passes[0].off.tolist() == g["off"]
    for b in range(2):
        u = oracle.segment_sums(art.passes[0].pi[b], art.passes[0].off[b], v)
        assert u.tolist() == g["u"][b]
    assert oracle.matvec(art, v).tolist() == g["out"]
    assert oracle.dense_matvec(M, v).tolist() == g["out"]


def test_hand_example_ternary_fused():
    g = _golden()["ternary_2x3_k2_fused"]
    M = np.array(g["M"], dtype=np.int8)
    v = np.array(g["v"], dtype=np.float64)
    assert oracle.encode(M, g["k"], oracle.MODE_FUSED3).tolist() == g["code"]
    art = oracle.preprocess(M, g["k"], oracle.TERNARY_FUSED)
    assert art.passes[0].pi.tolist() == g["pi"]
    assert art.passes[0].off.tolist() == g["off"]
    u = oracle.segment_sums(art.passes[0].pi[0], art.passes[0].off[0], v)
    assert u.tolist() == g["u"][0]
    assert oracle.matvec(art, v).tolist() == g["out"]
    assert oracle.dense_matvec(M, v).tolist() == g["out"]


def test_hand_example_ternary_twopass():
    g = _golden()["ternary_2x3_k2_twopass"]
    M = np.array(g["M"], dtype=np.int8)
    v = np.array(g["v"], dtype=np.float64)
    art = oracle.preprocess(M, g["k"], oracle.TERNARY_2PASS)
    assert [p.sign for p in art.passes] == [1.0, -1.0]
    for n in range(2):
        assert art.passes[n].pi.tolist() == g["pi"][n]
        assert art.passes[n].off.tolist() == g["off"][n]
    assert oracle.matvec(art, v).tolist() == g["out"]


def test_hand_example_pack2():
    g = _golden()["pack2_row"]
    M = np.array(g["M"], dtype=np.int8)
    assert oracle.pack2(M).tolist() == g["packed"]
    assert oracle.unpack2(np.array(g["packed"], dtype=np.uint8), M.shape[1]).tolist() == g["M"]


# ------------------------------------------------- dense vs library routine
@pytest.mark.parametrize("rows,cols,seed", [(1, 1, 1), (7, 13, 2), (64, 257, 3), (300, 129, 4)])
def test_dense_matches_numpy_matmul(rows, cols, seed):
    M = gen.ternary_matrix(rows, cols, 0.3, seed)
    v = gen.normal_f32(cols, seed + 100).astype(np.float64)
    ref = 0.75 * (M.astype(np.float64) @ v)
    got = oracle.dense_matvec(M, v, 0.75)
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-12)
    # integer-valued vector: exact
    vi = gen.integer_f32(cols, seed=seed).astype(np.float64)
    assert np.array_equal(oracle.dense_matvec(M, vi), (M.astype(np.int64) @ vi.astype(np.int64)))


# ------------------------------------------------- exhaustive enumeration
def _all_matrices(rows, cols, alphabet):
    n = rows * cols
    for cells in itertools.product(alphabet, repeat=n):
        yield np.array(cells, dtype=np.int8).reshape(rows, cols)


@pytest.mark.parametrize("rows,cols,ks", [
    (1, 4, (1, 2)), (2, 3, (1, 2, 3)), (3, 3, (1, 2, 3, 4)), (4, 3, (1, 2, 3, 4)),
    (3, 4, (1, 2, 3)), (5, 2, (2, 3, 4)), (4, 4, (3,)),
])
def test_exhaustive_binary_rsr_equals_definition(rows, cols, ks):
    v = (2.0 ** np.arange(cols)).astype(np.float64)
    vi = v.astype(np.int64)
    for M in _all_matrices(rows, cols, (0, 1)):
        want = M.astype(np.int64) @ vi          # library integer matmul
        for k in ks:
            art = oracle.preprocess(M, k, oracle.BINARY)
            got = oracle.matvec(art, v)
            assert np.array_equal(got, want), (M.tolist(), k)


@pytest.mark.parametrize("rows,cols,ks", [(2, 4, (1, 2, 3)), (3, 3, (1, 2, 3)), (4, 2, (3,))])
@pytest.mark.parametrize("kind", [oracle.TERNARY_2PASS, oracle.TERNARY_FUSED])
def test_exhaustive_ternary_rsr_equals_definition(rows, cols, ks, kind):
    v = (2.0 ** np.arange(cols)).astype(np.float64)
    vi = v.astype(np.int64)
    for M in _all_matrices(rows, cols, (-1, 0, 1)):
        want = M.astype(np.int64) @ vi
        for k in ks:
            got = oracle.matvec(oracle.preprocess(M, k, kind), v)
            assert np.array_equal(got, want), (M.tolist(), k, kind)


# ---------------------------------------- pi / offsets vs library routines
def _check_structure(p, cols, P):
    nb = p.pi.shape[0]
    assert p.off.shape == (nb, P + 1)
    for b in range(nb):
        pi, off = p.pi[b].astype(np.int64), p.off[b].astype(np.int64)
        assert np.array_equal(np.sort(pi), np.arange(cols))          # permutation
        assert off[0] == 0 and off[P] == cols and np.all(np.diff(off) >= 0)
        assert int(np.diff(off).sum()) == cols                        # sizes sum to n
        for c in np.nonzero(np.diff(off) > 1)[0]:
            seg = pi[off[c]:off[c + 1]]
            assert np.all(np.diff(seg) > 0)                           # ascending inside


@pytest.mark.parametrize("kind,rows,cols,k,seed", [
    (oracle.BINARY, 37, 200, 5, 11), (oracle.BINARY, 64, 1024, 8, 12),
    (oracle.TERNARY_2PASS, 50, 333, 6, 13), (oracle.TERNARY_FUSED, 50, 333, 4, 14),
    (oracle.TERNARY_FUSED, 22, 700, 6, 15), (oracle.BINARY, 9, 70, 10, 16),
])
def test_sort_matches_stable_argsort_and_bincount(kind, rows, cols, k, seed):
    M = gen.binary_matrix(rows, cols, 0.4, seed) if kind == oracle.BINARY \
        else gen.ternary_matrix(rows, cols, 0.4, seed)
    art = oracle.preprocess(M, k, kind)
    modes = {oracle.BINARY: [oracle.MODE_BINARY], oracle.TERNARY_2PASS: [oracle.MODE_POS, oracle.MODE_NEG],
             oracle.TERNARY_FUSED: [oracle.MODE_FUSED3]}[kind]
    for p, mode in zip(art.passes, modes):
        P = oracle.num_patterns(k, mode)
        _check_structure(p, cols, P)
        code = oracle.encode(M, k, mode).astype(np.int64)
        for b in range(code.shape[0]):
            assert np.array_equal(p.pi[b], np.argsort(code[b], kind="stable"))
            cnt = np.bincount(code[b], minlength=P)
            assert np.array_equal(p.off[b], np.concatenate([[0], np.cumsum(cnt)]))
            # codes along pi never decrease
            assert np.all(np.diff(code[b][p.pi[b].astype(np.int64)]) >= 0)


def test_encode_single_entry_closed_form():
    # One non-zero entry at (i, j): only block i//k, column j has a non-zero
    # code, and it is base^(i mod k) (x2 for a -1 in the fused code).
    rows, cols, k = 11, 6, 4
    for i in range(rows):
        for j in range(cols):
            M = np.zeros((rows, cols), dtype=np.int8)
            M[i, j] = 1
            cb = oracle.encode(M, k, oracle.MODE_BINARY)
            want = np.zeros_like(cb)
            want[i // k, j] = 2 ** (i % k)
            assert np.array_equal(cb, want)
            M[i, j] = -1
            cf = oracle.encode(M, k, oracle.MODE_FUSED3)
            want3 = np.zeros_like(cf)
            want3[i // k, j] = 2 * 3 ** (i % k)
            assert np.array_equal(cf, want3)
            assert np.array_equal(oracle.encode(M, k, oracle.MODE_NEG), want)
            assert not oracle.encode(M, k, oracle.MODE_POS).any()


def test_encode_rejects_foreign_entries():
    M = np.array([[0, 2], [1, 0]], dtype=np.int8)
    with pytest.raises(ValueError):
        oracle.encode(M, 2, oracle.MODE_BINARY)
    with pytest.raises(ValueError):
        oracle.encode(M, 2, oracle.MODE_FUSED3)
    with pytest.raises(ValueError):
        oracle.encode(np.array([[-1]], dtype=np.int8), 1, oracle.MODE_BINARY)


# -------------------------------------------------------------- closed forms
@pytest.mark.parametrize("kind", [oracle.BINARY, oracle.TERNARY_2PASS, oracle.TERNARY_FUSED])
def test_zero_matrix(kind):
    rows, cols, k = 10, 17, 4
    M = np.zeros((rows, cols), dtype=np.int8)
    v = gen.normal_f32(cols).astype(np.float64)
    art = oracle.preprocess(M, k, kind)
    assert not oracle.matvec(art, v).any()
    for p in art.passes:
        assert np.array_equal(p.pi, np.tile(np.arange(cols, dtype=np.uint32), (3, 1)))
        assert np.all(p.off[:, 0] == 0) and np.all(p.off[:, 1:] == cols)


def test_all_ones_binary():
    rows, cols, k = 8, 33, 4
    M = np.ones((rows, cols), dtype=np.int8)
    v = gen.integer_f32(cols).astype(np.float64)
    art = oracle.preprocess(M, k, oracle.BINARY)
    assert np.array_equal(oracle.matvec(art, v), np.full(rows, v.sum()))
    P = 2 ** k
    assert np.all(art.passes[0].off[:, :P] == 0) and np.all(art.passes[0].off[:, P] == cols)


def test_one_entry_per_column_is_a_gather():
    rows, cols, k = 12, 12, 5
    perm = np.random.default_rng(5).permutation(cols)
    M = np.zeros((rows, cols), dtype=np.int8)
    M[np.arange(rows), perm] = 1
    v = gen.integer_f32(cols).astype(np.float64)
    assert np.array_equal(oracle.matvec(oracle.preprocess(M, k, oracle.BINARY), v), v[perm])


def test_negated_matrix_swaps_passes_and_negates():
    M = gen.ternary_matrix(23, 90, 0.3, 77)
    v = gen.integer_f32(90).astype(np.float64)
    a = oracle.preprocess(M, 5, oracle.TERNARY_2PASS)
    b = oracle.preprocess(-M, 5, oracle.TERNARY_2PASS)
    assert np.array_equal(a.passes[0].pi, b.passes[1].pi)
    assert np.array_equal(a.passes[1].off, b.passes[0].off)
    assert np.array_equal(oracle.matvec(a, v), -oracle.matvec(b, v))


@pytest.mark.parametrize("rows,cols,seed", [(40, 300, 1), (4096 // 16, 512, 2)])
def test_kinds_and_block_heights_agree_exactly(rows, cols, seed):
    M = gen.ternary_matrix(rows, cols, 0.35, seed)
    v = gen.integer_f32(cols, seed=seed).astype(np.float64)
    want = M.astype(np.int64) @ v.astype(np.int64)
    for k in (1, 2, 3, 4, 6, 7):
        for kind in (oracle.TERNARY_2PASS, oracle.TERNARY_FUSED):
            assert np.array_equal(oracle.matvec(oracle.preprocess(M, k, kind), v), want)
    Mb = (M == 1).astype(np.int8)
    wantb = Mb.astype(np.int64) @ v.astype(np.int64)
    for k in (1, 3, 8, 10, 12):
        assert np.array_equal(oracle.matvec(oracle.preprocess(Mb, k, oracle.BINARY), v), wantb)


def test_float_vector_close_to_definition_and_scale():
    M = gen.ternary_matrix(130, 777, 0.4, 9)
    v = gen.normal_f32(777).astype(np.float64)
    ref = 0.37 * (M.astype(np.float64) @ v)
    for kind in (oracle.TERNARY_2PASS, oracle.TERNARY_FUSED):
        got = oracle.matvec(oracle.preprocess(M, 6, kind), v, 0.37)
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-11)


# ------------------------------------------------------ expansion u * B_k
@pytest.mark.parametrize("k", range(1, 11))
def test_expand_unit_vectors_binary(k):
    P = 2 ** k
    for c in range(P):
        u = np.zeros(P)
        u[c] = 1.0
        bits = [int(ch) for ch in reversed(np.binary_repr(c, width=k))]   # library digits
        assert oracle.expand(u, k, oracle.MODE_BINARY).tolist() == bits


@pytest.mark.parametrize("k", range(1, 7))
def test_expand_unit_vectors_ternary(k):
    P = 3 ** k
    sign = {"0": 0.0, "1": 1.0, "2": -1.0}
    for c in range(P):
        u = np.zeros(P)
        u[c] = 1.0
        digits = np.base_repr(c, 3).rjust(k, "0")
        want = [sign[ch] for ch in reversed(digits)]
        assert oracle.expand(u, k, oracle.MODE_FUSED3).tolist() == want


@pytest.mark.parametrize("k,mode", [(7, "t"), (8, "t"), (9, "t"), (10, "t"), (12, "b"), (15, "b")])
def test_expand_unit_vectors_large_k_sampled(k, mode):
    """The block heights the GPU tests use beyond the exhaustive range: a seeded sample of unit
    vectors (with the first and the last code) against the library's digit strings."""
    base = 3 if mode == "t" else 2
    P = base ** k
    sign = {"0": 0.0, "1": 1.0, "2": -1.0}
    codes = set(np.random.default_rng(k).integers(0, P, size=300).tolist()) | {0, 1, P - 1, P // 2}
    for c in sorted(codes):
        u = np.zeros(P)
        u[c] = 1.0
        digits = np.base_repr(c, base).rjust(k, "0")
        want = [sign[ch] for ch in reversed(digits)]
        got = oracle.expand(u, k, oracle.MODE_FUSED3 if mode == "t" else oracle.MODE_BINARY)
        assert got.tolist() == want


# -------------------------------------------------------------- 2-bit packing
def test_pack2_roundtrip_all_bytes():
    for byte in range(256):
        pairs = [(byte >> (2 * s)) & 3 for s in range(4)]
        packed = np.array([[byte]], dtype=np.uint8)
        if 2 in pairs:
            with pytest.raises(ValueError):
                oracle.unpack2(packed, 4)
            continue
        M = oracle.unpack2(packed, 4)
        assert M.tolist() == [[{0: 0, 1: 1, 3: -1}[p] for p in pairs]]
        assert oracle.pack2(M).tolist() == [[byte]]


def test_pack2_ragged_row():
    M = gen.ternary_matrix(5, 13, 0.3, 3)
    packed = oracle.pack2(M)
    assert packed.shape == (5, 4)
    assert np.array_equal(oracle.unpack2(packed, 13), M)
    assert np.all((packed[:, 3] >> 2) == 0)          # padding entries are zero


# --------------------------------------------------------------- generators
def test_to_bf16_is_round_to_nearest_even():
    import torch
    x = np.concatenate([gen.normal_f32(4096, 5), np.array([1.00390625, 1.01171875, 0.0, -0.0, 3.0e38], np.float32)])
    bits, vals = gen.to_bf16(x)
    t = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(t.view(torch.int16).numpy().view(np.uint16), bits)
    assert np.array_equal(t.to(torch.float32).numpy(), vals)
