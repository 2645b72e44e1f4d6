"""rsr_preprocess_into (the entry point that allocates nothing) against rsr_preprocess.

Through the C ABI: a handle refreshed in place with a new matrix must hold exactly what a
fresh rsr_preprocess of that matrix holds (pi, group boundaries, packed bytes: bit-exact;
integer-valued v: bit-exact; bf16 v: the tolerance of the other parity tests), on two calls
in a row, the second on a smaller input, so that whatever the first call left in the shared
scratch array is seen not to matter.  Needs an MI355X.
"""
import numpy as np
import pytest

import rsr_inputs as gen

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
rsr = pytest.importorskip("paper_2603_27462_amd")
DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _matrix(kind, rows, cols, seed):
    if kind == rsr.RSR_BINARY:
        return gen.binary_matrix(rows, cols, 0.4, seed)
    return gen.ternary_matrix(rows, cols, 0.4, seed)


def _same_as_fresh(h, M, kind, k, seed):
    """h was refreshed with M: compare with the handle rsr_preprocess makes of M."""
    cols = M.shape[1]
    fresh = rsr.rsr_preprocess(_dev(M), k, kind)
    if kind == rsr.RSR_DENSE_TERNARY_P2:
        assert np.array_equal(rsr.rsr_get_packed(h), rsr.rsr_get_packed(fresh))
    else:
        for ps in range(rsr.rsr_num_passes(fresh)):
            assert np.array_equal(rsr.rsr_get_perm(h, ps), rsr.rsr_get_perm(fresh, ps))
            assert np.array_equal(rsr.rsr_get_offsets(h, ps), rsr.rsr_get_offsets(fresh, ps))
    vi = _dev(gen.integer_f32(cols, seed=seed))
    assert torch.equal(rsr.rsr_matvec(h, vi), rsr.rsr_matvec(fresh, vi)), "integer v not exact"
    bits, vals = gen.normal_bf16(cols, seed=seed + 1)
    vb = torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    a = rsr.rsr_matvec_ex(h, vb, scale=0.5).cpu().numpy()
    b = rsr.rsr_matvec_ex(fresh, vb, scale=0.5).cpu().numpy()
    tol = 1e-4 * 0.5 * float(np.abs(vals.astype(np.float64)).sum())
    assert np.max(np.abs(a - b)) <= tol
    rsr.rsr_destroy(fresh)


@pytest.mark.parametrize("kind,k", [(rsr.RSR_TERNARY_FUSED, 6), (rsr.RSR_TERNARY_2PASS, 7),
                                    (rsr.RSR_BINARY, 8), (rsr.RSR_DENSE_TERNARY_P2, 0)])
def test_two_refreshes_in_a_row_second_one_smaller(kind, k):
    big, small = (300, 2560), (50, 333)
    hb = rsr.rsr_preprocess(_dev(_matrix(kind, *big, 1)), k, kind)
    hs = rsr.rsr_preprocess(_dev(_matrix(kind, *small, 2)), k, kind)
    Mb, Ms = _matrix(kind, *big, 3), _matrix(kind, *small, 4)
    rsr.rsr_preprocess_into(hb, _dev(Mb))
    rsr.rsr_preprocess_into(hs, _dev(Ms))          # right behind it, on the same scratch
    _same_as_fresh(hs, Ms, kind, k, 10)
    _same_as_fresh(hb, Mb, kind, k, 20)
    rsr.rsr_destroy(hb)
    rsr.rsr_destroy(hs)


def test_refusals_leave_the_library_usable():
    kind, k = rsr.RSR_TERNARY_FUSED, 5
    M = _matrix(kind, 64, 700, 5)
    h = rsr.rsr_preprocess(_dev(M), k, kind)
    v = _dev(gen.integer_f32(700, seed=6))
    before = rsr.rsr_matvec(h, v).clone()
    with pytest.raises(TypeError):
        rsr.rsr_preprocess_into(h, _dev(_matrix(kind, 64, 701, 5)))      # another shape
    bad = M.copy()
    bad[3, 5] = 2
    with pytest.raises(rsr.RsrError) as e:
        rsr.rsr_preprocess_into(h, _dev(bad))                           # entry outside the alphabet
    assert e.value.code == 2
    with pytest.raises(rsr.RsrError) as e:
        rsr.rsr_matvec(h, v)                                            # half-written: refused
    assert e.value.code == 1
    rsr.rsr_preprocess_into(h, _dev(M))
    assert torch.equal(rsr.rsr_matvec(h, v), before)
    rsr.rsr_destroy(h)
    # temporaries beyond the fixed scratch array: refused before anything is written
    rows, cols = 30000, 2048
    big = gen.binary_matrix(rows, cols, 0.3, 7)
    hb = rsr.rsr_preprocess(_dev(big), 4, rsr.RSR_BINARY)
    vb = _dev(gen.integer_f32(cols, seed=8))
    before = rsr.rsr_matvec(hb, vb).clone()
    with pytest.raises(rsr.RsrError) as e:
        rsr.rsr_preprocess_into(hb, _dev(big))
    assert e.value.code == 7
    assert torch.equal(rsr.rsr_matvec(hb, vb), before)
    rsr.rsr_destroy(hb)
