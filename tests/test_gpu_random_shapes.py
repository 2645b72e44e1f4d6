"""Seeded random shapes through the C ABI: whatever block height, kind, column count, entry
density and batch the draw gives, an integer-valued vector must come out exact (the oracle's
dense definition in float64 is the reference).  The draw is biased towards the borders between
the launch shapes of the multiply kernels (256 columns, short and long streams, pattern spaces
larger than the column count).  Needs an MI355X."""
import numpy as np
import pytest

import oracle
import rsr_inputs as gen

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
rsr = pytest.importorskip("paper_2603_27462_amd")
DEV = "cuda:0"


def _draw(rng):
    kind = int(rng.integers(0, 3))
    k = int(rng.integers(1, (10 if kind == rsr.RSR_TERNARY_FUSED else 15) + 1))
    cols = int(rng.choice([rng.integers(1, 300), rng.integers(250, 3000), rng.integers(3000, 20000),
                           rng.integers(20000, 32767)], p=[0.3, 0.4, 0.25, 0.05]))
    rows = int(rng.choice([rng.integers(1, 40), rng.integers(40, 600), rng.integers(600, 3000)],
                          p=[0.4, 0.4, 0.2]))
    rows = max(1, min(rows, 3_000_000 // cols))
    p_zero = float(rng.choice([0.02, 0.35, 0.5, 0.9, 0.99]))
    few_patterns = bool(rng.integers(0, 3) == 0)
    batch = int(rng.choice([1, 1, 3]))
    bf16 = bool(rng.integers(0, 2))
    return kind, k, rows, cols, p_zero, few_patterns, batch, bf16


@pytest.mark.parametrize("chunk", range(6))
def test_random_shapes_are_exact(chunk):
    rng = np.random.default_rng(gen.BASE_SEED + 7000 + chunk)
    for case in range(25):
        kind, k, rows, cols, p_zero, few, batch, bf16 = _draw(rng)
        seed = int(rng.integers(1 << 30))
        if kind == rsr.RSR_BINARY:
            M = gen.binary_matrix(rows, cols, 1.0 - p_zero, seed)
        else:
            M = gen.ternary_matrix(rows, cols, p_zero, seed)
        if few and cols > 8:      # few distinct columns: long groups, most patterns empty
            M = np.ascontiguousarray(M[:, :7][:, np.random.default_rng(seed).integers(0, 7, cols)])
        what = "chunk %d case %d: kind %d k %d %dx%d p0 %.2f few %d batch %d bf16 %d" % (
            chunk, case, kind, k, rows, cols, p_zero, few, batch, bf16)
        try:
            h = rsr.rsr_preprocess(torch.from_numpy(M).to(DEV), k, kind)
        except rsr.RsrError as e:
            assert e.code == 3, what          # only "outside the supported limits" may refuse
            continue
        vi = np.stack([gen.integer_f32(cols, seed=seed % 1000 + i) for i in range(batch)])
        v = torch.from_numpy(vi).to(DEV)
        if bf16:
            v = v.to(torch.bfloat16)
        got = rsr.rsr_matvec_ex(h, v if batch > 1 else v[0], scale=2.0).cpu().numpy().reshape(batch, rows)
        for i in range(batch):
            want = oracle.dense_matvec(M, vi[i].astype(np.float64), 2.0)
            assert np.array_equal(got[i].astype(np.float64), want), what + " vector %d" % i
        rsr.rsr_destroy(h)
