"""Full-size parity on the benchmark workloads (needs an MI355X).

Same bars as test_gpu_parity.py, at the sizes and in the launch configuration
bench.py times (bf16 vector, batch 1, the handle's own choice of waves per
block).  The C oracle is fast enough to check every output and every entry of
pi / group boundaries, so nothing is sampled.
"""
import numpy as np
import pytest

import oracle
import rsr_inputs as gen

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
rsr = pytest.importorskip("paper_2603_27462_amd")
DEV = "cuda:0"
OK = {rsr.RSR_BINARY: oracle.BINARY, rsr.RSR_TERNARY_2PASS: oracle.TERNARY_2PASS,
      rsr.RSR_TERNARY_FUSED: oracle.TERNARY_FUSED}


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _bf16_dev(bits):
    return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)


def _artifacts_equal(h, M, k, kind):
    art = oracle.preprocess(M, k, OK[kind])
    for n, p in enumerate(art.passes):
        assert np.array_equal(rsr.rsr_get_perm(h, n), p.pi)
        assert np.array_equal(rsr.rsr_get_offsets(h, n), p.off)


def _bf16_matvec_ok(h, M, seed, scale=1.0, batch=1):
    cols = M.shape[1]
    bits = np.stack([gen.normal_bf16(cols, seed=seed + i)[0] for i in range(batch)])
    vals = (bits.astype(np.uint32) << 16).view(np.float32)
    vd = _bf16_dev(bits if batch > 1 else bits[0])
    got = rsr.rsr_matvec_ex(h, vd, scale=scale).cpu().numpy().reshape(batch, -1)
    for i in range(batch):
        want = oracle.dense_matvec(M, vals[i].astype(np.float64), scale)
        tol = 1e-4 * abs(scale) * float(np.abs(vals[i].astype(np.float64)).sum())
        assert np.max(np.abs(got[i] - want)) <= tol


def _int_matvec_exact(h, M, seed):
    vi = gen.integer_f32(M.shape[1], seed=seed)
    got = rsr.rsr_matvec(h, _dev(vi)).cpu().numpy().astype(np.float64)
    assert np.array_equal(got, oracle.dense_matvec(M, vi.astype(np.float64)))


@pytest.mark.parametrize("kind,k", [(rsr.RSR_TERNARY_FUSED, 8), (rsr.RSR_TERNARY_2PASS, 8),
                                    (rsr.RSR_DENSE_TERNARY_P2, 0)])
def test_metric_workload(kind, k):
    M = gen.metric_matrix()                       # the matrix bench.py times first
    h = rsr.rsr_preprocess(_dev(M), k, kind)
    if kind == rsr.RSR_DENSE_TERNARY_P2:
        assert np.array_equal(rsr.rsr_get_packed(h), oracle.pack2(M))
    else:
        _artifacts_equal(h, M, k, kind)
    _int_matvec_exact(h, M, 3)
    _bf16_matvec_ok(h, M, gen.BASE_SEED + 41)
    fv = gen.normal_f32(M.shape[1], seed=9)
    got = rsr.rsr_matvec(h, _dev(fv)).cpu().numpy()
    want = oracle.dense_matvec(M, fv.astype(np.float64))
    assert np.max(np.abs(got - want)) <= 1e-4 * float(np.abs(fv.astype(np.float64)).sum())


@pytest.mark.parametrize("kind,k", [(rsr.RSR_TERNARY_2PASS, 4), (rsr.RSR_TERNARY_2PASS, 6),
                                    (rsr.RSR_TERNARY_2PASS, 8), (rsr.RSR_TERNARY_2PASS, 10),
                                    (rsr.RSR_TERNARY_FUSED, 4), (rsr.RSR_TERNARY_FUSED, 6),
                                    (rsr.RSR_TERNARY_FUSED, 8), (rsr.RSR_TERNARY_FUSED, 10)])
def test_uniform_ternary_4096_k_sweep(kind, k):
    M = gen.ternary_matrix(4096, 4096, 1.0 / 3.0, gen.BASE_SEED + 20)
    h = rsr.rsr_preprocess(_dev(M), k, kind)
    _artifacts_equal(h, M, k, kind)
    _int_matvec_exact(h, M, 5)
    fv = gen.normal_f32(4096, seed=6)
    got = rsr.rsr_matvec(h, _dev(fv)).cpu().numpy()
    want = oracle.dense_matvec(M, fv.astype(np.float64))
    assert np.max(np.abs(got - want)) <= 1e-4 * float(np.abs(fv.astype(np.float64)).sum())


def test_llm_2b_layer_sequence():
    for n, layer in enumerate(gen.LLM_2B_LAYERS):
        M = gen.ternary_matrix(layer.rows, layer.cols, gen.LLM_2B_P_ZERO, gen.BASE_SEED + 30 + n)
        for kind, k in ((rsr.RSR_TERNARY_FUSED, 7), (rsr.RSR_DENSE_TERNARY_P2, 0)):
            h = rsr.rsr_preprocess(_dev(M), k, kind)
            if kind != rsr.RSR_DENSE_TERNARY_P2:
                _artifacts_equal(h, M, k, kind)
            _bf16_matvec_ok(h, M, 100 + n, scale=0.0173)
            _int_matvec_exact(h, M, 200 + n)


def test_llm_8b_layers_batch_1_and_4():
    for n, layer in enumerate(gen.LLM_8B_LAYERS):
        M = gen.ternary_matrix(layer.rows, layer.cols, gen.LLM_8B_P_ZERO, gen.BASE_SEED + 50 + n)
        h = rsr.rsr_preprocess(_dev(M), 8, rsr.RSR_TERNARY_FUSED)
        _artifacts_equal(h, M, 8, rsr.RSR_TERNARY_FUSED)
        _bf16_matvec_ok(h, M, 300 + n, batch=1)
        _bf16_matvec_ok(h, M, 310 + n, batch=4)


def test_retrieval_table_binary():
    rows, cols, k = 1 << 20, 256, 8
    M = gen.column_density_binary(rows, cols, 0.05, 0.5, gen.BASE_SEED + 60)
    h = rsr.rsr_preprocess(_dev(M), k, rsr.RSR_BINARY)
    _artifacts_equal(h, M, k, rsr.RSR_BINARY)
    q = gen.uniform_f32(cols, seed=61)
    got = rsr.rsr_matvec(h, _dev(q)).cpu().numpy()
    want = oracle.dense_matvec(M, q.astype(np.float64))
    assert np.max(np.abs(got - want)) <= 1e-4 * float(np.abs(q.astype(np.float64)).sum())
    _int_matvec_exact(h, M, 62)
    # 64 queries streamed back to back on one stream, no host sync in between
    qs = np.stack([gen.uniform_f32(cols, seed=700 + i) for i in range(64)])
    qd = _dev(qs)
    outs = torch.empty((64, rows), dtype=torch.float32, device=DEV)
    for i in range(64):
        rsr.rsr_matvec(h, qd[i], out=outs[i])
    torch.cuda.synchronize()
    for i in (0, 31, 63):
        want = oracle.dense_matvec(M, qs[i].astype(np.float64))
        assert np.max(np.abs(outs[i].cpu().numpy() - want)) <= 1e-4 * float(qs[i].sum())
