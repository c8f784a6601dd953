"""CPU tests of the library's host-side helpers (no GPU needed) against the oracle's
definitions: threshold folding (Sec. 3.2.2) and the cost-aware masking priority (Sec. 3.1.2)."""
import numpy as np

from oracle import oracle as O
from paper_2601_11660_amd import binding as B


def test_library_threshold_folding_equals_batchnorm_sign():
    """mbu_fold_batchnorm (host code of the library) against the oracle's definition, for every
    integer sum a layer can produce."""
    rng = np.random.default_rng(22)
    C, fan_in = 96, 9 * 64
    g = rng.standard_normal(C)
    g[::7] = 0.0
    g[1::5] = -np.abs(g[1::5])
    b = rng.standard_normal(C) * 2
    m = rng.standard_normal(C) * 30
    v = rng.uniform(0.1, 90.0, C)
    bias = rng.standard_normal(C) * 2
    thresh, flip = B.fold_batchnorm(g, b, m, v, 1e-5, bias, fan_in)
    assert np.array_equal(flip != 0, g < 0)
    acc = np.arange(-fan_in, fan_in + 1)[:, None].repeat(C, 1)
    y, s = O.batchnorm_sign(acc, g, b, m, v, 1e-5, bias)
    got = np.where(np.where(flip[None, :] != 0, -acc, acc) >= thresh[None, :], 1, -1)
    sure = np.abs(y) > 1e-9          # away from the rounding noise of the float64 expressions
    assert sure.mean() > 0.999 and np.array_equal(got[sure], s[sure])
    assert (np.abs(thresh) <= fan_in + 1).all()
    # hand-solvable: acc - 1.5 + 0.3 >= 0 <=> acc >= 2;  -2 (acc - 1.5) + 0.3 >= 0 <=> -acc >= -1
    t, f = B.fold_batchnorm([1.0, -2.0, 0.0, 0.0], [0.3, 0.3, -1.0, 1.0], [1.5, 1.5, 0.0, 0.0],
                            [1.0, 1.0, 1.0, 1.0], 0.0, None, 576)
    assert t.tolist() == [2, -1, 577, -577] and f.tolist() == [0, 1, 0, 0]


def test_library_cost_ranking_equals_definition():
    rng = np.random.default_rng(23)
    ops = rng.uniform(1e6, 1e11, 12)
    par = rng.uniform(1e3, 1e7, 12)
    for w_op in (0.0, 0.3, 0.5, 1.0):
        s, order = O.cost_scores(ops, par, w_op)
        gs, go = B.cost_rank(ops, par, w_op)
        assert np.allclose(gs, s, rtol=1e-14, atol=0) and np.array_equal(go, order)
    # ties keep the lower index first; constant counts score 0
    gs, go = B.cost_rank([3, 3, 3], [7, 7, 7], 0.5)
    assert gs.tolist() == [0.0, 0.0, 0.0] and go.tolist() == [0, 1, 2]


def test_host_helper_argument_validation():
    import ctypes
    L = B.lib()
    d3 = (ctypes.c_double * 3)(1.0, 1.0, 1.0)
    t3 = (ctypes.c_int32 * 3)()
    f3 = (ctypes.c_int8 * 3)()
    o3 = (ctypes.c_int * 3)()
    assert L.mbu_fold_batchnorm(None, d3, d3, d3, 1e-5, None, 3, 576, t3, f3) == B.MBU_ERR_NULL
    assert L.mbu_fold_batchnorm(d3, d3, d3, d3, 1e-5, None, 0, 576, t3, f3) == B.MBU_ERR_SHAPE
    assert L.mbu_fold_batchnorm(d3, d3, d3, d3, -1.0, None, 3, 576, t3, f3) == B.MBU_ERR_ARG
    neg = (ctypes.c_double * 3)(1.0, -2.0, 1.0)
    assert L.mbu_fold_batchnorm(d3, d3, d3, neg, 0.0, None, 3, 576, t3, f3) == B.MBU_ERR_ARG
    assert L.mbu_cost_rank(d3, d3, 3, 1.5, d3, o3) == B.MBU_ERR_ARG
    assert L.mbu_cost_rank(d3, None, 3, 0.5, d3, o3) == B.MBU_ERR_NULL
    assert L.mbu_cost_rank(d3, d3, 0, 0.5, d3, o3) == B.MBU_ERR_SHAPE
