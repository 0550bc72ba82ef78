"""The library's analytical calculators (include/bf_calc.h, host arithmetic only) against the oracle's
exact-fraction model, which tests/test_oracle_formulas.py pins to the paper's conditions and printed values."""
import itertools
from fractions import Fraction

import pytest

import paper_2211_05953_amd as bf
from oracle import formulas as F

KIND = {bf.BF_METHOD_NO_PIPELINE: "plain", bf.BF_METHOD_NON_LOOPED: "GPIPE", bf.BF_METHOD_DEPTH_FIRST: "DF",
        bf.BF_METHOD_BREADTH_FIRST: "BF"}


def _valid(method, N_PP, N_loop, N_mb, N_layers):
    if method == bf.BF_METHOD_NO_PIPELINE and (N_PP != 1 or N_loop != 1):
        return False
    if method == bf.BF_METHOD_NON_LOOPED and N_loop != 1:
        return False
    if N_mb < N_PP or (method == bf.BF_METHOD_DEPTH_FIRST and N_mb % N_PP):
        return False
    return not (N_layers and N_layers % (N_PP * N_loop))


def test_efficiency_matches_the_oracle_on_a_grid():
    n = 0
    for method, N_PP, N_loop, N_TP, N_mb, S_mb, N_layers, sharded, overlap in itertools.product(
            KIND, (1, 2, 4), (1, 2, 4), (1, 2), (1, 2, 4, 6, 8, 16), (1, 3), (0, 16), (0, 1), (0, 1)):
        for beta_net in (Fraction(4), Fraction(6), Fraction(305, 100)):
            ok = _valid(method, N_PP, N_loop, N_mb, N_layers)
            if not ok:
                with pytest.raises(bf.BfError):
                    bf.bf_calc_efficiency(method, N_PP, N_loop, N_TP, N_layers, N_mb, S_mb, sharded, overlap, float(beta_net))
                continue
            if N_layers and N_layers == N_PP:
                continue
            got = bf.bf_calc_efficiency(method, N_PP, N_loop, N_TP, N_layers, N_mb, S_mb, sharded, overlap, float(beta_net))
            ref = F.efficiency(KIND[method], N_mb, S_mb, beta_net, N_PP=N_PP, N_loop=N_loop, N_TP=N_TP,
                               N_layers=N_layers or None, sharded=bool(sharded), overlap=bool(overlap))
            for k, v in ref.items():
                assert got[k] == pytest.approx(float(v), rel=1e-12, abs=1e-15), (k, method, N_PP, N_loop, N_mb, S_mb)
            n += 1
    assert n > 2000


def test_efficiency_curve_and_threshold():
    # Fig. 2's example: beta_net = 6, N_TP = 1, S_mb = 1, N_PP = 4
    counts = list(range(1, 33))
    for method, N_loop in ((bf.BF_METHOD_NON_LOOPED, 1), (bf.BF_METHOD_DEPTH_FIRST, 4), (bf.BF_METHOD_BREADTH_FIRST, 4)):
        pts = bf.bf_calc_efficiency_curve(method, 4, N_loop, 1, 0, 1, 0, 1, 6.0, counts)
        for N_mb, p in zip(counts, pts):
            if not _valid(method, 4, N_loop, N_mb, 0):
                assert p["efficiency"] == -1.0
                continue
            ref = F.efficiency(KIND[method], N_mb, 1, 6, N_PP=4, N_loop=N_loop)
            assert p["efficiency"] == pytest.approx(float(ref["efficiency"]), rel=1e-12)
            assert p["beta"] == pytest.approx(N_mb / 4)
    # thresholds: the right-hand sides of Eq. ddp_efficiency / Eq. pipeline_efficiency_3d / Eq. pipeline_efficiency_bf
    assert bf.bf_calc_beta_threshold(bf.BF_METHOD_NO_PIPELINE, 1, 1, 1, 0, 3, 1, 0, 1, 4.0) == pytest.approx(3 * 4.0)
    assert bf.bf_calc_beta_threshold(bf.BF_METHOD_NON_LOOPED, 4, 1, 2, 0, 8, 1, 0, 1, 4.0) == pytest.approx(8 * 4.0 / (4 * 2))
    assert bf.bf_calc_beta_threshold(bf.BF_METHOD_BREADTH_FIRST, 4, 2, 2, 0, 8, 1, 0, 1, 4.0) == pytest.approx(4.0 / (4 * 2))
    assert bf.bf_calc_beta_threshold(bf.BF_METHOD_BREADTH_FIRST, 4, 2, 2, 0, 8, 1, 1, 1, 4.0) == pytest.approx(1.5 * 4.0 / (4 * 2))
    assert bf.bf_calc_beta_threshold(bf.BF_METHOD_DEPTH_FIRST, 4, 2, 1, 0, 8, 1, 0, 1, 4.0) == pytest.approx(2 * 4.0 / 4)
    # and the model's overhead vanishes exactly from the threshold on
    for N_mb in (4, 8, 12):
        thr = bf.bf_calc_beta_threshold(bf.BF_METHOD_DEPTH_FIRST, 4, 2, 1, 0, N_mb, 1, 0, 1, 4.0)
        for S_mb in range(1, 8):
            p = bf.bf_calc_efficiency(bf.BF_METHOD_DEPTH_FIRST, 4, 2, 1, 0, N_mb, S_mb, 0, 1, 4.0)
            assert (p["net_overhead"] == 0.0) == (p["beta"] >= thr - 1e-12)


def test_cost_time():
    for beta, n_gpu, b_crit, eff in [(1.0, 1000.0, 10000.0, 1.0), (0.125, 4096.0, 6780.0, 0.4), (2.0, 512.0, 3430.0, 0.55)]:
        cost, time = bf.bf_calc_cost_time(beta, n_gpu, b_crit, eff)
        rc, rt = F.cost_time(Fraction(beta), Fraction(n_gpu), Fraction(b_crit), Fraction(eff))
        assert cost == pytest.approx(float(rc), rel=1e-12) and time == pytest.approx(float(rt), rel=1e-12)
    with pytest.raises(bf.BfError):
        bf.bf_calc_cost_time(1.0, 0.0, 10.0, 1.0)
    with pytest.raises(bf.BfError):
        bf.bf_calc_cost_time(1.0, 8.0, 10.0, 1.5)
