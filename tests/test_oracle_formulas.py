"""Pins for oracle/formulas.py: the values the paper prints for its worked examples."""
import json
import math
import os
from fractions import Fraction

from oracle import formulas as F

G = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_worked_values.json")))
MIB = 2 ** 20
GIB = 2 ** 30


def test_m_act_worked_examples():
    for name in ("gpt3", "1t"):
        m = G["models"][name]
        v = F.m_act(m["S_seq"], 1, m["S_hidden"], m["N_heads"], m["N_TP"]) / MIB
        assert round(float(v)) == G["m_act_mib_per_sample"][name]


def test_m_ckpt_worked_examples():
    for name in ("gpt3", "1t"):
        m = G["models"][name]
        v = F.m_ckpt("BF", 4, m["N_layers"], m["N_PP"], m["S_seq"], 1, m["S_hidden"], m["N_TP"]) / MIB
        assert v == G["m_ckpt_mib_at_beta_min"][name]


def test_intensities_worked_examples():
    g, t = G["models"]["gpt3"], G["models"]["1t"]
    ipp = G["i_pp"]
    assert abs(float(F.intensity_pp(g["S_hidden"], g["N_layers"], 4, 1)) / ipp["gpt3_nonlooped"] - 1) < 0.01
    assert abs(float(F.intensity_pp(t["S_hidden"], t["N_layers"], 4, 1)) / ipp["1t_nonlooped"] - 1) < 0.01
    # maximally looped: one layer per stage
    assert abs(float(F.intensity_pp(g["S_hidden"], g["N_layers"], 4, g["N_layers"] // 4)) / ipp["gpt3_maxlooped"] - 1) < 0.01
    assert abs(float(F.intensity_pp(t["S_hidden"], t["N_layers"], 4, t["N_layers"] // 4)) / ipp["1t_maxlooped"] - 1) < 0.01
    assert F.intensity_tp(g["S_hidden"], 8) == G["i_tp"]["gpt3"]
    assert F.intensity_tp(t["S_hidden"], 8) == G["i_tp"]["1t"]


def test_state_memory_worked_examples():
    g, t = G["models"]["gpt3"], G["models"]["1t"]
    lo, hi = F.state_memory("DP_PS", F.n_params(g["N_layers"], g["S_hidden"]), N_PP=4, N_TP=8)
    assert [round(float(lo) / GIB), round(float(hi) / GIB)] == G["state_gib"]["gpt3_dp_ps"]
    fs, _ = F.state_memory("DP_FS", F.n_params(t["N_layers"], t["S_hidden"]), N_layers=t["N_layers"], N_TP=8)
    assert round(float(fs) / GIB) == G["state_gib"]["1t_dp_fs"]


def test_hardware_intensity_and_beta_net():
    assert round(312e12 / (559 * GIB), -1) == G["hw_intensity"]["nvlink"]
    assert round(312e12 / (46.6 * GIB), -1) == G["hw_intensity"]["ib"]
    # intensity at beta_min equals the sequence length; ceil(I_hw / I_op)
    assert math.ceil(G["hw_intensity"]["ib"] / F.intensity_dp(1, 1, 2048)) == G["beta_net"]["value"]


def test_bubble_fig4():
    assert F.bubble(4, 8) == Fraction(*G["bubble_fig4"]["nonlooped"])
    assert F.bubble(4, 8, 4) == Fraction(*G["bubble_fig4"]["N_loop_4"])


def test_n_params():
    for k in ("52b", "6.6b"):
        e = G["n_params"][k]
        assert abs(F.n_params(e["N_layers"], e["S_hidden"]) / e["printed"] - 1) < 0.03
    # exact count = 12 N h^2 + 13 N h with S_mlp = 4 S_hidden
    assert F.n_params_exact(8, 8192, 32768) == 12 * 8 * 8192 ** 2 + 13 * 8 * 8192


def test_headline_speedups():
    s = G["speedup"]
    assert round((s["bf"] / s["df"] - 1) * 100) == s["vs_df_percent"]
    assert round((s["bf"] / s["nonlooped"] - 1) * 100) == s["vs_nonlooped_percent"]


def test_eq_compute_is_four_forward_passes():
    # Eq. compute x S_seq == 4 x (linear + full attention forward flops), exactly
    for (N_mb, S_mb, N_layers, h, S_seq) in [(16, 1, 8, 8192, 2048), (4, 4, 8, 8192, 2048), (3, 2, 5, 96, 24)]:
        lhs = F.c_gpu(N_mb, S_mb, N_layers, h, S_seq)
        rhs = 4 * F.fwd_flops_layer_mb(h, S_seq, S_mb) * N_layers * N_mb
        assert lhs == rhs
    # the approximate form: 96 N_mb S_mb N_layers h^2 = 8 flop per parameter and position
    assert 96 * 8192 ** 2 == 8 * F.n_params(1, 8192)


def test_fs_intensities():
    assert F.intensity_fs("plain", 8, 1, 2048) == Fraction(2 * 2048, 3)
    assert F.intensity_fs("DF", 8, 1, 2048, N_PP=4) == 4 * F.intensity_fs("plain", 8, 1, 2048)
    assert F.intensity_fs("BF", 8, 1, 2048) == 8 * F.intensity_fs("plain", 8, 1, 2048)


def test_tensor_parallel_overhead_worked_examples():
    g, t = G["models"]["gpt3"], G["models"]["1t"]
    nv = G["hw_intensity"]["nvlink"]
    assert round(float(F.tp_overhead(g["S_hidden"], 8, nv)) * 100) == G["tp_overhead_percent"]["gpt3"]
    assert round(float(F.tp_overhead(t["S_hidden"], 8, nv)) * 100) == G["tp_overhead_percent"]["1t"]


def test_data_parallel_efficiency_requirements():
    """App. A.3.1 on the worked hardware (I_IB = 6240, S_seq = 2048): beta_net = 4 sequences must be
    overlapped.  Plain accumulation needs them in one micro-batch, depth-first reaches them with
    N_PP = 4 micro-batches of one, breadth-first with any 4 micro-batches; fully sharded the bar
    rises by 3/2 and the micro-batch count stops helping everything but breadth-first."""
    ib = G["hw_intensity"]["ib"]
    assert not F.dp_efficient("plain", 8, 1, 2048, ib) and F.dp_efficient("plain", 1, 4, 2048, ib)
    assert F.dp_efficient("DF", 8, 1, 2048, ib, N_PP=4) and not F.dp_efficient("DF", 8, 1, 2048, ib, N_PP=2)
    assert F.dp_efficient("BF", 4, 1, 2048, ib) and not F.dp_efficient("BF", 3, 1, 2048, ib)
    assert not F.dp_efficient("BF", 4, 1, 2048, ib, sharded=True) and F.dp_efficient("BF", 5, 1, 2048, ib, sharded=True)
    assert not F.dp_efficient("plain", 64, 4, 2048, ib, sharded=True) and F.dp_efficient("plain", 1, 5, 2048, ib, sharded=True)
    # the threshold is where the intensity of App. A.3.1 crosses I_hw
    for n in range(1, 9):
        assert F.dp_efficient("BF", n, 1, 2048, ib) == (F.intensity_dp(n, 1, 2048) >= ib)
        assert F.dp_efficient("BF", n, 1, 2048, ib, sharded=True) == (F.intensity_fs("BF", n, 1, 2048) >= ib)


def test_batch_size_overhead_and_cost_worked_examples():
    """Eq. critical_batch / Eq. time_cost_tradeoff against the overheads the paper prints: GPT-3's batch of
    3 M tokens at a critical batch size of 10 M (Sec. 3.5), and a batch of 1024 at the critical batch
    sizes of the two evaluated models (Sec. 5.4).  cost - 1 of Eq. time_cost_tradeoff at beta N_gpu = B is
    that same overhead, however B is split into beta and N_gpu; time is cost / N_gpu."""
    for name in ("gpt3", "52b", "6.6b"):
        e = G["batch_overhead"][name]
        assert round(float(F.batch_overhead(e["B"], e["B_crit"])) * 100) == e["percent"], name
        for n_gpu in (64, 512, 4096):
            cost, time = F.cost_time(Fraction(e["B"], n_gpu), n_gpu, e["B_crit"])
            assert round(float(cost - 1) * 100) == e["percent"]
            assert time * n_gpu == cost
    # at a fixed batch size per GPU more GPUs cost more and finish sooner; a lower utilisation costs in proportion
    c1, t1 = F.cost_time(1, 1000, 10_000)
    c2, t2 = F.cost_time(1, 4000, 10_000)
    assert c2 > c1 and t2 < t1
    assert F.cost_time(1, 1000, 10_000, Fraction(1, 2))[0] == 2 * c1


def _eff(kind, N_mb, S_mb, beta_net, **kw):
    return F.efficiency(kind, N_mb, S_mb, beta_net, **kw)


def test_efficiency_model_thresholds_are_the_papers_conditions():
    """The network overhead of the overlapped model vanishes exactly where the paper's efficiency conditions
    hold: beta >= N_mb beta_net / (N_PP N_TP) without looping (Eq. ddp_efficiency, Eq. pipeline_efficiency_3d),
    beta >= beta_net / (N_PP N_TP) breadth-first (Eq. pipeline_efficiency_bf), N_PP micro-batches' worth
    depth-first (Sec. 4.2); fully sharded the bar is 3/2 higher (Sec. 3.1) and, except breadth-first, no longer
    helped by more micro-batches."""
    bn = G["efficiency_thresholds"]["beta_net_example"]
    fs = Fraction(*G["efficiency_thresholds"]["sharded_factor"])
    for N_PP, N_TP in [(1, 1), (4, 1), (4, 2), (8, 8)]:
        for N_mb in (N_PP, 2 * N_PP, 8 * N_PP):
            for S_mb in range(1, 13):
                beta = Fraction(N_mb * S_mb, N_PP * N_TP)
                kinds = ["plain"] if N_PP == 1 else ["GPIPE", "DF", "BF"]
                for kind in kinds:
                    e = _eff(kind, N_mb, S_mb, bn, N_PP=N_PP, N_TP=N_TP, N_loop=1 if kind in ("plain", "GPIPE") else 2)
                    assert e["beta"] == beta
                    bar = {"plain": N_mb * bn, "GPIPE": N_mb * bn, "DF": Fraction(N_mb, N_PP) * bn, "BF": bn}[kind]
                    assert (e["net_overhead"] == 0) == (beta >= Fraction(bar, N_PP * N_TP)), (kind, N_PP, N_mb, S_mb)
                    assert e["efficiency"] == 1 / (1 + e["bubble"] + e["net_overhead"])
                    s = _eff(kind, N_mb, S_mb, bn, N_PP=N_PP, N_TP=N_TP, sharded=True)
                    bar_s = {"plain": N_mb, "GPIPE": N_mb, "DF": Fraction(N_mb, N_PP), "BF": 1}[kind] * fs * bn
                    assert (s["net_overhead"] == 0) == (beta >= Fraction(bar_s, N_PP * N_TP)), (kind, "sharded")
    # lower bound on N_PP for efficient breadth-first training at beta_min = 1 / N_TP (Sec. 4.2): N_PP >= beta_net / beta_min
    for N_TP in (1, 2):
        for N_PP in range(1, 12):
            e = _eff("BF", N_PP, 1, bn, N_PP=N_PP, N_TP=N_TP, N_loop=4)     # N_mb = N_PP, S_mb = 1: beta = beta_min
            assert e["beta"] == Fraction(1, N_TP)
            assert (e["net_overhead"] == 0) == (N_PP >= bn)


def test_efficiency_model_limits_and_ordering():
    """Fig. 2, qualitatively: at equal batch size per GPU breadth-first >= depth-first >= non-looped once looped;
    without overlap the network time is paid in full (Eq. efficiency, second branch) and decays as 1 / beta;
    the bubble is Eq. bubble_looped; with the share of Table 4.1's overlap column the last stage's part is lost."""
    bn = G["efficiency_thresholds"]["beta_net_fig2"]
    N_PP = 4
    for N_mb in (4, 8, 16, 64):
        g = _eff("GPIPE", N_mb, 1, bn, N_PP=N_PP)
        d = _eff("DF", N_mb, 1, bn, N_PP=N_PP, N_loop=4)
        b = _eff("BF", N_mb, 1, bn, N_PP=N_PP, N_loop=4)
        assert b["efficiency"] >= d["efficiency"] >= g["efficiency"]
        assert b["bubble"] == d["bubble"] == F.bubble(N_PP, N_mb, 4) and g["bubble"] == F.bubble(N_PP, N_mb)
        # beta = N_mb / 4 < beta_net / N_PP = 1.5 only for N_mb = 4: breadth-first hides the reduction from N_mb = 6 on
        assert (b["net_overhead"] == 0) == (N_mb >= bn)
        for kind, e in (("GPIPE", g), ("DF", d), ("BF", b)):
            n = _eff(kind, N_mb, 1, bn, N_PP=N_PP, N_loop=1 if kind == "GPIPE" else 4, overlap=False)
            assert n["net_overhead"] == n["net_ratio"] == Fraction(bn, N_mb) and n["efficiency"] <= e["efficiency"]
    # Table 4.1, column "DP overlap", with a finite number of layers
    e = _eff("BF", 8, 1, 16, N_PP=4, N_loop=2, N_layers=16)
    assert e["overlap_share"] == F.dp_overlap("BF", 8, 16, 4) == Fraction(3, 4)
    assert e["net_overhead"] == Fraction(16, 8) - Fraction(3, 4)
    e = _eff("DF", 8, 1, 16, N_PP=4, N_loop=2, N_layers=16)
    assert e["overlap_share"] == Fraction(3, 4) * Fraction(4, 8)
    # network volume column: 2 / N_PP, fully sharded 3 / N_PP times the repetitions
    assert F.dp_network("BF", 8, 4) == Fraction(2, 4) and F.dp_network("BF", 8, 4, sharded=True) == Fraction(3, 4)
    assert F.dp_network("DF", 8, 4, sharded=True) == Fraction(3, 4) * 2 and F.dp_network("plain", 8, 1, sharded=True) == 24
