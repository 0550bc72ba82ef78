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
