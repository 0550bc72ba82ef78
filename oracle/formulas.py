"""The paper's closed forms (App. A), in exact integer / rational arithmetic.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).
"""
from fractions import Fraction


def n_params(N_layers, S_hidden):
    """App. A.1: N_params ~ 12 N_layers S_hidden^2 (weights of the four linears)."""
    return 12 * N_layers * S_hidden ** 2


def n_params_exact(N_layers, S_hidden, S_mlp):
    """All parameters of the layer stack built here, biases and LayerNorms included."""
    h, f = S_hidden, S_mlp
    per = (h * 3 * h + 3 * h) + (h * h + h) + (h * f + f) + (f * h + h) + 4 * h
    return N_layers * per


def bubble(N_PP, N_mb, N_loop=1):
    """Eq. bubble (Sec. 3.2) and Eq. bubble_looped (Sec. 4.1)."""
    return Fraction(N_PP - 1, N_mb * N_loop)


def m_act(S_seq, S_mb, S_hidden, N_heads, N_TP=1):
    """App. A.2.2: activation bytes of one layer and micro-batch (with dropout masks
    and unfused attention scores), as an exact fraction."""
    return S_seq * S_mb * S_hidden * (10 + Fraction(24, N_TP) + Fraction(5 * S_seq * N_heads, S_hidden * N_TP))


def ckpt_count(kind, N_mb, N_layers, N_PP):
    """Number of live checkpoints, first ratio of Eq. mem_ckpt with the caps the
    text gives for the backward-first schedules."""
    full = Fraction(N_mb * N_layers, N_PP)
    if kind in ("BF", "GPIPE"):
        return full
    if kind == "1F1B":
        return min(full, Fraction((2 * N_PP - 1) * N_layers, N_PP))
    if kind == "DF":
        return min(full, Fraction(N_layers + N_PP - 1))
    raise ValueError(kind)


def ckpt_bytes_each(S_seq, S_mb, S_hidden, N_TP=1):
    """Second ratio of Eq. mem_ckpt: one half-precision [S_mb, S_seq, S_hidden] tensor."""
    return Fraction(2 * S_seq * S_mb * S_hidden, N_TP)


def m_ckpt(kind, N_mb, N_layers, N_PP, S_seq, S_mb, S_hidden, N_TP=1):
    return ckpt_count(kind, N_mb, N_layers, N_PP) * ckpt_bytes_each(S_seq, S_mb, S_hidden, N_TP)


def c_gpu_per_position(N_mb, S_mb, N_layers, S_hidden, S_seq, S_voc=0, N_PP=1, N_TP=1):
    """Eq. compute exactly as printed (flop per GPU, per sequence position)."""
    return Fraction(96 * N_mb * S_mb * N_layers * S_hidden, N_PP * N_TP) * (
        S_hidden + Fraction(S_seq, 6) + Fraction(S_voc, 16 * N_layers))


def c_gpu(N_mb, S_mb, N_layers, S_hidden, S_seq, S_voc=0, N_PP=1, N_TP=1):
    """Eq. compute times S_seq: flop per GPU and batch.  (As printed the equation has
    no S_seq factor; with it the value is 4x the forward flops of the linears plus
    full attention, i.e. forward + recomputed forward + backward.)"""
    return c_gpu_per_position(N_mb, S_mb, N_layers, S_hidden, S_seq, S_voc, N_PP, N_TP) * S_seq


def fwd_flops_layer_mb(S_hidden, S_seq, S_mb):
    """Forward flops of one layer on one micro-batch with S_mlp = 4 S_hidden and full
    (non-causal) attention: 2 flop per multiply-add."""
    T = S_seq * S_mb
    return 24 * S_hidden ** 2 * T + 4 * S_seq * T * S_hidden


def state_memory(kind, N_params, N_layers=1, N_PP=1, N_TP=1):
    """App. A.2.1: (low, high) bytes of state memory."""
    if kind == "DP0":
        return Fraction(12 * N_params, N_PP * N_TP), Fraction(20 * N_params, N_PP * N_TP)
    if kind == "DP_PS":
        return Fraction(2 * N_params, N_PP * N_TP), Fraction(4 * N_params, N_PP * N_TP)
    if kind == "DP_FS":
        v = Fraction(8 * N_params, N_layers * N_TP)
        return v, v
    raise ValueError(kind)


def intensity_pp(S_hidden, N_layers, N_PP, N_loop):
    """Eq. intensity_pipeline: I_PP = 24 S_hidden N_layers / (N_PP N_loop)."""
    return Fraction(24 * S_hidden * N_layers, N_PP * N_loop)


def intensity_tp(S_hidden, N_TP):
    """App. A.3.3: I_TP = 2 S_hidden / N_TP."""
    return Fraction(2 * S_hidden, N_TP)


def tp_overhead(S_hidden, N_TP, I_hw):
    """App. A.3.3: two thirds of the tensor-parallel traffic cannot be overlapped, so the expected
    overhead is (2/3) T_net / T_comp = (2/3) I_hw / I_TP (App. A.3: T_comp / T_net ~ I_op / I_hw)."""
    return Fraction(2, 3) * Fraction(I_hw) / intensity_tp(S_hidden, N_TP)


def dp_efficient(kind, N_mb, S_mb, S_seq, I_hw, N_PP=1, sharded=False):
    """App. A.3.1, the overlapped branch of the efficiency requirements: the reduction (and, fully
    sharded, the reconstruction) hides behind the computation it can overlap with when that
    computation's intensity reaches the hardware intensity.  Non-looped / plain accumulation overlaps
    with one micro-batch, depth-first with N_PP of them, breadth-first with the whole batch."""
    n = {"plain": 1, "DF": N_PP, "BF": N_mb}[kind]
    i_op = Fraction(2 * n * S_mb * S_seq, 3) if sharded else n * S_mb * S_seq
    return i_op >= I_hw


def intensity_dp(N_mb, S_mb, S_seq):
    """App. A.3.1: I_DP0 ~ I_DP_PS = N_mb S_mb S_seq."""
    return N_mb * S_mb * S_seq


def intensity_fs(kind, N_mb, S_mb, S_seq, N_PP=1):
    """App. A.3.1: fully sharded intensities."""
    if kind == "plain":
        return Fraction(2 * S_mb * S_seq, 3)
    if kind == "DF":
        return Fraction(2 * N_PP * S_mb * S_seq, 3)
    if kind == "BF":
        return Fraction(2 * N_mb * S_mb * S_seq, 3)
    raise ValueError(kind)


def dp_overlap(kind, N_mb, N_stage, N_PP=1):
    """Table 4.1, column "DP overlap": the share of the backward pass that is still to run when the
    first stage's gradient is complete, i.e. the computation a gradient reduction can hide under.
    Stages of one layer each in the table (N_layers = N_stage)."""
    rest = 1 - Fraction(N_PP, N_stage)
    if kind == "BF":
        return rest
    if kind == "DF":
        return rest * Fraction(N_PP, N_mb)
    if kind in ("GPIPE", "1F1B", "plain"):       # non-looped pipelines / plain gradient accumulation
        return rest / N_mb
    raise ValueError(kind)


def batch_overhead(B, B_crit):
    """Sec. 3.5 (Eq. critical_batch): samples needed grow as 1 + B / B_crit; the relative overhead is B / B_crit."""
    return Fraction(B) / Fraction(B_crit)


def cost_time(beta, N_gpu, B_crit, efficiency=1):
    """Eq. time_cost_tradeoff: (cost, time) up to a common factor, at a fixed batch size per GPU beta
    (cost is proportional to the samples processed, Eq. critical_batch, over the utilisation)."""
    cost = (1 + Fraction(beta) * N_gpu / Fraction(B_crit)) / Fraction(efficiency)
    return cost, cost / N_gpu


# ------------------------------------------------------------------ efficiency model (Fig. 2)
def dp_network(kind, N_mb, N_PP=1, sharded=False):
    """Table 4.1, column "DP network": volume per GPU in units of the model size.  A reduction plus a
    reconstruction is 2; fully sharded it is 3 (Sec. 3.1: at least 50 % more), repeated for every
    micro-batch without looping, for every sequence of N_PP micro-batches depth-first (Sec. 4.2), and
    not repeated breadth-first.  A pipeline rank holds 1 / N_PP of the model.  (The table prints the
    sharded 1F1B entry without the 1 / N_PP; it is taken with it, like every other pipeline row.)"""
    if not sharded:
        return Fraction(2, N_PP)
    reps = {"plain": N_mb, "GPIPE": N_mb, "1F1B": N_mb, "DF": Fraction(N_mb, N_PP), "BF": 1}[kind]
    return Fraction(3, N_PP) * reps


def efficiency(kind, N_mb, S_mb, beta_net, N_PP=1, N_loop=1, N_TP=1, N_layers=None, sharded=False, overlap=True):
    """Theoretical efficiency behind Fig. 2, from the paper's own proportionalities.

    Footnote to Eq. ddp_efficiency: with plain data parallelism T_net / T_comp = beta_net / (N_mb S_mb).
    Other methods scale the network volume by Table 4.1's "DP network" column relative to its plain
    entry and the computation by 1 / N_PP.  Eq. efficiency: an overlapped operation costs what exceeds
    the computation it can hide under (Table 4.1, "DP overlap"; a repeated sharded operation hides under
    its own micro-batches each time, so under the whole pass in total); a non-overlapped one costs
    all of T_net.  The bubble of Eq. bubble / Eq. bubble_looped adds idle time.  Pipeline-parallel
    transfers are left out (the paper calls them mostly negligible and gives no figure).
    Returns dict(beta, bubble, net_ratio, overlap_share, net_overhead, efficiency) of Fractions."""
    beta_net = Fraction(beta_net)
    n_stage_for_tail = N_layers if N_layers else None
    t_comp = Fraction(N_mb * S_mb, N_PP)
    t_net = dp_network(kind, N_mb, N_PP, sharded) / dp_network("plain", 1) * beta_net
    net_ratio = t_net / t_comp
    if not overlap:
        share = Fraction(0)
    else:
        tail = 1 - Fraction(N_PP, n_stage_for_tail) if n_stage_for_tail else Fraction(1)
        if sharded:
            share = tail
        elif n_stage_for_tail:
            share = dp_overlap(kind, N_mb, n_stage_for_tail, N_PP)
        else:
            share = {"plain": Fraction(1, N_mb), "GPIPE": Fraction(1, N_mb), "1F1B": Fraction(1, N_mb),
                     "DF": Fraction(N_PP, N_mb), "BF": Fraction(1)}[kind]
    over = max(Fraction(0), net_ratio - share)
    b = bubble(N_PP, N_mb, N_loop)
    return dict(beta=Fraction(N_mb * S_mb, N_PP * N_TP), bubble=b, net_ratio=net_ratio, overlap_share=share,
                net_overhead=over, efficiency=1 / (1 + b + over))
