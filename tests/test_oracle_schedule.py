"""Pins for oracle/schedule.py and the event order of oracle/stack.py: the closed-form
bubble (Eq. bubble, Eq. bubble_looped) and checkpoint counts (Eq. mem_ckpt)."""
from fractions import Fraction

import pytest

from oracle import formulas as F
from oracle import schedule as S
from oracle import stack as K


@pytest.mark.parametrize("t_fwd,t_bwd", [(1, 2), (1, 3), (2, 3)])
def test_bf_bubble_equals_closed_form(t_fwd, t_bwd):
    for N_PP in (1, 2, 3, 4, 8):
        for N_loop in (1, 2, 4, 8):
            for N_mb in (N_PP, N_PP + 1, 2 * N_PP, 16):
                if N_mb < N_PP:
                    continue
                r = S.simulate("BF", N_PP, N_loop, N_mb, t_fwd, t_bwd)
                assert r["bubble"] == F.bubble(N_PP, N_mb, N_loop), (N_PP, N_loop, N_mb)
                # every stage input of the device is alive at the forward/backward turn
                assert r["peak_live"] == [N_loop * N_mb] * N_PP


def test_fig4_example():
    # 16 layers on 4 devices, 8 micro-batches: non-looped 3/8, 16 one-layer stages 3/32
    assert S.simulate("BF", 4, 1, 8)["bubble"] == Fraction(3, 8)
    assert S.simulate("BF", 4, 4, 8)["bubble"] == Fraction(3, 32)
    assert S.simulate("DF", 4, 1, 8)["bubble"] == Fraction(3, 8)
    assert S.simulate("DF", 4, 4, 8)["bubble"] == Fraction(3, 32)


def test_df_each_op_once_and_bubble():
    for N_PP in (1, 2, 4):
        for N_loop in (1, 2, 4):
            for mult in (1, 2, 3):
                N_mb = N_PP * mult
                r = S.simulate("DF", N_PP, N_loop, N_mb, 1, 2)
                seen = set()
                for dev in r["events"]:
                    for _, op, j, m in dev:
                        assert (op, j, m) not in seen
                        seen.add((op, j, m))
                assert len(seen) == 2 * N_PP * N_loop * N_mb
                assert r["bubble"] == F.bubble(N_PP, N_mb, N_loop), (N_PP, N_loop, N_mb)
                # backward-first keeps fewer inputs alive than forward-first
                assert max(r["peak_live"]) <= N_loop * N_mb


def test_checkpoint_counts_single_device():
    # N_PP = 1: BF holds N_mb * N_layers checkpoints, DF holds N_layers
    for N_layers, N_loop, N_mb in [(4, 2, 4), (8, 4, 16), (16, 16, 32), (6, 3, 8), (2, 1, 1)]:
        per_stage = N_layers // N_loop
        bf = S.simulate("BF", 1, N_loop, N_mb)
        df = S.simulate("DF", 1, N_loop, N_mb)
        assert bf["peak_live"][0] * per_stage == F.ckpt_count("BF", N_mb, N_layers, 1)
        assert df["peak_live"][0] * per_stage == F.ckpt_count("DF", N_mb, N_layers, 1) == min(N_layers, N_mb * N_layers)
        assert bf["bubble"] == df["bubble"] == 0


def test_stack_event_order_matches_simulator_at_npp1():
    for N_loop, N_mb in [(2, 4), (4, 16), (16, 32), (1, 3)]:
        for kind, code in (("BF", K.SCHED_BF), ("DF", K.SCHED_DF)):
            ev = [(op, s, m) for op, s, m in K.event_order(code, N_loop, N_mb) if op != K.OP_OPT]
            assert ev == S.device_order(kind, 1, N_loop, N_mb, 0)
            full = K.event_order(code, N_loop, N_mb)
            assert len(full) == 2 * N_loop * N_mb + N_loop
            # the optimizer step of a stage directly follows that stage's last backward
            for i, (op, s, m) in enumerate(full):
                if op == K.OP_OPT:
                    assert full[i - 1] == (K.OP_B, s, N_mb - 1)


def test_bf_needs_enough_microbatches_and_df_multiple():
    with pytest.raises(ValueError):
        S.device_order("BF", 4, 2, 3, 0)
    with pytest.raises(ValueError):
        S.device_order("DF", 4, 2, 6, 0)


def test_weight_intervals_match_the_sharded_intensities():
    """Fully sharded data parallelism reconstructs a stage once per interval of use.  Breadth-first:
    a single forward and a single backward interval per stage, whatever N_mb (Sec. 4.2); plain
    gradient accumulation (depth-first at N_PP = 1) repeats them for every micro-batch (Sec. 3.1).
    The ratio of the two counts is the ratio of the intensities I_FS-BF / I_FS of App. A.3.1."""
    for N_PP in (1, 2, 4):
        for N_loop in (1, 2, 3, 4, 8):
            for N_mb in (N_PP, 2 * N_PP, 4 * N_PP, 16 * N_PP):
                for rank in range(N_PP):
                    bf = S.weight_intervals(S.device_order("BF", N_PP, N_loop, N_mb, rank))
                    assert len(bf) == 2 * N_loop
                    assert sorted(st for _, st, _, _ in bf) == sorted(2 * [l * N_PP + rank for l in range(N_loop)])
                    assert all(n == N_mb for _, _, _, n in bf)
                    df = S.weight_intervals(S.device_order("DF", N_PP, N_loop, N_mb, rank))
                    # a sequence holds N_PP micro-batches: never fewer intervals than one per sequence
                    assert 2 * N_loop * N_mb // N_PP <= len(df) <= 2 * N_loop * N_mb
                    assert sum(n for _, _, _, n in df) == 2 * N_loop * N_mb
                    if N_PP == 1:
                        assert len(df) == 2 * N_loop * N_mb
                        assert Fraction(len(df), len(bf)) == F.intensity_fs("BF", N_mb, 1, 2048) / F.intensity_fs("plain", N_mb, 1, 2048)


def _count_misses_brute(stages, n_buffers):
    """Least-recently-used replacement written the slow way: time stamps, no list surgery."""
    last, held, misses = {}, set(), 0
    for t, st in enumerate(stages):
        if st not in held:
            misses += 1
            if len(held) == n_buffers:
                held.remove(min(held, key=lambda k: last[k]))
            held.add(st)
        last[st] = t
    return misses


def test_reconstruction_counts_with_a_double_buffer():
    """With the two most recent stages kept (App. D.1, double buffer) the turn-around from the last
    forward stage into the backward pass finds both stages in place."""
    for N_loop in (1, 2, 3, 4, 8):
        for N_mb in (1, 2, 5, 16):
            bf = S.device_order("BF", 1, N_loop, N_mb, 0)
            df = S.device_order("DF", 1, N_loop, N_mb, 0)
            n_bf, held_bf = S.reconstructions(bf)
            n_df, _ = S.reconstructions(df)
            assert n_bf == (N_loop if N_loop <= 2 else 2 * N_loop - 2)
            assert n_df == (N_loop if N_loop <= 2 else N_mb * (2 * N_loop - 4) + 2)
            assert held_bf[-1] == 0
            for order, n in ((bf, n_bf), (df, n_df)):
                assert n == _count_misses_brute([st for _, st, _, _ in S.weight_intervals(order)], 2)
            # one buffer: every interval but the forward-to-backward turn of the last stage reloads
            assert S.reconstructions(bf, n_buffers=1)[0] == 2 * N_loop - 1
            # a second step with nothing changed starts from what the first left behind
            again, _ = S.reconstructions(bf, resident=held_bf)
            assert again == (0 if N_loop <= 2 else 2 * N_loop - 4)


def _overlap_share(ops):
    """Backward ops still to run when the first stage of the rank has finished all its backwards."""
    n_mb = 1 + max(m for _, _, m in ops)
    done = {}
    total_b = sum(1 for op, _, _ in ops if op == S.OP_B)
    seen_b = 0
    for op, st, m in ops:
        if op != S.OP_B:
            continue
        seen_b += 1
        done[st] = done.get(st, 0) + 1
        if done[st] == n_mb:
            return Fraction(total_b - seen_b, total_b)
    raise AssertionError


def test_gradient_reduction_overlap_matches_the_method_table():
    """Table 4.1, "DP overlap": breadth-first can hide a stage's reduction under 1 - N_PP / N_stage of the
    backward pass, depth-first only under the last sequence's share, plain accumulation under one
    micro-batch's.  Read off the op orders the simulator and the stack execute."""
    for N_PP in (1, 2, 4):
        for N_loop in (1, 2, 4, 8):
            for mult in (1, 2, 4):
                N_mb = N_PP * mult
                N_stage = N_PP * N_loop
                for rank in range(N_PP):
                    assert _overlap_share(S.device_order("BF", N_PP, N_loop, N_mb, rank)) == F.dp_overlap("BF", N_mb, N_stage, N_PP)
                    if N_PP == 1 or rank == 0:
                        assert _overlap_share(S.device_order("DF", N_PP, N_loop, N_mb, rank)) == F.dp_overlap("DF", N_mb, N_stage, N_PP), (N_PP, N_loop, N_mb, rank)
    # at N_PP = 1 depth-first is plain gradient accumulation (App. C) and the stack's own event order agrees
    for N_loop, N_mb in [(2, 4), (4, 16), (8, 3)]:
        for kind, code in (("BF", K.SCHED_BF), ("DF", K.SCHED_DF)):
            full = K.event_order(code, N_loop, N_mb)
            first_opt = next(i for i, e in enumerate(full) if e[0] == K.OP_OPT)
            rest = sum(1 for e in full[first_opt:] if e[0] == K.OP_B)
            assert Fraction(rest, N_loop * N_mb) == F.dp_overlap(kind, N_mb, N_loop, 1)
        assert F.dp_overlap("DF", N_mb, N_loop, 1) == F.dp_overlap("plain", N_mb, N_loop, 1)
