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
