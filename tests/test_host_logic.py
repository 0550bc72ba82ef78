"""CPU-only checks of the C-ABI library: it loads, exports what include/*.h declares,
validates arguments, and its integer schedule generator matches the oracle's simulator
and the closed forms (Eq. bubble, Eq. bubble_looped, Eq. mem_ckpt)."""
import os
import re
from fractions import Fraction

import pytest

import paper_2211_05953_amd as bf
from oracle import formulas as F
from oracle import schedule as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = bf.load()
    declared = set()
    headers = sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))
    assert {"bf.h", "bf_ops.h", "bf_calc.h"} <= set(headers)
    for hdr in headers:
        text = open(os.path.join(ROOT, "include", hdr)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        declared |= set(re.findall(r"\b(bf_[a-z_0-9]+)\s*\(", text))
    assert len(declared) >= 20
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert set(bf.binding._SIGNATURES) == declared


def test_config_validation_without_a_device():
    good = bf.make_config(256, 4, 1024, 128, 4, 4, 1, dtype=bf.BF_FP32)
    assert bf.bf_workspace_bytes(good) > 0
    assert bf.bf_param_count(good) == F.n_params_exact(4, 256, 1024) == 3159040
    bad = bf.make_config(256, 4, 1024, 128, 4, 4, 1)
    bad.S_head = 60
    assert bf.bf_workspace_bytes(bad) == 0 and "N_heads" in bf.binding.last_error()
    bad = bf.make_config(256, 4, 1024, 128, 4, 0, 1)
    assert bf.bf_workspace_bytes(bad) == 0
    bad = bf.make_config(256, 4, 1024, 128, 4, 4, 1, dtype=7)
    assert bf.bf_workspace_bytes(bad) == 0
    # checkpointing shrinks the arena; bf16 shrinks activations
    none = bf.make_config(512, 4, 2048, 256, 4, 8, 1, ckpt_mode=bf.BF_CKPT_NONE)
    ck = bf.make_config(512, 4, 2048, 256, 4, 8, 1, ckpt_mode=bf.BF_CKPT_LAYER)
    assert bf.bf_workspace_bytes(ck) < bf.bf_workspace_bytes(none)
    # fully sharded weights: bf16 only; two stage-sized halves instead of every layer's bf16 copy
    assert bf.bf_workspace_bytes(bf.make_config(256, 4, 1024, 128, 4, 4, 1, dtype=bf.BF_FP32, dp_fs=1)) == 0
    assert "dp_fs" in bf.binding.last_error()
    res = bf.make_config(512, 4, 2048, 256, 8, 8, 1, N_loop_min=8)
    fs = bf.make_config(512, 4, 2048, 256, 8, 8, 1, N_loop_min=8, dp_fs=1)
    P = bf.bf_param_count(res)
    assert 0 < bf.bf_workspace_bytes(res) - bf.bf_workspace_bytes(fs) <= 2 * P
    assert bf.bf_workspace_bytes(res) - bf.bf_workspace_bytes(fs) >= 2 * P - 2 * 2 * (P // 8) - 4096
    # input / output layers: two [S_voc, S_hidden] matrices, the position table and the final LayerNorm
    voc = bf.make_config(256, 4, 1024, 128, 4, 4, 1, dtype=bf.BF_FP32, S_voc=1000)
    assert bf.bf_param_count(voc) - bf.bf_param_count(good) == 2 * 1000 * 256 + 128 * 256 + 2 * 256
    assert bf.bf_workspace_bytes(voc) > bf.bf_workspace_bytes(good)
    assert bf.bf_workspace_bytes(bf.make_config(256, 4, 1024, 128, 4, 4, 1, S_voc=-1)) == 0


def test_scratch_sizes_without_a_device():
    """Host arithmetic of the scratch areas the single kernels ask their callers for (include/bf_ops.h)."""
    # one-pass LayerNorm backward: one row of [3][h] per workgroup, at most 256 workgroups of ceil(T / 256)-row runs
    for T, h in [(1, 8), (255, 64), (256, 64), (257, 64), (2048, 8192), (8192, 8192), (3000, 100)]:
        run = -(-T // 256)
        assert bf.bf_op_layernorm_bwd_part_elems(T, h) == 3 * h * -(-T // run)
    assert bf.bf_op_layernorm_bwd_part_elems(0, 64) == 0 and bf.bf_op_layernorm_bwd_part_elems(64, 0) == 0
    # attention backward with the QKV bias gradient: a row of [S_hidden] per sequence and query block (256 queries when
    # S_seq is a multiple of 256, else 128) and a row of [2 S_hidden] per sequence and block of 128 keys; nothing for
    # shapes the matrix-core kernels do not serve
    for S_mb, S_seq, a, d in [(1, 2048, 64, 128), (4, 2048, 64, 128), (1, 384, 2, 128), (2, 128, 4, 64), (1, 1024, 16, 128)]:
        h = a * d
        q_rows = S_mb * (S_seq // (256 if S_seq % 256 == 0 else 128))
        assert bf.bf_op_attention_bwd_part_elems(S_mb, S_seq, a, d) == q_rows * h + S_mb * (S_seq // 128) * 2 * h
        assert bf.bf_op_attention_uses_mfma(S_seq, d)
    for S_mb, S_seq, a, d in [(1, 100, 3, 40), (1, 64, 4, 64), (1, 2048, 64, 96), (0, 2048, 64, 128), (1, 2048, 0, 128)]:
        assert bf.bf_op_attention_bwd_part_elems(S_mb, S_seq, a, d) == 0


@pytest.mark.parametrize("kind,code", [("BF", bf.BF_SCHED_BF), ("DF", bf.BF_SCHED_DF)])
def test_schedule_trace_matches_oracle_and_closed_forms(kind, code):
    for N_PP in (1, 2, 4, 8):
        for N_loop in (1, 2, 4):
            for N_mb in (N_PP, 2 * N_PP, 4 * N_PP):
                for t_fwd, t_bwd in ((1, 2), (1, 3)):
                    ref = S.simulate(kind, N_PP, N_loop, N_mb, t_fwd, t_bwd)
                    for rank in range(N_PP):
                        ev, st = bf.bf_schedule_trace(code, N_PP, N_loop, N_mb, rank, t_fwd, t_bwd)
                        assert [(o, j, m) for o, j, m, _ in ev] == S.device_order(kind, N_PP, N_loop, N_mb, rank)
                        assert Fraction(st.bubble_num, st.bubble_den) == F.bubble(N_PP, N_mb, N_loop) == ref["bubble"]
                        assert st.makespan == ref["makespan"] and st.busy == ref["busy"]
                        assert st.peak_live == ref["peak_live"][rank]
                        if kind == "BF":
                            # Eq. mem_ckpt first factor with one layer per stage
                            assert st.peak_live == F.ckpt_count("BF", N_mb, N_PP * N_loop, N_PP)
                        assert ev[-1][3] == 0 and max(e[3] for e in ev) == st.peak_live


def test_schedule_trace_fig4_and_errors():
    _, st = bf.bf_schedule_trace(bf.BF_SCHED_BF, 4, 1, 8, 0)
    assert (st.bubble_num, st.bubble_den) == (3, 8)
    _, st = bf.bf_schedule_trace(bf.BF_SCHED_BF, 4, 4, 8, 0)
    assert (st.bubble_num, st.bubble_den) == (3, 32)
    for args in [(bf.BF_SCHED_BF, 4, 2, 3, 0), (bf.BF_SCHED_DF, 4, 2, 6, 0), (5, 1, 1, 1, 0), (0, 2, 1, 2, 2),
                 (0, 0, 1, 1, 0)]:
        with pytest.raises(bf.BfError) as e:
            bf.bf_schedule_trace(*args)
        assert e.value.status == bf.BF_EINVAL


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2211_05953_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, os.path.join(dirpath, f)


def test_two_chain_configurations_are_validated_without_a_device():
    """mb_chains = 2 goes with the fused weight gradient, resident weights, no launch
    queue and no input / output layers; anything else is refused when the workspace is sized."""
    import paper_2211_05953_amd as bf
    ok = dict(dtype=bf.BF_BF16, fuse_wgrad=1, mb_chains=2)
    base = bf.bf_workspace_bytes(bf.make_config(256, 2, 1024, 128, 4, 4, 1, dtype=bf.BF_BF16, fuse_wgrad=1))
    assert bf.bf_workspace_bytes(bf.make_config(256, 2, 1024, 128, 4, 4, 1, **ok)) > base > 0
    for bad in (dict(fuse_wgrad=0), dict(dp_fs=1, N_loop_min=4), dict(queue_depth=4),
                dict(S_voc=512), dict(mb_chains=3), dict(mb_chains=-1)):
        assert bf.bf_workspace_bytes(bf.make_config(256, 2, 1024, 128, 4, 4, 1, **{**ok, **bad})) == 0, bad
        assert "mb_chains" in bf.binding.last_error(), bad
    assert bf.bf_workspace_bytes(bf.make_config(256, 2, 1024, 128, 4, 4, 1, ckpt_mode=bf.BF_CKPT_LAYER, **ok)) > 0


def test_tile_choice_invariants_without_a_device():
    """The tile a product runs on divides its output, the 192-column tile appears only for the layouts and epilogues
    that have it and only where it gives fewer rounds of the grid than 256 columns, and shapes outside the matrix-core
    kernel's reach report none."""
    import itertools
    import paper_2211_05953_amd as bf
    one_output = {(bf.BF_NT, bf.BF_EPI_NONE), (bf.BF_NN, bf.BF_EPI_NONE), (bf.BF_NN, bf.BF_EPI_BIAS), (bf.BF_NN, bf.BF_EPI_BIAS_RES)}
    combos = [(bf.BF_NN, e) for e in (bf.BF_EPI_NONE, bf.BF_EPI_BIAS, bf.BF_EPI_BIAS_RES, bf.BF_EPI_BIAS_GELU)] + \
             [(bf.BF_NT, bf.BF_EPI_NONE), (bf.BF_NT, bf.BF_EPI_GELU_BWD), (bf.BF_TN, bf.BF_EPI_ACCUM)]
    seen = set()
    for (layout, epi), M, N in itertools.product(combos, (128, 256, 1024, 2048, 8192), (128, 384, 768, 2048, 6144, 8192, 18432, 24576, 50304)):
        t = bf.bf_op_gemm_tile(layout, epi, M, N, 256)
        assert t in ((256, 256), (256, 128), (128, 128), (256, 192)), (layout, epi, M, N, t)
        assert M % t[0] == 0 and N % t[1] == 0
        if t == (256, 192):
            assert (layout, epi) in one_output
            rounds = lambda bn: -(-((M // 256) * (N // bn)) // 256)
            assert N % 256 or rounds(192) * 192 < rounds(256) * 256 * 1.2, (M, N)
        seen.add(t)
    assert seen == {(256, 256), (256, 128), (128, 128), (256, 192)}
    assert bf.bf_op_gemm_tile(bf.BF_NN, bf.BF_EPI_NONE, 100, 128, 64) is None      # rows not a multiple of 128
    assert bf.bf_op_gemm_tile(bf.BF_NN, bf.BF_EPI_NONE, 128, 128, 96) is None      # K not a multiple of 64
    assert bf.bf_op_gemm_tile(bf.BF_TN, bf.BF_EPI_NONE, 128, 128, 64) is None      # the weight-gradient layout stores fp32
