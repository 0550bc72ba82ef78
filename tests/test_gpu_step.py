"""GPU parity of the whole training step (bf_run_step) against the CPU oracle, in both
orders, plus the order invariants: BF == DF bitwise, event trace and checkpoint counts
equal to the oracle's and to Eq. mem_ckpt."""
import numpy as np
import pytest
import torch

import bf_inputs
import paper_2211_05953_amd as bf
from oracle import formulas as F
from oracle import stack as K
from util import TOL, TOL_RMS, rel_err, rms_err, to_dev, to_host

pytestmark = pytest.mark.gpu


def _run_gpu(cfg, params, x, dy, schedule, N_loop, N_mb, S_mb, apply_optimizer=0, steps=1):
    b16 = cfg.dtype == bf.BF_BF16
    st = bf.Stack(cfg)
    for l, p in enumerate(params):
        for name, tid in bf.TENSOR_IDS.items():
            st.bf_set_params(l, tid, p[name].reshape(-1))
    dX, dDY = to_dev(x, b16), to_dev(dy, b16)
    y, dx = torch.empty_like(dX), torch.empty_like(dX)
    for _ in range(steps):
        rep = st.bf_run_step(schedule, N_loop, N_mb, S_mb, dX, dDY, y, dx, apply_optimizer=apply_optimizer)
    torch.cuda.synchronize()
    out = dict(y=to_host(y), dx=to_host(dx), report=rep, trace=st.bf_get_trace(),
               grads=[{n: st.bf_get_grads(l, t) for n, t in bf.TENSOR_IDS.items()} for l in range(cfg.N_layers)],
               params=[{n: st.bf_get_params(l, t) for n, t in bf.TENSOR_IDS.items()} for l in range(cfg.N_layers)],
               m=[{n: st.bf_get_moments(l, t, 0) for n, t in bf.TENSOR_IDS.items()} for l in range(cfg.N_layers)],
               v=[{n: st.bf_get_moments(l, t, 1) for n, t in bf.TENSOR_IDS.items()} for l in range(cfg.N_layers)])
    st.close()
    return out


def _oracle(params, x, dy, schedule, N_loop, N_heads, causal=True, adam=None, steps=1):
    p64 = [{k: v.astype(np.float64) for k, v in p.items()} for p in params]
    state = None
    for t in range(1, steps + 1):
        a = dict(adam, t=t) if adam else None
        r = K.run_step(p64, x.astype(np.float64), dy.astype(np.float64), schedule, N_loop, N_heads, causal=causal,
                       adam=a, adam_state=state)
        p64, state = r["new_params"], r["new_adam_state"]
    return r


def _compare(gpu, ref, tol, N_layers):
    tol_rms = TOL_RMS["fp32" if tol == TOL["fp32"] else "bf16"]
    assert rel_err(gpu["y"], ref["y"]) <= tol
    assert rel_err(gpu["dx"], ref["dx"]) <= tol
    assert rms_err(gpu["dx"], ref["dx"]) <= tol_rms
    for l in range(N_layers):
        for name in bf.TENSOR_IDS:
            e = rel_err(gpu["grads"][l][name], ref["grads"][l][name].reshape(-1))
            assert e <= tol, (l, name, e)
            e = rms_err(gpu["grads"][l][name], ref["grads"][l][name].reshape(-1))
            assert e <= tol_rms, (l, name, "rms", e)


CASES = [
    # mode, dtype, ckpt, kernels, L, N_loop, h, a, f, S_seq, S_mb, N_mb
    ("fp32", bf.BF_FP32, bf.BF_CKPT_NONE, bf.BF_KERNELS_AUTO, 4, 2, 256, 4, 1024, 128, 1, 4),    # configs[0]
    ("fp32", bf.BF_FP32, bf.BF_CKPT_LAYER, bf.BF_KERNELS_AUTO, 4, 4, 256, 4, 1024, 128, 1, 4),
    ("fp32", bf.BF_FP32, bf.BF_CKPT_NONE, bf.BF_KERNELS_AUTO, 2, 1, 72, 3, 200, 50, 2, 3),       # ragged everything
    ("bf16", bf.BF_BF16, bf.BF_CKPT_NONE, bf.BF_KERNELS_PLAIN, 4, 2, 256, 4, 1024, 128, 1, 4),
    ("bf16", bf.BF_BF16, bf.BF_CKPT_NONE, bf.BF_KERNELS_AUTO, 4, 2, 256, 2, 1024, 256, 1, 4),
    ("bf16", bf.BF_BF16, bf.BF_CKPT_LAYER, bf.BF_KERNELS_AUTO, 2, 2, 512, 4, 2048, 256, 2, 2),
]


@pytest.mark.parametrize("mode,dtype,ckpt,kernels,Lyr,N_loop,h,a,f,S_seq,S_mb,N_mb", CASES)
def test_step_matches_oracle_in_both_orders(mode, dtype, ckpt, kernels, Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb):
    b16 = dtype == bf.BF_BF16
    params = bf_inputs.make_params(11, Lyr, h, f, bf16=b16)
    x, dy = bf_inputs.make_batch(11, N_mb, S_mb, S_seq, h, bf16=b16)
    cfg = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=dtype, ckpt_mode=ckpt, kernels=kernels)
    ref = _oracle(params, x, dy, K.SCHED_BF, N_loop, a)
    g_bf = _run_gpu(cfg, params, x, dy, bf.BF_SCHED_BF, N_loop, N_mb, S_mb)
    g_df = _run_gpu(cfg, params, x, dy, bf.BF_SCHED_DF, N_loop, N_mb, S_mb)
    _compare(g_bf, ref, TOL[mode], Lyr)
    _compare(g_df, ref, TOL[mode], Lyr)
    # the two orders add the same numbers in the same sequence
    assert np.array_equal(g_bf["y"], g_df["y"]) and np.array_equal(g_bf["dx"], g_df["dx"])
    for l in range(Lyr):
        for name in bf.TENSOR_IDS:
            assert np.array_equal(g_bf["grads"][l][name], g_df["grads"][l][name]), (l, name)
    # integer trace and checkpoint counts: the oracle's, and Eq. mem_ckpt at N_PP = 1
    assert g_bf["trace"] == [tuple(e) for e in ref["trace"]]
    assert g_bf["report"].peak_ckpt_count == F.ckpt_count("BF", N_mb, Lyr, 1) == ref["peak_ckpt"]
    assert g_df["report"].peak_ckpt_count == F.ckpt_count("DF", N_mb, Lyr, 1)
    assert [e[:3] for e in g_df["trace"]] == K.event_order(K.SCHED_DF, N_loop, N_mb)
    assert g_bf["report"].peak_ckpt_bytes == int(F.ckpt_count("BF", N_mb, Lyr, 1) * S_mb * S_seq * h * (2 if b16 else 4))
    if f == 4 * h:   # Eq. compute assumes S_mlp = 4 S_hidden
        assert g_bf["report"].flops_paper == float(F.c_gpu(N_mb, S_mb, Lyr, h, S_seq))


@pytest.mark.parametrize("mode,dtype,Lyr,N_loop,h,a,f,S_seq,S_mb,N_mb", [
    ("fp32", bf.BF_FP32, 4, 2, 256, 4, 1024, 128, 1, 4),
    ("fp32", bf.BF_FP32, 3, 1, 72, 3, 200, 50, 2, 3),
    ("bf16", bf.BF_BF16, 4, 2, 256, 2, 1024, 256, 1, 4),
    ("bf16", bf.BF_BF16, 4, 4, 512, 4, 2048, 128, 2, 3),
])
@pytest.mark.parametrize("ckpt,loop_hint", [(bf.BF_CKPT_NONE, 0), (bf.BF_CKPT_LAYER, 0), (bf.BF_CKPT_LAYER, -1), (bf.BF_CKPT_NONE, -1)])
def test_fused_weight_gradient_in_breadth_first_order(mode, dtype, Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb, ckpt, loop_hint):
    """fuse_wgrad = 1: one weight-gradient product per stage over all micro-batches (BF only).
    Same sum, one long contraction: equal to the oracle within the tolerance, equal to the
    per-micro-batch accumulation up to fp32 rounding; DF ignores the flag."""
    b16 = dtype == bf.BF_BF16
    params = bf_inputs.make_params(13, Lyr, h, f, bf16=b16)
    x, dy = bf_inputs.make_batch(13, N_mb, S_mb, S_seq, h, bf16=b16)
    hint = N_loop if loop_hint < 0 else 0     # per-stage buffers sized exactly for this N_loop, or for any
    fused = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=dtype, fuse_wgrad=1, ckpt_mode=ckpt, N_loop_min=hint)
    plain = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=dtype, fuse_wgrad=0, ckpt_mode=ckpt)
    if hint:
        assert bf.bf_workspace_bytes(fused) <= bf.bf_workspace_bytes(
            bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=dtype, fuse_wgrad=1, ckpt_mode=ckpt))
    ref = _oracle(params, x, dy, K.SCHED_BF, N_loop, a)
    g_f = _run_gpu(fused, params, x, dy, bf.BF_SCHED_BF, N_loop, N_mb, S_mb)
    g_p = _run_gpu(plain, params, x, dy, bf.BF_SCHED_BF, N_loop, N_mb, S_mb)
    g_df = _run_gpu(fused, params, x, dy, bf.BF_SCHED_DF, N_loop, N_mb, S_mb)
    _compare(g_f, ref, TOL[mode], Lyr)
    assert np.array_equal(g_f["y"], g_p["y"]) and np.array_equal(g_f["dx"], g_p["dx"])
    for l in range(Lyr):
        for name in bf.TENSOR_IDS:
            assert rel_err(g_f["grads"][l][name], g_p["grads"][l][name]) <= 2e-6, (l, name)
            assert np.array_equal(g_df["grads"][l][name], g_p["grads"][l][name]), (l, name)
    assert g_f["trace"] == g_p["trace"]
    if hint and N_loop % 2 == 0:
        # stages twice as large as the buffers were sized for: the step accumulates per micro-batch instead
        g_big = _run_gpu(fused, params, x, dy, bf.BF_SCHED_BF, N_loop // 2, N_mb, S_mb)
        for l in range(Lyr):
            for name in bf.TENSOR_IDS:
                assert np.array_equal(g_big["grads"][l][name], g_p["grads"][l][name]), (l, name)


@pytest.mark.parametrize("mode,dtype", [("fp32", bf.BF_FP32), ("bf16", bf.BF_BF16)])
@pytest.mark.parametrize("schedule", [bf.BF_SCHED_BF, bf.BF_SCHED_DF])
def test_two_optimizer_steps(mode, dtype, schedule):
    b16 = dtype == bf.BF_BF16
    Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb = 2, 2, 128, 2, 512, 64, 1, 3
    params = bf_inputs.make_params(12, Lyr, h, f, bf16=b16)
    x, dy = bf_inputs.make_batch(12, N_mb, S_mb, S_seq, h, bf16=b16)
    # the C ABI carries the constants as fp32: the oracle gets those exact values
    adam = {k: float(np.float32(v)) for k, v in dict(lr=1e-3, beta1=0.9, beta2=0.999, adam_eps=1e-8, weight_decay=0.0).items()}
    cfg = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=dtype, lr=adam["lr"])
    for steps in (1, 2):
        gpu = _run_gpu(cfg, params, x, dy, schedule, N_loop, N_mb, S_mb, apply_optimizer=1, steps=steps)
        ref = _oracle(params, x, dy, schedule, N_loop, a, adam=adam, steps=steps)
        tol = TOL[mode] * (1 if steps == 1 else 20)   # step 2 sees weights moved by +-lr where a gradient sign is ambiguous
        for l in range(Lyr):
            for name in bf.TENSOR_IDS:
                g_ref = ref["grads"][l][name].reshape(-1)
                m_ref, v_ref = (t.reshape(-1) for t in ref["new_adam_state"][l][name])
                assert rel_err(gpu["grads"][l][name], g_ref) <= tol, (steps, l, name)
                assert rel_err(gpu["m"][l][name], m_ref) <= tol, (steps, l, name)
                assert rel_err(gpu["v"][l][name], v_ref) <= 2 * tol, (steps, l, name)
                if steps == 1:
                    # where the gradient is well away from zero the first update is -lr * sign(g)
                    big = np.abs(g_ref) > 1e-2 * np.abs(g_ref).max()
                    upd = (gpu["params"][l][name].astype(np.float64) - params[l][name].reshape(-1))[big]
                    upd_ref = (ref["new_params"][l][name].reshape(-1) - params[l][name].reshape(-1))[big]
                    assert np.abs(upd - upd_ref).max() <= 1e-3 * adam["lr"] + 2e-7 * np.abs(params[l][name]).max()


@pytest.mark.parametrize("mode,dtype,Lyr,N_loop,h,a,f,S_seq,S_mb,N_mb", [
    ("fp32", bf.BF_FP32, 3, 3, 72, 3, 200, 50, 2, 3),          # generic kernels
    ("bf16", bf.BF_BF16, 4, 2, 256, 2, 1024, 256, 1, 4),       # MFMA kernels
    ("bf16", bf.BF_BF16, 2, 1, 512, 4, 2048, 128, 2, 3),
])
def test_optimizer_step_after_the_fused_weight_gradient(mode, dtype, Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb):
    """Breadth-first with fuse_wgrad = 1 and the optimizer on (the configuration the benchmark times),
    with weight decay: every parameter moves exactly once per step, the main-grads stay readable, and
    the result is the oracle's (Sec. 4.2, per-stage update)."""
    b16 = dtype == bf.BF_BF16
    params = bf_inputs.make_params(17, Lyr, h, f, bf16=b16)
    x, dy = bf_inputs.make_batch(17, N_mb, S_mb, S_seq, h, bf16=b16)
    adam = {k: float(np.float32(v)) for k, v in dict(lr=1e-3, beta1=0.9, beta2=0.999, adam_eps=1e-8, weight_decay=0.01).items()}
    mk = lambda fuse: bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=dtype, lr=adam["lr"],
                                     weight_decay=adam["weight_decay"], fuse_wgrad=fuse)
    for steps in (1, 2):
        fused = _run_gpu(mk(1), params, x, dy, bf.BF_SCHED_BF, N_loop, N_mb, S_mb, apply_optimizer=1, steps=steps)
        plain = _run_gpu(mk(0), params, x, dy, bf.BF_SCHED_BF, N_loop, N_mb, S_mb, apply_optimizer=1, steps=steps)
        ref = _oracle(params, x, dy, K.SCHED_BF, N_loop, a, adam=adam, steps=steps)
        tol = TOL[mode] * (1 if steps == 1 else 20)
        for l in range(Lyr):
            for name in bf.TENSOR_IDS:
                g_ref = ref["grads"][l][name].reshape(-1)
                m_ref, v_ref = (t.reshape(-1) for t in ref["new_adam_state"][l][name])
                assert rel_err(fused["grads"][l][name], g_ref) <= tol, (steps, l, name)
                assert rel_err(fused["m"][l][name], m_ref) <= tol, (steps, l, name)
                assert rel_err(fused["v"][l][name], v_ref) <= 2 * tol, (steps, l, name)
                if steps == 1:
                    # same gradients up to fp32 summation order: same moments, same -lr * sign(g) moves
                    assert rel_err(fused["m"][l][name], plain["m"][l][name]) <= 1e-5, (l, name)
                    assert rel_err(fused["v"][l][name], plain["v"][l][name]) <= 2e-5, (l, name)
                    big = np.abs(g_ref) > 1e-2 * np.abs(g_ref).max()
                    w0 = params[l][name].reshape(-1)
                    upd = (fused["params"][l][name].astype(np.float64) - w0)[big]
                    upd_ref = (ref["new_params"][l][name].reshape(-1) - w0)[big]
                    assert np.abs(upd - upd_ref).max() <= 1e-3 * adam["lr"] + 2e-7 * np.abs(w0).max(), (l, name)
                    # no parameter was skipped or stepped twice
                    moved = np.abs(fused["params"][l][name].astype(np.float64) - w0)[big]
                    assert moved.min() > 0.5 * adam["lr"] and moved.max() < 1.5 * adam["lr"], (l, name)


MATRICES = ("w_qkv", "w_o", "w_fc1", "w_fc2")


def _a_product_splits_its_contraction(dtype, T, h, f):
    """Whether one of a layer's forward / dgrad products runs as two slices of K in a one-chain step."""
    if dtype != bf.BF_BF16:
        return False
    shapes = [(bf.BF_NN, bf.BF_EPI_BIAS, T, 3 * h, h), (bf.BF_NN, bf.BF_EPI_BIAS_RES, T, h, h), (bf.BF_NN, bf.BF_EPI_BIAS_RES, T, h, f),
              (bf.BF_NT, bf.BF_EPI_NONE, T, h, f), (bf.BF_NT, bf.BF_EPI_NONE, T, h, h), (bf.BF_NT, bf.BF_EPI_NONE, T, h, 3 * h)]
    return any(bf.bf_op_gemm_splitk_slices(*sh) > 1 for sh in shapes)


@pytest.mark.parametrize("mode,dtype,Lyr,N_loop,h,a,f,S_seq,S_mb,N_mb", [
    ("fp32", bf.BF_FP32, 3, 3, 72, 3, 200, 50, 2, 3),          # generic kernels, odd N_mb
    ("fp32", bf.BF_FP32, 4, 2, 256, 4, 1024, 128, 1, 2),       # one micro-batch per chain
    ("bf16", bf.BF_BF16, 4, 2, 256, 2, 1024, 256, 1, 4),       # MFMA kernels
    ("bf16", bf.BF_BF16, 4, 4, 512, 4, 2048, 128, 2, 5),
    ("bf16", bf.BF_BF16, 4, 1, 256, 2, 1024, 256, 1, 3),       # one stage
])
@pytest.mark.parametrize("ckpt", [bf.BF_CKPT_NONE, bf.BF_CKPT_LAYER])
def test_two_chains_of_micro_batches_side_by_side(mode, dtype, Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb, ckpt):
    """mb_chains = 2: the micro-batches of a breadth-first step run on two streams (Sec. 4.2: within a stage
    they do not depend on each other), with stored activations or with per-layer checkpoints (then each chain
    recomputes into a record of its own).  Outputs and weight-matrix gradients are those of the one-chain step
    bit for bit (unless that step splits a contraction, which a two-chain step does not: then to the rounding of
    the outputs), the bias / LayerNorm gradients are two partial sums added in a fixed order (equal up to fp32
    rounding, the same bits on every run), and everything matches the oracle."""
    b16 = dtype == bf.BF_BF16
    params = bf_inputs.make_params(19, Lyr, h, f, bf16=b16)
    x, dy = bf_inputs.make_batch(19, N_mb, S_mb, S_seq, h, bf16=b16)
    mk = lambda chains: bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=dtype, fuse_wgrad=1, mb_chains=chains,
                                       ckpt_mode=ckpt)
    assert bf.bf_workspace_bytes(mk(2)) > bf.bf_workspace_bytes(mk(1)) == bf.bf_workspace_bytes(mk(0))
    ref = _oracle(params, x, dy, K.SCHED_BF, N_loop, a)
    two = _run_gpu(mk(2), params, x, dy, bf.BF_SCHED_BF, N_loop, N_mb, S_mb)
    again = _run_gpu(mk(2), params, x, dy, bf.BF_SCHED_BF, N_loop, N_mb, S_mb)
    one = _run_gpu(mk(1), params, x, dy, bf.BF_SCHED_BF, N_loop, N_mb, S_mb)
    assert two["report"].mb_chains == 2 and one["report"].mb_chains == 1
    _compare(two, ref, TOL[mode], Lyr)
    split = _a_product_splits_its_contraction(dtype, S_mb * S_seq, h, f)
    assert split == (h == 512)   # the cases cover both
    if split:
        assert rel_err(two["y"], one["y"]) <= TOL[mode] and rel_err(two["dx"], one["dx"]) <= TOL[mode]
    else:
        assert np.array_equal(two["y"], one["y"]) and np.array_equal(two["dx"], one["dx"])
    assert np.array_equal(two["y"], again["y"]) and np.array_equal(two["dx"], again["dx"])
    for l in range(Lyr):
        for name in bf.TENSOR_IDS:
            assert np.array_equal(two["grads"][l][name], again["grads"][l][name]), (l, name)
            if split:
                assert rel_err(two["grads"][l][name], one["grads"][l][name]) <= TOL[mode], (l, name)
            elif name in MATRICES:
                assert np.array_equal(two["grads"][l][name], one["grads"][l][name]), (l, name)
            else:
                assert rel_err(two["grads"][l][name], one["grads"][l][name]) <= 2e-6, (l, name)
    assert two["trace"] == one["trace"] == [tuple(e) for e in ref["trace"]]
    assert two["report"].peak_ckpt_count == one["report"].peak_ckpt_count
    # depth-first order has one micro-batch in flight per stage visit: the flag changes nothing there
    df2 = _run_gpu(mk(2), params, x, dy, bf.BF_SCHED_DF, N_loop, N_mb, S_mb)
    df1 = _run_gpu(mk(1), params, x, dy, bf.BF_SCHED_DF, N_loop, N_mb, S_mb)
    assert df2["report"].mb_chains == 1
    for l in range(Lyr):
        for name in bf.TENSOR_IDS:
            assert np.array_equal(df2["grads"][l][name], df1["grads"][l][name]), (l, name)
    # a single micro-batch leaves nothing to run beside it
    solo = _run_gpu(mk(2), params, x[:1], dy[:1], bf.BF_SCHED_BF, N_loop, 1, S_mb)
    solo1 = _run_gpu(mk(1), params, x[:1], dy[:1], bf.BF_SCHED_BF, N_loop, 1, S_mb)
    assert solo["report"].mb_chains == 1
    for l in range(Lyr):
        for name in bf.TENSOR_IDS:
            assert np.array_equal(solo["grads"][l][name], solo1["grads"][l][name]), (l, name)


@pytest.mark.parametrize("mode,dtype,Lyr,N_loop,h,a,f,S_seq,S_mb,N_mb", [
    ("fp32", bf.BF_FP32, 3, 3, 72, 3, 200, 50, 2, 3),
    ("bf16", bf.BF_BF16, 4, 2, 256, 2, 1024, 256, 1, 4),
])
def test_optimizer_steps_with_two_chains(mode, dtype, Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb):
    """Two steps with the per-stage update between the chains' work: the update of a stage runs while the other
    chain is already in the stage below, and the next step's forward must see every updated weight."""
    b16 = dtype == bf.BF_BF16
    params = bf_inputs.make_params(23, Lyr, h, f, bf16=b16)
    x, dy = bf_inputs.make_batch(23, N_mb, S_mb, S_seq, h, bf16=b16)
    adam = {k: float(np.float32(v)) for k, v in dict(lr=1e-3, beta1=0.9, beta2=0.999, adam_eps=1e-8, weight_decay=0.01).items()}
    mk = lambda chains: bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=dtype, lr=adam["lr"],
                                       weight_decay=adam["weight_decay"], fuse_wgrad=1, mb_chains=chains)
    for steps in (1, 2):
        two = _run_gpu(mk(2), params, x, dy, bf.BF_SCHED_BF, N_loop, N_mb, S_mb, apply_optimizer=1, steps=steps)
        again = _run_gpu(mk(2), params, x, dy, bf.BF_SCHED_BF, N_loop, N_mb, S_mb, apply_optimizer=1, steps=steps)
        one = _run_gpu(mk(1), params, x, dy, bf.BF_SCHED_BF, N_loop, N_mb, S_mb, apply_optimizer=1, steps=steps)
        ref = _oracle(params, x, dy, K.SCHED_BF, N_loop, a, adam=adam, steps=steps)
        assert two["report"].mb_chains == 2
        tol = TOL[mode] * (1 if steps == 1 else 20)
        for l in range(Lyr):
            for name in bf.TENSOR_IDS:
                g_ref = ref["grads"][l][name].reshape(-1)
                m_ref, v_ref = (t.reshape(-1) for t in ref["new_adam_state"][l][name])
                assert rel_err(two["grads"][l][name], g_ref) <= tol, (steps, l, name)
                assert rel_err(two["m"][l][name], m_ref) <= tol, (steps, l, name)
                assert rel_err(two["v"][l][name], v_ref) <= 2 * tol, (steps, l, name)
                for k in ("grads", "params", "m", "v"):
                    assert np.array_equal(two[k][l][name], again[k][l][name]), (steps, k, l, name)
                if steps == 1 and name in MATRICES:
                    for k in ("grads", "params", "m", "v"):
                        assert np.array_equal(two[k][l][name], one[k][l][name]), (k, l, name)
                elif steps == 1:
                    assert rel_err(two["m"][l][name], one["m"][l][name]) <= 1e-5, (l, name)


def test_run_step_argument_errors():
    cfg = bf.make_config(64, 2, 256, 16, 4, 2, 1, dtype=bf.BF_FP32)
    st = bf.Stack(cfg)
    t = torch.zeros(2, 1, 16, 64, device="cuda")
    with pytest.raises(bf.BfError) as e:
        st.bf_get_grads(0, 2)
    assert e.value.status == bf.BF_ESTATE
    for kw in [dict(N_loop=3), dict(N_mb=3), dict(S_mb=2), dict(schedule=5), dict(x=None)]:
        args = dict(schedule=0, N_loop=2, N_mb=2, S_mb=1, x=t, dy=t)
        args.update(kw)
        with pytest.raises(bf.BfError) as e:
            st.bf_run_step(**args)
        assert e.value.status == bf.BF_EINVAL
    with pytest.raises(bf.BfError):
        st.bf_set_params(9, 0, np.zeros(64, np.float32))
    with pytest.raises(bf.BfError):
        st.bf_set_params(0, 0, np.zeros(63, np.float32))
    st.close()
    # workspace too small
    import ctypes as C
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    h = C.c_void_p()
    rc = bf.load().bf_create_stack(C.byref(cfg), small.data_ptr(), 1024, None, C.byref(h))
    assert rc == bf.BF_ENOMEM


def _fs_expected(schedule, N_loop, N_mb, resident=()):
    from oracle import schedule as S
    order = S.device_order("BF" if schedule == bf.BF_SCHED_BF else "DF", 1, N_loop, N_mb, 0)
    n, held = S.reconstructions(order, resident=resident)
    return len(S.weight_intervals(order)), n, held


@pytest.mark.parametrize("schedule", [bf.BF_SCHED_BF, bf.BF_SCHED_DF])
@pytest.mark.parametrize("Lyr,N_loop,N_mb,fuse,ckpt", [
    (4, 4, 3, 0, bf.BF_CKPT_NONE), (4, 2, 4, 1, bf.BF_CKPT_NONE), (3, 3, 2, 1, bf.BF_CKPT_LAYER), (2, 1, 3, 0, bf.BF_CKPT_NONE),
    (6, 3, 2, 0, bf.BF_CKPT_LAYER),
])
def test_fully_sharded_double_buffer_is_bit_identical_and_counts_reconstructions(schedule, Lyr, N_loop, N_mb, fuse, ckpt):
    """dp_fs = 1: bf16 stage weights are rebuilt from the fp32 master copy into a two-stage double
    buffer before each interval of use (Sec. 3.1, App. D.1).  Same bf16 weights reach the same kernels:
    outputs, gradients, and two optimizer steps are bit-identical to the resident copy; the interval
    and reconstruction counts are the oracle's (BF 2 N_loop intervals, DF 2 N_loop N_mb, Sec. 4.2)."""
    h, a, f, S_seq, S_mb = 256, 2, 1024, 128, 1
    params = bf_inputs.make_params(19, Lyr, h, f, bf16=True)
    x, dy = bf_inputs.make_batch(19, N_mb, S_mb, S_seq, h, bf16=True)
    mk = lambda fs: bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=bf.BF_BF16, lr=1e-3, fuse_wgrad=fuse,
                                   ckpt_mode=ckpt, N_loop_min=N_loop, dp_fs=fs)
    if N_loop > 2:
        saved = bf.bf_workspace_bytes(mk(0)) - bf.bf_workspace_bytes(mk(1))
        P = bf.bf_param_count(mk(0))
        assert 0 < saved <= 2 * P and saved >= 2 * P * (N_loop - 2) // N_loop - 1024
    for opt in (0, 1):
        g1 = _run_gpu(mk(1), params, x, dy, schedule, N_loop, N_mb, S_mb, apply_optimizer=opt, steps=2)
        g0 = _run_gpu(mk(0), params, x, dy, schedule, N_loop, N_mb, S_mb, apply_optimizer=opt, steps=2)
        assert np.array_equal(g1["y"], g0["y"]) and np.array_equal(g1["dx"], g0["dx"])
        for l in range(Lyr):
            for name in bf.TENSOR_IDS:
                for key in ("grads", "params", "m", "v"):
                    assert np.array_equal(g1[key][l][name], g0[key][l][name]), (opt, key, l, name)
        assert g1["trace"] == g0["trace"]
        if not opt:
            _compare(g1, _oracle(params, x, dy, K.SCHED_BF, N_loop, a), TOL["bf16"], Lyr)
        # second step: without an optimizer step the stages left in the buffer are still good
        _, _, held = _fs_expected(schedule, N_loop, N_mb)
        n_iv, n_rec, _ = _fs_expected(schedule, N_loop, N_mb, resident=() if opt else held)
        r = g1["report"]
        assert (r.n_weight_intervals, r.n_reconstruct) == (n_iv, n_rec)
        assert r.reconstruct_bytes == n_rec * 6 * (bf.bf_param_count(mk(1)) // N_loop)
        assert g0["report"].n_reconstruct == 0 and g0["report"].weight_buffer_bytes == 0
        assert r.weight_buffer_bytes >= 2 * 2 * (bf.bf_param_count(mk(1)) // N_loop)


def test_fully_sharded_argument_errors():
    assert bf.bf_workspace_bytes(bf.make_config(64, 2, 256, 16, 4, 2, 1, dtype=bf.BF_FP32, dp_fs=1)) == 0
    cfg = bf.make_config(128, 2, 512, 64, 4, 2, 1, dtype=bf.BF_BF16, dp_fs=1, N_loop_min=4)
    st = bf.Stack(cfg)
    x = torch.zeros(2, 1, 64, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(bf.BfError, match="dp_fs"):
        st.bf_run_step(bf.BF_SCHED_BF, 2, 2, 1, x, x, None, None)     # stages of 2 layers, halves of 1
    st.bf_run_step(bf.BF_SCHED_BF, 4, 2, 1, x, x, None, None)
    st.close()


def _run_gpu_rank(cfg, params, x, dy, schedule, N_PP, rank, N_loop, N_mb, S_mb):
    b16 = cfg.dtype == bf.BF_BF16
    st = bf.Stack(cfg)
    for l, p in enumerate(params):
        for name, tid in bf.TENSOR_IDS.items():
            st.bf_set_params(l, tid, p[name].reshape(-1))
    dX, dDY = to_dev(x, b16), to_dev(dy, b16)
    y, dx = torch.empty_like(dX), torch.empty_like(dX)
    rep = st.bf_run_rank_step(schedule, N_PP, rank, N_loop, N_mb, S_mb, dX, dDY, y, dx)
    torch.cuda.synchronize()
    out = dict(y=to_host(y), dx=to_host(dx), report=rep, trace=st.bf_get_trace(),
               grads=[{n: st.bf_get_grads(l, t) for n, t in bf.TENSOR_IDS.items()} for l in range(cfg.N_layers)])
    st.close()
    return out


@pytest.mark.parametrize("mode,dtype,N_PP,rank,Lyr,N_loop,h,a,f,S_seq,S_mb,N_mb,fuse,ckpt,fs", [
    ("fp32", bf.BF_FP32, 2, 0, 4, 2, 128, 2, 512, 64, 1, 4, 0, bf.BF_CKPT_NONE, 0),
    ("fp32", bf.BF_FP32, 2, 1, 4, 2, 128, 2, 512, 64, 1, 4, 1, bf.BF_CKPT_LAYER, 0),
    ("fp32", bf.BF_FP32, 4, 2, 3, 3, 72, 3, 200, 50, 2, 8, 0, bf.BF_CKPT_NONE, 0),
    ("fp32", bf.BF_FP32, 1, 0, 4, 2, 128, 2, 512, 64, 1, 3, 1, bf.BF_CKPT_NONE, 0),
    ("bf16", bf.BF_BF16, 4, 3, 4, 2, 256, 2, 1024, 128, 1, 8, 1, bf.BF_CKPT_NONE, 1),
    ("bf16", bf.BF_BF16, 2, 0, 4, 4, 256, 2, 1024, 128, 1, 2, 0, bf.BF_CKPT_LAYER, 1),
])
def test_rank_of_a_deeper_pipeline_matches_oracle(mode, dtype, N_PP, rank, Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb,
                                                  fuse, ckpt, fs):
    """bf_run_rank_step: the rank's order for N_PP > 1 (Sec. 4.2), its stages fed from the caller's
    buffers.  Numbers against the oracle's rank step; the trace is the oracle's device order; the
    peak checkpoint count is the simulator's and respects Eq. mem_ckpt and its depth-first cap."""
    from oracle import schedule as S
    b16 = dtype == bf.BF_BF16
    params = bf_inputs.make_params(23, Lyr, h, f, bf16=b16)
    p64 = [{k: v.astype(np.float64) for k, v in p.items()} for p in params]
    xs, dys = zip(*[bf_inputs.make_batch(100 + l, N_mb, S_mb, S_seq, h, bf16=b16) for l in range(N_loop)])
    x, dy = np.stack(xs), np.stack(dys)
    cfg = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=dtype, fuse_wgrad=fuse, ckpt_mode=ckpt, N_loop_min=N_loop,
                         dp_fs=fs)
    per_stage = Lyr // N_loop
    N_layers_total = Lyr * N_PP
    got = {}
    for kind, code in (("BF", bf.BF_SCHED_BF), ("DF", bf.BF_SCHED_DF)):
        ref = K.run_rank_step(p64, x.astype(np.float64), dy.astype(np.float64), kind, N_PP, rank, N_loop, a)
        g = got[kind] = _run_gpu_rank(cfg, params, x, dy, code, N_PP, rank, N_loop, N_mb, S_mb)
        _compare(g, ref, TOL[mode], Lyr)
        assert g["trace"] == [tuple(e) for e in ref["trace"]]
        assert [e[:3] for e in g["trace"] if e[0] != 2] == S.device_order(kind, N_PP, N_loop, N_mb, rank)
        peak = g["report"].peak_ckpt_count
        assert peak == ref["peak_ckpt"] == S.simulate(kind, N_PP, N_loop, N_mb)["peak_live"][rank] * per_stage
        if kind == "BF":
            assert peak == F.ckpt_count("BF", N_mb, N_layers_total, N_PP)
        else:
            # the cap of Eq. mem_ckpt counts stages of one layer: here a stage is per_stage layers
            assert peak <= F.ckpt_count("DF" if N_loop > 1 else "1F1B", N_mb, N_PP * N_loop, N_PP) * per_stage
        if fs:
            order = S.device_order(kind, N_PP, N_loop, N_mb, rank)
            assert g["report"].n_weight_intervals == len(S.weight_intervals(order))
            assert g["report"].n_reconstruct == S.reconstructions(order)[0]
    # the two orders add each stage's micro-batches in the same sequence (fused: one long contraction instead)
    assert np.array_equal(got["BF"]["y"], got["DF"]["y"]) and np.array_equal(got["BF"]["dx"], got["DF"]["dx"])
    for l in range(Lyr):
        for name in bf.TENSOR_IDS:
            if fuse:
                assert rel_err(got["BF"]["grads"][l][name], got["DF"]["grads"][l][name]) <= 1e-5, (l, name)
            else:
                assert np.array_equal(got["BF"]["grads"][l][name], got["DF"]["grads"][l][name]), (l, name)


@pytest.mark.parametrize("mode,dtype,N_PP,rank,Lyr,N_loop,h,a,f,S_seq,S_mb,N_mb,ckpt", [
    ("fp32", bf.BF_FP32, 2, 1, 4, 2, 128, 2, 512, 64, 1, 4, bf.BF_CKPT_LAYER),
    ("fp32", bf.BF_FP32, 4, 2, 3, 3, 72, 3, 200, 50, 2, 8, bf.BF_CKPT_NONE),
    ("bf16", bf.BF_BF16, 4, 3, 4, 2, 256, 2, 1024, 128, 1, 7, bf.BF_CKPT_NONE),
])
def test_rank_of_a_deeper_pipeline_with_two_chains(mode, dtype, N_PP, rank, Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb, ckpt):
    """A rank's breadth-first order (Sec. 4.2) also has every micro-batch of a stage in a row, so the two chains
    of mb_chains = 2 apply to bf_run_rank_step as well: the oracle's numbers and trace, outputs and
    weight-matrix gradients those of the one-chain step bit for bit."""
    b16 = dtype == bf.BF_BF16
    params = bf_inputs.make_params(31, Lyr, h, f, bf16=b16)
    p64 = [{k: v.astype(np.float64) for k, v in p.items()} for p in params]
    xs, dys = zip(*[bf_inputs.make_batch(200 + l, N_mb, S_mb, S_seq, h, bf16=b16) for l in range(N_loop)])
    x, dy = np.stack(xs), np.stack(dys)
    mk = lambda chains: bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=dtype, fuse_wgrad=1, ckpt_mode=ckpt,
                                       N_loop_min=N_loop, mb_chains=chains)
    ref = K.run_rank_step(p64, x.astype(np.float64), dy.astype(np.float64), "BF", N_PP, rank, N_loop, a)
    two = _run_gpu_rank(mk(2), params, x, dy, bf.BF_SCHED_BF, N_PP, rank, N_loop, N_mb, S_mb)
    one = _run_gpu_rank(mk(1), params, x, dy, bf.BF_SCHED_BF, N_PP, rank, N_loop, N_mb, S_mb)
    assert two["report"].mb_chains == 2 and one["report"].mb_chains == 1
    _compare(two, ref, TOL[mode], Lyr)
    assert two["trace"] == one["trace"] == [tuple(e) for e in ref["trace"]]
    assert not _a_product_splits_its_contraction(dtype, S_mb * S_seq, h, f)
    assert np.array_equal(two["y"], one["y"]) and np.array_equal(two["dx"], one["dx"])
    for l in range(Lyr):
        for name in bf.TENSOR_IDS:
            if name in MATRICES:
                assert np.array_equal(two["grads"][l][name], one["grads"][l][name]), (l, name)
            else:
                assert rel_err(two["grads"][l][name], one["grads"][l][name]) <= 2e-6, (l, name)
    # the rank's depth-first order has one micro-batch of a stage at a time
    df = _run_gpu_rank(mk(2), params, x, dy, bf.BF_SCHED_DF, N_PP, rank, N_loop, N_mb if N_mb % N_PP == 0 else N_PP, S_mb) \
        if N_mb % N_PP == 0 else None
    assert df is None or df["report"].mb_chains == 1


def test_rank_step_argument_errors():
    cfg = bf.make_config(64, 2, 256, 16, 4, 4, 1, dtype=bf.BF_FP32)
    st = bf.Stack(cfg)
    x = torch.zeros(2, 4, 1, 16, 64, device="cuda")
    with pytest.raises(bf.BfError):
        st.bf_run_rank_step(bf.BF_SCHED_BF, 2, 2, 2, 4, 1, x, x)      # rank outside 0..N_PP-1
    with pytest.raises(bf.BfError):
        st.bf_run_rank_step(bf.BF_SCHED_DF, 2, 0, 2, 3, 1, x, x)      # depth-first needs N_mb % N_PP == 0
    with pytest.raises(bf.BfError):
        st.bf_run_rank_step(bf.BF_SCHED_BF, 4, 0, 2, 2, 1, x, x)      # breadth-first needs N_mb >= N_PP
    st.bf_run_rank_step(bf.BF_SCHED_BF, 2, 1, 2, 4, 1, x, x)
    st.close()


def _random_cases(n, seed):
    """Seeded draw of step configurations: ragged fp32 shapes on the generic kernels, tile-aligned
    bf16 shapes on the MFMA kernels, every flag of the configuration that changes the path."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        b16 = bool(i % 2)
        if b16:
            d = int(rng.choice([64, 128]))
            a = int(rng.choice([1, 2, 4]))
            h = a * d
            if h % 128:
                a, h = 2, 2 * d
            f = int(rng.choice([2, 4])) * h
            S_seq = int(rng.choice([128, 256, 384]))
            S_mb = int(rng.choice([1, 2]))
        else:
            a = int(rng.choice([1, 2, 3]))
            h = a * int(rng.choice([8, 20, 24]))
            f = int(rng.integers(h, 4 * h))
            S_seq = int(rng.integers(5, 70))
            S_mb = int(rng.choice([1, 2, 3]))
        N_loop = int(rng.choice([1, 2, 3, 4]))
        Lyr = N_loop * int(rng.choice([1, 2]))
        N_mb = int(rng.integers(1, 6))
        cases.append(dict(b16=b16, h=h, a=a, f=f, S_seq=S_seq, S_mb=S_mb, Lyr=Lyr, N_loop=N_loop, N_mb=N_mb,
                          ckpt=int(rng.choice([bf.BF_CKPT_NONE, bf.BF_CKPT_LAYER])), fuse=int(rng.integers(0, 2)),
                          fs=int(rng.integers(0, 2)) if b16 else 0, causal=int(rng.integers(0, 2)),
                          hint=int(rng.integers(0, 2)), seed=100 + i))
    return cases


@pytest.mark.parametrize("c", _random_cases(14, 20221105), ids=lambda c: "h%d_a%d_f%d_S%d_b%d_L%d_l%d_m%d_%s" % (
    c["h"], c["a"], c["f"], c["S_seq"], c["S_mb"], c["Lyr"], c["N_loop"], c["N_mb"], "bf16" if c["b16"] else "fp32"))
def test_randomly_drawn_configurations(c):
    """Both orders on configurations nobody picked by hand: outputs, input gradients and every
    main-grad against the oracle; the two orders bit-identical in y and dx."""
    mode, dtype = ("bf16", bf.BF_BF16) if c["b16"] else ("fp32", bf.BF_FP32)
    params = bf_inputs.make_params(c["seed"], c["Lyr"], c["h"], c["f"], bf16=c["b16"])
    x, dy = bf_inputs.make_batch(c["seed"], c["N_mb"], c["S_mb"], c["S_seq"], c["h"], bf16=c["b16"])
    cfg = bf.make_config(c["h"], c["a"], c["f"], c["S_seq"], c["Lyr"], c["N_mb"], c["S_mb"], dtype=dtype, ckpt_mode=c["ckpt"],
                         fuse_wgrad=c["fuse"], dp_fs=c["fs"], causal=c["causal"], N_loop_min=c["N_loop"] if c["hint"] else 0)
    ref = _oracle(params, x, dy, K.SCHED_BF, c["N_loop"], c["a"], causal=bool(c["causal"]))
    g_bf = _run_gpu(cfg, params, x, dy, bf.BF_SCHED_BF, c["N_loop"], c["N_mb"], c["S_mb"])
    g_df = _run_gpu(cfg, params, x, dy, bf.BF_SCHED_DF, c["N_loop"], c["N_mb"], c["S_mb"])
    _compare(g_bf, ref, TOL[mode], c["Lyr"])
    _compare(g_df, ref, TOL[mode], c["Lyr"])
    assert np.array_equal(g_bf["y"], g_df["y"]) and np.array_equal(g_bf["dx"], g_df["dx"])
    assert g_bf["report"].peak_ckpt_count == F.ckpt_count("BF", c["N_mb"], c["Lyr"], 1)
    assert g_df["report"].peak_ckpt_count == F.ckpt_count("DF", c["N_mb"], c["Lyr"], 1)
    if c["fuse"] and not c["fs"]:
        # the same step with two chains of micro-batches, where the configuration allows them
        cfg.mb_chains = 2
        g_two = _run_gpu(cfg, params, x, dy, bf.BF_SCHED_BF, c["N_loop"], c["N_mb"], c["S_mb"])
        assert g_two["report"].mb_chains == (2 if c["N_mb"] >= 2 else 1)
        _compare(g_two, ref, TOL[mode], c["Lyr"])
        assert g_two["trace"] == g_bf["trace"]


def _random_rank_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        b16 = bool(i % 2)
        N_PP = int(rng.choice([1, 2, 3, 4]))
        rank = int(rng.integers(0, N_PP))
        N_loop = int(rng.choice([1, 2, 3]))
        Lyr = N_loop * int(rng.choice([1, 2]))
        N_mb = N_PP * int(rng.integers(1, 4))       # depth-first runs sequences of N_PP
        if b16:
            h, a, f, S_seq, S_mb = 256, int(rng.choice([2, 4])), 1024, int(rng.choice([128, 256])), 1
        else:
            a = int(rng.choice([1, 2, 3]))
            h, S_seq, S_mb = a * int(rng.choice([8, 24])), int(rng.integers(5, 50)), int(rng.choice([1, 2]))
            f = int(rng.integers(h, 3 * h))
        cases.append((("bf16", bf.BF_BF16) if b16 else ("fp32", bf.BF_FP32)) + (
            N_PP, rank, Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb, int(rng.integers(0, 2)),
            int(rng.choice([bf.BF_CKPT_NONE, bf.BF_CKPT_LAYER])), int(rng.integers(0, 2)) if b16 else 0))
    return cases


@pytest.mark.parametrize("c", _random_rank_cases(10, 5953), ids=lambda c: "%s_pp%d_r%d_L%d_l%d_h%d_S%d_m%d" % (
    c[0], c[2], c[3], c[4], c[5], c[6], c[9], c[11]))
def test_randomly_drawn_pipeline_ranks(c):
    """The checks of the rank-step test on drawn pipeline depths, ranks, loop counts and flags."""
    test_rank_of_a_deeper_pipeline_matches_oracle(*c)


@pytest.mark.parametrize("schedule,chains", [(bf.BF_SCHED_BF, 1), (bf.BF_SCHED_DF, 1), (bf.BF_SCHED_BF, 2)])
def test_gradient_step_replays_from_a_hip_graph(schedule, chains):
    """With timing = 0 and queue_depth = 0 a step is kernel launches and event record / wait only
    (everything pre-allocated, App. D.2; buffers cleared by fill kernels): it can be captured into a HIP graph.
    Three replays, with unrelated eager work and synchronisations in between, each bit-identical to the
    eager step.  With two chains of micro-batches the second stream forks from the captured one at the start of
    the step and joins it at the end, so the recording holds both."""
    Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb = 4, 2, 256, 2, 1024, 128, 1, 3
    params = bf_inputs.make_params(29, Lyr, h, f, bf16=True)
    x, dy = bf_inputs.make_batch(29, N_mb, S_mb, S_seq, h, bf16=True)
    cfg = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=bf.BF_BF16, fuse_wgrad=1, queue_depth=0, mb_chains=chains)
    st = bf.Stack(cfg)
    for l, p in enumerate(params):
        for name, tid in bf.TENSOR_IDS.items():
            st.bf_set_params(l, tid, p[name].reshape(-1))
    dX, dDY = to_dev(x, True), to_dev(dy, True)
    y, dx = torch.empty_like(dX), torch.empty_like(dX)
    run = lambda: st.bf_run_step(schedule, N_loop, N_mb, S_mb, dX, dDY, y, dx, apply_optimizer=0, timing=0)
    run()
    torch.cuda.synchronize()
    want = dict(y=y.clone(), dx=dx.clone(),
                grads=[{n: st.bf_get_grads(l, t) for n, t in bf.TENSOR_IDS.items()} for l in range(Lyr)])
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for replay in range(3):
        y.zero_()
        dx.zero_()
        noise = torch.randn(1 << 20, device="cuda").cumsum(0).sum().item()   # eager work and a synchronisation
        assert np.isfinite(noise)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want["y"]) and torch.equal(dx, want["dx"]), replay
        for l in range(Lyr):
            for n, t in bf.TENSOR_IDS.items():
                assert np.array_equal(st.bf_get_grads(l, t), want["grads"][l][n]), (replay, l, n)
    del graph
    st.close()


@pytest.mark.parametrize("chains,N_mb", [(1, 2), (2, 2), (2, 5)])
def test_optimizer_steps_replay_from_a_hip_graph(chains, N_mb):
    """The optimizer's step count lives on the device and is advanced by the step itself, so a recorded
    training step (breadth-first, Adam per stage as soon as its gradient is final) keeps its bias corrections right
    from replay to replay: eager step 1, then the graph replayed as steps 2 and 3, equals three eager steps.
    Also with two chains of micro-batches, whose second stream is part of the recording."""
    Lyr, N_loop, h, a, f, S_seq, S_mb = 4, 2, 256, 2, 1024, 128, 1
    params = bf_inputs.make_params(31, Lyr, h, f, bf16=True)
    x, dy = bf_inputs.make_batch(31, N_mb, S_mb, S_seq, h, bf16=True)
    cfg = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=bf.BF_BF16, fuse_wgrad=1, queue_depth=0, lr=1e-3,
                         weight_decay=0.01, mb_chains=chains)
    dX, dDY = to_dev(x, True), to_dev(dy, True)

    def fresh():
        st = bf.Stack(cfg)
        for l, p in enumerate(params):
            for name, tid in bf.TENSOR_IDS.items():
                st.bf_set_params(l, tid, p[name].reshape(-1))
        y, dx = torch.empty_like(dX), torch.empty_like(dX)
        return st, y, dx, (lambda: st.bf_run_step(bf.BF_SCHED_BF, N_loop, N_mb, S_mb, dX, dDY, y, dx, apply_optimizer=1, timing=0))

    def state(st):
        torch.cuda.synchronize()
        return [(st.bf_get_params(l, t), st.bf_get_moments(l, t, 0), st.bf_get_moments(l, t, 1))
                for l in range(Lyr) for t in bf.TENSOR_IDS.values()]

    st, y, dx, run = fresh()
    for _ in range(3):
        run()
    want, want_y = state(st), y.clone()
    st.close()

    st, y, dx, run = fresh()
    run()                                   # step 1, eager
    snap = state(st)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):           # records step 2 (capture does not execute it)
        run()
    assert all(np.array_equal(a, b) for s0, s1 in zip(snap, state(st)) for a, b in zip(s0, s1)), "capture ran the step"
    for _ in range(2):                      # steps 2 and 3
        assert np.isfinite(torch.randn(1 << 18, device="cuda").sum().item())
        graph.replay()
    got = state(st)
    assert torch.equal(y, want_y)
    for (pw, mw, vw), (pg, mg, vg) in zip(want, got):
        assert np.array_equal(pw, pg) and np.array_equal(mw, mg) and np.array_equal(vw, vg)
    del graph
    st.close()


@pytest.mark.parametrize("chains", [1, 2])
def test_timing_modes_fill_the_report_and_leave_the_numbers_alone(chains):
    """timing 1: step time; 2: an event pair around every launch, per-class sums in the report; 3: around
    the weight-gradient products only.  Launch counts follow from the layer structure (4 forward, 4 dgrad and 4
    weight-gradient products, 2 LayerNorms each way, 1 attention each way per layer and micro-batch; one
    fused weight-gradient product per weight and stage); the results do not depend on the mode.  With two chains
    of micro-batches the event pairs sit on two streams and the counts are the same."""
    Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb = 4, 2, 256, 2, 1024, 128, 1, 3
    params = bf_inputs.make_params(37, Lyr, h, f, bf16=True)
    x, dy = bf_inputs.make_batch(37, N_mb, S_mb, S_seq, h, bf16=True)
    cfg = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=bf.BF_BF16, fuse_wgrad=1, mb_chains=chains)
    st = bf.Stack(cfg)
    for l, p in enumerate(params):
        for name, tid in bf.TENSOR_IDS.items():
            st.bf_set_params(l, tid, p[name].reshape(-1))
    dX, dDY = to_dev(x, True), to_dev(dy, True)
    y, dx = torch.empty_like(dX), torch.empty_like(dX)
    K_ = {n: i for i, n in enumerate(bf.binding.KERNEL_CLASSES)}
    outs = []
    for timing in (0, 1, 2, 3):
        rep = st.bf_run_step(bf.BF_SCHED_BF, N_loop, N_mb, S_mb, dX, dDY, y, dx, apply_optimizer=0, timing=timing)
        torch.cuda.synchronize()
        outs.append((y.clone(), dx.clone(), st.bf_get_grads(1, bf.TENSOR_IDS["w_fc1"])))
        n = lambda cls: int(rep.kernel_launches[K_[cls]])
        lm = Lyr * N_mb
        assert rep.mb_chains == chains
        if timing == 0:
            assert rep.timed == 0
        else:
            assert rep.timed == 1 and rep.gpu_ms > 0
        if timing in (2, 3):
            assert n("gemm_wgrad") == 4 * Lyr
            assert rep.kernel_ms[K_["gemm_wgrad"]] > 0 and rep.kernel_flops[K_["gemm_wgrad"]] > 0
        if timing == 2:
            assert (n("gemm_fwd"), n("gemm_dgrad")) == (4 * lm, 4 * lm)
            assert all(rep.kernel_ms[K_[c]] > 0 and rep.kernel_flops[K_[c]] > 0 for c in ("gemm_fwd", "gemm_dgrad"))
            assert rep.kernel_flops[K_["gemm_fwd"]] == rep.kernel_flops[K_["gemm_dgrad"]] == rep.kernel_flops[K_["gemm_wgrad"]]
            # the only separate column-sum launch left is the one per micro-batch for the top layer's incoming gradient:
            # FC1's bias gradient is taken inside the FC2 dgrad product, the QKV one inside the attention backward, the
            # out-projection's and the lower layers' FC2 ones inside the LayerNorm backward that writes the tensor
            assert (n("attn_fwd"), n("attn_bwd"), n("ln_fwd"), n("ln_bwd"), n("colsum")) == (lm, lm, 2 * lm, 2 * lm, N_mb)
        if timing in (0, 1):
            assert sum(int(v) for v in rep.kernel_launches) == 0
        if timing == 3:
            assert n("gemm_fwd") == n("gemm_dgrad") == n("attn_fwd") == n("ln_fwd") == n("colsum") == n("adam") == 0
    for yy, dd, gg in outs[1:]:
        assert torch.equal(yy, outs[0][0]) and torch.equal(dd, outs[0][1]) and np.array_equal(gg, outs[0][2])
    with pytest.raises(bf.BfError):
        st.bf_run_step(bf.BF_SCHED_BF, N_loop, N_mb, S_mb, dX, dDY, y, dx, timing=4)
    st.close()


@pytest.mark.parametrize("depth", [1, 3, 64])
def test_bounded_launch_queue_changes_nothing_but_the_host_pace(depth):
    """queue_depth > 0: the host waits for the op issued `depth` ops earlier before issuing the next one
    (pre-allocation with a bounded kernel queue, App. D.2).  Same launches in the same order: outputs
    and main-grads bit-identical to the unbounded queue, in both orders, optimizer on."""
    Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb = 4, 2, 256, 2, 1024, 128, 1, 3
    params = bf_inputs.make_params(41, Lyr, h, f, bf16=True)
    x, dy = bf_inputs.make_batch(41, N_mb, S_mb, S_seq, h, bf16=True)
    got = {}
    for qd in (0, depth):
        cfg = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=bf.BF_BF16, fuse_wgrad=1, queue_depth=qd, lr=1e-3)
        for code in (bf.BF_SCHED_BF, bf.BF_SCHED_DF):
            got[qd, code] = _run_gpu(cfg, params, x, dy, code, N_loop, N_mb, S_mb, apply_optimizer=1, steps=2)
    for code in (bf.BF_SCHED_BF, bf.BF_SCHED_DF):
        a0, a1 = got[0, code], got[depth, code]
        assert np.array_equal(a0["y"], a1["y"]) and np.array_equal(a0["dx"], a1["dx"])
        assert a0["trace"] == a1["trace"]
        for l in range(Lyr):
            for name in bf.TENSOR_IDS:
                assert np.array_equal(a0["grads"][l][name], a1["grads"][l][name]), (l, name)
                assert np.array_equal(a0["params"][l][name], a1["params"][l][name]), (l, name)


@pytest.mark.parametrize("ckpt", [bf.BF_CKPT_NONE, bf.BF_CKPT_LAYER])
def test_activation_bytes_count_what_the_fused_weight_gradient_keeps(ckpt):
    """peak_act_bytes from the sizes of the stored tensors (bf16, S_mlp = 4 S_hidden: 32 S_hidden T bytes per layer
    and micro-batch without checkpointing, the input alone with, App. A.2.1 / A.2.2 less the dropout masks and the
    attention scores), plus what fuse_wgrad keeps per layer of a stage and micro-batch until the stage completes:
    the gradients dy, du, dx1, dqkv (18 S_hidden T bytes) and, with checkpointing, the recomputed a, ctx, c, g (14)."""
    Lyr, N_loop, h, a, S_seq, S_mb, N_mb = 4, 2, 256, 2, 128, 2, 3
    f, T, per_stage = 4 * h, S_mb * S_seq, Lyr // N_loop
    x, dy = bf_inputs.make_batch(3, N_mb, S_mb, S_seq, h, bf16=True)
    dX, dDY = to_dev(x, True), to_dev(dy, True)
    stats = 2 * (T * 2 * 4) + S_mb * a * S_seq * 4            # LayerNorm statistics twice, log-sum-exp
    record = 30 * h * T + stats                               # a, qkv, ctx, x1, c, u, g
    for fuse in (0, 1):
        st = bf.Stack(bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, ckpt_mode=ckpt, fuse_wgrad=fuse, N_loop_min=N_loop))
        for sched in (bf.BF_SCHED_BF, bf.BF_SCHED_DF):
            rep = st.bf_run_step(sched, N_loop, N_mb, S_mb, dX, dDY)
            torch.cuda.synchronize()
            live = rep.peak_ckpt_count
            assert live == (Lyr * N_mb if sched == bf.BF_SCHED_BF else Lyr)
            kept = 0
            if fuse and sched == bf.BF_SCHED_BF:
                kept = per_stage * N_mb * (18 + (14 if ckpt == bf.BF_CKPT_LAYER else 0)) * h * T
            assert rep.fused_wgrad_bytes == kept
            stored = live * (record + 2 * h * T) if ckpt == bf.BF_CKPT_NONE else live * 2 * h * T + record
            assert rep.peak_act_bytes == stored + kept, (fuse, sched, rep.peak_act_bytes, stored, kept)
        st.close()
