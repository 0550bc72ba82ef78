"""Pins for oracle/stack.py: order invariance of the accumulated gradient, event trace
counts, checkpoint counts (Eq. mem_ckpt), Adam closed form and library cross-check."""
import numpy as np
import torch

import bf_inputs
from oracle import formulas as F
from oracle import stack as K


def _setup(N_layers=4, h=16, a=2, f=64, S_seq=8, S_mb=2, N_mb=3, seed=3):
    params = [{k: v.astype(np.float64) for k, v in p.items()}
              for p in bf_inputs.make_params(seed, N_layers, h, f, init_std=0.3, bias_std=0.2)]
    x, dy = bf_inputs.make_batch(seed, N_mb, S_mb, S_seq, h)
    return params, x.astype(np.float64), dy.astype(np.float64), a


def test_bf_equals_df_bitwise_and_equals_one_big_batch():
    params, x, dy, a = _setup()
    bf = K.run_step(params, x, dy, K.SCHED_BF, 2, a)
    df = K.run_step(params, x, dy, K.SCHED_DF, 2, a)
    bf4 = K.run_step(params, x, dy, K.SCHED_BF, 4, a)
    big = K.run_one_big_batch(params, x, dy, a)
    assert np.array_equal(bf["y"], df["y"]) and np.array_equal(bf["dx"], df["dx"])
    assert np.array_equal(bf["y"], bf4["y"]) and np.array_equal(bf["dx"], bf4["dx"])
    assert np.allclose(bf["y"], big["y"], rtol=1e-12, atol=1e-12)
    assert np.allclose(bf["dx"], big["dx"], rtol=1e-12, atol=1e-12)
    for l in range(len(params)):
        for k in params[l]:
            assert np.array_equal(bf["grads"][l][k], df["grads"][l][k]), (l, k)
            assert np.array_equal(bf["grads"][l][k], bf4["grads"][l][k]), (l, k)
            ref = big["grads"][l][k]
            assert np.allclose(bf["grads"][l][k], ref, rtol=1e-10, atol=1e-10 * np.abs(ref).max()), (l, k)


def test_stack_gradient_finite_differences():
    params, x, dy, a = _setup(N_layers=2, N_mb=2)
    r = K.run_step(params, x, dy, K.SCHED_BF, 2, a)

    def loss():
        return float((K.run_step(params, x, dy, K.SCHED_DF, 1, a)["y"] * dy).sum())

    rng = np.random.default_rng(0)
    eps = 1e-5
    for l in (0, 1):
        for k in ("w_qkv", "b_fc1", "ln1_g", "w_fc2"):
            flat = params[l][k].reshape(-1)
            for i in rng.choice(flat.size, 4, replace=False):
                old = flat[i]
                flat[i] = old + eps; lp = loss()
                flat[i] = old - eps; lm = loss()
                flat[i] = old
                an = r["grads"][l][k].reshape(-1)[i]
                assert abs((lp - lm) / (2 * eps) - an) <= 2e-6 * max(1.0, abs(an)), (l, k, i)


def test_trace_and_checkpoint_counts():
    params, x, dy, a = _setup(N_layers=4, N_mb=3)
    for N_loop in (1, 2, 4):
        bf = K.run_step(params, x, dy, K.SCHED_BF, N_loop, a)
        df = K.run_step(params, x, dy, K.SCHED_DF, N_loop, a)
        assert len(bf["trace"]) == len(df["trace"]) == 2 * N_loop * 3 + N_loop
        assert bf["peak_ckpt"] == F.ckpt_count("BF", 3, 4, 1) == 12
        assert df["peak_ckpt"] == F.ckpt_count("DF", 3, 4, 1) == 4
        assert bf["trace"][-1][3] == 0 and df["trace"][-1][3] == 0


def test_adam_first_step_closed_form_and_torch():
    rng = np.random.default_rng(5)
    w = rng.standard_normal(50)
    g = rng.standard_normal(50) * 10.0 ** rng.integers(-6, 2, 50)
    lr, eps = 1e-3, 1e-8
    w1, m1, v1 = K.adam_update(w, g, np.zeros(50), np.zeros(50), 1, lr, 0.9, 0.999, eps)
    # with bias correction the first step moves by -lr * sign(g) / (1 + eps/|g|)
    assert np.allclose(w1 - w, -lr * np.sign(g) / (1.0 + eps / np.abs(g)), rtol=1e-7, atol=0)
    # three steps against the library optimizer
    tw = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([tw], lr=lr, betas=(0.9, 0.999), eps=eps)
    ww, mm, vv = w.copy(), np.zeros(50), np.zeros(50)
    for t in (1, 2, 3):
        gt = g * t
        tw.grad = torch.tensor(gt)
        opt.step()
        ww, mm, vv = K.adam_update(ww, gt, mm, vv, t, lr, 0.9, 0.999, eps)
        assert np.allclose(ww, tw.detach().numpy(), rtol=1e-12, atol=1e-14)
    # decoupled weight decay against AdamW
    tw = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([tw], lr=lr, betas=(0.9, 0.999), eps=eps, weight_decay=0.1)
    tw.grad = torch.tensor(g)
    opt.step()
    w2, _, _ = K.adam_update(w, g, np.zeros(50), np.zeros(50), 1, lr, 0.9, 0.999, eps, 0.1)
    assert np.allclose(w2, tw.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_optimizer_fires_per_stage_and_uses_final_gradient():
    params, x, dy, a = _setup(N_layers=2, N_mb=2)
    adam = dict(lr=1e-2, beta1=0.9, beta2=0.999, adam_eps=1e-8, weight_decay=0.0, t=1)
    bf = K.run_step(params, x, dy, K.SCHED_BF, 2, a, adam=adam)
    df = K.run_step(params, x, dy, K.SCHED_DF, 2, a, adam=adam)
    for l in range(2):
        for k in params[l]:
            assert np.array_equal(bf["new_params"][l][k], df["new_params"][l][k])
            g = bf["grads"][l][k]
            ref = params[l][k] - 1e-2 * g / (np.abs(g) + 1e-8)
            assert np.allclose(bf["new_params"][l][k], ref, rtol=1e-9, atol=1e-12)
    # weights used by the backward are the old ones: y does not depend on the optimizer
    noopt = K.run_step(params, x, dy, K.SCHED_BF, 2, a)
    assert np.array_equal(noopt["dx"], bf["dx"])


def test_rank_step_composes_to_the_chained_step_and_keeps_the_pipeline_order():
    """A pipeline rank's stages, fed by hand with what their neighbours would send, must give what the
    chained stack gives (the stack pinned above by finite differences and the one-big-batch run): the
    two ranks of an N_PP = 2 pipeline over 4 layers in 4 stages, forward rank by rank and backward in
    reverse, reproduce the N_loop = 4 single-device step.  The order changes nothing but the trace."""
    from oracle import schedule as S
    params, x, dy, a = _setup(N_layers=4, N_mb=4)
    whole = K.run_step(params, x, dy, K.SCHED_BF, 4, a)
    N_PP, N_loop, N_mb = 2, 2, 4
    # layers of rank r, local stage l: global stage l * N_PP + r = layer index here (one layer per stage)
    rank_params = [[params[l * N_PP + r] for l in range(N_loop)] for r in range(N_PP)]
    zeros = np.zeros((N_loop,) + x.shape)
    # forward sweep: stage j's input is stage j-1's output; run ranks with the inputs known so far
    xin = [zeros.copy() for _ in range(N_PP)]
    xin[0][0] = x
    for j in range(N_PP * N_loop):
        r, l = j % N_PP, j // N_PP
        out = K.run_rank_step(rank_params[r], xin[r], zeros, "BF", N_PP, r, N_loop, a)
        if j + 1 < N_PP * N_loop:
            xin[(j + 1) % N_PP][(j + 1) // N_PP] = out["y"][l]
    assert np.array_equal(out["y"][N_loop - 1], whole["y"])
    # backward sweep: stage j's incoming gradient is what stage j+1 hands back
    din = [zeros.copy() for _ in range(N_PP)]
    din[N_PP - 1][N_loop - 1] = dy
    for j in reversed(range(N_PP * N_loop)):
        r, l = j % N_PP, j // N_PP
        out = K.run_rank_step(rank_params[r], xin[r], din[r], "BF", N_PP, r, N_loop, a)
        if j > 0:
            din[(j - 1) % N_PP][(j - 1) // N_PP] = out["dx"][l]
    assert np.array_equal(out["dx"][0], whole["dx"])
    for r in range(N_PP):
        res = {kind: K.run_rank_step(rank_params[r], xin[r], din[r], kind, N_PP, r, N_loop, a) for kind in ("BF", "DF")}
        for l in range(N_loop):
            for k in params[0]:
                assert np.array_equal(res["BF"]["grads"][l][k], whole["grads"][l * N_PP + r][k]), (r, l, k)
                assert np.array_equal(res["DF"]["grads"][l][k], res["BF"]["grads"][l][k]), (r, l, k)
        for kind in ("BF", "DF"):
            ops = [e[:3] for e in res[kind]["trace"] if e[0] != K.OP_OPT]
            assert ops == S.device_order(kind, N_PP, N_loop, N_mb, r)
            assert res[kind]["peak_ckpt"] == S.simulate(kind, N_PP, N_loop, N_mb)["peak_live"][r]
        # Eq. mem_ckpt: breadth-first holds every micro-batch of every local stage, depth-first at most
        # N_layers + N_PP - 1 checkpoints
        assert res["BF"]["peak_ckpt"] == F.ckpt_count("BF", N_mb, 4, N_PP)
        assert res["DF"]["peak_ckpt"] <= F.ckpt_count("DF", N_mb, 4, N_PP)
        assert res["DF"]["peak_ckpt"] < res["BF"]["peak_ckpt"]
