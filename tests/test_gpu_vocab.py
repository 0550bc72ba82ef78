"""GPU parity of the input / output layers (token + position embedding, final LayerNorm, output
projection, cross-entropy) and of the step on token ids against the CPU oracle.
Tolerance: max|gpu - oracle| / max|oracle| <= 1e-5 in fp32 mode, 2e-2 in bf16 mode, per tensor."""
import numpy as np
import pytest
import torch

import bf_inputs
import paper_2211_05953_amd as bf
from oracle import stack as K
from oracle import vocab as V
from util import TOL, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu

MODES = [("fp32", bf.BF_FP32), ("bf16", bf.BF_BF16)]


def _itensor(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


@pytest.mark.parametrize("mode,dtype", MODES)
@pytest.mark.parametrize("S_mb,S_seq,S_voc,h", [(2, 64, 97, 72), (1, 128, 1000, 256), (3, 50, 7, 40), (1, 1, 1, 1)])
def test_embedding_forward_and_backward(mode, dtype, S_mb, S_seq, S_voc, h):
    b16 = dtype == bf.BF_BF16
    vp = bf_inputs.make_vocab_params(3, S_voc, S_seq, h, bf16=b16)
    vp64 = {k: v.astype(np.float64) for k, v in vp.items()}
    tokens, _ = bf_inputs.make_tokens(3, 1, S_mb, S_seq, S_voc)
    tokens = tokens[0]
    d = bf_inputs.normal(3, 0, (S_mb, S_seq, h), bf16=b16)
    T = S_mb * S_seq
    dtok, e_tok, e_pos = _itensor(tokens), to_dev(vp["e_tok"], False), to_dev(vp["e_pos"], False)
    x = torch.empty(S_mb, S_seq, h, dtype=torch.bfloat16 if b16 else torch.float32, device="cuda")
    bf.bf_op_embedding_fwd(dtype, T, S_seq, S_voc, h, dtok, e_tok, e_pos, x)
    assert rel_err(to_host(x), V.embedding_fwd(vp64, tokens)) <= (TOL[mode] if b16 else 1e-7)
    # gradient: start from a non-zero g_tok (it is added to) and from garbage in g_pos (it is overwritten)
    g0 = bf_inputs.normal(3, 1, (S_voc, h))
    g_tok, g_pos = to_dev(g0, False), torch.full((S_seq, h), 7.0, device="cuda")
    bf.bf_op_embedding_bwd(dtype, S_mb, S_seq, S_voc, h, dtok, to_dev(d, b16), g_tok, g_pos, 0)
    ref = V.embedding_bwd(vp64, tokens, d.astype(np.float64))
    assert rel_err(to_host(g_tok) - g0, ref["e_tok"]) <= 1e-5
    assert rel_err(to_host(g_pos), ref["e_pos"]) <= 1e-5
    first = to_host(g_pos).copy()
    bf.bf_op_embedding_bwd(dtype, S_mb, S_seq, S_voc, h, dtok, to_dev(d, b16), g_tok, g_pos, 1)
    assert rel_err(to_host(g_pos), 2 * ref["e_pos"]) <= 1e-5
    # fixed summation order: a second run from the same start gives the same bits
    g_tok2, g_pos2 = to_dev(g0, False), torch.zeros(S_seq, h, device="cuda")
    bf.bf_op_embedding_bwd(dtype, S_mb, S_seq, S_voc, h, dtok, to_dev(d, b16), g_tok2, g_pos2, 0)
    assert np.array_equal(to_host(g_pos2), first)
    unused = np.setdiff1d(np.arange(S_voc), np.unique(tokens))
    assert np.array_equal(to_host(g_tok2)[unused], g0[unused])


def test_embedding_ignores_ids_out_of_range():
    S_mb, S_seq, S_voc, h = 1, 8, 5, 16
    vp = bf_inputs.make_vocab_params(4, S_voc, S_seq, h)
    tokens = np.array([[0, 4, -1, 5, 2, 2, 1 << 30, 3]], dtype=np.int32)
    x = torch.empty(S_mb, S_seq, h, device="cuda")
    bf.bf_op_embedding_fwd(bf.BF_FP32, S_seq, S_seq, S_voc, h, _itensor(tokens), to_dev(vp["e_tok"], False),
                           to_dev(vp["e_pos"], False), x)
    ok = (tokens[0] >= 0) & (tokens[0] < S_voc)
    ref = vp["e_pos"].copy()
    ref[ok] += vp["e_tok"][tokens[0][ok]]
    assert np.array_equal(to_host(x)[0], ref)
    g_tok, g_pos = torch.zeros(S_voc, h, device="cuda"), torch.zeros(S_seq, h, device="cuda")
    d = bf_inputs.normal(4, 0, (S_mb, S_seq, h))
    bf.bf_op_embedding_bwd(bf.BF_FP32, S_mb, S_seq, S_voc, h, _itensor(tokens), to_dev(d, False), g_tok, g_pos, 0)
    ref_g = np.zeros((S_voc, h), dtype=np.float32)
    for i in np.nonzero(ok)[0]:
        ref_g[tokens[0, i]] += d[0, i]
    assert rel_err(to_host(g_tok), ref_g) <= 1e-6


@pytest.mark.parametrize("mode,dtype", MODES)
@pytest.mark.parametrize("T,S_voc", [(64, 1000), (33, 97), (5, 3), (16, 50304), (1, 1)])
def test_cross_entropy_rows(mode, dtype, T, S_voc):
    b16 = dtype == bf.BF_BF16
    z = bf_inputs.normal(5, 0, (T, S_voc), 3.0, bf16=b16)
    labels = np.random.Generator(np.random.PCG64(5)).integers(0, S_voc, size=T).astype(np.int32)
    scale = 1.0 / (3 * T)
    z64 = z.astype(np.float64)
    lse = np.log(np.exp(z64 - z64.max(1, keepdims=True)).sum(1)) + z64.max(1)
    ref_rows = (lse - z64[np.arange(T), labels]) * scale
    ref_dz = np.exp(z64 - lse[:, None])
    ref_dz[np.arange(T), labels] -= 1
    ref_dz *= scale
    dz, row_loss, loss = to_dev(z, b16), torch.empty(T, device="cuda"), torch.empty(1, device="cuda")
    bf.bf_op_ce_loss(dtype, T, S_voc, dz, _itensor(labels), scale, row_loss, loss)
    assert rel_err(to_host(row_loss), ref_rows) <= 1e-5
    assert abs(loss.item() - ref_rows.sum()) <= 1e-5 * abs(ref_rows.sum())
    assert rel_err(to_host(dz), ref_dz) <= TOL[mode]
    # every row of the gradient sums to zero (softmax sums to one), up to the storage rounding
    assert np.abs(to_host(dz).astype(np.float64).sum(1)).max() <= (2e-2 if b16 else 1e-5) * scale
    # a label out of range drops its row
    labels[0] = S_voc
    dz = to_dev(z, b16)
    bf.bf_op_ce_loss(dtype, T, S_voc, dz, _itensor(labels), scale, row_loss, loss)
    assert to_host(row_loss)[0] == 0 and np.abs(to_host(dz)[0]).max() == 0
    assert abs(loss.item() - ref_rows[1:].sum()) <= 1e-5 * abs(ref_rows.sum()) + 1e-12


def _run_lm(cfg, params, vp, tokens, labels, schedule, N_loop, N_mb, S_mb, apply_optimizer=0, steps=1):
    st = bf.Stack(cfg)
    for l, p in enumerate(params):
        for name, tid in bf.TENSOR_IDS.items():
            st.bf_set_params(l, tid, p[name].reshape(-1))
    for name, tid in bf.VOCAB_TENSOR_IDS.items():
        st.bf_set_params(cfg.N_layers, tid, vp[name].reshape(-1))
    dtok, dlab = _itensor(tokens), _itensor(labels)
    loss = torch.zeros(N_mb, device="cuda")
    for _ in range(steps):
        rep = st.bf_run_lm_step(schedule, N_loop, N_mb, S_mb, dtok, dlab, loss, apply_optimizer=apply_optimizer)
    torch.cuda.synchronize()
    out = dict(loss_mb=to_host(loss), report=rep, trace=st.bf_get_trace(),
               grads=[{n: st.bf_get_grads(l, t) for n, t in bf.TENSOR_IDS.items()} for l in range(cfg.N_layers)],
               vgrads={n: st.bf_get_grads(cfg.N_layers, t) for n, t in bf.VOCAB_TENSOR_IDS.items()},
               vparams={n: st.bf_get_params(cfg.N_layers, t) for n, t in bf.VOCAB_TENSOR_IDS.items()},
               vm={n: st.bf_get_moments(cfg.N_layers, t, 0) for n, t in bf.VOCAB_TENSOR_IDS.items()})
    st.close()
    return out


LM_CASES = [
    # mode, dtype, ckpt, fuse, fs, L, N_loop, h, a, f, S_seq, S_mb, N_mb, S_voc
    ("fp32", bf.BF_FP32, bf.BF_CKPT_NONE, 0, 0, 2, 2, 64, 2, 256, 32, 2, 3, 97),
    ("fp32", bf.BF_FP32, bf.BF_CKPT_LAYER, 1, 0, 4, 2, 128, 2, 512, 64, 1, 4, 1000),
    ("bf16", bf.BF_BF16, bf.BF_CKPT_NONE, 1, 0, 4, 2, 256, 2, 1024, 128, 1, 4, 1024),
    ("bf16", bf.BF_BF16, bf.BF_CKPT_NONE, 0, 1, 2, 2, 256, 2, 1024, 128, 2, 2, 640),
    ("bf16", bf.BF_BF16, bf.BF_CKPT_LAYER, 0, 0, 2, 1, 128, 2, 512, 64, 1, 3, 333),
]


@pytest.mark.parametrize("mode,dtype,ckpt,fuse,fs,Lyr,N_loop,h,a,f,S_seq,S_mb,N_mb,S_voc", LM_CASES)
def test_lm_step_matches_oracle_in_both_orders(mode, dtype, ckpt, fuse, fs, Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb, S_voc):
    b16 = dtype == bf.BF_BF16
    params = bf_inputs.make_params(29, Lyr, h, f, bf16=b16)
    vp = bf_inputs.make_vocab_params(29, S_voc, S_seq, h, init_std=0.1, bf16=b16)
    tokens, labels = bf_inputs.make_tokens(29, N_mb, S_mb, S_seq, S_voc)
    p64 = [{k: v.astype(np.float64) for k, v in p.items()} for p in params]
    vp64 = {k: v.astype(np.float64) for k, v in vp.items()}
    ref = K.run_lm_step(p64, vp64, tokens, labels, K.SCHED_BF, N_loop, a)
    cfg = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=dtype, ckpt_mode=ckpt, fuse_wgrad=fuse, dp_fs=fs,
                         N_loop_min=N_loop, S_voc=S_voc)
    got = {}
    for name, code in (("BF", bf.BF_SCHED_BF), ("DF", bf.BF_SCHED_DF)):
        g = got[name] = _run_lm(cfg, params, vp, tokens, labels, code, N_loop, N_mb, S_mb)
        tol = TOL[mode]
        assert rel_err(g["loss_mb"], ref["loss_mb"]) <= tol
        assert abs(g["loss_mb"].astype(np.float64).sum() - ref["loss"]) <= tol * ref["loss"]
        for l in range(Lyr):
            for k in bf.TENSOR_IDS:
                assert rel_err(g["grads"][l][k], ref["grads"][l][k].reshape(-1)) <= tol, (name, l, k)
        for k in bf.VOCAB_TENSOR_IDS:
            assert rel_err(g["vgrads"][k], ref["vgrads"][k].reshape(-1)) <= tol, (name, k)
    # same per-tensor sums in both orders wherever the micro-batches are added one by one
    assert np.array_equal(got["BF"]["loss_mb"], got["DF"]["loss_mb"])
    for k in bf.VOCAB_TENSOR_IDS:
        assert np.array_equal(got["BF"]["vgrads"][k], got["DF"]["vgrads"][k]), k
    # the output projection is priced as Eq. compute's S_voc term: 6 S_voc S_hidden flop per token
    plain = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=dtype, S_voc=0)
    st = bf.Stack(plain)
    x = torch.zeros(N_mb, S_mb, S_seq, h, dtype=torch.bfloat16 if b16 else torch.float32, device="cuda")
    base = st.bf_run_step(bf.BF_SCHED_BF, N_loop, N_mb, S_mb, x, x).flops_model
    st.close()
    assert got["BF"]["report"].flops_model - base == 6.0 * S_voc * h * N_mb * S_mb * S_seq


def test_lm_optimizer_moves_input_and_output_layers_once():
    Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb, S_voc = 2, 2, 64, 2, 256, 32, 1, 3, 50
    params = bf_inputs.make_params(31, Lyr, h, f)
    vp = bf_inputs.make_vocab_params(31, S_voc, S_seq, h, init_std=0.1)
    tokens, labels = bf_inputs.make_tokens(31, N_mb, S_mb, S_seq, S_voc)
    lr = float(np.float32(1e-3))
    cfg = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=bf.BF_FP32, S_voc=S_voc, lr=lr)
    for code in (bf.BF_SCHED_BF, bf.BF_SCHED_DF):
        g = _run_lm(cfg, params, vp, tokens, labels, code, N_loop, N_mb, S_mb, apply_optimizer=1)
        for k in bf.VOCAB_TENSOR_IDS:
            grad = g["vgrads"][k].astype(np.float64)
            # first Adam step: m = (1 - beta1) g, and the weight moves by lr * sign(g) where g is well off zero
            assert rel_err(g["vm"][k], 0.1 * grad) <= 1e-5, k
            big = np.abs(grad) > 1e-2 * np.abs(grad).max()
            moved = g["vparams"][k].astype(np.float64) - vp[k].reshape(-1)
            assert np.abs(moved[big] + lr * np.sign(grad[big])).max() <= 2e-2 * lr, k
            assert np.abs(moved[grad == 0]).max(initial=0) == 0, k      # rows of tokens never seen stay put


def test_lm_step_argument_errors():
    cfg = bf.make_config(64, 2, 256, 16, 2, 2, 1, dtype=bf.BF_FP32)
    st = bf.Stack(cfg)
    t = torch.zeros(2, 1, 16, dtype=torch.int32, device="cuda")
    with pytest.raises(bf.BfError, match="S_voc"):
        st.bf_run_lm_step(bf.BF_SCHED_BF, 2, 2, 1, t, t, torch.zeros(2, device="cuda"))
    st.close()
    cfg = bf.make_config(64, 2, 256, 16, 2, 2, 1, dtype=bf.BF_FP32, S_voc=11)
    st = bf.Stack(cfg)
    with pytest.raises(bf.BfError):
        st.bf_run_lm_step(bf.BF_SCHED_BF, 2, 2, 1, t, None, torch.zeros(2, device="cuda"))
    assert st.bf_tensor_elems(bf.VOCAB_TENSOR_IDS["w_out"]) == 11 * 64
    with pytest.raises(bf.BfError):
        st.bf_get_params(0, bf.VOCAB_TENSOR_IDS["w_out"])       # the vocabulary tensors live in pseudo-layer N_layers
    st.close()
