"""Pins for oracle/vocab.py and oracle.stack.run_lm_step: torch's embedding / layer_norm / linear /
cross_entropy with autograd (library routines, float64), finite differences of the loss, and the
decomposition of the batch loss into micro-batch contributions."""
import numpy as np
import torch

import bf_inputs
from oracle import stack as K
from oracle import vocab as V


def _setup(S_voc=37, S_seq=6, h=16, f=64, N_layers=2, N_mb=3, S_mb=2, seed=5):
    params = [{k: v.astype(np.float64) for k, v in p.items()}
              for p in bf_inputs.make_params(seed, N_layers, h, f, init_std=0.3, bias_std=0.2)]
    vp = {k: v.astype(np.float64) for k, v in bf_inputs.make_vocab_params(seed, S_voc, S_seq, h, init_std=0.5).items()}
    tokens, labels = bf_inputs.make_tokens(seed, N_mb, S_mb, S_seq, S_voc)
    return params, vp, tokens, labels


def test_tokens_are_in_range_repeat_and_labels_are_shifted():
    tokens, labels = bf_inputs.make_tokens(1, 4, 2, 64, 1000)
    assert tokens.dtype == np.int32 and tokens.min() >= 0 and tokens.max() < 1000
    assert np.array_equal(tokens[..., 1:], labels[..., :-1])
    assert len(np.unique(tokens[0])) < tokens[0].size          # frequent tokens repeat inside a micro-batch


def test_embedding_and_head_against_torch_autograd():
    _, vp, tokens, labels = _setup()
    rng = np.random.default_rng(0)
    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in vp.items()}
    tok, lab = torch.tensor(tokens[0], dtype=torch.long), torch.tensor(labels[0], dtype=torch.long)
    # input layer
    x = V.embedding_fwd(vp, tokens[0])
    xt = torch.nn.functional.embedding(tok, t["e_tok"]) + t["e_pos"][None]
    assert np.allclose(x, xt.detach().numpy(), rtol=0, atol=1e-15)
    dx = rng.standard_normal(x.shape)
    xt.backward(torch.tensor(dx))
    G = V.embedding_bwd(vp, tokens[0], dx)
    assert np.allclose(G["e_tok"], t["e_tok"].grad.numpy(), rtol=1e-13, atol=1e-13)
    assert np.allclose(G["e_pos"], t["e_pos"].grad.numpy(), rtol=1e-13, atol=1e-13)
    # output layer and loss: this micro-batch is a third of the batch
    n_total = 3 * tok.numel()
    y = rng.standard_normal(x.shape)
    yt = torch.tensor(y, requires_grad=True)
    hn = torch.nn.functional.layer_norm(yt, (y.shape[-1],), t["lnf_g"], t["lnf_b"], 1e-5)
    z = torch.nn.functional.linear(hn, t["w_out"])
    loss_t = torch.nn.functional.cross_entropy(z.reshape(-1, z.shape[-1]), lab.reshape(-1), reduction="sum") / n_total
    for k in t:
        t[k].grad = None
    loss_t.backward()
    loss, dy, G = V.head_loss_fwd_bwd(vp, y, labels[0], n_total)
    assert abs(loss - loss_t.item()) <= 1e-13 * abs(loss)
    assert np.allclose(dy, yt.grad.numpy(), rtol=1e-11, atol=1e-14)
    for k in ("lnf_g", "lnf_b", "w_out"):
        assert np.allclose(G[k], t[k].grad.numpy(), rtol=1e-11, atol=1e-14), k


def test_uniform_logits_give_log_vocabulary():
    """w_out = 0: every token is equally likely, the loss is log S_voc whatever the input."""
    _, vp, tokens, labels = _setup()
    vp["w_out"] = np.zeros_like(vp["w_out"])
    y = np.random.default_rng(1).standard_normal((2, 6, 16))
    loss, dy, G = V.head_loss_fwd_bwd(vp, y, labels[0], labels[0].size)
    assert abs(loss - np.log(37)) < 1e-12
    assert np.abs(dy).max() == 0


def test_lm_step_loss_gradient_by_finite_differences_and_both_orders():
    params, vp, tokens, labels = _setup()
    r = K.run_lm_step(params, vp, tokens, labels, K.SCHED_BF, 2, 2)
    d = K.run_lm_step(params, vp, tokens, labels, K.SCHED_DF, 2, 2)
    assert r["loss"] == d["loss"] and abs(r["loss_mb"].sum() - r["loss"]) < 1e-15
    for k in vp:
        assert np.array_equal(r["vgrads"][k], d["vgrads"][k]), k
    for l in range(2):
        for k in params[l]:
            assert np.array_equal(r["grads"][l][k], d["grads"][l][k]), (l, k)
    # one batch of N_mb * S_mb samples gives the same loss: the micro-batch split is only bookkeeping
    flat = lambda a: a.reshape(1, -1, a.shape[-1])
    one = K.run_lm_step(params, vp, flat(tokens), flat(labels), K.SCHED_BF, 1, 2)
    assert abs(one["loss"] - r["loss"]) < 1e-13
    for k in vp:
        assert np.allclose(one["vgrads"][k], r["vgrads"][k], rtol=1e-10, atol=1e-13), k

    def loss_at(vp2, params2):
        return K.run_lm_step(params2, vp2, tokens, labels, K.SCHED_BF, 2, 2)["loss"]

    rng = np.random.default_rng(2)
    eps = 1e-6
    used = np.unique(tokens)
    for k in vp:
        for _ in range(3):
            idx = tuple(rng.integers(0, n) for n in vp[k].shape)
            if k == "e_tok":
                idx = (int(rng.choice(used)),) + idx[1:]       # a row that is looked up at least once
            hi, lo = {**vp}, {**vp}
            hi[k] = vp[k].copy(); hi[k][idx] += eps
            lo[k] = vp[k].copy(); lo[k][idx] -= eps
            fd = (loss_at(hi, params) - loss_at(lo, params)) / (2 * eps)
            assert abs(fd - r["vgrads"][k][idx]) <= 1e-6 * max(1e-3, abs(fd)), (k, idx, fd, r["vgrads"][k][idx])
    # a layer weight, through the whole stack: the head's dy feeds the stages' backward
    for k in ("w_fc2", "ln1_g", "w_qkv"):
        idx = tuple(rng.integers(0, n) for n in params[1][k].shape)
        hi = [dict(p) for p in params]; lo = [dict(p) for p in params]
        hi[1][k] = params[1][k].copy(); hi[1][k][idx] += eps
        lo[1][k] = params[1][k].copy(); lo[1][k][idx] -= eps
        fd = (loss_at(vp, hi) - loss_at(vp, lo)) / (2 * eps)
        assert abs(fd - r["grads"][1][k][idx]) <= 1e-6 * max(1e-3, abs(fd)), (k, idx)
    # a token never looked up gets no gradient
    unused = np.setdiff1d(np.arange(37), used)
    if unused.size:
        assert np.abs(r["vgrads"]["e_tok"][unused]).max() == 0
