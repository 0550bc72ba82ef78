"""Input and output layers of the language model, forward and backward, in float64 numpy.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

App. A.1 ("Setup") names them only as the input and output layers that may be attached to
the first and last stage; Eq. compute prices the output projection with its
S_voc / (16 N_layers) term.  Readings taken here (GPT-2 style, nothing fused):

  * input:   x[b, i, :] = E_tok[token[b, i], :] + E_pos[i, :]
  * output:  z = LN_f(y) W_out^T,  W_out [S_voc, S_hidden] separate from E_tok (untied)
  * loss:    mean over every token of the batch of the cross-entropy of softmax(z) against
             the label; a micro-batch contributes sum(ce) / n_tokens_total, so the
             micro-batch losses add up to the batch loss and their gradients to its gradient
  * labels are token ids in 0..S_voc-1 (no ignored positions)
"""
import numpy as np

from . import layer as L

VOCAB_PARAM_NAMES = ("e_tok", "e_pos", "lnf_g", "lnf_b", "w_out")


def vocab_param_shapes(S_voc, S_seq, S_hidden):
    return {"e_tok": (S_voc, S_hidden), "e_pos": (S_seq, S_hidden), "lnf_g": (S_hidden,), "lnf_b": (S_hidden,),
            "w_out": (S_voc, S_hidden)}


def embedding_fwd(vp, tokens):
    """tokens int [S_mb, S_seq] -> x [S_mb, S_seq, S_hidden]."""
    S_seq = tokens.shape[1]
    return vp["e_tok"][tokens] + vp["e_pos"][:S_seq][None, :, :]


def embedding_bwd(vp, tokens, dx):
    """Gradients of e_tok and e_pos: every use of a row adds its dx row (ascending position)."""
    g_tok = np.zeros_like(vp["e_tok"])
    g_pos = np.zeros_like(vp["e_pos"])
    S_mb, S_seq = tokens.shape
    for b in range(S_mb):
        for i in range(S_seq):
            g_tok[tokens[b, i]] += dx[b, i]
            g_pos[i] += dx[b, i]
    return {"e_tok": g_tok, "e_pos": g_pos}


def head_loss_fwd_bwd(vp, y, labels, n_tokens_total, eps=1e-5):
    """Final LayerNorm, output projection, softmax cross-entropy.

    y [S_mb, S_seq, S_hidden], labels int [S_mb, S_seq].
    Returns (loss contribution of this micro-batch, dy, grads of lnf_g / lnf_b / w_out)."""
    hn, saved = L.layernorm_fwd(y, vp["lnf_g"], vp["lnf_b"], eps)
    z = hn @ vp["w_out"].T                                   # [S_mb, S_seq, S_voc]
    zmax = z.max(axis=-1, keepdims=True)
    lse = zmax[..., 0] + np.log(np.exp(z - zmax).sum(axis=-1))
    picked = np.take_along_axis(z, labels[..., None], axis=-1)[..., 0]
    loss = (lse - picked).sum() / n_tokens_total
    p = np.exp(z - lse[..., None])
    dz = p
    np.put_along_axis(dz, labels[..., None], np.take_along_axis(p, labels[..., None], axis=-1) - 1.0, axis=-1)
    dz = dz / n_tokens_total
    S_voc, h = vp["w_out"].shape
    g_w = dz.reshape(-1, S_voc).T @ hn.reshape(-1, h)
    dhn = dz @ vp["w_out"]
    dy, dg, db = L.layernorm_bwd(dhn, vp["lnf_g"], saved)
    return loss, dy, {"lnf_g": dg, "lnf_b": db, "w_out": g_w}
