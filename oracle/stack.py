"""One pipeline rank's training step in breadth-first or depth-first order.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The rank holds N_layers identical layers split into N_loop contiguous stages
(Sec. 4.1: N_loop = N_stage / N_PP).  On one device the stages are chained, which
is the N_PP = 1 case the paper calls breadth-first gradient accumulation (App. C).
What is computed is ordinary gradient accumulation over N_mb micro-batches:

    Y_m = Layer_{N-1}( ... Layer_0(X_m)),    L = sum_m <Y_m, dY_m>
    G_l = sum_{m ascending} d<Y_m, dY_m>/d theta_l,   dX_m = dL/dX_m
    then one Adam step per parameter with G (plain sum, no 1/N_mb).

The two orders (Sec. 4.1):
  BF  every micro-batch through a stage before the next stage, forward first;
      backward stage by stage from the last, a stage's gradient is final after
      its N_mb backwards and its optimizer step fires there.
  DF  (N_PP = 1) each micro-batch goes through the whole forward and the whole
      backward before the next one starts; a stage's gradient is final only in
      the last micro-batch's backward.
Within a stage the micro-batches are always taken in ascending order, so both
orders add the same numbers in the same sequence and G is bitwise equal.

The integer event trace records (op, stage, mb, live) where live is the number
of activation checkpoints (one per layer and micro-batch, Eq. mem_ckpt in
App. A.2.2) alive after the event.
"""
import numpy as np

from . import layer as L

OP_F, OP_B, OP_OPT = 0, 1, 2
SCHED_BF, SCHED_DF = 0, 1


def stage_layers(N_layers, N_loop, s):
    if N_layers % N_loop:
        raise ValueError("N_layers must be a multiple of N_loop")
    per = N_layers // N_loop
    return range(s * per, (s + 1) * per)


def event_order(schedule, N_loop, N_mb):
    """The ordered (op, stage, mb) list of one step; OPT events carry mb = -1."""
    ev = []
    if schedule == SCHED_BF:
        for s in range(N_loop):
            for m in range(N_mb):
                ev.append((OP_F, s, m))
        for s in reversed(range(N_loop)):
            for m in range(N_mb):
                ev.append((OP_B, s, m))
            ev.append((OP_OPT, s, -1))
    elif schedule == SCHED_DF:
        for m in range(N_mb):
            for s in range(N_loop):
                ev.append((OP_F, s, m))
            for s in reversed(range(N_loop)):
                ev.append((OP_B, s, m))
                if m == N_mb - 1:
                    ev.append((OP_OPT, s, -1))
    else:
        raise ValueError("schedule")
    return ev


def adam_update(w, g, m, v, t, lr, beta1, beta2, adam_eps, weight_decay=0.0):
    """Bias-corrected Adam (Kingma & Ba, Alg. 1), step counter t >= 1.

    weight_decay is the decoupled (AdamW) kind: w -= lr * weight_decay * w.
    Returns new (w, m, v).
    """
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    w = w - lr * (mhat / (np.sqrt(vhat) + adam_eps) + weight_decay * w)
    return w, m, v


def run_step(params, x, dy, schedule, N_loop, N_heads, eps=1e-5, causal=True,
             gelu_form="tanh", adam=None, adam_state=None):
    """Executes one step in the given order.

    params: list (one per layer) of dicts name -> float64 array
    x, dy:  [N_mb, S_mb, S_seq, S_hidden]; dy may instead be a function (m, y_m) -> dy_m that is
            called when micro-batch m leaves the last stage (an output layer and loss attached to it)
    adam:   None (no optimizer step) or dict(lr, beta1, beta2, adam_eps, weight_decay, t)
    adam_state: list of dicts name -> (m, v); zeros if None
    Returns dict(y, dx, grads, trace, peak_ckpt, new_params, new_adam_state)
    """
    N_layers = len(params)
    N_mb = x.shape[0]
    y = np.zeros_like(x)
    dx = np.zeros_like(x)
    grads = [None] * N_layers                 # main-grad buffers, created by the first micro-batch
    caches = {}                               # (layer, mb) -> cache; its presence = one live checkpoint
    hand = {}                                 # mb -> tensor handed from stage s to s+1 (forward) / s to s-1 (backward)
    bhand = {}
    dy_of = {}
    new_params = [dict(p) for p in params]
    if adam_state is None:
        adam_state = [{k: (np.zeros_like(v), np.zeros_like(v)) for k, v in p.items()} for p in params]
    new_state = [dict(s) for s in adam_state]
    trace = []
    peak = 0

    for op, s, m in event_order(schedule, N_loop, N_mb):
        if op == OP_F:
            t = x[m] if s == 0 else hand[m]
            for l in stage_layers(N_layers, N_loop, s):
                t, caches[(l, m)] = L.layer_fwd(params[l], t, N_heads, eps, causal, gelu_form)
            hand[m] = t
            if s == N_loop - 1:
                y[m] = t
                if callable(dy):
                    dy_of[m] = dy(m, t)
        elif op == OP_B:
            d = (dy_of[m] if callable(dy) else dy[m]) if s == N_loop - 1 else bhand[m]
            for l in reversed(stage_layers(N_layers, N_loop, s)):
                d, G = L.layer_bwd(params[l], caches.pop((l, m)), d, N_heads)
                if grads[l] is None:
                    grads[l] = G                       # first micro-batch writes
                else:
                    for k in G:
                        grads[l][k] = grads[l][k] + G[k]   # later ones add, ascending m
            bhand[m] = d
            if s == 0:
                dx[m] = d
        else:  # OP_OPT: this stage's gradients are final
            if adam is not None:
                for l in stage_layers(N_layers, N_loop, s):
                    for k in params[l]:
                        mm, vv = adam_state[l][k]
                        w2, m2, v2 = adam_update(params[l][k], grads[l][k], mm, vv, adam["t"], adam["lr"],
                                                 adam["beta1"], adam["beta2"], adam["adam_eps"],
                                                 adam.get("weight_decay", 0.0))
                        new_params[l][k] = w2
                        new_state[l][k] = (m2, v2)
        live = len(caches)
        peak = max(peak, live)
        trace.append((op, s, m, live))
    return dict(y=y, dx=dx, grads=grads, trace=trace, peak_ckpt=peak,
                new_params=new_params, new_adam_state=new_state)


def run_one_big_batch(params, x, dy, N_heads, eps=1e-5, causal=True, gelu_form="tanh"):
    """The same gradient computed without any schedule: all N_mb*S_mb samples as
    one batch through all layers.  Used only as a pin for run_step."""
    N_mb, S_mb = x.shape[:2]
    t = x.reshape((N_mb * S_mb,) + x.shape[2:])
    d = dy.reshape(t.shape)
    caches = []
    for p in params:
        t, c = L.layer_fwd(p, t, N_heads, eps, causal, gelu_form)
        caches.append(c)
    grads = [None] * len(params)
    for l in reversed(range(len(params))):
        d, grads[l] = L.layer_bwd(params[l], caches[l], d, N_heads)
    return dict(y=t.reshape(x.shape), dx=d.reshape(x.shape), grads=grads)


def run_rank_step(params, x, dy, kind, N_PP, rank, N_loop, N_heads, eps=1e-5, causal=True, gelu_form="tanh"):
    """One step of rank `rank` of an N_PP-deep looped pipeline (Sec. 4.1, Sec. 4.2), the other ranks
    absent: the rank's local stage l (global stage l N_PP + rank, the layers stage_layers(.., l) of
    `params`) takes its input x[l, m] and the gradient dy[l, m] of its output from outside and hands
    y[l, m], dx[l, m] back.  Ops run in the order of schedule.device_order (kind "BF" or "DF").

    x, dy: [N_loop, N_mb, S_mb, S_seq, S_hidden].
    Returns dict(y, dx, grads, trace, peak_ckpt); trace entries (op, global stage, mb, live
    checkpoints), with an OP_OPT entry after the last backward of each stage."""
    from . import schedule as S
    N_layers = len(params)
    N_mb = x.shape[1]
    y = np.zeros_like(x)
    dx = np.zeros_like(x)
    grads = [None] * N_layers
    caches = {}
    trace = []
    peak = 0
    for op, stage, m in S.device_order(kind, N_PP, N_loop, N_mb, rank):
        l_loc = (stage - rank) // N_PP
        if op == OP_F:
            t = x[l_loc, m]
            for l in stage_layers(N_layers, N_loop, l_loc):
                t, caches[(l, m)] = L.layer_fwd(params[l], t, N_heads, eps, causal, gelu_form)
            y[l_loc, m] = t
        else:
            d = dy[l_loc, m]
            for l in reversed(stage_layers(N_layers, N_loop, l_loc)):
                d, G = L.layer_bwd(params[l], caches.pop((l, m)), d, N_heads)
                if grads[l] is None:
                    grads[l] = G
                else:
                    for k in G:
                        grads[l][k] = grads[l][k] + G[k]
            dx[l_loc, m] = d
        peak = max(peak, len(caches))
        trace.append((op, stage, m, len(caches)))
        if op == OP_B and m == N_mb - 1:
            trace.append((OP_OPT, stage, -1, len(caches)))
    return dict(y=y, dx=dx, grads=grads, trace=trace, peak_ckpt=peak)


def run_lm_step(params, vparams, tokens, labels, schedule, N_loop, N_heads, eps=1e-5, causal=True, gelu_form="tanh"):
    """The step on token ids: input layer attached to the first stage, output layer and loss to
    the last (App. A.1; Eq. compute's S_voc term).  The loss gradient of a micro-batch is taken as
    soon as the micro-batch leaves the last stage's forward; the input layer's gradient after the
    first stage's backward.

    vparams: dict e_tok, e_pos, lnf_g, lnf_b, w_out (float64); tokens, labels int [N_mb, S_mb, S_seq].
    Returns run_step's dict plus loss (batch mean), loss_mb [N_mb], vgrads (dict like vparams)."""
    from . import vocab as V
    N_mb = tokens.shape[0]
    n_total = tokens.size
    x = np.stack([V.embedding_fwd(vparams, tokens[m]) for m in range(N_mb)])
    loss_mb = np.zeros(N_mb)
    vgrads = {}

    def add(G):
        for k, g in G.items():
            vgrads[k] = g if k not in vgrads else vgrads[k] + g      # ascending micro-batch order

    def head(m, y_m):
        loss_mb[m], dy_m, G = V.head_loss_fwd_bwd(vparams, y_m, labels[m], n_total, eps)
        add(G)
        return dy_m

    r = run_step(params, x, head, schedule, N_loop, N_heads, eps, causal, gelu_form)
    for m in range(N_mb):
        add(V.embedding_bwd(vparams, tokens[m], r["dx"][m]))
    r.update(loss=loss_mb.sum(), loss_mb=loss_mb, vgrads=vgrads, x=x)
    return r
