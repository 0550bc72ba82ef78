"""Unit-time simulation of the four pipeline schedules for N_PP >= 1.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

N_stage = N_PP * N_loop stages are wrapped round N_PP devices (Sec. 4.1): stage j
lives on device j mod N_PP.  A forward of one stage for one micro-batch takes
t_fwd ticks, a backward t_bwd; transfers take no time.  Each device walks a
fixed op list and starts an op as soon as it is free and the op's producer is
done:  F(j, m) needs F(j-1, m);  B(j, m) needs B(j+1, m) (and F(j, m)).

Orders
  "BF"  forward-first, earlier stages first, all micro-batches at once
        (GPipe when N_loop = 1).
  "DF"  backward-first, earlier micro-batches first, in sequences of N_PP
        micro-batches (1F1B when N_loop = 1); needs N_mb % N_PP == 0.  The paper
        takes this schedule from earlier work and does not restate its warm-up
        depth; the one used here is the usual interleaved one: device r runs
        2 (N_PP - r - 1) + (N_loop - 1) N_PP forwards (N_PP - r - 1 when
        N_loop = 1), then alternates one forward, one backward.  With N_PP = 1
        there is nothing to interleave and the order is the one of App. C: each
        micro-batch through every stage forward and backward before the next.

Reported: the bubble as an exact fraction idle / busy of one device (Eq. bubble,
Eq. bubble_looped) and the peak number of live (stage, micro-batch) inputs per
device, from which the checkpoint count of Eq. mem_ckpt follows by multiplying
with the layers per stage.
"""
from fractions import Fraction

OP_F, OP_B = 0, 1


def device_order(kind, N_PP, N_loop, N_mb, rank):
    """Ordered list of (op, global stage, mb) that device `rank` executes."""
    if kind == "BF":
        if N_mb < N_PP:
            raise ValueError("BF needs N_mb >= N_PP")
        ops = [(OP_F, l * N_PP + rank, m) for l in range(N_loop) for m in range(N_mb)]
        ops += [(OP_B, l * N_PP + rank, m) for l in reversed(range(N_loop)) for m in range(N_mb)]
        return ops
    if kind != "DF":
        raise ValueError(kind)
    if N_mb % N_PP:
        raise ValueError("DF needs N_mb to be a multiple of N_PP")
    if N_PP == 1:
        # App. C: a micro-batch runs its whole forward and backward before the next begins
        ops = []
        for m in range(N_mb):
            ops += [(OP_F, l, m) for l in range(N_loop)]
            ops += [(OP_B, l, m) for l in reversed(range(N_loop))]
        return ops
    total = N_loop * N_mb
    seq = N_PP * N_loop                       # slots per sequence of N_PP micro-batches

    def slot(i, backward):
        g, r = divmod(i, seq)
        l, j = divmod(r, N_PP)
        if backward:
            l = N_loop - 1 - l
        return l * N_PP + rank, g * N_PP + j

    fwd = [(OP_F,) + slot(i, False) for i in range(total)]
    bwd = [(OP_B,) + slot(i, True) for i in range(total)]
    if N_loop == 1:
        warm = N_PP - rank - 1
    else:
        warm = 2 * (N_PP - rank - 1) + (N_loop - 1) * N_PP
    warm = min(warm, total)
    ops = fwd[:warm]
    fi, bi = warm, 0
    while fi < total:
        ops.append(fwd[fi]); fi += 1
        ops.append(bwd[bi]); bi += 1
    ops += bwd[bi:]
    return ops


def simulate(kind, N_PP, N_loop, N_mb, t_fwd=1, t_bwd=2):
    """Runs the schedule; returns dict(makespan, busy, bubble, peak_live, events).

    events: per device, list of (start, op, stage, mb); peak_live: per device, the
    largest number of (stage, mb) pairs whose forward has started and whose
    backward has not finished.
    """
    N_stage = N_PP * N_loop
    orders = [device_order(kind, N_PP, N_loop, N_mb, r) for r in range(N_PP)]
    ptr = [0] * N_PP
    free = [0] * N_PP
    done = {}                                  # (op, stage, mb) -> finish time
    events = [[] for _ in range(N_PP)]
    remaining = sum(len(o) for o in orders)
    while remaining:
        progressed = False
        for r in range(N_PP):
            while ptr[r] < len(orders[r]):
                op, j, m = orders[r][ptr[r]]
                if op == OP_F:
                    dep = None if j == 0 else (OP_F, j - 1, m)
                else:
                    dep = (OP_F, j, m) if j == N_stage - 1 else (OP_B, j + 1, m)
                if dep is not None and dep not in done:
                    break
                ready = 0 if dep is None else done[dep]
                start = max(free[r], ready)
                dur = t_fwd if op == OP_F else t_bwd
                free[r] = start + dur
                done[(op, j, m)] = free[r]
                events[r].append((start, op, j, m))
                ptr[r] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise RuntimeError("schedule deadlocks")
    makespan = max(free)
    busy = N_loop * N_mb * (t_fwd + t_bwd)
    peak_live = []
    for r in range(N_PP):
        live = peak = 0
        for _, op, _, _ in events[r]:          # in issue order on this device
            if op == OP_F:
                live += 1
                peak = max(peak, live)
            else:
                live -= 1
        peak_live.append(peak)
    return dict(makespan=makespan, busy=busy, bubble=Fraction(makespan - busy, busy),
                peak_live=peak_live, events=events)


def weight_intervals(ops):
    """Intervals over which a device needs one stage's weights: maximal runs of consecutive
    ops of one stage in one direction.  With fully sharded data parallelism the stage is
    reconstructed for each such interval (Sec. 3.1: before every use, forward and backward);
    breadth-first has one forward and one backward interval per stage, the other orders
    repeat them per micro-batch or micro-batch sequence (Sec. 4.2).
    Returns the list of (op, stage, first index, length)."""
    out = []
    for i, (op, stage, _m) in enumerate(ops):
        if out and out[-1][0] == op and out[-1][1] == stage:
            out[-1][3] += 1
        else:
            out.append([op, stage, i, 1])
    return [tuple(v) for v in out]


def reconstructions(ops, n_buffers=2, resident=()):
    """Reconstructions a device runs when it keeps the weights of the n_buffers most recently
    used stages (App. D.1: a double buffer, one half computing while the other is restored):
    an interval whose stage is still held costs nothing, otherwise the stage replaces the one
    unused for longest.  `resident`: stages held at the start, least recently used first.
    Returns (count, stages held at the end in the same order)."""
    held = list(resident)[-n_buffers:]
    count = 0
    for _op, stage, _i, _n in weight_intervals(ops):
        if stage in held:
            held.remove(stage)
        else:
            count += 1
            if len(held) == n_buffers:
                held.pop(0)
        held.append(stage)
    return count, tuple(held)
