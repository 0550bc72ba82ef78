"""ctypes binding of libbf.so: argument marshalling only.  Every step of the path runs in
the library's HIP kernels; torch is used for device memory and streams.  There is no CPU
fallback: a missing library is an ImportError at load()."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libbf.so")

BF_OK, BF_EINVAL, BF_ENOMEM, BF_ESTATE, BF_EDEVICE = 0, -1, -2, -3, -4
BF_SCHED_BF, BF_SCHED_DF = 0, 1
BF_FP32, BF_BF16 = 0, 1
BF_CKPT_NONE, BF_CKPT_LAYER = 0, 1
BF_KERNELS_AUTO, BF_KERNELS_PLAIN = 0, 1
BF_NN, BF_NT, BF_TN = 0, 1, 2
BF_EPI_NONE, BF_EPI_BIAS, BF_EPI_BIAS_RES, BF_EPI_BIAS_GELU, BF_EPI_GELU_BWD, BF_EPI_ACCUM = range(6)
VOCAB_TENSOR_IDS = {"e_tok": 12, "e_pos": 13, "lnf_g": 14, "lnf_b": 15, "w_out": 16}
TENSOR_IDS = {"ln1_g": 0, "ln1_b": 1, "w_qkv": 2, "b_qkv": 3, "w_o": 4, "b_o": 5,
              "ln2_g": 6, "ln2_b": 7, "w_fc1": 8, "b_fc1": 9, "w_fc2": 10, "b_fc2": 11}


class bf_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("S_hidden", "N_heads", "S_head", "S_mlp", "S_seq", "N_layers", "N_mb_max",
                                         "S_mb_max", "dtype", "ckpt_mode", "causal", "kernels", "queue_depth",
                                         "fuse_wgrad", "N_loop_min", "dp_fs", "S_voc")] + \
               [("seed", C.c_uint64)] + \
               [(n, C.c_float) for n in ("init_std", "ln_eps", "lr", "beta1", "beta2", "adam_eps", "weight_decay")] + \
               [("mb_chains", C.c_int32)]


class bf_event(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("op", "stage", "mb", "live_ckpt")]


class bf_step_report(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("gpu_ms", "adam_ms", "flops_model", "flops_paper", "flops_executed")] + \
               [(n, C.c_int64) for n in ("peak_ckpt_count", "peak_ckpt_bytes", "peak_act_bytes", "state_bytes")] + \
               [("n_events", C.c_int32), ("timed", C.c_int32)] + \
               [("kernel_ms", C.c_double * 11), ("kernel_flops", C.c_double * 11), ("kernel_bytes", C.c_double * 11),
                ("kernel_launches", C.c_int64 * 11)] + \
               [(n, C.c_int64) for n in ("n_weight_intervals", "n_reconstruct", "reconstruct_bytes", "weight_buffer_bytes",
                                         "fused_wgrad_bytes", "mb_chains")]


KERNEL_CLASSES = ("gemm_fwd", "gemm_dgrad", "gemm_wgrad", "attn_fwd", "attn_bwd", "ln_fwd", "ln_bwd", "colsum", "adam",
                  "reconstruct", "vocab")


BF_METHOD_NO_PIPELINE, BF_METHOD_NON_LOOPED, BF_METHOD_DEPTH_FIRST, BF_METHOD_BREADTH_FIRST = range(4)


class bf_calc_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("method", "N_PP", "N_loop", "N_TP", "N_layers", "N_mb", "S_mb", "sharded",
                                         "overlap")] + [("beta_net", C.c_double)]


class bf_calc_point(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("beta", "bubble", "net_ratio", "overlap_share", "net_overhead", "efficiency")]


class bf_sched_stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("makespan", "busy", "bubble_num", "bubble_den", "peak_live")]


_P = C.c_void_p
_FP = C.POINTER(C.c_float)
_SIGNATURES = {
    "bf_workspace_bytes": (C.c_size_t, [C.POINTER(bf_config)]),
    "bf_create_stack": (C.c_int, [C.POINTER(bf_config), _P, C.c_size_t, _P, C.POINTER(_P)]),
    "bf_destroy_stack": (C.c_int, [_P]),
    "bf_tensor_elems": (C.c_size_t, [_P, C.c_int]),
    "bf_set_params": (C.c_int, [_P, C.c_int, C.c_int, _P, C.c_size_t]),
    "bf_get_params": (C.c_int, [_P, C.c_int, C.c_int, _P, C.c_size_t]),
    "bf_get_grads": (C.c_int, [_P, C.c_int, C.c_int, _P, C.c_size_t]),
    "bf_get_moments": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, _P, C.c_size_t]),
    "bf_reset_optimizer": (C.c_int, [_P]),
    "bf_run_step": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, C.c_int, _P, _P, _P, _P, C.c_int, C.c_int, _P,
                              C.POINTER(bf_step_report)]),
    "bf_run_lm_step": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, C.c_int, _P, _P, _P, C.c_int, C.c_int, _P,
                                 C.POINTER(bf_step_report)]),
    "bf_run_rank_step": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _P, _P, _P, _P, C.c_int, C.c_int, _P,
                              C.POINTER(bf_step_report)]),
    "bf_get_trace": (C.c_int, [_P, C.POINTER(bf_event), C.c_size_t, C.POINTER(C.c_size_t)]),
    "bf_schedule_trace": (C.c_int, [C.c_int] * 7 + [C.POINTER(bf_event), C.c_size_t, C.POINTER(C.c_size_t),
                                                    C.POINTER(bf_sched_stats)]),
    "bf_param_count": (C.c_int64, [C.POINTER(bf_config)]),
    "bf_calc_efficiency": (C.c_int, [C.POINTER(bf_calc_config), C.POINTER(bf_calc_point)]),
    "bf_calc_efficiency_curve": (C.c_int, [C.POINTER(bf_calc_config), C.POINTER(C.c_int32), C.c_size_t,
                                           C.POINTER(bf_calc_point)]),
    "bf_calc_beta_threshold": (C.c_int, [C.POINTER(bf_calc_config), C.POINTER(C.c_double)]),
    "bf_calc_cost_time": (C.c_int, [C.c_double] * 4 + [C.POINTER(C.c_double)] * 2),
    "bf_last_error": (C.c_char_p, []),
    "bf_op_gemm": (C.c_int, [C.c_int] * 7 + [_P] * 6 + [C.c_int, _P]),
    "bf_op_gemm_gelu_bwd_colsum": (C.c_int, [C.c_int] * 5 + [_P] * 6 + [C.c_int, _P]),
    "bf_op_gemm_uses_mfma": (C.c_int, [C.c_int] * 5),
    "bf_op_gemm_tile": (C.c_int, [C.c_int] * 5 + [C.POINTER(C.c_int)] * 2),
    "bf_op_wgrad": (C.c_int, [C.c_int] * 6 + [_P, C.c_size_t, _P, C.c_size_t, _P, _P, C.c_int, _P]),
    "bf_op_layernorm_fwd": (C.c_int, [C.c_int, C.c_int, C.c_int, _P, _P, _P, C.c_float, _P, _P, _P]),
    "bf_op_layernorm_bwd": (C.c_int, [C.c_int, C.c_int, C.c_int] + [_P] * 8 + [C.c_int, _P]),
    "bf_op_layernorm_bwd_fused": (C.c_int, [C.c_int, C.c_int, C.c_int] + [_P] * 10 + [C.c_int, _P]),
    "bf_op_layernorm_bwd_part_elems": (C.c_size_t, [C.c_int, C.c_int]),
    "bf_op_colsum": (C.c_int, [C.c_int, C.c_int, C.c_int, _P, _P, C.c_int, _P]),
    "bf_op_attention_fwd": (C.c_int, [C.c_int] * 7 + [_P] * 4),
    "bf_op_attention_bwd": (C.c_int, [C.c_int] * 7 + [_P] * 7),
    "bf_op_attention_bwd_static": (C.c_int, [C.c_int] * 7 + [_P] * 6),
    "bf_op_gemm_splitk": (C.c_int, [C.c_int] * 7 + [_P] * 6 + [C.c_size_t, _P]),
    "bf_op_gemm_splitk_slices": (C.c_int, [C.c_int] * 5),
    "bf_op_attention_bwd_bias": (C.c_int, [C.c_int] * 7 + [_P] * 8 + [C.c_int, _P]),
    "bf_op_attention_bwd_part_elems": (C.c_size_t, [C.c_int] * 4),
    "bf_op_attention_uses_mfma": (C.c_int, [C.c_int, C.c_int]),
    "bf_op_embedding_fwd": (C.c_int, [C.c_int] * 5 + [_P, _P, _P, _P, _P]),
    "bf_op_embedding_bwd": (C.c_int, [C.c_int] * 5 + [_P, _P, _P, _P, C.c_int, _P]),
    "bf_op_ce_loss": (C.c_int, [C.c_int] * 3 + [_P, _P, C.c_float, _P, _P, _P]),
    "bf_op_adam": (C.c_int, [C.c_size_t, _P, _P, _P, _P, _P, C.c_int] + [C.c_float] * 5 + [_P]),
}

_lib = None


class BfError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("libbf status %d: %s" % (status, text))
        self.status = status


def load():
    """Loads libbf.so (built by paper_2211_05953_amd.build); raises ImportError if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libbf.so is not built: run `python -m paper_2211_05953_amd.build`")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def last_error():
    return load().bf_last_error().decode()


def check(status):
    if status != BF_OK:
        raise BfError(status, last_error())


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / None."""
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def make_config(S_hidden, N_heads, S_mlp, S_seq, N_layers, N_mb_max, S_mb_max, dtype=BF_BF16, ckpt_mode=BF_CKPT_NONE,
                causal=1, kernels=BF_KERNELS_AUTO, queue_depth=0, fuse_wgrad=0, N_loop_min=0, dp_fs=0, S_voc=0, seed=0x221105953, init_std=0.02, ln_eps=1e-5,
                lr=1e-4, beta1=0.9, beta2=0.999, adam_eps=1e-8, weight_decay=0.0, mb_chains=1):
    return bf_config(S_hidden, N_heads, S_hidden // N_heads, S_mlp, S_seq, N_layers, N_mb_max, S_mb_max, dtype,
                     ckpt_mode, causal, kernels, queue_depth, fuse_wgrad, N_loop_min, dp_fs, S_voc, seed, init_std, ln_eps, lr, beta1, beta2, adam_eps,
                     weight_decay, mb_chains)


def bf_workspace_bytes(cfg):
    return load().bf_workspace_bytes(C.byref(cfg))


def bf_param_count(cfg):
    return load().bf_param_count(C.byref(cfg))


class Stack:
    """Owns the torch-allocated workspace and the opaque bf_stack handle."""

    def __init__(self, cfg, device="cuda:0"):
        import torch
        lib = load()
        self.cfg = cfg
        n = lib.bf_workspace_bytes(C.byref(cfg))
        if n == 0:
            raise BfError(BF_EINVAL, last_error())
        self.workspace = torch.empty(n, dtype=torch.uint8, device=device)
        self.handle = _P()
        with torch.cuda.device(self.workspace.device):
            check(lib.bf_create_stack(C.byref(cfg), self.workspace.data_ptr(), n, _stream(), C.byref(self.handle)))
        self.torch_dtype = torch.bfloat16 if cfg.dtype == BF_BF16 else torch.float32

    def close(self):
        if self.handle:
            load().bf_destroy_stack(self.handle)
            self.handle = _P()
            self.workspace = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def bf_tensor_elems(self, tensor_id):
        return load().bf_tensor_elems(self.handle, tensor_id)

    def _xfer(self, fn, layer, tensor_id, arr, *extra):
        import numpy as np
        assert arr.dtype == np.float32 and arr.flags["C_CONTIGUOUS"]
        check(fn(self.handle, layer, tensor_id, *extra, arr.ctypes.data, arr.size))

    def bf_set_params(self, layer, tensor_id, host_src):
        import numpy as np
        self._xfer(load().bf_set_params, layer, tensor_id, np.ascontiguousarray(host_src, dtype=np.float32))

    def _get(self, fn, layer, tensor_id, *extra):
        import numpy as np
        out = np.empty(self.bf_tensor_elems(tensor_id), dtype=np.float32)
        self._xfer(fn, layer, tensor_id, out, *extra)
        return out

    def bf_get_params(self, layer, tensor_id):
        return self._get(load().bf_get_params, layer, tensor_id)

    def bf_get_grads(self, layer, tensor_id):
        return self._get(load().bf_get_grads, layer, tensor_id)

    def bf_get_moments(self, layer, tensor_id, which):
        return self._get(load().bf_get_moments, layer, tensor_id, which)

    def bf_reset_optimizer(self):
        check(load().bf_reset_optimizer(self.handle))

    def bf_run_step(self, schedule, N_loop, N_mb, S_mb, x, dy, y=None, dx=None, apply_optimizer=0, timing=0):
        rep = bf_step_report()
        check(load().bf_run_step(self.handle, schedule, N_loop, N_mb, S_mb, _ptr(x), _ptr(dy), _ptr(y), _ptr(dx),
                                 apply_optimizer, timing, _stream(), C.byref(rep)))
        return rep

    def bf_run_lm_step(self, schedule, N_loop, N_mb, S_mb, tokens, labels, loss, apply_optimizer=0, timing=0):
        rep = bf_step_report()
        check(load().bf_run_lm_step(self.handle, schedule, N_loop, N_mb, S_mb, _ptr(tokens), _ptr(labels), _ptr(loss),
                                    apply_optimizer, timing, _stream(), C.byref(rep)))
        return rep

    def bf_run_rank_step(self, schedule, N_PP, rank, N_loop, N_mb, S_mb, x, dy, y=None, dx=None, apply_optimizer=0,
                         timing=0):
        rep = bf_step_report()
        check(load().bf_run_rank_step(self.handle, schedule, N_PP, rank, N_loop, N_mb, S_mb, _ptr(x), _ptr(dy), _ptr(y),
                                      _ptr(dx), apply_optimizer, timing, _stream(), C.byref(rep)))
        return rep

    def bf_get_trace(self):
        n = C.c_size_t(0)
        check(load().bf_get_trace(self.handle, None, 0, C.byref(n)))
        buf = (bf_event * max(1, n.value))()
        check(load().bf_get_trace(self.handle, buf, n.value, C.byref(n)))
        return [(e.op, e.stage, e.mb, e.live_ckpt) for e in buf[:n.value]]


def bf_schedule_trace(schedule, N_PP, N_loop, N_mb, rank, t_fwd=1, t_bwd=2):
    """Returns (events, stats) of the pure-host schedule generator."""
    lib = load()
    n = C.c_size_t(0)
    check(lib.bf_schedule_trace(schedule, N_PP, N_loop, N_mb, rank, t_fwd, t_bwd, None, 0, C.byref(n), None))
    buf = (bf_event * max(1, n.value))()
    st = bf_sched_stats()
    check(lib.bf_schedule_trace(schedule, N_PP, N_loop, N_mb, rank, t_fwd, t_bwd, buf, n.value, C.byref(n), C.byref(st)))
    return [(e.op, e.stage, e.mb, e.live_ckpt) for e in buf[:n.value]], st


# ---- analytical calculators (include/bf_calc.h); host arithmetic only ------------------------
def _point(p):
    return {n: getattr(p, n) for n, _ in bf_calc_point._fields_}


def bf_calc_efficiency(method, N_PP, N_loop, N_TP, N_layers, N_mb, S_mb, sharded, overlap, beta_net):
    cfg = bf_calc_config(method, N_PP, N_loop, N_TP, N_layers, N_mb, S_mb, sharded, overlap, beta_net)
    out = bf_calc_point()
    check(load().bf_calc_efficiency(C.byref(cfg), C.byref(out)))
    return _point(out)


def bf_calc_efficiency_curve(method, N_PP, N_loop, N_TP, N_layers, S_mb, sharded, overlap, beta_net, n_mb):
    cfg = bf_calc_config(method, N_PP, N_loop, N_TP, N_layers, 1, S_mb, sharded, overlap, beta_net)
    counts = (C.c_int32 * len(n_mb))(*n_mb)
    out = (bf_calc_point * max(1, len(n_mb)))()
    check(load().bf_calc_efficiency_curve(C.byref(cfg), counts, len(n_mb), out))
    return [_point(p) for p in out[:len(n_mb)]]


def bf_calc_beta_threshold(method, N_PP, N_loop, N_TP, N_layers, N_mb, S_mb, sharded, overlap, beta_net):
    cfg = bf_calc_config(method, N_PP, N_loop, N_TP, N_layers, N_mb, S_mb, sharded, overlap, beta_net)
    out = C.c_double(0.0)
    check(load().bf_calc_beta_threshold(C.byref(cfg), C.byref(out)))
    return out.value


def bf_calc_cost_time(beta, N_gpu, B_crit, efficiency=1.0):
    cost, time = C.c_double(0.0), C.c_double(0.0)
    check(load().bf_calc_cost_time(beta, N_gpu, B_crit, efficiency, C.byref(cost), C.byref(time)))
    return cost.value, time.value


# ---- single kernels (include/bf_ops.h); tensors are torch CUDA tensors ----------------------
def bf_op_gemm(dtype, kernels, layout, epilogue, M, N, K, A, B, Cout, bias=None, R=None, C2=None, accumulate=0):
    check(load().bf_op_gemm(dtype, kernels, layout, epilogue, M, N, K, _ptr(A), _ptr(B), _ptr(Cout), _ptr(bias), _ptr(R),
                            _ptr(C2), accumulate, _stream()))


def bf_op_wgrad(dtype, kernels, M, N, K, n_seg, X, stride_x, dY, stride_dy, G, db=None, accumulate=0):
    check(load().bf_op_wgrad(dtype, kernels, M, N, K, n_seg, _ptr(X), stride_x, _ptr(dY), stride_dy, _ptr(G), _ptr(db),
                             accumulate, _stream()))


def bf_op_gemm_gelu_bwd_colsum(dtype, kernels, M, N, K, A, Bt, Cout, R, db, part=None, accumulate=0):
    check(load().bf_op_gemm_gelu_bwd_colsum(dtype, kernels, M, N, K, _ptr(A), _ptr(Bt), _ptr(Cout), _ptr(R), _ptr(db),
                                            _ptr(part), accumulate, _stream()))


def bf_op_gemm_splitk(dtype, kernels, layout, epilogue, M, N, K, A, B, Cout, bias=None, R=None, planes=None):
    opt = lambda t: _ptr(t) if t is not None else None
    check(load().bf_op_gemm_splitk(dtype, kernels, layout, epilogue, M, N, K, _ptr(A), _ptr(B), _ptr(Cout), opt(bias), opt(R),
                                   opt(planes), planes.numel() if planes is not None else 0, _stream()))


def bf_op_gemm_splitk_slices(layout, epilogue, M, N, K):
    return load().bf_op_gemm_splitk_slices(layout, epilogue, M, N, K)


def bf_op_gemm_uses_mfma(layout, epilogue, M, N, K):
    return bool(load().bf_op_gemm_uses_mfma(layout, epilogue, M, N, K))


def bf_op_gemm_tile(layout, epilogue, M, N, K):
    """(rows, columns) of the MFMA kernel's tile for this product, or None where the plain kernel runs."""
    bm, bn = C.c_int(0), C.c_int(0)
    ok = load().bf_op_gemm_tile(layout, epilogue, M, N, K, C.byref(bm), C.byref(bn))
    return (bm.value, bn.value) if ok else None


def bf_op_layernorm_fwd(dtype, T, h, x, g, b, eps, y, stats):
    check(load().bf_op_layernorm_fwd(dtype, T, h, _ptr(x), _ptr(g), _ptr(b), eps, _ptr(y), _ptr(stats), _stream()))


def bf_op_layernorm_bwd(dtype, T, h, dy, x, g, stats, dres, dx, dg, db, accumulate=0):
    check(load().bf_op_layernorm_bwd(dtype, T, h, _ptr(dy), _ptr(x), _ptr(g), _ptr(stats), _ptr(dres), _ptr(dx),
                                     _ptr(dg), _ptr(db), accumulate, _stream()))


def bf_op_layernorm_bwd_fused(dtype, T, h, dy, x, g, stats, dres, dx, dg, db, dcs=None, part=None, accumulate=0):
    check(load().bf_op_layernorm_bwd_fused(dtype, T, h, _ptr(dy), _ptr(x), _ptr(g), _ptr(stats), _ptr(dres), _ptr(dx),
                                           _ptr(dg), _ptr(db), _ptr(dcs), _ptr(part), accumulate, _stream()))


def bf_op_layernorm_bwd_part_elems(T, h):
    return load().bf_op_layernorm_bwd_part_elems(T, h)


def bf_op_colsum(dtype, T, N, dY, out, accumulate=0):
    check(load().bf_op_colsum(dtype, T, N, _ptr(dY), _ptr(out), accumulate, _stream()))


def bf_op_attention_fwd(dtype, kernels, S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse):
    check(load().bf_op_attention_fwd(dtype, kernels, S_mb, S_seq, N_heads, S_head, causal, _ptr(qkv), _ptr(ctx),
                                     _ptr(lse), _stream()))


def bf_op_attention_bwd(dtype, kernels, S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, dctx, dqkv, delta):
    check(load().bf_op_attention_bwd(dtype, kernels, S_mb, S_seq, N_heads, S_head, causal, _ptr(qkv), _ptr(ctx),
                                     _ptr(lse), _ptr(dctx), _ptr(dqkv), _ptr(delta), _stream()))


def bf_op_attention_bwd_bias(dtype, kernels, S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, dctx, dqkv, delta, db_qkv,
                             part=None, accumulate=0):
    check(load().bf_op_attention_bwd_bias(dtype, kernels, S_mb, S_seq, N_heads, S_head, causal, _ptr(qkv), _ptr(ctx),
                                          _ptr(lse), _ptr(dctx), _ptr(dqkv), _ptr(delta), _ptr(db_qkv),
                                          _ptr(part) if part is not None else None, int(accumulate), _stream()))


def bf_op_attention_bwd_part_elems(S_mb, S_seq, N_heads, S_head):
    return load().bf_op_attention_bwd_part_elems(S_mb, S_seq, N_heads, S_head)


def bf_op_attention_bwd_static(dtype, kernels, S_mb, S_seq, N_heads, S_head, causal, qkv, ctx, lse, dctx, dqkv):
    check(load().bf_op_attention_bwd_static(dtype, kernels, S_mb, S_seq, N_heads, S_head, causal, _ptr(qkv), _ptr(ctx),
                                            _ptr(lse), _ptr(dctx), _ptr(dqkv), _stream()))


def bf_op_attention_uses_mfma(S_seq, S_head):
    return bool(load().bf_op_attention_uses_mfma(S_seq, S_head))


def bf_op_embedding_fwd(dtype, n_rows, S_seq, S_voc, S_hidden, tokens, e_tok, e_pos, x):
    check(load().bf_op_embedding_fwd(dtype, n_rows, S_seq, S_voc, S_hidden, _ptr(tokens), _ptr(e_tok), _ptr(e_pos), _ptr(x),
                                     _stream()))


def bf_op_embedding_bwd(dtype, S_mb, S_seq, S_voc, S_hidden, tokens, d, g_tok, g_pos, accumulate_pos):
    check(load().bf_op_embedding_bwd(dtype, S_mb, S_seq, S_voc, S_hidden, _ptr(tokens), _ptr(d), _ptr(g_tok), _ptr(g_pos),
                                     accumulate_pos, _stream()))


def bf_op_ce_loss(dtype, n_rows, S_voc, z, labels, scale, row_loss, loss_out):
    check(load().bf_op_ce_loss(dtype, n_rows, S_voc, _ptr(z), _ptr(labels), scale, _ptr(row_loss), _ptr(loss_out), _stream()))


def bf_op_adam(n, w, m, v, g, w_lp, t, lr, beta1, beta2, adam_eps, weight_decay):
    check(load().bf_op_adam(n, _ptr(w), _ptr(m), _ptr(v), _ptr(g), _ptr(w_lp), t, lr, beta1, beta2, adam_eps,
                            weight_decay, _stream()))
