"""GPU parity of the single kernels against the CPU oracle, element by element.
Tolerance: max|gpu - oracle| / max|oracle| <= 1e-5 in fp32 mode, 2e-2 in bf16 mode."""
import math

import numpy as np
import pytest
import torch

import bf_inputs
import paper_2211_05953_amd as bf
from oracle import layer as L
from oracle import stack as K
from util import TOL, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu

MODES = [("fp32", bf.BF_FP32), ("bf16", bf.BF_BF16)]


def _dt(bf16):
    return torch.bfloat16 if bf16 else torch.float32


@pytest.mark.parametrize("mode,dtype", MODES)
@pytest.mark.parametrize("kernels", [bf.BF_KERNELS_PLAIN, bf.BF_KERNELS_AUTO])
@pytest.mark.parametrize("M,N,K", [(128, 768, 256), (200, 136, 72), (256, 512, 384), (2048, 256, 512), (64, 64, 2048), (1, 1, 1)])
def test_gemm_all_layouts_and_epilogues(mode, dtype, kernels, M, N, K):
    b16 = dtype == bf.BF_BF16
    A = bf_inputs.normal(1, 0, (M, K), bf16=b16)
    B = bf_inputs.normal(1, 1, (K, N), 0.05, bf16=b16)
    bias = bf_inputs.normal(1, 2, (N,), 0.5)
    R = bf_inputs.normal(1, 3, (M, N), bf16=b16)
    A64, B64, R64 = A.astype(np.float64), B.astype(np.float64), R.astype(np.float64)
    acc = A64 @ B64
    dA, dB, dR, dbias = to_dev(A, b16), to_dev(B, b16), to_dev(R, b16), to_dev(bias, False)
    out = torch.empty(M, N, dtype=_dt(b16), device="cuda")
    out2 = torch.empty_like(out)
    # forward layouts
    bf.bf_op_gemm(dtype, kernels, bf.BF_NN, bf.BF_EPI_NONE, M, N, K, dA, dB, out)
    assert rel_err(to_host(out), acc) <= TOL[mode]
    bf.bf_op_gemm(dtype, kernels, bf.BF_NN, bf.BF_EPI_BIAS, M, N, K, dA, dB, out, bias=dbias)
    assert rel_err(to_host(out), acc + bias) <= TOL[mode]
    bf.bf_op_gemm(dtype, kernels, bf.BF_NN, bf.BF_EPI_BIAS_RES, M, N, K, dA, dB, out, bias=dbias, R=dR)
    assert rel_err(to_host(out), acc + bias + R64) <= TOL[mode]
    bf.bf_op_gemm(dtype, kernels, bf.BF_NN, bf.BF_EPI_BIAS_GELU, M, N, K, dA, dB, out, bias=dbias, C2=out2)
    assert rel_err(to_host(out), acc + bias) <= TOL[mode]
    assert rel_err(to_host(out2), L.gelu(acc + bias)) <= TOL[mode]
    # dgrad layout: B passed as [N, K]
    dBt = to_dev(np.ascontiguousarray(B.T), b16)
    bf.bf_op_gemm(dtype, kernels, bf.BF_NT, bf.BF_EPI_NONE, M, N, K, dA, dBt, out)
    assert rel_err(to_host(out), acc) <= TOL[mode]
    bf.bf_op_gemm(dtype, kernels, bf.BF_NT, bf.BF_EPI_GELU_BWD, M, N, K, dA, dBt, out, R=dR)
    assert rel_err(to_host(out), acc * L.gelu_grad(R64)) <= TOL[mode]
    # wgrad layout: A passed as [K, M], fp32 output, overwrite then accumulate
    dAt = to_dev(np.ascontiguousarray(A.T), b16)
    G = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    bf.bf_op_gemm(dtype, kernels, bf.BF_TN, bf.BF_EPI_ACCUM, M, N, K, dAt, dB, G, accumulate=0)
    assert rel_err(to_host(G), acc) <= TOL["fp32"] * (1 if not b16 else 1)
    bf.bf_op_gemm(dtype, kernels, bf.BF_TN, bf.BF_EPI_ACCUM, M, N, K, dAt, dB, G, accumulate=1)
    assert rel_err(to_host(G), 2 * acc) <= TOL["fp32"]


@pytest.mark.parametrize("mode,dtype", MODES)
@pytest.mark.parametrize("kernels", [bf.BF_KERNELS_PLAIN, bf.BF_KERNELS_AUTO])
@pytest.mark.parametrize("M,N,K", [(128, 768, 256), (200, 136, 72), (512, 512, 128), (1280, 384, 192), (2048, 256, 512)])
def test_gelu_backward_product_with_the_bias_gradient_on_the_way(mode, dtype, kernels, M, N, K):
    """dU = (dY W^T) gelu'(U) and db = column sums of dU: in the MFMA kernel's epilogue (per-tile partial sums in a
    scratch buffer, then a fixed-order reduction), or as a second pass when there is no scratch or the plain kernel
    runs; overwriting and accumulating.  Shapes cover the 128-, 256 x 128- and 256 x 256-tile forms, several tile
    rows, and a ragged one."""
    b16 = dtype == bf.BF_BF16
    A = bf_inputs.normal(4, 0, (M, K), bf16=b16)
    Bt = bf_inputs.normal(4, 1, (N, K), 0.05, bf16=b16)
    R = bf_inputs.normal(4, 3, (M, N), bf16=b16)
    ref = (A.astype(np.float64) @ Bt.astype(np.float64).T) * L.gelu_grad(R.astype(np.float64))
    dA, dBt, dR = to_dev(A, b16), to_dev(Bt, b16), to_dev(R, b16)
    for with_part in (True, False):
        out = torch.empty(M, N, dtype=_dt(b16), device="cuda")
        db = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
        part = torch.full(((M + 127) // 128, N), float("nan"), dtype=torch.float32, device="cuda") if with_part else None
        bf.bf_op_gemm_gelu_bwd_colsum(dtype, kernels, M, N, K, dA, dBt, out, dR, db, part, accumulate=0)
        assert rel_err(to_host(out), ref) <= TOL[mode]
        assert rel_err(to_host(db), ref.sum(axis=0)) <= TOL[mode]
        # the sums are those of the stored output, up to fp32 summation order
        assert rel_err(to_host(db), to_host(out).astype(np.float64).sum(axis=0)) <= 1e-5
        first = to_host(db).copy()
        bf.bf_op_gemm_gelu_bwd_colsum(dtype, kernels, M, N, K, dA, dBt, out, dR, db, part, accumulate=1)
        assert rel_err(to_host(db), 2.0 * first.astype(np.float64)) <= 1e-6
        # same launch, same bits
        db2 = torch.empty_like(db)
        bf.bf_op_gemm_gelu_bwd_colsum(dtype, kernels, M, N, K, dA, dBt, out, dR, db2, part, accumulate=0)
        assert np.array_equal(to_host(db2), first)


@pytest.mark.parametrize("mode,dtype", MODES)
@pytest.mark.parametrize("T,h", [(128, 256), (77, 100), (300, 2048), (1024, 6144), (2048, 8192), (520, 1000), (3, 8200), (64, 16384)])
def test_layernorm_backward_in_one_pass(mode, dtype, T, h):
    """bf_op_layernorm_bwd_fused: dx, the gain / bias gradients and the column sums of dx from one pass over dy and x
    (workgroups of consecutive rows with partial sums in a scratch buffer, then a fixed-order reduction), or in separate
    passes when there is no scratch or the row does not fit; overwriting and accumulating; row counts that do not
    divide into equal runs; widths with idle lanes (256), of 3 and 4 vectors per thread, and beyond the one-pass form."""
    b16 = dtype == bf.BF_BF16
    x = bf_inputs.normal(6, 0, (T, h), 2.0, bf16=b16) + np.float32(0.5)
    if b16:
        x = bf_inputs.round_bf16(x)
    g = 1 + bf_inputs.normal(6, 1, (h,), 0.2)
    dy = bf_inputs.normal(6, 3, (T, h), bf16=b16)
    dres = bf_inputs.normal(6, 4, (T, h), bf16=b16)
    eps = 1e-5
    g64 = g.astype(np.float64)
    _, saved = L.layernorm_fwd(x.astype(np.float64), g64, np.zeros(h), eps)
    dx_ref, dg_ref, db_ref = L.layernorm_bwd(dy.astype(np.float64), g64, saved)
    dx_ref = dx_ref + dres.astype(np.float64)
    dX, dG, dDY, dRES = to_dev(x, b16), to_dev(g, False), to_dev(dy, b16), to_dev(dres, b16)
    stats = torch.empty(T, 2, dtype=torch.float32, device="cuda")
    bf.bf_op_layernorm_fwd(dtype, T, h, dX, dG, torch.zeros(h, device="cuda"), eps, torch.empty_like(dX), stats)
    n_part = bf.bf_op_layernorm_bwd_part_elems(T, h)
    assert n_part == 3 * h * -(-T // -(-T // 256)) and n_part <= 3 * h * 256
    results = []
    for with_part in (True, False):
        part = torch.full((n_part,), float("nan"), dtype=torch.float32, device="cuda") if with_part else None
        dx = torch.empty_like(dX)
        dg, db, dcs = (torch.full((h,), float("nan"), dtype=torch.float32, device="cuda") for _ in range(3))
        bf.bf_op_layernorm_bwd_fused(dtype, T, h, dDY, dX, dG, stats, dRES, dx, dg, db, dcs, part, accumulate=0)
        assert rel_err(to_host(dx), dx_ref) <= TOL[mode]
        assert rel_err(to_host(dg), dg_ref) <= TOL[mode] and rel_err(to_host(db), db_ref) <= TOL[mode]
        assert rel_err(to_host(dcs), dx_ref.sum(axis=0)) <= TOL[mode]
        assert rel_err(to_host(dcs), to_host(dx).astype(np.float64).sum(axis=0)) <= 1e-5   # sums of the stored dx
        first = [to_host(t).copy() for t in (dg, db, dcs)]
        bf.bf_op_layernorm_bwd_fused(dtype, T, h, dDY, dX, dG, stats, dRES, dx, dg, db, dcs, part, accumulate=1)
        for t, f0 in zip((dg, db, dcs), first):
            assert rel_err(to_host(t), 2.0 * f0.astype(np.float64)) <= 1e-6
        # without the residual gradient and without the column sums of dx
        dx2 = torch.empty_like(dX)
        bf.bf_op_layernorm_bwd_fused(dtype, T, h, dDY, dX, dG, stats, None, dx2, dg, db, None, part, accumulate=0)
        assert rel_err(to_host(dx2), dx_ref - dres.astype(np.float64)) <= TOL[mode]
        assert np.array_equal(to_host(dg), first[0]) and np.array_equal(to_host(db), first[1])
        results.append((to_host(dx), first))
    # the two forms agree to the rounding of the output (their fused multiply-adds may associate differently)
    assert rel_err(results[0][0], results[1][0].astype(np.float64)) <= (2.0 ** -8 if b16 else 1e-6)


@pytest.mark.parametrize("mode,dtype", MODES)
@pytest.mark.parametrize("T,h", [(128, 256), (77, 100), (512, 2048), (3, 8200)])
def test_layernorm_fwd_bwd_and_colsum(mode, dtype, T, h):
    b16 = dtype == bf.BF_BF16
    x = bf_inputs.normal(2, 0, (T, h), 2.0, bf16=b16) + np.float32(0.5)
    if b16:
        x = bf_inputs.round_bf16(x)
    g = 1 + bf_inputs.normal(2, 1, (h,), 0.2)
    b = bf_inputs.normal(2, 2, (h,), 0.2)
    dy = bf_inputs.normal(2, 3, (T, h), bf16=b16)
    dres = bf_inputs.normal(2, 4, (T, h), bf16=b16)
    eps = 1e-5
    y_ref, saved = L.layernorm_fwd(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64), eps)
    dx_ref, dg_ref, db_ref = L.layernorm_bwd(dy.astype(np.float64), g.astype(np.float64), saved)
    dX, dG, dB, dDY, dRES = to_dev(x, b16), to_dev(g, False), to_dev(b, False), to_dev(dy, b16), to_dev(dres, b16)
    y = torch.empty(T, h, dtype=_dt(b16), device="cuda")
    stats = torch.empty(T, 2, dtype=torch.float32, device="cuda")
    bf.bf_op_layernorm_fwd(dtype, T, h, dX, dG, dB, eps, y, stats)
    assert rel_err(to_host(y), y_ref) <= TOL[mode]
    st = to_host(stats).astype(np.float64)
    assert rel_err(st[:, 0], x.astype(np.float64).mean(-1)) <= 1e-5
    assert rel_err(st[:, 1], saved[1][:, 0]) <= 1e-5
    dx = torch.empty_like(y)
    dg = torch.full((h,), float("nan"), dtype=torch.float32, device="cuda")
    db = torch.full((h,), float("nan"), dtype=torch.float32, device="cuda")
    bf.bf_op_layernorm_bwd(dtype, T, h, dDY, dX, dG, stats, dRES, dx, dg, db, 0)
    assert rel_err(to_host(dx), dx_ref + dres) <= TOL[mode]
    assert rel_err(to_host(dg), dg_ref) <= 1e-5 and rel_err(to_host(db), db_ref) <= 1e-5
    bf.bf_op_layernorm_bwd(dtype, T, h, dDY, dX, dG, stats, None, dx, dg, db, 1)
    assert rel_err(to_host(dx), dx_ref) <= TOL[mode]
    assert rel_err(to_host(dg), 2 * dg_ref) <= 1e-5 and rel_err(to_host(db), 2 * db_ref) <= 1e-5
    out = torch.full((h,), float("nan"), dtype=torch.float32, device="cuda")
    bf.bf_op_colsum(dtype, T, h, dDY, out, 0)
    assert rel_err(to_host(out), dy.astype(np.float64).sum(0)) <= 1e-5
    bf.bf_op_colsum(dtype, T, h, dDY, out, 1)
    assert rel_err(to_host(out), 2 * dy.astype(np.float64).sum(0)) <= 1e-5


@pytest.mark.parametrize("mode,dtype", MODES)
@pytest.mark.parametrize("kernels", [bf.BF_KERNELS_PLAIN, bf.BF_KERNELS_AUTO])
@pytest.mark.parametrize("causal", [1, 0])
@pytest.mark.parametrize("S_mb,S_seq,a,d", [(1, 128, 4, 64), (2, 256, 2, 128), (2, 100, 3, 40), (1, 1, 1, 8), (1, 384, 2, 128)])
def test_attention_fwd_bwd(mode, dtype, kernels, causal, S_mb, S_seq, a, d):
    b16 = dtype == bf.BF_BF16
    h = a * d
    qkv = bf_inputs.normal(3, 0, (S_mb, S_seq, 3 * h), bf16=b16)
    dctx = bf_inputs.normal(3, 1, (S_mb, S_seq, h), bf16=b16)
    ctx_ref, saved = L.attention_fwd(qkv.astype(np.float64), a, bool(causal))
    dqkv_ref = L.attention_bwd(dctx.astype(np.float64), saved, a)
    dQKV, dDC = to_dev(qkv, b16), to_dev(dctx, b16)
    ctx = torch.empty(S_mb, S_seq, h, dtype=_dt(b16), device="cuda")
    lse = torch.empty(S_mb, a, S_seq, dtype=torch.float32, device="cuda")
    bf.bf_op_attention_fwd(dtype, kernels, S_mb, S_seq, a, d, causal, dQKV, ctx, lse)
    assert rel_err(to_host(ctx), ctx_ref) <= TOL[mode]
    # log-sum-exp of the scaled masked scores, from the definition
    q, k, v, p = saved
    s = np.matmul(q, k.transpose(0, 1, 3, 2)) / math.sqrt(d)
    if causal:
        s = np.where(np.tril(np.ones((S_seq, S_seq), dtype=bool)), s, -np.inf)
    lse_ref = np.log(np.exp(s - s.max(-1, keepdims=True)).sum(-1)) + s.max(-1)
    assert np.abs(to_host(lse) - lse_ref).max() <= (1e-4 if not b16 else 2e-2)
    dqkv = torch.empty(S_mb, S_seq, 3 * h, dtype=_dt(b16), device="cuda")
    delta = torch.empty(S_mb * a * S_seq, dtype=torch.float32, device="cuda")
    bf.bf_op_attention_bwd(dtype, kernels, S_mb, S_seq, a, d, causal, dQKV, ctx, lse, dDC, dqkv, delta)
    got = to_host(dqkv)
    for i, name in enumerate(("dq", "dk", "dv")):
        assert rel_err(got[..., i * h:(i + 1) * h], dqkv_ref[..., i * h:(i + 1) * h]) <= TOL[mode], name
    # the same with the QKV bias gradient (column sums of dqkv) on the way: with the scratch for the kernels' partial
    # sums (where the matrix-core kernels serve the shape) and without it (dqkv read a second time); overwrite, then add
    n_part = bf.bf_op_attention_bwd_part_elems(S_mb, S_seq, a, d)
    mfma = bf.bf_op_attention_uses_mfma(S_seq, d)
    q_rows = S_mb * (S_seq // (256 if S_seq % 256 == 0 else 128)) if mfma else 0
    assert n_part == (q_rows * h + S_mb * (S_seq // 128) * 2 * h if mfma else 0)
    db_ref = dqkv_ref.reshape(-1, 3 * h).sum(axis=0)
    for with_part in (True, False):
        part = torch.full((max(n_part, 1),), float("nan"), dtype=torch.float32, device="cuda") if with_part and n_part else None
        dqkv2 = torch.full_like(dqkv, float("nan"))
        db = torch.full((3 * h,), float("nan"), dtype=torch.float32, device="cuda")
        bf.bf_op_attention_bwd_bias(dtype, kernels, S_mb, S_seq, a, d, causal, dQKV, ctx, lse, dDC, dqkv2, delta, db, part, 0)
        assert torch.equal(dqkv2, dqkv)
        first = to_host(db).copy()
        # (the K third is zero in exact arithmetic: a softmax row does not move when every score of it is shifted by the
        # same amount, which is all a key bias does; so the thirds are judged together, on the scale of the whole vector)
        assert rel_err(first, db_ref) <= TOL[mode]
        for i, name in ((0, "dq"), (2, "dv")):
            assert rel_err(first[i * h:(i + 1) * h], db_ref[i * h:(i + 1) * h]) <= TOL[mode], name
        # against the sums of what was stored: the fused form adds the values before they are rounded to bf16
        stored = got.astype(np.float64).reshape(-1, 3 * h).sum(axis=0)
        assert rel_err(first, stored) <= (2.0 ** -8 if b16 else 1e-5)
        bf.bf_op_attention_bwd_bias(dtype, kernels, S_mb, S_seq, a, d, causal, dQKV, ctx, lse, dDC, dqkv2, delta, db, part, 1)
        assert rel_err(to_host(db), 2.0 * first.astype(np.float64)) <= 1e-6


@pytest.mark.parametrize("M,N,K", [(2048, 2048, 8192), (2048, 2048, 6144), (1024, 1024, 4096), (256, 128, 2048)])
def test_gemm_with_a_split_contraction(M, N, K):
    """bf_op_gemm_splitk: few tiles and a long contraction run K in two slices into fp32 planes that a second kernel adds
    in order, with each of the epilogues it serves, in both layouts; the result agrees with the unsplit product to the
    rounding of the output (the fp32 sum associates differently) and with the fp64 product to the bf16 bar."""
    assert bf.bf_op_gemm_splitk_slices(bf.BF_NN, bf.BF_EPI_BIAS_RES, M, N, K) == 2
    assert bf.bf_op_gemm_splitk_slices(bf.BF_NT, bf.BF_EPI_NONE, M, N, K) == 2
    A = bf_inputs.normal(15, 0, (M, K), bf16=True)
    B = bf_inputs.normal(15, 1, (K, N), 0.05, bf16=True)
    bias = bf_inputs.normal(15, 2, (N,), 0.5)
    R = bf_inputs.normal(15, 3, (M, N), bf16=True)
    acc = A.astype(np.float64) @ B.astype(np.float64)
    dA, dB, dBt, dR, dbias = to_dev(A, True), to_dev(B, True), to_dev(np.ascontiguousarray(B.T), True), to_dev(R, True), to_dev(bias, False)
    planes = torch.full((2 * M * N,), float("nan"), dtype=torch.float32, device="cuda")
    for layout, Bd in ((bf.BF_NN, dB), (bf.BF_NT, dBt)):
        for epi, want in ((bf.BF_EPI_NONE, acc), (bf.BF_EPI_BIAS, acc + bias), (bf.BF_EPI_BIAS_RES, acc + bias + R)):
            out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
            ref = torch.empty_like(out)
            bf.bf_op_gemm_splitk(bf.BF_BF16, 0, layout, epi, M, N, K, dA, Bd, out, bias=dbias, R=dR, planes=planes)
            bf.bf_op_gemm(bf.BF_BF16, 0, layout, epi, M, N, K, dA, Bd, ref, bias=dbias, R=dR)
            assert rel_err(to_host(out), want) <= TOL["bf16"], (layout, epi)
            assert rel_err(to_host(out), to_host(ref).astype(np.float64)) <= 2.0 ** -7, (layout, epi)
            # deterministic: a second call gives the same bits
            again = torch.empty_like(out)
            bf.bf_op_gemm_splitk(bf.BF_BF16, 0, layout, epi, M, N, K, dA, Bd, again, bias=dbias, R=dR, planes=planes)
            assert torch.equal(out, again)
    # without the scratch, or with too little of it, the call is the plain product
    out, ref = torch.empty((M, N), dtype=torch.bfloat16, device="cuda"), torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    bf.bf_op_gemm(bf.BF_BF16, 0, bf.BF_NN, bf.BF_EPI_BIAS, M, N, K, dA, dB, ref, bias=dbias)
    bf.bf_op_gemm_splitk(bf.BF_BF16, 0, bf.BF_NN, bf.BF_EPI_BIAS, M, N, K, dA, dB, out, bias=dbias, planes=None)
    assert torch.equal(out, ref)
    bf.bf_op_gemm_splitk(bf.BF_BF16, 0, bf.BF_NN, bf.BF_EPI_BIAS, M, N, K, dA, dB, out, bias=dbias, planes=planes[:M * N])
    assert torch.equal(out, ref)


def test_split_contraction_is_chosen_only_where_it_pays():
    s = bf.bf_op_gemm_splitk_slices
    assert s(bf.BF_NN, bf.BF_EPI_BIAS_RES, 2048, 2048, 2048) == 2
    assert s(bf.BF_NN, bf.BF_EPI_BIAS_RES, 2048, 2048, 1024) == 1      # contraction too short
    assert s(bf.BF_NN, bf.BF_EPI_BIAS, 2048, 8192, 8192) == 1          # a full round of tiles already
    assert s(bf.BF_NT, bf.BF_EPI_NONE, 2048, 6144, 18432) == 1
    assert s(bf.BF_NN, bf.BF_EPI_BIAS_GELU, 2048, 2048, 8192) == 1     # epilogues with a second output are not split
    assert s(bf.BF_NT, bf.BF_EPI_GELU_BWD, 2048, 2048, 8192) == 1
    assert s(bf.BF_TN, bf.BF_EPI_ACCUM, 2048, 2048, 8192) == 1
    assert s(bf.BF_NN, bf.BF_EPI_NONE, 2000, 2048, 8192) == 1          # not a shape of the matrix-core kernel
    assert s(bf.BF_NN, bf.BF_EPI_NONE, 2048, 2048, 8192 + 64) == 1     # slices must be whole k-tiles


@pytest.mark.parametrize("M,N,K", [(2048, 4096, 512), (4096, 2048, 192), (512, 16384, 128)])
def test_gemm_mfma_large_tile(M, N, K):
    """Shapes that take the 256 x 256 workgroup tile of the MFMA kernel, all layouts."""
    assert bf.bf_op_gemm_uses_mfma(bf.BF_NN, bf.BF_EPI_NONE, M, N, K)
    A = bf_inputs.normal(5, 0, (M, K), bf16=True)
    B = bf_inputs.normal(5, 1, (K, N), 0.05, bf16=True)
    bias = bf_inputs.normal(5, 2, (N,), 0.5)
    R = bf_inputs.normal(5, 3, (M, N), bf16=True)
    acc = A.astype(np.float64) @ B.astype(np.float64)
    dA, dB, dR, dbias = to_dev(A, True), to_dev(B, True), to_dev(R, True), to_dev(bias, False)
    out = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    out2 = torch.empty_like(out)
    bf.bf_op_gemm(bf.BF_BF16, 0, bf.BF_NN, bf.BF_EPI_BIAS_RES, M, N, K, dA, dB, out, bias=dbias, R=dR)
    assert rel_err(to_host(out), acc + bias + R) <= TOL["bf16"]
    bf.bf_op_gemm(bf.BF_BF16, 0, bf.BF_NN, bf.BF_EPI_BIAS_GELU, M, N, K, dA, dB, out, bias=dbias, C2=out2)
    assert rel_err(to_host(out2), L.gelu(acc + bias)) <= TOL["bf16"]
    bf.bf_op_gemm(bf.BF_BF16, 0, bf.BF_NT, bf.BF_EPI_GELU_BWD, M, N, K, dA, to_dev(np.ascontiguousarray(B.T), True), out, R=dR)
    assert rel_err(to_host(out), acc * L.gelu_grad(R.astype(np.float64))) <= TOL["bf16"]
    G = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    dAt = to_dev(np.ascontiguousarray(A.T), True)
    bf.bf_op_gemm(bf.BF_BF16, 0, bf.BF_TN, bf.BF_EPI_ACCUM, M, N, K, dAt, dB, G, accumulate=0)
    bf.bf_op_gemm(bf.BF_BF16, 0, bf.BF_TN, bf.BF_EPI_ACCUM, M, N, K, dAt, dB, G, accumulate=1)
    assert rel_err(to_host(G), 2 * acc) <= 1e-5   # bf16 products are exact in fp32; only the summation order differs


@pytest.mark.parametrize("M,N,K", [(4096, 3072, 192), (2048, 6144, 64), (256, 49152, 128), (2048, 6144, 320)])
def test_gemm_mfma_tile_of_192_columns(M, N, K):
    """Forward and dgrad products with a one-output epilogue whose column count is a multiple of 192 take a 256 x 192
    tile where that fills the rounds better (6144 columns: 32 tiles where 256-column tiles give 24); the epilogues
    with a second output or with column sums, and the weight-gradient layout, keep their tiles."""
    for layout, epi in ((bf.BF_NT, bf.BF_EPI_NONE), (bf.BF_NN, bf.BF_EPI_NONE), (bf.BF_NN, bf.BF_EPI_BIAS), (bf.BF_NN, bf.BF_EPI_BIAS_RES)):
        assert bf.bf_op_gemm_tile(layout, epi, M, N, K) == (256, 192), (layout, epi)
    for layout, epi in ((bf.BF_NT, bf.BF_EPI_GELU_BWD), (bf.BF_NN, bf.BF_EPI_BIAS_GELU), (bf.BF_TN, bf.BF_EPI_ACCUM)):
        assert bf.bf_op_gemm_tile(layout, epi, M, N, K)[1] != 192, (layout, epi)
    assert bf.bf_op_gemm_tile(bf.BF_NT, bf.BF_EPI_NONE, 2048, 8192, 8192) == (256, 256)   # 8192 is no multiple of 192
    assert bf.bf_op_gemm_tile(bf.BF_NN, bf.BF_EPI_BIAS, 2048, 24576, 8192) == (256, 256)  # three whole rounds already
    assert bf.bf_op_gemm_tile(bf.BF_NT, bf.BF_EPI_NONE, 100, 72, 64) is None
    A = bf_inputs.normal(6, 0, (M, K), bf16=True)
    B = bf_inputs.normal(6, 1, (K, N), 0.05, bf16=True)
    bias = bf_inputs.normal(6, 2, (N,), 0.5)
    R = bf_inputs.normal(6, 3, (M, N), bf16=True)
    acc = A.astype(np.float64) @ B.astype(np.float64)
    dA, dB, dBt = to_dev(A, True), to_dev(B, True), to_dev(np.ascontiguousarray(B.T), True)
    dR, dbias = to_dev(R, True), to_dev(bias, False)
    cases = (("dgrad", bf.BF_NT, bf.BF_EPI_NONE, dBt, acc), ("fwd", bf.BF_NN, bf.BF_EPI_NONE, dB, acc),
             ("fwd+bias", bf.BF_NN, bf.BF_EPI_BIAS, dB, acc + bias), ("fwd+bias+res", bf.BF_NN, bf.BF_EPI_BIAS_RES, dB, acc + bias + R))
    for name, layout, epi, dOp, ref in cases:
        out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        bf.bf_op_gemm(bf.BF_BF16, 0, layout, epi, M, N, K, dA, dOp, out, bias=dbias, R=dR)
        got = to_host(out)
        assert np.isfinite(got).all() and rel_err(got, ref) <= TOL["bf16"], name
        # one rounding of the fp32 result: the plain kernel (fp32 FMA over the same bf16 products) agrees to that rounding
        plain = torch.empty_like(out)
        bf.bf_op_gemm(bf.BF_BF16, bf.BF_KERNELS_PLAIN, layout, epi, M, N, K, dA, dOp, plain, bias=dbias, R=dR)
        assert rel_err(got, to_host(plain)) <= 2.0 ** -7, name


@pytest.mark.parametrize("mode,dtype,kernels", [("fp32", bf.BF_FP32, bf.BF_KERNELS_AUTO), ("bf16", bf.BF_BF16, bf.BF_KERNELS_PLAIN),
                                                ("bf16", bf.BF_BF16, bf.BF_KERNELS_AUTO)])
@pytest.mark.parametrize("M,N,K,n_seg,gap", [(256, 512, 128, 3, 0), (1024, 768, 128, 2, 64), (128, 384, 64, 2, 8), (512, 256, 192, 4, 0),
                                             (768, 128, 64, 1, 0), (200, 136, 72, 3, 16), (256, 256, 64, 2, 4)])
def test_wgrad_over_the_micro_batches_of_a_stage(mode, dtype, kernels, M, N, K, n_seg, gap):
    """G = sum_i X_i^T dY_i and db = sum_i colsum(dY_i) in one call (Sec. 4.2: the gradient of a stage
    is needed only after all its micro-batches); segments lie `gap` elements apart beyond their size."""
    b16 = dtype == bf.BF_BF16
    sx, sy = K * M + gap, K * N + gap
    X = bf_inputs.normal(9, 0, (n_seg * sx,), bf16=b16)
    dY = bf_inputs.normal(9, 1, (n_seg * sy,), 0.3, bf16=b16)
    G_ref, db_ref = np.zeros((M, N)), np.zeros(N)
    for i in range(n_seg):
        Xi = X[i * sx:i * sx + K * M].reshape(K, M).astype(np.float64)
        dYi = dY[i * sy:i * sy + K * N].reshape(K, N).astype(np.float64)
        G_ref += Xi.T @ dYi
        db_ref += dYi.sum(0)
    dX, ddY = to_dev(X, b16), to_dev(dY, b16)
    G = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    db = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
    bf.bf_op_wgrad(dtype, kernels, M, N, K, n_seg, dX, sx, ddY, sy, G, db, accumulate=0)
    assert rel_err(to_host(G), G_ref) <= 1e-5 and rel_err(to_host(db), db_ref) <= 1e-5
    bf.bf_op_wgrad(dtype, kernels, M, N, K, n_seg, dX, sx, ddY, sy, G, db, accumulate=1)
    assert rel_err(to_host(G), 2 * G_ref) <= 1e-5 and rel_err(to_host(db), 2 * db_ref) <= 1e-5
    # without the bias gradient: db is left alone
    keep = to_host(db).copy()
    bf.bf_op_wgrad(dtype, kernels, M, N, K, n_seg, dX, sx, ddY, sy, G, None, accumulate=0)
    assert rel_err(to_host(G), G_ref) <= 1e-5 and np.array_equal(to_host(db), keep)


@pytest.mark.parametrize("n", [1, 1000, 4096 * 33 + 4])
def test_adam_kernel(n):
    rng = np.random.default_rng(4)
    w = rng.standard_normal(n).astype(np.float32)
    g = (rng.standard_normal(n) * 10.0 ** rng.integers(-4, 2, n)).astype(np.float32)
    m0 = (rng.standard_normal(n) * 0.1).astype(np.float32)
    v0 = (rng.random(n) * 0.1).astype(np.float32)
    dW, dM, dV, dGr = (torch.from_numpy(t).cuda() for t in (w, m0, v0, g))
    wlp = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    args = dict(lr=1e-2, beta1=0.9, beta2=0.999, adam_eps=1e-8, weight_decay=0.01)
    bf.bf_op_adam(n, dW, dM, dV, dGr, wlp, 3, **args)
    # the C ABI carries the constants as fp32: the oracle gets those exact values
    f32 = {k: float(np.float32(v)) for k, v in args.items()}
    w1, m1, v1 = K.adam_update(w.astype(np.float64), g.astype(np.float64), m0.astype(np.float64), v0.astype(np.float64),
                               3, f32["lr"], f32["beta1"], f32["beta2"], f32["adam_eps"], f32["weight_decay"])
    assert rel_err(to_host(dM), m1) <= 1e-6 and rel_err(to_host(dV), v1) <= 1e-6
    assert rel_err(to_host(dW) - w, w1 - w) <= 1e-4          # the update itself
    assert np.array_equal(to_host(wlp), bf_inputs.round_bf16(to_host(dW)))  # recast = RNE of the new master


def test_op_argument_errors():
    t = torch.zeros(16, device="cuda")
    with pytest.raises(bf.BfError) as e:
        bf.bf_op_gemm(bf.BF_FP32, 0, bf.BF_NN, bf.BF_EPI_BIAS, 4, 4, 4, t, t, t)   # bias missing
    assert e.value.status == bf.BF_EINVAL
    with pytest.raises(bf.BfError):
        bf.bf_op_gemm(bf.BF_FP32, 0, bf.BF_TN, bf.BF_EPI_NONE, 4, 4, 4, t, t, t)
    with pytest.raises(bf.BfError):
        bf.bf_op_gemm(9, 0, bf.BF_NN, bf.BF_EPI_NONE, 4, 4, 4, t, t, t)
    with pytest.raises(bf.BfError):
        bf.bf_op_layernorm_fwd(bf.BF_FP32, 0, 4, t, t, t, 1e-5, t, t)
    with pytest.raises(bf.BfError):
        bf.bf_op_attention_fwd(bf.BF_FP32, 0, 1, 5000, 1, 4, 1, t, t, t)
