"""GPU parity of the individual kernels against the CPU oracle (through the C ABI)."""
import math

import numpy as np
import pytest
import torch

from oracle import stage_oracle as O
from paper_2507_21276_amd import binding as Bd
from paper_2507_21276_amd import synth_inputs as S
from parity_util import TOL, assert_close, dev, host, out_rounding_bound

pytestmark = pytest.mark.gpu

DT = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
# tolerance by operand type: fp16 operands are held to the bf16 bar too
KTOL = {"f32": 1e-4, "bf16": 2e-2, "f16": 2e-2}


def otol(name, ref, f32_tol=1e-5):
    """Tolerance for a kernel whose *output* is stored in `name`: the bar plus the
    unavoidable rounding of the result itself (half an ulp of the largest element
    over the tensor RMS; this alone exceeds 2e-2 for bf16 tensors with outliers)."""
    return f32_tol if name == "f32" else KTOL[name] + out_rounding_bound(ref, name)


def q(x, name):
    """Round host data to what the kernel will read."""
    if name == "f32":
        return np.asarray(x, np.float32)
    if name == "bf16":
        return S.round_bf16(x)
    return np.asarray(x, np.float32).astype(np.float16).astype(np.float32)


@pytest.mark.parametrize("name", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("M,N,K", [(300, 264, 328), (512, 768, 256), (64, 1048, 136), (5, 8, 8), (257, 520, 1000)])
def test_gemm_forward_layout_with_bias_and_residual(name, M, N, K):
    A = q(S.normal(1, "A", (M, K)), name)
    W = q(S.normal(1, "W", (N, K), 0.05), name)
    bias = q(S.normal(1, "b", (N,)), "f32" if name == "f32" else "bf16")
    R = S.normal(1, "R", (M, N))
    ref = A.astype(np.float64) @ W.astype(np.float64).T + bias + R
    out = torch.empty(M, N, dtype=torch.float32, device="cuda")
    Bd.lsk_gemm(dev(A, DT[name]), dev(W, DT[name]), out, M=M, N=N, K=K,
                bias=dev(bias, torch.float32 if name == "f32" else torch.bfloat16), resid=dev(R, torch.float32))
    assert_close(host(out), ref, KTOL[name] if name == "f32" else 1e-5, f"gemm NT {name}")
    if name != "f32":   # operand-typed output, no residual
        out16 = torch.empty(M, N, dtype=DT[name], device="cuda")
        Bd.lsk_gemm(dev(A, DT[name]), dev(W, DT[name]), out16, M=M, N=N, K=K)
        r_ = A.astype(np.float64) @ W.astype(np.float64).T
        assert_close(host(out16), r_, otol(name, r_), f"gemm NT16 {name}")


@pytest.mark.parametrize("name", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("T,N,K", [(300, 264, 328), (130, 512, 768), (7, 16, 24)])
def test_gemm_input_and_weight_gradient_layouts(name, T, N, K):
    dY = q(S.normal(2, "dY", (T, N)), name)
    W = q(S.normal(2, "W", (N, K), 0.05), name)
    X = q(S.normal(2, "X", (T, K)), name)
    dYd, Wd, Xd = dev(dY, DT[name]), dev(W, DT[name]), dev(X, DT[name])
    # dX = dY W : contraction over N, B is k-strided
    dX = torch.empty(T, K, dtype=torch.float32, device="cuda")
    Bd.lsk_gemm(dYd, Wd, dX, M=T, N=K, K=N, a_kmajor=True, b_kmajor=False, lda=N, ldb=K)
    assert_close(host(dX), dY.astype(np.float64) @ W.astype(np.float64), 1e-5 if name != "f32" else 1e-4, "dX")
    # dW = dY^T X : contraction over tokens, both k-strided; accumulate twice
    dW = torch.zeros(N, K, dtype=torch.float32, device="cuda")
    for acc in (False, True):
        Bd.lsk_gemm(dYd, Xd, dW, M=N, N=K, K=T, a_kmajor=False, b_kmajor=False, lda=N, ldb=K, accumulate=acc)
    assert_close(host(dW), 2.0 * dY.astype(np.float64).T @ X.astype(np.float64), 1e-5 if name != "f32" else 1e-4, "dW")


@pytest.mark.parametrize("name", ["bf16", "f16"])
@pytest.mark.parametrize("K", [64, 192])
@pytest.mark.parametrize("M,N", [(4104, 2568),    # 17 x 11 = 187 tiles of 256 x 256, 8 rows and 8 columns in the last ones
                                  (2056, 8200)])   # 9 x 33 = 297 tiles: a second, nearly empty round of workgroups
def test_gemm_large_tile_kernels_with_ragged_edges(name, K, M, N):
    """More than 160 tiles of 256 x 256 with partial tiles on both edges and one or three k tiles: the
    16x16x32 kernel (forward and input-gradient layouts) and the 32x32x16 kernel (weight gradient),
    every element against float64."""
    A = q(S.normal(5, "A", (M, K)), name)
    W = q(S.normal(5, "W", (N, K), 0.05), name)
    bias = q(S.normal(5, "b", (N,)), "bf16")
    R = S.normal(5, "R", (M, N))
    Ad, Wd = dev(A, DT[name]), dev(W, DT[name])
    ref = A.astype(np.float64) @ W.astype(np.float64).T
    out = torch.empty(M, N, dtype=torch.float32, device="cuda")
    Bd.lsk_gemm(Ad, Wd, out, M=M, N=N, K=K, bias=dev(bias, torch.bfloat16), resid=dev(R, torch.float32))
    assert_close(host(out), ref + bias + R, 1e-5, "forward, bias and residual")
    out16 = torch.empty(M, N, dtype=DT[name], device="cuda")
    Bd.lsk_gemm(Ad, Wd, out16, M=M, N=N, K=K, bias=dev(bias, torch.bfloat16))
    assert_close(host(out16), ref + bias, otol(name, ref + bias), "forward, 16-bit result")
    # input-gradient layout: C[M, N] = A[M, K] B[K, N], B k-strided
    Bk = q(S.normal(5, "Bk", (K, N), 0.05), name)
    out16.zero_()
    Bd.lsk_gemm(Ad, dev(Bk, DT[name]), out16, M=M, N=N, K=K, a_kmajor=True, b_kmajor=False, lda=K, ldb=N)
    r2 = A.astype(np.float64) @ Bk.astype(np.float64)
    assert_close(host(out16), r2, otol(name, r2), "input-gradient layout")
    # weight-gradient layout: C[M, N] = At[K, M]^T Bk[K, N], both k-strided, fp32 result
    At = q(S.normal(5, "At", (K, M)), name)
    Bd.lsk_gemm(dev(At, DT[name]), dev(Bk, DT[name]), out, M=M, N=N, K=K, a_kmajor=False, b_kmajor=False, lda=M, ldb=N)
    r3 = At.astype(np.float64).T @ Bk.astype(np.float64)
    assert_close(host(out), r3, 1e-5, "weight-gradient layout")
    # accumulating fp32 results: a second launch adds to what the first one wrote (both kernels fetch the old
    # values of an epilogue pass before they stage the accumulators)
    Bd.lsk_gemm(dev(At, DT[name]), dev(Bk, DT[name]), out, M=M, N=N, K=K, a_kmajor=False, b_kmajor=False, lda=M, ldb=N,
                accumulate=True)
    assert_close(host(out), 2.0 * r3, 1e-5, "weight-gradient layout, accumulated")
    out.copy_(dev(R, torch.float32))
    Bd.lsk_gemm(Ad, Wd, out, M=M, N=N, K=K, accumulate=True)
    assert_close(host(out), ref + R, 1e-5, "forward layout, fp32 result added to the buffer")
    out.copy_(dev(R, torch.float32))
    Bd.lsk_gemm(Ad, dev(Bk, DT[name]), out, M=M, N=N, K=K, a_kmajor=True, b_kmajor=False, lda=K, ldb=N, accumulate=True)
    assert_close(host(out), r2 + R, 1e-5, "input-gradient layout, fp32 result added to the buffer")


@pytest.mark.parametrize("name", ["bf16", "f16"])
def test_gemm_accumulates_into_fp32_buffers_with_128_tiles(name):
    """Few tiles (the 128 x 128 kernel), partial tiles on both edges: a launch with accumulate adds to the
    buffer in the forward, input-gradient and weight-gradient layouts, and the residual mode adds the residual."""
    M, N, K = 520, 392, 256
    A = q(S.normal(6, "A", (M, K)), name)
    W = q(S.normal(6, "W", (N, K), 0.05), name)
    Bk = q(S.normal(6, "Bk", (K, N), 0.05), name)
    At = q(S.normal(6, "At", (K, M)), name)
    R = S.normal(6, "R", (M, N))
    Rd = dev(R, torch.float32)
    out = torch.empty(M, N, dtype=torch.float32, device="cuda")
    f64 = lambda x: x.astype(np.float64)
    out.copy_(Rd)
    Bd.lsk_gemm(dev(A, DT[name]), dev(W, DT[name]), out, M=M, N=N, K=K, accumulate=True)
    assert_close(host(out), f64(A) @ f64(W).T + R, 1e-5, "forward layout")
    Bd.lsk_gemm(dev(A, DT[name]), dev(W, DT[name]), out, M=M, N=N, K=K, resid=Rd)
    assert_close(host(out), f64(A) @ f64(W).T + R, 1e-5, "forward layout, residual")
    out.copy_(Rd)
    Bd.lsk_gemm(dev(A, DT[name]), dev(Bk, DT[name]), out, M=M, N=N, K=K, a_kmajor=True, b_kmajor=False, lda=K, ldb=N,
                accumulate=True)
    assert_close(host(out), f64(A) @ f64(Bk) + R, 1e-5, "input-gradient layout")
    out.copy_(Rd)
    Bd.lsk_gemm(dev(At, DT[name]), dev(Bk, DT[name]), out, M=M, N=N, K=K, a_kmajor=False, b_kmajor=False, lda=M, ldb=N,
                accumulate=True)
    assert_close(host(out), f64(At).T @ f64(Bk) + R, 1e-5, "weight-gradient layout")
    Bd.lsk_gemm(dev(At, DT[name]), dev(Bk, DT[name]), out, M=M, N=N, K=K, a_kmajor=False, b_kmajor=False, lda=M, ldb=N)
    assert_close(host(out), f64(At).T @ f64(Bk), 1e-5, "weight-gradient layout, overwriting")


@pytest.mark.parametrize("name", ["f16", "bf16"])
@pytest.mark.parametrize("M,N,K,out,res", [(512, 4096, 4096, "f32", True), (512, 4096, 11008, "f32", True),
                                            (300, 520, 2048, "op", False), (256, 264, 4096, "op", False),
                                            # decode batches: weight-streaming kernel, 32 weight rows per workgroup
                                            (64, 4096, 4096, "f32", True), (64, 12288, 4096, "op", False),
                                            (33, 264, 1024, "op", False), (1, 128, 512, "f32", True),
                                            (7, 1048, 11008, "op", False), (64, 22016, 4096, "op", False),
                                            (64, 4096, 11008, "f32", True), (32, 72, 64, "op", False),
                                            (17, 40, 320, "f32", False), (64, 8, 192, "op", True),
                                            (48, 2000, 1600, "f32", True), (128, 5120, 13824, "f32", True),
                                            (100, 15360, 5120, "op", False)])
def test_gemm_split_k_through_a_workspace(name, M, N, K, out, res):
    """Few output tiles: the contraction is split over workgroups and summed in a fixed order."""
    dt = DT[name]
    x = S.normal_torch(31, "x", (M, K), 1.0, dtype=dt)
    w = S.normal_torch(31, "w", (N, K), K ** -0.5, dtype=dt)
    bias = S.normal_torch(31, "b", (N,), 1.0, dtype=torch.float32)
    resid = S.normal_torch(31, "r", (M, N), 1.0, dtype=torch.float32) if res else None
    c = torch.empty(M, N, dtype=torch.float32 if out == "f32" else dt, device="cuda")
    scratch = torch.empty(8 * M * N, dtype=torch.float32, device="cuda")
    Bd.lsk_gemm_ws(x, w, c, scratch, bias=bias, resid=resid)
    ref = host(x) @ host(w).T + host(bias)[None, :]
    if res:
        ref = ref + host(resid)
    tol = KTOL[name] if out == "f32" else otol(name, ref)
    assert_close(host(c), ref, tol, "split-K gemm")
    c2 = torch.empty_like(c)
    Bd.lsk_gemm_ws(x, w, c2, scratch, bias=bias, resid=resid)
    assert torch.equal(c, c2)   # deterministic
    # without a workspace the same call takes the plain path
    c3 = torch.empty_like(c)
    Bd.lsk_gemm_ws(x, w, c3, torch.empty(0, dtype=torch.float32, device="cuda"), bias=bias, resid=resid)
    assert_close(host(c3), ref, tol, "gemm_ws without workspace")


@pytest.mark.parametrize("name", ["f16", "bf16"])
def test_gemm_full_size_launch_configuration_on_sampled_outputs(name):
    """The LLaMA-7B-shaped projections at the training micro-batch size (the
    256 x 256 tile kernel with direct-to-LDS loads and all three operand
    layouts): sampled rows of each result against float64 dot products."""
    T, d, F = 4096, 4096, 11008
    # one row of every 16-row block of a 256-row tile (the blocks of the 16x16x32 kernel), and the edges
    rows = sorted(set(list(range(3, 256, 16)) + [0, 1, 255, 256, 2047, 3000, 4095]))
    dt = DT[name]
    X = S.normal_torch(11, "X", (T, d), 1.0, "cuda", dt)
    dY = S.normal_torch(11, "dY", (T, 2 * F), 1.0, "cuda", dt)
    W = S.normal_torch(11, "W", (2 * F, d), 0.02, "cuda", dt)
    R = S.normal_torch(11, "R", (T, 2 * F), 1.0, "cuda")
    Xh, dYh, Wh = (host(t) for t in (X, dY, W))
    # forward, 16-bit output
    Y = torch.empty(T, 2 * F, dtype=dt, device="cuda")
    Bd.lsk_gemm(X, W, Y, M=T, N=2 * F, K=d)
    ref = Xh[rows] @ Wh.T
    assert_close(host(Y[rows]), ref, otol(name, ref), "fwd rows")
    # forward, fp32 output with residual
    Yf = torch.empty(T, 2 * F, dtype=torch.float32, device="cuda")
    Bd.lsk_gemm(X, W, Yf, M=T, N=2 * F, K=d, resid=R)
    assert_close(host(Yf[rows]), ref + host(R[rows]), 1e-5, "fwd+resid rows")
    # input gradient dX = dY W
    dX = torch.empty(T, d, dtype=dt, device="cuda")
    Bd.lsk_gemm(dY, W, dX, M=T, N=d, K=2 * F, a_kmajor=True, b_kmajor=False, lda=2 * F, ldb=d)
    ref = dYh[rows] @ Wh
    assert_close(host(dX[rows]), ref, otol(name, ref), "dX rows")
    # weight gradient dW = dY^T X, sampled rows of dW (= columns of dY)
    dW = torch.empty(2 * F, d, dtype=torch.float32, device="cuda")
    Bd.lsk_gemm(dY, X, dW, M=2 * F, N=d, K=T, a_kmajor=False, b_kmajor=False, lda=2 * F, ldb=d)
    wrows = [0, 7, 256, 11007, 11008, 22015]
    ref = dYh[:, wrows].T @ Xh
    assert_close(host(dW[wrows]), ref, 1e-5, "dW rows")


def test_gemm_rejects_unaligned_operands():
    a = torch.zeros(16, 12, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(16, 12, dtype=torch.bfloat16, device="cuda")
    c = torch.zeros(16, 16, dtype=torch.float32, device="cuda")
    with pytest.raises(Bd.LsError) as e:
        Bd.lsk_gemm(a, w, c, M=16, N=16, K=12)
    assert e.value.status == Bd.LS_EINVAL


@pytest.mark.parametrize("kind", [0, 1])
@pytest.mark.parametrize("hname", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("T,d", [(37, 128), (70, 768), (33, 4096), (70, 1600), (19, 2560), (9, 8192), (600, 1024)])
def test_norm_forward_and_backward(kind, hname, T, d):
    x = S.normal(3, "x", (T, d)) * 1.7 + 0.3
    pn = "f32" if hname == "f32" else "bf16"
    g = q(1.0 + S.normal(3, "g", (d,), 0.1), pn)
    b = q(S.normal(3, "b", (d,), 0.1), pn)
    dh = q(S.normal(3, "dh", (T, d)), hname)
    dres = S.normal(3, "dres", (T, d))
    x64 = x.astype(np.float64)
    if kind == 0:
        ref, xhat, r = O.layer_norm(x64, g.astype(np.float64), b.astype(np.float64), 1e-5)
        dxr, dgr, dbr = O.layer_norm_bwd(dh.astype(np.float64), xhat, r, g.astype(np.float64))
    else:
        ref, xhat, r = O.rms_norm(x64, g.astype(np.float64), 1e-5)
        dxr, dgr = O.rms_norm_bwd(dh.astype(np.float64), xhat, r, g.astype(np.float64))
    xd = dev(x, torch.float32)
    h = torch.empty(T, d, dtype=DT[hname], device="cuda")
    mean = torch.zeros(T, dtype=torch.float32, device="cuda")
    rstd = torch.zeros(T, dtype=torch.float32, device="cuda")
    gd, bd = dev(g, DT[pn]), dev(b, DT[pn])
    Bd.lsk_norm_fwd(kind, xd, gd, bd if kind == 0 else None, 1e-5, h, mean, rstd)
    assert_close(host(h), ref, otol(hname, ref, 1e-4), "norm fwd")
    assert_close(host(rstd), r[:, 0], 1e-5, "rstd")
    dx = torch.empty(T, d, dtype=torch.float32, device="cuda")
    dx16 = torch.empty(T, d, dtype=DT[hname], device="cuda")
    dgam = torch.full((d,), 1.0, dtype=torch.float32, device="cuda")
    dbet = torch.full((d,), 1.0, dtype=torch.float32, device="cuda")
    Bd.lsk_norm_bwd(kind, dev(dh, DT[hname]), xd, mean, rstd, gd, dev(dres, torch.float32), dx, dx16, dgam,
                    dbet if kind == 0 else None, True)
    assert_close(host(dx), dxr + dres, 1e-5, "norm bwd dx")
    assert_close(host(dx16), dxr + dres, otol(hname, dxr + dres, 1e-4), "norm bwd dx16")
    assert_close(host(dgam), dgr + 1.0, 1e-5, "dgamma (accumulated)")
    if kind == 0:
        assert_close(host(dbet), dbr + 1.0, 1e-5, "dbeta (accumulated)")


def rope_table(max_pos, dh, theta=1e4):
    i = np.arange(dh // 2, dtype=np.float64)
    ang = np.arange(max_pos, dtype=np.float64)[:, None] * theta ** (-2.0 * i / dh)[None, :]
    return np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)


@pytest.mark.parametrize("name", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("sign", [1.0, -1.0])
def test_rope_in_place(name, sign):
    T, h, dh = 50, 3, 128
    d = h * dh
    qkv = q(S.normal(4, "qkv", (T, 3 * d)), name)
    pos = S.uniform_ints(4, "pos", T, 0, 4095)
    ref = qkv.astype(np.float64).copy()
    for part in (0, 1):
        blk = ref[:, part * d:(part + 1) * d].reshape(T, h, dh)
        ref[:, part * d:(part + 1) * d] = O.rope(blk, pos, 1e4, sign).reshape(T, d)
    t = dev(qkv, DT[name])
    Bd.lsk_rope(t, h, dh, torch.as_tensor(pos, dtype=torch.int32, device="cuda"),
                dev(rope_table(4096, dh), torch.float32), sign)
    assert_close(host(t), ref, otol(name, ref), "rope")
    assert np.array_equal(host(t)[:, 2 * d:], qkv[:, 2 * d:].astype(np.float64))   # v untouched


@pytest.mark.parametrize("name", ["f32", "f16", "bf16"])
def test_activations(name):
    T, F = 33, 264
    u = q(S.normal(5, "u", (T, F)) * 2.0, name)
    dg = q(S.normal(5, "dg", (T, F)), name)
    for kind, kname in ((Bd.LS_ACT_GELU_TANH, "gelu_tanh"), (Bd.LS_ACT_GELU_ERF, "gelu_erf")):
        g = torch.empty(T, F, dtype=DT[name], device="cuda")
        Bd.lsk_gelu_fwd(dev(u, DT[name]), g, kind)
        r_ = O.gelu(u.astype(np.float64), kname)
        assert_close(host(g), r_, otol(name, r_), kname)
        du = torch.empty(T, F, dtype=DT[name], device="cuda")
        Bd.lsk_gelu_bwd(dev(dg, DT[name]), dev(u, DT[name]), du, kind)
        r_ = dg * O.gelu_grad(u.astype(np.float64), kname)
        assert_close(host(du), r_, otol(name, r_), kname + " bwd")
    gu = q(S.normal(5, "gu", (T, 2 * F)) * 2.0, name)
    gate, up = gu[:, :F].astype(np.float64), gu[:, F:].astype(np.float64)
    a = torch.empty(T, F, dtype=DT[name], device="cuda")
    Bd.lsk_swiglu_fwd(dev(gu, DT[name]), a)
    assert_close(host(a), O.silu(gate) * up, otol(name, O.silu(gate) * up), "swiglu")
    dgu = torch.empty(T, 2 * F, dtype=DT[name], device="cuda")
    Bd.lsk_swiglu_bwd(dev(dg, DT[name]), dev(gu, DT[name]), dgu)
    sg = O.sigmoid(gate)
    ref = np.concatenate([dg * up * sg * (1 + gate * (1 - sg)), dg * gate * sg], axis=1)
    assert_close(host(dgu), ref, otol(name, ref), "swiglu bwd")


def test_grad_scale_is_a_power_of_two_that_brings_the_maximum_to_8_16():
    for amax in (3.7e-6, 1e-2, 1.0, 15.9, 16.0, 4.0e4):
        x = torch.zeros(10000, dtype=torch.float32, device="cuda")
        x[1234] = -amax
        out = torch.zeros(3, dtype=torch.float32, device="cuda")
        Bd.lsk_grad_scale(x, out)
        sc, inv, m = out.cpu().tolist()
        assert m == np.float32(amax) and sc * inv == 1.0 and np.log2(sc) == round(np.log2(sc))
        assert 8.0 < np.float32(amax) * sc <= 16.0
    x = torch.zeros(100, dtype=torch.float16, device="cuda")
    out = torch.zeros(3, dtype=torch.float32, device="cuda")
    Bd.lsk_grad_scale(x, out)
    assert out.cpu().tolist()[:2] == [1.0, 1.0]          # all-zero gradient: no scaling
    # 16-bit input on the eight-wide path, and a ragged length on the element-wise one
    for dt, n in ((torch.bfloat16, 4096), (torch.float16, 8 * 333), (torch.float32, 1001)):
        x = (S.normal_torch(52, "gs", (n,), 1.0, dtype=torch.float32) * 0.01).to(dt)
        out = torch.zeros(3, dtype=torch.float32, device="cuda")
        Bd.lsk_grad_scale(x, out)
        assert out[2].item() == x.float().abs().max().item()


@pytest.mark.parametrize("name", ["f16", "bf16"])
@pytest.mark.parametrize("T,F,d", [(4104, 2568, 192),     # 17 x 11 tiles of 256 with ragged edges: the fused epilogue
                                    (2056, 8200, 64),      # 297 tiles, two rounds of workgroups
                                    (300, 264, 128)])      # few tiles: product, then the element-wise kernel
def test_ffn_down_input_gradient_with_swiglu_backward_in_one_call(name, T, F, d):
    """d(gate | up) of a = SiLU(gate) * up from dY and W_d, against the chain rule in float64, and bit for bit
    against the two-step route (product rounded to 16 bits, then lsk_swiglu_bwd)."""
    dt = DT[name]
    dY = q(S.normal(41, "dY", (T, d)), name)
    Wd = q(S.normal(41, "Wd", (d, F), 0.05), name)
    pre = q(S.normal(41, "pre", (T, 2 * F)), name)
    dYd, Wdd, pred = dev(dY, dt), dev(Wd, dt), dev(pre, dt)
    grad = torch.full((T, 2 * F), 7.0, dtype=dt, device="cuda")
    scratch = torch.empty(T, F, dtype=dt, device="cuda")
    Bd.lsk_gemm_swiglu_bwd(dYd, Wdd, pred, grad, scratch)
    da = dY.astype(np.float64) @ Wd.astype(np.float64)
    gate, up = pre[:, :F].astype(np.float64), pre[:, F:].astype(np.float64)
    sg = O.sigmoid(gate)
    ref = np.concatenate([da * up * sg * (1.0 + gate * (1.0 - sg)), da * gate * sg], axis=1)
    # two 16-bit roundings: da before the derivative, then the result (the products of three Gaussians have
    # elements fifty times the tensor RMS, and half an ulp of those is the whole error)
    assert_close(host(grad), ref, otol(name, ref) + out_rounding_bound(ref, name), "d(gate | up)")
    two = torch.empty_like(grad)
    Bd.lsk_gemm(dYd, Wdd, scratch, M=T, N=F, K=d, a_kmajor=True, b_kmajor=False, lda=d, ldb=F)
    Bd.lsk_swiglu_bwd(scratch, pred, two)
    assert torch.equal(grad, two), "the fused epilogue and the two-step route differ"


@pytest.mark.parametrize("name", ["f32", "f16"])
def test_colsum(name):
    T, N = 333, 520
    x = q(S.normal(6, "x", (T, N)), name)
    out = torch.ones(N, dtype=torch.float32, device="cuda")
    Bd.lsk_colsum(dev(x, DT[name]), out, accumulate=True)
    assert_close(host(out), x.astype(np.float64).sum(axis=0) + 1.0, 1e-5, "colsum")


def attn_ref(qkv, B, L, h, dh):
    d = h * dh
    o = np.empty((B * L, d))
    lse = np.empty((B * L, h))
    Ps = []
    for b in range(B):
        blk = qkv[b * L:(b + 1) * L].astype(np.float64)
        qq, kk, vv = (blk[:, i * d:(i + 1) * d].reshape(L, h, dh) for i in range(3))
        ob, P = O.attention(qq, kk, vv, 0)
        o[b * L:(b + 1) * L] = ob.reshape(L, d)
        for j in range(h):
            s = (qq[:, j] @ kk[:, j].T) / math.sqrt(dh)
            s = np.where(np.tril(np.ones((L, L), bool)), s, -np.inf)
            m = s.max(1)
            lse[b * L:(b + 1) * L, j] = m + np.log(np.exp(s - m[:, None]).sum(1))
        Ps.append((qq, kk, vv, P))
    return o, lse, Ps


@pytest.mark.parametrize("impl", [0, 1])
@pytest.mark.parametrize("name,B,L,h,dh", [("f32", 2, 64, 4, 32), ("f16", 2, 200, 3, 64), ("bf16", 1, 300, 2, 128),
                                             ("f16", 3, 129, 2, 128), ("f16", 1, 1, 2, 64),
                                             # longer than 512: 256 queries per workgroup, several key tiles in the ring
                                             ("f16", 1, 700, 2, 128), ("bf16", 2, 600, 1, 64), ("f16", 1, 1025, 1, 128)])
def test_attention_forward_and_backward(impl, name, B, L, h, dh):
    if impl == 1 and name == "f32":
        pytest.skip("matrix-core attention is 16-bit only")
    d = h * dh
    qkv = q(S.normal(7, "qkv", (B * L, 3 * d)), name)
    dO = q(S.normal(7, "dO", (B * L, d)), name)
    o_ref, lse_ref, Ps = attn_ref(qkv, B, L, h, dh)
    qd = dev(qkv, DT[name])
    o = torch.empty(B * L, d, dtype=DT[name], device="cuda")
    lse = torch.empty(B * L, h, dtype=torch.float32, device="cuda")
    Bd.lsk_attn_fwd(impl, qd, B, L, h, dh, o, lse)
    assert_close(host(o), o_ref, otol(name, o_ref, 1e-4), "attention o")
    assert np.abs(host(lse) - lse_ref).max() < (1e-4 if name == "f32" else 2e-2)
    dqkv_ref = np.empty((B * L, 3 * d))
    for b, (qq, kk, vv, P) in enumerate(Ps):
        dq, dk, dv = O.attention_bwd(dO[b * L:(b + 1) * L].astype(np.float64).reshape(L, h, dh), qq, kk, vv, P)
        dqkv_ref[b * L:(b + 1) * L] = np.concatenate([dq.reshape(L, d), dk.reshape(L, d), dv.reshape(L, d)], 1)
    dqkv = torch.empty(B * L, 3 * d, dtype=DT[name], device="cuda")
    # backward consumes the forward's own o and lse
    Bd.lsk_attn_bwd(impl, qd, o, dev(dO, DT[name]), lse, B, L, h, dh, dqkv)
    got = host(dqkv)
    for i, nm in enumerate(("dq", "dk", "dv")):
        r_ = dqkv_ref[:, i * d:(i + 1) * d]
        # L = 1: dq and dk are exactly zero in the definition; allow fp32 cancellation noise
        assert_close(got[:, i * d:(i + 1) * d], r_, otol(name, r_, 1e-4), nm, atol=1e-5 if L == 1 else 0.0)


@pytest.mark.parametrize("impl", [0, 1])
@pytest.mark.parametrize("name,B,L,h,dh", [("f32", 2, 40, 2, 32), ("f16", 2, 200, 3, 64), ("bf16", 1, 300, 2, 128),
                                             ("f16", 3, 129, 2, 128)])
def test_attention_backward_with_rotary_backward(impl, name, B, L, h, dh):
    """dq and dk leave the kernel rotated back by their positions (rotation transposed)."""
    if impl == 1 and name == "f32":
        pytest.skip("matrix-core attention is 16-bit only")
    d = h * dh
    qkv = q(S.normal(17, "qkv", (B * L, 3 * d)), name)
    dO = q(S.normal(17, "dO", (B * L, d)), name)
    _, _, Ps = attn_ref(qkv, B, L, h, dh)
    pos = np.tile(np.arange(L), B)
    ref = np.empty((B * L, 3 * d))
    for b, (qq, kk, vv, P) in enumerate(Ps):
        dq, dk, dv = O.attention_bwd(dO[b * L:(b + 1) * L].astype(np.float64).reshape(L, h, dh), qq, kk, vv, P)
        dq, dk = (O.rope(g, np.arange(L), 1e4, -1.0) for g in (dq, dk))
        ref[b * L:(b + 1) * L] = np.concatenate([dq.reshape(L, d), dk.reshape(L, d), dv.reshape(L, d)], 1)
    qd = dev(qkv, DT[name])
    o = torch.empty(B * L, d, dtype=DT[name], device="cuda")
    lse = torch.empty(B * L, h, dtype=torch.float32, device="cuda")
    Bd.lsk_attn_fwd(impl, qd, B, L, h, dh, o, lse)
    dqkv = torch.empty(B * L, 3 * d, dtype=DT[name], device="cuda")
    Bd.lsk_attn_bwd_rope(impl, qd, o, dev(dO, DT[name]), lse, B, L, h, dh, dqkv,
                         torch.as_tensor(pos, dtype=torch.int32, device="cuda"),
                         dev(rope_table(L + 3, dh), torch.float32))
    got = host(dqkv)
    for i, nm in enumerate(("dq", "dk", "dv")):
        r_ = ref[:, i * d:(i + 1) * d]
        assert_close(got[:, i * d:(i + 1) * d], r_, otol(name, r_, 1e-4), nm + " (rotary backward)")


@pytest.mark.parametrize("name,B,L,h,heads", [
    ("f16", 2, 2048, 32, [(0, 0), (0, 17), (1, 31)]),      # the training micro-batch of the LLaMA-7B-shaped stage
    ("bf16", 1, 2048, 32, [(0, 5)]),                       # config 4's training stream, bf16 operands
    ("f16", 1, 4096, 40, [(0, 0), (0, 39)]),               # LLaMA-13B-shaped stage, one sequence of 4096
    ("f16", 1, 4096, 2, [(0, 0), (0, 1)]),                 # few heads: every (sequence, head) pair checked
    # launches in which a forward workgroup takes several query tiles of a head in a row: three of nine (the last
    # tile short, with an odd number of key tiles), all four (sequence end inside a key tile)
    ("f16", 5, 1064, 32, [(0, 3), (2, 16), (4, 31)]),
    ("f16", 8, 500, 32, [(0, 0), (7, 31)]),
])
def test_attention_at_the_benchmarked_sizes_on_sampled_heads(name, B, L, h, heads):
    """The launches bench.py times (head_dim 128, all heads, L = 2048 and 4096: 16 and 32 query tiles
    per head, dispatched heaviest first over every head, one or several to a workgroup), forward and both backward
    kernels, with and without the fused rotary backward.  The float64 definition is formed for the sampled (sequence,
    head) pairs only: heads do not interact, and one head's 4096 x 4096 probability matrix is 134 MB."""
    dh = 128
    d = h * dh
    dt = DT[name]
    qd = S.normal_torch(23, "qkv", (B * L, 3 * d), 1.0, "cuda", dt)
    dOd = S.normal_torch(23, "dO", (B * L, d), 1.0, "cuda", dt)
    o = torch.empty(B * L, d, dtype=dt, device="cuda")
    lse = torch.empty(B * L, h, dtype=torch.float32, device="cuda")
    Bd.lsk_attn_fwd(1, qd, B, L, h, dh, o, lse)
    dqkv = torch.empty(B * L, 3 * d, dtype=dt, device="cuda")
    Bd.lsk_attn_bwd(1, qd, o, dOd, lse, B, L, h, dh, dqkv)
    dqkv_r = torch.empty_like(dqkv)
    pos = torch.arange(L, dtype=torch.int32, device="cuda").repeat(B)
    Bd.lsk_attn_bwd_rope(1, qd, o, dOd, lse, B, L, h, dh, dqkv_r, pos, dev(rope_table(L, dh), torch.float32))
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all() and torch.isfinite(dqkv.float()).all()
    for b, j in heads:
        rows = slice(b * L, (b + 1) * L)
        col = lambda part: slice(part * d + j * dh, part * d + (j + 1) * dh)
        qq, kk, vv = (host(qd[rows, col(i)]).reshape(L, 1, dh) for i in range(3))
        do = host(dOd[rows, col(0)]).reshape(L, 1, dh)
        o_ref, P = O.attention(qq, kk, vv, 0)
        what = f"{name} L={L} sequence {b} head {j}: "
        assert_close(host(o[rows, col(0)]), o_ref.reshape(L, dh), otol(name, o_ref, 1e-4), what + "o")
        sc = (qq[:, 0] @ kk[:, 0].T) / math.sqrt(dh)
        sc = np.where(np.tril(np.ones((L, L), bool)), sc, -np.inf)
        m = sc.max(1)
        lse_ref = m + np.log(np.exp(sc - m[:, None]).sum(1))
        assert np.abs(host(lse[rows, j]) - lse_ref).max() < 2e-2
        dq, dk, dv = O.attention_bwd(do, qq, kk, vv, P)
        for i, (nm, r_) in enumerate((("dq", dq), ("dk", dk), ("dv", dv))):
            r_ = r_.reshape(L, dh)
            assert_close(host(dqkv[rows, col(i)]), r_, otol(name, r_, 1e-4), what + nm)
            if i < 2:
                r_ = O.rope(r_.reshape(L, 1, dh), np.arange(L), 1e4, -1.0).reshape(L, dh)
            assert_close(host(dqkv_r[rows, col(i)]), r_, otol(name, r_, 1e-4), what + nm + " (rotary backward)")


@pytest.mark.parametrize("name", ["f16", "bf16"])
@pytest.mark.parametrize("B,L,h,heads", [(5, 1064, 32, [(0, 3), (2, 16), (4, 31)]), (8, 500, 32, [(0, 0), (3, 9), (7, 31)]),
                                         (4, 2048, 32, [(0, 0), (3, 31)]), (16, 2048, 32, [(0, 0), (9, 20), (15, 31)])])
def test_attention_forward_over_several_query_tiles_per_workgroup(name, B, L, h, heads):
    """Forward launches (head_dim 128) whose workgroups take 3, 4, 8 and all 16 query tiles of a head in a row, the key
    tiles of one flowing into the next: o and the log-sum-exp of sampled (sequence, head) pairs against the
    definition, in both 16-bit formats."""
    dh = 128
    d = h * dh
    dt = DT[name]
    qd = S.normal_torch(29, "qkv", (B * L, 3 * d), 1.0, "cuda", dt)
    o = torch.empty(B * L, d, dtype=dt, device="cuda")
    lse = torch.empty(B * L, h, dtype=torch.float32, device="cuda")
    Bd.lsk_attn_fwd(1, qd, B, L, h, dh, o, lse)
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all() and torch.isfinite(lse).all()
    for b, j in heads:
        rows = slice(b * L, (b + 1) * L)
        qq, kk, vv = (host(qd[rows, i * d + j * dh:i * d + (j + 1) * dh]).reshape(L, 1, dh) for i in range(3))
        o_ref, _ = O.attention(qq, kk, vv, 0)
        what = f"{name} B={B} L={L} sequence {b} head {j}: "
        assert_close(host(o[rows, j * dh:(j + 1) * dh]), o_ref.reshape(L, dh), otol(name, o_ref, 1e-4), what + "o")
        sc = (qq[:, 0] @ kk[:, 0].T) / math.sqrt(dh)
        sc = np.where(np.tril(np.ones((L, L), bool)), sc, -np.inf)
        m = sc.max(1)
        assert np.abs(host(lse[rows, j]) - (m + np.log(np.exp(sc - m[:, None]).sum(1)))).max() < 2e-2, what + "lse"


@pytest.mark.parametrize("name", ["f16", "bf16"])
@pytest.mark.parametrize("T,h,dh", [(70, 2, 64), (300, 3, 128), (4096, 32, 128), (2304, 16, 128), (2048, 32, 128)])
def test_qkv_projection_with_fused_rotary_embedding(name, T, h, dh):
    """(4096, 32, 128) is the training launch configuration with the rotation in the GEMM epilogue
    (checked on sampled rows); the small shapes take the GEMM + in-place rotation route."""
    d = h * dh
    dt = DT[name]
    hd = S.normal_torch(21, "h", (T, d), 1.0, dtype=dt)
    wd = S.normal_torch(21, "w", (3 * d, d), d ** -0.5, dtype=dt)
    pos = S.uniform_ints(21, "pos", T, 0, 2047).astype(np.int32)
    qkv = torch.empty(T, 3 * d, dtype=dt, device="cuda")
    Bd.lsk_gemm_qkv_rope(hd, wd, qkv, h, dh, torch.as_tensor(pos, device="cuda"),
                         dev(rope_table(2048, dh), torch.float32))
    rows = np.arange(T) if T <= 300 else np.unique(np.concatenate(
        [[0, 1, 127, 128, 255, 256, T - 1], S.uniform_ints(22, "rows", 40, 0, T - 1)]))
    W = host(wd)
    ref = host(hd[torch.as_tensor(rows, device="cuda")]) @ W.T
    for part in (0, 1):
        blk = ref[:, part * d:(part + 1) * d].reshape(len(rows), h, dh)
        ref[:, part * d:(part + 1) * d] = O.rope(blk, pos[rows], 1e4, 1.0).reshape(len(rows), d)
    got = host(qkv[torch.as_tensor(rows, device="cuda")])
    # two 16-bit roundings on the unfused route (GEMM output, then the rotated value)
    tol = otol(name, ref) + out_rounding_bound(ref, name)
    for part, nm in enumerate(("q", "k", "v")):
        sl = slice(part * d, (part + 1) * d)
        assert_close(got[:, sl], ref[:, sl], tol, "qkv+rope " + nm)


@pytest.mark.parametrize("fill", ["gauss", "nan", "inf"])
@pytest.mark.parametrize("impl", [0, 1])
@pytest.mark.parametrize("name,h,dh,P", [("f32", 4, 32, 16), ("f16", 2, 128, 16), ("bf16", 3, 64, 8)])
def test_paged_attention_ragged(impl, name, h, dh, P, fill):
    """`fill`: what the slots that no request has written hold - the tail of every last page and the spare
    pages.  A pool straight from the allocator may hold any bit pattern there, NaN and infinity included,
    and none of it may reach a result."""
    if impl == 1 and name == "f32":
        pytest.skip("optimised paged attention is 16-bit only")
    d = h * dh
    ctx = np.array([0, 5, 16, 100, 333, 47])          # cached tokens per request
    new = np.array([1, 1, 3, 1, 20, 40])              # decode rows and prefill chunks mixed
    table, n_pages = S.page_tables(ctx, new, P, seed=3)
    rng = np.random.default_rng(0)
    T = int(new.sum())
    qkv = q(S.normal(8, "qkv", (T, 3 * d)), name)
    kp = q(rng.normal(0, 1, (n_pages, h, P, dh)), name)   # garbage everywhere, real rows overwritten below
    vp = q(rng.normal(0, 1, (n_pages, h, P, dh)), name)
    if fill == "nan":
        kp[:], vp[:] = np.nan, np.nan
    elif fill == "inf":
        kp[:] = np.where(rng.random(kp.shape) < 0.5, np.inf, -np.inf)
        vp[:] = np.where(rng.random(vp.shape) < 0.5, np.inf, -np.inf)
    Kc = [q(S.normal(8, f"K{b}", (int(c), h, dh)), name) for b, c in enumerate(ctx)]
    Vc = [q(S.normal(8, f"V{b}", (int(c), h, dh)), name) for b, c in enumerate(ctx)]
    for b in range(len(ctx)):
        for j in range(int(ctx[b])):
            kp[table[b, j // P], :, j % P] = Kc[b][j]
            vp[table[b, j // P], :, j % P] = Vc[b][j]
    pos = np.concatenate([ctx[b] + np.arange(new[b]) for b in range(len(ctx))]).astype(np.int32)
    req = np.concatenate([np.full(new[b], b) for b in range(len(ctx))]).astype(np.int32)
    kd, vd = dev(kp, DT[name]), dev(vp, DT[name])
    qd = dev(qkv, DT[name])
    bt = torch.as_tensor(table, dtype=torch.int32, device="cuda")
    posd, reqd = torch.as_tensor(pos, device="cuda"), torch.as_tensor(req, device="cuda")
    Bd.lsk_kv_write(qd, h, dh, posd, reqd, kd, vd, bt, P)
    o = torch.empty(T, d, dtype=DT[name], device="cuda")
    Bd.lsk_attn_paged(impl, qd, h, dh, posd, reqd, kd, vd, bt, P, int((ctx + new).max()), o)
    ref = np.empty((T, d))
    t0 = 0
    for b in range(len(ctx)):
        rows = qkv[t0:t0 + new[b]].astype(np.float64)
        qq, kn, vn = (rows[:, i * d:(i + 1) * d].reshape(-1, h, dh) for i in range(3))
        K = np.concatenate([Kc[b].astype(np.float64), kn]); V = np.concatenate([Vc[b].astype(np.float64), vn])
        ob, _ = O.attention(qq, K, V, int(ctx[b]))
        ref[t0:t0 + new[b]] = ob.reshape(-1, d)
        # the new rows landed in the right page slots, bit-exactly
        kh = host(kd)
        for i in range(new[b]):
            j = int(ctx[b]) + i
            assert np.array_equal(kh[table[b, j // P], :, j % P], kn[i])
        t0 += new[b]
    assert_close(host(o), ref, otol(name, ref, 1e-4), "paged attention")


@pytest.mark.parametrize("name,h,dh,P", [("f32", 2, 32, 16), ("f16", 3, 128, 16), ("bf16", 2, 64, 8), ("f16", 2, 36, 4)])
@pytest.mark.parametrize("rotate", [True, False])
def test_rope_and_page_write_in_one_pass(name, h, dh, P, rotate):
    """q and k rotated in place as the oracle's rope does, the (rotated) k rows and the v rows bit-exactly in
    their page slots, every other slot untouched; 16-bit data with head_dim % 8 == 0 takes the vectorised
    kernel, head_dim 36 and fp32 the scalar one."""
    d = h * dh
    ctx = np.array([0, 7, 16, 250])
    new = np.array([1, 3, 33, 70])
    table, n_pages = S.page_tables(ctx, new, P, seed=5)
    T = int(new.sum())
    qkv = q(S.normal(11, "qkv", (T, 3 * d)), name)
    rng = np.random.default_rng(1)
    kp = q(rng.normal(0, 1, (n_pages, h, P, dh)), name)
    vp = q(rng.normal(0, 1, (n_pages, h, P, dh)), name)
    pos = np.concatenate([ctx[b] + np.arange(new[b]) for b in range(len(ctx))]).astype(np.int32)
    req = np.concatenate([np.full(new[b], b) for b in range(len(ctx))]).astype(np.int32)
    qd, kd, vd = dev(qkv, DT[name]), dev(kp, DT[name]), dev(vp, DT[name])
    bt = torch.as_tensor(table, dtype=torch.int32, device="cuda")
    Bd.lsk_rope_kv_write(qd, h, dh, torch.as_tensor(pos, device="cuda"), torch.as_tensor(req, device="cuda"),
                         dev(rope_table(512, dh), torch.float32) if rotate else None, kd, vd, bt, P)
    out, kh, vh = host(qd), host(kd), host(vd)
    ref = qkv.astype(np.float64).copy()
    if rotate:
        for part in (0, 1):
            blk = ref[:, part * d:(part + 1) * d].reshape(T, h, dh)
            ref[:, part * d:(part + 1) * d] = O.rope(blk, pos, 1e4, 1.0).reshape(T, d)
        assert_close(out, ref, otol(name, ref), "q and k rotated in place")
    else:
        assert np.array_equal(out, ref)
    assert np.array_equal(out[:, 2 * d:], qkv[:, 2 * d:].astype(np.float64))   # v untouched
    written = np.zeros((n_pages, P), dtype=bool)
    for t in range(T):
        pg, slot = table[req[t], pos[t] // P], pos[t] % P
        written[pg, slot] = True
        assert np.array_equal(kh[pg, :, slot], out[t, d:2 * d].reshape(h, dh)), t
        assert np.array_equal(vh[pg, :, slot], out[t, 2 * d:].reshape(h, dh)), t
    keep = ~written
    assert np.array_equal(kh.transpose(0, 2, 1, 3)[keep], kp.astype(np.float64).transpose(0, 2, 1, 3)[keep])
    assert np.array_equal(vh.transpose(0, 2, 1, 3)[keep], vp.astype(np.float64).transpose(0, 2, 1, 3)[keep])


@pytest.mark.parametrize("src,dst", [("f32", "bf16"), ("f32", "f16"), ("bf16", "f32"), ("f16", "f32"), ("bf16", "f16"),
                                     ("f16", "bf16"), ("f32", "f32")])
@pytest.mark.parametrize("n,offset", [(8 * 1000, 0), (8 * 1000 + 3, 0), (4096, 1), (5, 0)])
def test_convert_is_the_rounding_of_each_element(src, dst, n, offset):
    """Bit-exact against the host conversion (round to nearest even), on the 8-wide path (length a multiple of
    8, 16-byte aligned) and on the element-wise path (ragged length, misaligned views)."""
    x = S.normal_torch(51, "cv", (n + offset,), 3.0, dtype=DT[src])[offset:]
    y = torch.full((n + offset,), 7.0, dtype=DT[dst], device="cuda")[offset:]
    Bd.lsk_convert(x, y)
    assert torch.equal(y, x.to(DT[dst]))
