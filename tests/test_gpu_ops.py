"""Kernel-by-kernel parity through the C interface against the float64
reference functions, in the fp32 tier (1e-4) and the bf16 tier."""
import numpy as np
import pytest
import torch

import oracle
from oracle import model as om
import synth
from helpers import grad_norm_err

pytestmark = pytest.mark.gpu
FP32_TOL, BF16_TOL = 1e-4, 3e-2


def _env(**kw):
    from paper_2503_22673_amd import binding as B
    import gpu_util as G
    sh = synth.CONFIGS[1].replace(**kw)
    return B, G, B.Context(B.make_config(sh)), sh


# (M, N, K1, K2): several tiles + ragged tails, and the shapes of the tiny config
GEMM_SHAPES = [(512, 128, 128, 64), (512, 344, 128, 0), (512, 128, 344, 64), (300, 200, 72, 0), (1, 7, 8, 8),
               (700, 1024, 256, 64), (64, 520, 1024, 0), (1000, 520, 192, 64), (1024, 512, 256, 64), (768, 256, 64, 0),
               (512, 256, 128, 128), (300, 256, 192, 64), (700, 64, 256, 0), (515, 48, 136, 64)]


@pytest.mark.parametrize("shape", GEMM_SHAPES)
@pytest.mark.parametrize("tier", ["fp32", "bf16_fma", "bf16_mfma", "bf16_mfma_dlds", "bf16_mfma_rs"])
def test_gemm_with_lora_segment_and_residual(shape, tier):
    B, G, ctx, _ = _env()
    M, N, K1, K2 = shape
    bf16 = tier != "fp32"
    dt = torch.bfloat16 if bf16 else torch.float32
    g = synth.rng(1, 20)
    A1, B1 = G.quantise(g.standard_normal((M, K1)), bf16), G.quantise(g.standard_normal((N, K1)), bf16)
    R = G.quantise(g.standard_normal((M, N)), bf16)
    ref = A1 @ B1.T
    A2 = B2 = None
    if K2:
        A2, B2 = G.quantise(g.standard_normal((M, K2)), bf16), G.quantise(g.standard_normal((N, K2)), bf16)
        ref = ref + A2 @ B2.T
    ref = 0.5 * ref + R
    variant = {"fp32": 1, "bf16_fma": 1, "bf16_mfma": 2, "bf16_mfma_dlds": 30, "bf16_mfma_rs": 34}[tier]
    out = ctx.op_gemm(G.to_dev(A1, dt), G.to_dev(B1, dt), G.to_dev(A2, dt) if K2 else None,
                      G.to_dev(B2, dt) if K2 else None, alpha=0.5, R=G.to_dev(R, dt), out_f32=True, variant=variant,
                      mode=B.AS_BF16 if bf16 else B.AS_FP32)
    torch.cuda.synchronize()
    # float accumulation of exact products: only summation rounding remains
    assert grad_norm_err(G.to_np(out), ref) < 2e-6 * max(1, (K1 + K2)) ** 0.5 + 1e-6


@pytest.mark.parametrize("with_residual", [False, True])
@pytest.mark.parametrize("shape", [(512, 512, 256, 64), (768, 256, 128, 0), (1280, 768, 64, 64)])
def test_hand_scheduled_gemm_bf16_output(shape, with_residual):
    """bf16 results of the hand-scheduled kernel leave through LDS (residual included): one rounding of alpha * sum + R"""
    B, G, ctx, _ = _env()
    M, N, K1, K2 = shape
    g = synth.rng(5, 20)
    A1, B1 = G.quantise(g.standard_normal((M, K1)), True), G.quantise(g.standard_normal((N, K1)), True)
    R = G.quantise(g.standard_normal((M, N)), True) if with_residual else None
    ref = A1 @ B1.T
    A2 = B2 = None
    if K2:
        A2, B2 = G.quantise(g.standard_normal((M, K2)), True), G.quantise(g.standard_normal((N, K2)), True)
        ref = ref + A2 @ B2.T
    ref = 0.25 * ref + (R if with_residual else 0.0)
    dt = torch.bfloat16
    args = (G.to_dev(A1, dt), G.to_dev(B1, dt), G.to_dev(A2, dt) if K2 else None, G.to_dev(B2, dt) if K2 else None)
    kw = dict(alpha=0.25, R=G.to_dev(R, dt) if with_residual else None, mode=B.AS_BF16)
    out = ctx.op_gemm(*args, variant=34, **kw)
    torch.cuda.synchronize()
    assert out.dtype == torch.bfloat16
    got = G.to_np(out)
    # one rounding to bf16 of a float sum of exact products: half an ulp plus the summation error
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-4 * (K1 + K2) ** 0.5)
    # same summation order as the eight-wave kernel: the same bits
    other = ctx.op_gemm(*args, variant=30, **kw)
    torch.cuda.synchronize()
    assert torch.equal(out, other)


@pytest.mark.parametrize("out_f32,with_residual", [(False, True), (False, False), (True, True)])
def test_hand_scheduled_gemm_split_last_round(out_f32, with_residual):
    """17 x 16 = 272 tiles on 256 CUs: one full round, then 16 tiles whose contraction (2048 + the 64-wide adapter segment)
    is split over two workgroups each and summed by the second launch; every entry against float64."""
    B, G, ctx, _ = _env()
    M, N, K1, K2 = 4352, 4096, 2048, 64
    g = synth.rng(9, 20)
    A1, B1 = G.quantise(g.standard_normal((M, K1)), True), G.quantise(g.standard_normal((N, K1)), True)
    A2, B2 = G.quantise(g.standard_normal((M, K2)), True), G.quantise(g.standard_normal((N, K2)), True)
    R = G.quantise(g.standard_normal((M, N)), True) if with_residual else None
    ref = 0.5 * (A1 @ B1.T + A2 @ B2.T) + (R if with_residual else 0.0)
    dt = torch.bfloat16
    args = (G.to_dev(A1, dt), G.to_dev(B1, dt), G.to_dev(A2, dt), G.to_dev(B2, dt))
    kw = dict(alpha=0.5, R=G.to_dev(R, dt) if with_residual else None, out_f32=out_f32, mode=B.AS_BF16, variant=34)
    scratch = torch.empty(B.GEMM_TAIL_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
    out = ctx.op_gemm(*args, tail_scratch=scratch, **kw)
    plain = ctx.op_gemm(*args, **kw)
    torch.cuda.synchronize()
    got = G.to_np(out)
    if out_f32:
        assert grad_norm_err(got, ref) < 2e-6 * (K1 + K2) ** 0.5 + 1e-6
    else:
        assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-4 * (K1 + K2) ** 0.5)
    # the tiles of the full round are the same bits with and without the split; the split ones differ in summation order only
    same = (out == plain).float().mean().item()
    assert 0.9 < same < 1.0 or out_f32 is False, same
    assert np.abs(got - G.to_np(plain)).max() <= (1e-4 if out_f32 else 2.0 ** -7) * np.abs(ref).max()


@pytest.mark.parametrize("out_f32", [False, True])
@pytest.mark.parametrize("variant", [0, 30, 34])
@pytest.mark.parametrize("row_off,live", [(0, 700), (128, 896), (0, 0), (256, 1)])
def test_gemm_over_a_device_side_row_count(variant, out_f32, row_off, live):
    """rows row_off .. row_off + live - 1 are computed (the count lives on the device), the others keep their contents;
    variant 34 is the hand-scheduled kernel, which moves its last, ragged tile up inside the M rows it may read"""
    B, G, ctx, _ = _env()
    M, N, K = 1024, 512, 192
    g = synth.rng(6, 20)
    A, W, R = (G.quantise(g.standard_normal(s), True) for s in ((M, K), (N, K), (M, N)))
    dt = torch.bfloat16
    dA, dW, dR = G.to_dev(A, dt), G.to_dev(W, dt), G.to_dev(R, dt)
    Cm = torch.full((M, N), 7.0, dtype=torch.float32 if out_f32 else dt, device="cuda")
    rows = torch.tensor([row_off + live], dtype=torch.int32, device="cuda")
    ctx.op_gemm_rows(dA[row_off:], dW, Cm[row_off:], alpha=0.5, R=dR[row_off:], d_rows=rows, row_off=row_off, M=M - row_off,
                     variant=variant, mode=B.AS_BF16)
    torch.cuda.synchronize()
    got = G.to_np(Cm)
    ref = np.full((M, N), 7.0)
    ref[row_off:row_off + live] = 0.5 * (A[row_off:row_off + live] @ W.T) + R[row_off:row_off + live]
    assert np.array_equal(got[:row_off], ref[:row_off]) and np.array_equal(got[row_off + live:], ref[row_off + live:])
    tol = 1e-5 if out_f32 else 2.0 ** -8
    assert np.all(np.abs(got - ref) <= tol * np.abs(ref) + 1e-4 * K ** 0.5)


@pytest.mark.parametrize("out_f32", [False, True])
@pytest.mark.parametrize("variant", [0, 30, 34])
def test_gemm_over_the_rows_of_one_group(variant, out_f32):
    """one launch per group of rows (an expert's rows), the table on the device: an empty group, ragged ones, and a last
    group whose final tile would reach past the rows_cap rows of the buffers"""
    B, G, ctx, _ = _env()
    cap, N, K = 1300, 256, 128
    off_host = [0, 300, 300, 1000, 1300]
    g = synth.rng(7, 20)
    A, R = G.quantise(g.standard_normal((cap, K)), True), G.quantise(g.standard_normal((cap, N)), True)
    Ws = [G.quantise(g.standard_normal((N, K)), True) for _ in range(4)]
    dt = torch.bfloat16
    dA, dR = G.to_dev(A, dt), G.to_dev(R, dt)
    Cm = torch.full((cap, N), 7.0, dtype=torch.float32 if out_f32 else dt, device="cuda")
    off = torch.tensor(off_host, dtype=torch.int32, device="cuda")
    ref = np.full((cap, N), 7.0)
    for e in (2, 0, 1):                                   # group 3 is left out: its rows must stay untouched
        ctx.op_gemm_rows(dA, G.to_dev(Ws[e], dt), Cm, R=dR, d_group_off=off, group=e, rows_cap=cap, M=cap, variant=variant, mode=B.AS_BF16)
        ref[off_host[e]:off_host[e + 1]] = A[off_host[e]:off_host[e + 1]] @ Ws[e].T + R[off_host[e]:off_host[e + 1]]
    torch.cuda.synchronize()
    got = G.to_np(Cm)
    assert np.array_equal(got[1000:], ref[1000:])
    tol = 1e-5 if out_f32 else 2.0 ** -8
    assert np.all(np.abs(got - ref) <= tol * np.abs(ref) + 1e-4 * K ** 0.5)
    ctx.op_gemm_rows(dA, G.to_dev(Ws[3], dt), Cm, R=dR, d_group_off=off, group=3, rows_cap=cap, M=cap, variant=variant, mode=B.AS_BF16)
    torch.cuda.synchronize()
    got = G.to_np(Cm)
    ref[1000:] = A[1000:] @ Ws[3].T + R[1000:]
    assert np.all(np.abs(got - ref) <= tol * np.abs(ref) + 1e-4 * K ** 0.5)
    # every group in one call, the matrices stacked
    C2 = torch.full((cap, N), 7.0, dtype=Cm.dtype, device="cuda")
    ctx.op_gemm_rows(dA, G.to_dev(np.stack(Ws), dt), C2, R=dR, d_group_off=off, n_groups=4, rows_cap=cap, M=cap, variant=variant, mode=B.AS_BF16)
    torch.cuda.synchronize()
    assert torch.equal(C2, Cm)
    # ... and with a table that leaves rows out at both ends
    off2 = torch.tensor([40, 300, 300, 1000, 1290], dtype=torch.int32, device="cuda")
    C3 = torch.full((cap, N), 7.0, dtype=Cm.dtype, device="cuda")
    ctx.op_gemm_rows(dA, G.to_dev(np.stack(Ws), dt), C3, R=dR, d_group_off=off2, n_groups=4, rows_cap=cap, M=cap, variant=variant, mode=B.AS_BF16)
    torch.cuda.synchronize()
    assert torch.equal(C3[40:1290], Cm[40:1290]) and bool((C3[:40] == 7.0).all()) and bool((C3[1290:] == 7.0).all())


def test_gemm_mfma_typed_output_and_strides():
    B, G, ctx, _ = _env()
    g = synth.rng(2, 20)
    M, N, K = 520, 300, 128
    big = G.to_dev(G.quantise(g.standard_normal((M, 3 * K)), True), torch.bfloat16)
    A = big[:, K:2 * K]                                   # row stride 3K
    Bm = G.to_dev(G.quantise(g.standard_normal((N, K)), True), torch.bfloat16)
    out = ctx.op_gemm(A, Bm, variant=2, mode=B.AS_BF16)
    torch.cuda.synchronize()
    ref = G.to_np(A) @ G.to_np(Bm).T
    assert out.dtype == torch.bfloat16
    assert grad_norm_err(G.to_np(out), ref) < 2 ** -8


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("n,d", [(512, 128), (37, 344), (5, 12), (130, 4096)])
def test_rmsnorm_forward_and_backward(bf16, n, d):
    B, G, ctx, _ = _env()
    dt = torch.bfloat16 if bf16 else torch.float32
    g = synth.rng(3, 21)
    x, gain, dy = (G.quantise(g.standard_normal((n, d)), bf16), G.quantise(1 + 0.1 * g.standard_normal(d), bf16),
                   G.quantise(g.standard_normal((n, d)), bf16))
    add = G.quantise(g.standard_normal((n, d)), bf16)
    y_ref, rho = om.rmsnorm(x, gain, 1e-5)
    dx_ref, _ = om.rmsnorm_bwd(dy, x, gain, rho)
    mode = B.AS_BF16 if bf16 else B.AS_FP32
    y, rstd = ctx.op_rmsnorm_fwd(G.to_dev(x, dt), G.to_dev(gain, dt), 1e-5, mode=mode)
    dx = ctx.op_rmsnorm_bwd(G.to_dev(dy, dt), G.to_dev(x, dt), G.to_dev(gain, dt), rstd, add=G.to_dev(add, dt), mode=mode)
    torch.cuda.synchronize()
    tol = 2 ** -8 if bf16 else 1e-6
    assert grad_norm_err(G.to_np(rstd), rho) < 1e-6
    assert grad_norm_err(G.to_np(y), y_ref) < tol
    assert grad_norm_err(G.to_np(dx), dx_ref + add) < tol


def _attn_case(seed, n_seg, Hq, Hkv, dh, lens):
    g = synth.rng(seed, 22)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    n = int(cu[-1])
    return g, cu, n


@pytest.mark.parametrize("tier", ["fp32", "bf16_plain", "bf16_mfma", "bf16_mfma_two_pass"])
@pytest.mark.parametrize("Hq,Hkv,dh,lens,late_gain", [(4, 4, 32, [100, 1, 63, 200, 148], 1.0), (8, 2, 64, [130, 257, 64, 5], 1.0),
                                                      (4, 1, 128, [300, 70, 129], 1.0), (2, 2, 64, [200, 90], 1.0),
                                                      (4, 2, 128, [65, 190], 1.0), (4, 1, 128, [700, 3, 420], 5.0),
                                                      (2, 1, 64, [515, 333], 5.0), (2, 2, 128, [333, 97, 260], 1.0)])
def test_attention_forward_and_backward(tier, Hq, Hkv, dh, lens, late_gain):
    """late_gain > 1 scales the keys of the last third of every segment, so that the running maximum of
    the online softmax jumps by many octaves late in a row (the rare rescale path of the MFMA kernels)."""
    B, G, ctx, sh = _env(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=dh)
    bf16 = tier != "fp32"
    variant = {"fp32": 1, "bf16_plain": 1, "bf16_mfma": 2, "bf16_mfma_two_pass": 4}[tier]
    if tier.startswith("bf16_mfma") and dh == 32:
        pytest.skip("the MFMA attention kernels cover head_dim 64 and 128")
    dt = torch.bfloat16 if bf16 else torch.float32
    g, cu, n = _attn_case(4, len(lens), Hq, Hkv, dh, lens)
    q = G.quantise(g.standard_normal((n, Hq, dh)), bf16)
    k = g.standard_normal((n, Hkv, dh))
    for s0, s1 in zip(cu[:-1], cu[1:]):
        k[s0 + 2 * (s1 - s0) // 3:s1] *= late_gain
    k = G.quantise(k, bf16)
    v = G.quantise(g.standard_normal((n, Hkv, dh)), bf16)
    do = G.quantise(g.standard_normal((n, Hq, dh)), bf16)
    o_ref, probs = om.attention(q, k, v, cu, Hq // Hkv)
    dq_ref, dk_ref, dv_ref = om.attention_bwd(do, q, k, v, o_ref, probs, cu, Hq // Hkv)
    qkv = np.concatenate([q.reshape(n, -1), k.reshape(n, -1), v.reshape(n, -1)], axis=1)
    seg = om.segment_ids(cu, n)
    seg_start = torch.from_numpy(cu[seg].astype(np.int32)).cuda()
    seg_end = torch.from_numpy(cu[seg + 1].astype(np.int32)).cuda()
    mode = B.AS_BF16 if bf16 else B.AS_FP32
    qkv_d = G.to_dev(qkv, dt)
    o, lse = ctx.op_attention_fwd(qkv_d, seg_start, variant=variant, mode=mode)
    # feed the backward the reference output rounded to the device type, so
    # the two checks are independent
    o_in = G.to_dev(o_ref.reshape(n, -1), dt)
    dqkv = ctx.op_attention_bwd(qkv_d, seg_start, seg_end, o_in, lse, G.to_dev(do.reshape(n, -1), dt), variant=variant, mode=mode)
    torch.cuda.synchronize()
    tol = 2e-2 if bf16 else 1e-5
    assert grad_norm_err(G.to_np(o), o_ref.reshape(n, -1)) < tol
    D, Dkv = Hq * dh, Hkv * dh
    got = G.to_np(dqkv)
    assert grad_norm_err(got[:, :D], dq_ref.reshape(n, -1)) < tol
    assert grad_norm_err(got[:, D:D + Dkv], dk_ref.reshape(n, -1)) < tol
    assert grad_norm_err(got[:, D + Dkv:], dv_ref.reshape(n, -1)) < tol
    # lse against the definition on a few rows
    for t in (0, n // 2, n - 1):
        s0 = cu[seg[t]]
        sc = (k[s0:t + 1, 0] @ q[t, 0]) / np.sqrt(dh)
        ref = sc.max() + np.log(np.exp(sc - sc.max()).sum())
        assert abs(float(lse[t, 0]) - ref) < (2e-2 if bf16 else 1e-4)
