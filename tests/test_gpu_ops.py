"""GPU parity of the single kernels against their definitions (numpy fp64 /
the oracle's block pieces): GEMM layouts and epilogues, LayerNorm, column sums,
attention forward and backward."""

import math

import numpy as np
import pytest
import torch

from oracle import block as OB
from paper_2308_15762_amd import hanayo as hn
from paper_2308_15762_amd import synth
from helpers import TOL, dev, host, perr

pytestmark = pytest.mark.gpu

DT = {"fp32": hn.FP32, "bf16": hn.BF16}


def rnd(rng, shape, dtype, scale=1.0):
    a = (scale * rng.normal(size=shape)).astype(np.float32)
    return synth.bf16_round(a) if dtype == "bf16" else a


GEMM_SHAPES = [
    # M, N, K
    (256, 256, 128),        # one or a few tiles
    (384, 640, 192),        # several 128-tiles
    (200, 136, 72),         # ragged in every dimension
    (4096, 4096, 128),      # enough tiles for the 256 x 256 configuration
    (4104, 4120, 136),      # the same with ragged edges
    (128, 256, 2048),       # long reduction (split K for the accumulate epilogue)
]
LAYOUTS = {"fwd": (False, True), "dx": (False, False), "dw": (True, True)}
EPIS = {"fwd": [hn.EPI_BIAS, hn.EPI_BIAS_GELU, hn.EPI_BIAS_RES],
        "dx": [hn.EPI_NONE, hn.EPI_MUL_DGELU, hn.EPI_ADD],
        "dw": [hn.EPI_ACCUM_F32]}


@pytest.fixture
def gemm_config(request):
    hn.hanayo_op_gemm_config(request.param)
    yield request.param
    hn.hanayo_op_gemm_config(-1)


# every bf16 MFMA kernel variant on shapes that are whole numbers of its tile
@pytest.mark.parametrize("gemm_config", [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11], indirect=True)
@pytest.mark.parametrize("layout", list(LAYOUTS))
@pytest.mark.parametrize("shape", [(512, 768, 256), (256, 256, 32), (1024, 512, 96), (512, 512, 192), (256, 512, 64)])
def test_gemm_kernel_variants(gemm_config, layout, shape):
    run_gemm_case("bf16", layout, shape)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("layout", list(LAYOUTS))
@pytest.mark.parametrize("shape", GEMM_SHAPES)
def test_gemm(dtype, layout, shape):
    run_gemm_case(dtype, layout, shape)


@pytest.mark.parametrize("dtype,shapes", [
    ("bf16", [(512, 384, 256), (128, 128, 256), (256, 1024, 256), (1024, 128, 256)]),   # one tiled launch
    ("bf16", [(256, 256, 512), (200, 136, 96)]),                                        # ragged member: one by one
    ("fp32", [(96, 64, 80), (40, 72, 56), (64, 64, 64)]),
])
def test_gemm_group_weight_gradients(dtype, shapes):
    """hanayo_op_gemm_group on weight-gradient problems of different sizes: every C += A^T B and
    every column sum against numpy, the rows of C a neighbouring problem owns untouched."""
    rng = np.random.default_rng(len(shapes) * 1009 + shapes[0][0])
    probs, checks = [], []
    for (M, N, K) in shapes:
        A = rnd(rng, (K, M), dtype)
        B = rnd(rng, (K, N), dtype, 0.05)
        C0 = rng.normal(size=(M, N)).astype(np.float32)
        cs0 = rng.normal(size=N).astype(np.float32)
        t = dict(A=dev(A, dtype), B=dev(B, dtype), C=torch.from_numpy(C0).cuda(), M=M, N=N, K=K, lda=M, ldb=N, ldc=N,
                 colsum=torch.from_numpy(cs0).cuda(), colsum_scratch=torch.empty(64 * N, dtype=torch.float32, device="cuda"))
        probs.append(t)
        checks.append((C0 + A.astype(np.float64).T @ B.astype(np.float64), cs0 + B.astype(np.float64).sum(0)))
    hn.hanayo_op_gemm_group(DT[dtype], True, True, hn.EPI_ACCUM_F32, probs)
    torch.cuda.synchronize()
    for t, (want, want_cs) in zip(probs, checks):
        assert perr(t["C"].cpu().numpy(), want) <= TOL[dtype]
        assert perr(t["colsum"].cpu().numpy(), want_cs) <= 1e-4
    with pytest.raises(hn.HanayoError):
        hn.hanayo_op_gemm_group(DT[dtype], True, True, hn.EPI_ACCUM_F32, (probs * 3)[:5])   # more than 4


def run_gemm_case(dtype, layout, shape):
    M, N, K = shape
    if dtype == "fp32" and M * N * K > 4096 * 4096 * 64:
        M, N = M // 4, N // 4
    a_t, b_t = LAYOUTS[layout]
    rng = np.random.default_rng(hash((dtype, layout, shape)) % (2 ** 32))
    A = rnd(rng, (M, K), dtype)
    B = rnd(rng, (K, N), dtype, 0.05)
    bias = rnd(rng, (N,), dtype)
    aux = rnd(rng, (M, N), dtype)
    ref = A.astype(np.float64) @ B.astype(np.float64)
    Ad = dev(A.T.copy() if a_t else A, dtype)
    Bd = dev(B if b_t else B.T.copy(), dtype)
    for epi in EPIS[layout]:
        bd, xd = dev(bias, dtype), dev(aux, dtype)
        if epi == hn.EPI_ACCUM_F32:
            C0 = rng.normal(size=(M, N)).astype(np.float32)
            Cd = torch.from_numpy(C0).cuda()
            want = C0 + ref
        else:
            Cd = torch.empty((M, N), dtype=Ad.dtype, device="cuda")
            want = {hn.EPI_NONE: ref, hn.EPI_BIAS: ref + bias, hn.EPI_BIAS_GELU: OB.gelu(ref + bias),
                    hn.EPI_BIAS_RES: ref + bias + aux, hn.EPI_MUL_DGELU: ref * OB.gelu_grad(aux.astype(np.float64)),
                    hn.EPI_ADD: ref + aux}[epi]
        out2 = torch.empty((M, N), dtype=Ad.dtype, device="cuda") if epi == hn.EPI_BIAS_GELU else None
        cs = cs0 = scratch = None
        if epi == hn.EPI_ACCUM_F32 and N % 8 == 0:   # the bias gradient rides along: column sums of B
            cs0 = rng.normal(size=N).astype(np.float32)
            cs = torch.from_numpy(cs0).cuda()
            scratch = torch.empty(64 * N, dtype=torch.float32, device="cuda")
        hn.hanayo_op_gemm(DT[dtype], Ad, Bd, Cd, M, N, K, M if a_t else K, N if b_t else K, N, a_t, b_t, epi,
                          bd, xd, out2, cs, scratch)
        torch.cuda.synchronize()
        if cs is not None:
            want_cs = B.astype(np.float64).sum(0)
            assert perr(cs.cpu().numpy() - cs0, want_cs) <= 1e-4, "column sums"
        e = perr(host(Cd), want)
        assert e <= TOL[dtype], "epilogue %d: %.3g" % (epi, e)
        if out2 is not None:
            assert perr(host(out2), ref + bias) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("rows,H", [(64, 256), (300, 1024), (37, 2560), (130, 4096), (1030, 512), (5, 72),
                                    # wide rows: several trips of a workgroup's row loop with a ragged last one,
                                    # every width class above 2048, a width that is no multiple of 512, one row
                                    (2100, 4096), (1601, 2560), (700, 3072), (530, 3584), (41, 2600), (1, 4096)])
def test_layernorm_forward_backward(dtype, rows, H):
    rng = np.random.default_rng(rows * 7 + H)
    x = rnd(rng, (rows, H), dtype, 2.0) + (0.5 if dtype == "fp32" else 0.0)
    x = synth.bf16_round(x) if dtype == "bf16" else x
    g = rnd(rng, (H,), dtype) * 0.2 + 1.0
    g = synth.bf16_round(g) if dtype == "bf16" else g
    b = rnd(rng, (H,), dtype, 0.2)
    dout = rnd(rng, (rows, H), dtype)
    add = rnd(rng, (rows, H), dtype)
    x64, g64 = x.astype(np.float64), g.astype(np.float64)
    out_ref, cache = OB.ln_fwd(x64, g64, b.astype(np.float64), 1e-5)
    dz_ref, dg_ref, db_ref = OB.ln_bwd(dout.astype(np.float64), g64, cache)
    xd, gd, bd, dd, ad = (dev(t, dtype) for t in (x, g, b, dout, add))
    out = torch.empty_like(xd)
    cp = torch.empty_like(xd)
    stats = torch.empty((rows, 2), dtype=torch.float32, device="cuda")
    hn.hanayo_op_layernorm_forward(DT[dtype], xd, gd, bd, out, stats, cp, rows, H, 1e-5)
    torch.cuda.synchronize()
    assert perr(host(out), out_ref) <= TOL[dtype]
    assert torch.equal(cp, xd)
    st = stats.cpu().numpy().astype(np.float64)
    assert np.allclose(st[:, 0], x64.mean(-1), atol=1e-5)
    assert np.allclose(st[:, 1], cache[1][:, 0], rtol=1e-4)
    dz = torch.empty_like(xd)
    dg0, db0 = rng.normal(size=H).astype(np.float32), rng.normal(size=H).astype(np.float32)
    dgd, dbd = torch.from_numpy(dg0).cuda(), torch.from_numpy(db0).cuda()
    scratch = torch.empty(1024 * H, dtype=torch.float32, device="cuda")
    for addend, want in ((None, dz_ref), (ad, dz_ref + add)):
        hn.hanayo_op_layernorm_backward(DT[dtype], dd, xd, gd, stats, addend, dz, dgd, dbd, scratch, rows, H)
        torch.cuda.synchronize()
        assert perr(host(dz), want) <= TOL[dtype]
    # gamma / beta gradients were accumulated twice on top of their initial values
    assert perr(dgd.cpu().numpy() - dg0, 2 * dg_ref) <= 1e-4
    assert perr(dbd.cpu().numpy() - db0, 2 * db_ref) <= 1e-4


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("rows,N", [(256, 768), (1000, 3072), (33, 264), (4096, 1024)])
def test_colsum(dtype, rows, N):
    rng = np.random.default_rng(rows + N)
    a = rnd(rng, (rows, N), dtype)
    o0 = rng.normal(size=N).astype(np.float32)
    od = torch.from_numpy(o0).cuda()
    scratch = torch.empty(64 * N, dtype=torch.float32, device="cuda")
    hn.hanayo_op_colsum_add(DT[dtype], dev(a, dtype), rows, N, od, scratch)
    torch.cuda.synchronize()
    assert perr(od.cpu().numpy() - o0, a.astype(np.float64).sum(0)) <= 1e-5


ATTN_CASES = [
    # b, s, heads, d, causal, padded
    (2, 128, 4, 64, True, False),
    (3, 160, 2, 64, False, True),
    (1, 256, 2, 128, True, False),
    (2, 200, 3, 64, True, True),
    (2, 96, 2, 80, True, False),
    (2, 300, 3, 80, False, True),
    (1, 264, 2, 96, True, True),
    (2, 130, 2, 48, True, False),          # a head dim the register-staged kernels take
    (2, 77, 2, 64, False, False),
    (1, 512, 1, 64, True, False),
    (2, 320, 2, 128, False, True),
]


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("case", ATTN_CASES)
def test_attention_forward_backward(dtype, case):
    b, s, h, d, causal, padded = case
    H = h * d
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    qkv = rnd(rng, (b, s, 3 * H), dtype)
    dctx = rnd(rng, (b, s, H), dtype)
    vl = rng.integers(s // 3, s + 1, size=b).astype(np.int32) if padded else None
    # the oracle's attention with identity projections: Wqkv = I-like split, Wo = I
    cfg = OB.BlockCfg(H, h, 4 * H, causal=causal)
    p = {"wqkv": np.eye(3 * H)[: 3 * H], "bqkv": np.zeros(3 * H), "wo": np.eye(H), "bo": np.zeros(H)}
    q64 = qkv.astype(np.float64)
    split = lambda t: t.reshape(b, s, h, d).transpose(0, 2, 1, 3)
    q, k, v = (split(q64[..., i * H:(i + 1) * H]) for i in range(3))
    ok = OB._allowed(s, causal, vl, b)
    sc = np.where(ok, q @ k.transpose(0, 1, 3, 2) / math.sqrt(d), -np.inf)
    mx = sc.max(-1, keepdims=True)
    e = np.where(ok, np.exp(sc - mx), 0.0)
    prob = e / e.sum(-1, keepdims=True)
    ctx_ref = (prob @ v).transpose(0, 2, 1, 3).reshape(b, s, H)
    lse_ref = (mx + np.log(e.sum(-1, keepdims=True)))[..., 0]
    dc = split(dctx.astype(np.float64))
    dv = prob.transpose(0, 1, 3, 2) @ dc
    dp = dc @ v.transpose(0, 1, 3, 2)
    ds = prob * (dp - (dp * prob).sum(-1, keepdims=True))
    dq = ds @ k / math.sqrt(d)
    dk = ds.transpose(0, 1, 3, 2) @ q / math.sqrt(d)
    dqkv_ref = np.concatenate([t.transpose(0, 2, 1, 3).reshape(b, s, H) for t in (dq, dk, dv)], -1)

    qd, dd = dev(qkv, dtype), dev(dctx, dtype)
    vld = None if vl is None else torch.from_numpy(vl).cuda()
    ctx = torch.empty((b, s, H), dtype=qd.dtype, device="cuda")
    lse = torch.empty((b, h, s), dtype=torch.float32, device="cuda")
    hn.hanayo_op_attention_forward(DT[dtype], qd, vld, ctx, lse, b, s, h, d, causal)
    torch.cuda.synchronize()
    assert perr(host(ctx), ctx_ref) <= TOL[dtype]
    assert np.abs(lse.cpu().numpy() - lse_ref).max() <= (2e-2 if dtype == "bf16" else 1e-4)
    dqkv = torch.full((b, s, 3 * H), float("nan"), dtype=qd.dtype, device="cuda")
    delta = torch.empty((b, h, s), dtype=torch.float32, device="cuda")
    hn.hanayo_op_attention_backward(DT[dtype], qd, vld, ctx, lse, dd, dqkv, delta, b, s, h, d, causal)
    torch.cuda.synchronize()
    got = host(dqkv)
    assert np.isfinite(got).all()
    for i, name in enumerate("qkv"):
        e = perr(got[..., i * H:(i + 1) * H], dqkv_ref[..., i * H:(i + 1) * H])
        assert e <= TOL[dtype], "d%s: %.3g" % (name, e)


@pytest.mark.parametrize("nbytes", [0, 16, 4096 + 16, (3 << 20) + 48, 70 << 20])
def test_copy_kernel(nbytes):
    """The plain copy kernel: byte-exact, nothing written past the end."""
    src = torch.randint(0, 256, (nbytes + 64,), dtype=torch.uint8, device="cuda")
    dst = torch.full((nbytes + 64,), 7, dtype=torch.uint8, device="cuda")
    hn.hanayo_op_copy(dst, src, nbytes)
    torch.cuda.synchronize()
    assert torch.equal(dst[:nbytes], src[:nbytes])
    assert bool((dst[nbytes:] == 7).all())
    if nbytes:
        with pytest.raises(hn.HanayoError):
            hn.hanayo_op_copy(dst, src, nbytes - 8)
