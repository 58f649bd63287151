"""GPU parity of the single operators against the numpy oracle (through the C ABI)."""
import math

import numpy as np
import pytest

from oracle import block_oracle as bo
from paper_2107_06925_amd import binding as b
from paper_2107_06925_amd import synth
from gpu_util import TOL, assert_close, to_dev, to_np

pytestmark = pytest.mark.gpu
DTYPES = [b.F32, b.BF16]
IMPLS = [0, 1]


def _rand(shape, seed, dtype, scale=1.0):
    a = np.random.default_rng(seed).standard_normal(shape).astype(np.float32) * scale
    return synth.round_to_bf16(a) if dtype == b.BF16 else a


GEMM_SHAPES = [(128, 384, 128), (200, 136, 72), (512, 512, 256), (304, 1600, 320), (1024, 264, 1032), (8, 8, 8),
               (512, 520, 2048)]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("impl", IMPLS)
@pytest.mark.parametrize("m,n,k", GEMM_SHAPES)
@pytest.mark.parametrize("layout", ["fwd", "dgrad", "wgrad"])
def test_gemm_layouts(dtype, impl, m, n, k, layout):
    import torch
    print("gemm", dtype, impl, m, n, k, layout, flush=True)
    a_kc, b_kc = {"fwd": (1, 0), "dgrad": (1, 1), "wgrad": (0, 0)}[layout]
    A = _rand((m, k), 1, dtype)
    B = _rand((k, n), 2, dtype)
    a_store = A if a_kc else np.ascontiguousarray(A.T)
    b_store = np.ascontiguousarray(B.T) if b_kc else B
    want = A.astype(np.float64) @ B.astype(np.float64)
    da, db = to_dev(a_store, dtype), to_dev(b_store, dtype)
    if layout == "wgrad":
        c0 = np.random.default_rng(3).standard_normal((m, n)).astype(np.float32)
        dc = torch.from_numpy(c0.copy()).cuda()
        b.chimera_op_gemm(da, db, dc, m, n, k, a_kc, b_kc, b.EPI_ACCUM_F32, impl=impl)
        b.chimera_op_gemm(da, db, dc, m, n, k, a_kc, b_kc, b.EPI_ACCUM_F32, impl=impl)
        torch.cuda.synchronize()
        assert_close(to_np(dc) - c0, 2 * want, dtype, "accumulated twice")
    else:
        dc = torch.empty((m, n), dtype=da.dtype, device="cuda")
        b.chimera_op_gemm(da, db, dc, m, n, k, a_kc, b_kc, b.EPI_NONE, impl=impl)
        torch.cuda.synchronize()
        assert_close(to_np(dc), want, dtype)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("impl", IMPLS)
@pytest.mark.parametrize("gelu_erf", [False, True])
def test_gemm_epilogues(dtype, impl, gelu_erf):
    import torch
    m, n, k = 264, 520, 136
    kind = "erf" if gelu_erf else "tanh"
    A, B = _rand((m, k), 1, dtype), _rand((k, n), 2, dtype, 0.2)
    bias, R = _rand((n,), 3, dtype), _rand((m, n), 4, dtype)
    acc = A.astype(np.float64) @ B.astype(np.float64)
    da, db, dbias, dr = to_dev(A, dtype), to_dev(B, dtype), to_dev(bias, dtype), to_dev(R, dtype)
    c = torch.empty((m, n), dtype=da.dtype, device="cuda")
    c2 = torch.empty_like(c)
    b.chimera_op_gemm(da, db, c, m, n, k, 1, 0, b.EPI_BIAS, bias=dbias, impl=impl)
    assert_close(to_np(c), acc + bias, dtype, "bias")
    b.chimera_op_gemm(da, db, c, m, n, k, 1, 0, b.EPI_BIAS_GELU, bias=dbias, c2=c2, impl=impl, gelu_erf=gelu_erf)
    assert_close(to_np(c), acc + bias, dtype, "bias+gelu: u")
    assert_close(to_np(c2), bo.gelu_fwd(acc + bias, kind), dtype, "bias+gelu: g")
    b.chimera_op_gemm(da, db, c, m, n, k, 1, 0, b.EPI_BIAS_RESIDUAL, bias=dbias, r=dr, impl=impl)
    assert_close(to_np(c), acc + bias + R, dtype, "bias+residual")
    b.chimera_op_gemm(da, db, c, m, n, k, 1, 0, b.EPI_DGELU, r=dr, impl=impl, gelu_erf=gelu_erf)
    assert_close(to_np(c), acc * bo.gelu_grad(R.astype(np.float64), kind), dtype, "dgelu")


def test_gemm_last_row_bands_on_small_tiles():
    """272 tiles of 256x256 are one round of the 256 CUs plus 16 tiles: the last band of 256 rows
    (here 200 of them exist) goes out as a second launch of 128x128 tiles.  Every epilogue has
    to find its row-offset operands (residual, second output, float output) in that launch."""
    import torch
    m, n, k = 16 * 256 + 200, 4096, 64
    A, B = _rand((m, k), 1, b.BF16), _rand((k, n), 2, b.BF16, 0.2)
    bias, R = _rand((n,), 3, b.BF16), _rand((m, n), 4, b.BF16)
    acc = A.astype(np.float64) @ B.astype(np.float64)
    da, db, dbias, dr = to_dev(A, b.BF16), to_dev(B, b.BF16), to_dev(bias, b.BF16), to_dev(R, b.BF16)
    c = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    c2 = torch.empty_like(c)
    b.chimera_op_gemm(da, db, c, m, n, k, 1, 0, b.EPI_BIAS_GELU, bias=dbias, c2=c2)
    assert_close(to_np(c), acc + bias, b.BF16, "bias+gelu: u")
    assert_close(to_np(c2), bo.gelu_fwd(acc + bias, "tanh"), b.BF16, "bias+gelu: g")
    b.chimera_op_gemm(da, db, c, m, n, k, 1, 0, b.EPI_BIAS_RESIDUAL, bias=dbias, r=dr)
    assert_close(to_np(c), acc + bias + R, b.BF16, "bias+residual")
    b.chimera_op_gemm(da, db, c, m, n, k, 1, 0, b.EPI_DGELU, r=dr)
    assert_close(to_np(c), acc * bo.gelu_grad(R.astype(np.float64), "tanh"), b.BF16, "dgelu")
    # dgrad layout (both operands k-contiguous) and the float-accumulating weight-gradient layout
    dbt = to_dev(np.ascontiguousarray(B.T), b.BF16)
    b.chimera_op_gemm(da, dbt, c, m, n, k, 1, 1, b.EPI_NONE)
    assert_close(to_np(c), acc, b.BF16, "k-contiguous B")
    dat = to_dev(np.ascontiguousarray(A.T), b.BF16)
    dw = torch.ones((m, n), device="cuda")
    b.chimera_op_gemm(dat, db, dw, m, n, k, 0, 0, b.EPI_ACCUM_F32)
    assert_close(to_np(dw) - 1.0, acc, b.BF16, "index-contiguous A, float accumulate")


def test_gemm_split_k_matches_unsplit_and_is_reproducible():
    """On request (tile override plus a workspace) the bf16 kernel splits k over several
    workgroups per tile; partial sums are added in a fixed order, so two runs agree bit
    for bit, and the result matches the oracle like the unsplit one."""
    import torch
    m, n, k = 1024, 1024, 4096
    assert b.lib().chimera_op_gemm_workspace_bytes(m, n, k) > 0
    b.check(b.lib().chimera_op_gemm_tuning(256, 256, 4, 0))
    try:
        _split_k_body(m, n, k)
    finally:
        b.check(b.lib().chimera_op_gemm_tuning(0, 0, 0, 0))


def _split_k_body(m, n, k):
    import torch
    A, B = _rand((m, k), 1, b.BF16), _rand((k, n), 2, b.BF16)
    want = A.astype(np.float64) @ B.astype(np.float64)
    da, db = to_dev(A, b.BF16), to_dev(B, b.BF16)
    outs = []
    for ws in ("auto", "auto", None):
        c = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
        b.chimera_op_gemm(da, db, c, m, n, k, 1, 0, workspace=ws)
        torch.cuda.synchronize()
        assert_close(to_np(c), want, b.BF16)
        outs.append(c)
    assert torch.equal(outs[0], outs[1])
    # accumulate epilogue through the split path, twice
    dw = torch.zeros((m, n), device="cuda")
    at = to_dev(np.ascontiguousarray(A.T), b.BF16)
    for _ in range(2):
        b.chimera_op_gemm(at, db, dw, m, n, k, 0, 0, b.EPI_ACCUM_F32)
    assert_close(to_np(dw), 2 * want, b.BF16)


GROUPS = [
    # (k, [(m, n), ...]): one block's weight gradients in miniature; ragged tiles; a single product
    (256, [(128, 512), (512, 128), (128, 128), (128, 384)]),
    (192, [(200, 136), (8, 8), (264, 520)]),
    (64, [(136, 72)]),
    (1024, [(256, 1024), (1024, 256), (256, 256), (256, 768)]),     # 48 tiles: the k-sliced 8-wavefront variant
    (128, [(1024, 4096), (4096, 1024), (1024, 1024), (1024, 3072)]),   # 768 tiles: the two-workgroups-per-CU variant
    (64, [(2048, 4096), (4096, 2056), (2048, 2048)]),                  # enough 256x256 tiles for the whole chip, ragged edge
    (64, [(1024, 3080), (1024, 1032), (1032, 4096), (2056, 1024)]),    # 188 tiles of 256x256: fewer than CUs, not a multiple of 8
    (64, [(2048, 2048), (2048, 2048), (2048, 2048), (2248, 2048)]),    # 264 tiles: the last 200 rows of one product go to a 128x128 launch
]


@pytest.mark.parametrize("with_bsum", [False, True])
@pytest.mark.parametrize("k,shapes", GROUPS)
def test_gemm_group_accumulate(k, shapes, with_bsum):
    """One launch for several dW += X^T dY equals the per-product oracle, twice in a row."""
    import torch
    print("gemm group", k, shapes, flush=True)
    probs, want, c0s, bs, bs0, want_b = [], [], [], [], [], []
    for i, (m, n) in enumerate(shapes):
        X = _rand((k, m), 10 + i, b.BF16)
        dY = _rand((k, n), 20 + i, b.BF16)
        c0 = np.random.default_rng(30 + i).standard_normal((m, n)).astype(np.float32)
        probs.append((to_dev(X, b.BF16), to_dev(dY, b.BF16), torch.from_numpy(c0.copy()).cuda()))
        want.append(X.astype(np.float64).T @ dY.astype(np.float64))
        c0s.append(c0)
        # bias gradient of the same layer (column sums of dY); the odd products go without
        b0 = np.random.default_rng(60 + i).standard_normal(n).astype(np.float32)
        bs0.append(b0)
        bs.append(torch.from_numpy(b0.copy()).cuda() if with_bsum and i % 2 == 0 else None)
        want_b.append(dY.astype(np.float64).sum(axis=0))
    b.chimera_op_gemm_group_accumulate(probs, k, bs if with_bsum else None)
    b.chimera_op_gemm_group_accumulate(probs, k, bs if with_bsum else None)
    torch.cuda.synchronize()
    for i, (_, _, c) in enumerate(probs):
        assert_close(to_np(c) - c0s[i], 2 * want[i], b.BF16, "product %d" % i)
        if bs[i] is not None:
            assert_close(to_np(bs[i]) - bs0[i], 2 * want_b[i], b.BF16, "column sums %d" % i)


def test_gemm_group_overwrite():
    """overwrite: C and the column sums receive the results whatever they held (NaN here)."""
    import torch
    k, shapes = 192, [(136, 264), (128, 128), (264, 136)]
    probs, bs, want, want_b = [], [], [], []
    for i, (m, n) in enumerate(shapes):
        X, dY = _rand((k, m), 70 + i, b.BF16), _rand((k, n), 80 + i, b.BF16)
        probs.append((to_dev(X, b.BF16), to_dev(dY, b.BF16), torch.full((m, n), float("nan"), device="cuda")))
        bs.append(torch.full((n,), float("nan"), device="cuda"))
        want.append(X.astype(np.float64).T @ dY.astype(np.float64))
        want_b.append(dY.astype(np.float64).sum(axis=0))
    b.chimera_op_gemm_group_accumulate(probs, k, bs, overwrite=True)
    b.chimera_op_gemm_group_accumulate(probs, k, bs)              # and a second micro-batch accumulates
    torch.cuda.synchronize()
    for i, (_, _, c) in enumerate(probs):
        assert_close(to_np(c), 2 * want[i], b.BF16, "product %d" % i)
        assert_close(to_np(bs[i]), 2 * want_b[i], b.BF16, "column sums %d" % i)
    # a single product with the float-accumulate epilogue never overwrites, whatever the GeLU flag says
    X, dY, c = probs[1][0], probs[1][1], torch.ones((128, 128), device="cuda")
    b.chimera_op_gemm(X, dY, c, 128, 128, k, 0, 0, b.EPI_ACCUM_F32, gelu_erf=True)
    torch.cuda.synchronize()
    assert_close(to_np(c) - 1.0, want[1], b.BF16, "accumulate with gelu flag set")


def test_gemm_group_matches_single_launches_bitwise():
    import torch
    k, shapes = 320, [(136, 264), (264, 136), (128, 128)]
    probs, singles = [], []
    for i, (m, n) in enumerate(shapes):
        X = to_dev(_rand((k, m), 40 + i, b.BF16), b.BF16)
        dY = to_dev(_rand((k, n), 50 + i, b.BF16), b.BF16)
        probs.append((X, dY, torch.zeros((m, n), device="cuda")))
        singles.append(torch.zeros((m, n), device="cuda"))
        b.chimera_op_gemm(X, dY, singles[-1], m, n, k, 0, 0, b.EPI_ACCUM_F32)
    b.chimera_op_gemm_group_accumulate(probs, k)
    torch.cuda.synchronize()
    for (_, _, c), s1 in zip(probs, singles):
        assert torch.equal(c, s1)


def test_gemm_group_argument_errors():
    import torch
    X = torch.zeros((64, 16), device="cuda", dtype=torch.bfloat16)
    c = torch.zeros((16, 16), device="cuda")
    with pytest.raises(b.ChimeraError):
        b.chimera_op_gemm_group_accumulate([(X, X, c)] * 5, 64)            # more than four products
    with pytest.raises(b.ChimeraError):
        b.chimera_op_gemm_group_accumulate([(X[:40], X[:40], c)], 40)      # k not a multiple of 64
    Y = torch.zeros((64, 4), device="cuda", dtype=torch.bfloat16)
    with pytest.raises(b.ChimeraError):
        b.chimera_op_gemm_group_accumulate([(X, Y, torch.zeros((16, 4), device="cuda"))], 64)   # n < 8
    with pytest.raises(b.ChimeraError):
        b.chimera_op_gemm_group_accumulate([], 64)


def test_gemm_argument_errors():
    import torch
    a = torch.zeros((16, 16), device="cuda")
    with pytest.raises(b.ChimeraError):
        b.chimera_op_gemm(a, a, a, 16, 12, 16, 1, 0)           # n not a multiple of 8
    with pytest.raises(b.ChimeraError):
        b.chimera_op_gemm(a, a, a, 16, 16, 16, 1, 0, b.EPI_BIAS)  # bias missing
    with pytest.raises(b.ChimeraError):
        b.chimera_op_gemm(a, a, a, 0, 16, 16, 1, 0)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("rows,cols", [(128, 128), (37, 1600), (515, 1024), (64, 2048), (5, 8), (21, 4096), (300, 3072)])
def test_layernorm(dtype, rows, cols):
    if dtype == b.F32 and cols > 2048:
        with pytest.raises(b.ChimeraError):        # float rows are limited to 2048 columns (8 chunks per lane)
            import torch
            z = torch.zeros((rows, cols), device="cuda")
            b.chimera_op_layernorm_fwd(z, z[0], z[0], z.clone(), z[:, 0].clone(), z[:, 0].clone())
        return
    import torch
    print("layernorm", dtype, rows, cols, flush=True)
    x = _rand((rows, cols), 1, dtype, 2.0) + (0.5 if dtype == b.F32 else 0.0)
    x = synth.round_to_bf16(x) if dtype == b.BF16 else x
    g, be = _rand((cols,), 2, dtype), _rand((cols,), 3, dtype)
    dy, res = _rand((rows, cols), 4, dtype), _rand((rows, cols), 5, dtype)
    y64, cache = bo.layernorm_fwd(x.astype(np.float64), g.astype(np.float64), be.astype(np.float64))
    dx64, dg64, db64 = bo.layernorm_bwd(dy.astype(np.float64), cache, g.astype(np.float64))
    dxd = to_dev(x, dtype)
    y = torch.empty_like(dxd)
    mean = torch.empty(rows, device="cuda")
    rstd = torch.empty(rows, device="cuda")
    b.chimera_op_layernorm_fwd(dxd, to_dev(g, dtype), to_dev(be, dtype), y, mean, rstd)
    assert_close(to_np(y), y64, dtype, "y")
    assert_close(to_np(mean), x.astype(np.float64).mean(-1), b.F32, "mean")
    assert_close(to_np(rstd), cache[1][:, 0], b.F32, "rstd")
    dx = torch.empty_like(dxd)
    dgam = torch.full((cols,), 1.0, device="cuda")
    dbet = torch.full((cols,), -2.0, device="cuda")
    b.chimera_op_layernorm_bwd(to_dev(dy, dtype), dxd, mean, rstd, to_dev(g, dtype), to_dev(res, dtype), dx, dgam, dbet)
    assert_close(to_np(dx), res + dx64, dtype, "dx")
    assert_close(to_np(dgam) - 1.0, dg64, dtype, "dgamma")
    assert_close(to_np(dbet) + 2.0, db64, dtype, "dbeta")


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("rows,cols", [(128, 384), (1000, 1600), (70, 8), (4096, 4096)])
def test_colsum(dtype, rows, cols):
    import torch
    x = _rand((rows, cols), 1, dtype)
    out = torch.full((cols,), 3.0, device="cuda")
    b.chimera_op_colsum(to_dev(x, dtype), out)
    assert_close(to_np(out) - 3.0, x.astype(np.float64).sum(0), b.F32, "colsum", scale=10.0)


ATTN_SHAPES = [(2, 64, 4, 32), (1, 100, 2, 64), (2, 256, 3, 64), (1, 192, 2, 128), (3, 1, 2, 64), (1, 77, 1, 16),
               (8, 200, 32, 64), (2, 333, 2, 128)]        # many (sequence, head) pairs; a ragged last tile at head dim 128


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("impl", IMPLS)
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("batch,seq,heads,d", ATTN_SHAPES)
def test_attention(dtype, impl, causal, batch, seq, heads, d):
    import torch
    print("attention", dtype, impl, causal, batch, seq, heads, d, flush=True)
    H = heads * d
    qkv = _rand((batch * seq, 3 * H), 1, dtype, 1.5)       # peaked softmax: scores ~ N(0, 2.25 d)/sqrt(d)
    dctx = _rand((batch * seq, H), 2, dtype)
    ctx64, probs = bo.attention_fwd(qkv.astype(np.float64), batch, seq, heads, causal)
    dqkv64 = bo.attention_bwd(dctx.astype(np.float64), qkv.astype(np.float64), probs, batch, seq, heads)
    dq = to_dev(qkv, dtype)
    ctx = torch.empty((batch * seq, H), dtype=dq.dtype, device="cuda")
    lse = torch.empty((batch, heads, seq), device="cuda")
    b.chimera_op_attention_fwd(dq, ctx, lse, batch, seq, heads, d, causal, impl=impl)
    assert_close(to_np(ctx), ctx64, dtype, "ctx")
    # lse: log-sum-exp of the scaled, masked scores
    q = qkv.astype(np.float64)
    bb, hh = batch - 1, heads - 1
    s = q[bb * seq:(bb + 1) * seq, hh * d:(hh + 1) * d] @ q[bb * seq:(bb + 1) * seq, H + hh * d:H + (hh + 1) * d].T / math.sqrt(d)
    if causal:
        s = np.where(np.tril(np.ones((seq, seq), dtype=bool)), s, -np.inf)
    want_lse = np.log(np.exp(s - s.max(-1, keepdims=True)).sum(-1)) + s.max(-1)
    assert np.max(np.abs(to_np(lse)[bb, hh] - want_lse)) < (1e-4 if dtype == b.F32 else 2e-2)
    dqkv = torch.empty_like(dq)
    delta = torch.empty((batch, heads, seq), device="cuda")
    # the backward reads the forward's own ctx and lse, as the stage does
    b.chimera_op_attention_bwd(dq, ctx, lse, to_dev(dctx, dtype), dqkv, delta, batch, seq, heads, d, causal, impl=impl)
    got = to_np(dqkv)
    for name, lo in (("dq", 0), ("dk", H), ("dv", 2 * H)):
        assert_close(got[:, lo:lo + H], dqkv64[:, lo:lo + H], dtype, name)


def test_measured_ceiling_probes():
    import torch
    sink = torch.zeros(1, device="cuda")
    tf = b.chimera_probe_mfma_bf16(sink, 500)
    assert 200.0 < tf < 2600.0, tf              # below the published dense bf16 peak, far above vector rates
    assert float(sink.item()) == 0.0
    src = torch.arange(1 << 22, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    gbs = b.chimera_probe_copy(src, dst)
    assert torch.equal(src, dst)
    assert 100.0 < gbs < 8200.0, gbs
    with pytest.raises(b.ChimeraError):
        b.chimera_probe_copy(src[1:], dst[1:])    # 4-byte offset: not 16-byte aligned
