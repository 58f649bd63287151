"""The allocation-free LayerNorm backward (partial sums in the library's static device array)
against the ordinary entry point, which takes the same scratch from the caller: same kernels,
so the results must agree bit for bit - on two calls in a row, the second on a smaller input
(the array then still holds the first call's partial sums beyond what the second overwrites)."""
import numpy as np
import pytest

from paper_2107_06925_amd import binding as b

pytestmark = pytest.mark.gpu


def _case(rows, cols, dtype, seed):
    import torch
    tdt = torch.float32 if dtype == b.F32 else torch.bfloat16
    gen = torch.Generator(device="cuda").manual_seed(seed)
    rnd = lambda *shape: torch.randn(shape, device="cuda", generator=gen)
    x, dy, res = rnd(rows, cols).to(tdt), rnd(rows, cols).to(tdt), rnd(rows, cols).to(tdt)
    gamma = (1.0 + 0.02 * rnd(cols)).to(tdt)
    mean = x.float().mean(dim=1).contiguous()
    rstd = (1.0 / torch.sqrt(x.float().var(dim=1, unbiased=False) + 1e-5)).contiguous()
    out = []
    for f in (b.chimera_op_layernorm_bwd, b.chimera_op_layernorm_bwd_noalloc):
        dx = torch.full((rows, cols), float("nan"), device="cuda", dtype=tdt)
        dg, db = torch.full((cols,), 0.5, device="cuda"), torch.full((cols,), -0.25, device="cuda")   # accumulated into
        f(dy, x, mean, rstd, gamma, res, dx, dg, db)
        torch.cuda.synchronize()
        out.append((dx, dg, db))
    for want, got, what in zip(out[0], out[1], ("dx", "dgamma", "dbeta")):
        assert torch.isfinite(got.float()).all(), what
        assert torch.equal(want, got), "%s differs for %d x %d" % (what, rows, cols)
    # and the ordinary entry point is itself checked against the oracle in test_gpu_ops.py


@pytest.mark.parametrize("dtype", [b.BF16, b.F32], ids=["bf16", "f32"])
def test_no_alloc_layernorm_backward_twice_in_a_row(dtype):
    _case(4096, 1600, dtype, 1)       # wide rows, 1.6 M scratch floats
    _case(333, 1024, dtype, 2)        # smaller, ragged, narrow-row kernel
    _case(2048, 2048, dtype, 3)


def test_no_alloc_rejects_sizes_beyond_the_static_scratch():
    import torch
    lim = b.lib().chimera_op_layernorm_bwd_noalloc_max_scratch_floats()
    rows, cols = 8192, 2048
    assert b.lib().chimera_op_layernorm_bwd_scratch_floats(rows, cols) > lim
    z = torch.zeros((8, 8), device="cuda")           # never touched: the size check comes first
    with pytest.raises(b.ChimeraError) as e:
        b.check(b.lib().chimera_op_layernorm_bwd_noalloc(b.F32, rows, cols, *[z.data_ptr()] * 9, None))
    assert e.value.code == b.ENOMEM
