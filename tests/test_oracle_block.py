"""Pins of the numeric oracle (CPU only): finite differences, the
micro-batch-sum identity, closed-form special cases, invariants and an
independent autograd library.  Each would fail on a dropped term, a wrong
sign or index, or a transposed operand somewhere in oracle/block_oracle.py."""
import math

import numpy as np
import pytest
import torch

from oracle import block_oracle as bo
from paper_2107_06925_amd import synth

H, HEADS, S, BATCH = 16, 2, 5, 2


def _params(hidden=H, layers=1, seed=1, qk_gain=20.0):
    ps = synth.make_stage_params(hidden, layers, 0, seed=seed, qk_gain=qk_gain)
    # larger weights than the 0.02 recipe so that every term matters
    out = []
    for p in ps:
        q = {}
        for k, v in p.items():
            v = v.astype(np.float64)
            if k.startswith("w_") and k != "w_qkv":
                v = v * 10.0
            if k == "w_qkv":
                v = v.copy()
                v[:, 2 * hidden:] *= 10.0
            if k.startswith("b_") or k.endswith("_b"):
                v = v * 10.0
            q[k] = v
        out.append(q)
    return out


def _io(tokens, hidden, seed=0):
    x, dy = synth.make_microbatch(tokens, hidden, seed)
    return x.astype(np.float64), dy.astype(np.float64)


def _loss(x, params, G, causal, gelu):
    y, _ = bo.stage_fwd(x, params, BATCH, S, HEADS, causal, gelu)
    return float((y * G).sum())


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("gelu", ["tanh", "erf"])
def test_finite_differences(causal, gelu):
    """Central differences of l = sum(Y * G) for dX and for every parameter tensor."""
    params = _params(layers=2)
    x, G = _io(BATCH * S, H)
    y, caches = bo.stage_fwd(x, params, BATCH, S, HEADS, causal, gelu)
    dx, grads = bo.stage_bwd(G, caches, params)
    rng = np.random.default_rng(5)
    h = 1e-5

    def probe(arr, analytic, n):
        flat = arr.reshape(-1)
        for idx in rng.choice(flat.size, size=min(n, flat.size), replace=False):
            old = flat[idx]
            flat[idx] = old + h
            lp = _loss(x, params, G, causal, gelu)
            flat[idx] = old - h
            lm = _loss(x, params, G, causal, gelu)
            flat[idx] = old
            fd = (lp - lm) / (2 * h)
            an = analytic.reshape(-1)[idx]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (idx, fd, an)

    probe(x, dx, 12)
    for layer in range(2):
        for name in bo.PARAM_ORDER:
            probe(params[layer][name], grads[layer][name], 6)


def test_microbatch_sum_equals_full_batch():
    """Synchronous schedule = plain mini-batch gradient: sum over micro-batches of
    dtheta equals dtheta of the concatenated batch (no op mixes samples)."""
    params = _params(layers=2)
    xs, dys = zip(*[_io(BATCH * S, H, seed=g) for g in range(3)])
    total = None
    ys, dxs = [], []
    for x, dy in zip(xs, dys):
        y, dx, g = bo.stage_pass(x, dy, params, BATCH, S, HEADS)
        ys.append(y), dxs.append(dx)
        total = bo.add_grads(total, g)
    Y, DX, G = bo.stage_pass(np.concatenate(xs), np.concatenate(dys), params, 3 * BATCH, S, HEADS)
    np.testing.assert_allclose(np.concatenate(ys), Y, rtol=0, atol=1e-12)
    np.testing.assert_allclose(np.concatenate(dxs), DX, rtol=0, atol=1e-12)
    np.testing.assert_allclose(bo.flatten_grads(total), bo.flatten_grads(G), rtol=1e-11, atol=1e-11)


def test_worker_iteration_partition():
    """Worker sums: down stage gets the first half of each unit, up stage the second."""
    D, N = 2, 4
    pd, pu = _params(seed=3), _params(seed=4)
    xs, dys = zip(*[_io(BATCH * S, H, seed=g) for g in range(N)])
    ys, dxs, gd, gu = bo.worker_iteration(0, D, N, pd, pu, xs, dys, BATCH, S, HEADS)
    want_d = want_u = None
    for g in range(N):
        p = pd if g % 2 == 0 else pu
        y, dx, gr = bo.stage_pass(xs[g], dys[g], p, BATCH, S, HEADS)
        np.testing.assert_array_equal(ys[g], y)
        if g % 2 == 0:
            want_d = bo.add_grads(want_d, gr)
        else:
            want_u = bo.add_grads(want_u, gr)
    np.testing.assert_array_equal(bo.flatten_grads(gd), bo.flatten_grads(want_d))
    np.testing.assert_array_equal(bo.flatten_grads(gu), bo.flatten_grads(want_u))


def _torch_block(x, p, causal, gelu):
    F = torch.nn.functional
    Hh = x.shape[-1]
    d = Hh // HEADS
    h1 = F.layer_norm(x, (Hh,), p["ln1_g"], p["ln1_b"], eps=1e-5)
    qkv = torch.addmm(p["b_qkv"], h1, p["w_qkv"])
    q, k, v = [t.reshape(BATCH, S, HEADS, d).transpose(1, 2) for t in qkv.split(Hh, dim=-1)]
    ctx = F.scaled_dot_product_attention(q, k, v, is_causal=causal)
    ctx = ctx.transpose(1, 2).reshape(BATCH * S, Hh)
    x1 = x + torch.addmm(p["b_o"], ctx, p["w_o"])
    h2 = F.layer_norm(x1, (Hh,), p["ln2_g"], p["ln2_b"], eps=1e-5)
    u = torch.addmm(p["b_fc1"], h2, p["w_fc1"])
    g = F.gelu(u, approximate="tanh" if gelu == "tanh" else "none")
    return x1 + torch.addmm(p["b_fc2"], g, p["w_fc2"])


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("gelu", ["tanh", "erf"])
def test_against_library_autograd(causal, gelu):
    """The block reduces to library routines (layer_norm, SDPA, gelu, addmm) + autograd."""
    params = _params(layers=2, seed=7)
    x, G = _io(BATCH * S, H, seed=9)
    y, dx, grads = bo.stage_pass(x, G, params, BATCH, S, HEADS, causal, gelu)
    tp = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()} for p in params]
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    t = tx
    for p in tp:
        t = _torch_block(t, p, causal, gelu)
    (t * torch.tensor(G)).sum().backward()
    np.testing.assert_allclose(y, t.detach().numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-9, atol=1e-10)
    for layer in range(2):
        for name in bo.PARAM_ORDER:
            np.testing.assert_allclose(grads[layer][name], tp[layer][name].grad.numpy(),
                                       rtol=1e-9, atol=1e-10, err_msg=name)


def test_seq_one_attention_is_value():
    """S = 1: softmax of one score is 1, so ctx = V whatever Q, K and the mask are."""
    qkv = np.random.default_rng(0).standard_normal((3, 3 * H))
    for causal in (True, False):
        ctx, probs = bo.attention_fwd(qkv, 3, 1, HEADS, causal)
        np.testing.assert_array_equal(ctx, qkv[:, 2 * H:])
        assert np.all(probs == 1.0)


def test_zero_projections_give_identity():
    """Wo = W2 = 0 and bo = b2 = 0: the block is the identity and dX = dY."""
    p = _params()[0]
    for k in ("w_o", "b_o", "w_fc2", "b_fc2"):
        p[k] = np.zeros_like(p[k])
    x, dy = _io(BATCH * S, H)
    y, dx, gr = bo.stage_pass(x, dy, [p], BATCH, S, HEADS)
    np.testing.assert_array_equal(y, x)
    np.testing.assert_array_equal(dx, dy)
    np.testing.assert_allclose(gr[0]["b_fc2"], dy.sum(0), atol=1e-12)


def test_layernorm_closed_forms():
    x = np.random.default_rng(1).standard_normal((7, H)) * 3 + 2
    g = np.random.default_rng(2).standard_normal(H)
    b = np.random.default_rng(3).standard_normal(H)
    y, (xhat, rstd) = bo.layernorm_fwd(x, np.zeros(H), b)
    np.testing.assert_array_equal(y, np.broadcast_to(b, y.shape))       # gamma = 0
    y, (xhat, rstd) = bo.layernorm_fwd(x, np.ones(H), np.zeros(H))
    np.testing.assert_allclose(y.mean(-1), 0, atol=1e-12)
    np.testing.assert_allclose((y ** 2).mean(-1), 1 - 1e-5 * rstd[:, 0] ** 2, rtol=1e-12)
    np.testing.assert_allclose(rstd[:, 0], 1 / np.sqrt(x.var(-1) + 1e-5), rtol=1e-12)
    # backward is orthogonal to 1 and (nearly) to xhat when gamma = 1
    dy = np.random.default_rng(4).standard_normal(x.shape)
    dx, dg, db = bo.layernorm_bwd(dy, (xhat, rstd), np.ones(H))
    np.testing.assert_allclose(dx.sum(-1), 0, atol=1e-12)
    # ... up to the eps term: sum(dx*xhat) = eps * rstd^3 * sum(dy*xhat)
    np.testing.assert_allclose((dx * xhat).sum(-1), 1e-5 * rstd[:, 0] ** 3 * (dy * xhat).sum(-1), atol=1e-12)
    # shift invariance: LN(x + c) = LN(x)
    y2, _ = bo.layernorm_fwd(x + 5.0, g, b)
    y1, _ = bo.layernorm_fwd(x, g, b)
    np.testing.assert_allclose(y1, y2, atol=1e-10)


def test_gelu_values():
    u = np.array([-3.0, -1.0, 0.0, 0.5, 2.0])
    # exact form: x * Phi(x), with Phi the normal CDF
    phi = np.array([0.5 * math.erfc(-v / math.sqrt(2)) for v in u])
    np.testing.assert_allclose(bo.gelu_fwd(u, "erf"), u * phi, rtol=1e-14, atol=1e-16)
    # tanh form stays within 5e-4 of the exact one and shares gelu(0)=0, gelu'(0)=1/2
    assert np.max(np.abs(bo.gelu_fwd(u, "tanh") - u * phi)) < 5e-4
    assert bo.gelu_fwd(np.zeros(1))[0] == 0 and bo.gelu_grad(np.zeros(1))[0] == 0.5
    for kind in ("tanh", "erf"):
        h = 1e-6
        fd = (bo.gelu_fwd(u + h, kind) - bo.gelu_fwd(u - h, kind)) / (2 * h)
        np.testing.assert_allclose(bo.gelu_grad(u, kind), fd, rtol=1e-8, atol=1e-9)
        # large |u|: gelu -> u or 0
        assert abs(bo.gelu_fwd(np.array([30.0]), kind)[0] - 30.0) < 1e-12
        assert abs(bo.gelu_fwd(np.array([-30.0]), kind)[0]) < 1e-12


def test_attention_invariants():
    rng = np.random.default_rng(11)
    qkv = rng.standard_normal((BATCH * S, 3 * H)) * 2
    dctx = rng.standard_normal((BATCH * S, H))
    d = H // HEADS
    for causal in (True, False):
        ctx, probs = bo.attention_fwd(qkv, BATCH, S, HEADS, causal)
        np.testing.assert_allclose(probs.sum(-1), 1.0, atol=1e-14)
        if causal:
            assert np.all(np.triu(probs, 1) == 0)
            # first query of every sequence sees only itself
            for b in range(BATCH):
                np.testing.assert_allclose(ctx[b * S], qkv[b * S, 2 * H:], atol=1e-14)
        # brute force, element by element, of one head
        b, j = 1, 1
        for i in range(S):
            last = i if causal else S - 1
            sc = [sum(qkv[b * S + i, j * d + t] * qkv[b * S + n, H + j * d + t] for t in range(d)) / math.sqrt(d)
                  for n in range(last + 1)]
            z = sum(math.exp(v) for v in sc)
            for t in range(d):
                want = sum(math.exp(sc[n]) / z * qkv[b * S + n, 2 * H + j * d + t] for n in range(last + 1))
                assert abs(ctx[b * S + i, j * d + t] - want) < 1e-12
        # softmax Jacobian rows sum to zero: adding a constant to a score row changes nothing,
        # so dQ . q-direction of a uniform key shift vanishes: check via dS row sums
        dqkv = bo.attention_bwd(dctx, qkv, probs, BATCH, S, HEADS)
        assert dqkv.shape == qkv.shape
    # causal: output at position i ignores later tokens
    q2 = qkv.copy()
    q2[S - 1] += 1.0                                   # last token of sequence 0
    a, _ = bo.attention_fwd(qkv, BATCH, S, HEADS, True)
    b_, _ = bo.attention_fwd(q2, BATCH, S, HEADS, True)
    np.testing.assert_array_equal(a[:S - 1], b_[:S - 1])
    np.testing.assert_array_equal(a[S:], b_[S:])       # and sequences do not mix


def test_equivariances():
    """Bidirectional block: permuting the sequence permutes the output (no positional
    term inside a stage); permuting the batch permutes the output for any mask."""
    params = _params(layers=2, seed=21)
    x, dy = _io(BATCH * S, H, seed=22)
    y, dx, gr = bo.stage_pass(x, dy, params, BATCH, S, HEADS, causal=False)
    perm = np.random.default_rng(0).permutation(S)
    idx = np.concatenate([b * S + perm for b in range(BATCH)])
    y2, dx2, gr2 = bo.stage_pass(x[idx], dy[idx], params, BATCH, S, HEADS, causal=False)
    np.testing.assert_allclose(y2, y[idx], atol=1e-11)
    np.testing.assert_allclose(dx2, dx[idx], atol=1e-11)
    np.testing.assert_allclose(bo.flatten_grads(gr2), bo.flatten_grads(gr), atol=1e-10)
    idx = np.concatenate([np.arange(S) + S, np.arange(S)])
    y3, dx3, gr3 = bo.stage_pass(x[idx], dy[idx], params, BATCH, S, HEADS, causal=True)
    y0, dx0, gr0 = bo.stage_pass(x, dy, params, BATCH, S, HEADS, causal=True)
    np.testing.assert_allclose(y3, y0[idx], atol=1e-11)
    np.testing.assert_allclose(bo.flatten_grads(gr3), bo.flatten_grads(gr0), atol=1e-10)


def test_bf16_rounding_helper():
    a = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.3, 3.1415926], dtype=np.float32)
    r = synth.round_to_bf16(a)
    want = torch.tensor(a).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(r, want)
    assert r[1] == 1.0 and r[3] == np.float32(1.0 + 2 ** -6)   # ties go to even


# ------------------------------------------------------------ op-by-op replay (sections 3.5, 3.6)
def _replay_case(D, N, f, batch):
    from oracle import schedule_oracle as so
    hidden, heads, seq, layers = 16, 2, 4, 1
    rng = np.random.default_rng(5)
    xs = {g: rng.standard_normal((batch * seq, hidden)) for g in range(N)}
    dys = {g: rng.standard_normal((batch * seq, hidden)) for g in range(N)}
    stage_params = {s: _params(hidden, layers, seed=10 + s) for s in range(D)}
    return so, xs, dys, stage_params, (batch, seq, heads)


def _sum_by_stage(D, N, xs, dys, stage_params, shape, stage_of_mb):
    """Per-stage gradient sums and per-micro-batch outputs from the plain stage pass."""
    batch, seq, heads = shape
    ys, dxs, grads = {}, {}, {}
    for g in range(N):
        s = stage_of_mb(g)
        y, dx, gr = bo.stage_pass(xs[g], dys[g], stage_params[s], batch, seq, heads)
        ys[g], dxs[g] = y, dx
        grads[s] = bo.add_grads(grads.get(s), gr)
    return ys, dxs, grads


@pytest.mark.parametrize("mode", ["direct", "doubling", "halving", "2f"])
def test_worker_replay_is_order_independent(mode):
    """Whatever the schedule, a synchronous iteration gives every micro-batch's stage pass and
    the per-stage sum of gradients (section 2: one weight version per iteration)."""
    D, f, batch = (8, 2, 2) if mode == "2f" else (4, 1, 2)
    N = 2 * D if mode == "doubling" else D
    rank = 1
    so, xs, dys, stage_params, shape = _replay_case(D, N, f, batch)
    lists = {"direct": lambda: so.chimera_schedule(D, N), "doubling": lambda: so.forward_doubling_schedule(D, N),
             "halving": lambda: so.backward_halving_schedule(D, N), "2f": lambda: so.chimera_schedule(D, N, f)}[mode]()
    ops = lists[rank]
    stage_of_pipe = {pipe: s for _, pipe, _, s in ops}
    pipe_of_mb = {}
    for kind, pipe, g, s in ops:
        pipe_of_mb[g] = pipe
        if kind == so.F2:
            pipe_of_mb[g + 1] = pipe
    ys, dxs, grads = bo.worker_replay(ops, {p: stage_params[s] for p, s in stage_of_pipe.items()}, xs, dys, *shape)
    want_y, want_dx, want_g = _sum_by_stage(D, N, xs, dys, stage_params, shape, lambda g: stage_of_pipe[pipe_of_mb[g]])
    assert sorted(ys) == sorted(dxs) == list(range(N))
    for g in range(N):
        np.testing.assert_allclose(ys[g], want_y[g], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(dxs[g], want_dx[g], rtol=1e-10, atol=1e-12)
    for pipe, s in stage_of_pipe.items():
        for got_layer, want_layer in zip(grads[pipe], want_g[s]):
            for k in want_layer:
                np.testing.assert_allclose(got_layer[k], want_layer[k], rtol=1e-9, atol=1e-11)


def test_doubled_forward_equals_two_forwards():
    # sequences never mix inside a block: a forward over the concatenation is the two forwards
    hidden, heads, seq, batch = 16, 2, 5, 3
    rng = np.random.default_rng(8)
    p = bo._f64(_params(hidden, 2, seed=3))
    xa, xb = rng.standard_normal((batch * seq, hidden)), rng.standard_normal((batch * seq, hidden))
    y2, _ = bo.stage_fwd(np.concatenate([xa, xb]), p, 2 * batch, seq, heads)
    ya, _ = bo.stage_fwd(xa, p, batch, seq, heads)
    yb, _ = bo.stage_fwd(xb, p, batch, seq, heads)
    np.testing.assert_allclose(y2, np.concatenate([ya, yb]), rtol=1e-13, atol=1e-13)
