"""Numeric oracle: forward and backward of one pipeline stage (a stack of
Transformer blocks) and of one Chimera worker, in float64 numpy.

TEST INFRASTRUCTURE ONLY.  Plain and slow on purpose; the tests, the smoke
check and the bench's cpu_baseline leg are its only callers.  It shares no
code with the HIP library and the product never imports it.

What it follows.  The Chimera paper treats a stage's compute as a black box
(section 3.4 measures its forward time F_t and models the backward as 2 F_t)
and states that the method is synchronous: every micro-batch of an iteration
sees the same weights and the weight gradient of a stage is the sum over the
micro-batches that pass through it (section 2, "Convergence friendliness";
the mini-batch gradient formula at the start of section 2).  Chimera only
reorders that work, so the oracle is the plain definition:

    Y_g  = Stage(X_g; theta)                       for each micro-batch g
    dX_g = (dStage/dX)^T dY_g
    dtheta = sum_g (dStage/dtheta)^T dY_g          over the stage's micro-batches

The paper says only "Transformer", "Bert", "GPT-2" about the block (section
3.1, section 4).  The reading used here, and by the library:

  * pre-LayerNorm block: x1 = x + Proj(Attn(LN1(x))),  y = x1 + FC2(GeLU(FC1(LN2(x1))))
  * biases on all four linear maps; weights stored [in, out], y = x W + b
  * LayerNorm over the hidden dimension, biased variance, eps = 1e-5
  * attention scores scaled by 1/sqrt(head_dim); causal mask lets query i see
    keys j <= i; no dropout, no padding mask, no positional term inside a stage
  * the fused QKV weight has columns [Q | K | V], head j owns columns
    j*d .. (j+1)*d-1 of each of the three blocks
  * GeLU in tanh form (default) or exact erf form
  * no 1/b loss scaling: the upstream gradient dY is an input.

Every backward formula is the textbook derivative written out; the tests pin
them with central finite differences, with the full-batch = sum-of-micro-
batches identity, with closed-form special cases and with an independent
autograd library.
"""
import math

import numpy as np
from scipy.special import erf as _erf

PARAM_ORDER = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")
LN_EPS = 1e-5


# ---------------------------------------------------------------- LayerNorm
def layernorm_fwd(x, gamma, beta, eps=LN_EPS):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)      # biased variance
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * gamma + beta, (xhat, rstd)


def layernorm_bwd(dy, cache, gamma):
    xhat, rstd = cache
    dgamma = (dy * xhat).sum(axis=0)
    dbeta = dy.sum(axis=0)
    dxhat = dy * gamma
    # d/dx of (x - mean) * rstd: remove the components along 1 and along xhat
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, dgamma, dbeta


# --------------------------------------------------------------------- GeLU
_K0 = math.sqrt(2.0 / math.pi)
_K1 = 0.044715


def gelu_fwd(u, kind="tanh"):
    if kind == "tanh":
        return 0.5 * u * (1.0 + np.tanh(_K0 * (u + _K1 * u ** 3)))
    if kind == "erf":
        return 0.5 * u * (1.0 + _erf(u / math.sqrt(2.0)))
    raise ValueError(kind)


def gelu_grad(u, kind="tanh"):
    if kind == "tanh":
        t = np.tanh(_K0 * (u + _K1 * u ** 3))
        return 0.5 * (1.0 + t) + 0.5 * u * (1.0 - t * t) * _K0 * (1.0 + 3.0 * _K1 * u * u)
    if kind == "erf":
        return 0.5 * (1.0 + _erf(u / math.sqrt(2.0))) + u * np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)
    raise ValueError(kind)


# ---------------------------------------------------------------- attention
def attention_fwd(qkv, batch, seq, heads, causal):
    """qkv [batch*seq, 3H] -> ctx [batch*seq, H]; returns the softmax matrices too."""
    M, H3 = qkv.shape
    H = H3 // 3
    d = H // heads
    assert M == batch * seq and H == heads * d
    ctx = np.zeros((M, H))
    probs = np.zeros((batch, heads, seq, seq))
    allowed = np.tril(np.ones((seq, seq), dtype=bool)) if causal else np.ones((seq, seq), dtype=bool)
    for b in range(batch):
        rows = slice(b * seq, (b + 1) * seq)
        for j in range(heads):
            q = qkv[rows, j * d:(j + 1) * d]
            k = qkv[rows, H + j * d:H + (j + 1) * d]
            v = qkv[rows, 2 * H + j * d:2 * H + (j + 1) * d]
            s = (q @ k.T) / math.sqrt(d)
            s = np.where(allowed, s, -np.inf)
            s = s - s.max(axis=-1, keepdims=True)
            e = np.exp(s)
            p = e / e.sum(axis=-1, keepdims=True)
            probs[b, j] = p
            ctx[rows, j * d:(j + 1) * d] = p @ v
    return ctx, probs


def attention_bwd(dctx, qkv, probs, batch, seq, heads):
    M, H3 = qkv.shape
    H = H3 // 3
    d = H // heads
    dqkv = np.zeros_like(qkv)
    for b in range(batch):
        rows = slice(b * seq, (b + 1) * seq)
        for j in range(heads):
            q = qkv[rows, j * d:(j + 1) * d]
            k = qkv[rows, H + j * d:H + (j + 1) * d]
            v = qkv[rows, 2 * H + j * d:2 * H + (j + 1) * d]
            p = probs[b, j]
            do = dctx[rows, j * d:(j + 1) * d]
            dv = p.T @ do
            dp = do @ v.T
            # softmax Jacobian, row by row: ds = p * (dp - sum_j p_j dp_j)
            ds = p * (dp - (p * dp).sum(axis=-1, keepdims=True))
            dq = (ds @ k) / math.sqrt(d)
            dk = (ds.T @ q) / math.sqrt(d)
            dqkv[rows, j * d:(j + 1) * d] = dq
            dqkv[rows, H + j * d:H + (j + 1) * d] = dk
            dqkv[rows, 2 * H + j * d:2 * H + (j + 1) * d] = dv
    return dqkv


# -------------------------------------------------------------------- block
def block_fwd(x, p, batch, seq, heads, causal=True, gelu="tanh"):
    """One pre-LN Transformer block.  x [batch*seq, H].  Returns (y, cache)."""
    h1, ln1 = layernorm_fwd(x, p["ln1_g"], p["ln1_b"])
    qkv = h1 @ p["w_qkv"] + p["b_qkv"]
    ctx, probs = attention_fwd(qkv, batch, seq, heads, causal)
    x1 = x + ctx @ p["w_o"] + p["b_o"]
    h2, ln2 = layernorm_fwd(x1, p["ln2_g"], p["ln2_b"])
    u = h2 @ p["w_fc1"] + p["b_fc1"]
    g = gelu_fwd(u, gelu)
    y = x1 + g @ p["w_fc2"] + p["b_fc2"]
    cache = dict(ln1=ln1, h1=h1, qkv=qkv, probs=probs, ctx=ctx, ln2=ln2, h2=h2, u=u, g=g,
                 batch=batch, seq=seq, heads=heads, gelu=gelu)
    return y, cache


def block_bwd(dy, cache, p):
    """Returns (dx, grads) with grads keyed like the parameters."""
    c = cache
    gr = {}
    # y = x1 + g W2 + b2
    gr["w_fc2"] = c["g"].T @ dy
    gr["b_fc2"] = dy.sum(axis=0)
    dg = dy @ p["w_fc2"].T
    du = dg * gelu_grad(c["u"], c["gelu"])
    gr["w_fc1"] = c["h2"].T @ du
    gr["b_fc1"] = du.sum(axis=0)
    dh2 = du @ p["w_fc1"].T
    dln2, gr["ln2_g"], gr["ln2_b"] = layernorm_bwd(dh2, c["ln2"], p["ln2_g"])
    dx1 = dy + dln2
    # x1 = x + ctx Wo + bo
    gr["w_o"] = c["ctx"].T @ dx1
    gr["b_o"] = dx1.sum(axis=0)
    dctx = dx1 @ p["w_o"].T
    dqkv = attention_bwd(dctx, c["qkv"], c["probs"], c["batch"], c["seq"], c["heads"])
    gr["w_qkv"] = c["h1"].T @ dqkv
    gr["b_qkv"] = dqkv.sum(axis=0)
    dh1 = dqkv @ p["w_qkv"].T
    dln1, gr["ln1_g"], gr["ln1_b"] = layernorm_bwd(dh1, c["ln1"], p["ln1_g"])
    dx = dx1 + dln1
    return dx, gr


# -------------------------------------------------------------------- stage
def _f64(params):
    return [{k: np.asarray(v, dtype=np.float64) for k, v in layer.items()} for layer in params]


def stage_fwd(x, params, batch, seq, heads, causal=True, gelu="tanh"):
    """params: list (one per block) of dicts keyed by PARAM_ORDER."""
    caches = []
    x = np.asarray(x, dtype=np.float64)
    for p in params:
        x, c = block_fwd(x, p, batch, seq, heads, causal, gelu)
        caches.append(c)
    return x, caches


def stage_bwd(dy, caches, params):
    grads = [None] * len(params)
    dy = np.asarray(dy, dtype=np.float64)
    for i in range(len(params) - 1, -1, -1):
        dy, grads[i] = block_bwd(dy, caches[i], params[i])
    return dy, grads


def stage_pass(x, dy, params, batch, seq, heads, causal=True, gelu="tanh"):
    """Forward then backward of one micro-batch through one stage."""
    params = _f64(params)
    y, caches = stage_fwd(x, params, batch, seq, heads, causal, gelu)
    dx, grads = stage_bwd(dy, caches, params)
    return y, dx, grads


def add_grads(total, grads):
    if total is None:
        return [{k: v.copy() for k, v in layer.items()} for layer in grads]
    for t, g in zip(total, grads):
        for k in t:
            t[k] += g[k]
    return total


def worker_iteration(rank, D, N, params_down, params_up, xs, dys, batch, seq, heads,
                     causal=True, gelu="tanh", only=None):
    """One training iteration of Chimera worker `rank` (section 3.1).

    The worker owns stage `rank` of the down pipeline (weights params_down)
    and stage D-1-rank of the up pipeline (weights params_up).  In every unit
    of D micro-batches the first half belongs to the down pipeline and the
    second half to the up pipeline.  xs[g], dys[g] are the activation arriving
    from the previous stage and the gradient arriving from the next stage for
    micro-batch g.  Being synchronous, the result does not depend on the order
    of execution, so micro-batches are simply taken in ascending order.
    `only`: optional set of micro-batch ids to restrict the sum to.
    Returns (ys, dxs, grads_down, grads_up); ys/dxs are dicts keyed by g.
    """
    assert D % 2 == 0 and N % D == 0 and 0 <= rank < D
    pd, pu = _f64(params_down), _f64(params_up)
    ys, dxs = {}, {}
    gd = gu = None
    for g in range(N):
        if only is not None and g not in only:
            continue
        down = (g % D) < D // 2
        p = pd if down else pu
        y, caches = stage_fwd(xs[g], p, batch, seq, heads, causal, gelu)
        dx, grads = stage_bwd(dys[g], caches, p)
        ys[g], dxs[g] = y, dx
        if down:
            gd = add_grads(gd, grads)
        else:
            gu = add_grads(gu, grads)
    return ys, dxs, gd, gu


def worker_replay(ops, params_by_pipe, xs, dys, batch, seq, heads, causal=True, gelu="tanh"):
    """Executes one worker's op list literally, op by op (sections 3.1, 3.5, 3.6).

    ops: [(kind, pipe, g, stage), ...] as the schedule oracle lists them, with
    kind 0 forward, 1 backward, 2 forward of micro-batches g and g+1 together
    (forward doubling), 3 / 4 backward of the first / second half of the
    micro-batch's sequences (backward halving).  params_by_pipe[pipe] are the
    weights of the stage this worker holds for that pipeline.

    A doubled forward runs the stage once on the 2*batch sequences of the two
    micro-batches and keeps no activations; the backward of such a micro-batch
    first runs its forward again (activation recomputation), then the
    backward.  A half backward is the backward of those sequences alone: every
    operation of a block acts within one sequence, so the forward of a half
    equals the matching rows of the whole forward and is simply recomputed here
    instead of slicing the kept activations.

    Returns (ys, dxs, grads_by_pipe): ys, dxs keyed by micro-batch id.
    """
    params = {p: _f64(v) for p, v in params_by_pipe.items()}
    tokens = batch * seq
    ys, dxs, kept, grads = {}, {}, {}, {p: None for p in params}
    for kind, pipe, g, _stage in ops:
        p = params[pipe]
        if kind == 0:
            ys[g], kept[g] = stage_fwd(xs[g], p, batch, seq, heads, causal, gelu)
        elif kind == 2:
            y2, _ = stage_fwd(np.concatenate([xs[g], xs[g + 1]], axis=0), p, 2 * batch, seq, heads, causal, gelu)
            ys[g], ys[g + 1] = y2[:tokens], y2[tokens:]
        elif kind == 1:
            caches = kept.pop(g) if g in kept else stage_fwd(xs[g], p, batch, seq, heads, causal, gelu)[1]
            dxs[g], gr = stage_bwd(dys[g], caches, p)
            grads[pipe] = add_grads(grads[pipe], gr)
        elif kind in (3, 4):
            assert batch % 2 == 0 and g in kept
            lo = (kind - 3) * (tokens // 2)
            rows = slice(lo, lo + tokens // 2)
            _, caches = stage_fwd(xs[g][rows], p, batch // 2, seq, heads, causal, gelu)
            dx_half, gr = stage_bwd(dys[g][rows], caches, p)
            dxs.setdefault(g, np.zeros_like(np.asarray(xs[g], dtype=np.float64)))[rows] = dx_half
            grads[pipe] = add_grads(grads[pipe], gr)
            if kind == 4:
                kept.pop(g)
        else:
            raise ValueError("unknown op kind %r" % (kind,))
    assert not kept, "forward without backward"
    return ys, dxs, grads


def flatten_grads(grads):
    """Concatenate per-layer gradients in the library's flat parameter order."""
    return np.concatenate([layer[k].reshape(-1) for layer in grads for k in PARAM_ORDER])
