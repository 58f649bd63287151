"""Numeric oracle for the two ends of the pipeline: the embedding in front of
the first stage and the language-model head with its loss behind the last one,
in float64 numpy.

TEST INFRASTRUCTURE ONLY.  It shares no code with the HIP library and the
product never imports it.

What it follows.  The Chimera paper trains Bert-48 and GPT-2 (section 4, Table
4) and only remarks about the ends that "the first stage ... includes an extra
embedding layer" (section 4.1, memory consumption); the last stage of a
language model turns hidden states into a loss.  Nothing else is specified, so
the reading is the GPT-2 one, written out as plain definitions:

  embedding   x[t] = wte[token[t]] + wpe[t mod S]              (token + learned position table)
  head        h    = LayerNorm(y; g, b)                         (final LayerNorm, eps 1e-5, biased variance)
              z    = h W                                        (W stored [H, V], no bias, not tied)
              loss = scale * sum_t ( logsumexp(z[t]) - z[t, target[t]] )

`scale` is the caller's weight of this micro-batch's tokens in the mini-batch
loss (1 / number of tokens for a mean); the oracle does not choose it.  The
backward formulas are the textbook derivatives:

  dz = scale * (softmax(z) - onehot(target)),  dW = h^T dz,  dh = dz W^T,
  dy, dg, db = LayerNorm backward of dh;        dwte[v] = sum of dx[t] over t with token[t] = v,
  dwpe[p] = sum of dx[t] over t with t mod S = p.

Pinned by the tests with central finite differences, closed forms (uniform
logits give log V; a shift of a row of logits changes nothing; every row of dz
sums to zero; scatter = one-hot matrix product) and an independent autograd
library.
"""
import numpy as np

LN_EPS = 1e-5


def embedding_fwd(tokens, seq, wte, wpe):
    """tokens: int array [M] (M = batch*seq, token index b*seq + s); returns x [M, H]."""
    tokens = np.asarray(tokens)
    pos = np.arange(tokens.shape[0]) % seq
    return np.asarray(wte, dtype=np.float64)[tokens] + np.asarray(wpe, dtype=np.float64)[pos]


def embedding_bwd(dx, tokens, seq, vocab):
    """Returns (dwte [vocab, H], dwpe [seq, H]): plain scatter-additions in token order."""
    dx = np.asarray(dx, dtype=np.float64)
    tokens = np.asarray(tokens)
    dwte = np.zeros((vocab, dx.shape[1]))
    dwpe = np.zeros((seq, dx.shape[1]))
    for t in range(dx.shape[0]):
        dwte[tokens[t]] += dx[t]
        dwpe[t % seq] += dx[t]
    return dwte, dwpe


def softmax_xent(z, targets, scale):
    """loss = scale * sum_t (logsumexp(z[t]) - z[t, target[t]]); returns (loss, dz)."""
    z = np.asarray(z, dtype=np.float64)
    targets = np.asarray(targets)
    m = z.max(axis=1, keepdims=True)
    e = np.exp(z - m)
    s = e.sum(axis=1, keepdims=True)
    lse = (m + np.log(s))[:, 0]
    rows = np.arange(z.shape[0])
    loss = scale * float(np.sum(lse - z[rows, targets]))
    dz = e / s
    dz[rows, targets] -= 1.0
    return loss, scale * dz


def head_fwd_bwd(y, targets, lnf_g, lnf_b, w_head, scale):
    """Final LayerNorm, vocabulary projection, cross-entropy; forward and backward.

    Returns dict(loss, dy, dlnf_g, dlnf_b, dw_head, logits).
    """
    y = np.asarray(y, dtype=np.float64)
    g = np.asarray(lnf_g, dtype=np.float64)
    b = np.asarray(lnf_b, dtype=np.float64)
    w = np.asarray(w_head, dtype=np.float64)
    mu = y.mean(axis=1, keepdims=True)
    var = ((y - mu) ** 2).mean(axis=1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + LN_EPS)
    xh = (y - mu) * rstd
    h = xh * g + b
    z = h @ w
    loss, dz = softmax_xent(z, targets, scale)
    dw = h.T @ dz
    dh = dz @ w.T
    dg = (dh * xh).sum(axis=0)
    db = dh.sum(axis=0)
    dxh = dh * g
    dy = rstd * (dxh - dxh.mean(axis=1, keepdims=True) - xh * (dxh * xh).mean(axis=1, keepdims=True))
    return dict(loss=loss, dy=dy, dlnf_g=dg, dlnf_b=db, dw_head=dw, logits=z)
