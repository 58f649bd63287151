"""Pins of the oracle for the pipeline's two ends (embedding; LM head and loss); CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import edges_oracle as eo

V, H, S, B = 37, 12, 5, 3
M = B * S


def _case(seed=0):
    rng = np.random.default_rng(seed)
    return dict(tokens=rng.integers(0, V, size=M), targets=rng.integers(0, V, size=M),
                wte=rng.standard_normal((V, H)), wpe=rng.standard_normal((S, H)),
                y=rng.standard_normal((M, H)) * 2 + 0.3, g=1 + 0.3 * rng.standard_normal(H), b=0.2 * rng.standard_normal(H),
                w=rng.standard_normal((H, V)) * 0.7, dx=rng.standard_normal((M, H)))


def test_embedding_is_one_hot_product():
    c = _case()
    x = eo.embedding_fwd(c["tokens"], S, c["wte"], c["wpe"])
    onehot = np.eye(V)[c["tokens"]]
    posmat = np.eye(S)[np.arange(M) % S]
    np.testing.assert_allclose(x, onehot @ c["wte"] + posmat @ c["wpe"], rtol=0, atol=1e-14)
    dwte, dwpe = eo.embedding_bwd(c["dx"], c["tokens"], S, V)
    np.testing.assert_allclose(dwte, onehot.T @ c["dx"], rtol=0, atol=1e-12)
    np.testing.assert_allclose(dwpe, posmat.T @ c["dx"], rtol=0, atol=1e-12)
    # position p of every sequence shares one row of the position table
    assert np.allclose(x[2] - c["wte"][c["tokens"][2]], x[S + 2] - c["wte"][c["tokens"][S + 2]])


def test_softmax_xent_closed_forms():
    z = np.zeros((4, V))
    t = np.array([0, 5, 7, V - 1])
    loss, dz = eo.softmax_xent(z, t, 1.0 / 4)
    assert loss == pytest.approx(math.log(V))                      # uniform prediction
    c = _case(1)
    z = c["y"] @ c["w"]
    loss, dz = eo.softmax_xent(z, c["targets"], 0.5)
    np.testing.assert_allclose(dz.sum(axis=1), 0.0, atol=1e-14)     # probabilities sum to one
    shifted = z + np.random.default_rng(2).standard_normal((M, 1)) * 50
    loss2, dz2 = eo.softmax_xent(shifted, c["targets"], 0.5)
    assert loss2 == pytest.approx(loss, rel=1e-12) and np.allclose(dz, dz2, atol=1e-12)
    # brute force on one row
    p = np.exp(z[3]) / np.exp(z[3]).sum()
    assert -math.log(p[c["targets"][3]]) * 0.5 == pytest.approx(eo.softmax_xent(z[3:4], c["targets"][3:4], 0.5)[0])
    # a confident correct prediction costs nothing and pushes nothing
    big = np.full((1, V), -60.0); big[0, 9] = 60.0
    loss3, dz3 = eo.softmax_xent(big, np.array([9]), 1.0)
    assert loss3 == pytest.approx(0.0, abs=1e-12) and np.abs(dz3).max() < 1e-12


def test_head_finite_differences():
    c = _case(3)
    scale = 1.0 / M
    out = eo.head_fwd_bwd(c["y"], c["targets"], c["g"], c["b"], c["w"], scale)
    f = lambda **kw: eo.head_fwd_bwd(kw.get("y", c["y"]), c["targets"], kw.get("g", c["g"]), kw.get("b", c["b"]),
                                     kw.get("w", c["w"]), scale)["loss"]
    rng = np.random.default_rng(4)
    for name, grad in (("y", out["dy"]), ("g", out["dlnf_g"]), ("b", out["dlnf_b"]), ("w", out["dw_head"])):
        base = c[name]
        for _ in range(6):
            idx = tuple(rng.integers(0, n) for n in base.shape)
            eps = 1e-6
            hi, lo = base.copy(), base.copy()
            hi[idx] += eps
            lo[idx] -= eps
            num = (f(**{name: hi}) - f(**{name: lo})) / (2 * eps)
            assert num == pytest.approx(grad[idx], rel=2e-5, abs=1e-9), (name, idx)


def test_against_library_autograd():
    c = _case(5)
    scale = 0.25
    t = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    wte, wpe, g, b, w = t(c["wte"]), t(c["wpe"]), t(c["g"]), t(c["b"]), t(c["w"])
    tok = torch.tensor(c["tokens"])
    x = torch.nn.functional.embedding(tok, wte) + wpe[torch.arange(M) % S]
    np.testing.assert_allclose(x.detach().numpy(), eo.embedding_fwd(c["tokens"], S, c["wte"], c["wpe"]), atol=1e-14)
    h = torch.nn.functional.layer_norm(x, (H,), g, b, 1e-5)
    loss = scale * torch.nn.functional.cross_entropy(h @ w, torch.tensor(c["targets"]), reduction="sum")
    loss.backward()
    xs = x.detach().numpy()
    out = eo.head_fwd_bwd(xs, c["targets"], c["g"], c["b"], c["w"], scale)
    assert out["loss"] == pytest.approx(float(loss.detach()), rel=1e-12)
    np.testing.assert_allclose(out["dw_head"], w.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(out["dlnf_g"], g.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(out["dlnf_b"], b.grad.numpy(), rtol=1e-10, atol=1e-12)
    dwte, dwpe = eo.embedding_bwd(out["dy"], c["tokens"], S, V)
    np.testing.assert_allclose(dwte, wte.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dwpe, wpe.grad.numpy(), rtol=1e-10, atol=1e-12)
