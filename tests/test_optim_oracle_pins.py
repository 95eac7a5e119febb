"""Pins for the optimizer oracle (numpy, float64): the stock optimizers of PyTorch on the CPU in
float64 are the library routines these rules reduce to; closed forms cover single steps."""
import numpy as np
import pytest
import torch

import oracle


def _torch_run(kind, M0, grads, **kw):
    p = torch.nn.Parameter(torch.tensor(M0, dtype=torch.float64))
    if kind == "sgd":
        opt = torch.optim.SGD([p], lr=kw["lr"], weight_decay=kw.get("weight_decay", 0.0))
    elif kind == "adagrad":
        opt = torch.optim.Adagrad([p], lr=kw["lr"], weight_decay=kw.get("weight_decay", 0.0), eps=kw["eps"])
    else:
        opt = torch.optim.Adam([p], lr=kw["lr"], betas=(kw["beta1"], kw["beta2"]), eps=kw["eps"],
                               weight_decay=kw.get("weight_decay", 0.0))
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
    return p.detach().numpy()


@pytest.mark.parametrize("wd", [0.0, 0.01])
def test_sgd_adagrad_adam_match_the_stock_optimizers(wd):
    rng = np.random.default_rng(5)
    M0 = rng.standard_normal(257) * 0.02
    grads = [rng.standard_normal(257) * s for s in (1.0, 0.1, 3.0, 1e-3)]
    # SGD
    M = M0.copy()
    for g in grads:
        M = oracle.optim.sgd(M, g, 0.05, wd)
    assert np.allclose(M, _torch_run("sgd", M0, grads, lr=0.05, weight_decay=wd), rtol=1e-13, atol=0)
    # Adagrad
    M, s = M0.copy(), np.zeros_like(M0)
    for g in grads:
        M, s = oracle.optim.adagrad(M, g, s, 0.05, wd, 1e-10)
    assert np.allclose(M, _torch_run("adagrad", M0, grads, lr=0.05, weight_decay=wd, eps=1e-10), rtol=1e-12, atol=0)
    # Adam
    M, m, v = M0.copy(), np.zeros_like(M0), np.zeros_like(M0)
    for t, g in enumerate(grads, start=1):
        M, m, v = oracle.optim.adam(M, g, m, v, t, 1e-3, 0.9, 0.999, 1e-8, wd)
    ref = _torch_run("adam", M0, grads, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=wd)
    assert np.allclose(M, ref, rtol=1e-12, atol=0)


def test_closed_forms_of_a_first_step():
    g = np.array([2.0, -0.5, 0.0])
    M = np.array([1.0, 1.0, 1.0])
    assert np.allclose(oracle.optim.sgd(M, g, 0.1), [0.8, 1.05, 1.0])
    # first Adagrad step with eps -> 0 moves every non-zero coordinate by exactly lr * sign(g)
    Mn, s = oracle.optim.adagrad(M, g, np.zeros(3), 0.1, 0.0, 0.0 + 1e-300)
    assert np.allclose(Mn, [0.9, 1.1, 1.0]) and np.allclose(s, g * g)
    # first Adam step: bias correction makes m_hat = g and v_hat = g^2, so the move is lr * sign(g) (eps -> 0)
    Mn, m, v = oracle.optim.adam(M, g, np.zeros(3), np.zeros(3), 1, 0.1, 0.9, 0.999, 1e-300)
    assert np.allclose(Mn, [0.9, 1.1, 1.0])
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)
