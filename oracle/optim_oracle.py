"""Optimizer step on the shared array M -- TEST INFRASTRUCTURE ONLY (numpy, float64).

The paper times the weight update of its training workload with stock SGD, Adagrad and Adam on
the |M|-sized parameter (Appendix "training" tables, "update weights (optim.step())"); it defines no
update rule of its own, so these are the textbook rules in the form those stock optimizers use:

  g = dM + weight_decay * M
  SGD      : M <- M - lr * g
  Adagrad  : s <- s + g*g ;                M <- M - lr * g / (sqrt(s) + eps)
  Adam     : m <- b1*m + (1-b1)*g ; v <- b2*v + (1-b2)*g*g ;
             M <- M - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)       (t = 1, 2, ...)

Every function returns new arrays and leaves its inputs alone.
"""
import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def sgd(M, dM, lr, weight_decay=0.0):
    M, g = _f64(M), _f64(dM) + weight_decay * _f64(M)
    return M - lr * g


def adagrad(M, dM, state_sum, lr, weight_decay=0.0, eps=1e-10):
    M = _f64(M)
    g = _f64(dM) + weight_decay * M
    s = _f64(state_sum) + g * g
    return M - lr * g / (np.sqrt(s) + eps), s


def adam(M, dM, exp_avg, exp_avg_sq, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    M = _f64(M)
    g = _f64(dM) + weight_decay * M
    m = beta1 * _f64(exp_avg) + (1.0 - beta1) * g
    v = beta2 * _f64(exp_avg_sq) + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    return M - lr * mhat / (np.sqrt(vhat) + eps), m, v
