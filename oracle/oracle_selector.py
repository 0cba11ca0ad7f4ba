"""CPU oracle of the saturation-aware chunk-size selection (Optimus Sec. 5).

TEST INFRASTRUCTURE ONLY: numpy fp64, exhaustive search, no code shared with the library.

Sec. 5.2 models the step latency over x = batch * chunk as one curve that passes through a
memory-bound, a transition and a compute-bound regime, affine in each, with coefficients from
offline profiling; it does not give the fitting procedure.  Reading: the curve is continuous
(it is one latency curve, the regimes meet at their boundaries), the two boundaries lie at
profiled loads strictly between the smallest and the largest one, and for a pair of boundaries
b0 < b1 the four free parameters of
    T(x) = alpha + beta * x + gamma0 * max(0, x - b0) + gamma1 * max(0, x - b1)
are the ordinary least-squares solution (numpy.linalg.lstsq); the pair with the smallest
squared error wins (the first such pair in (b0, b1) order).  The model is handed out per
regime: T(x) = beta1[k] * x + beta0[k], k = 0 for x < b0, 1 for x < b1, else 2.
Sec. 5.1: c* = argmax over the candidates of N_commit(c) * b / T(c * b).
"""
import numpy as np


def _hinge_fit(x, t, b0, b1):
    A = np.stack([np.ones_like(x), x, np.maximum(0.0, x - b0), np.maximum(0.0, x - b1)], axis=1)
    sol = np.linalg.lstsq(A, t, rcond=None)[0]
    r = t - A @ sol
    return sol, float(r @ r)


def latency_fit(x, t):
    """Returns dict(x_break [2], beta1 [3], beta0 [3], sse)."""
    x = np.asarray(x, dtype=np.float64)
    t = np.asarray(t, dtype=np.float64)
    loads = np.unique(x)                      # distinct loads, ascending
    inner = loads[1:-1]                       # a boundary has a profiled load on either side
    best = None
    for i in range(len(inner)):
        for j in range(i + 1, len(inner)):
            b0, b1 = inner[i], inner[j]
            (alpha, beta, g0, g1), sse = _hinge_fit(x, t, b0, b1)
            if best is None or sse < best["sse"]:
                best = dict(x_break=np.array([b0, b1]),
                            beta1=np.array([beta, beta + g0, beta + g0 + g1]),
                            beta0=np.array([alpha, alpha - g0 * b0, alpha - g0 * b0 - g1 * b1]), sse=sse)
    if best is None:
        raise ValueError("fewer than four distinct loads")
    return best


def latency_eval(model, x):
    k = 0 if x < model["x_break"][0] else (1 if x < model["x_break"][1] else 2)
    return model["beta1"][k] * x + model["beta0"][k]


def select_chunk(model, batch, chunk_sizes, n_commit):
    """Returns (index of the best candidate, objective values)."""
    rates = np.array([n_commit[i] * batch / latency_eval(model, float(batch) * chunk_sizes[i])
                      for i in range(len(chunk_sizes))])
    return int(np.argmax(rates)), rates
