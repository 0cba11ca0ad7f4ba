"""CPU oracle of the saturation-aware chunk-size selection (Optimus Sec. 5).

TEST INFRASTRUCTURE ONLY: numpy fp64, exhaustive search, no code shared with the library.

Sec. 5.2 models the step latency as three affine regimes over x = batch * chunk and says the
coefficients come from offline profiling without giving the fitting procedure.  Reading: order
the samples by x, try every pair of cuts that leaves three runs with at least two distinct x
each and never separates equal x, fit each run with an ordinary least-squares line
(numpy.linalg.lstsq), keep the pair of smallest total squared error (the first such pair); the
regime boundary is the midpoint of the two samples a cut separates.
Sec. 5.1: c* = argmax over the candidates of N_commit(c) * b / T(c * b).
"""
import numpy as np


def _line(x, t):
    A = np.stack([x, np.ones_like(x)], axis=1)
    sol = np.linalg.lstsq(A, t, rcond=None)[0]
    r = t - A @ sol
    return sol[0], sol[1], float(r @ r)


def latency_fit(x, t):
    """Returns dict(x_break [2], beta1 [3], beta0 [3], sse, cuts (a, b))."""
    x = np.asarray(x, dtype=np.float64)
    t = np.asarray(t, dtype=np.float64)
    order = np.argsort(x, kind="stable")
    x, t = x[order], t[order]
    n = len(x)
    best = None
    for a in range(1, n):
        if x[a] == x[a - 1] or len(np.unique(x[:a])) < 2:
            continue
        l0 = _line(x[:a], t[:a])
        for b in range(a + 1, n):
            if x[b] == x[b - 1] or len(np.unique(x[a:b])) < 2 or len(np.unique(x[b:])) < 2:
                continue
            l1, l2 = _line(x[a:b], t[a:b]), _line(x[b:], t[b:])
            sse = l0[2] + l1[2] + l2[2]
            if best is None or sse < best["sse"]:
                best = dict(x_break=np.array([(x[a - 1] + x[a]) / 2, (x[b - 1] + x[b]) / 2]),
                            beta1=np.array([l0[0], l1[0], l2[0]]),
                            beta0=np.array([l0[1], l1[1], l2[1]]), sse=sse, cuts=(a, b))
    if best is None:
        raise ValueError("no admissible pair of cuts")
    return best


def latency_eval(model, x):
    k = 0 if x < model["x_break"][0] else (1 if x < model["x_break"][1] else 2)
    return model["beta1"][k] * x + model["beta0"][k]


def select_chunk(model, batch, chunk_sizes, n_commit):
    """Returns (index of the best candidate, objective values)."""
    rates = np.array([n_commit[i] * batch / latency_eval(model, float(batch) * chunk_sizes[i])
                      for i in range(len(chunk_sizes))])
    return int(np.argmax(rates)), rates
