"""Chunk-size selection (Sec. 5): pins of the numpy oracle, then the C-ABI host functions against
the oracle.  No GPU is involved: the functions are host code."""
import numpy as np
import pytest
import scipy.stats

from paper_2605_24832_amd import OptimusError, latency_eval, latency_fit, select_chunk

# a latency curve with the three regimes of Sec. 5.2: flat (memory-bound), steeper transition,
# proportional to the load (compute-bound); continuous at the two boundaries 256 and 1024
TRUE = dict(x_break=[256.0, 1024.0], beta1=[0.001, 0.01, 0.03], beta0=[10.0, 7.696, -12.784])


def true_latency(x):
    x = np.asarray(x, dtype=np.float64)
    k = (x >= TRUE["x_break"][0]).astype(int) + (x >= TRUE["x_break"][1]).astype(int)
    return np.asarray(TRUE["beta1"])[k] * x + np.asarray(TRUE["beta0"])[k]


def sample_loads():
    # batch x chunk grid of the profiling sweep: b in 1..256, c in 1..32, duplicates kept
    return np.array(sorted(b * c for b in (1, 2, 4, 8, 16, 32, 64, 128, 256) for c in (1, 2, 4, 8, 16, 32)
                           if b * c <= 8192), dtype=np.float64)


# ---------------------------------------------------------------- oracle pins

def constrained_three_lines(x, t, b0, b1):
    """Independent formulation of the same fit: three separate lines (slope, intercept) on the
    samples x < b0, b0 <= x < b1, x >= b1, minimising the total squared error subject to the two
    equality constraints that neighbours meet at b0 and b1; solved as one KKT linear system.
    Returns (params [s0, i0, s1, i1, s2, i2], squared error)."""
    k = (x >= b0).astype(int) + (x >= b1).astype(int)
    A = np.zeros((len(x), 6))
    A[np.arange(len(x)), 2 * k] = x
    A[np.arange(len(x)), 2 * k + 1] = 1.0
    C = np.array([[b0, 1.0, -b0, -1.0, 0.0, 0.0], [0.0, 0.0, b1, 1.0, -b1, -1.0]])
    K = np.block([[2 * A.T @ A, C.T], [C, np.zeros((2, 2))]])
    sol = np.linalg.solve(K, np.concatenate([2 * A.T @ t, np.zeros(2)]))[:6]
    r = t - A @ sol
    return sol, float(r @ r)


def test_oracle_recovers_an_exact_three_regime_curve(oracle_mod):
    x = sample_loads()
    m = oracle_mod.selector.latency_fit(x, true_latency(x))
    np.testing.assert_array_equal(m["x_break"], TRUE["x_break"])   # both boundaries are profiled loads
    np.testing.assert_allclose(m["beta1"], TRUE["beta1"], rtol=1e-9)
    np.testing.assert_allclose(m["beta0"], TRUE["beta0"], rtol=1e-9, atol=1e-9)
    assert m["sse"] < 1e-16
    for q in (1, 100, 128, 256, 300, 512, 1024, 2048, 5000):
        assert abs(oracle_mod.selector.latency_eval(m, q) - true_latency(q)) < 1e-9


def test_oracle_fit_is_continuous_and_optimal(oracle_mod):
    rng = np.random.RandomState(3)
    x = sample_loads()
    t = true_latency(x) * (1 + 0.02 * rng.standard_normal(len(x)))
    m = oracle_mod.selector.latency_fit(x, t)
    b0, b1 = m["x_break"]
    # one curve: the regimes meet at the boundaries
    for k, b in enumerate((b0, b1)):
        left = m["beta1"][k] * b + m["beta0"][k]
        right = m["beta1"][k + 1] * b + m["beta0"][k + 1]
        assert abs(left - right) < 1e-9 * abs(left)
    # the same numbers from the constrained three-line formulation at these boundaries
    sol, sse = constrained_three_lines(x, t, b0, b1)
    np.testing.assert_allclose(sol[0::2], m["beta1"], rtol=1e-8)
    np.testing.assert_allclose(sol[1::2], m["beta0"], rtol=1e-8, atol=1e-9)
    assert abs(sse - m["sse"]) < 1e-9 * sse
    # no admissible pair of boundaries does better (exhaustive, through the other formulation),
    # and the boundaries are interior profiled loads
    loads = np.unique(x)
    assert b0 in loads[1:-1] and b1 in loads[1:-1] and b0 < b1
    best = min(constrained_three_lines(x, t, p, q)[1] for i, p in enumerate(loads[1:-1]) for q in loads[2 + i:-1])
    assert abs(best - m["sse"]) < 1e-9 * best
    # the continuity constraint can only cost: never below three unconstrained regressions
    free = 0.0
    for lo, hi in ((-np.inf, b0), (b0, b1), (b1, np.inf)):
        sel = (x >= lo) & (x < hi)
        r = scipy.stats.linregress(x[sel], t[sel])
        free += float(np.sum((t[sel] - (r.slope * x[sel] + r.intercept)) ** 2))
    assert m["sse"] >= free * (1 - 1e-12)


def test_oracle_single_line_and_sample_order(oracle_mod):
    x = np.arange(1, 13, dtype=np.float64)
    m = oracle_mod.selector.latency_fit(x[::-1], 2.5 * x[::-1] + 4)   # order of the samples is free
    np.testing.assert_allclose(m["beta1"], [2.5] * 3, rtol=1e-9)
    np.testing.assert_allclose(m["beta0"], [4.0] * 3, rtol=1e-9)
    # one boundary is enough for two regimes: the second one is then free; whatever it is, the
    # curve is recovered and the boundaries never sit at the extreme loads
    t2 = np.where(x < 7, 3.0, 3.0 + 2.0 * (x - 7))
    m2 = oracle_mod.selector.latency_fit(x, t2)
    assert m2["sse"] < 1e-18 and 7.0 in m2["x_break"]
    assert x.min() < m2["x_break"][0] < m2["x_break"][1] < x.max()
    for q in (1, 5, 7, 9.5, 12, 20):
        want = 3.0 if q < 7 else 3.0 + 2.0 * (q - 7)
        assert abs(oracle_mod.selector.latency_eval(m2, q) - want) < 1e-9
    # four distinct loads are the fewest that leave room for two interior boundaries
    m3 = oracle_mod.selector.latency_fit([1, 2, 3, 4, 4, 1], [5, 5, 6, 9, 9, 5])
    np.testing.assert_array_equal(m3["x_break"], [2.0, 3.0])
    assert m3["sse"] < 1e-20
    with pytest.raises(ValueError):
        oracle_mod.selector.latency_fit([1, 1, 2, 2, 3, 3], [1, 1, 2, 2, 3, 3])  # three distinct loads only


def test_oracle_selection_follows_the_two_limits_of_sec_5(oracle_mod):
    sel = oracle_mod.selector
    cs = [2, 4, 8, 16, 32]
    n_commit = np.array([1.4, 2.0, 2.6, 3.0, 3.2])        # grows with c, diminishing returns
    flat = dict(x_break=np.array([1e9, 2e9]), beta1=np.zeros(3), beta0=np.full(3, 5.0))
    prop = dict(x_break=np.array([1e9, 2e9]), beta1=np.full(3, 0.01), beta0=np.zeros(3))
    # memory-bound (latency does not depend on the load): the most committed tokens win
    i, r = sel.select_chunk(flat, 4, cs, n_commit)
    assert i == 4 and np.allclose(r, n_commit * 4 / 5.0)
    # compute-bound (latency proportional to b*c): the best token utilisation N/c wins
    i, r = sel.select_chunk(prop, 64, cs, n_commit)
    assert i == 0 and np.allclose(r, n_commit / (0.01 * np.array(cs)))
    # hand-worked mixed case, batch 8: T = 10 ms up to x = 64, then 10 + 0.5 (x - 64)
    mixed = dict(x_break=np.array([64.0, 1e9]), beta1=np.array([0.0, 0.5, 0.5]),
                 beta0=np.array([10.0, -22.0, -22.0]))
    i, r = sel.select_chunk(mixed, 8, cs, n_commit)
    # x = 16, 32, 64, 128, 256 -> T = 10, 10, 10, 42, 106 -> rate = 1.12, 1.6, 2.08, 0.571, 0.2415
    np.testing.assert_allclose(r, [1.12, 1.6, 2.08, 24 / 42, 25.6 / 106], rtol=1e-12)
    assert i == 2
    # as the batch grows the chosen chunk never grows (saturation reached with fewer tokens per request)
    m = dict(x_break=np.array(TRUE["x_break"]), beta1=np.array(TRUE["beta1"]), beta0=np.array(TRUE["beta0"]))
    picks = [cs[sel.select_chunk(m, b, cs, n_commit)[0]] for b in (1, 4, 16, 64, 256, 1024)]
    assert picks[0] == 32 and picks[-1] == 2 and all(p >= q for p, q in zip(picks, picks[1:]))


# ---------------------------------------------------------------- library vs oracle

def model_dict(m):
    return dict(x_break=np.array(m.x_break[:]), beta1=np.array(m.beta1[:]), beta0=np.array(m.beta0[:]))


@pytest.mark.parametrize("seed,noise", [(0, 0.0), (1, 0.01), (2, 0.05), (3, 0.2)])
def test_library_fit_matches_oracle(oracle_mod, seed, noise):
    rng = np.random.RandomState(seed)
    x = sample_loads()
    t = true_latency(x) * (1 + noise * rng.standard_normal(len(x)))
    perm = rng.permutation(len(x))
    m, sse = latency_fit(x[perm], t[perm])
    ref = oracle_mod.selector.latency_fit(x[perm], t[perm])
    # squared errors agree to rounding of the sums they are differences of
    assert abs(sse - ref["sse"]) <= 1e-8 * ref["sse"] + 1e-13 * float(np.sum((t - t.mean()) ** 2))
    got = model_dict(m)
    np.testing.assert_array_equal(got["x_break"], ref["x_break"])
    np.testing.assert_allclose(got["beta1"], ref["beta1"], rtol=1e-7, atol=1e-12)
    np.testing.assert_allclose(got["beta0"], ref["beta0"], rtol=1e-7, atol=1e-8)
    for k, b in enumerate(got["x_break"]):     # continuous at its own boundaries
        left = got["beta1"][k] * b + got["beta0"][k]
        assert abs(left - (got["beta1"][k + 1] * b + got["beta0"][k + 1])) <= 1e-9 * abs(left)
    for q in (1, 77, 256, 900, 4096, 1e5):
        assert abs(latency_eval(m, q) - oracle_mod.selector.latency_eval(ref, q)) <= 1e-7 * abs(true_latency(q)) + 1e-9


def test_library_fit_small_and_degenerate_sets(oracle_mod):
    x = np.array([1, 2, 3, 4, 4, 1], dtype=np.float64)
    t = np.array([5, 5, 6, 9, 9, 5], dtype=np.float64)
    m, sse = latency_fit(x, t)
    ref = oracle_mod.selector.latency_fit(x, t)
    np.testing.assert_array_equal(model_dict(m)["x_break"], ref["x_break"])
    assert sse < 1e-18
    for q in (1, 2, 2.5, 3, 3.5, 4, 6):
        assert abs(latency_eval(m, q) - oracle_mod.selector.latency_eval(ref, q)) < 1e-9
    # a straight line: every pair of boundaries fits exactly, the curve is what counts
    xl = np.arange(1, 13.0)
    ml, _ = latency_fit(xl, 2.5 * xl + 4)
    np.testing.assert_allclose(model_dict(ml)["beta1"], [2.5] * 3, rtol=1e-9)
    np.testing.assert_allclose(model_dict(ml)["beta0"], [4.0] * 3, rtol=1e-8)


def test_library_selection_matches_oracle(oracle_mod):
    rng = np.random.RandomState(11)
    x = sample_loads()
    m, _ = latency_fit(x, true_latency(x))
    ref = oracle_mod.selector.latency_fit(x, true_latency(x))
    cs = np.array([1, 2, 4, 8, 16, 32])
    for trial in range(40):
        n_commit = np.sort(rng.uniform(0.5, 6.0, size=len(cs)))
        b = int(rng.choice([1, 2, 3, 7, 16, 50, 128, 256, 1000]))
        i, r = select_chunk(m, b, cs, n_commit)
        j, rr = oracle_mod.selector.select_chunk(ref, b, cs, n_commit)
        np.testing.assert_allclose(r, rr, rtol=1e-8)
        order = np.sort(rr)
        if order[-1] - order[-2] > 1e-7 * order[-1]:
            assert i == j
        else:
            assert rr[i] >= order[-1] * (1 - 1e-7)
    # ties go to the first candidate
    flat, _ = latency_fit(np.arange(1, 13.0), np.full(12, 3.0))
    assert select_chunk(flat, 4, [2, 4, 8], [2.0, 2.0, 1.0])[0] == 0


def test_library_rejects_bad_input():
    x = np.arange(1, 13.0)
    for bad_x, bad_t in [(x[:5], x[:5]), ([1, 1, 2, 2, 3, 3], [1, 1, 2, 2, 3, 3]),
                         (np.r_[x[:-1], np.nan], x), (np.r_[x[:-1], -1.0], x), (x, np.r_[x[:-1], np.inf])]:
        with pytest.raises(OptimusError) as e:
            latency_fit(bad_x, bad_t)
        assert e.value.status == -1
    m, _ = latency_fit(x, 2 * x + 1)
    for kw in [dict(batch=0), dict(chunk_sizes=[0, 2]), dict(n_commit=[-1.0, 1.0]), dict(n_commit=[np.nan, 1.0])]:
        args = dict(batch=2, chunk_sizes=[1, 2], n_commit=[1.0, 1.5])
        args.update(kw)
        with pytest.raises(OptimusError) as e:
            select_chunk(m, args["batch"], args["chunk_sizes"], args["n_commit"])
        assert e.value.status == -1
    neg, _ = latency_fit(x, x - 5.0)                     # non-positive latency at small loads
    with pytest.raises(OptimusError):
        select_chunk(neg, 1, [1, 2], [1.0, 1.5])
