"""CPU tests that pin the oracle to facts fixed by the paper and by arithmetic,
none of which come from the oracle itself (nor from the GPU path).

Each test names the passage of the ABS-SGD paper it rests on.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import abs_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
F32 = np.float32


def _f32(*vals):
    return np.array(vals, dtype=np.float32)


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [Fraction(v) for v in vals]
    return out


# ---------------------------------------------------------------------------
# 1. worked example (Algorithm 1 Step 1 + update), values derived by hand
# ---------------------------------------------------------------------------

def test_worked_example_weighted_average_and_three_updates():
    gold = _read_golden("worked_example.txt")
    M_r = 32
    G0 = np.zeros(2)
    G1 = np.zeros(2)
    orc.accumulate(G0, _f32(0.5, 1.0), M_r)
    for g in (_f32(0.1, 0.2), _f32(0.3, -0.2), _f32(0.2, 0.6)):
        orc.accumulate(G1, g, M_r)
    M = [32, 96]
    # fp32 inputs 0.1, 0.3 ... are not exact decimals: tolerance is fp32 input rounding
    np.testing.assert_allclose(G0, [16.0, 32.0], rtol=1e-7)
    np.testing.assert_allclose(G1, [19.2, 19.2], rtol=1e-7)

    x = np.array([1.0, -2.0])
    v = np.zeros(2)
    for step in (1, 2, 3):
        assert orc.sync_update(x, v, [G0, G1], M, 0.1, 0.9, 0.0005)
        np.testing.assert_allclose(v, [float(f) for f in gold[f"v{step}"]], rtol=2e-7)
        np.testing.assert_allclose(x, [float(f) for f in gold[f"x{step}"]], rtol=2e-7)

    # the weighted average is NOT the plain mean of worker means here
    x = np.zeros(2)
    v = np.zeros(2)
    orc.sync_update(x, v, [G0, G1], M, 1.0, 0.0, 0.0)   # x = -Gbar
    np.testing.assert_allclose(-x, [float(f) for f in gold["gbar"]], rtol=2e-7)
    unweighted = np.array([float(f) for f in gold["unweighted"]])
    assert np.all(np.abs(-x - unweighted) > 0.05)


def test_worked_example_exact_with_dyadic_inputs():
    """Same structure with inputs that are exact in binary, so the double oracle
    must hit the rational result exactly (to 1 ulp of double)."""
    M_r = 32
    G0, G1 = np.zeros(2), np.zeros(2)
    orc.accumulate(G0, _f32(0.5, 1.0), M_r)
    for g in (_f32(0.125, 0.25), _f32(0.375, -0.25), _f32(0.25, 0.5)):
        orc.accumulate(G1, g, M_r)
    assert G0.tolist() == [16.0, 32.0]
    assert G1.tolist() == [24.0, 16.0]
    x, v = np.zeros(2), np.zeros(2)
    orc.sync_update(x, v, [G0, G1], [32, 96], 1.0, 0.0, 0.0)
    assert (-x).tolist() == [40.0 / 128.0, 48.0 / 128.0]


# ---------------------------------------------------------------------------
# 2. equal batch sizes => plain mean (weighted gradient averaging mechanism)
# ---------------------------------------------------------------------------

def test_equal_counts_reduce_to_plain_mean():
    rng = np.random.default_rng(1)
    P, N, M_r, m = 257, 5, 32, 3
    means = rng.standard_normal((N, m, P)).astype(F32)
    G = [np.zeros(P) for _ in range(N)]
    for i in range(N):
        for j in range(m):
            orc.accumulate(G[i], means[i, j], M_r)
    x, v = np.zeros(P), np.zeros(P)
    orc.sync_update(x, v, G, [m * M_r] * N, 1.0, 0.0, 0.0)
    worker_means = means.astype(np.float64).mean(axis=1)       # each worker's own mean
    np.testing.assert_allclose(-x, worker_means.mean(axis=0), rtol=0, atol=1e-14)


def test_unequal_counts_weight_by_sample_share():
    rng = np.random.default_rng(2)
    P, M_r = 64, 32
    m = [1, 2, 5]
    means = [rng.standard_normal((mi, P)).astype(F32) for mi in m]
    G = [np.zeros(P) for _ in m]
    for i, mm in enumerate(means):
        for g in mm:
            orc.accumulate(G[i], g, M_r)
    x, v = np.zeros(P), np.zeros(P)
    orc.sync_update(x, v, G, [mi * M_r for mi in m], 1.0, 0.0, 0.0)
    # sum_i (M_i / M) * (worker i's mean)
    total = sum(m)
    expect = sum((mi / total) * mm.astype(np.float64).mean(axis=0) for mi, mm in zip(m, means))
    np.testing.assert_allclose(-x, expect, rtol=0, atol=1e-14)
    plain = np.mean([mm.astype(np.float64).mean(axis=0) for mm in means], axis=0)
    assert np.max(np.abs(-x - plain)) > 1e-3


# ---------------------------------------------------------------------------
# 3. N = 1, mu = 0, wd = 0  =>  SGD with exactly one iteration of delay
#    (Algorithm 1 with G_{-1} = 0; Appendix, proof of Theorem 1, first display)
# ---------------------------------------------------------------------------

def test_single_worker_is_one_step_delayed_sgd():
    rng = np.random.default_rng(3)
    P, T, M_r, gamma = 33, 6, 32, 0.05
    g = rng.standard_normal((T, P)).astype(F32)
    x0 = rng.standard_normal(P).astype(F32)

    xs = []
    orc.run(x0, 1, T, M_r, gamma, 0.0, 0.0, lambda t, i: [g[t]],
            record=lambda t, x, v: xs.append(x.copy()))

    # independent five-line delayed SGD: x_{t+1} = x_t - gamma * gbar_{t-1}, gbar_{-1} = 0
    ref = x0.astype(np.float64)
    prev = np.zeros(P)
    for t in range(T):
        ref = ref - gamma * prev
        prev = g[t].astype(np.float64)
        np.testing.assert_allclose(xs[t], ref, rtol=0, atol=1e-14)
    # first iteration applied nothing
    np.testing.assert_array_equal(xs[0], x0.astype(np.float64))


def test_first_iteration_is_a_noop_even_with_weight_decay():
    """G_{-1} = 0 and no batch size exists for it: nothing is applied, the state
    is untouched (Algorithm 1, initialisation)."""
    x = np.array([1.0, -3.0])
    v = np.array([0.25, 0.5])
    G = [np.zeros(2), np.zeros(2)]
    assert orc.sync_update(x, v, G, [0, 0], 0.1, 0.9, 0.01) is False
    assert x.tolist() == [1.0, -3.0] and v.tolist() == [0.25, 0.5]


# ---------------------------------------------------------------------------
# 4. delay invariant: x_{t+1} does not depend on the gradients of iteration t
# ---------------------------------------------------------------------------

def test_update_ignores_current_iteration_gradients():
    rng = np.random.default_rng(4)
    P, N, T, M_r = 40, 3, 4, 32
    g = rng.standard_normal((T, N, 2, P)).astype(F32)
    x0 = rng.standard_normal(P).astype(F32)

    def run(gg):
        return orc.run(x0, N, T, M_r, 0.1, 0.9, 5e-4, lambda t, i: list(gg[t, i]))[0]

    base = run(g)
    g2 = g.copy()
    g2[T - 1] += 7.0                       # perturb only the last iteration's gradients
    np.testing.assert_array_equal(run(g2), base)
    g3 = g.copy()
    g3[T - 2] += 7.0                       # the one before is applied in the last iteration
    assert np.max(np.abs(run(g3) - base)) > 0.1


# ---------------------------------------------------------------------------
# 5. closed forms of the update recursion
# ---------------------------------------------------------------------------

def test_constant_gradient_momentum_closed_form():
    gbar, mu, gamma, steps = 0.375, 0.9, 0.1, 25
    G = [np.full(3, 32 * gbar)]
    x, v = np.array([1.0, 0.0, -1.0]), np.zeros(3)
    x_init = x.copy()
    for n in range(1, steps + 1):
        orc.sync_update(x, v, G, [32], gamma, mu, 0.0)
        v_n = gbar * (1 - mu ** n) / (1 - mu)
        x_n = x_init - gamma * gbar * (n - mu * (1 - mu ** n) / (1 - mu)) / (1 - mu)
        np.testing.assert_allclose(v, v_n, rtol=1e-13)
        np.testing.assert_allclose(x, x_n, rtol=1e-12, atol=1e-13)


def test_pure_weight_decay_closed_form():
    gamma, wd, steps = 0.1, 0.05, 12
    G = [np.zeros(2)]
    x, v = np.array([2.0, -0.5]), np.zeros(2)
    for _ in range(steps):
        orc.sync_update(x, v, G, [32], gamma, 0.0, wd)
    np.testing.assert_allclose(x, np.array([2.0, -0.5]) * (1 - gamma * wd) ** steps, rtol=1e-13)


def test_momentum_and_weight_decay_match_two_term_linear_recurrence():
    """With constant Gbar = g the pair (x, v) follows a 2x2 affine map; compare
    with that map applied through numpy matrix algebra."""
    g, gamma, mu, wd, steps = -0.2, 0.1, 0.9, 0.01, 9
    A = np.array([[1 - gamma * wd, -gamma * mu], [wd, mu]])   # acts on (x, v)
    b = np.array([-gamma * g, g])
    s = np.array([0.7, 0.0])
    G = [np.full(1, 64 * g)]
    x, v = np.array([0.7]), np.zeros(1)
    for _ in range(steps):
        s = A @ s + b
        orc.sync_update(x, v, G, [64], gamma, mu, wd)
    np.testing.assert_allclose([x[0], v[0]], s, rtol=1e-12)


# ---------------------------------------------------------------------------
# 6. regrouping invariants: Gbar is (sum of all per-sample gradients)/(samples)
# ---------------------------------------------------------------------------

def _gbar(groups, M_r_of):
    """groups[i] = list of (mean_gradient, samples) for worker i."""
    P = groups[0][0][0].size
    G, M = [], []
    for batches in groups:
        Gi, Mi = np.zeros(P), 0
        for g, m in batches:
            orc.accumulate(Gi, g, m)
            Mi += m
        G.append(Gi)
        M.append(Mi)
    x, v = np.zeros(P), np.zeros(P)
    orc.sync_update(x, v, G, M, 1.0, 0.0, 0.0)
    return -x


def test_regrouping_leaves_average_unchanged():
    rng = np.random.default_rng(6)
    P = 50
    a, b, c, d = (rng.standard_normal(P).astype(F32) for _ in range(4))
    base = _gbar([[(a, 32), (b, 32)], [(c, 32)], [(d, 64)]], None)
    # permute workers
    np.testing.assert_allclose(_gbar([[(d, 64)], [(a, 32), (b, 32)], [(c, 32)]], None), base,
                               rtol=0, atol=1e-15)
    # move a micro-batch to another worker
    np.testing.assert_allclose(_gbar([[(a, 32)], [(c, 32), (b, 32)], [(d, 64)]], None), base,
                               rtol=0, atol=1e-15)
    # split a 64-sample batch into two 32-sample batches with the same mean
    np.testing.assert_allclose(_gbar([[(a, 32), (b, 32)], [(c, 32)], [(d, 32), (d, 32)]], None),
                               base, rtol=0, atol=1e-15)
    # an idle worker changes nothing
    np.testing.assert_allclose(_gbar([[(a, 32), (b, 32)], [], [(c, 32)], [(d, 64)]], None), base,
                               rtol=0, atol=1e-15)


# ---------------------------------------------------------------------------
# 7. brute force on tiny inputs, in exact rational arithmetic, from per-sample
#    gradients (Algorithm 1 Step 2 sums PER-SAMPLE gradients)
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("seed", [0, 1, 2])
def test_brute_force_per_sample_rational(seed):
    rng = np.random.default_rng(100 + seed)
    P, N, T, M_r = 5, 3, 4, 4
    gamma, mu, wd = F32(0.1), F32(0.9), F32(5e-4)
    fg, fm, fw = Fraction(float(gamma)), Fraction(float(mu)), Fraction(float(wd))
    m = rng.integers(0 if seed == 2 else 1, 4, size=(T, N))      # seed 2 allows idle workers
    if seed == 2:
        m[1, :] = 0                                              # a whole iteration with no samples
    # per-sample gradients are multiples of 1/256 so every micro-batch mean is exact in fp32
    samples = {(t, i, j): rng.integers(-512, 513, size=(M_r, P))
               for t in range(T) for i in range(N) for j in range(int(m[t, i]))}
    x0 = (rng.integers(-1024, 1025, size=P) / 512.0).astype(F32)

    def batches(t, i):
        return [(samples[(t, i, j)].sum(axis=0) / (256.0 * M_r)).astype(F32)
                for j in range(int(m[t, i]))]

    x_o, v_o, hist = orc.run(x0, N, T, M_r, gamma, mu, wd, batches)

    # brute force: expand every sample, average them all at once, exact rationals
    x = [Fraction(float(a)) for a in x0]
    v = [Fraction(0)] * P
    for t in range(T):
        if t >= 1:
            all_samples = [samples[(t - 1, i, j)][s]
                           for i in range(N) for j in range(int(m[t - 1, i])) for s in range(M_r)]
            if all_samples:
                cnt = len(all_samples)
                for p in range(P):
                    gbar = Fraction(int(sum(int(s[p]) for s in all_samples)), 256 * cnt)
                    d = gbar + fw * x[p]
                    v[p] = fm * v[p] + d
                    x[p] = x[p] - fg * v[p]
        assert hist[t] == [int(mm) * M_r for mm in m[t]]         # batch sizes are exact integers
    np.testing.assert_allclose(x_o, [float(a) for a in x], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(v_o, [float(a) for a in v], rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------------------
# 7b. Step 2's initialisation G_t^i = 0 (Algorithm 1, Step 2, "Initialization")
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("n", [0, 1, 2, 7, 1000, 100_003])
def test_zero_clears_every_element_and_nothing_else(n):
    """Whatever the accumulator holds (NaN, infinities, old sums), every one of its
    n elements is +0.0 afterwards, the last one included; the memory on either
    side of it is untouched; n = 0 touches nothing."""
    guard = 3
    buf = np.empty(n + 2 * guard)
    buf[:] = np.nan
    buf[guard + n // 2:] = -np.inf
    buf[:guard] = [11.0, 12.0, 13.0]
    buf[guard + n:] = [21.0, 22.0, 23.0]
    G = buf[guard:guard + n]
    orc.zero(G)
    assert G.size == n
    assert np.array_equal(G.view(np.uint64), np.zeros(n, dtype=np.uint64))      # +0.0 bit patterns
    assert buf[:guard].tolist() == [11.0, 12.0, 13.0]
    assert buf[guard + n:].tolist() == [21.0, 22.0, 23.0]


def test_zero_makes_the_generation_forget_the_one_before_last():
    """Algorithm 1 re-initialises G_t^i at the start of every Step 2, so what a worker
    summed two iterations ago (the same buffer, with two generations alive) must not
    reach Step 1 when that worker sits an iteration out.  Checked against the
    definition written out with fresh arrays, not against the oracle's own loop."""
    P, N, T, M_r = 6, 2, 5, 8
    rng = np.random.default_rng(77)
    g = (rng.integers(-64, 65, size=(T, N, P)) / 32.0).astype(F32)      # exact in fp32
    m = np.array([[1, 1], [1, 1], [1, 0], [0, 1], [1, 1]])               # worker 1 idle at t=2, worker 0 at t=3
    x0 = (rng.integers(-32, 33, size=P) / 16.0).astype(F32)

    def batches(t, i):
        return [g[t, i]] * int(m[t, i])

    x_o, _, hist = orc.run(x0, N, T, M_r, 0.25, 0.0, 0.0, batches)
    x = x0.astype(np.float64)
    for t in range(1, T):                                                # plain delayed SGD on the weighted mean
        tot = int(m[t - 1].sum()) * M_r
        s = sum(float(M_r) * g[t - 1, i].astype(np.float64) for i in range(N) if m[t - 1, i])
        x = x - 0.25 * (s / tot)
    np.testing.assert_allclose(x_o, x, rtol=0, atol=1e-15)
    assert hist == [[int(a) * M_r for a in row] for row in m]


# ---------------------------------------------------------------------------
# 8. bf16 gradients widen exactly
# ---------------------------------------------------------------------------

def test_bf16_gradients_widen_exactly():
    vals = np.array([1.0, -2.5, 0.00390625, 3.0e-5, -1.0e10, 0.0], dtype=F32)
    bits = (vals.view(np.uint32) >> 16).astype(np.uint16)        # truncate: these ARE bf16 values now
    widened = (bits.astype(np.uint32) << 16).view(F32).astype(np.float64)
    G = np.zeros(vals.size)
    orc.accumulate(G, bits, 3)
    np.testing.assert_array_equal(G, 3.0 * widened)
    # 1.0 and -2.5 are representable: survive unchanged
    assert G[0] == 3.0 and G[1] == -7.5


# ---------------------------------------------------------------------------
# 9. the fixed-order fp32 restatement stays within fp32 rounding of the definition
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fp32_family_tracks_double_family(dtype):
    import abs_workloads as wl
    rng = np.random.default_rng(9)
    P, N, T, M_r = 4099, 4, 6, 32
    gamma, mu, wd = F32(0.1), F32(0.9), F32(5e-4)
    m = rng.integers(0, 4, size=(T, N))
    pool = [(rng.standard_normal(P) * 0.01).astype(F32) for _ in range(8)]
    if dtype == "bf16":
        pool = [wl.to_bf16_bits(g) for g in pool]
    x0 = (rng.standard_normal(P) * 0.05).astype(F32)

    def batches(t, i):
        return [pool[(3 * t + 5 * i + j) % 8] for j in range(int(m[t, i]))]

    x64, v64, h64 = orc.run(x0, N, T, M_r, gamma, mu, wd, batches, precision="f64")
    x32, v32, h32 = orc.run(x0, N, T, M_r, gamma, mu, wd, batches, precision="f32")
    assert h64 == h32
    assert x32.dtype == F32
    # norm-wise: a handful of fp32 roundings per step on O(0.05) values
    assert np.max(np.abs(x32 - x64)) <= 1e-6 * np.max(np.abs(x64))
    assert np.max(np.abs(v32 - v64)) <= 1e-6 * np.max(np.abs(v64))
    # and it really is a different precision
    assert np.max(np.abs(x32 - x64)) > 0


def test_fp32_family_first_batch_overwrites_stale_accumulator():
    G = np.full(4, 123.0, dtype=F32)
    g = _f32(1.0, 2.0, -3.0, 0.5)
    orc.accumulate32(G, g, 32, first=True)
    np.testing.assert_array_equal(G, _f32(32, 64, -96, 16))
    orc.accumulate32(G, g, 32, first=False)
    np.testing.assert_array_equal(G, _f32(64, 128, -192, 32))


def test_fp32_family_skips_idle_workers():
    Ga = _f32(32.0, 64.0)
    stale = _f32(1e30, -1e30)
    x, v = _f32(0, 0), _f32(0, 0)
    assert orc.sync_update32(x, v, [stale, Ga], [0, 32], 1.0, 0.0, 0.0)
    np.testing.assert_array_equal(x, _f32(-1.0, -2.0))
    assert orc.sync_update32(x, v, [stale, Ga], [0, 0], 1.0, 0.0, 0.0) is False


# ---------------------------------------------------------------------------
# 10. delayed gradient compensation (third mechanism of Section "Algorithm")
# ---------------------------------------------------------------------------

def test_compensation_worked_example():
    gold = _read_golden("worked_example.txt")
    x = np.array([0.9, -1.9])
    x_prev = np.array([1.0, -2.0])
    v = np.zeros(2)
    G = [np.array([0.5, -0.25]) * 64]
    assert orc.sync_update_dc(x, x_prev, v, G, [64], 0.1, 0.0, 0.0, 0.5)
    np.testing.assert_allclose(v, [float(f) for f in gold["dc_gtilde"]], rtol=1e-15)   # mu = wd = 0: v is Gtilde
    np.testing.assert_allclose(x, [float(f) for f in gold["dc_x_next"]], rtol=1e-15)
    np.testing.assert_array_equal(x_prev, [0.9, -1.9])                                  # now holds x_t


def test_compensation_vanishes_for_lambda_zero_and_for_equal_iterates():
    rng = np.random.default_rng(10)
    P = 31
    G = [rng.standard_normal(P) * 10, rng.standard_normal(P) * 10]
    M = [32, 64]
    x0 = rng.standard_normal(P)
    xp = rng.standard_normal(P)
    v0 = rng.standard_normal(P)
    xa, va = x0.copy(), v0.copy()
    orc.sync_update(xa, va, G, M, 0.1, 0.9, 5e-4)
    # lambda = 0: any x_prev gives the uncompensated update
    xb, vb, xpb = x0.copy(), v0.copy(), xp.copy()
    orc.sync_update_dc(xb, xpb, vb, G, M, 0.1, 0.9, 5e-4, 0.0)
    np.testing.assert_array_equal(xb, xa)
    np.testing.assert_array_equal(vb, va)
    np.testing.assert_array_equal(xpb, x0)
    # x_prev == x (first applied step): any lambda gives the uncompensated update
    xc, vc, xpc = x0.copy(), v0.copy(), x0.copy()
    orc.sync_update_dc(xc, xpc, vc, G, M, 0.1, 0.9, 5e-4, 0.5)
    np.testing.assert_array_equal(xc, xa)
    np.testing.assert_array_equal(vc, va)
    # and a non-trivial case really differs
    xd, vd, xpd = x0.copy(), v0.copy(), xp.copy()
    orc.sync_update_dc(xd, xpd, vd, G, M, 0.1, 0.9, 5e-4, 0.5)
    assert np.max(np.abs(xd - xa)) > 1e-4


def test_compensation_constant_gradient_closed_form():
    """Plain SGD with constant Gbar = g: the increments d_t = x_t - x_{t-1} obey
    d_{t+1} = -gamma*g + r*d_t with r = -gamma*lambda*g^2, a geometric series."""
    g, gamma, lam, steps = 1.5, 0.1, 0.5, 15
    r = -gamma * lam * g * g
    G = [np.full(1, 32 * g)]
    x, xp, v = np.array([2.0]), np.array([2.0]), np.zeros(1)
    for n in range(1, steps + 1):
        orc.sync_update_dc(x, xp, v, G, [32], gamma, 0.0, 0.0, lam)
        d_n = -gamma * g * (1 - r ** n) / (1 - r)
        np.testing.assert_allclose(x - xp, d_n, rtol=1e-12)
    x_n = 2.0 - gamma * g * (steps - r * (1 - r ** steps) / (1 - r)) / (1 - r)
    np.testing.assert_allclose(x, x_n, rtol=1e-12)


def test_compensation_is_elementwise():
    rng = np.random.default_rng(12)
    P = 9
    G = [rng.standard_normal(P) * 32]
    x0, xp0 = rng.standard_normal(P), rng.standard_normal(P)
    xa, xpa, va = x0.copy(), xp0.copy(), np.zeros(P)
    orc.sync_update_dc(xa, xpa, va, G, [32], 0.1, 0.9, 1e-3, 0.5)
    G2 = [G[0].copy()]
    G2[0][4] += 100.0
    xp2 = xp0.copy()
    xp2[4] -= 3.0
    xb, vb = x0.copy(), np.zeros(P)
    orc.sync_update_dc(xb, xp2, vb, G2, [32], 0.1, 0.9, 1e-3, 0.5)
    others = np.arange(P) != 4
    np.testing.assert_array_equal(xb[others], xa[others])
    assert xb[4] != xa[4]


def test_compensation_empty_step_still_advances_previous_iterate():
    x = np.array([1.0, 2.0])
    xp = np.array([0.0, 0.0])
    v = np.array([0.5, 0.5])
    assert orc.sync_update_dc(x, xp, v, [np.zeros(2)], [0], 0.1, 0.9, 0.0, 0.5) is False
    assert x.tolist() == [1.0, 2.0] and v.tolist() == [0.5, 0.5] and xp.tolist() == [1.0, 2.0]


@pytest.mark.parametrize("seed", [0, 1])
def test_compensation_brute_force_rational(seed):
    """Whole loop with compensation against exact rationals from per-sample gradients."""
    rng = np.random.default_rng(200 + seed)
    P, N, T, M_r = 4, 2, 5, 4
    gamma, mu, wd, lam = F32(0.1), F32(0.9), F32(5e-4), F32(0.5)
    fg, fm, fw, fl = (Fraction(float(t)) for t in (gamma, mu, wd, lam))
    m = rng.integers(1, 3, size=(T, N))
    samples = {(t, i, j): rng.integers(-512, 513, size=(M_r, P))
               for t in range(T) for i in range(N) for j in range(int(m[t, i]))}
    x0 = (rng.integers(-1024, 1025, size=P) / 512.0).astype(F32)

    def batches(t, i):
        return [(samples[(t, i, j)].sum(axis=0) / (256.0 * M_r)).astype(F32)
                for j in range(int(m[t, i]))]

    x_o, v_o, _ = orc.run(x0, N, T, M_r, gamma, mu, wd, batches, lam=lam)

    x = [Fraction(float(a)) for a in x0]
    xprev = list(x)
    v = [Fraction(0)] * P
    for t in range(T):
        if t >= 1:
            alls = [samples[(t - 1, i, j)][s]
                    for i in range(N) for j in range(int(m[t - 1, i])) for s in range(M_r)]
            for p in range(P):
                gbar = Fraction(int(sum(int(s[p]) for s in alls)), 256 * len(alls))
                gt = gbar + fl * gbar * gbar * (x[p] - xprev[p])
                d = gt + fw * x[p]
                v[p] = fm * v[p] + d
                xprev[p] = x[p]
                x[p] = x[p] - fg * v[p]
    np.testing.assert_allclose(x_o, [float(a) for a in x], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(v_o, [float(a) for a in v], rtol=1e-13, atol=1e-15)


def test_compensation_fp32_family_tracks_double_family():
    rng = np.random.default_rng(13)
    P, N, T, M_r = 2051, 3, 6, 32
    m = rng.integers(1, 4, size=(T, N))
    pool = [(rng.standard_normal(P) * 0.5).astype(F32) for _ in range(8)]   # large gradients: a visible correction
    x0 = (rng.standard_normal(P) * 0.05).astype(F32)

    def batches(t, i):
        return [pool[(3 * t + 5 * i + j) % 8] for j in range(int(m[t, i]))]

    args = (x0, N, T, M_r, F32(0.1), F32(0.9), F32(5e-4), batches)
    x64, v64, _ = orc.run(*args, precision="f64", lam=F32(0.5))
    x32, v32, _ = orc.run(*args, precision="f32", lam=F32(0.5))
    xb, _, _ = orc.run(*args, precision="f64")
    assert np.max(np.abs(x64 - xb)) > 1e-4                       # the compensation is active here
    assert np.max(np.abs(x32 - x64)) <= 2e-6 * np.max(np.abs(x64))
    assert np.max(np.abs(v32 - v64)) <= 2e-6 * np.max(np.abs(v64))


# The same correction with x_t - x_{t-1} read off the momentum (every applied
# update is x_t = x_{t-1} - gamma_{t-1} v_t).  Pinned against the stored-iterate
# form, which the pins above tie to Algorithm 1.

def test_compensation_from_momentum_worked_example():
    """x_t - x_{t-1} = (-0.1, +0.1), given once as stored iterates (the golden
    example) and once as gamma_prev = 0.1, v = (1, -1)."""
    gold = _read_golden("worked_example.txt")
    x = np.array([0.9, -1.9])
    v = np.array([1.0, -1.0])
    G = [np.array([0.5, -0.25]) * 64]
    assert orc.sync_update_dcm(x, v, G, [64], 0.1, 0.0, 0.0, 0.5, 0.1)
    np.testing.assert_allclose(v, [float(f) for f in gold["dc_gtilde"]], rtol=1e-15)
    np.testing.assert_allclose(x, [float(f) for f in gold["dc_x_next"]], rtol=1e-15)


def test_compensation_from_momentum_equals_stored_iterate_form():
    """Step by step with a step size that changes every iteration, an iteration
    that applies nothing in the middle, momentum and weight decay on."""
    rng = np.random.default_rng(14)
    P, N = 257, 3
    x0 = rng.standard_normal(P)
    xa, xpa, va = x0.copy(), x0.copy(), np.zeros(P)
    xb, vb = x0.copy(), np.zeros(P)
    gamma_prev = 0.0
    moved = 0.0
    for t in range(9):
        G = [rng.standard_normal(P) * 40 for _ in range(N)]
        M = [0, 0, 0] if t == 4 else [32, 64, 32 * (1 + t % 3)]
        gamma = 0.05 * (1 + t % 4)
        x_before = xa.copy()
        ra = orc.sync_update_dc(xa, xpa, va, G, M, gamma, 0.9, 5e-4, 0.5)
        rb = orc.sync_update_dcm(xb, vb, G, M, gamma, 0.9, 5e-4, 0.5, gamma_prev)
        assert ra == rb == (t != 4)
        gamma_prev = gamma if rb else 0.0
        np.testing.assert_allclose(xb, xa, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(vb, va, rtol=1e-12, atol=1e-13)
        moved = max(moved, float(np.max(np.abs(xa - x_before))))
    assert moved > 1e-2


def test_compensation_from_momentum_whole_loop_and_no_previous_update():
    rng = np.random.default_rng(15)
    P, N, T, M_r = 513, 2, 7, 32
    m = rng.integers(0, 3, size=(T, N))
    m[3] = 0                                                    # an iteration with no samples at all
    pool = [(rng.standard_normal(P) * 0.5).astype(F32) for _ in range(8)]
    x0 = (rng.standard_normal(P) * 0.05).astype(F32)

    def batches(t, i):
        return [pool[(3 * t + 5 * i + j) % 8] for j in range(int(m[t, i]))]

    args = (x0, N, T, M_r, F32(0.1), F32(0.9), F32(5e-4), batches)
    xa, va, _ = orc.run(*args, lam=F32(0.5))
    xb, vb, _ = orc.run(*args, lam=F32(0.5), lam_from_momentum=True)
    xn, _, _ = orc.run(*args)
    assert np.max(np.abs(xa - xn)) > 1e-4
    np.testing.assert_allclose(xb, xa, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(vb, va, rtol=1e-11, atol=1e-13)
    # gamma_prev = 0 (nothing applied before): the uncompensated update
    x1, v1 = x0.astype(np.float64), rng.standard_normal(P)
    x2, v2 = x1.copy(), v1.copy()
    G = [pool[0].astype(np.float64) * 32]
    orc.sync_update(x1, v1, G, [32], 0.1, 0.9, 5e-4)
    orc.sync_update_dcm(x2, v2, G, [32], 0.1, 0.9, 5e-4, 0.5, 0.0)
    np.testing.assert_array_equal(x2, x1)
    np.testing.assert_array_equal(v2, v1)
    # sum(M) == 0 touches nothing
    assert orc.sync_update_dcm(x2, v2, G, [0], 0.1, 0.9, 5e-4, 0.5, 0.1) is False
    np.testing.assert_array_equal(x2, x1)
    np.testing.assert_array_equal(v2, v1)


def test_compensation_from_momentum_fp32_family_tracks_double_family():
    rng = np.random.default_rng(16)
    P, N, T, M_r = 2051, 3, 6, 32
    m = rng.integers(1, 4, size=(T, N))
    pool = [(rng.standard_normal(P) * 0.5).astype(F32) for _ in range(8)]
    x0 = (rng.standard_normal(P) * 0.05).astype(F32)

    def batches(t, i):
        return [pool[(3 * t + 5 * i + j) % 8] for j in range(int(m[t, i]))]

    args = (x0, N, T, M_r, F32(0.1), F32(0.9), F32(5e-4), batches)
    x64, v64, _ = orc.run(*args, precision="f64", lam=F32(0.5))                      # stored-iterate form, double
    x32, v32, _ = orc.run(*args, precision="f32", lam=F32(0.5), lam_from_momentum=True)
    assert np.max(np.abs(x32 - x64)) <= 2e-6 * np.max(np.abs(x64))
    assert np.max(np.abs(v32 - v64)) <= 2e-6 * np.max(np.abs(v64))
    # one update whose step size differs from the previous one's
    g32 = [pool[1] * F32(32), pool[2] * F32(64)]
    xs, vs = x0.copy(), (pool[3] * F32(4)).astype(F32)
    xd, vd = xs.astype(np.float64), vs.astype(np.float64)
    assert orc.sync_update32_dcm(xs, vs, g32, [32, 64], F32(0.1), F32(0.9), F32(5e-4), F32(0.5), F32(0.03))
    assert orc.sync_update_dcm(xd, vd, [g.astype(np.float64) for g in g32], [32, 64], F32(0.1), F32(0.9),
                               F32(5e-4), F32(0.5), F32(0.03))
    xu, vu = x0.astype(np.float64), (pool[3] * F32(4)).astype(np.float64)
    orc.sync_update(xu, vu, [g.astype(np.float64) for g in g32], [32, 64], F32(0.1), F32(0.9), F32(5e-4))
    assert np.max(np.abs(vd - vu)) > 1e-3                        # a visible correction
    assert np.max(np.abs(vs - vd)) <= 1e-6 * np.max(np.abs(vd))
    assert np.max(np.abs(xs - xd)) <= 1e-6 * np.max(np.abs(xd))
    # idle workers are skipped, stale buffers and all
    stale = np.full(P, 1e30, dtype=F32)
    xa, va = x0.copy(), np.ones(P, dtype=F32)
    xb, vb = x0.copy(), np.ones(P, dtype=F32)
    assert orc.sync_update32_dcm(xa, va, [stale, pool[0] * F32(32)], [0, 32], 0.1, 0.9, 5e-4, 0.5, 0.1)
    assert orc.sync_update32_dcm(xb, vb, [pool[0] * F32(32)], [32], 0.1, 0.9, 5e-4, 0.5, 0.1)
    np.testing.assert_array_equal(xa, xb)
    np.testing.assert_array_equal(va, vb)


# ---------------------------------------------------------------------------
# 11. Adam behind the delayed synchronous mechanism (Section "Conclusions and
#     Future Work" names it; the recursion is the published Adam algorithm)
# ---------------------------------------------------------------------------

def test_adam_constant_gradient_closed_form():
    """With a constant gradient the bias-corrected moments are exactly g and g^2,
    so every step moves x by gamma * g / (|g| + eps)."""
    g = np.array([0.25, -3.0, 1e-3])
    gamma, b1, b2, eps = 0.01, 0.9, 0.999, 1e-8
    G = [g * 96]
    x, m, v = np.zeros(3), np.zeros(3), np.zeros(3)
    for t in range(1, 13):
        assert orc.sync_update_adam(x, m, v, G, [96], gamma, b1, b2, eps, 0.0, t)
        np.testing.assert_allclose(x, -t * gamma * g / (np.abs(g) + eps), rtol=1e-12)
        np.testing.assert_allclose(m, g * (1 - b1 ** t), rtol=1e-12)
        np.testing.assert_allclose(v, g * g * (1 - b2 ** t), rtol=1e-12)


def test_adam_matches_a_library_adam_on_delayed_averaged_gradients():
    """The same gradients fed to torch.optim.Adam (double, CPU): an independent
    implementation of the published recursion, including coupled weight decay."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(21)
    P, N, T, M_r = 37, 3, 7, 32
    gamma, b1, b2, eps, wd = 0.01, 0.9, 0.999, 1e-8, 5e-3
    m = rng.integers(0, 4, size=(T, N))
    m[2, :] = 0                                              # an iteration without samples: no Adam step
    means = {(t, i, j): (rng.standard_normal(P) * 0.1).astype(F32)
             for t in range(T) for i in range(N) for j in range(int(m[t, i]))}
    x0 = rng.standard_normal(P).astype(F32)

    x_o, (m_o, v_o), _ = orc.run(x0, N, T, M_r, gamma, 0.0, wd,
                                 lambda t, i: [means[(t, i, j)] for j in range(int(m[t, i]))],
                                 adam=(b1, b2, eps))

    p = torch.tensor(x0.astype(np.float64), requires_grad=True)
    opt = torch.optim.Adam([p], lr=gamma, betas=(b1, b2), eps=eps, weight_decay=wd)
    for t in range(1, T):                                    # iteration t applies the average of t-1
        batch = [means[(t - 1, i, j)].astype(np.float64) for i in range(N) for j in range(int(m[t - 1, i]))]
        if not batch:
            continue
        p.grad = torch.tensor(np.mean(batch, axis=0))        # equal-size batches: the sample-weighted mean
        opt.step()
    np.testing.assert_allclose(x_o, p.detach().numpy(), rtol=1e-11, atol=1e-13)
    st = opt.state[p]
    np.testing.assert_allclose(m_o, st["exp_avg"].numpy(), rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(v_o, st["exp_avg_sq"].numpy(), rtol=1e-11, atol=1e-18)


def test_adam_brute_force_high_precision():
    """Per-sample gradients expanded and the recursion evaluated in 60-digit decimals."""
    from decimal import Decimal, getcontext
    getcontext().prec = 60
    rng = np.random.default_rng(22)
    P, N, T, M_r = 3, 2, 5, 4
    gamma, b1, b2, eps, wd = F32(0.01), F32(0.9), F32(0.999), F32(1e-8), F32(1e-2)
    D = lambda t: Decimal(float(t))
    m = rng.integers(1, 3, size=(T, N))
    samples = {(t, i, j): rng.integers(-512, 513, size=(M_r, P))
               for t in range(T) for i in range(N) for j in range(int(m[t, i]))}
    x0 = (rng.integers(-1024, 1025, size=P) / 512.0).astype(F32)

    def batches(t, i):
        return [(samples[(t, i, j)].sum(axis=0) / (256.0 * M_r)).astype(F32) for j in range(int(m[t, i]))]

    x_o, (m_o, v_o), _ = orc.run(x0, N, T, M_r, gamma, 0.0, wd, batches, adam=(b1, b2, eps))
    x = [D(a) for a in x0]
    mm = [Decimal(0)] * P
    vv = [Decimal(0)] * P
    step = 0
    for t in range(1, T):
        alls = [samples[(t - 1, i, j)][s] for i in range(N) for j in range(int(m[t - 1, i])) for s in range(M_r)]
        step += 1
        for p in range(P):
            gbar = Decimal(int(sum(int(s[p]) for s in alls))) / Decimal(256 * len(alls))
            g = gbar + D(wd) * x[p]
            mm[p] = D(b1) * mm[p] + (1 - D(b1)) * g
            vv[p] = D(b2) * vv[p] + (1 - D(b2)) * g * g
            mh = mm[p] / (1 - D(b1) ** step)
            vh = vv[p] / (1 - D(b2) ** step)
            x[p] = x[p] - D(gamma) * mh / (vh.sqrt() + D(eps))
    np.testing.assert_allclose(x_o, [float(a) for a in x], rtol=1e-12)
    np.testing.assert_allclose(m_o, [float(a) for a in mm], rtol=1e-12)
    np.testing.assert_allclose(v_o, [float(a) for a in vv], rtol=1e-12)


def test_adam_is_invariant_to_gradient_scale_and_skips_empty_steps():
    rng = np.random.default_rng(23)
    P = 11
    G = [rng.standard_normal(P) * 32]
    xa, ma, va = np.zeros(P), np.zeros(P), np.zeros(P)
    xb, mb, vb = np.zeros(P), np.zeros(P), np.zeros(P)
    for t in (1, 2, 3):
        orc.sync_update_adam(xa, ma, va, G, [32], 0.01, 0.9, 0.999, 0.0, 0.0, t)
        orc.sync_update_adam(xb, mb, vb, [G[0] * 1000.0], [32], 0.01, 0.9, 0.999, 0.0, 0.0, t)
    np.testing.assert_allclose(xa, xb, rtol=1e-12)           # eps = 0: only the direction matters
    before = xa.copy()
    assert orc.sync_update_adam(xa, ma, va, G, [0], 0.01, 0.9, 0.999, 0.0, 0.0, 4) is False
    np.testing.assert_array_equal(xa, before)


def test_adam_fp32_family_tracks_double_family():
    rng = np.random.default_rng(24)
    P, N, T, M_r = 2051, 3, 8, 32
    m = rng.integers(1, 4, size=(T, N))
    pool = [(rng.standard_normal(P) * 0.01).astype(F32) for _ in range(8)]
    x0 = (rng.standard_normal(P) * 0.05).astype(F32)

    def batches(t, i):
        return [pool[(3 * t + 5 * i + j) % 8] for j in range(int(m[t, i]))]

    args = (x0, N, T, M_r, F32(0.001), 0.0, F32(1e-2), batches)
    ad = (F32(0.9), F32(0.999), F32(1e-8))
    x64, (m64, v64), _ = orc.run(*args, precision="f64", adam=ad)
    x32, (m32, v32), _ = orc.run(*args, precision="f32", adam=ad)
    assert np.max(np.abs(x32 - x64)) <= 2e-6 * np.max(np.abs(x64))
    assert np.max(np.abs(m32 - m64)) <= 2e-6 * np.max(np.abs(m64))
    assert np.max(np.abs(v32 - v64)) <= 2e-6 * np.max(np.abs(v64))
    assert np.max(np.abs(x64 - x0)) > 1e-3                     # seven updates of ~lr each


# ---------------------------------------------------------------------------
# 12. LARS behind the delayed synchronous mechanism (named with Adam in Section
#     "Conclusions and Future Work"; the recursion is the published layer-wise rule)
# ---------------------------------------------------------------------------

def test_lars_worked_example():
    gold = _read_golden("worked_example.txt")
    x, v = np.array([3.0, 4.0]), np.zeros(2)
    assert orc.sync_update_lars(x, v, [np.array([0.6, 0.8]) * 64], [64], [2], 0.5, 0.0, 0.1, 0.02)
    np.testing.assert_allclose(v, [float(f) for f in gold["lars_v"]], rtol=1e-14)
    np.testing.assert_allclose(x, [float(f) for f in gold["lars_x"]], rtol=1e-14)


def test_lars_matches_an_independent_numpy_statement():
    rng = np.random.default_rng(31)
    sizes = [7, 1, 30, 12]
    P = sum(sizes)
    G = [rng.standard_normal(P) * 32, rng.standard_normal(P) * 64, rng.standard_normal(P) * 96]
    M = [32, 64, 96]
    x0, v0 = rng.standard_normal(P), rng.standard_normal(P) * 0.01
    gamma, mu, wd, eta = 0.1, 0.9, 5e-4, 0.001
    x, v = x0.copy(), v0.copy()
    orc.sync_update_lars(x, v, G, M, sizes, gamma, mu, wd, eta)
    gbar = sum(G) / sum(M)
    off = np.cumsum([0] + sizes)
    for a, b in zip(off[:-1], off[1:]):
        wn, gn = np.linalg.norm(x0[a:b]), np.linalg.norm(gbar[a:b])
        rate = eta * wn / (gn + wd * wn)
        v_ref = mu * v0[a:b] + gamma * rate * (gbar[a:b] + wd * x0[a:b])
        np.testing.assert_allclose(v[a:b], v_ref, rtol=1e-12)
        np.testing.assert_allclose(x[a:b], x0[a:b] - v_ref, rtol=1e-12, atol=1e-15)


def test_lars_step_length_ignores_gradient_scale_and_layers_are_independent():
    rng = np.random.default_rng(32)
    sizes = [16, 16]
    G = [rng.standard_normal(32) * 32]
    x0 = rng.standard_normal(32)
    xa, va = x0.copy(), np.zeros(32)
    orc.sync_update_lars(xa, va, G, [32], sizes, 0.1, 0.0, 0.0, 0.01)
    # wd = 0: the step is gamma * eta * ||x_l|| * g_l / ||g_l||, whatever the gradient's scale
    xb, vb = x0.copy(), np.zeros(32)
    orc.sync_update_lars(xb, vb, [G[0] * 1e3], [32], sizes, 0.1, 0.0, 0.0, 0.01)
    np.testing.assert_allclose(xa, xb, rtol=1e-12)
    for sl in (slice(0, 16), slice(16, 32)):
        np.testing.assert_allclose(np.linalg.norm(va[sl]), 0.1 * 0.01 * np.linalg.norm(x0[sl]), rtol=1e-12)
    # changing layer 1's gradients leaves layer 0 alone
    G2 = [G[0].copy()]
    G2[0][16:] *= -3.0
    xc, vc = x0.copy(), np.zeros(32)
    orc.sync_update_lars(xc, vc, G2, [32], sizes, 0.1, 0.0, 0.0, 0.01)
    np.testing.assert_array_equal(xc[:16], xa[:16])
    assert np.max(np.abs(xc[16:] - xa[16:])) > 1e-4


def test_lars_degenerate_norms_and_empty_step():
    x, v = np.zeros(3), np.zeros(3)
    G = [np.array([32.0, -64.0, 0.0])]
    orc.sync_update_lars(x, v, G, [32], [3], 0.1, 0.9, 0.0, 0.01)       # ||x|| = 0: rate 1, a plain step
    np.testing.assert_allclose(x, [-0.1, 0.2, 0.0], rtol=1e-15)
    x2, v2 = np.array([1.0, 2.0]), np.array([0.5, 0.5])
    orc.sync_update_lars(x2, v2, [np.zeros(2)], [32], [2], 0.1, 0.0, 0.01, 0.5)   # ||g|| = 0: rate 1
    np.testing.assert_allclose(v2, [0.001, 0.002], rtol=1e-14)
    x3, v3 = np.array([1.0, 2.0]), np.array([0.5, 0.5])
    assert orc.sync_update_lars(x3, v3, [np.zeros(2)], [0], [2], 0.1, 0.9, 0.01, 0.5) is False
    assert x3.tolist() == [1.0, 2.0] and v3.tolist() == [0.5, 0.5]


def test_lars_one_layer_per_element_is_sign_like():
    """With one element per layer and wd = 0 the step is gamma*eta*|x| in the direction of g."""
    x0 = np.array([2.0, -3.0, 0.5])
    g = np.array([0.1, 5.0, -7.0])
    x, v = x0.copy(), np.zeros(3)
    orc.sync_update_lars(x, v, [g * 32], [32], [1, 1, 1], 0.1, 0.0, 0.0, 0.05)
    np.testing.assert_allclose(x, x0 - 0.1 * 0.05 * np.abs(x0) * np.sign(g), rtol=1e-14)
