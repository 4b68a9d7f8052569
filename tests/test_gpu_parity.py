"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.

Bars:
  * sample counts: exact integers;
  * against the fixed-order fp32 oracle: bit for bit;
  * against the double oracle (the judge of accuracy):
      - norm-wise   max|d| <= 1e-5 * max|ref|,
      - element-wise |d_i| <= 1e-5 * (magnitude of the operands that formed element i),
        which is the relative-error bar wherever no cancellation occurs.
    The naive element-wise relative error is printed for information: where
    x - lr*v cancels to ~0 it is unbounded for ANY fp32 implementation.
"""
import numpy as np
import pytest

import abs_workloads as wl
from oracle import abs_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

RTOL = 1e-5
F32 = np.float32


@pytest.fixture(scope="module")
def absgd():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2308_15164_amd as m
    m.lib()                      # fails loudly if the HIP library is missing
    return m


def _up(a):
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _bits(a):
    return np.ascontiguousarray(a, dtype=F32).view(np.uint32)


def _assert_bitexact(got, want, what):
    gb, wb = _bits(got), _bits(want)
    bad = np.nonzero(gb != wb)[0]
    assert bad.size == 0, (f"{what}: {bad.size} of {gb.size} elements differ in bits; first at {bad[0]}: "
                           f"got {got[bad[0]]!r} want {want[bad[0]]!r}")


def _assert_close64(got, ref, scale, what):
    """got fp32, ref float64, scale = per-element operand magnitude (float64)."""
    d = np.abs(got.astype(np.float64) - ref)
    assert np.max(d) <= RTOL * max(np.max(np.abs(ref)), 1e-300), f"{what}: norm-wise bar missed"
    bad = np.nonzero(d > RTOL * scale + 1e-300)[0]
    assert bad.size == 0, f"{what}: {bad.size} elements beyond 1e-5 of their operands; first {bad[0]}"
    with np.errstate(divide="ignore", invalid="ignore"):
        naive = np.where(ref != 0, d / np.abs(ref), 0.0)
    return float(np.max(naive)), int(np.count_nonzero(naive > RTOL))


def _grad(rng, P, dtype, sigma=0.01):
    g = (rng.standard_normal(P) * sigma).astype(F32)
    return wl.to_bf16_bits(g) if dtype == "bf16" else g


# ---------------------------------------------------------------------------
# abs_accumulate, call by call
# ---------------------------------------------------------------------------

SIZES = [1, 3, 4, 7, 255, 1024, 4095, 4096, 4097, 3 * 4096 + 5, 8 * 4096, 100_003, 1_048_576 + 13]


@pytest.fixture
def tuned(absgd, request):
    """Launch shapes that force multi-row tiles (whole groups + a partial group +
    a vector tail) already at small sizes."""
    blocks_per_cu, max_rows = request.param
    absgd.abs_set_launch_tuning(blocks_per_cu, max_rows)
    yield request.param
    absgd.abs_set_launch_tuning(0, 4)      # the defaults


MULTI_ROW_SIZES = [700_001, 1_048_576, 1_048_576 + 13, 2_500_007]
TUNINGS = [(1, 0), (1, 3), (2, 5)]


@pytest.mark.parametrize("tuned", TUNINGS, indirect=True)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("P", MULTI_ROW_SIZES)
def test_accumulate_multi_row_tiles(absgd, tuned, dtype, P):
    test_accumulate_matches_oracle(absgd, dtype, P)


@pytest.mark.parametrize("tuned", TUNINGS, indirect=True)
@pytest.mark.parametrize("K", [3, 9, 16, 19])
@pytest.mark.parametrize("P", MULTI_ROW_SIZES[:3])
def test_sync_update_multi_row_tiles(absgd, tuned, K, P):
    print(f"[case] sync_update multi-row K={K} P={P} tuning={tuned}", flush=True)
    _sync_case(absgd, K, P, [32 * (1 + k % 3) for k in range(K)], seed=K + P)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("P", SIZES)
def test_accumulate_matches_oracle(absgd, dtype, P):
    print(f"[case] accumulate dtype={dtype} P={P}", flush=True)
    rng = np.random.default_rng(P * 2 + (dtype == "bf16"))
    grads = [_grad(rng, P, dtype) for _ in range(3)]
    n_list = [32, 64, 7]
    acc_d = torch.full((P,), float("nan"), device="cuda")       # stale garbage before the first call
    cnt = absgd.Count(0)
    G64 = np.zeros(P)
    G32 = np.zeros(P, dtype=F32)
    M = 0
    for j, (g, n) in enumerate(zip(grads, n_list)):
        g_d = _up(g)
        absgd.abs_accumulate(acc_d, g_d, n, cnt)
        orc.accumulate(G64, g, n)
        orc.accumulate32(G32, g, n, first=(M == 0))
        M += n
        assert cnt.value == M
        got = acc_d.cpu().numpy()
        _assert_bitexact(got, G32, f"accumulate call {j}")
        gf = (g.astype(np.uint32) << 16).view(F32) if dtype == "bf16" else g
        scale = np.abs(G64) + n * np.abs(gf.astype(np.float64))
        _assert_close64(got, G64, scale, f"accumulate call {j}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shift", [1, 2, 3])
def test_accumulate_unaligned_views(absgd, dtype, shift):
    """Bases that are element-aligned but not 16-byte aligned take the
    element-wise path and must give the same bits."""
    print(f"[case] accumulate unaligned dtype={dtype} shift={shift}", flush=True)
    P = 2 * 4096 + 37
    rng = np.random.default_rng(77 + shift)
    g1, g2 = _grad(rng, P, dtype), _grad(rng, P, dtype)
    acc_buf = torch.full((P + 8,), float("nan"), device="cuda")
    acc_d = acc_buf[shift:shift + P]
    cnt = absgd.Count(0)
    G32 = np.zeros(P, dtype=F32)
    for j, g in enumerate((g1, g2)):
        pad = np.zeros(P + 8, dtype=g.dtype)
        pad[shift:shift + P] = g
        g_d = _up(pad)[shift:shift + P]
        absgd.abs_accumulate(acc_d, g_d, 32, cnt)
        orc.accumulate32(G32, g, 32, first=(j == 0))
    _assert_bitexact(acc_d.cpu().numpy(), G32, "unaligned accumulate")
    guard = acc_buf.cpu().numpy()
    assert np.all(np.isnan(guard[:shift])) and np.all(np.isnan(guard[shift + P:]))   # nothing written outside


def test_accumulate_zero_length_and_large_count(absgd):
    cnt = absgd.Count(2**40)
    acc_d = torch.zeros(4, device="cuda")
    absgd.abs_accumulate(acc_d, acc_d, 32, cnt, P=0)
    assert cnt.value == 2**40 + 32


# ---------------------------------------------------------------------------
# abs_accumulate_batch: J gradients in one pass == J calls, bit for bit
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("J", [1, 2, 3, 4, 5, 6, 7, 8, 9, 19])
def test_accumulate_batch_equals_sequential(absgd, dtype, J):
    print(f"[case] accumulate_batch dtype={dtype} J={J}", flush=True)
    P = 5 * 4096 + 1031
    rng = np.random.default_rng(1000 + J)
    grads = [_grad(rng, P, dtype) for _ in range(J)]
    ns = [int(v) for v in rng.integers(1, 200, size=J)]
    g_d = [_up(g) for g in grads]
    for start_count in (0, 64):                        # batch that starts an accumulator / continues one
        base = (rng.standard_normal(P)).astype(F32)
        acc_b = _up(base) if start_count else torch.full((P,), float("nan"), device="cuda")
        acc_s = acc_b.clone()
        cb, cs = absgd.Count(start_count), absgd.Count(start_count)
        absgd.abs_accumulate_batch(acc_b, g_d, ns, cb)
        for g, n in zip(g_d, ns):
            absgd.abs_accumulate(acc_s, g, n, cs)
        G32 = base.copy() if start_count else np.zeros(P, dtype=F32)
        G64 = G32.astype(np.float64)
        M = start_count
        for g, n in zip(grads, ns):
            orc.accumulate32(G32, g, n, first=(M == 0))
            orc.accumulate(G64, g, n)
            M += n
        assert cb.value == cs.value == M
        got = acc_b.cpu().numpy()
        _assert_bitexact(got, acc_s.cpu().numpy(), "batch vs sequential launches")
        _assert_bitexact(got, G32, "batch vs fp32 oracle")
        assert np.max(np.abs(got - G64)) <= RTOL * np.max(np.abs(G64))


@pytest.mark.parametrize("tuned", [(1, 0), (1, 3)], indirect=True)
@pytest.mark.parametrize("J", [2, 4, 8])
def test_accumulate_batch_multi_row_and_unaligned(absgd, tuned, J):
    print(f"[case] accumulate_batch multi-row J={J} tuning={tuned}", flush=True)
    P = 1_048_576 + 13
    rng = np.random.default_rng(1100 + J)
    for shift in (0, 1):
        grads = [_grad(rng, P, "bf16" if J == 4 else "f32") for _ in range(J)]
        def up(a):
            pad = np.zeros(P + 8, dtype=a.dtype)
            pad[shift:shift + P] = a
            return _up(pad)[shift:shift + P]
        acc = torch.full((P + 8,), float("nan"), device="cuda")[shift:shift + P]
        cnt = absgd.Count(0)
        absgd.abs_accumulate_batch(acc, [up(g) for g in grads], [32] * J, cnt)
        G32 = np.zeros(P, dtype=F32)
        for j, g in enumerate(grads):
            orc.accumulate32(G32, g, 32, first=(j == 0))
        _assert_bitexact(acc.cpu().numpy(), G32, f"batch J={J} shift={shift}")


def test_accumulate_batch_rejects_bad_arguments(absgd):
    acc = torch.zeros(16, device="cuda")
    g = torch.zeros(16, device="cuda")
    with pytest.raises(absgd.AbsError):
        absgd.abs_accumulate_batch(acc, [g, g], [32, 0], absgd.Count(0))       # a zero sample count
    import ctypes
    c = ctypes.c_int64(0)
    rc = absgd.lib().abs_accumulate_batch(acc.data_ptr(), (ctypes.c_void_p * 1)(g.data_ptr()), 0, 0, 16,
                                          (ctypes.c_int64 * 1)(32), ctypes.byref(c), None)
    assert rc == absgd.ABS_EINVAL and c.value == 0                              # J < 1


# ---------------------------------------------------------------------------
# abs_accumulate_jobs: Step 2 of several workers in one launch == each worker's
# gradients taken one by one by the oracle, bit for bit
# ---------------------------------------------------------------------------

def _jobs_case(absgd, P, Js, dtype, fold, seed, start_counts=None, shift=0):
    """Js[w] gradients for worker w; start_counts[w] > 0 continues an accumulator."""
    rng = np.random.default_rng(seed)
    W = len(Js)
    start_counts = [0] * W if start_counts is None else start_counts
    grads = [[_grad(rng, P, dtype) for _ in range(J)] for J in Js]
    ns = [[int(v) for v in rng.integers(1, 200, size=J)] for J in Js]
    bases = [rng.standard_normal(P).astype(F32) for _ in range(W)]

    def up(a):
        if not shift:
            return _up(a)
        pad = np.zeros(P + 8, dtype=a.dtype)
        pad[shift:shift + P] = a
        return _up(pad.view(np.int16) if a.dtype == np.uint16 else pad)[shift:shift + P]

    accs = [up(bases[w]) if start_counts[w] else up(np.full(P, np.nan, dtype=F32)) for w in range(W)]
    g_d = [[up(g) for g in gs] for gs in grads]
    counts = [absgd.Count(c) for c in start_counts]
    absgd.abs_accumulate_jobs(accs, g_d, ns, counts, fold=fold, P=P,
                              grad_dtype=absgd.ABS_BF16 if dtype == "bf16" else absgd.ABS_F32)
    for w in range(W):
        G32 = bases[w].copy() if start_counts[w] else np.zeros(P, dtype=F32)
        G64 = G32.astype(np.float64)
        M = start_counts[w]
        for g, n in zip(grads[w], ns[w]):
            orc.accumulate32(G32, g, n, first=(M == 0))
            orc.accumulate(G64, g, n)
            M += n
        assert counts[w].value == M, f"job {w}: count"
        got = accs[w].cpu().numpy()
        if Js[w] == 0 and not start_counts[w]:
            assert np.all(np.isnan(got)), f"job {w}: an idle worker's buffer was touched"
            continue
        _assert_bitexact(got, G32, f"job {w} (J={Js[w]}, fold={fold}) vs fp32 oracle")
        assert np.max(np.abs(got - G64)) <= RTOL * max(np.max(np.abs(G64)), 1e-30)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("fold", [1, 2, 3, 8])
def test_accumulate_jobs_matches_oracle(absgd, dtype, fold):
    print(f"[case] accumulate_jobs dtype={dtype} fold={fold}", flush=True)
    # adaptive batch sizes: every worker brings another number of gradients, one sits out,
    # one continues an accumulator that already holds samples
    _jobs_case(absgd, 5 * 4096 + 1031, [2, 2, 4, 8, 0, 1, 11], dtype, fold, seed=2000 + fold,
               start_counts=[0, 64, 0, 0, 0, 32, 0])


@pytest.mark.parametrize("P", [1, 3, 4, 7, 1023, 4096, 4097, 100_003])
def test_accumulate_jobs_sizes(absgd, P):
    print(f"[case] accumulate_jobs P={P}", flush=True)
    _jobs_case(absgd, P, [3, 1, 5], "f32", 2, seed=2100 + P)
    _jobs_case(absgd, P, [1, 6], "bf16", 8, seed=2200 + P)


def test_accumulate_jobs_more_jobs_than_one_launch_carries(absgd):
    print("[case] accumulate_jobs 37 workers", flush=True)
    Js = [1 + (w * 7) % 9 for w in range(37)]                  # 1..9: some need two launches at fold 8
    _jobs_case(absgd, 3 * 4096 + 5, Js, "bf16", 8, seed=2300)
    _jobs_case(absgd, 3 * 4096 + 5, Js, "f32", 1, seed=2301)
    print("[case] accumulate_jobs 64 workers (the most a call takes)", flush=True)
    _jobs_case(absgd, 4096 + 9, [(w * 5) % 4 for w in range(64)], "f32", 2, seed=2302,
               start_counts=[32 * (w % 2) for w in range(64)])


@pytest.mark.parametrize("shift", [1, 2, 3])
def test_accumulate_jobs_unaligned_views(absgd, shift):
    print(f"[case] accumulate_jobs unaligned shift={shift}", flush=True)
    _jobs_case(absgd, 2 * 4096 + 77, [2, 5, 1], "f32", 4, seed=2400 + shift, shift=shift)
    _jobs_case(absgd, 2 * 4096 + 77, [2, 5, 1], "bf16", 4, seed=2410 + shift, shift=shift)


@pytest.mark.parametrize("tuned", TUNINGS, indirect=True)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_accumulate_jobs_multi_row_tiles(absgd, tuned, dtype):
    print(f"[case] accumulate_jobs multi-row dtype={dtype} tuning={tuned}", flush=True)
    _jobs_case(absgd, 1_048_576 + 13, [1, 3, 8], dtype, 8, seed=2500)
    _jobs_case(absgd, 700_001, [2, 2], dtype, 1, seed=2501)


@pytest.mark.parametrize("policy", [(0, 0), (1, 1)], indirect=True)
def test_accumulate_jobs_cache_flavours(absgd, policy):
    print(f"[case] accumulate_jobs policy={policy}", flush=True)
    _jobs_case(absgd, 3 * 4096 + 9, [4, 1, 2], "f32", 2, seed=2600)
    _jobs_case(absgd, 3 * 4096 + 9, [4, 1, 2], "bf16", 8, seed=2601)


def test_accumulate_jobs_rejects_shared_buffers(absgd):
    acc = torch.zeros(64, device="cuda")
    g = torch.zeros(64, device="cuda")
    c = [absgd.Count(0), absgd.Count(0)]
    with pytest.raises(absgd.AbsError):                       # two jobs into overlapping accumulators
        absgd.abs_accumulate_jobs([acc[:32], acc[16:48]], [[g[:32]], [g[32:]]], [[32], [32]], c, P=32)
    with pytest.raises(absgd.AbsError):                       # a gradient that is another job's accumulator
        absgd.abs_accumulate_jobs([acc[:32], acc[32:]], [[g[:32]], [acc[:32]]], [[32], [32]], c, P=32)
    assert [x.value for x in c] == [0, 0]
    assert torch.count_nonzero(acc).item() == 0


# ---------------------------------------------------------------------------
# abs_sync_update, call by call
# ---------------------------------------------------------------------------

def _sync_case(absgd, K, P, counts, seed, lr=0.1, mu=0.9, wd=5e-4):
    rng = np.random.default_rng(seed)
    x0 = (rng.standard_normal(P) * 0.05).astype(F32)
    v0 = (rng.standard_normal(P) * 0.02).astype(F32)
    accs = [(rng.standard_normal(P) * 0.3 * max(c, 1) / 32).astype(F32) for c in counts]
    x_d, v_d = _up(x0), _up(v0)
    acc_d = [_up(a) if c > 0 else torch.full((P,), float("nan"), device="cuda")
             for a, c in zip(accs, counts)]
    applied = absgd.abs_sync_update(x_d, v_d, acc_d, counts, lr, mu, wd)
    x32, v32 = x0.copy(), v0.copy()
    ok32 = orc.sync_update32(x32, v32, accs, counts, lr, mu, wd)
    x64, v64 = x0.astype(np.float64), v0.astype(np.float64)
    # the double oracle sums every worker: idle workers hold zeros there (Step 2 initialisation)
    G64 = [a.astype(np.float64) if c > 0 else np.zeros(P) for a, c in zip(accs, counts)]
    lr32, mu32, wd32 = (float(F32(t)) for t in (lr, mu, wd))
    ok64 = orc.sync_update(x64, v64, G64, counts, lr32, mu32, wd32)
    assert applied == ok32 == ok64
    gx, gv = x_d.cpu().numpy(), v_d.cpu().numpy()
    _assert_bitexact(gx, x32, f"sync x K={K} P={P}")
    _assert_bitexact(gv, v32, f"sync v K={K} P={P}")
    if applied:
        M = float(sum(counts))
        gbar_mag = sum(np.abs(g) for g in G64) / M
        v_scale = mu32 * np.abs(v0.astype(np.float64)) + gbar_mag + wd32 * np.abs(x0.astype(np.float64))
        x_scale = np.abs(x0.astype(np.float64)) + lr32 * v_scale
        _assert_close64(gv, v64, v_scale, "sync v")
        _assert_close64(gx, x64, x_scale, "sync x")
    else:
        _assert_bitexact(gx, x0, "untouched x")
        _assert_bitexact(gv, v0, "untouched v")


@pytest.mark.parametrize("K", list(range(1, 18)) + [33, 64])
def test_sync_update_every_worker_count(absgd, K):
    print(f"[case] sync_update K={K}", flush=True)
    counts = [32 * (1 + (3 * k) % 5) for k in range(K)]
    _sync_case(absgd, K, 3 * 4096 + 1029, counts, seed=K)


@pytest.mark.parametrize("P", [1, 5, 4096, 4097, 100_003, 1_048_576])
def test_sync_update_sizes(absgd, P):
    print(f"[case] sync_update P={P}", flush=True)
    _sync_case(absgd, 4, P, [64, 64, 128, 256], seed=P)


def test_sync_update_idle_workers_and_empty_step(absgd):
    print("[case] sync_update idle workers", flush=True)
    _sync_case(absgd, 5, 9001, [0, 96, 0, 32, 0], seed=5)        # stale NaN buffers must not be read
    _sync_case(absgd, 3, 9001, [0, 0, 0], seed=6)                # first iteration: nothing applied
    _sync_case(absgd, 20, 9001, [0] * 3 + [32] * 17, seed=7)     # 17 non-empty: the run-time-K kernel


def test_sync_update_paper_rule_plain_sgd(absgd):
    print("[case] sync_update plain SGD", flush=True)
    _sync_case(absgd, 4, 50_000, [384, 192, 128, 96], seed=8, lr=0.01, mu=0.0, wd=0.0)


def test_sync_update_huge_total_count(absgd):
    print("[case] sync_update huge counts", flush=True)
    _sync_case(absgd, 2, 5000, [2**33 + 1, 2**31 + 7], seed=9)   # (float)M rounds; both sides round alike


def test_sync_update_unaligned_views(absgd):
    print("[case] sync_update unaligned", flush=True)
    P, K = 4096 + 11, 3
    rng = np.random.default_rng(11)
    x0 = (rng.standard_normal(P) * 0.05).astype(F32)
    v0 = (rng.standard_normal(P) * 0.02).astype(F32)
    accs = [(rng.standard_normal(P)).astype(F32) for _ in range(K)]

    def shifted(a, s):
        pad = np.zeros(P + 8, dtype=F32)
        pad[s:s + P] = a
        return _up(pad)[s:s + P]

    x_d, v_d = shifted(x0, 1), shifted(v0, 0)
    acc_d = [shifted(a, s) for a, s in zip(accs, (0, 3, 2))]
    absgd.abs_sync_update(x_d, v_d, acc_d, [32, 64, 32], 0.1, 0.9, 5e-4)
    x32, v32 = x0.copy(), v0.copy()
    orc.sync_update32(x32, v32, accs, [32, 64, 32], 0.1, 0.9, 5e-4)
    _assert_bitexact(x_d.cpu().numpy(), x32, "unaligned sync x")
    _assert_bitexact(v_d.cpu().numpy(), v32, "unaligned sync v")


# ---------------------------------------------------------------------------
# abs_sync_update_dc: delayed gradient compensation, call by call
# ---------------------------------------------------------------------------

def _sync_dc_case(absgd, K, P, counts, seed, lam=0.5, lr=0.1, mu=0.9, wd=5e-4, shifts=None):
    rng = np.random.default_rng(seed)
    x0 = (rng.standard_normal(P) * 0.05).astype(F32)
    xp0 = (x0 + rng.standard_normal(P).astype(F32) * F32(0.02)).astype(F32)
    v0 = (rng.standard_normal(P) * 0.02).astype(F32)
    accs = [(rng.standard_normal(P) * 20.0 * max(c, 1) / 32).astype(F32) for c in counts]   # |Gbar| ~ 1..10

    def up(a, s):
        if not s:
            return _up(a)
        pad = np.zeros(P + 8, dtype=F32)
        pad[s:s + P] = a
        return _up(pad)[s:s + P]

    sh = shifts or [0] * (K + 3)
    x_d, xp_d, v_d = up(x0, sh[0]), up(xp0, sh[1]), up(v0, sh[2])
    acc_d = [up(a, sh[3 + k]) if c > 0 else torch.full((P,), float("nan"), device="cuda")
             for k, (a, c) in enumerate(zip(accs, counts))]
    applied = absgd.abs_sync_update_dc(x_d, xp_d, v_d, acc_d, counts, lr, mu, wd, lam)
    x32, xp32, v32 = x0.copy(), xp0.copy(), v0.copy()
    ok32 = orc.sync_update32_dc(x32, xp32, v32, accs, counts, lr, mu, wd, lam)
    x64, xp64, v64 = (a.astype(np.float64) for a in (x0, xp0, v0))
    G64 = [a.astype(np.float64) if c > 0 else np.zeros(P) for a, c in zip(accs, counts)]
    f = lambda t: float(F32(t))
    ok64 = orc.sync_update_dc(x64, xp64, v64, G64, counts, f(lr), f(mu), f(wd), f(lam))
    assert applied == ok32 == ok64
    gx, gp, gv = x_d.cpu().numpy(), xp_d.cpu().numpy(), v_d.cpu().numpy()
    _assert_bitexact(gx, x32, f"dc x K={K} P={P}")
    _assert_bitexact(gv, v32, f"dc v K={K} P={P}")
    _assert_bitexact(gp, xp32, f"dc x_prev K={K} P={P}")
    _assert_bitexact(gp, x0, "x_prev takes the value x had on entry")
    if applied:
        M = float(sum(counts))
        gbar = sum(g for g in G64) / M
        gbar_mag = sum(np.abs(g) for g in G64) / M
        corr = f(lam) * gbar * gbar * np.abs(x0.astype(np.float64) - xp0.astype(np.float64))
        v_scale = f(mu) * np.abs(v0.astype(np.float64)) + gbar_mag + np.abs(corr) + f(wd) * np.abs(x0.astype(np.float64))
        # squaring Gbar doubles its relative error: allow for it in the operand scale
        v_scale = v_scale + 2 * np.abs(corr) * gbar_mag / np.maximum(np.abs(gbar), 1e-30)
        x_scale = np.abs(x0.astype(np.float64)) + f(lr) * v_scale
        _assert_close64(gv, v64, v_scale, "dc v")
        _assert_close64(gx, x64, x_scale, "dc x")
        if P >= 1000 and lam != 0:
            assert np.max(np.abs(corr)) > 1e-3 * np.max(gbar_mag)      # the correction is not negligible here
    else:
        _assert_bitexact(gx, x0, "untouched x")
        _assert_bitexact(gv, v0, "untouched v")


@pytest.mark.parametrize("K", [1, 2, 4, 7, 8, 11, 16, 17, 40])
def test_sync_update_dc_worker_counts(absgd, K):
    print(f"[case] sync_update_dc K={K}", flush=True)
    _sync_dc_case(absgd, K, 3 * 4096 + 1029, [32 * (1 + (3 * k) % 5) for k in range(K)], seed=100 + K)


@pytest.mark.parametrize("P", [1, 5, 4097, 100_003, 1_048_576 + 13])
def test_sync_update_dc_sizes(absgd, P):
    print(f"[case] sync_update_dc P={P}", flush=True)
    _sync_dc_case(absgd, 4, P, [64, 64, 128, 256], seed=200 + P % 1000)


def test_sync_update_dc_edges(absgd):
    print("[case] sync_update_dc edges", flush=True)
    _sync_dc_case(absgd, 3, 9001, [0, 0, 0], seed=301)                       # empty step: x_prev <- x, nothing else
    _sync_dc_case(absgd, 5, 9001, [0, 96, 0, 32, 0], seed=302)               # idle workers skipped
    _sync_dc_case(absgd, 4, 9001, [32] * 4, seed=303, lam=0.0)               # lambda = 0
    _sync_dc_case(absgd, 4, 50_000, [384, 192, 128, 96], seed=304, lr=0.01, mu=0.0, wd=0.0)   # the paper's plain SGD
    _sync_dc_case(absgd, 3, 4096 + 11, [32, 64, 32], seed=305, shifts=[1, 2, 0, 0, 3, 2])     # unaligned views
    _sync_dc_case(absgd, 18, 4096 + 11, [32] * 18, seed=306, shifts=[1] + [0] * 20)           # run-time K, unaligned


@pytest.mark.parametrize("tuned", TUNINGS, indirect=True)
@pytest.mark.parametrize("K", [3, 9, 16])
def test_sync_update_dc_multi_row_tiles(absgd, tuned, K):
    print(f"[case] sync_update_dc multi-row K={K} tuning={tuned}", flush=True)
    _sync_dc_case(absgd, K, 1_048_576 + 13, [32 * (1 + k % 3) for k in range(K)], seed=400 + K)


# ---------------------------------------------------------------------------
# abs_sync_update_dcm: the compensation with x_t - x_{t-1} taken from the momentum
# ---------------------------------------------------------------------------

def _sync_dcm_case(absgd, K, P, counts, seed, lam=0.5, lr=0.1, lr_prev=0.07, mu=0.9, wd=5e-4, shifts=None):
    rng = np.random.default_rng(seed)
    x0 = (rng.standard_normal(P) * 0.05).astype(F32)
    v0 = (rng.standard_normal(P) * 0.3).astype(F32)                     # x_t - x_{t-1} = -lr_prev * v0 ~ 0.02
    accs = [(rng.standard_normal(P) * 20.0 * max(c, 1) / 32).astype(F32) for c in counts]   # |Gbar| ~ 1..10

    def up(a, s):
        if not s:
            return _up(a)
        pad = np.zeros(P + 8, dtype=F32)
        pad[s:s + P] = a
        return _up(pad)[s:s + P]

    sh = shifts or [0] * (K + 2)
    x_d, v_d = up(x0, sh[0]), up(v0, sh[1])
    acc_d = [up(a, sh[2 + k]) if c > 0 else torch.full((P,), float("nan"), device="cuda")
             for k, (a, c) in enumerate(zip(accs, counts))]
    applied = absgd.abs_sync_update_dcm(x_d, v_d, acc_d, counts, lr, mu, wd, lam, lr_prev)
    x32, v32 = x0.copy(), v0.copy()
    ok32 = orc.sync_update32_dcm(x32, v32, accs, counts, lr, mu, wd, lam, lr_prev)
    f = lambda t: float(F32(t))
    # the judge: the stored-iterate form of Algorithm 1 in double, with x_{t-1} = x_t + lr_prev * v_t
    x64, v64 = x0.astype(np.float64), v0.astype(np.float64)
    xp64 = x64 + f(lr_prev) * v64
    G64 = [a.astype(np.float64) if c > 0 else np.zeros(P) for a, c in zip(accs, counts)]
    ok64 = orc.sync_update_dc(x64, xp64, v64, G64, counts, f(lr), f(mu), f(wd), f(lam))
    assert applied == ok32 == ok64
    gx, gv = x_d.cpu().numpy(), v_d.cpu().numpy()
    _assert_bitexact(gx, x32, f"dcm x K={K} P={P}")
    _assert_bitexact(gv, v32, f"dcm v K={K} P={P}")
    if applied:
        M = float(sum(counts))
        gbar = sum(g for g in G64) / M
        gbar_mag = sum(np.abs(g) for g in G64) / M
        corr = f(lam) * gbar * gbar * f(lr_prev) * np.abs(v0.astype(np.float64))
        v_scale = f(mu) * np.abs(v0.astype(np.float64)) + gbar_mag + np.abs(corr) + f(wd) * np.abs(x0.astype(np.float64))
        v_scale = v_scale + 2 * np.abs(corr) * gbar_mag / np.maximum(np.abs(gbar), 1e-30)
        x_scale = np.abs(x0.astype(np.float64)) + f(lr) * v_scale
        _assert_close64(gv, v64, v_scale, "dcm v")
        _assert_close64(gx, x64, x_scale, "dcm x")
        if P >= 1000 and lam != 0 and lr_prev != 0:
            assert np.max(np.abs(corr)) > 1e-3 * np.max(gbar_mag)
    else:
        _assert_bitexact(gx, x0, "untouched x")
        _assert_bitexact(gv, v0, "untouched v")


@pytest.mark.parametrize("K", [1, 2, 4, 7, 8, 11, 16, 17, 40])
def test_sync_update_dcm_worker_counts(absgd, K):
    print(f"[case] sync_update_dcm K={K}", flush=True)
    _sync_dcm_case(absgd, K, 3 * 4096 + 1029, [32 * (1 + (3 * k) % 5) for k in range(K)], seed=500 + K)


@pytest.mark.parametrize("P", [1, 5, 4097, 100_003, 1_048_576 + 13])
def test_sync_update_dcm_sizes(absgd, P):
    print(f"[case] sync_update_dcm P={P}", flush=True)
    _sync_dcm_case(absgd, 4, P, [64, 64, 128, 256], seed=600 + P % 1000)


def test_sync_update_dcm_edges(absgd):
    print("[case] sync_update_dcm edges", flush=True)
    _sync_dcm_case(absgd, 3, 9001, [0, 0, 0], seed=701)                      # empty step: nothing touched
    _sync_dcm_case(absgd, 5, 9001, [0, 96, 0, 32, 0], seed=702)              # idle workers skipped
    _sync_dcm_case(absgd, 4, 9001, [32] * 4, seed=703, lam=0.0)              # lambda = 0
    _sync_dcm_case(absgd, 4, 9001, [32] * 4, seed=704, lr_prev=0.0)          # no previous update
    _sync_dcm_case(absgd, 4, 50_000, [384, 192, 128, 96], seed=705, lr=0.01, lr_prev=0.01, mu=0.0, wd=0.0)
    _sync_dcm_case(absgd, 3, 4096 + 11, [32, 64, 32], seed=706, shifts=[1, 2, 0, 3, 2])      # unaligned views
    _sync_dcm_case(absgd, 18, 4096 + 11, [32] * 18, seed=707, shifts=[1] + [0] * 20)         # run-time K, unaligned


@pytest.mark.parametrize("tuned", TUNINGS, indirect=True)
@pytest.mark.parametrize("K", [3, 16])
def test_sync_update_dcm_multi_row_tiles(absgd, tuned, K):
    print(f"[case] sync_update_dcm multi-row K={K} tuning={tuned}", flush=True)
    _sync_dcm_case(absgd, K, 1_048_576 + 13, [32 * (1 + k % 3) for k in range(K)], seed=800 + K)


# ---------------------------------------------------------------------------
# abs_sync_update_adam, call by call
# ---------------------------------------------------------------------------

def _sync_adam_case(absgd, K, P, counts, seed, step=3, lr=1e-3, b1=0.9, b2=0.999, eps=1e-8, wd=1e-2, shifts=None):
    rng = np.random.default_rng(seed)
    x0 = (rng.standard_normal(P) * 0.05).astype(F32)
    m0 = (rng.standard_normal(P) * 0.01).astype(F32)
    v0 = (rng.standard_normal(P) ** 2 * 1e-4).astype(F32)
    accs = [(rng.standard_normal(P) * 0.3 * max(c, 1) / 32).astype(F32) for c in counts]

    def up(a, s):
        if not s:
            return _up(a)
        pad = np.zeros(P + 8, dtype=F32)
        pad[s:s + P] = a
        return _up(pad)[s:s + P]

    sh = shifts or [0] * (K + 3)
    x_d, m_d, v_d = up(x0, sh[0]), up(m0, sh[1]), up(v0, sh[2])
    acc_d = [up(a, sh[3 + k]) if c > 0 else torch.full((P,), float("nan"), device="cuda")
             for k, (a, c) in enumerate(zip(accs, counts))]
    applied = absgd.abs_sync_update_adam(x_d, m_d, v_d, acc_d, counts, lr, b1, b2, eps, wd, step)
    x32, m32, v32 = x0.copy(), m0.copy(), v0.copy()
    ok32 = orc.sync_update32_adam(x32, m32, v32, accs, counts, lr, b1, b2, eps, wd, step)
    x64, m64, v64 = (a.astype(np.float64) for a in (x0, m0, v0))
    G64 = [a.astype(np.float64) if c > 0 else np.zeros(P) for a, c in zip(accs, counts)]
    f = lambda t: float(F32(t))
    ok64 = orc.sync_update_adam(x64, m64, v64, G64, counts, f(lr), f(b1), f(b2), f(eps), f(wd), step)
    assert applied == ok32 == ok64
    gx, gm, gv = x_d.cpu().numpy(), m_d.cpu().numpy(), v_d.cpu().numpy()
    _assert_bitexact(gx, x32, f"adam x K={K} P={P}")
    _assert_bitexact(gm, m32, f"adam m K={K} P={P}")
    _assert_bitexact(gv, v32, f"adam v K={K} P={P}")
    if applied:
        M = float(sum(counts))
        g_mag = sum(np.abs(g) for g in G64) / M + f(wd) * np.abs(x64)
        m_scale = np.abs(m0.astype(np.float64)) + g_mag
        v_scale = np.abs(v0.astype(np.float64)) + g_mag ** 2
        _assert_close64(gm, m64, m_scale, "adam m")
        _assert_close64(gv, v64, 2 * v_scale, "adam v")
        # x moves by lr * mh / (sqrt(vh) + eps): relative errors of m and v carry over once and half
        upd = f(lr) * (np.abs(m64) + 1e-5 * m_scale) / (1 - f(b1) ** step) / (np.sqrt(v64 / (1 - f(b2) ** step)) + f(eps))
        assert np.all(np.abs(gx - x64) <= RTOL * (np.abs(x0) + 4 * upd * np.maximum(1.0, m_scale / np.maximum(np.abs(m64), 1e-30) * 1e-0)) + 1e-30)
        assert np.max(np.abs(gx - x64)) <= RTOL * np.max(np.abs(x64))
    else:
        _assert_bitexact(gx, x0, "untouched x")
        _assert_bitexact(gm, m0, "untouched m")
        _assert_bitexact(gv, v0, "untouched v")


@pytest.mark.parametrize("K", [1, 2, 4, 7, 8, 11, 16, 17, 40])
def test_sync_update_adam_worker_counts(absgd, K):
    print(f"[case] sync_update_adam K={K}", flush=True)
    _sync_adam_case(absgd, K, 3 * 4096 + 1029, [32 * (1 + (3 * k) % 5) for k in range(K)], seed=500 + K, step=1 + K % 5)


@pytest.mark.parametrize("P", [1, 5, 4097, 100_003, 1_048_576 + 13])
def test_sync_update_adam_sizes(absgd, P):
    print(f"[case] sync_update_adam P={P}", flush=True)
    _sync_adam_case(absgd, 4, P, [64, 64, 128, 256], seed=600 + P % 1000)


def test_sync_update_adam_edges(absgd):
    print("[case] sync_update_adam edges", flush=True)
    _sync_adam_case(absgd, 3, 9001, [0, 0, 0], seed=701)                               # nothing applied, nothing touched
    _sync_adam_case(absgd, 5, 9001, [0, 96, 0, 32, 0], seed=702)                       # idle workers skipped
    _sync_adam_case(absgd, 4, 9001, [32] * 4, seed=703, step=1, wd=0.0)                # first step
    _sync_adam_case(absgd, 4, 9001, [32] * 4, seed=704, step=100_000)                  # bias corrections ~ 1
    _sync_adam_case(absgd, 3, 4096 + 11, [32, 64, 32], seed=705, shifts=[1, 2, 0, 0, 3, 2])
    x = torch.zeros(8, device="cuda")
    with pytest.raises(absgd.AbsError):
        absgd.abs_sync_update_adam(x, x.clone(), x.clone(), [x.clone()], [32], 1e-3, 0.9, 0.999, 1e-8, 0.0, 0)   # step < 1
    with pytest.raises(absgd.AbsError):
        absgd.abs_sync_update_adam(x, x.clone(), x.clone(), [x.clone()], [32], 1e-3, 1.0, 0.999, 1e-8, 0.0, 1)   # beta1 = 1


@pytest.mark.parametrize("tuned", TUNINGS, indirect=True)
@pytest.mark.parametrize("K", [3, 9, 16])
def test_sync_update_adam_multi_row_tiles(absgd, tuned, K):
    print(f"[case] sync_update_adam multi-row K={K} tuning={tuned}", flush=True)
    _sync_adam_case(absgd, K, 1_048_576 + 13, [32 * (1 + k % 3) for k in range(K)], seed=800 + K)


ADAM = (0.9, 0.999, 1e-8)


@pytest.mark.parametrize("name", ["cfg1_small", "tiny_tail_bf16", "ragged_odd_f32", "ragged_odd_bf16"])
def test_trajectory_adam(absgd, name):
    """Algorithm 1's loop with Adam as the update rule, serial and overlapped, against both oracles."""
    from paper_2308_15164_amd.driver import DeviceRun
    w = wl.WORKLOADS[name]
    steps = w.steps
    x0, pool, sched = wl.initial_params(w), wl.gradient_pool(w), wl.schedule(w, steps)
    lr = 1e-3
    res = []
    for overlap in (False, True):
        print(f"[case] adam trajectory {name} overlap={overlap}", flush=True)
        run = DeviceRun(w, x0, pool, sched, overlap=overlap, adam=ADAM)
        run.lr = lr
        run.run(steps)
        res.append(run.read_state() + (run.read_second_state(), run.count_history, run.adam_step))
        run.close()
    for a, b in zip(res[0][:3], res[1][:3]):
        _assert_bitexact(b, a, "adam overlap vs serial")
    assert res[0][4] == steps - 1                                  # one-iteration delay: T - 1 updates applied
    R = len(pool)

    def batches(t, i):
        return [pool[wl.pool_index(w, t, i, j, R)] for j in range(int(sched[t, i]))]

    f = lambda t: float(F32(t))
    args = (x0, w.K, steps, w.n, f(lr), 0.0, f(w.wd), batches)
    ad = tuple(f(t) for t in ADAM)
    x32, (m32, v32), h32 = orc.run(*args, precision="f32", adam=ad)
    x64, (m64, v64), _ = orc.run(*args, precision="f64", adam=ad)
    gx, gm, gv = res[1][:3]
    assert res[1][3] == h32
    _assert_bitexact(gx, x32, f"{name} adam x")
    _assert_bitexact(gm, m32, f"{name} adam m")
    _assert_bitexact(gv, v32, f"{name} adam v")
    for got, ref, what in ((gm, m64, "m"), (gv, v64, "v")):
        assert np.max(np.abs(got - ref)) <= RTOL * np.max(np.abs(ref)), what
    # x: Adam's step lr * mh / sqrt(vh) is scale-free in the gradient, so where the K-way sum
    # cancels to nearly zero its fp32 rounding is amplified to a visible fraction of lr per
    # step -- for any fp32 implementation, the fp32 oracle included.  Bar: all but 0.1 % of
    # the elements within 1e-5 of (|x| + the distance travelled), none further than 5 % of it.
    dx = np.abs(gx - x64)
    travelled = steps * lr
    assert np.mean(dx > RTOL * (np.abs(x64) + travelled)) < 1e-3
    assert np.max(dx) <= 0.05 * travelled
    print(f"[info] {name} adam: max|dx| = {np.max(dx):.2e} over a distance of {travelled:.1e}; "
          f"{np.mean(dx > RTOL * np.abs(x64)):.2e} of the elements beyond 1e-5 relative", flush=True)


# ---------------------------------------------------------------------------
# both memory flavours of every kernel (cached / streaming) at sizes with tails: the
# size-based choice only reaches the streaming flavour above 40 M parameters
# ---------------------------------------------------------------------------

@pytest.fixture
def policy(absgd, request):
    absgd.abs_set_cache_policy(*request.param)
    yield request.param
    absgd.abs_set_cache_policy(-1, -1)


@pytest.mark.parametrize("policy", [(0, 0), (1, 1), (1, 0), (0, 1)], indirect=True)
def test_cache_flavours_give_the_same_bits(absgd, policy):
    print(f"[case] cache policy {policy}", flush=True)
    for dtype in ("f32", "bf16"):
        test_accumulate_matches_oracle(absgd, dtype, 3 * 4096 + 1029)
        test_accumulate_batch_equals_sequential(absgd, dtype, 5)
    _sync_case(absgd, 4, 100_003, [64, 64, 128, 256], seed=1401)
    _sync_case(absgd, 18, 4096 + 11, [32] * 18, seed=1402)
    _sync_dc_case(absgd, 3, 100_003, [32, 64, 32], seed=1403)
    _sync_dcm_case(absgd, 3, 100_003, [32, 64, 32], seed=1404)
    _sync_adam_case(absgd, 3, 100_003, [32, 64, 32], seed=1405)
    _ragged_case(absgd, [4096 + 11, 8192, 4095, 2], [32, 64, 32], seed=1406, dtype="bf16", misalign=True)
    _lars_case(absgd, [4096 * 3 + 5, 1, 700], [32, 64], seed=1407)
    _trajectory_case(absgd, "tiny_tail_bf16", lam=0.5)


# ---------------------------------------------------------------------------
# the ragged (_mt) entry points, call by call: every tensor a separate allocation
# ---------------------------------------------------------------------------

def _ragged_case(absgd, sizes, counts, seed, dtype="f32", misalign=False):
    """accumulate_mt (overwrite, then on top), accumulate_batch_mt, and every update rule
    with a fixed-order fp32 restatement over one layout; the oracle sees the concatenation."""
    rng = np.random.default_rng(seed)
    P, K, T = int(sum(sizes)), len(counts), len(sizes)
    off = wl.tensor_offsets(sizes)
    print(f"[case] ragged T={T} P={P} K={K} {dtype} misalign={misalign}", flush=True)

    def split(a, fill=None):
        """One allocation per tensor; misalign: start one element into a larger buffer."""
        out = []
        for t in range(T):
            part = np.ascontiguousarray(a[off[t]:off[t + 1]])
            if misalign and t % 2 == 0:
                pad = np.zeros(part.size + 3, dtype=part.dtype)
                pad[1:1 + part.size] = part
                out.append(_up(pad)[1:1 + part.size])
            else:
                out.append(_up(part))
        return out

    cat = lambda ts: np.concatenate([t.cpu().numpy() for t in ts]) if P else np.zeros(0, dtype=F32)
    lay = absgd.Layout(sizes)
    gdt = absgd.ABS_BF16 if dtype == "bf16" else absgd.ABS_F32
    grads = [_grad(rng, P, dtype) for _ in range(4)]
    gsets = [absgd.TensorSet(lay, split(g), dtype=gdt) for g in grads]

    # Step 2 into NaN-filled accumulators: overwrite, one on top, then a batch of two
    acc_t = split(np.full(P, np.nan, dtype=F32))
    aset = absgd.TensorSet(lay, acc_t)
    cnt = absgd.Count(0)
    absgd.abs_accumulate_mt(lay, aset, gsets[0], 32, cnt)
    absgd.abs_accumulate_mt(lay, aset, gsets[1], 64, cnt)
    absgd.abs_accumulate_batch_mt(lay, aset, [gsets[2], gsets[3]], [32, 16], cnt)
    assert cnt.value == 144
    want = np.zeros(P, dtype=F32)
    orc.accumulate32(want, grads[0], 32, first=True)
    for g, n in ((grads[1], 64), (grads[2], 32), (grads[3], 16)):
        orc.accumulate32(want, g, n, first=False)
    _assert_bitexact(cat(acc_t), want, "accumulate_mt + accumulate_batch_mt")

    # Step 2 of several workers as one job list: a fresh accumulator, a worker that sits the
    # call out, and the accumulator from above carried on; at most two gradients per launch
    acc2_t, idle_t = split(np.full(P, np.nan, dtype=F32)), split(np.full(P, np.nan, dtype=F32))
    aset2, iset = absgd.TensorSet(lay, acc2_t), absgd.TensorSet(lay, idle_t)
    c2, ci = absgd.Count(0), absgd.Count(0)
    absgd.abs_accumulate_jobs_mt(lay, [aset2, iset, aset], [[gsets[0], gsets[1], gsets[2]], [], [gsets[3], gsets[0]]],
                                 [[32, 8, 16], [], [64, 32]], [c2, ci, cnt], fold=2)
    assert (c2.value, ci.value, cnt.value) == (56, 0, 240)
    want2 = np.zeros(P, dtype=F32)
    for j, (g, n) in enumerate(((grads[0], 32), (grads[1], 8), (grads[2], 16))):
        orc.accumulate32(want2, g, n, first=(j == 0))
    for g, n in ((grads[3], 64), (grads[0], 32)):
        orc.accumulate32(want, g, n, first=False)
    _assert_bitexact(cat(acc2_t), want2, "accumulate_jobs_mt, fresh accumulator")
    _assert_bitexact(cat(acc_t), want, "accumulate_jobs_mt, accumulator carried on")
    if P:
        assert np.all(np.isnan(cat(idle_t))), "accumulate_jobs_mt touched an idle worker's buffers"

    # Step 1 + update, every rule
    x0 = (rng.standard_normal(P) * 0.05).astype(F32)
    v0 = (rng.standard_normal(P) * 0.3).astype(F32)
    p0 = (x0 + rng.standard_normal(P).astype(F32) * F32(0.02)).astype(F32)
    q0 = np.abs(rng.standard_normal(P) * 1e-4).astype(F32)
    accs = [(rng.standard_normal(P) * 20.0 * max(c, 1) / 32).astype(F32) for c in counts]
    asets = [absgd.TensorSet(lay, split(a) if c > 0 else split(np.full(P, np.nan, dtype=F32)))
             for a, c in zip(accs, counts)]

    def state(*arrays):
        ts = [split(a) for a in arrays]
        return ts, [absgd.TensorSet(lay, t) for t in ts]

    (xt, vt), (xs, vs) = state(x0, v0)
    ok = absgd.abs_sync_update_mt(lay, xs, vs, asets, counts, 0.1, 0.9, 5e-4)
    xw, vw = x0.copy(), v0.copy()
    assert ok == orc.sync_update32(xw, vw, accs, counts, 0.1, 0.9, 5e-4)
    _assert_bitexact(cat(xt), xw, "sync_update_mt x")
    _assert_bitexact(cat(vt), vw, "sync_update_mt v")

    (xt, pt, vt), (xs, ps, vs) = state(x0, p0, v0)
    ok = absgd.abs_sync_update_dc_mt(lay, xs, ps, vs, asets, counts, 0.1, 0.9, 5e-4, 0.5)
    xw, pw, vw = x0.copy(), p0.copy(), v0.copy()
    assert ok == orc.sync_update32_dc(xw, pw, vw, accs, counts, 0.1, 0.9, 5e-4, 0.5)
    _assert_bitexact(cat(xt), xw, "sync_update_dc_mt x")
    _assert_bitexact(cat(vt), vw, "sync_update_dc_mt v")
    _assert_bitexact(cat(pt), pw, "sync_update_dc_mt x_prev")

    (xt, vt), (xs, vs) = state(x0, v0)
    ok = absgd.abs_sync_update_dcm_mt(lay, xs, vs, asets, counts, 0.1, 0.9, 5e-4, 0.5, 0.07)
    xw, vw = x0.copy(), v0.copy()
    assert ok == orc.sync_update32_dcm(xw, vw, accs, counts, 0.1, 0.9, 5e-4, 0.5, 0.07)
    _assert_bitexact(cat(xt), xw, "sync_update_dcm_mt x")
    _assert_bitexact(cat(vt), vw, "sync_update_dcm_mt v")

    (xt, mt, qt), (xs, ms, qs) = state(x0, v0, q0)
    ok = absgd.abs_sync_update_adam_mt(lay, xs, ms, qs, asets, counts, 1e-3, 0.9, 0.999, 1e-8, 1e-2, 2)
    xw, mw, qw = x0.copy(), v0.copy(), q0.copy()
    assert ok == orc.sync_update32_adam(xw, mw, qw, accs, counts, 1e-3, 0.9, 0.999, 1e-8, 1e-2, 2)
    _assert_bitexact(cat(xt), xw, "sync_update_adam_mt x")
    _assert_bitexact(cat(mt), mw, "sync_update_adam_mt m")
    _assert_bitexact(cat(qt), qw, "sync_update_adam_mt v")


@pytest.mark.parametrize("K", [1, 2, 5, 16, 17, 40])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_calls_worker_counts(absgd, K, dtype):
    _ragged_case(absgd, [4096 * 3 + 5, 1, 700, 65_537, 12], [32 * (1 + k % 3) for k in range(K)], seed=1100 + K,
                 dtype=dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_calls_layouts_and_edges(absgd, dtype):
    _ragged_case(absgd, [5, 0, 9000, 3], [32, 32], seed=1201, dtype=dtype)                           # an empty tensor
    _ragged_case(absgd, [1], [32], seed=1202, dtype=dtype)                                           # one element
    _ragged_case(absgd, [300, 5000, 70], [0, 64, 0, 32], seed=1203, dtype=dtype)                     # idle workers
    _ragged_case(absgd, [300, 5000, 70], [0, 0, 0], seed=1204, dtype=dtype)                          # nothing to apply
    _ragged_case(absgd, [4096 + 11, 8192, 4095, 2], [32, 64, 32], seed=1205, dtype=dtype, misalign=True)
    _ragged_case(absgd, [4096 + 11, 8192, 4095, 2], [32] * 18, seed=1206, dtype=dtype, misalign=True)   # run-time K
    _ragged_case(absgd, list(wl.WORKLOADS["ragged_odd_f32"].tensor_sizes), [32, 96, 64], seed=1207, dtype=dtype)
    many = [int(v) for v in np.random.default_rng(1208).integers(0, 40, size=2000)]                     # 2,000 tiny tensors
    _ragged_case(absgd, many, [32, 64], seed=1208, dtype=dtype)


def test_ragged_calls_reject_mismatched_arguments(absgd):
    """Argument errors are reported before anything is launched; the state is untouched."""
    print("[case] ragged argument errors", flush=True)
    sizes = [300, 5000, 70]
    lay, other = absgd.Layout(sizes), absgd.Layout([300, 5000, 71])
    mk = lambda n=None, dt=torch.float32: [torch.ones(s if n is None else n[i], device="cuda", dtype=dt)
                                           for i, s in enumerate(sizes)]
    xt, vt, at, gt = mk(), mk(), mk(), mk()
    xs, vs, a, g = (absgd.TensorSet(lay, t) for t in (xt, vt, at, gt))
    foreign = absgd.TensorSet(other, mk(n=[300, 5000, 71]))
    half = absgd.TensorSet(lay, mk(dt=torch.bfloat16))
    cnt = absgd.Count(0)
    with pytest.raises(absgd.AbsError):
        absgd.abs_accumulate_mt(lay, a, foreign, 32, cnt)              # gradient set of another layout
    with pytest.raises(absgd.AbsError):
        absgd.abs_accumulate_mt(lay, half, g, 32, cnt)                 # accumulators are fp32
    with pytest.raises(absgd.AbsError):
        absgd.abs_accumulate_mt(lay, a, g, 0, cnt)                     # a batch has samples
    with pytest.raises(absgd.AbsError):
        absgd.abs_accumulate_batch_mt(lay, a, [g, half], [32, 32], cnt)   # one element type per batch
    assert cnt.value == 0
    with pytest.raises(absgd.AbsError):
        absgd.abs_sync_update_mt(lay, xs, xs, [a], [32], 0.1, 0.9, 0.0)       # params and momentum alias
    with pytest.raises(absgd.AbsError):
        absgd.abs_sync_update_mt(lay, xs, vs, [foreign], [32], 0.1, 0.9, 0.0)
    with pytest.raises(absgd.AbsError):
        absgd.abs_sync_update_mt(lay, xs, vs, [a], [-1], 0.1, 0.9, 0.0)
    with pytest.raises(absgd.AbsError):
        absgd.abs_sync_update_dc_mt(lay, xs, xs, vs, [a], [32], 0.1, 0.9, 0.0, 0.5)   # x_prev aliases x
    with pytest.raises(absgd.AbsError):
        absgd.abs_sync_update_adam_mt(lay, xs, vs, g, [a], [32], 1e-3, 0.9, 0.999, 1e-8, 0.0, 0)   # step >= 1
    with pytest.raises(absgd.AbsError):
        absgd.abs_sync_update_lars_mt(lay, xs, vs, vs, [a], [32], 0.1, 0.9, 0.0, 0.001)   # workspace aliases v
    torch.cuda.synchronize()
    for t in xt + vt + at + gt:
        assert bool((t == 1).all())


@pytest.mark.parametrize("tuned", TUNINGS, indirect=True)
def test_ragged_calls_multi_row_tiles(absgd, tuned):
    _ragged_case(absgd, [1_048_576 + 13, 300_007, 5], [32, 64, 32, 32, 96], seed=1300, dtype="bf16")


# ---------------------------------------------------------------------------
# abs_sync_update_lars_mt: per-tensor norms + update.  Double oracle only (the norm
# reductions have no fixed-order fp32 restatement); results must not depend on timing.
# ---------------------------------------------------------------------------

def _lars_case(absgd, sizes, counts, seed, lr=0.1, mu=0.9, wd=5e-4, eta=0.001, zero_tensor=None):
    rng = np.random.default_rng(seed)
    P, K = int(sum(sizes)), len(counts)
    off = wl.tensor_offsets(sizes)
    x0 = (rng.standard_normal(P) * 0.05).astype(F32)
    v0 = (rng.standard_normal(P) * 0.001).astype(F32)
    accs = [(rng.standard_normal(P) * 0.3 * max(c, 1) / 32).astype(F32) for c in counts]
    if zero_tensor is not None:                        # a layer whose parameters are all zero: rate 1
        x0[off[zero_tensor]:off[zero_tensor + 1]] = 0

    def split(a):
        return [_up(np.ascontiguousarray(a[off[t]:off[t + 1]])) for t in range(len(sizes))]

    lay = absgd.Layout(sizes)
    outs = []
    for rep in range(2):
        xt, vt = split(x0), split(v0)
        gt = [torch.full_like(t, float("nan")) for t in xt]
        at = [split(a) if c > 0 else [torch.full_like(t, float("nan")) for t in xt] for a, c in zip(accs, counts)]
        xs, vs, gs = absgd.TensorSet(lay, xt), absgd.TensorSet(lay, vt), absgd.TensorSet(lay, gt)
        asets = [absgd.TensorSet(lay, a) for a in at]
        applied = absgd.abs_sync_update_lars_mt(lay, xs, vs, gs, asets, counts, lr, mu, wd, eta)
        torch.cuda.synchronize()
        cat = lambda ts: np.concatenate([t.cpu().numpy() for t in ts]) if ts else np.zeros(0, dtype=F32)
        outs.append((cat(xt), cat(vt), cat(gt)))
    _assert_bitexact(outs[1][0], outs[0][0], "LARS x, second run")         # fixed reduction order
    _assert_bitexact(outs[1][1], outs[0][1], "LARS v, second run")
    gx, gv, gg = outs[0]
    x64, v64 = x0.astype(np.float64), v0.astype(np.float64)
    G64 = [a.astype(np.float64) if c > 0 else np.zeros(P) for a, c in zip(accs, counts)]
    f = lambda t: float(F32(t))
    ok = orc.sync_update_lars(x64, v64, G64, counts, sizes, f(lr), f(mu), f(wd), f(eta))
    assert applied == ok
    if not ok:
        _assert_bitexact(gx, x0, "untouched x")
        _assert_bitexact(gv, v0, "untouched v")
        return
    M = float(sum(counts))
    gbar = sum(G64) / M
    gmag = sum(np.abs(g) for g in G64) / M
    assert np.max(np.abs(gg - gbar)) <= RTOL * np.max(gmag)                # the workspace holds Gbar
    step = np.abs(v64 - f(mu) * v0.astype(np.float64))                     # |lr*rate*(g + wd x)| per element
    rel = step / np.maximum(np.abs(gbar + f(wd) * x0), 1e-300)             # lr*rate of the element's layer
    v_scale = f(mu) * np.abs(v0.astype(np.float64)) + rel * (gmag + f(wd) * np.abs(x0))
    x_scale = np.abs(x0.astype(np.float64)) + v_scale
    _assert_close64(gv, v64, v_scale, "LARS v")
    _assert_close64(gx, x64, x_scale, "LARS x")


@pytest.mark.parametrize("K", [1, 3, 4, 5, 8, 16, 17])
def test_lars_worker_counts(absgd, K):
    print(f"[case] lars K={K}", flush=True)
    _lars_case(absgd, [4096 * 3 + 5, 1, 700, 65_537, 12], [32 * (1 + k % 3) for k in range(K)], seed=900 + K)


def test_lars_layouts_and_edges(absgd):
    print("[case] lars layouts", flush=True)
    _lars_case(absgd, [1_048_576 + 13], [64, 32], seed=921)                               # one layer = a flat vector
    _lars_case(absgd, list(wl.WORKLOADS["ragged_odd_f32"].tensor_sizes), [32, 96, 64], seed=922)
    _lars_case(absgd, [5, 0, 9000, 3], [32, 32], seed=923)                                # an empty tensor
    _lars_case(absgd, [300, 5000, 70], [0, 64, 0, 32], seed=924)                          # idle workers (NaN buffers)
    _lars_case(absgd, [300, 5000, 70], [0, 0], seed=925)                                  # nothing to apply
    _lars_case(absgd, [300, 5000, 70], [32, 32], seed=926, zero_tensor=1)                 # ||x_l|| = 0: rate 1
    _lars_case(absgd, [300, 5000], [32, 32], seed=927, mu=0.0, wd=0.0, eta=0.02)


@pytest.mark.parametrize("tuned", [(1, 0), (1, 3)], indirect=True)
def test_lars_multi_row_tiles(absgd, tuned):
    print(f"[case] lars multi-row tuning={tuned}", flush=True)
    _lars_case(absgd, [1_048_576 + 13, 300_007, 5], [32, 64, 32], seed=930)


@pytest.mark.parametrize("name", ["ragged_odd_f32", "ragged_odd_bf16"])
def test_trajectory_lars(absgd, name):
    from paper_2308_15164_amd.driver import DeviceRun
    w = wl.WORKLOADS[name]
    steps, eta = w.steps, 0.02
    x0, pool, sched = wl.initial_params(w), wl.gradient_pool(w), wl.schedule(w, steps)
    res = []
    for overlap in (False, True):
        print(f"[case] lars trajectory {name} overlap={overlap}", flush=True)
        run = DeviceRun(w, x0, pool, sched, overlap=overlap, lars=eta)
        run.run(steps)
        res.append(run.read_state() + (run.count_history,))
        run.close()
    _assert_bitexact(res[1][0], res[0][0], "lars overlap vs serial x")
    _assert_bitexact(res[1][1], res[0][1], "lars overlap vs serial v")
    R = len(pool)

    def batches(t, i):
        return [pool[wl.pool_index(w, t, i, j, R)] for j in range(int(sched[t, i]))]

    f = lambda t: float(F32(t))
    x64, v64, h = orc.run(x0, w.K, steps, w.n, f(w.lr), f(w.mu), f(w.wd), batches,
                          lars=(list(w.tensor_sizes), f(eta)))
    assert res[1][2] == h
    gx, gv = res[1][:2]
    # norm-wise and element by element, each element against the magnitude of the operands that
    # formed it over the run (v: its own size plus one typical step of its layer; x: where it
    # started and what was subtracted from it)
    off = wl.tensor_offsets(w.tensor_sizes)
    rms = np.concatenate([np.full(off[t + 1] - off[t], np.sqrt(np.mean(x64[off[t]:off[t + 1]] ** 2)))
                          for t in range(len(w.tensor_sizes))])
    typical_step = w.lr * eta * rms                    # lr * rate_l * |g| is of this size in layer l
    scale_v = np.abs(v64) + typical_step
    scale_x = np.abs(x0.astype(np.float64)) + np.abs(x64) + steps * scale_v
    _assert_close64(gx, x64, scale_x, f"{name} lars x vs double oracle")
    _assert_close64(gv, v64, scale_v, f"{name} lars v vs double oracle")
    assert np.max(np.abs(x64 - x0)) > 1e-5                                                # it moved


# ---------------------------------------------------------------------------
# whole trajectories through the double-buffered context (Algorithm 1 loop)
# ---------------------------------------------------------------------------

def _oracle_trajectory(w, x0, pool, sched, steps, precision, R=None, lam=None, lam_from_momentum=False):
    R = len(pool) if R is None else R

    def batches(t, i):
        return [pool[wl.pool_index(w, t, i, j, R)] for j in range(int(sched[t, i]))]

    return orc.run(x0, w.K, steps, w.n, float(F32(w.lr)), float(F32(w.mu)), float(F32(w.wd)), batches,
                   precision=precision, lam=None if lam is None else float(F32(lam)),
                   lam_from_momentum=lam_from_momentum)


def _trajectory_case(absgd, name, steps=None, P=None, lam=None, batched=False, lam_from_momentum=False,
                     step_fold=None):
    from paper_2308_15164_amd.driver import DeviceRun
    w = wl.WORKLOADS[name]
    steps = w.steps if steps is None else steps
    size = w.P if P is None else P
    x0 = wl.initial_params(w, size)
    pool = wl.gradient_pool(w, size)
    sched = wl.schedule(w, steps)
    out = {}
    for overlap in (False, True):
        print(f"[case] trajectory {name} overlap={overlap}", flush=True)
        run = DeviceRun(w, x0, pool, sched, overlap=overlap, P=size, lam=lam, batched=batched,
                        lam_from_momentum=lam_from_momentum, step_fold=step_fold)
        run.run(steps)
        out[overlap] = run.read_state() + (run.count_history, run.applied)
        run.close()
        del run
        torch.cuda.empty_cache()
    (xs, vs, cs, aps), (xo, vo, co, apo) = out[False], out[True]
    # serial == overlapped, bit for bit: the double buffer has no race
    _assert_bitexact(xo, xs, "overlap vs serial x")
    _assert_bitexact(vo, vs, "overlap vs serial v")
    assert cs == co and aps == apo
    assert aps == [False] + [True] * (steps - 1)       # one-iteration delay: step 0 applies nothing

    x32, v32, h32 = _oracle_trajectory(w, x0, pool, sched, steps, "f32", lam=lam,
                                       lam_from_momentum=lam_from_momentum)
    # the judge is always Algorithm 1 as printed (x_{t-1} stored), in double
    x64, v64, h64 = _oracle_trajectory(w, x0, pool, sched, steps, "f64", lam=lam)
    assert cs == h32 == h64                            # sample counts: exact
    _assert_bitexact(xo, x32, f"{name} x vs fp32 oracle")
    _assert_bitexact(vo, v32, f"{name} v vs fp32 oracle")
    scale_x = np.abs(x0.astype(np.float64)) + np.abs(x64) + w.lr * np.abs(v64) * steps
    scale_v = np.abs(v64) + 10 * w.sigma_g
    nx = _assert_close64(xo, x64, scale_x, f"{name} x vs double oracle")
    nv = _assert_close64(vo, v64, scale_v, f"{name} v vs double oracle")
    print(f"[info] {name}: naive max rel err x={nx[0]:.3e} ({nx[1]} elems > 1e-5), "
          f"v={nv[0]:.3e} ({nv[1]} elems > 1e-5)", flush=True)


def test_trajectory_cfg1(absgd):
    _trajectory_case(absgd, "cfg1_small")


@pytest.mark.parametrize("tuned", [(1, 0), (1, 2)], indirect=True)
@pytest.mark.parametrize("name", ["cfg1_small", "ragged_odd_bf16"])
def test_trajectory_multi_row_tiles(absgd, tuned, name):
    _trajectory_case(absgd, name)


def test_trajectory_worker_streams(absgd):
    """The K workers' accumulations spread over several streams give the same bits."""
    from paper_2308_15164_amd.driver import DeviceRun
    w = wl.WORKLOADS["cfg1_small"]
    x0, pool, sched = wl.initial_params(w), wl.gradient_pool(w), wl.schedule(w)
    res = []
    for n_streams in (1, 2, 4):
        print(f"[case] worker streams n={n_streams}", flush=True)
        run = DeviceRun(w, x0, pool, sched, overlap=True, acc_streams=n_streams)
        run.run(w.steps)
        res.append(run.read_state() + (run.count_history,))
        run.close()
    for r in res[1:]:
        _assert_bitexact(r[0], res[0][0], "worker streams x")
        _assert_bitexact(r[1], res[0][1], "worker streams v")
        assert r[2] == res[0][2]


@pytest.mark.parametrize("name", ["tiny_tail_f32", "tiny_tail_bf16", "ragged_odd_f32", "ragged_odd_bf16"])
def test_trajectory_tails_and_ragged(absgd, name):
    _trajectory_case(absgd, name)


def test_trajectory_paper_rule(absgd):
    """The paper's own setting (plain SGD, 12:6:4:3 micro-batches) on a short vector."""
    _trajectory_case(absgd, "paper_static", steps=6, P=300_007)


@pytest.mark.parametrize("name,kw", [("paper_static", dict(steps=6, P=300_007)), ("cfg1_small", {}),
                                     ("tiny_tail_bf16", {}), ("ragged_odd_f32", {}), ("ragged_odd_bf16", dict(lam=0.5))])
def test_trajectory_batched_accumulate(absgd, name, kw):
    """One accumulate launch per worker and step; the oracle still takes the gradients one by one."""
    _trajectory_case(absgd, name, batched=True, **kw)


@pytest.mark.parametrize("fold", [1, 3, 8])
@pytest.mark.parametrize("name,kw", [("paper_static", dict(steps=6, P=300_007)), ("cfg1_small", {}),
                                     ("tiny_tail_bf16", {}), ("ragged_odd_f32", {}), ("ragged_odd_bf16", dict(lam=0.5))])
def test_trajectory_one_accumulate_call_per_step(absgd, name, kw, fold):
    """Step 2 of all K workers in one abs_ctx_accumulate_step call per iteration (a job list);
    the oracle still takes every worker's gradients one by one."""
    _trajectory_case(absgd, name, step_fold=fold, **kw)


@pytest.mark.parametrize("name,kw", [("paper_static", dict(steps=6, P=300_007)), ("cfg1_small", {}),
                                     ("tiny_tail_bf16", {}), ("ragged_odd_f32", {}), ("ragged_odd_bf16", {})])
def test_trajectory_with_compensation(absgd, name, kw):
    """Algorithm 1 complete: delayed update + weighted averaging + compensation, lambda = 0.5."""
    _trajectory_case(absgd, name, lam=0.5, **kw)


@pytest.mark.parametrize("name,kw", [("paper_static", dict(steps=6, P=300_007)), ("cfg1_small", {}),
                                     ("tiny_tail_bf16", {}), ("ragged_odd_f32", {}), ("ragged_odd_bf16", {})])
def test_trajectory_with_compensation_from_momentum(absgd, name, kw):
    """The same, with x_t - x_{t-1} read off the momentum: bit-exact against that
    order in fp32, and within the bar of Algorithm 1's stored-iterate form in double."""
    _trajectory_case(absgd, name, lam=0.5, lam_from_momentum=True, **kw)


def test_trajectory_delay_invariant_on_gpu(absgd):
    """x after step t does not depend on step t's gradients."""
    from paper_2308_15164_amd.driver import DeviceRun
    print("[case] delay invariant", flush=True)
    w = wl.WORKLOADS["tiny_tail_f32"]
    x0 = wl.initial_params(w)
    pool = wl.gradient_pool(w)
    sched = wl.schedule(w, 4)
    res = []
    for bump in (1, 5):
        s2 = sched.copy()
        s2[3] = bump                                        # only the LAST step's accumulation differs
        run = DeviceRun(w, x0, pool, s2, overlap=True)
        run.run(4)
        res.append(run.read_state())
        run.close()
    _assert_bitexact(res[0][0], res[1][0], "delay invariant x")
    _assert_bitexact(res[0][1], res[1][1], "delay invariant v")


# ---------------------------------------------------------------------------
# the full stated sizes in the benchmark's launch configuration, sampled outputs
# ---------------------------------------------------------------------------

# every element where the oracle needs only seconds for the whole vector; a sample elsewhere
FULL_VECTOR = ("cfg2_resnet18", "cfg3_resnet50_bf16")


@pytest.mark.parametrize("name,lam,batched", [("cfg2_resnet18", None, False), ("cfg3_resnet50_bf16", None, False),
                                              ("cfg4_vgg16", None, False), ("cfg5_gpt2_ragged_bf16", None, False),
                                              ("cfg2_resnet18", 0.5, False), ("cfg5_gpt2_ragged_bf16", 0.5, False),
                                              ("cfg2_resnet18", None, True), ("cfg3_resnet50_bf16", None, True),
                                              ("cfg5_gpt2_ragged_bf16", None, True),
                                              ("cfg2_resnet18", "0.5 from momentum", False),
                                              ("cfg5_gpt2_ragged_bf16", "0.5 from momentum", True),
                                              ("cfg2_resnet18", None, "step 8"), ("cfg3_resnet50_bf16", None, "step 1"),
                                              ("cfg4_vgg16", None, "step 8"), ("cfg4_vgg16", None, "step 1"),
                                              ("cfg5_gpt2_ragged_bf16", None, "step 8")])
def test_full_size(absgd, name, lam, batched):
    """The stated configurations at full size, in the launch configuration the benchmark times.
    cfg 2 and cfg 3: every element against the oracle.  cfg 4 and cfg 5: every output element
    depends only on the same index of the inputs, so the oracle runs on a sample of indices
    gathered from the very same host arrays.  batched "step f": one abs_ctx_accumulate_step call
    per iteration folding at most f gradients per worker and launch."""
    from paper_2308_15164_amd.driver import DeviceRun
    w = wl.WORKLOADS[name]
    dcm = isinstance(lam, str)                   # compensation with x_t - x_{t-1} taken from the momentum
    lam = float(lam.split()[0]) if dcm else lam
    fold = int(batched.split()[1]) if isinstance(batched, str) else None
    print(f"[case] full size {name}: generating inputs", flush=True)
    x0 = wl.initial_params(w)
    R = 4
    pool = wl.gradient_pool(w, pool=R)
    sched = wl.schedule(w)
    # the stream plan bench.py times for this workload: the step call runs on one stream; separate
    # calls on what abs_suggest_accumulate_streams names
    n_acc = 1 if fold is not None else absgd.abs_suggest_accumulate_streams(w.P, w.K)
    overlap = n_acc > 1
    print(f"[case] full size {name}: device run, overlap={overlap}, {n_acc} accumulate stream(s), fold={fold}",
          flush=True)
    run = DeviceRun(w, x0, pool, sched, overlap=overlap, acc_streams=n_acc, lam=lam,
                    batched=batched is True, lam_from_momentum=dcm, step_fold=fold)
    run.run(w.steps)
    if name in FULL_VECTOR:
        idx = None
        gx, gv = run.read_state()
    else:
        idx = wl.sample_indices(w.P, 200_000, w.seed)
        if w.tensor_sizes is not None:       # both sides of every tensor boundary
            off = wl.tensor_offsets(w.tensor_sizes)
            extra = np.concatenate([off[:-1], off[1:] - 1, np.minimum(off[:-1] + 1, w.P - 1)])
            idx = np.unique(np.concatenate([idx, extra]))
        gx, gv = run.read_state_at(idx)
    counts = run.count_history
    run.close()
    del run
    torch.cuda.empty_cache()
    print(f"[case] full size {name}: oracle on {w.P if idx is None else idx.size} elements", flush=True)
    x0s = x0 if idx is None else np.ascontiguousarray(x0[idx])
    pools = pool if idx is None else [np.ascontiguousarray(g[idx]) for g in pool]
    x32, v32, h32 = _oracle_trajectory(w, x0s, pools, sched, w.steps, "f32", R, lam=lam, lam_from_momentum=dcm)
    _assert_bitexact(gx, x32, f"{name} x vs fp32 oracle")
    _assert_bitexact(gv, v32, f"{name} v vs fp32 oracle")
    del x32, v32
    x64, v64, h64 = _oracle_trajectory(w, x0s, pools, sched, w.steps, "f64", R, lam=lam)   # Algorithm 1 as printed
    assert counts == h32 == h64
    scale_x = np.abs(x0s.astype(np.float64)) + np.abs(x64) + w.lr * np.abs(v64) * w.steps
    scale_v = np.abs(v64) + 10 * w.sigma_g
    nx = _assert_close64(gx, x64, scale_x, f"{name} x vs double oracle")
    nv = _assert_close64(gv, v64, scale_v, f"{name} v vs double oracle")
    print(f"[info] {name}: naive max rel err x={nx[0]:.3e} ({nx[1]} > 1e-5), v={nv[0]:.3e} ({nv[1]} > 1e-5)",
          flush=True)


# ---------------------------------------------------------------------------
# vectors longer than 2^31 elements: 64-bit indexing end to end
# ---------------------------------------------------------------------------

def test_more_than_2_31_elements(absgd):
    """P = 2^31 + 3 tiles + 5 elements (8.6 GB per fp32 vector).  Inputs are made on the device
    with PyTorch (an input generator, not the path under test); the oracle runs on elements
    sampled around 0, 2^31, the 2^32-byte boundaries and the tail."""
    P = 2**31 + 3 * 4096 + 5
    print(f"[case] P = {P}: allocating", flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0x15164)

    def fill_normal(t, sigma):
        step = 1 << 28
        for a in range(0, t.numel(), step):
            t[a:a + step].normal_(0.0, sigma, generator=gen)
        return t

    acc0 = torch.empty(P, device="cuda")
    acc1 = fill_normal(torch.empty(P, device="cuda"), 3.0)
    g_bf = fill_normal(torch.empty(P, device="cuda", dtype=torch.bfloat16), 0.01)
    g_f32 = fill_normal(torch.empty(P, device="cuda"), 0.01)
    x = fill_normal(torch.empty(P, device="cuda"), 0.05)
    v = torch.zeros(P, device="cuda")
    idx = np.unique(np.concatenate([
        wl.sample_indices(P, 20000, 99),
        np.arange(2**30 - 8, 2**30 + 8), np.arange(2**31 - 4100, 2**31 + 4100), np.arange(P - 9000, P)]))
    idx = idx[(idx >= 0) & (idx < P)]
    it = torch.from_numpy(idx).cuda()

    def at(t):
        h = t[it].cpu()
        return h.view(torch.int16).numpy().view(np.uint16).copy() if t.dtype == torch.bfloat16 else h.numpy().copy()

    g_bf_s, g_f32_s, x_s, acc1_s = at(g_bf), at(g_f32), at(x), at(acc1)
    torch.cuda.synchronize()
    print("[case] accumulate (overwrite with bf16, then fp32 on top)", flush=True)
    cnt = absgd.Count(0)
    absgd.abs_accumulate(acc0, g_bf, 32, cnt)
    absgd.abs_accumulate(acc0, g_f32, 64, cnt)
    assert cnt.value == 96
    print("[case] sync-update K = 2", flush=True)
    absgd.abs_sync_update(x, v, [acc0, acc1], [96, 160], 0.1, 0.9, 5e-4)
    torch.cuda.synchronize()
    G0 = np.zeros(idx.size, dtype=F32)
    orc.accumulate32(G0, g_bf_s, 32, first=True)
    orc.accumulate32(G0, g_f32_s, 64, first=False)
    _assert_bitexact(at(acc0), G0, "accumulate beyond 2^31")
    xo, vo = x_s.copy(), np.zeros(idx.size, dtype=F32)
    orc.sync_update32(xo, vo, [G0, acc1_s], [96, 160], 0.1, 0.9, 5e-4)
    _assert_bitexact(at(x), xo, "sync-update x beyond 2^31")
    _assert_bitexact(at(v), vo, "sync-update v beyond 2^31")
    # against the double oracle, norm-wise
    x64, v64 = x_s.astype(np.float64), np.zeros(idx.size)
    G64 = np.zeros(idx.size)
    orc.accumulate(G64, g_bf_s, 32)
    orc.accumulate(G64, g_f32_s, 64)
    orc.sync_update(x64, v64, [G64, acc1_s.astype(np.float64)], [96, 160], float(F32(0.1)), float(F32(0.9)), float(F32(5e-4)))
    assert np.max(np.abs(at(x) - x64)) <= RTOL * np.max(np.abs(x64))
    assert np.max(np.abs(at(v) - v64)) <= RTOL * np.max(np.abs(v64))
    del acc0, acc1, g_bf, g_f32, x, v
    torch.cuda.empty_cache()


# ---------------------------------------------------------------------------
# the paper's own setting, long run: drift of the fp32 path against the double oracle
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("name,steps,dcm", [("paper_static", 6200, False), ("paper_dynamic", 1500, False),
                                            ("paper_static_dynamic", 1500, False), ("paper_dynamic", 3000, True)])
def test_paper_setting_long_run(absgd, name, steps, dcm):
    """N = 4 workers, reference batch 32, plain SGD with lr 0.01 and compensation 0.5
    (Section "Hyper-parameters"), the three heterogeneity structures of Section
    "Experiments", full ResNet18-sized vector, the paper's 6,200 iterations for the static
    cluster.  Sampled elements against both oracles.  dcm: the compensation reads
    x_t - x_{t-1} off the momentum; the double oracle stays Algorithm 1 as printed."""
    from paper_2308_15164_amd.driver import DeviceRun
    w = wl.WORKLOADS[name]
    lam = 0.5
    print(f"[case] long run {name} steps={steps}: inputs", flush=True)
    x0 = wl.initial_params(w)
    R = 8
    pool = wl.gradient_pool(w, pool=R)
    sched = wl.schedule(w, steps)
    run = DeviceRun(w, x0, pool, sched, overlap=True, acc_streams=2, lam=lam, lam_from_momentum=dcm)
    print(f"[case] long run {name}: device", flush=True)
    for t in range(steps):
        run.step(t)
        if t % 1000 == 999:
            torch.cuda.synchronize()
            print(f"[progress] {name} step {t + 1}", flush=True)
    idx = wl.sample_indices(w.P, 6000, w.seed + 77)
    gx, gv = run.read_state_at(idx)
    counts = run.ctx.counts(1)
    run.close()
    del run
    torch.cuda.empty_cache()
    assert counts == [int(m) * w.n for m in sched[steps - 1]]
    print(f"[case] long run {name}: oracle on {idx.size} sampled elements", flush=True)
    x0s = np.ascontiguousarray(x0[idx])
    pools = [np.ascontiguousarray(g[idx]) for g in pool]
    x32, v32, _ = _oracle_trajectory(w, x0s, pools, sched, steps, "f32", R, lam=lam, lam_from_momentum=dcm)
    x64, v64, _ = _oracle_trajectory(w, x0s, pools, sched, steps, "f64", R, lam=lam)
    _assert_bitexact(gx, x32, f"{name} long run x")
    _assert_bitexact(gv, v32, f"{name} long run v")
    drift_x = np.max(np.abs(gx - x64)) / np.max(np.abs(x64))
    drift_v = np.max(np.abs(gv - v64)) / np.max(np.abs(v64))
    print(f"[info] {name}: after {steps} delayed steps max|dx|/max|x| = {drift_x:.3e}, "
          f"max|dv|/max|v| = {drift_v:.3e}", flush=True)
    # the 1e-5 bar still holds after thousands of delayed steps (rounding errors of the
    # fp32 iterate add up like a random walk, far below the linear worst case steps * 2^-24)
    assert drift_x <= 1e-5
    assert drift_v <= 1e-5


# ---------------------------------------------------------------------------
# special values: subnormals, signed zeros, the largest finite values, infinities, NaN
# ---------------------------------------------------------------------------

_SPECIALS = np.array([0.0, -0.0, 1e-45, -1e-45, 1e-40, -3e-39, 1.1754944e-38, -1.1754944e-38, 1e-30, -1e-20,
                      1.0, -1.0, 3.0, 1e20, -1e30, 3.4028235e38, -3.4028235e38, np.inf, -np.inf, np.nan],
                     dtype=F32)


def _assert_same_ieee(got, want, what):
    """Bit-exact, except that any NaN matches any NaN (payloads are not part of the contract)."""
    gn, wn = np.isnan(got), np.isnan(want)
    assert np.array_equal(gn, wn), f"{what}: NaN positions differ"
    _assert_bitexact(np.where(gn, F32(0), got), np.where(wn, F32(0), want), what)


def test_special_values(absgd):
    """Every pair (and for the update, a sample of triples) of special fp32 values through
    accumulate and the update rules: IEEE semantics on both sides, subnormals kept."""
    S = _SPECIALS
    n = S.size
    a0, g0 = (t.ravel().astype(F32) for t in np.meshgrid(S, S, indexing="ij"))      # all pairs
    P = a0.size
    print(f"[case] special values, {P} pairs", flush=True)
    with np.errstate(all="ignore"):
        for nn in (1, 32, 3):
            for dtype in ("f32", "bf16"):
                g = g0 if dtype == "f32" else wl.to_bf16_bits(np.where(np.isnan(g0), F32(0), g0))
                for first in (True, False):
                    acc_d = _up(a0)
                    cnt = absgd.Count(0 if first else 32)
                    absgd.abs_accumulate(acc_d, _up(g), nn, cnt, grad_dtype=absgd.ABS_BF16 if dtype == "bf16" else absgd.ABS_F32)
                    want = a0.copy()
                    orc.accumulate32(want, g, nn, first=first)
                    _assert_same_ieee(acc_d.cpu().numpy(), want, f"accumulate {dtype} n={nn} first={first}")
        # update rules: x from one axis, the accumulators from the other, v cycling through the table
        x0, s0 = a0, g0
        v0 = S[(np.arange(P) * 7 + 3) % n].astype(F32)
        s1 = S[(np.arange(P) * 11 + 5) % n].astype(F32)
        for counts in ([32, 64], [1, 0], [3, 5]):
            x_d, v_d = _up(x0), _up(v0)
            absgd.abs_sync_update(x_d, v_d, [_up(s0), _up(s1)], counts, 0.1, 0.9, 5e-4)
            xw, vw = x0.copy(), v0.copy()
            orc.sync_update32(xw, vw, [s0, s1], counts, 0.1, 0.9, 5e-4)
            _assert_same_ieee(x_d.cpu().numpy(), xw, f"sync-update x counts={counts}")
            _assert_same_ieee(v_d.cpu().numpy(), vw, f"sync-update v counts={counts}")
            x_d, v_d, p_d = _up(x0), _up(v0), _up(s1)
            absgd.abs_sync_update_dc(x_d, p_d, v_d, [_up(s0), _up(s1)], counts, 0.1, 0.9, 5e-4, 0.5)
            xw, vw, pw = x0.copy(), v0.copy(), s1.copy()
            orc.sync_update32_dc(xw, pw, vw, [s0, s1], counts, 0.1, 0.9, 5e-4, 0.5)
            _assert_same_ieee(x_d.cpu().numpy(), xw, f"dc x counts={counts}")
            _assert_same_ieee(v_d.cpu().numpy(), vw, f"dc v counts={counts}")
            _assert_same_ieee(p_d.cpu().numpy(), pw, f"dc x_prev counts={counts}")
            x_d, v_d = _up(x0), _up(v0)
            absgd.abs_sync_update_dcm(x_d, v_d, [_up(s0), _up(s1)], counts, 0.1, 0.9, 5e-4, 0.5, 0.07)
            xw, vw = x0.copy(), v0.copy()
            orc.sync_update32_dcm(xw, vw, [s0, s1], counts, 0.1, 0.9, 5e-4, 0.5, 0.07)
            _assert_same_ieee(x_d.cpu().numpy(), xw, f"dcm x counts={counts}")
            _assert_same_ieee(v_d.cpu().numpy(), vw, f"dcm v counts={counts}")
            # Adam: second moment must be non-negative for the square root to mean anything
            m0, q0 = v0, np.abs(s1)
            x_d, m_d, q_d = _up(x0), _up(m0), _up(q0)
            absgd.abs_sync_update_adam(x_d, m_d, q_d, [_up(s0), _up(s1)], counts, 1e-3, 0.9, 0.999, 1e-8, 1e-2, 3)
            xw, mw, qw = x0.copy(), m0.copy(), q0.copy()
            orc.sync_update32_adam(xw, mw, qw, [s0, s1], counts, 1e-3, 0.9, 0.999, 1e-8, 1e-2, 3)
            _assert_same_ieee(m_d.cpu().numpy(), mw, f"adam m counts={counts}")
            _assert_same_ieee(q_d.cpu().numpy(), qw, f"adam v counts={counts}")
            _assert_same_ieee(x_d.cpu().numpy(), xw, f"adam x counts={counts}")


# ---------------------------------------------------------------------------
# calls cut into several launches over consecutive workgroup ranges
# ---------------------------------------------------------------------------

@pytest.fixture
def sliced(absgd, request):
    """One-row tiles, one resident workgroup per CU and a tiny launch length: calls over a
    million elements or more go in 4 to 40 launches (the default cuts only multi-GB calls)."""
    absgd.abs_set_launch_tuning(1, request.param)
    absgd.abs_set_launch_slice_bytes(1 << 20)
    yield request.param
    absgd.abs_set_launch_slice_bytes()     # the defaults
    absgd.abs_set_launch_tuning(0, 4)


@pytest.mark.parametrize("sliced", [1, 2], indirect=True)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sliced_accumulate(absgd, sliced, dtype):
    for P in (1_048_576 + 13, 2_500_007):
        test_accumulate_matches_oracle(absgd, dtype, P)
    print(f"[case] sliced accumulate_jobs {dtype}", flush=True)
    _jobs_case(absgd, 700_001, [2, 5, 1, 0, 3], dtype, 1, seed=7400, start_counts=[0, 32, 0, 0, 64])
    _jobs_case(absgd, 700_001, [2, 9, 1, 0, 3], dtype, 8, seed=7401)


@pytest.mark.parametrize("sliced", [1, 2], indirect=True)
@pytest.mark.parametrize("K", [3, 9, 16, 19])
def test_sliced_sync_update(absgd, sliced, K):
    P = 1_048_576 + 13
    counts = [32 * (1 + k % 3) for k in range(K)]
    print(f"[case] sliced sync_update K={K} rows per tile <= {sliced}", flush=True)
    _sync_case(absgd, K, P, counts, seed=7500 + K)
    _sync_dc_case(absgd, K, P, counts, seed=7510 + K)
    _sync_dcm_case(absgd, K, P, counts, seed=7520 + K)
    _sync_adam_case(absgd, K, P, counts, seed=7530 + K)


@pytest.mark.parametrize("sliced", [1], indirect=True)
@pytest.mark.parametrize("K,dtype", [(3, "f32"), (17, "bf16")])
def test_sliced_ragged_calls(absgd, sliced, K, dtype):
    _ragged_case(absgd, [700_001, 5, 300_000, 1_048_576 + 13, 0, 77], [32 * (1 + k % 3) for k in range(K)],
                 seed=7600 + K, dtype=dtype)
    _lars_case(absgd, [700_001, 5, 300_000, 1_048_576 + 13, 0, 77], [32 * (1 + k % 3) for k in range(K)],
               seed=7610 + K)


@pytest.mark.parametrize("sliced", [1], indirect=True)
@pytest.mark.parametrize("fold", [None, 1, 8])
def test_sliced_trajectory(absgd, sliced, fold):
    _trajectory_case(absgd, "cfg1_small", step_fold=fold)


# ---------------------------------------------------------------------------
# seeded random draws: the grids above vary one thing at a time, these vary all at once
# ---------------------------------------------------------------------------

def _draw_P(rng):
    lo, hi = [(1, 64), (64, 5000), (5000, 70_000)][int(rng.integers(0, 3))]
    return int(rng.integers(lo, hi))


def test_random_draws_accumulate_jobs(absgd):
    rng = np.random.default_rng(0x5EED)
    for case in range(36):
        P, W = _draw_P(rng), int(rng.integers(1, 21))
        Js = [int(j) for j in rng.integers(0, 11, size=W)]
        if sum(Js) == 0:
            Js[0] = 1
        start = [32 * int(rng.integers(1, 4)) if rng.integers(0, 2) else 0 for _ in range(W)]
        fold, dtype = int(rng.integers(1, 9)), ("f32", "bf16")[int(rng.integers(0, 2))]
        shift = int(rng.choice([0, 0, 1, 2, 3]))
        print(f"[case] draw {case}: accumulate_jobs P={P} Js={Js} start={start} fold={fold} {dtype} shift={shift}",
              flush=True)
        _jobs_case(absgd, P, Js, dtype, fold, seed=7000 + case, start_counts=start, shift=shift)


def test_random_draws_sync_update_rules(absgd):
    rng = np.random.default_rng(0xD1CE)
    rules = [("sgd", _sync_case), ("dc", _sync_dc_case), ("dcm", _sync_dcm_case), ("adam", _sync_adam_case)]
    for case in range(40):
        P, K = _draw_P(rng), int(rng.integers(1, 41))
        counts = [32 * int(c) for c in rng.integers(0, 4, size=K)]       # about a quarter of the workers idle
        if sum(counts) == 0:
            counts[int(rng.integers(0, K))] = 64
        name, fn = rules[case % 4]
        print(f"[case] draw {case}: {name} P={P} K={K} counts={counts}", flush=True)
        fn(absgd, K, P, counts, seed=7100 + case)


def test_random_draws_ragged_layouts(absgd):
    rng = np.random.default_rng(0xFACE)
    for case in range(12):
        T = int(rng.integers(1, 13))
        sizes = [0 if rng.integers(0, 6) == 0 else _draw_P(rng) for _ in range(T)]
        if sum(sizes) == 0:
            sizes[0] = 17
        K = int(rng.integers(1, 25))
        counts = [32 * int(c) for c in rng.integers(0, 4, size=K)]
        if sum(counts) == 0:
            counts[0] = 32
        dtype, misalign = ("f32", "bf16")[case % 2], bool(rng.integers(0, 2))
        print(f"[case] draw {case}: ragged sizes={sizes} counts={counts}", flush=True)
        _ragged_case(absgd, sizes, counts, seed=7200 + case, dtype=dtype, misalign=misalign)
        if case % 3 == 0:
            _lars_case(absgd, sizes, counts, seed=7300 + case)


# ---------------------------------------------------------------------------
# the C ABI from plain C: no Python binding, no PyTorch in the process
# ---------------------------------------------------------------------------

def test_c_abi_from_plain_c(absgd):
    """tests/c_abi/abi_check.c: hipMalloc'ed buffers, the library's calls, the C oracle."""
    import subprocess
    from tests.c_abi.build_check import build_abi_check
    exe = build_abi_check()
    print(f"[case] {exe}", flush=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0
    assert r.stdout.strip().endswith("abi_check: OK")


# ---------------------------------------------------------------------------
# the usage example of the README runs as printed
# ---------------------------------------------------------------------------

def test_readme_example_runs(absgd):
    import os
    import torch
    readme = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "README.md")
    code = open(readme).read().split("```python")[1].split("```")[0]
    print("[case] README example", flush=True)
    ns = {}
    exec(compile(code, "README.md", "exec"), ns)
    x, v, ctx = ns["x"], ns["v"], ns["ctx"]
    assert bool(torch.isfinite(x).all()) and bool(torch.isfinite(v).all())
    assert float(v.abs().max()) > 0.0                       # updates were applied
    assert ctx.counts(0) == [0] * ns["K"]                   # after the last swap: nothing accumulated yet
    assert ctx.counts(1) == [32 * (1 + k) for k in range(ns["K"])]
