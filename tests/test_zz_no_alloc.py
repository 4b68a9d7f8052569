"""The allocation-free entry point, abs_sync_update_lars_mt_noalloc, through the C ABI against
the entry point it is a variant of (abs_sync_update_lars_mt): same inputs, two calls in a row,
the second on a smaller layout, every output compared bit for bit (the two share their
kernels and the order of every sum is fixed, so nothing less than equal bits is expected).
The existing entry point is itself checked against the oracle in test_gpu_parity.py."""

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

F32 = np.float32


@pytest.fixture(scope="module")
def absgd():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2308_15164_amd as m
    m.lib()
    return m


def _bits(ts):
    return np.concatenate([t.cpu().numpy().view(np.uint32) for t in ts]) if ts else np.zeros(0, np.uint32)


def _pair(absgd, sizes, counts, seed, lr=0.1, mu=0.9, wd=5e-4, eta=0.02):
    """Run both entry points on copies of the same state; return what each left behind."""
    rng = np.random.default_rng(seed)
    K = len(counts)
    lay = absgd.Layout(sizes)

    def tensors(sigma, fill=None):
        return [torch.from_numpy(np.full(s, fill, dtype=F32) if fill is not None
                                 else (rng.standard_normal(s) * sigma).astype(F32)).cuda() for s in sizes]

    x0, v0 = tensors(0.05), tensors(0.01)
    accs = [tensors(20.0 * max(c, 1) / 32) if c > 0 else tensors(0, fill=np.nan) for c in counts]
    asets = [absgd.TensorSet(lay, a) for a in accs]
    out = []
    for fn in (absgd.abs_sync_update_lars_mt, absgd.abs_sync_update_lars_mt_noalloc):
        xt, vt = [t.clone() for t in x0], [t.clone() for t in v0]
        gt = [torch.full_like(t, float("nan")) for t in x0]                  # workspace: stale garbage
        torch.cuda.synchronize()
        xs, vs, gs = (absgd.TensorSet(lay, t) for t in (xt, vt, gt))
        applied = fn(lay, xs, vs, gs, asets, counts, lr, mu, wd, eta)
        torch.cuda.synchronize()
        out.append((applied, _bits(xt), _bits(vt), _bits(gt)))
    x0b = _bits(x0)
    lay_chunks = lay.num_chunks()
    return out, x0b, lay_chunks


def test_noalloc_lars_recorded_into_a_graph_and_replayed(absgd):
    """What the entry point is for: a caller under graph capture.  The call is recorded with no call
    before it (the scratch array's address was looked up when the layout's tables went to the device),
    replayed three times with eager work between the replays, and every replay is compared bit for
    bit with the allocating entry point applied eagerly to a copy of the same state."""
    rng = np.random.default_rng(77)
    sizes, counts = [4096 * 5 + 3, 700, 1, 65_537], [32, 64, 0, 96]
    hyper = (0.1, 0.9, 5e-4, 0.02)
    lay = absgd.Layout(sizes)
    mk = lambda sigma: [torch.from_numpy((rng.standard_normal(s) * sigma).astype(F32)).cuda() for s in sizes]
    x0, v0 = mk(0.05), mk(0.01)
    accs = [mk(20.0 * max(c, 1) / 32) for c in counts]
    asets = [absgd.TensorSet(lay, a) for a in accs]
    state = lambda: ([t.clone() for t in x0], [t.clone() for t in v0], [torch.zeros_like(t) for t in x0])
    xr, vr, gr = state()          # eager, allocating entry point
    xg, vg, gg = state()          # replays of the recorded allocation-free call
    xw, vw, gw = state()          # eager allocation-free calls between the replays
    rs, gs, ws = ([absgd.TensorSet(lay, t) for t in trio] for trio in ((xr, vr, gr), (xg, vg, gg), (xw, vw, gw)))
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    print("[case] noalloc lars: capture", flush=True)
    with torch.cuda.graph(graph, stream=side):
        assert absgd.abs_sync_update_lars_mt_noalloc(lay, gs[0], gs[1], gs[2], asets, counts, *hyper)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(xg), _bits(x0)), "recording a call must not run it"
    for r in range(3):
        print(f"[case] noalloc lars: replay {r}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert absgd.abs_sync_update_lars_mt(lay, rs[0], rs[1], rs[2], asets, counts, *hyper)
        torch.cuda.synchronize()
        assert np.array_equal(_bits(xg), _bits(xr)), f"x differs after replay {r}"
        assert np.array_equal(_bits(vg), _bits(vr)), f"v differs after replay {r}"
        # the program's own eager work between replays, a call that shares the scratch array included
        assert absgd.abs_sync_update_lars_mt_noalloc(lay, ws[0], ws[1], ws[2], asets, counts, *hyper)
        float(torch.randn(1 << 20, device="cuda").sum())
        torch.cuda.synchronize()
    assert not np.array_equal(_bits(xg), _bits(x0))


def test_noalloc_lars_equals_the_allocating_entry_point_twice_in_a_row(absgd):
    cases = [([1_048_576 + 13, 300_007, 5, 0, 70_001, 1], [32, 64, 0, 96], 31),    # larger first
             ([5000, 3, 700], [64, 32], 32),                                     # then smaller: stale scratch beyond it
             ([4096 * 9 + 1, 2], [0, 0, 0], 33)]                                 # nothing to apply
    for sizes, counts, seed in cases:
        print(f"[case] noalloc lars sizes={sizes} counts={counts}", flush=True)
        (ref, new), x0b, chunks = _pair(absgd, sizes, counts, seed)
        assert ref[0] == new[0] == (sum(counts) > 0)
        for what, a, b in zip(("x", "v", "gbar"), ref[1:], new[1:]):
            bad = np.nonzero(a != b)[0]
            assert bad.size == 0, f"{what}: {bad.size} elements differ in bits, first at {bad[0]} ({chunks} chunks)"
        if sum(counts) > 0:
            assert np.any(ref[1] != x0b), "the update moved nothing"
        else:
            assert np.array_equal(new[1], x0b), "an empty step touched x"


def test_noalloc_lars_rejects_layouts_beyond_its_scratch(absgd):
    print("[case] noalloc lars limits", flush=True)
    T = 4097                                                   # one tensor more than the fixed array holds
    buf = lambda: torch.ones(3 * T, device="cuda")
    lay = absgd.Layout([3] * T)
    bx, bv, bg, ba = buf(), buf(), buf(), buf()
    sets = [absgd.TensorSet(lay, [b[3 * i:3 * i + 3] for i in range(T)]) for b in (bx, bv, bg, ba)]
    with pytest.raises(absgd.AbsError):
        absgd.abs_sync_update_lars_mt_noalloc(lay, sets[0], sets[1], sets[2], [sets[3]], [32], 0.1, 0.9, 0.0, 0.02)
    torch.cuda.synchronize()
    for b in (bx, bv, bg, ba):
        assert bool((b == 1).all())
    # the allocating entry point takes the same layout
    assert absgd.abs_sync_update_lars_mt(lay, sets[0], sets[1], sets[2], [sets[3]], [32], 0.1, 0.9, 0.0, 0.02)
    torch.cuda.synchronize()
    assert not bool((bx == 1).all())
    L = absgd.lib()
    assert L.abs_sync_update_lars_mt_noalloc(None, None, None, None, None, None, 1, 0.1, 0.9, 0.0, 0.02,
                                             None) == absgd.ABS_EINVAL
