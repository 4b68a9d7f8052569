"""CPU tests of the boundary: the C-ABI library loads, exports every symbol the
header declares, and its host-side logic (argument checks, ragged chunk table,
empty-step detection) behaves as the header states.  No kernel is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2308_15164_amd as absgd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "abs_sgd.h")


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(abs_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = absgd.lib()
    declared = _declared_symbols()
    assert len(declared) >= 20
    for name in declared:
        assert hasattr(L, name), f"{name} declared in abs_sgd.h but not exported"
    # and the binding marshals exactly that set
    assert sorted(absgd.SYMBOLS) == declared


def test_version_tile_and_error_strings():
    assert absgd.abs_version() >= 100
    row = absgd.abs_row_elems()
    assert row > 0 and row % 256 == 0
    L = absgd.lib()
    assert b"invalid" in L.abs_error_string(absgd.ABS_EINVAL)
    assert L.abs_error_string(absgd.ABS_OK) == b"ok"


def _rc_accumulate(acc, grad, dtype, P, n, count):
    c = ctypes.c_int64(count)
    rc = absgd.lib().abs_accumulate(acc, grad, dtype, P, n, ctypes.byref(c), None)
    return rc, c.value


def test_accumulate_rejects_bad_arguments_before_touching_the_gpu():
    assert _rc_accumulate(None, 16, absgd.ABS_F32, 8, 32, 0)[0] == absgd.ABS_EINVAL     # null acc
    assert _rc_accumulate(16, None, absgd.ABS_F32, 8, 32, 0)[0] == absgd.ABS_EINVAL     # null grad
    assert _rc_accumulate(16, 32, absgd.ABS_F32, -1, 32, 0)[0] == absgd.ABS_EINVAL      # P < 0
    assert _rc_accumulate(16, 32, absgd.ABS_F32, 8, 0, 0)[0] == absgd.ABS_EINVAL        # n <= 0
    assert _rc_accumulate(16, 32, absgd.ABS_F32, 8, 32, -5)[0] == absgd.ABS_EINVAL      # count < 0
    assert _rc_accumulate(18, 32, absgd.ABS_F32, 8, 32, 0)[0] == absgd.ABS_EINVAL       # acc not 4-aligned
    assert _rc_accumulate(16, 33, absgd.ABS_BF16, 8, 32, 0)[0] == absgd.ABS_EINVAL      # bf16 not 2-aligned
    assert _rc_accumulate(16, 32, 7, 8, 32, 0)[0] == absgd.ABS_EINVAL                   # dtype
    assert _rc_accumulate(16, 32, absgd.ABS_F32, 8, 2, 2**63 - 2)[0] == absgd.ABS_EINVAL  # overflow
    # failed calls leave the count alone
    assert _rc_accumulate(None, 16, absgd.ABS_F32, 8, 32, 64)[1] == 64
    # P == 0: nothing to launch, only the integer moves (bit-exact counts)
    rc, cnt = _rc_accumulate(None, None, absgd.ABS_F32, 0, 32, 64)
    assert rc == absgd.ABS_OK and cnt == 96


def _rc_sync(x, v, ptrs, counts, P, K=None):
    K = len(ptrs) if K is None else K
    arr = (ctypes.c_void_p * max(1, len(ptrs)))(*ptrs)
    cnt = (ctypes.c_int64 * max(1, len(counts)))(*counts)
    return absgd.lib().abs_sync_update(x, v, arr, cnt, K, P, 0.1, 0.9, 5e-4, None)


def test_sync_update_empty_and_bad_arguments():
    # total count zero: the first iteration applies nothing, whatever the pointers are
    assert _rc_sync(16, 32, [48, 64], [0, 0], 8) == absgd.ABS_EMPTY
    assert _rc_sync(16, 32, [48, 64], [32, -1], 8) == absgd.ABS_EINVAL
    assert _rc_sync(16, 32, [48], [32], 8, K=0) == absgd.ABS_EINVAL
    assert _rc_sync(16, 32, [48] * 65, [32] * 65, 8) == absgd.ABS_EINVAL      # K > ABS_MAX_K
    assert _rc_sync(None, 32, [48], [32], 8) == absgd.ABS_EINVAL
    assert _rc_sync(16, 16, [48], [32], 8) == absgd.ABS_EINVAL                 # x aliases v
    assert _rc_sync(16, 32, [None], [32], 8) == absgd.ABS_EINVAL               # non-empty worker, null buffer
    assert _rc_sync(16, 32, [48], [32], -3) == absgd.ABS_EINVAL
    assert _rc_sync(16, 32, [48], [32], 0) == absgd.ABS_OK                     # P == 0


@pytest.mark.parametrize("sizes", [[1], [0, 5, 0], [4096], [4097, 1, 8192, 3], [12289, 768, 100000],
                                   [5_000_000, 1, 1023, 1025, 3_000_001]])
def test_layout_chunk_table_partitions_every_tensor(sizes):
    lay = absgd.Layout(sizes)
    tile = lay.tile()
    assert tile > 0 and tile % absgd.abs_row_elems() == 0
    assert lay.num_tensors() == len(sizes)
    assert lay.total() == sum(sizes)
    expected = sum((s + tile - 1) // tile for s in sizes)
    assert lay.num_chunks() == expected
    covered = [np.zeros(s, dtype=np.int32) for s in sizes]
    for c in range(lay.num_chunks()):
        t, off, ln = lay.chunk(c)
        assert 0 < ln <= tile and off % tile == 0 and off + ln <= sizes[t]
        covered[t][off:off + ln] += 1
    for cov in covered:
        assert np.all(cov == 1)          # every element in exactly one chunk
    assert absgd.lib().abs_layout_chunk(lay.handle, lay.num_chunks(), None, None, None) == absgd.ABS_EINVAL
    lay.close()


def test_layout_tile_fills_whole_rounds():
    """Large layouts get one chunk per resident workgroup (about), small ones one row per chunk."""
    row = absgd.abs_row_elems()
    small = absgd.Layout([row * 10, 5])
    assert small.tile() == row
    absgd.abs_set_launch_tuning(0, 0)              # no cap: one round
    big = absgd.Layout([row * 2048 * 7 + 3])
    assert big.tile() == 8 * row and big.num_chunks() <= 2048
    absgd.abs_set_launch_tuning(0, 4)              # the default cap of 4 rows: two rounds of 2048
    capped = absgd.Layout([row * 2048 * 7 + 3])
    assert capped.tile() == 4 * row and 2048 < capped.num_chunks() <= 4096
    with pytest.raises(absgd.AbsError):
        absgd.abs_set_launch_tuning(-1, 0)


def test_layout_rejects_bad_sizes():
    h = ctypes.c_void_p()
    L = absgd.lib()
    assert L.abs_layout_create(ctypes.byref(h), 0, (ctypes.c_int64 * 1)(1)) == absgd.ABS_EINVAL
    assert L.abs_layout_create(ctypes.byref(h), 2, (ctypes.c_int64 * 2)(5, -1)) == absgd.ABS_EINVAL
    assert L.abs_layout_create(None, 1, (ctypes.c_int64 * 1)(1)) == absgd.ABS_EINVAL


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(absgd, "_lib", None)
    monkeypatch.setattr(absgd, "LIB_PATH", "/nonexistent/libabs_sgd.so")
    with pytest.raises(ImportError, match="no CPU or PyTorch fallback"):
        absgd.lib()


def test_bench_refuses_more_than_one_gpu():
    """One GPU per box: the benchmark says so instead of starting ranks."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_accumulate_batch_host_checks():
    L = absgd.lib()
    c = ctypes.c_int64(32)
    n2 = (ctypes.c_int64 * 2)(32, 64)
    g2 = (ctypes.c_void_p * 2)(64, 128)
    # P == 0: only the count moves, by the sum of the batch
    assert L.abs_accumulate_batch(None, g2, absgd.ABS_F32, 2, 0, n2, ctypes.byref(c), None) == absgd.ABS_OK
    assert c.value == 128
    assert L.abs_accumulate_batch(16, g2, absgd.ABS_F32, 0, 8, n2, ctypes.byref(c), None) == absgd.ABS_EINVAL
    bad = (ctypes.c_void_p * 2)(64, None)
    assert L.abs_accumulate_batch(16, bad, absgd.ABS_F32, 2, 8, n2, ctypes.byref(c), None) == absgd.ABS_EINVAL
    assert c.value == 128


def test_update_rule_host_checks():
    L = absgd.lib()
    arr = (ctypes.c_void_p * 1)(64)
    cnt = (ctypes.c_int64 * 1)(32)
    zero = (ctypes.c_int64 * 1)(0)
    # compensation: the previous-iterate buffer must be distinct
    assert L.abs_sync_update_dc(16, 16, 32, arr, cnt, 1, 8, 0.1, 0.9, 0.0, 0.5, None) == absgd.ABS_EINVAL
    assert L.abs_sync_update_dc(16, None, 32, arr, cnt, 1, 8, 0.1, 0.9, 0.0, 0.5, None) == absgd.ABS_EINVAL
    # compensation from the momentum: no third vector; an empty step touches nothing and says so
    assert L.abs_sync_update_dcm(16, 32, arr, zero, 1, 8, 0.1, 0.9, 0.0, 0.5, 0.1, None) == absgd.ABS_EMPTY
    assert L.abs_sync_update_dcm(16, 16, arr, cnt, 1, 8, 0.1, 0.9, 0.0, 0.5, 0.1, None) == absgd.ABS_EINVAL
    assert L.abs_sync_update_dcm(None, 32, arr, cnt, 1, 8, 0.1, 0.9, 0.0, 0.5, 0.1, None) == absgd.ABS_EINVAL
    assert L.abs_sync_update_dcm(16, 32, arr, cnt, 1, 0, 0.1, 0.9, 0.0, 0.5, 0.1, None) == absgd.ABS_OK   # P == 0
    # Adam: step >= 1, betas in [0, 1), eps >= 0; an empty step is reported before anything else happens
    assert L.abs_sync_update_adam(16, 32, 48, arr, cnt, 1, 8, 1e-3, 0.9, 0.999, 1e-8, 0.0, 0, None) == absgd.ABS_EINVAL
    assert L.abs_sync_update_adam(16, 32, 48, arr, cnt, 1, 8, 1e-3, 1.5, 0.999, 1e-8, 0.0, 1, None) == absgd.ABS_EINVAL
    assert L.abs_sync_update_adam(16, 32, 48, arr, cnt, 1, 8, 1e-3, 0.9, 0.999, -1.0, 0.0, 1, None) == absgd.ABS_EINVAL
    assert L.abs_sync_update_adam(16, 32, 48, arr, zero, 1, 8, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, None) == absgd.ABS_EMPTY
    assert L.abs_sync_update_adam(16, 32, 32, arr, cnt, 1, 8, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, None) == absgd.ABS_EINVAL


def test_header_is_strict_c99_and_the_c_caller_builds():
    """include/abs_sgd.h compiles as ISO C99 with every warning an error, and the
    plain-C test program links against the library (no GPU needed to build)."""
    import subprocess
    hdr = os.path.join(ROOT, "include", "abs_sgd.h")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c", hdr],
                   check=True, timeout=60)
    from oracle.abs_oracle import build_oracle
    from tests.c_abi.build_check import build_abi_check
    build_oracle()
    exe = build_abi_check(force=True)
    assert os.access(exe, os.X_OK)


def test_double_buffer_bookkeeping_without_a_gpu():
    """With P = 0 no kernel is launched, so the context's host side runs anywhere:
    per-generation sample counts, the flip, the empty first iteration (G_{-1} = 0 has
    no samples), and the argument checks."""
    L = absgd.lib()
    K = 3
    null = (ctypes.c_void_p * K)()
    ctx = ctypes.c_void_p()
    assert L.abs_ctx_create(ctypes.byref(ctx), K, 0, null, null, None, None) == absgd.ABS_OK
    out = (ctypes.c_int64 * K)()

    def counts(which):
        assert L.abs_ctx_counts(ctx, which, out) == absgd.ABS_OK
        return list(out)

    # iteration 0: nothing to apply yet
    assert L.abs_ctx_sync_update(ctx, None, None, 0.1, 0.9, 0.0) == absgd.ABS_EMPTY
    for k, m in enumerate((2, 0, 3)):
        for _ in range(m):
            assert L.abs_ctx_accumulate(ctx, k, None, absgd.ABS_F32, 32) == absgd.ABS_OK
    n2 = (ctypes.c_int64 * 2)(16, 48)
    g2 = (ctypes.c_void_p * 2)()
    assert L.abs_ctx_accumulate_batch(ctx, 1, g2, absgd.ABS_F32, 2, n2) == absgd.ABS_OK
    assert counts(0) == [64, 64, 96] and counts(1) == [0, 0, 0]
    assert L.abs_ctx_accumulate(ctx, K, None, absgd.ABS_F32, 32) == absgd.ABS_EINVAL        # no such worker
    assert L.abs_ctx_accumulate(ctx, 0, None, absgd.ABS_F32, 0) == absgd.ABS_EINVAL        # a batch has samples
    assert L.abs_ctx_set_accumulate_streams(ctx, null, 2) == absgd.ABS_EINVAL              # too late: counts moved
    assert counts(0) == [64, 64, 96]
    assert L.abs_swap_buffers(ctx) == absgd.ABS_OK
    # iteration 1: the previous generation is what was accumulated, the current one starts empty
    assert counts(0) == [0, 0, 0] and counts(1) == [64, 64, 96]
    assert L.abs_ctx_sync_update(ctx, None, None, 0.1, 0.9, 0.0) == absgd.ABS_OK            # P = 0: nothing to launch
    assert L.abs_ctx_accumulate(ctx, 2, None, absgd.ABS_BF16, 8) == absgd.ABS_OK
    assert L.abs_swap_buffers(ctx) == absgd.ABS_OK
    assert counts(0) == [0, 0, 0] and counts(1) == [0, 0, 8]
    assert L.abs_swap_buffers(ctx) == absgd.ABS_OK
    # an iteration in which no worker accumulated anything applies nothing
    assert counts(1) == [0, 0, 0]
    assert L.abs_ctx_sync_update(ctx, None, None, 0.1, 0.9, 0.0) == absgd.ABS_EMPTY
    assert L.abs_ctx_sync_update_dcm(ctx, None, None, 0.1, 0.9, 0.0, 0.5) == absgd.ABS_EMPTY
    # flat contexts refuse the ragged calls and the other way round
    assert L.abs_ctx_sync_update_mt(ctx, None, None, 0.1, 0.9, 0.0) == absgd.ABS_EINVAL
    assert L.abs_ctx_counts(ctx, 2, out) == absgd.ABS_EINVAL
    assert L.abs_ctx_destroy(ctx) == absgd.ABS_OK
    assert L.abs_ctx_create(ctypes.byref(ctx), 0, 0, null, null, None, None) == absgd.ABS_EINVAL
    assert L.abs_ctx_create(ctypes.byref(ctx), 65, 0, null, null, None, None) == absgd.ABS_EINVAL


def test_python_wrappers_marshal_every_flat_call_without_a_gpu():
    """P = 0 launches nothing, and the wrappers accept raw integer addresses: every flat
    wrapper is called once through its Python signature (argument order and count)."""
    cnt = absgd.Count(0)
    assert absgd.abs_accumulate(16, 32, 8, cnt, P=0, grad_dtype=absgd.ABS_F32, stream=0) is True
    assert absgd.abs_accumulate_batch(16, [32, 48], [8, 8], cnt, P=0, grad_dtype=absgd.ABS_BF16, stream=0) is True
    assert cnt.value == 24
    acc, counts = [64, 128], [32, 0]
    assert absgd.abs_sync_update(16, 32, acc, counts, 0.1, 0.9, 5e-4, P=0, stream=0) is True
    assert absgd.abs_sync_update(16, 32, acc, [0, 0], 0.1, 0.9, 5e-4, P=0, stream=0) is False
    assert absgd.abs_sync_update_dc(16, 48, 32, acc, counts, 0.1, 0.9, 5e-4, 0.5, P=0, stream=0) is True
    assert absgd.abs_sync_update_dcm(16, 32, acc, counts, 0.1, 0.9, 5e-4, 0.5, 0.1, P=0, stream=0) is True
    assert absgd.abs_sync_update_adam(16, 32, 48, acc, counts, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, P=0, stream=0) is True
    with pytest.raises(absgd.AbsError):
        absgd.abs_sync_update_adam(16, 32, 48, acc, counts, 1e-3, 0.9, 0.999, 1e-8, 0.0, 0, P=0, stream=0)
    assert absgd.abs_set_cache_policy(-1, -1) is True
    assert absgd.abs_set_launch_tuning(0, 4) is True
    ctx = absgd.Context([0, 0], [0, 0], 0, 0, P=0)         # stream handle 0: the null stream
    assert ctx.abs_sync_update(0, 0, 0.1, 0.9, 0.0) is False
    assert ctx.abs_accumulate(1, 0, 32, grad_dtype=absgd.ABS_F32) is True
    assert ctx.abs_accumulate_batch(0, [0, 0], [16, 16], grad_dtype=absgd.ABS_F32) is True
    assert ctx.counts(0) == [32, 32] and ctx.counts(1) == [0, 0]
    assert absgd.abs_swap_buffers(ctx) is True
    assert ctx.counts(1) == [32, 32]
    assert ctx.abs_sync_update(0, 0, 0.1, 0.9, 0.0) is True
    assert ctx.abs_sync_update_dc(0, 0, 0, 0.1, 0.9, 0.0, 0.5) is True
    assert ctx.abs_sync_update_dcm(0, 0, 0.1, 0.9, 0.0, 0.5) is True
    assert ctx.abs_sync_update_adam(0, 0, 0, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1) is True
    ctx.close()


def test_suggested_accumulate_streams_for_the_stated_configurations():
    import abs_workloads as wl
    want = {"cfg1_small": 1, "cfg2_resnet18": 2, "cfg3_resnet50_bf16": 2, "cfg4_vgg16": 1,
            "cfg5_gpt2_ragged_bf16": 1, "paper_static": 2}
    for name, n in want.items():
        w = wl.WORKLOADS[name]
        assert absgd.abs_suggest_accumulate_streams(w.P, w.K) == n, name
    assert absgd.abs_suggest_accumulate_streams(11_689_512, 1) == 1        # one worker: nothing to spread
    assert absgd.abs_suggest_accumulate_streams(0, 4) == 1


def test_flat_calls_reject_overlapping_buffers():
    """A buffer a call writes may not share a byte with another buffer of the call: partial
    overlaps are refused like exact aliases, before anything is enqueued."""
    L = absgd.lib()
    P = 8                                       # 32 bytes per fp32 vector, 16 per bf16 vector
    c = ctypes.c_int64(0)
    # the gradient starts inside the accumulator / the accumulator starts inside the gradient
    assert L.abs_accumulate(1024, 1024 + 16, absgd.ABS_F32, P, 32, ctypes.byref(c), None) == absgd.ABS_EINVAL
    assert L.abs_accumulate(1024 + 8, 1024, absgd.ABS_BF16, P, 32, ctypes.byref(c), None) == absgd.ABS_EINVAL
    assert c.value == 0
    one, cnt = (ctypes.c_void_p * 1)(4096), (ctypes.c_int64 * 1)(32)
    sync = lambda x, v, a=one: L.abs_sync_update(x, v, a, cnt, 1, P, 0.1, 0.9, 0.0, None)
    assert sync(1024, 1024 + 28) == absgd.ABS_EINVAL                            # v starts in x's last element
    assert sync(1024, 2048, (ctypes.c_void_p * 1)(1024 + 16)) == absgd.ABS_EINVAL   # an accumulator inside x
    assert sync(1024, 2048, (ctypes.c_void_p * 1)(2048 - 4)) == absgd.ABS_EINVAL    # ... reaching into v
    assert L.abs_sync_update_dc(1024, 2048 + 4, 2048, one, cnt, 1, P, 0.1, 0.9, 0.0, 0.5, None) == absgd.ABS_EINVAL
    assert L.abs_sync_update_adam(1024, 2048, 1024 + 20, one, cnt, 1, P, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1,
                                  None) == absgd.ABS_EINVAL
    # the 2K accumulators of a context are all written
    ctx = ctypes.c_void_p()
    A, B = (ctypes.c_void_p * 2)(1024, 2048), (ctypes.c_void_p * 2)(4096, 2048 + 16)
    assert L.abs_ctx_create(ctypes.byref(ctx), 2, P, A, B, None, None) == absgd.ABS_EINVAL
    A2 = (ctypes.c_void_p * 2)(1024, 1024 + 4)
    assert L.abs_ctx_create(ctypes.byref(ctx), 2, P, A2, (ctypes.c_void_p * 2)(4096, 8192), None, None) == absgd.ABS_EINVAL


def test_python_default_launch_tuning_is_the_librarys():
    """abs_set_launch_tuning() without arguments restores what the library starts with (tiles of
    at most 4 rows), not the uncapped shape."""
    row = absgd.abs_row_elems()
    absgd.abs_set_launch_tuning(0, 0)
    absgd.abs_set_launch_tuning()
    lay = absgd.Layout([row * 2048 * 7 + 3])
    assert lay.tile() == 4 * row
    lay.close()


def test_job_list_host_side_without_a_gpu():
    """P = 0 launches nothing: the job list's counts, its argument checks, and the one-call Step 2
    of a context run anywhere."""
    L = absgd.lib()
    counts = [absgd.Count(0), absgd.Count(32), absgd.Count(0)]
    ns = [[32, 32], [], [8, 16, 24]]
    assert absgd.abs_accumulate_jobs([0, 0, 0], [[0, 0], [], [0, 0, 0]], ns, counts, fold=2, P=0,
                                     grad_dtype=absgd.ABS_F32, stream=0) is True
    assert [c.value for c in counts] == [64, 32, 48]
    for bad_fold in (0, 9):
        with pytest.raises(absgd.AbsError):
            absgd.abs_accumulate_jobs([0], [[0]], [[32]], [absgd.Count(0)], fold=bad_fold, P=0,
                                      grad_dtype=absgd.ABS_F32, stream=0)
    with pytest.raises(absgd.AbsError):                       # a batch has samples
        absgd.abs_accumulate_jobs([0], [[0]], [[0]], [absgd.Count(0)], P=0, grad_dtype=absgd.ABS_F32, stream=0)
    shared = absgd.Count(0)
    with pytest.raises(absgd.AbsError):                       # two jobs, one count
        absgd.abs_accumulate_jobs([0, 0], [[0], [0]], [[32], [32]], [shared, shared], P=0,
                                  grad_dtype=absgd.ABS_F32, stream=0)
    assert shared.value == 0
    # two jobs into one accumulator, or a gradient that is another job's accumulator: refused at P > 0
    c2 = [absgd.Count(0), absgd.Count(0)]
    with pytest.raises(absgd.AbsError):
        absgd.abs_accumulate_jobs([1024, 1024 + 16], [[4096], [8192]], [[32], [32]], c2, P=8,
                                  grad_dtype=absgd.ABS_F32, stream=0)
    with pytest.raises(absgd.AbsError):
        absgd.abs_accumulate_jobs([1024, 2048], [[2048 + 4], [8192]], [[32], [32]], c2, P=8,
                                  grad_dtype=absgd.ABS_F32, stream=0)
    assert [c.value for c in c2] == [0, 0]
    assert L.abs_accumulate_jobs(None, 1, absgd.ABS_F32, 0, 8, None) == absgd.ABS_EINVAL
    # the context's one-call Step 2
    ctx = absgd.Context([0, 0, 0], [0, 0, 0], 0, 0, P=0)
    assert ctx.abs_accumulate_step([0] * 5, [2, 0, 3], [32] * 5, fold=1, grad_dtype=absgd.ABS_F32) is True
    assert ctx.counts(0) == [64, 0, 96]
    assert ctx.abs_accumulate_step([0], [0, 1, 0], [7], fold=8, grad_dtype=absgd.ABS_BF16) is True
    assert ctx.counts(0) == [64, 7, 96]
    with pytest.raises(absgd.AbsError):
        ctx.abs_accumulate_step([0], [0, -1, 0], [7], grad_dtype=absgd.ABS_F32)
    assert absgd.abs_swap_buffers(ctx) is True
    assert ctx.counts(1) == [64, 7, 96] and ctx.counts(0) == [0, 0, 0]
    # settings of its own: same argument checks as the process-wide calls
    assert ctx.abs_set_cache_policy(1, 0) is True and ctx.abs_set_launch_tuning(2, 3) is True
    with pytest.raises(absgd.AbsError):
        ctx.abs_set_cache_policy(2, 0)
    with pytest.raises(absgd.AbsError):
        ctx.abs_set_launch_tuning(0, -1)
    ctx.close()


def test_launch_slicing_rule():
    """abs_slice_workgroups: a call is cut into floor(bytes / slice_bytes) launches (one below
    twice the unit), every launch but the last a whole number of resident rounds, together
    covering every workgroup once; 0 switches the cutting off."""
    L = absgd.lib()
    rng = np.random.default_rng(5)
    try:
        for unit in (1 << 30, 1 << 20, 12345):
            absgd.abs_set_launch_slice_bytes(unit)
            for _ in range(300):
                wgs = int(rng.integers(0, 200_000))
                nbytes = int(rng.integers(0, 40 * unit))
                resident = int(rng.integers(1, 3000))
                per = L.abs_slice_workgroups(wgs, nbytes, resident)
                if nbytes < 2 * unit or wgs <= resident:
                    assert per == wgs
                    continue
                assert 1 <= per <= max(wgs, resident) and per % resident == 0
                launches = -(-wgs // per)
                assert 1 <= launches <= nbytes // unit
                # cutting never makes launches smaller than half of what was asked for, except the last
                assert per >= wgs // (nbytes // unit)
        absgd.abs_set_launch_slice_bytes(0)
        assert L.abs_slice_workgroups(10**6, 10**15, 7) == 10**6
        assert L.abs_set_launch_slice_bytes(-1) == absgd.ABS_EINVAL
        assert L.abs_slice_workgroups(-1, 0, 1) == absgd.ABS_EINVAL
        assert L.abs_slice_workgroups(1, -1, 1) == absgd.ABS_EINVAL
        assert L.abs_slice_workgroups(1, 1, 0) == absgd.ABS_EINVAL
    finally:
        absgd.abs_set_launch_slice_bytes()
    # the default: the VGG16-sized accumulate (1.66 GB) goes in one launch, the sync-update over
    # 16 such accumulators (11 GB, ten units) in nine launches of five resident rounds each
    assert L.abs_slice_workgroups(33_779, 12 * 138_357_544, 2048) == 33_779
    per = L.abs_slice_workgroups(33_779, 80 * 138_357_544, 768)
    assert per == 5 * 768 and -(-33_779 // per) == 9
