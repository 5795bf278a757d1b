"""GPU parity of the batched (several plans, one launch) entry points: bit-identical to the per-plan calls,
and checked against the oracle on the decode-step append of the d = 96 workload."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2605_05699_amd import workloads as W
from tests import parity_util as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2605_05699_amd import binding
    binding.lib()
    return binding


def _make(B, d, g, counts, seed0, cap=None):
    """Plans with distinct signs and lambda, inputs of the given lengths, and the per-plan results."""
    plans, xs, ref = [], [], []
    for i, n in enumerate(counts):
        lam = W.lognormal_lambda(d, seed=seed0 + 7 * i)
        plan = B.Plan(d, g, seed0 + i, lam)
        plan.lam = lam
        x = torch.from_numpy(W.gaussian_with_outliers(max(n, 1), d, seed=seed0 + 13 * i, outliers=1))[:n].cuda()
        if n:
            codes, scales = plan.quantize(x)
            out = plan.dequantize(codes, scales)
        else:
            codes = torch.empty(0, d // 2, dtype=torch.uint8, device="cuda")
            scales = torch.empty(0, d // g, dtype=torch.float32, device="cuda")
            out = torch.empty(0, d, dtype=torch.float16, device="cuda")
        if cap:
            B.srft_plan_set_max_workgroups(plan.handle, cap)
        plans.append(plan)
        xs.append(x)
        ref.append((codes, scales, out))
    return plans, xs, ref


def _batched(B, plans, xs, d, g):
    codes = [torch.full((x.shape[0], d // 2), 0xAB, dtype=torch.uint8, device="cuda") for x in xs]
    scales = [torch.full((x.shape[0], d // g), -1.0, dtype=torch.float32, device="cuda") for x in xs]
    outs = [torch.full((x.shape[0], d), 77.0, dtype=torch.float16, device="cuda") for x in xs]
    h = [p.handle for p in plans]
    B.srft_kv_quantize_batched(B.BatchTable(h, xs, codes, scales))
    B.srft_kv_dequantize_batched(B.BatchTable(h, outs, codes, scales))
    torch.cuda.synchronize()
    return codes, scales, outs


def _assert_same(ref, got):
    for i, (r, c, s, o) in enumerate(zip(ref, *got)):
        assert torch.equal(r[0], c), f"codes of entry {i}"
        assert torch.equal(r[1].view(torch.int32), s.view(torch.int32)), f"scales of entry {i}"
        assert torch.equal(r[2].view(torch.int16), o.view(torch.int16)), f"output of entry {i}"


@pytest.mark.parametrize("d,g", [(64, 32), (96, 32), (128, 32), (256, 32), (128, 16), (128, 128), (96, 96)])
def test_batched_equals_per_plan_calls(B, d, g):
    counts = [1, 31, 32, 33, 0, 257, 1000, 64]
    plans, xs, ref = _make(B, d, g, counts, seed0=100 * d + g)
    _assert_same(ref, _batched(B, plans, xs, d, g))
    for p in plans:
        p.close()


def test_more_entries_than_one_launch_holds(B):
    d, g = 96, 32
    counts = [8 + (i % 5) for i in range(101)]          # 101 entries: launches of 64 + 37
    plans, xs, ref = _make(B, d, g, counts, seed0=4242)
    _assert_same(ref, _batched(B, plans, xs, d, g))
    for p in plans:
        p.close()


def test_workgroups_are_shared_out_when_tiles_exceed_the_grid(B):
    d, g = 128, 32
    counts = [5000, 40, 90000, 1, 2049]
    for cap in (3, 64):                                  # 3 < number of entries: every entry still gets one
        plans, xs, ref = _make(B, d, g, counts, seed0=77, cap=cap)
        _assert_same(ref, _batched(B, plans, xs, d, g))
        for p in plans:
            p.close()
    plans, xs, ref = _make(B, d, g, [400000, 300000, 500000], seed0=78)     # default grid < 37,500 tiles
    _assert_same(ref, _batched(B, plans, xs, d, g))
    for p in plans:
        p.close()


def test_decode_append_of_the_d96_workload_against_the_oracle(B):
    """All 64 plans of the workload append their step's 512 vectors in one call per direction."""
    w = W.WORKLOADS["decode-d96"]
    n = w.append_vectors_per_plan
    plans, lams, xs = [], [], []
    for pi in range(w.n_plans):
        seed, lam, _ = W.plan_constants(w, pi)
        plans.append(B.Plan(w.d, w.g, seed, lam))
        lams.append(lam)
        xs.append(W.make_kv(w, pi, n_vec=n, device="cuda"))
    codes, scales, outs = _batched(B, plans, xs, w.d, w.g)
    mism = tot = 0
    for pi in range(w.n_plans):
        xh, c, sc, o = (t.cpu().numpy() for t in (xs[pi], codes[pi], scales[pi], outs[pi]))
        q = P.check_quantize(xh, plans[pi].signs, lams[pi], w.g, c, sc)
        assert q["ill_conditioned_groups"] == 0
        P.check_dequantize(c, sc, plans[pi].signs, lams[pi], w.g, o)
        mism += q["mismatches"]
        tot += q["n"] * w.d
    print(f"decode-d96 append, batched: {w.n_plans} plans x {n} vectors, {mism} boundary mismatches of {tot}")
    assert mism / tot < 1e-4
    for p in plans:
        p.close()


def test_counts_can_shrink_between_calls_and_untouched_rows_stay(B):
    d, g = 96, 32
    plans, xs, ref = _make(B, d, g, [300, 300, 300], seed0=9)
    h = [p.handle for p in plans]
    codes = [torch.full((300, d // 2), 0xAB, dtype=torch.uint8, device="cuda") for _ in xs]
    scales = [torch.full((300, d // g), -1.0, dtype=torch.float32, device="cuda") for _ in xs]
    table = B.BatchTable(h, xs, codes, scales)
    table.set_counts([300, 0, 45])
    B.srft_kv_quantize_batched(table)
    torch.cuda.synchronize()
    assert torch.equal(codes[0], ref[0][0])
    assert bool((codes[1] == 0xAB).all()) and bool((scales[1] == -1.0).all())
    assert torch.equal(codes[2][:45], ref[2][0][:45]) and bool((codes[2][45:] == 0xAB).all())
    assert torch.equal(scales[2][:45], ref[2][1][:45]) and bool((scales[2][45:] == -1.0).all())
    for p in plans:
        p.close()


def test_batched_argument_errors(B):
    L = B.lib()
    p96, p128, p96g = B.Plan(96, 32, 1), B.Plan(128, 32, 1), B.Plan(96, 96, 1)
    x = torch.zeros(64, 96, dtype=torch.float16, device="cuda")
    c = torch.full((64, 48), 0xAB, dtype=torch.uint8, device="cuda")
    s = torch.zeros(64, 3, dtype=torch.float32, device="cuda")

    def call(handles, xp, n, cp, sp, count=None):
        k = len(handles)
        return L.srft_kv_quantize_batched((C.c_void_p * k)(*handles), (C.c_void_p * k)(*xp), (C.c_int64 * k)(*n),
                                          (C.c_void_p * k)(*cp), (C.c_void_p * k)(*sp), k if count is None else count,
                                          None)

    ptrs = (x.data_ptr(), c.data_ptr(), s.data_ptr())
    assert call([p96.handle, p128.handle], [ptrs[0]] * 2, [4, 4], [ptrs[1]] * 2, [ptrs[2]] * 2) == -8
    assert call([p96.handle, p96g.handle], [ptrs[0]] * 2, [4, 4], [ptrs[1]] * 2, [ptrs[2]] * 2) == -8
    assert call([p96.handle, None], [ptrs[0]] * 2, [4, 4], [ptrs[1]] * 2, [ptrs[2]] * 2) == -1
    assert call([p96.handle, p96.handle], [ptrs[0], None], [4, 4], [ptrs[1]] * 2, [ptrs[2]] * 2) == -1
    assert call([p96.handle, p96.handle], [ptrs[0], None], [4, 0], [ptrs[1]] * 2, [ptrs[2]] * 2) == 0   # skipped entry
    assert call([p96.handle, p96.handle], [ptrs[0]] * 2, [4, -1], [ptrs[1]] * 2, [ptrs[2]] * 2) == -7
    assert call([p96.handle, p96.handle], [ptrs[0], ptrs[0] + 8], [4, 4], [ptrs[1]] * 2, [ptrs[2]] * 2) == -5
    assert call([p96.handle], [ptrs[0]], [4], [ptrs[1]], [ptrs[2]], count=-1) == -7
    torch.cuda.synchronize()
    # a rejected batch enqueued nothing: only the accepted call's 4 rows (zero vectors -> zero codes) were written
    assert bool((c[:4] == 0).all()) and bool((c[4:] == 0xAB).all())
    with pytest.raises(B.SrftError):
        B.srft_kv_quantize_batched(B.BatchTable([p96.handle, p128.handle], [x, x], [c, c], [s, s]))
    for p in (p96, p128, p96g):
        p.close()


def test_full_size_plans_in_the_launch_shape_the_benchmark_times(B):
    """Three plans of the Llama-70B-shaped workload at their full 1,048,576 vectors: the batched read path (what
    bench.py launches) gives the bytes of the per-plan calls, which the parity tests check against the oracle on a
    sample; the batched write path likewise."""
    w = W.WORKLOADS["llama3-70b-128k"]
    n = w.vectors_per_plan
    plans, xs = [], []
    for pi in (0, 1, 159):
        seed, lam, _ = W.plan_constants(w, pi)
        plans.append(B.Plan(w.d, w.g, seed, lam))
        xs.append(W.make_kv(w, pi, n_vec=n, device="cuda"))
    ref = []
    for p, x in zip(plans, xs):
        c, s = p.quantize(x)
        ref.append((c, s, p.dequantize(c, s)))
    got = _batched(B, plans, xs, w.d, w.g)
    _assert_same(ref, got)
    # oracle on a sample of the batched output (first and last tile of every plan included)
    rng = np.random.RandomState(0)
    for i, p in enumerate(plans):
        idx = np.unique(np.concatenate([np.arange(32), np.arange(n - 32, n), rng.randint(0, n, size=4096)]))
        it = torch.from_numpy(idx).cuda()
        _, lam, _ = W.plan_constants(w, (0, 1, 159)[i])
        c, s, o = (t[it].cpu().numpy() for t in got[0][i:i + 1] + got[1][i:i + 1] + got[2][i:i + 1])
        assert P.check_quantize(xs[i][it].cpu().numpy(), p.signs, lam, w.g, c, s)["ill_conditioned_groups"] == 0
        P.check_dequantize(c, s, p.signs, lam, w.g, o)
    for p in plans:
        p.close()
