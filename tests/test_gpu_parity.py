"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import srft_oracle as O
from paper_2605_05699_amd import workloads as W
from tests import parity_util as P

pytestmark = pytest.mark.gpu

ALL_D = [32, 64, 96, 128, 160, 192, 224, 256]
MAIN_D = [96, 128, 256]


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2605_05699_amd import binding
    binding.lib()      # raises if the HIP library is not built: no fallback
    return binding


def _run_both(B, d, n, seed, lam=None, x=None, g=32):
    if x is None:
        x = W.gaussian_with_outliers(n, d, seed=seed, outliers=max(1, d // 64), gain=20.0)
    lam = W.lognormal_lambda(d, seed=seed + 1) if lam is None else lam
    plan = B.Plan(d, g, seed, lam)
    s = plan.signs
    xd = torch.from_numpy(x).cuda()
    codes, scales = plan.quantize(xd)
    out = plan.dequantize(codes, scales)
    torch.cuda.synchronize()
    res = (x, s, lam, codes.cpu().numpy(), scales.cpu().numpy(), out.cpu().numpy())
    plan.close()
    return res


@pytest.mark.parametrize("d", ALL_D)
def test_signs_come_from_the_same_stream_as_the_oracles(B, d):
    for seed in (0, 1, 2 ** 63 + 5, 2 ** 64 - 1):
        plan = B.Plan(d, 32, seed)
        assert np.array_equal(plan.signs, O.signs_from_seed(seed, d))
        plan.close()


@pytest.mark.parametrize("d", ALL_D)
def test_transform_alone_matches_eq1_eq2(B, d):
    n = 203
    x = W.gaussian_with_outliers(n, d, seed=d)
    lam = W.lognormal_lambda(d, seed=5)
    plan = B.Plan(d, 32, 99, lam)
    w = plan.forward_f32(torch.from_numpy(x).cuda()).cpu().numpy().astype(np.float64)
    ref = O.srft_forward(x, plan.signs) * lam.astype(np.float64)
    scale = np.abs(ref).max(axis=1, keepdims=True)
    assert (np.abs(w - ref) / scale).max() < 2e-6
    plan.close()
    # lambda = 1: orthonormal on the GPU as well
    plan = B.Plan(d, 32, 7)
    z = plan.forward_f32(torch.from_numpy(x).cuda()).cpu().numpy().astype(np.float64)
    xf = x.astype(np.float64)
    assert np.abs(np.linalg.norm(z, axis=1) / np.linalg.norm(xf, axis=1) - 1).max() < 1e-5
    plan.close()


@pytest.mark.parametrize("d", ALL_D)
@pytest.mark.parametrize("n", [1, 31, 32, 33, 1003])
def test_quantize_and_dequantize_match_oracle(B, d, n):
    x, s, lam, codes, scales, out = _run_both(B, d, n, seed=1000 * d + n)
    q = P.check_quantize(x, s, lam, 32, codes, scales)
    r = P.check_dequantize(codes, scales, s, lam, 32, out)
    if n * d >= 10_000:        # rates mean something only with enough elements
        assert q["mismatch_rate"] < 1e-3
        assert r["bit_identical_fraction"] > 0.99


GROUP_CASES = [(128, 16), (128, 64), (128, 128), (96, 16), (96, 96), (256, 16), (256, 64), (256, 128), (256, 256),
               (64, 16), (64, 64), (192, 96), (32, 16), (160, 160)]


@pytest.mark.parametrize("d,g", GROUP_CASES)
@pytest.mark.parametrize("n", [33, 2531])
def test_other_group_sizes_match_oracle(B, d, g, n):
    # g = 16, multiples of 32, and the per-token quantizer g = d (Sec. 3.2 step 3)
    x, s, lam, codes, scales, out = _run_both(B, d, n, seed=7 * d + g + n, g=g)
    assert scales.shape == (n, d // g)
    q = P.check_quantize(x, s, lam, g, codes, scales)
    r = P.check_dequantize(codes, scales, s, lam, g, out)
    if n > 1000:
        assert q["mismatch_rate"] < 1e-3 and r["bit_identical_fraction"] > 0.99


def test_group_sizes_do_not_depend_on_the_grid(B):
    d, n = 128, 3000
    x = torch.from_numpy(W.gaussian_with_outliers(n, d, seed=5)).cuda()
    for g in (16, 64, 128):
        plan = B.Plan(d, g, 5, W.lognormal_lambda(d, 5))
        c0, s0 = plan.quantize(x)
        o0 = plan.dequantize(c0, s0)
        for cap in (1, 5):
            B.srft_plan_set_max_workgroups(plan.handle, cap)
            c1, s1 = plan.quantize(x)
            o1 = plan.dequantize(c1, s1)
            assert torch.equal(c0, c1) and torch.equal(s0, s1) and torch.equal(o0, o1)
        plan.close()


@pytest.mark.parametrize("d", MAIN_D)
def test_larger_batch_spanning_many_workgroups(B, d):
    n = 70_001                     # > 2000 tiles with a ragged tail: every workgroup loops
    x, s, lam, codes, scales, out = _run_both(B, d, n, seed=d)
    q = P.check_quantize(x, s, lam, 32, codes, scales)
    r = P.check_dequantize(codes, scales, s, lam, 32, out)
    print(f"d={d} n={n} code mismatch rate {q['mismatch_rate']:.2e} scale rel {q['scale_max_rel']:.2e} "
          f"fp16-identical {r['bit_identical_fraction']:.6f} worst/tol {r['worst_over_tol']:.3f}")
    assert q["mismatch_rate"] < 1e-4


@pytest.mark.parametrize("d", MAIN_D)
def test_every_nibble_value_at_every_position_is_decoded(B, d):
    # one non-zero nibble per vector: the output is q * scale * (a column of the inverse), which identifies
    # both the position and the 4-bit two's-complement value, -8 included.
    vals = list(range(-8, 8))
    n = d * len(vals)
    q = np.zeros((n, d), dtype=np.int8)
    for k in range(d):
        for i, v in enumerate(vals):
            q[k * len(vals) + i, k] = v
    codes = O.pack_nibbles(q)
    rng = np.random.RandomState(0)
    scales = rng.uniform(0.5, 2.0, size=(n, d // 32)).astype(np.float32)
    lam = W.lognormal_lambda(d, seed=3)
    plan = B.Plan(d, 32, 11, lam)
    out = plan.dequantize(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda()).cpu().numpy()
    P.check_dequantize(codes, scales, plan.signs, lam, 32, out)
    plan.close()


@pytest.mark.parametrize("d,g", [(128, 32), (128, 64), (128, 128), (256, 32), (256, 128), (256, 256)])
def test_codes_the_twice_folded_read_form_treats_apart(B, d, g):
    # The read kernel at d = 128 / 256 contracts cosine and sine rows, even and odd packed indices, in four separate
    # classes, brings Nyquist (p = d/2) in as an addend and takes the outputs n = d/4, 3d/4 from a row of its own.
    # One-hot records at the indices where those paths meet, every code value, wide groups included; also two vectors
    # in which only one class is populated.  Element by element against the oracle (n = 0, d/4, d/2, 3d/4 included).
    h = d // 2
    special = [0, 1, 2, 3, h // 2, h - 2, h - 1, h, h + 1, h + 2, h + h // 2, d - 2, d - 1]
    vals = list(range(-8, 8))
    q = np.zeros((len(special) * len(vals) + 4, d), dtype=np.int8)
    for a, p in enumerate(special):
        for i, v in enumerate(vals):
            q[a * len(vals) + i, p] = v
    rng = np.random.RandomState(d + g)
    tail = len(special) * len(vals)
    q[tail + 0, 0:h:2] = rng.randint(-7, 8, size=h // 2)          # even cosine codes only
    q[tail + 1, 1:h:2] = rng.randint(-7, 8, size=h // 2)          # odd cosine codes only
    q[tail + 2, h + 2:d:2] = rng.randint(-7, 8, size=h // 2 - 1)  # even sine codes only (Nyquist left out)
    q[tail + 3, h + 1:d:2] = rng.randint(-7, 8, size=h // 2)      # odd sine codes only
    codes = O.pack_nibbles(q)
    scales = rng.uniform(0.25, 4.0, size=(q.shape[0], d // g)).astype(np.float32)
    lam = W.lognormal_lambda(d, seed=d)
    plan = B.Plan(d, g, 21, lam)
    assert B.lib().srft_plan_form(plan.handle, 1) == 2
    out = plan.dequantize(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda()).cpu().numpy()
    P.check_dequantize(codes, scales, plan.signs, lam, g, out)
    plan.close()


@pytest.mark.parametrize("d", MAIN_D)
def test_random_bytes_are_decoded(B, d):
    rng = np.random.RandomState(d)
    n = 4099
    codes = rng.randint(0, 256, size=(n, d // 2)).astype(np.uint8)
    scales = np.exp(rng.standard_normal((n, d // 32))).astype(np.float32)
    scales[::7, 0] = 0.0
    lam = W.lognormal_lambda(d, seed=9)
    plan = B.Plan(d, 32, 12, lam)
    out = plan.dequantize(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda()).cpu().numpy()
    P.check_dequantize(codes, scales, plan.signs, lam, 32, out)
    plan.close()


def test_zero_vectors_zero_groups_and_empty_input(B):
    d = 128
    plan = B.Plan(d, 32, 3, W.lognormal_lambda(d, 1))
    x = W.gaussian_with_outliers(64, d, seed=2)
    x[5] = 0
    x[6] = -0.0
    xd = torch.from_numpy(x).cuda()
    codes, scales = plan.quantize(xd)
    out = plan.dequantize(codes, scales)
    c, sc, o = codes.cpu().numpy(), scales.cpu().numpy(), out.cpu().numpy()
    assert not c[5].any() and not sc[5].any() and not o[5].any()
    assert not c[6].any() and not sc[6].any() and not o[6].any()
    P.check_quantize(x, plan.signs, W.lognormal_lambda(d, 1), 32, c, sc)
    # a vector whose transform has an all-zero group: x = s * cos(2 pi 3 n / d) has a single packed coefficient
    nn = np.arange(d)
    x1 = (plan.signs * np.cos(2 * np.pi * 3 * nn / d) * 4).astype(np.float16)[None]
    c1, s1 = plan.quantize(torch.from_numpy(x1).cuda())
    s1 = s1.cpu().numpy()
    assert s1[0, 0] > 0 and np.all(s1[0, 1:] < 1e-3 * s1[0, 0])
    P.check_quantize(x1, plan.signs, W.lognormal_lambda(d, 1), 32, c1.cpu().numpy(), s1)
    # n = 0 is a successful no-op
    e_codes, e_scales = plan.quantize(torch.empty(0, d, dtype=torch.float16, device="cuda"))
    assert e_codes.shape == (0, d // 2) and e_scales.shape == (0, 4)
    assert plan.dequantize(e_codes, e_scales).shape == (0, d)
    plan.close()


def test_large_magnitudes_and_tiny_magnitudes(B):
    d = 128
    lam = np.ones(d, dtype=np.float32)
    plan = B.Plan(d, 32, 21, lam)
    rng = np.random.RandomState(1)
    x = rng.standard_normal((256, d))
    x[:128] *= 500.0            # |x| up to ~2000: far from fp16 overflow after the inverse
    x[128:] *= 1e-4             # includes fp16 subnormals
    x = x.astype(np.float16)
    codes, scales = plan.quantize(torch.from_numpy(x).cuda())
    out = plan.dequantize(codes, scales)
    c, sc = codes.cpu().numpy(), scales.cpu().numpy()
    P.check_quantize(x, plan.signs, lam, 32, c, sc)
    P.check_dequantize(c, sc, plan.signs, lam, 32, out.cpu().numpy())
    plan.close()


def test_lambda_spanning_several_orders_of_magnitude(B):
    d = 128
    rng = np.random.RandomState(4)
    lam = np.exp(rng.uniform(np.log(1e-2), np.log(1e2), size=d)).astype(np.float32)
    x, s, lam, codes, scales, out = _run_both(B, d, 2000, seed=77, lam=lam)
    P.check_quantize(x, s, lam, 32, codes, scales)
    P.check_dequantize(codes, scales, s, lam, 32, out)


def test_grid_cap_and_side_stream_give_identical_bytes(B):
    d, n = 128, 5000
    x = W.gaussian_with_outliers(n, d, seed=8)
    lam = W.lognormal_lambda(d, 8)
    plan = B.Plan(d, 32, 8, lam)
    xd = torch.from_numpy(x).cuda()
    c0, s0 = plan.quantize(xd)
    o0 = plan.dequantize(c0, s0)
    torch.cuda.synchronize()
    for cap in (1, 7, 100):
        B.srft_plan_set_max_workgroups(plan.handle, cap)
        c1, s1 = plan.quantize(xd)
        o1 = plan.dequantize(c1, s1)
        assert torch.equal(c0, c1) and torch.equal(s0, s1) and torch.equal(o0, o1)
    B.srft_plan_set_max_workgroups(plan.handle, 0)
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        c2, s2 = plan.quantize(xd, stream=st)
        o2 = plan.dequantize(c2, s2, stream=st)
    st.synchronize()
    assert torch.equal(c0, c2) and torch.equal(s0, s2) and torch.equal(o0, o2)
    plan.close()


@pytest.mark.parametrize("d,g,bits", [(128, 32, 4), (256, 32, 4), (192, 32, 4), (96, 32, 4), (64, 32, 4),
                                      (128, 128, 4), (256, 64, 8), (128, 16, 4)])
def test_every_pipeline_length_of_one_workgroup(B, d, g, bits):
    # One workgroup walks m tiles, m = 1..7 (odd and even numbers of stages, with and without a ragged last
    # tile): prologue, steady state and every epilogue of the software pipelines.  The reference is the same
    # input on the full grid (one tile per workgroup), which the other tests hold against the oracle.
    lam = W.lognormal_lambda(d, d + g)
    plan = B.Plan(d, g, 3, lam, bits=bits)
    for m in range(1, 8):
        for n in (32 * m, 32 * m - 13):
            x = torch.from_numpy(W.gaussian_with_outliers(n, d, seed=100 * m + n % 7, outliers=1, gain=25.0)).cuda()
            B.srft_plan_set_max_workgroups(plan.handle, 0)
            c0, s0 = plan.quantize(x)
            o0 = plan.dequantize(c0, s0)
            B.srft_plan_set_max_workgroups(plan.handle, 1)
            c1, s1 = plan.quantize(x)
            o1 = plan.dequantize(c1, s1)
            assert torch.equal(c0, c1) and torch.equal(s0, s1) and torch.equal(o0, o1), (m, n)
            if m in (1, 2, 5):
                P.check_quantize(x.cpu().numpy(), plan.signs, lam, g, c1.cpu().numpy(), s1.cpu().numpy(), bits=bits)
    plan.close()


def test_argument_errors_on_device_pointers(B):
    d = 128
    plan = B.Plan(d, 32, 1)
    x = torch.zeros(9, d, dtype=torch.float16, device="cuda")
    codes = torch.zeros(8 * d // 2 + 16, dtype=torch.uint8, device="cuda")
    scales = torch.zeros(8, 4, dtype=torch.float32, device="cuda")
    L = B.lib()
    # misaligned input (offset by one fp16) and misaligned codes (offset by one byte)
    assert L.srft_kv_quantize(plan.handle, x.data_ptr() + 2, 8, codes.data_ptr(), scales.data_ptr(), None) == -5
    assert L.srft_kv_quantize(plan.handle, x.data_ptr(), 8, codes.data_ptr() + 1, scales.data_ptr(), None) == -5
    assert L.srft_kv_quantize(plan.handle, None, 8, codes.data_ptr(), scales.data_ptr(), None) == -1
    assert L.srft_kv_quantize(plan.handle, x.data_ptr(), -1, codes.data_ptr(), scales.data_ptr(), None) == -7
    assert L.srft_kv_dequantize(plan.handle, codes.data_ptr(), scales.data_ptr(), 8, x.data_ptr() + 2, None) == -5
    assert L.srft_kv_dequantize(None, codes.data_ptr(), scales.data_ptr(), 8, x.data_ptr(), None) == -1
    # more vectors than the kernels' 32-bit tile indices cover (2^33) are refused before anything is launched
    too_many = 2 ** 33 + 1
    assert L.srft_kv_quantize(plan.handle, x.data_ptr(), too_many, codes.data_ptr(), scales.data_ptr(), None) == -7
    assert L.srft_kv_dequantize(plan.handle, codes.data_ptr(), scales.data_ptr(), too_many, x.data_ptr(), None) == -7
    assert L.srft_kv_forward_f32(plan.handle, x.data_ptr(), too_many, scales.data_ptr(), None) == -7
    torch.cuda.synchronize()
    plan.close()


# ----------------------------------------------------------------------------- the five workloads
def _plan_for(B, w, plan_idx):
    seed, lam, _ = W.plan_constants(w, plan_idx)
    return B.Plan(w.d, w.g, seed, lam), lam


def _full_parity(B, w, plans, n_vec=None):
    stats = []
    for pi in plans:
        plan, lam = _plan_for(B, w, pi)
        x = W.make_kv(w, pi, n_vec=n_vec, device="cuda")
        codes, scales = plan.quantize(x)
        out = plan.dequantize(codes, scales)
        xh, c, sc, o = x.cpu().numpy(), codes.cpu().numpy(), scales.cpu().numpy(), out.cpu().numpy()
        q = P.check_quantize(xh, plan.signs, lam, w.g, c, sc)
        r = P.check_dequantize(c, sc, plan.signs, lam, w.g, o)
        # the workloads' data has no cancellation-dominated group: nothing is exempt from the relative checks
        assert q["ill_conditioned_groups"] == 0, (w.name, pi, q["ill_conditioned_groups"])
        stats.append((pi, q["n"], q["mismatches"], q["scale_max_rel"], r["bit_identical_fraction"]))
        plan.close()
    tot = sum(s[1] for s in stats) * w.d
    mism = sum(s[2] for s in stats)
    print(f"{w.name}: {len(stats)} plans, {tot} codes, {mism} boundary mismatches ({mism / tot:.2e}), "
          f"max scale rel err {max(s[3] for s in stats):.2e}, min fp16-identical {min(s[4] for s in stats):.6f}")
    assert mism / tot < 1e-4


def test_workload_tiny_full(B):
    _full_parity(B, W.WORKLOADS["tiny"], plans=[0, 1])


def test_workload_qwen_full(B):
    w = W.WORKLOADS["qwen2.5-1.5b-4k"]
    _full_parity(B, w, plans=range(w.n_plans))


def test_workload_gemma_full(B):
    w = W.WORKLOADS["gemma3-1b-4k"]
    _full_parity(B, w, plans=range(w.n_plans))


def _sampled_parity(B, w, plan_idx, n_vec, quant=True):
    """One launch at full size; oracle on a seeded >= 1% sample that includes the first and last tile."""
    plan, lam = _plan_for(B, w, plan_idx)
    x = W.make_kv(w, plan_idx, n_vec=n_vec, device="cuda")
    codes, scales = plan.quantize(x)
    out = plan.dequantize(codes, scales)
    torch.cuda.synchronize()
    rng = np.random.RandomState(plan_idx)
    k = max(4096, n_vec // 100)
    idx = np.unique(np.concatenate([np.arange(32), np.arange(n_vec - 32, n_vec),
                                    rng.randint(0, n_vec, size=k)]))
    it = torch.from_numpy(idx).cuda()
    xh, c, sc, o = (t[it].cpu().numpy() for t in (x, codes, scales, out))
    q = P.check_quantize(xh, plan.signs, lam, w.g, c, sc)
    r = P.check_dequantize(c, sc, plan.signs, lam, w.g, o)
    assert q["ill_conditioned_groups"] == 0, (w.name, plan_idx, q["ill_conditioned_groups"])
    # whole-tensor properties that hold at any size: code range and (scale == 0) <=> (all codes zero)
    lo, hi = codes & 0xF, codes >> 4
    assert int(((lo == 8) | (hi == 8)).sum()) == 0, "nibble -8 produced by the write path"
    grp = codes.view(n_vec, w.d // w.g, w.g // 2)
    zero_grp = (grp == 0).all(dim=-1)
    assert torch.equal(zero_grp, scales == 0)
    assert torch.isfinite(out).all() and torch.isfinite(scales).all()
    # every non-zero group contains a code of magnitude 7
    mag7 = ((lo == 7) | (lo == 9) | (hi == 7) | (hi == 9)).view(n_vec, w.d // w.g, w.g // 2).any(dim=-1)
    assert torch.equal(mag7, scales > 0)
    # round-trip error bound from orthogonality, evaluated on the GPU for every vector:
    # ||xhat - x||^2 <= sum_k (scale_j / (2 lambda_k))^2, plus fp16 output rounding
    lam_t = torch.from_numpy(lam).cuda().double()
    bound = ((scales.double().repeat_interleave(w.g, dim=1) / (2 * lam_t)) ** 2).sum(1)
    err = ((out.double() - x.double()) ** 2).sum(1)
    slack = out.double().norm(dim=1) * 2.0 ** -11 * 1.01 + 1e-7       # |fp16(v) - v| <= 2^-11 |v|
    assert bool((err.sqrt() <= bound.sqrt() * (1 + 1e-4) + slack).all())
    print(f"{w.name} plan {plan_idx}: {n_vec} vectors in one launch, {len(idx)} checked one by one, "
          f"{q['mismatches']} boundary mismatches, fp16-identical {r['bit_identical_fraction']:.6f}")
    plan.close()


def test_workload_decode_append_and_prefix(B):
    w = W.WORKLOADS["decode-d96"]
    # append step: 512 new vectors per plan; full parity on a few plans
    _full_parity(B, w, plans=[0, 1, 62, 63], n_vec=w.append_vectors_per_plan)
    # prefix read: one plan's full 4,194,304-vector prefix in one launch, three more plans at 262,144 vectors
    _sampled_parity(B, w, 5, w.vectors_per_plan)
    for pi in (0, 31, 63):
        _sampled_parity(B, w, pi, 262_144)


def test_workload_llama70b_full_size_launch(B):
    w = W.WORKLOADS["llama3-70b-128k"]
    # two plans at the full 1,048,576 vectors of a launch, six more spread over the 160 at 65,536 vectors
    for pi in (0, 159):
        _sampled_parity(B, w, pi, w.vectors_per_plan)
    for pi in (1, 40, 41, 80, 119, 158):
        _sampled_parity(B, w, pi, 65_536)


def test_d256_at_the_launch_size_the_bench_times(B):
    # d = 256 (the Gemma-shaped plans' constants and data) at 1,048,576 vectors per launch: the shape of the bench's
    # d = 256 line.  Write path per plan, read path through the batched entry point over all plans at once, which
    # must give the same bytes as the per-plan launches that the sampled check holds against the oracle.
    w = W.WORKLOADS["gemma3-1b-4k"]
    n = 1 << 20
    for pi in (0, 51):
        _sampled_parity(B, w, pi, n)
    plans, xs = [], []
    for pi in (2, 3, 4):
        plan, _ = _plan_for(B, w, pi)
        plans.append(plan)
        xs.append(W.make_kv(w, pi, n_vec=n, device="cuda"))
    recs = [pl.quantize(x) for pl, x in zip(plans, xs)]
    outs = [pl.dequantize(c, sc) for pl, (c, sc) in zip(plans, recs)]
    batched = [torch.empty_like(o) for o in outs]
    table = B.BatchTable([pl.handle for pl in plans], batched, [c for c, _ in recs], [sc for _, sc in recs])
    B.srft_kv_dequantize_batched(table)
    torch.cuda.synchronize()
    for a, b in zip(outs, batched):
        assert torch.equal(a, b)
    for pl in plans:
        pl.close()


@pytest.mark.parametrize("name,n_write,n_read", [("llama3-70b-128k", 16, 4), ("gemma3-1b-4k", 8, 4)])
def test_plans_per_launch_as_the_bench_times_them(B, name, n_write, n_read):
    # bench.py puts 16 (write path) and 4 (read path) plans of 1,048,576 vectors into every launch of the headline
    # workload (d = 128), and 8 (write: all of its plans) and 4 (read) into its d = 256 side measurement.  The batched launches must produce the
    # bytes of the per-plan launches, which _sampled_parity holds against the oracle at this size (plans 0 and 159 /
    # 0 and 51 above).
    w = W.WORKLOADS[name]
    n = 1 << 20
    ids = list(range(n_write // 2)) + list(range(w.n_plans - n_write // 2, w.n_plans))
    plans, xs = [], []
    for pi in ids:
        plan, _ = _plan_for(B, w, pi)
        plans.append(plan)
        xs.append(W.make_kv(w, pi, n_vec=n, device="cuda"))
    recs = [pl.quantize(x) for pl, x in zip(plans, xs)]
    h = [pl.handle for pl in plans]
    codes_b = [torch.empty_like(c) for c, _ in recs]
    scales_b = [torch.empty_like(sc) for _, sc in recs]
    B.srft_kv_quantize_batched(B.BatchTable(h, xs, codes_b, scales_b))
    torch.cuda.synchronize()
    for (c, sc), cb, sb in zip(recs, codes_b, scales_b):
        assert torch.equal(c, cb) and torch.equal(sc, sb)
    del xs
    pick = [0, 1, len(ids) - 2, len(ids) - 1][:n_read]
    outs = [plans[i].dequantize(*recs[i]) for i in pick]
    outs_b = [torch.empty_like(o) for o in outs]
    B.srft_kv_dequantize_batched(B.BatchTable([h[i] for i in pick], outs_b, [codes_b[i] for i in pick],
                                              [scales_b[i] for i in pick]))
    torch.cuda.synchronize()
    for o, ob in zip(outs, outs_b):
        assert torch.equal(o, ob)
    for pl in plans:
        pl.close()


def test_single_launch_beyond_4_gib(B):
    # 20,000,003 vectors of d = 128: 5.1 GB of fp16 in one launch, so tile bases pass 2^32 bytes (64-bit scalar
    # base + 32-bit lane offset) and the last tile is ragged; sampled rows against the oracle, properties on all.
    _sampled_parity(B, W.WORKLOADS["llama3-70b-128k"], 7, 20_000_003)



def test_plan_form_reports_the_factorisation_each_plan_runs(B):
    """srft_plan_form is what bench.py names the timed kernel by: once-folded write path at d = 128, twice-folded at
    d = 256 with g = 32, plain elsewhere; twice-folded read path at d = 128 and 256, once-folded at d = 192, with g >= 32."""
    L = B.lib()
    expect = {(128, 32, "dft"): (1, 2), (256, 32, "dft"): (2, 2), (256, 64, "dft"): (1, 2), (96, 32, "dft"): (0, 0),
              (192, 32, "dft"): (0, 1), (64, 32, "dft"): (0, 0), (128, 16, "dft"): (0, 0), (128, 32, "hadamard"): (0, 0)}
    for (d, g, tr), (fw, fr) in expect.items():
        plan = B.Plan(d, g, 1, None, transform=tr)
        assert (L.srft_plan_form(plan.handle, 0), L.srft_plan_form(plan.handle, 1)) == (fw, fr), (d, g, tr)
        assert L.srft_plan_form(plan.handle, 2) == -7
        plan.close()
    assert L.srft_plan_form(None, 0) == -1
