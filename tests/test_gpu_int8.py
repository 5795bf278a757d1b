"""GPU parity of the 8-bit code width (scale = abs-max / 127, one byte per value) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import srft_oracle as O
from paper_2605_05699_amd import workloads as W
from tests import parity_util as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2605_05699_amd import binding
    binding.lib()
    return binding


def _run(B, d, g, n, seed):
    x = W.gaussian_with_outliers(n, d, seed=seed, outliers=max(1, d // 64), gain=20.0)
    lam = W.lognormal_lambda(d, seed=seed + 1)
    plan = B.Plan(d, g, seed, lam, bits=8)
    assert plan.code_bytes == d and B.lib().srft_plan_bits(plan.handle) == 8
    codes, scales = plan.quantize(torch.from_numpy(x).cuda())
    out = plan.dequantize(codes, scales)
    torch.cuda.synchronize()
    res = (x, plan.signs, lam, codes.cpu().numpy(), scales.cpu().numpy(), out.cpu().numpy())
    plan.close()
    return res


@pytest.mark.parametrize("d", [32, 64, 96, 128, 160, 192, 224, 256])
@pytest.mark.parametrize("n", [1, 33, 2531])
def test_int8_quantize_and_dequantize_match_oracle(B, d, n):
    x, s, lam, codes, scales, out = _run(B, d, 32, n, seed=3000 * d + n)
    q = P.check_quantize(x, s, lam, 32, codes, scales, bits=8)
    r = P.check_dequantize(codes, scales, s, lam, 32, out, bits=8)
    if n * d >= 10_000:
        assert q["mismatch_rate"] < 5e-3           # the paper reports 99.997 - 99.999 % identical int8 values
        assert r["bit_identical_fraction"] > 0.99
        # the 8-bit reconstruction is far closer to the input than 4 bits allow
        err = np.linalg.norm(out.astype(np.float64) - x.astype(np.float64)) / np.linalg.norm(x.astype(np.float64))
        assert err < 0.02


@pytest.mark.parametrize("d,g", [(128, 16), (128, 64), (128, 128), (96, 96), (256, 16), (256, 256), (64, 64)])
def test_int8_other_group_sizes(B, d, g):
    x, s, lam, codes, scales, out = _run(B, d, g, 700, seed=17 * d + g)
    P.check_quantize(x, s, lam, g, codes, scales, bits=8)
    P.check_dequantize(codes, scales, s, lam, g, out, bits=8)


@pytest.mark.parametrize("d", [96, 128, 256])
def test_every_byte_value_is_decoded(B, d):
    """One-hot codes: every byte value at every position, scale 1, lambda 1 -> column of Q^T times the value."""
    plan = B.Plan(d, 32, 5, bits=8)
    s = plan.signs
    vals = np.arange(256, dtype=np.uint8)
    for pos in (0, 1, 2, 3, d // 2 - 1, d // 2, d - 2, d - 1, 37 % d):
        codes = np.zeros((256, d), dtype=np.uint8)
        codes[:, pos] = vals
        scales = np.ones((256, d // 32), dtype=np.float32)
        out = plan.dequantize(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda()).cpu().numpy()
        P.check_dequantize(codes, scales, s, np.ones(d, dtype=np.float32), 32, out, bits=8)
    rng = np.random.RandomState(1)
    codes = rng.randint(0, 256, size=(999, d)).astype(np.uint8)
    scales = np.exp(rng.standard_normal((999, d // 32))).astype(np.float32)
    out = plan.dequantize(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda()).cpu().numpy()
    P.check_dequantize(codes, scales, s, np.ones(d, dtype=np.float32), 32, out, bits=8)
    plan.close()


def test_int8_batched_cache_and_errors(B):
    d, g = 128, 32
    L = B.lib()
    import ctypes as C
    h = C.c_void_p()
    for bits in (0, 2, 5, 16):
        assert L.srft_plan_create_bits(C.byref(h), d, g, bits, 0, None) == -9
    # batched == per-plan, bitwise; a 4-bit and an 8-bit plan do not mix
    plans = [B.Plan(d, g, 40 + i, W.lognormal_lambda(d, seed=i), bits=8) for i in range(3)]
    xs = [torch.from_numpy(W.gaussian_with_outliers(n, d, seed=60 + i)).cuda() for i, n in enumerate((33, 1000, 64))]
    ref = [p.quantize(x) for p, x in zip(plans, xs)]
    codes = [torch.zeros_like(r[0]) for r in ref]
    scales = [torch.zeros_like(r[1]) for r in ref]
    outs = [torch.zeros(x.shape[0], d, dtype=torch.float16, device="cuda") for x in xs]
    hs = [p.handle for p in plans]
    B.srft_kv_quantize_batched(B.BatchTable(hs, xs, codes, scales))
    B.srft_kv_dequantize_batched(B.BatchTable(hs, outs, codes, scales))
    torch.cuda.synchronize()
    for i in range(3):
        assert torch.equal(codes[i], ref[i][0]) and torch.equal(scales[i], ref[i][1])
        assert torch.equal(outs[i], plans[i].dequantize(*ref[i]))
    p4 = B.Plan(d, g, 1)
    with pytest.raises(B.SrftError):
        B.srft_kv_quantize_batched(B.BatchTable([hs[0], p4.handle], xs[:2], codes[:2], scales[:2]))
    # cache manager with 8-bit plans
    from oracle import cache_oracle as CO
    n_seq, R, T = 4, 16, 37
    x = [W.gaussian_with_outliers(n_seq * T, d, seed=80 + i).reshape(n_seq, T, d) for i in range(3)]
    cache = B.Cache(plans, n_seq, 48, R)
    cache.append([torch.from_numpy(v).cuda() for v in x])
    torch.cuda.synchronize()
    assert cache.quantized_tokens == 32
    for i in range(3):
        cg = cache.codes[i].permute(1, 0, 2, 3).reshape(n_seq, 48, d)[:, :32].cpu().numpy().reshape(-1, d)
        sg = cache.scales[i].permute(1, 0, 2, 3).reshape(n_seq, 48, d // g)[:, :32].cpu().numpy().reshape(-1, d // g)
        vw = cache.view[i].permute(1, 0, 2, 3).reshape(n_seq, 48, d)[:, :T].cpu().numpy()
        lam = W.lognormal_lambda(d, seed=i)
        P.check_quantize(x[i][:, :32].reshape(-1, d), plans[i].signs, lam, g, cg, sg, bits=8)
        P.check_dequantize(cg, sg, plans[i].signs, lam, g, vw[:, :32].reshape(-1, d), bits=8)
        assert np.array_equal(vw[:, 32:].view(np.uint16), x[i][:, 32:].view(np.uint16))
    cache.close()
    p4.close()
    for p in plans:
        p.close()
