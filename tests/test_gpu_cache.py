"""GPU parity of the cache manager (int4 store + fp16 residual window + dequantized-prefix view) against the
cache model in oracle/cache_oracle.py."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import cache_oracle as CO
from paper_2605_05699_amd import workloads as W
from tests import parity_util as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2605_05699_amd import binding
    binding.lib()
    return binding


def _tokens(paged, T):
    """[pages, n_seq, R, w] -> [n_seq, T, w] in token order (test-side layout conversion only)."""
    pages, n_seq, R, w = paged.shape
    return paged.permute(1, 0, 2, 3).reshape(n_seq, pages * R, w)[:, :T]


def _setup(B, d, g, n_plans, n_seq, seed):
    plans, lams, xs = [], [], []
    for p in range(n_plans):
        lam = W.lognormal_lambda(d, seed=seed + 10 * p)
        plans.append(B.Plan(d, g, seed + p, lam))
        lams.append(lam)
    return plans, lams


@pytest.mark.parametrize("d,R", [(128, 16), (96, 16), (256, 8), (64, 5)])
def test_cache_matches_the_model_through_a_ragged_append_schedule(B, d, R):
    g, n_plans, n_seq = 32, 3, 6
    schedule = [1, 1, 3, R, 2 * R + 1, 1, 7, R - 1, 1, 40]
    T = sum(schedule)
    capacity = -(-T // R) * R
    plans, lams = _setup(B, d, g, n_plans, n_seq, seed=31 * d + R)
    x = [W.gaussian_with_outliers(n_seq * T, d, seed=d + p, outliers=1).reshape(n_seq, T, d) for p in range(n_plans)]
    cache = B.Cache(plans, n_seq, capacity, R)
    models = [CO.ResidualWindowCache(d, g, plans[p].signs, lams[p], n_seq, R) for p in range(n_plans)]
    pos = 0
    for t in schedule:
        cache.append([torch.from_numpy(np.ascontiguousarray(x[p][:, pos:pos + t])).cuda() for p in range(n_plans)])
        for p in range(n_plans):
            models[p].append(x[p][:, pos:pos + t])
        pos += t
        assert cache.tokens == pos == models[0].tokens
        assert cache.quantized_tokens == models[0].quantized_tokens == pos // R * R
    torch.cuda.synchronize()
    n_q = cache.quantized_tokens
    for p in range(n_plans):
        view = _tokens(cache.view[p], T).cpu().numpy()
        codes = _tokens(cache.codes[p], n_q).cpu().numpy()
        scales = _tokens(cache.scales[p], n_q).cpu().numpy()
        ref = models[p].view()
        # the window is an exact copy
        assert np.array_equal(view[:, n_q:].view(np.uint16), x[p][:, n_q:].view(np.uint16))
        assert np.array_equal(view[:, n_q:].view(np.uint16), ref[:, n_q:].view(np.uint16))
        # the store against the oracle's quantizer, the prefix against the oracle's read path of the GPU's codes
        q = P.check_quantize(x[p][:, :n_q].reshape(-1, d), plans[p].signs, lams[p], g, codes.reshape(-1, d // 2),
                             scales.reshape(-1, d // g))
        assert q["ill_conditioned_groups"] == 0
        P.check_dequantize(codes.reshape(-1, d // 2), scales.reshape(-1, d // g), plans[p].signs, lams[p], g,
                           view[:, :n_q].reshape(-1, d))
        # and the prefix is what the library's own read path gives for the stored record (bitwise)
        again = plans[p].dequantize(torch.from_numpy(codes.reshape(-1, d // 2)).cuda(),
                                    torch.from_numpy(scales.reshape(-1, d // g)).cuda()).cpu().numpy()
        assert np.array_equal(again.view(np.uint16), view[:, :n_q].reshape(-1, d).view(np.uint16))
    cache.close()
    for pl in plans:
        pl.close()


def test_chunking_does_not_change_a_byte_and_the_view_can_be_rebuilt(B):
    d, g, R, n_plans, n_seq, T = 128, 32, 16, 2, 4, 83
    plans, lams = _setup(B, d, g, n_plans, n_seq, seed=5)
    x = [torch.from_numpy(W.gaussian_with_outliers(n_seq * T, d, seed=70 + p).reshape(n_seq, T, d)).cuda()
         for p in range(n_plans)]
    a = B.Cache(plans, n_seq, 96, R)
    a.append(x)                                              # everything at once: five pages flushed in one go
    b = B.Cache(plans, n_seq, 96, R)
    for j in range(T):                                       # one token at a time
        b.append([xp[:, j:j + 1].contiguous() for xp in x])
    torch.cuda.synchronize()
    assert a.tokens == b.tokens == T and a.quantized_tokens == b.quantized_tokens == 80
    for p in range(n_plans):
        assert torch.equal(a.codes[p], b.codes[p])
        assert torch.equal(a.scales[p].view(torch.int32), b.scales[p].view(torch.int32))
        assert torch.equal(a.view[p].view(torch.int16), b.view[p].view(torch.int16))
    # wipe the prefix part of the view; rebuild restores it and leaves the window alone
    keep = [v.clone() for v in a.view]
    for v in a.view:
        v[:5].fill_(7.0)
    a.rebuild_view()
    torch.cuda.synchronize()
    for p in range(n_plans):
        assert torch.equal(a.view[p].view(torch.int16), keep[p].view(torch.int16))
    a.close()
    b.close()
    for pl in plans:
        pl.close()


def test_decode_workload_shape_and_capacity_errors(B):
    """Config 4's append shape: 8 kv heads x 64 sequences, one token per step, many plans."""
    w = W.WORKLOADS["decode-d96"]
    n_plans, n_seq, R = 8, w.batch * w.kv_heads, 16
    plans, lams = [], []
    for p in range(n_plans):
        seed, lam, _ = W.plan_constants(w, p)
        plans.append(B.Plan(w.d, w.g, seed, lam))
        lams.append(lam)
    cache = B.Cache(plans, n_seq, 32, R)
    steps = [[W.make_kv(w, p, n_vec=n_seq, device="cuda").view(n_seq, 1, w.d) * (1 + 0.01 * j) for p in range(n_plans)]
             for j in range(20)]
    steps = [[t.to(torch.float16).contiguous() for t in st] for st in steps]
    for st in steps:
        cache.append(st)
    torch.cuda.synchronize()
    assert cache.tokens == 20 and cache.quantized_tokens == 16
    p = 5
    xs = torch.stack([st[p][:, 0] for st in steps], dim=1).cpu().numpy()          # [n_seq, 20, d]
    model = CO.ResidualWindowCache(w.d, w.g, plans[p].signs, lams[p], n_seq, R)
    model.append(xs)
    view = _tokens(cache.view[p], 20).cpu().numpy()
    codes = _tokens(cache.codes[p], 16).cpu().numpy().reshape(-1, w.d // 2)
    scales = _tokens(cache.scales[p], 16).cpu().numpy().reshape(-1, w.d // w.g)
    assert P.check_quantize(xs[:, :16].reshape(-1, w.d), plans[p].signs, lams[p], w.g, codes,
                            scales)["ill_conditioned_groups"] == 0
    P.check_dequantize(codes, scales, plans[p].signs, lams[p], w.g, view[:, :16].reshape(-1, w.d))
    assert np.array_equal(view[:, 16:].view(np.uint16), model.view()[:, 16:].view(np.uint16))
    # capacity: 12 more tokens fit, 13 do not, and a refused append changes nothing
    L = B.lib()
    big = [torch.zeros(n_seq, 13, w.d, dtype=torch.float16, device="cuda") for _ in range(n_plans)]
    with pytest.raises(B.SrftError):
        cache.append(big)
    assert cache.tokens == 20
    cache.append([b[:, :12].contiguous() for b in big])
    assert cache.tokens == 32 and cache.quantized_tokens == 32
    assert L.srft_cache_append(cache.handle, None, 0, None) == 0
    assert L.srft_cache_append(cache.handle, None, -1, None) == -7
    torch.cuda.synchronize()
    cache.close()
    for pl in plans:
        pl.close()
