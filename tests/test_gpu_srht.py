"""GPU parity of the SRHT comparator (Walsh-Hadamard in place of the DFT) against the oracle."""
import ctypes as C

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


@pytest.mark.parametrize("d", [32, 64, 128, 256])
@pytest.mark.parametrize("bits", [4, 8])
def test_srht_matches_oracle(B, d, bits):
    n = 1500
    x = W.gaussian_with_outliers(n, d, seed=d + bits, outliers=2, gain=25.0)
    lam = W.lognormal_lambda(d, seed=d)
    plan = B.Plan(d, 32, 99 + d, lam, bits=bits, transform="hadamard")
    s = plan.signs
    xd = torch.from_numpy(x).cuda()
    # the transform alone: H (s * x) scaled by lambda
    w = plan.forward_f32(xd).cpu().numpy().astype(np.float64)
    ref = O.srft_forward(x, s, form="hadamard") * lam.astype(np.float64)
    assert (np.abs(w - ref) / np.abs(ref).max(axis=1, keepdims=True)).max() < 2e-6
    codes, scales = plan.quantize(xd)
    out = plan.dequantize(codes, scales)
    c, sc = codes.cpu().numpy(), scales.cpu().numpy()
    P.check_quantize(x, s, lam, 32, c, sc, bits=bits, form="hadamard")
    P.check_dequantize(c, sc, s, lam, 32, out.cpu().numpy(), bits=bits, form="hadamard")
    plan.close()


def test_srft_and_srht_reconstruct_alike_on_the_gpu(B):
    """The comparison the paper draws (Sec. 1, Sec. 3.1), on config 3's heavy-tailed channels: 4-bit round-trip
    errors of the two transforms agree within 10 %."""
    w = W.WORKLOADS["gemma3-1b-4k"]
    x = W.make_kv(w, 0, device="cuda")
    xf = x.double()
    err = {}
    for name in ("dft", "hadamard"):
        plan = B.Plan(w.d, w.g, 7, None, transform=name)
        out = plan.dequantize(*plan.quantize(x))
        err[name] = float(((out.double() - xf) ** 2).mean())
        plan.close()
    assert abs(err["dft"] - err["hadamard"]) / err["dft"] < 0.1, err


def test_srht_argument_errors(B):
    L = B.lib()
    h = C.c_void_p()
    assert L.srft_plan_create_ex(C.byref(h), 96, 32, 4, 1, 0, None) == -2          # not a power of two
    assert L.srft_plan_create_ex(C.byref(h), 128, 32, 4, 2, 0, None) == -10
    assert L.srft_plan_create_ex(C.byref(h), 128, 32, 4, -1, 0, None) == -10
    a, b = B.Plan(128, 32, 1), B.Plan(128, 32, 1, transform="hadamard")
    x = torch.zeros(32, 128, dtype=torch.float16, device="cuda")
    c = torch.zeros(32, 64, dtype=torch.uint8, device="cuda")
    s = torch.zeros(32, 4, dtype=torch.float32, device="cuda")
    with pytest.raises(B.SrftError):
        B.srft_kv_quantize_batched(B.BatchTable([a.handle, b.handle], [x, x], [c, c], [s, s]))
    a.close()
    b.close()
