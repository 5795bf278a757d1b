"""Shared checks of the HIP path against the CPU oracle (used by the GPU tests and the smoke check).

Acceptance (per vector, element by element):
  (a) bytes: where the GPU's integer codes equal the oracle's, the packed bytes are identical -- checked by
      unpacking the GPU bytes with the oracle's unpacker and by comparing whole rows byte for byte;
  (b) codes: identical to the oracle's except where the oracle's pre-rounding ratio r = w / scale lies within
      BOUNDARY_WINDOW of a half-integer; every mismatch must be off by exactly one and inside the window;
  (c) scales within SCALE_RTOL relative, dequantized fp16 within OUT_RTOL relative plus a small floor
      tied to the vector's largest magnitude (fp32 accumulation error does not shrink with the element).
"""
from __future__ import annotations

import numpy as np

from oracle import srft_oracle as O

BOUNDARY_WINDOW = 1e-4     # in units of the group's scale, at 4 bits
# At 8 bits one code step is 7/127 of the 4-bit step for the same accuracy of w, so the same relative error of w
# moves r = w / scale by 127/7 as much: the window is the 4-bit one scaled by that ratio (1.8e-3).
BOUNDARY_WINDOW_8 = BOUNDARY_WINDOW * 127.0 / 7.0
SCALE_RTOL = 2e-3          # stated bar; the measured error is reported alongside
SCALE_RTOL_TIGHT = 2e-6    # what fp32 arithmetic on the abs-max actually delivers
W_ABS_ERR = 1e-6           # bound on |w_gpu - w| in units of lambda_k * ||x||_2 (fp32 accumulation of d terms)
COND_MIN = 1e-3            # a group below this fraction of its typical magnitude is cancellation-dominated
OUT_RTOL = 2e-3            # relative, per element (one fp16 ulp is at most 9.8e-4 relative)
OUT_FLOOR = 8e-6           # times max |ref| of the vector: fp32 accumulation over d <= 256 terms
FP16_TINY = 1.2e-7         # two fp16 subnormal quanta


def check_quantize(x_f16: np.ndarray, s, lam, g, codes_gpu: np.ndarray, scales_gpu: np.ndarray, bits: int = 4,
                   form: str = "dense") -> dict:
    """x_f16 [n, d] float16; GPU outputs as numpy.  Raises AssertionError on any violation.

    A group is "cancellation-dominated" when its abs-max is below COND_MIN of what its lambdas and the
    vector's norm make typical (lambda ||x|| / sqrt(d) is the typical coefficient): there the
    coefficients are rounding noise of the fp32 transform, relative agreement is not defined, and the
    group is held to the absolute checks only.  Random data has no such groups; the count is reported.
    """
    ref = O.quantize(x_f16, s, lam, g, bits=bits, form=form)
    n, d = x_f16.shape
    G = d // g
    qmax = 2 ** (bits - 1) - 1
    window = BOUNDARY_WINDOW if bits == 4 else BOUNDARY_WINDOW_8
    assert codes_gpu.shape == (n, d * bits // 8) and codes_gpu.dtype == np.uint8
    assert scales_gpu.shape == (n, G) and scales_gpu.dtype == np.float32
    lam64 = np.asarray(lam, dtype=np.float64)
    xn = np.linalg.norm(x_f16.astype(np.float64), axis=1)                       # [n]
    typical = lam64.reshape(G, g).max(axis=1)[None, :] * xn[:, None]             # [n, G]
    sr = ref["scales"].astype(np.float64)
    sg = scales_gpu.astype(np.float64)
    well = sr > COND_MIN * typical / np.sqrt(d)
    q_gpu = O.unpack_nibbles(codes_gpu) if bits == 4 else codes_gpu.view(np.int8)
    q_ref = ref["q"]
    assert q_gpu.min(initial=0) >= -qmax and q_gpu.max(initial=0) <= qmax, "code outside the symmetric range"
    # every group, absolute: scale within the fp32 error of the transform; codes are a nearest rounding of w
    assert np.all(np.abs(sg - sr) <= SCALE_RTOL_TIGHT * sr + W_ABS_ERR * typical / qmax), "scale abs err"
    sg_k = np.repeat(sg, g, axis=1)
    e_k = W_ABS_ERR * lam64[None, :] * xn[:, None]
    assert np.all(np.abs(q_gpu * sg_k - ref["w"]) <= 0.5 * sg_k * (1 + 1e-5) + e_k), "codes are not a nearest rounding"
    assert not q_gpu[np.repeat(sg == 0, g, axis=1)].any(), "non-zero code under a zero scale"
    # (c) scales of well-conditioned groups, relative
    rel = np.where(well, np.abs(sg - sr) / np.where(sr > 0, sr, 1.0), 0.0)
    assert rel.max(initial=0.0) <= SCALE_RTOL_TIGHT, f"scale rel err {rel.max():.3e}"
    # (b) codes of well-conditioned groups
    well_k = np.repeat(well, g, axis=1)
    mism = (q_gpu != q_ref) & well_k
    n_mism = int(mism.sum())
    if n_mism:
        r = ref["r"][mism]
        dist = np.abs(np.abs(r - np.floor(r)) - 0.5)        # distance to the nearest half-integer
        step = np.abs(q_gpu[mism].astype(np.int32) - q_ref[mism].astype(np.int32))
        assert np.all(step == 1), "code mismatch larger than one step"
        assert np.all(dist < window), f"code mismatch {dist.max():.3e} away from a rounding boundary"
    # (a) bytes: rows whose codes all agree must agree byte for byte; and re-packing the GPU codes is the identity
    rows_equal = ~(q_gpu != q_ref).any(axis=1)
    assert np.array_equal(codes_gpu[rows_equal], ref["codes"][rows_equal])
    if bits == 4:
        assert np.array_equal(O.pack_nibbles(q_gpu), codes_gpu)
    return {
        "n": n, "mismatches": n_mism, "mismatch_rate": n_mism / max(1, n * d),
        "scale_max_rel": float(rel.max(initial=0.0)), "ill_conditioned_groups": int((~well & (sr > 0)).sum()),
        "ref": ref,
    }


def out_tolerance(ref64: np.ndarray) -> np.ndarray:
    vmax = np.abs(ref64).max(axis=1, keepdims=True)
    return OUT_RTOL * np.abs(ref64) + OUT_FLOOR * vmax + FP16_TINY


def check_dequantize(codes: np.ndarray, scales: np.ndarray, s, lam, g, out_gpu: np.ndarray, bits: int = 4,
                     form: str = "dense") -> dict:
    """GPU read path on (codes, scales) against the oracle's read path on the same bytes."""
    ref64 = O.dequantize_f64(codes, scales, s, lam, g, bits=bits, form=form)
    ref16 = ref64.astype(np.float16)
    assert out_gpu.dtype == np.float16 and out_gpu.shape == ref16.shape
    assert np.isfinite(out_gpu.astype(np.float32)).all()
    err = np.abs(out_gpu.astype(np.float64) - ref16.astype(np.float64))
    tol = out_tolerance(ref64)
    worst = float((err / tol).max(initial=0.0))
    assert worst <= 1.0, f"dequantized output off by {worst:.2f}x the tolerance"
    exact = float((out_gpu == ref16).mean()) if out_gpu.size else 1.0
    vmax = np.abs(ref64).max(axis=1, keepdims=True)
    # error before the fp16 rounding cannot be seen; report the fp16-level figures
    return {"bit_identical_fraction": exact, "worst_over_tol": worst,
            "max_err_over_vmax": float((err / np.where(vmax > 0, vmax, 1.0)).max(initial=0.0))}
