"""CPU oracle for the SRFT int4 KV-cache quantizer.  TEST INFRASTRUCTURE ONLY.

A plain, slow, double-precision statement of what the write path and the read
path compute, written from the paper's definitions.  Nothing in the product
(the HIP library and its Python binding) imports, calls or links this module;
only the tests, the smoke check and the benchmark's CPU-baseline leg do.  It
shares no code, table or constant generator with the HIP path.

What each function follows:

* ``signs_from_seed``      -- Sec. 3.1: "s is a fixed random sign vector drawn
                              at initialization".  The paper does not name a
                              generator; ours is the published splitmix64
                              stream (Steele, Lea, Flood 2014), top bit of the
                              n-th output = 1 means s_n = -1.
* ``srft_matrix``          -- Eq. 1 and Eq. 2 written out as one real d x d
                              matrix Q (unitary DFT, rfft sign convention,
                              sqrt(2) on the middle bins).
* ``srft_forward`` /
  ``srft_inverse``         -- Eq. 1, Eq. 2 and the sentence after them
                              ("unpack, irfft, apply s"): z = Q (s * x) and
                              x = s * (Q^T z), as a dense product (``dense``)
                              or through a recursive mixed-radix FFT followed
                              by the Eq. 2 packing (``fft``).
* ``quantize``             -- Sec. 3.2 steps 1-4 with b = 4, the lambda
                              rescale of Sec. 5.1 item 1 and the per-group
                              abs-max of Sec. 5.6 / Sec. 7.1 (g values per
                              group, groups are runs of the packed index).
* ``dequantize``           -- the matching inverse named in Sec. 7.1: unpack,
                              times scale, divide by lambda clamped at 1e-6
                              (Sec. 5.1 item 1), inverse SRFT, unsign.
* ``pack_nibbles`` /
  ``unpack_nibbles``       -- Sec. 3.2 detail (ii):
                              byte = (q[2i+1] << 4) | (q[2i] & 0xF).
* ``hadamard_matrix``      -- the SRHT the paper compares against (Sec. 1,
                              Sec. 3.1): ``form="hadamard"`` swaps it in for Q
                              everywhere.
* ``attention_scores``     -- the consumer of the stored keys (Sec. 1, "each decode
                              step streams the stored prefix ... before attention
                              can read it"): inner products of queries with the
                              reconstructed keys, written as exactly that.
* ``attention_output`` /
  ``softmax_rows`` /
  ``decode_attention``     -- the rest of that consumer (Sec. 1; Sec. 7.2, where
                              attention reads the dequantized prefix): weights times
                              the reconstructed values, the row softmax between the
                              two, and their composition, each as its plain definition.
* ``channel_absmax`` /
  ``lambda_from_absmax``   -- Sec. 7.1: lambda_d = 1 / per_channel_max(SRFT
                              output)_d, the maximum taken over a calibration
                              batch (Sec. 7.2: over whole windows).
* ``record_bytes``         -- Sec. 3.2 step 4, Sec. 4.5 and Sec. 7.2 item (i):
                              d/2 code bytes plus one fp32 scale per group.

Parity status: every function above is pinned by tests that do not go through
this module's own formulas (brute-force DFT sums, numpy's rfft, closed forms,
orthogonality, exhaustive pack/unpack, the paper's printed compression ratios
and memory table, error bounds).  The paper prints no worked numeric example of
codes or scales, so there is no stored code/scale fixture from the paper.
"""
from __future__ import annotations

import numpy as np

QMAX = 7            # 2^(b-1) - 1 for b = 4  (Sec. 3.2 step 3)
LAMBDA_FLOOR = 1e-6  # read-path clamp on lambda (Sec. 5.1 item 1)
_MASK64 = (1 << 64) - 1


# --------------------------------------------------------------------------
# sign diagonal
# --------------------------------------------------------------------------
def splitmix64_stream(seed: int, n: int) -> list[int]:
    """First n outputs of splitmix64 started at ``seed`` (published algorithm)."""
    state = seed & _MASK64
    out = []
    for _ in range(n):
        state = (state + 0x9E3779B97F4A7C15) & _MASK64
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
        z = z ^ (z >> 31)
        out.append(z)
    return out


def signs_from_seed(seed: int, d: int) -> np.ndarray:
    """s in {-1,+1}^d (int8): s_n = -1 iff the top bit of the n-th output is set."""
    return np.array([-1 if (v >> 63) else 1 for v in splitmix64_stream(seed, d)],
                    dtype=np.int8)


# --------------------------------------------------------------------------
# the transform
# --------------------------------------------------------------------------
def srft_matrix(d: int) -> np.ndarray:
    """Q in R^{d x d} with z = Q u equal to pack(F u) of Eq. 1-2.

    F is the unitary DFT, Y_k = d^{-1/2} sum_n u_n exp(-2 pi i k n / d), so
    Re Y_k = d^{-1/2} sum u_n cos(2 pi k n/d), Im Y_k = -d^{-1/2} sum u_n sin(.).
    Rows: k = 0 -> Re Y_0; k = d/2 -> Re Y_{d/2}; 1 <= k < d/2 -> sqrt2 Re Y_k;
    d/2 < k < d -> sqrt2 Im Y_{k - d/2}.
    """
    if d < 2 or d % 2:
        raise ValueError("d must be even and >= 2")
    h = d // 2
    n = np.arange(d, dtype=np.float64)
    Q = np.empty((d, d), dtype=np.float64)
    for k in range(d):
        if k == 0:
            Q[k] = 1.0 / np.sqrt(d)
        elif k == h:
            Q[k] = np.cos(np.pi * n) / np.sqrt(d)          # (-1)^n
        elif k < h:
            Q[k] = np.sqrt(2.0 / d) * np.cos(2.0 * np.pi * k * n / d)
        else:
            Q[k] = -np.sqrt(2.0 / d) * np.sin(2.0 * np.pi * (k - h) * n / d)
    return Q


def hadamard_matrix(d: int) -> np.ndarray:
    """The orthonormal Walsh-Hadamard matrix in natural (Sylvester) order, H_{2m} = [[H_m, H_m], [H_m, -H_m]] / sqrt 2.

    With it in place of Q the pipeline is the SRHT the paper compares the SRFT against (Sec. 1 contribution list,
    Sec. 3.1): same sign diagonal, same quantizer, another orthogonal mixing matrix.  d must be a power of two.
    """
    if d < 1 or d & (d - 1):
        raise ValueError("the Hadamard comparator needs a power-of-two d")
    H = np.ones((1, 1), dtype=np.float64)
    while H.shape[0] < d:
        H = np.block([[H, H], [H, -H]])
    return H / np.sqrt(d)


def _smallest_factor(n: int) -> int:
    p = 2
    while p * p <= n:
        if n % p == 0:
            return p
        p += 1
    return n


def fft_mixed_radix(a: np.ndarray) -> np.ndarray:
    """Unnormalised forward DFT along the last axis, any length.

    Decimation in time on the smallest prime factor p of n: the p interleaved
    subsequences a[r::p] are transformed recursively (length m = n/p) and
    recombined as X[k + m q] = sum_r W_n^{r (k + m q)} A_r[k]; a prime length is
    the direct sum.  W_n = exp(-2 pi i / n).
    """
    a = np.asarray(a, dtype=np.complex128)
    n = a.shape[-1]
    if n == 1:
        return a.copy()
    p = _smallest_factor(n)
    if p == n:  # prime length: direct O(n^2) sum
        k = np.arange(n)
        W = np.exp(-2j * np.pi * np.outer(k, k) / n)
        return a @ W.T
    m = n // p
    subs = [fft_mixed_radix(a[..., r::p]) for r in range(p)]
    out = np.empty_like(a)
    k = np.arange(m)
    for q in range(p):
        acc = np.zeros(a.shape[:-1] + (m,), dtype=np.complex128)
        for r in range(p):
            acc = acc + np.exp(-2j * np.pi * r * (k + m * q) / n) * subs[r]
        out[..., m * q:m * (q + 1)] = acc
    return out


def pack_spectrum(Y: np.ndarray, d: int) -> np.ndarray:
    """Eq. 2: half spectrum Y_0..Y_{d/2} (complex) -> z in R^d."""
    h = d // 2
    z = np.empty(Y.shape[:-1] + (d,), dtype=np.float64)
    z[..., 0] = Y[..., 0].real
    z[..., h] = Y[..., h].real
    z[..., 1:h] = np.sqrt(2.0) * Y[..., 1:h].real
    z[..., h + 1:] = np.sqrt(2.0) * Y[..., 1:h].imag
    return z


def unpack_spectrum(z: np.ndarray) -> np.ndarray:
    """Inverse of Eq. 2: z in R^d -> the full length-d conjugate-symmetric spectrum."""
    d = z.shape[-1]
    h = d // 2
    Y = np.zeros(z.shape[:-1] + (d,), dtype=np.complex128)
    Y[..., 0] = z[..., 0]
    Y[..., h] = z[..., h]
    mid = (z[..., 1:h] + 1j * z[..., h + 1:]) / np.sqrt(2.0)
    Y[..., 1:h] = mid
    Y[..., h + 1:] = np.conj(mid[..., ::-1])   # Y_{d-k} = conj(Y_k)
    return Y


def srft_forward(x, s, form: str = "dense", dtype=np.float64) -> np.ndarray:
    """z = pack(F diag(s) x) for x of shape [..., d]  (Eq. 1-2)."""
    x = np.asarray(x)
    d = x.shape[-1]
    u = x.astype(dtype) * np.asarray(s).astype(dtype)
    if form == "dense":
        return u @ srft_matrix(d).astype(dtype).T
    if form == "fft":
        Y = fft_mixed_radix(u.astype(np.float64)) / np.sqrt(d)
        return pack_spectrum(Y[..., :d // 2 + 1], d)
    if form == "hadamard":                       # the SRHT comparator: H in place of Q
        return u @ hadamard_matrix(d).astype(dtype).T
    raise ValueError(form)


def srft_inverse(z, s, form: str = "dense", dtype=np.float64) -> np.ndarray:
    """x = s * (Q^T z): unpack, unitary inverse DFT, apply s (sentence after Eq. 2)."""
    z = np.asarray(z)
    d = z.shape[-1]
    if form == "dense":
        u = z.astype(dtype) @ srft_matrix(d).astype(dtype)
    elif form == "fft":
        Y = unpack_spectrum(z.astype(np.float64))
        # inverse unitary DFT through the forward routine: ifft(Y) = conj(fft(conj Y)) / d
        u = np.conj(fft_mixed_radix(np.conj(Y))).real / np.sqrt(d)
    elif form == "hadamard":
        u = z.astype(dtype) @ hadamard_matrix(d).astype(dtype)
    else:
        raise ValueError(form)
    return u * np.asarray(s).astype(u.dtype)


# --------------------------------------------------------------------------
# int4 codes
# --------------------------------------------------------------------------
def pack_nibbles(q: np.ndarray) -> np.ndarray:
    """[..., d] integers in [-8, 7] -> [..., d/2] uint8, byte_i = (q[2i+1] << 4) | (q[2i] & 0xF)."""
    q = np.asarray(q).astype(np.int64)
    lo = q[..., 0::2] & 0xF
    hi = q[..., 1::2] & 0xF
    return ((hi << 4) | lo).astype(np.uint8)


def unpack_nibbles(b: np.ndarray) -> np.ndarray:
    """[..., d/2] uint8 -> [..., d] int8, each nibble read as 4-bit two's complement."""
    b = np.asarray(b, dtype=np.uint8).astype(np.int64)
    lo = b & 0xF
    hi = (b >> 4) & 0xF
    lo = np.where(lo >= 8, lo - 16, lo)
    hi = np.where(hi >= 8, hi - 16, hi)
    q = np.empty(b.shape[:-1] + (2 * b.shape[-1],), dtype=np.int8)
    q[..., 0::2] = lo
    q[..., 1::2] = hi
    return q


def record_bytes(d: int, g: int, bits: int = 4) -> int:
    """Stored bytes per vector: d/2 code bytes (d at 8 bits) + one fp32 scale per group of g."""
    if d % 2 or d % g:
        raise ValueError("d must be even and divisible by g")
    return d * bits // 8 + 4 * (d // g)


# --------------------------------------------------------------------------
# write path / read path
# --------------------------------------------------------------------------
def quantize(x_f16, s, lam, g: int, form: str = "dense", bits: int = 4) -> dict:
    """Write path for x_f16 of shape [n, d] (fp16 values).

    1. u = s * x                      (Sec. 3.2 step 1)
    2. z = pack(F u)                  (Eq. 1-2; Sec. 3.2 step 2)
    3. w = lambda * z                 (Sec. 5.1 item 1, Sec. 7.1)
    4. per group j of g packed indices: a_j = max |w_k|,
       scale_j = fp32(a_j / 7)        (Sec. 3.2 step 3 with b = 4; Sec. 7.1)
    5. q_k = clip(rint(w_k / scale_j), -7, 7), rint = round half to even
       (Sec. 7.1 names rint); an all-zero group gives scale 0 and codes 0
    6. nibble pack                    (Sec. 3.2 detail (ii))

    Returns codes [n, d/2] uint8, scales [n, d/g] float32, and for the parity
    tests q [n, d] int8, the pre-rounding ratios r [n, d] and w [n, d].

    bits = 8 is the paper's other output width (Sec. 3.2 steps 3-4 with b = 8): scale = a / 127, codes in
    [-127, 127], "one byte per value" (two's complement), codes [n, d] uint8.
    """
    if bits not in (4, 8):
        raise ValueError("bits must be 4 or 8")
    qmax = 2 ** (bits - 1) - 1
    x = np.asarray(x_f16).astype(np.float64)
    n, d = x.shape
    if d % g:
        raise ValueError("g must divide d")
    lam = np.asarray(lam, dtype=np.float64)
    z = srft_forward(x, s, form=form)
    w = z * lam
    wg = w.reshape(n, d // g, g)
    a = np.abs(wg).max(axis=-1)
    scales = (a / qmax).astype(np.float32)
    sc = scales.astype(np.float64)[..., None]
    safe = np.where(sc > 0, sc, 1.0)
    r = np.where(sc > 0, wg / safe, 0.0)
    q = np.clip(np.rint(r), -qmax, qmax).astype(np.int8)
    q = q.reshape(n, d)
    return {
        "codes": pack_nibbles(q) if bits == 4 else q.view(np.uint8).copy(),
        "scales": scales,
        "q": q,
        "r": r.reshape(n, d),
        "w": w,
    }


def dequantize_f64(codes, scales, s, lam, g: int, form: str = "dense", bits: int = 4) -> np.ndarray:
    """Read path up to, not including, the final fp16 rounding.  Returns [n, d] float64."""
    if bits == 4:
        q = unpack_nibbles(codes).astype(np.float64)
    else:                                        # one byte per value, two's complement
        q = np.asarray(codes, dtype=np.uint8).view(np.int8).astype(np.float64)
    n, d = q.shape
    sc = np.asarray(scales, dtype=np.float32).astype(np.float64)
    w = (q.reshape(n, d // g, g) * sc[..., None]).reshape(n, d)
    lam = np.maximum(np.asarray(lam, dtype=np.float64), LAMBDA_FLOOR)
    z = w / lam
    return srft_inverse(z, s, form=form)


def dequantize(codes, scales, s, lam, g: int, form: str = "dense", bits: int = 4) -> np.ndarray:
    """Read path: unpack, times scale, / max(lambda, 1e-6), inverse SRFT, unsign, fp16 (RNE)."""
    return dequantize_f64(codes, scales, s, lam, g, form=form, bits=bits).astype(np.float16)


def channel_absmax(x_f16, s, lam=None, running=None) -> np.ndarray:
    """Per-channel abs-max of w = lambda * pack(F (s * x)) over the rows of x_f16 ([n, d]); float64 [d].

    Sec. 7.1 names this statistic ("per_channel_max(SRFT-output)"); Sec. 7.2 takes it over whole calibration
    windows, batch after batch, hence ``running``: the maxima so far (element-wise maximum with them).
    """
    x = np.asarray(x_f16, dtype=np.float64)
    d = x.shape[-1]
    w = srft_forward(x, s)
    if lam is not None:
        w = w * np.asarray(lam, dtype=np.float64)
    amax = np.abs(w).max(axis=0) if x.shape[0] else np.zeros(d)
    if running is not None:
        amax = np.maximum(amax, np.asarray(running, dtype=np.float64))
    return amax


def lambda_from_absmax(amax) -> np.ndarray:
    """lambda_k = 1 / amax_k (Sec. 7.1), float64.

    The paper does not say what a channel that never moved gets; reading taken here: channels below 2^-16 of
    the largest abs-max are treated as if they were at that floor, and an all-zero statistic gives lambda = 1.
    """
    a = np.asarray(amax, dtype=np.float64)
    top = a.max(initial=0.0)
    if top <= 0.0:
        return np.ones_like(a)
    return 1.0 / np.maximum(a, top * 2.0 ** -16)


def attention_scores(q_f16, codes, scales, s, lam, g: int, form: str = "dense", bits: int = 4) -> np.ndarray:
    """scores[i, t] = <q_i, k_t>, k_t the read path's reconstruction of key t before its fp16 rounding; float64
    [n_q, n_keys].  The plain definition: reconstruct every key, take the inner products.  (A kernel may use the
    orthogonality of the transform and contract in the rotated domain instead; the result is the same number.)
    """
    q = np.asarray(q_f16).astype(np.float64)
    keys = dequantize_f64(codes, scales, s, lam, g, form=form, bits=bits)
    return q @ keys.T



def attention_output(weights, codes, scales, s, lam, g: int, form: str = "dense", bits: int = 4) -> np.ndarray:
    """out[i] = sum_t weights[i, t] * v_t, v_t the read path's reconstruction of value t before its fp16 rounding;
    float64 [n_q, d].  The plain definition: reconstruct every value, take the weighted sums.  (A kernel may sum in
    the rotated domain and apply one inverse transform per query instead: the transform is linear.)
    """
    w = np.asarray(weights, dtype=np.float64)
    values = dequantize_f64(codes, scales, s, lam, g, form=form, bits=bits)
    return w @ values


def softmax_rows(scores, scale: float = 1.0) -> np.ndarray:
    """Row-wise softmax of scale * scores in float64: exp(x - max x) / sum exp(x - max x)."""
    x = np.asarray(scores, dtype=np.float64) * float(scale)
    e = np.exp(x - x.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def decode_attention(q_f16, k_codes, k_scales, s_k, lam_k, v_codes, v_scales, s_v, lam_v, g: int, scale: float,
                     form: str = "dense", bits: int = 4) -> np.ndarray:
    """One decode step of attention over a stored cache: softmax(scale * q K^T) V with K and V the reconstructions
    of the two records (each with its own signs and lambda); float64 [n_q, d]."""
    scores = attention_scores(q_f16, k_codes, k_scales, s_k, lam_k, g, form=form, bits=bits)
    return attention_output(softmax_rows(scores, scale), v_codes, v_scales, s_v, lam_v, g, form=form, bits=bits)
