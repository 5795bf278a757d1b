"""Pins of the cache model (oracle/cache_oracle.py); no GPU."""
import numpy as np
import pytest

from oracle import cache_oracle as CO
from oracle import srft_oracle as O


def _inputs(n_seq, T, d, seed):
    rng = np.random.RandomState(seed)
    x = rng.standard_normal((n_seq, T, d)).astype(np.float16)
    x[:, :, 3] *= np.float16(12.0)                       # one loud channel
    lam = np.exp(0.4 * rng.standard_normal(d)).astype(np.float32)
    return x, O.signs_from_seed(seed, d), lam


@pytest.mark.parametrize("T", [0, 1, 15, 16, 17, 31, 32, 33, 100])
def test_view_is_quantized_prefix_then_exact_window(T):
    d, g, n_seq, R = 32, 32, 3, 16
    x, s, lam = _inputs(n_seq, T, d, seed=T + 1)
    c = CO.ResidualWindowCache(d, g, s, lam, n_seq, R)
    c.append(x)
    n_q = (T // R) * R                                   # "re-quantized when full": every complete window is flushed
    assert c.tokens == T and c.quantized_tokens == n_q and c.flushes == T // R
    v = c.view()
    assert v.shape == (n_seq, T, d) and v.dtype == np.float16
    # the definition written out on the whole tensor, independent of the model's token loop
    q = O.quantize(x[:, :n_q].reshape(-1, d), s, lam, g)
    want = O.dequantize(q["codes"], q["scales"], s, lam, g).reshape(n_seq, n_q, d)
    assert np.array_equal(v[:, :n_q].view(np.uint16), want.view(np.uint16))
    assert np.array_equal(c.codes.reshape(-1, d // 2), q["codes"])
    assert np.array_equal(v[:, n_q:].view(np.uint16), x[:, n_q:].view(np.uint16))     # the window is exact
    if n_q:
        assert not np.array_equal(v[:, :n_q], x[:, :n_q])                             # the prefix is not


def test_result_does_not_depend_on_how_appends_are_chunked():
    d, g, n_seq, R, T = 32, 16, 2, 8, 45
    x, s, lam = _inputs(n_seq, T, d, seed=9)
    a = CO.ResidualWindowCache(d, g, s, lam, n_seq, R)
    a.append(x)
    b = CO.ResidualWindowCache(d, g, s, lam, n_seq, R)
    pos = 0
    for t in (1, 1, 1, 5, 8, 0, 13, 16):
        b.append(x[:, pos:pos + t])
        pos += t
    assert pos == T
    assert np.array_equal(a.view().view(np.uint16), b.view().view(np.uint16))
    assert np.array_equal(a.codes, b.codes) and np.array_equal(a.scales, b.scales)
    # the dequantized prefix never changes afterwards (it can be cached between steps); window tokens stay exact
    # until the append that fills the window, which replaces them by their reconstruction
    before = b.view().copy()
    n_q = b.quantized_tokens                                             # 40, with 5 tokens in the window
    b.append(np.zeros((n_seq, 2, d), dtype=np.float16))                  # 7 of 8: no flush
    assert np.array_equal(b.view()[:, :T].view(np.uint16), before.view(np.uint16))
    b.append(np.zeros((n_seq, 1, d), dtype=np.float16))                  # full: flushed
    assert b.quantized_tokens == n_q + R
    assert np.array_equal(b.view()[:, :n_q].view(np.uint16), before[:, :n_q].view(np.uint16))
    assert not np.array_equal(b.view()[:, n_q:T], before[:, n_q:T])


def test_stored_bytes_behind_the_papers_compression_figures():
    """d = 128, g = 32: 80 bytes per quantized token against 256 in fp16 (3.2x); with a 16-token window a
    cache of about a thousand tokens stays above 3x, with a 32-token window it can drop below 3x
    (cache section item (i) and the residual-window paragraph)."""
    d, g = 128, 32
    s, lam = O.signs_from_seed(1, d), np.ones(d, dtype=np.float32)

    def ratio(T, R):
        c = CO.ResidualWindowCache(d, g, s, lam, 1, R)
        c.codes = np.zeros((1, (T // R) * R, d // 2), dtype=np.uint8)        # bookkeeping only: no arithmetic needed
        c.window = np.zeros((1, T % R, d), dtype=np.float16)
        assert c.tokens == T
        return T * 2 * d / c.stored_bytes_per_sequence()

    assert ratio(16 * 4096, 16) == pytest.approx(3.2)
    assert all(ratio(T, 16) >= 3.0 for T in range(512, 1100))
    assert min(ratio(T, 32) for T in range(512, 1024)) < 3.0
    assert ratio(1024 + 15, 16) == pytest.approx(265984 / 85760)
