"""CPU model of the int4 KV cache with an fp16 residual window.  TEST INFRASTRUCTURE ONLY.

Follows the paper's description of its cache class (Sec. 7.2, items (i)-(iv), and the "Residual window"
paragraph of the design-choices section): keys/values are stored as int4 codes plus fp32 group scales; the most
recent tokens are kept in fp16 in a residual window and are quantized ("re-quantized when full") once the window
holds R tokens (R = 16 in the paper); what attention reads is the dequantized prefix followed by the window.
The dequantized prefix is a cache of the int4 store: it changes only when the window is flushed.

Plain Python/numpy, one token at a time, no blocking: only tests, the smoke check and the benchmark's CPU leg
may import it; it shares nothing with the HIP library except the seeded input generators' outputs.

Parity status: pinned in tests/test_oracle_cache.py by the definition written out independently (whole-tensor
quantize/dequantize of the flushed part, exact copy of the rest), by the stored-byte counts behind the paper's
3.2x figure and its statement about a 32-token window, and by chunking invariance.
"""
from __future__ import annotations

import numpy as np

from oracle import srft_oracle as O


class ResidualWindowCache:
    """One (layer, K|V) cache for n_seq independent sequences (batch x kv_heads) that grow in lock-step."""

    def __init__(self, d: int, g: int, s, lam, n_seq: int, residual_tokens: int = 16):
        if residual_tokens < 1:
            raise ValueError("the residual window holds at least one token")
        self.d, self.g, self.s, self.lam = d, g, np.asarray(s), np.asarray(lam, dtype=np.float32)
        self.n_seq, self.R = n_seq, residual_tokens
        self.codes = np.zeros((n_seq, 0, d // 2), dtype=np.uint8)       # the int4 store
        self.scales = np.zeros((n_seq, 0, d // g), dtype=np.float32)
        self.prefix = np.zeros((n_seq, 0, d), dtype=np.float16)         # dequantized store, refreshed on flush
        self.window = np.zeros((n_seq, 0, d), dtype=np.float16)         # recent tokens, exact
        self.flushes = 0

    @property
    def tokens(self) -> int:
        return self.codes.shape[1] + self.window.shape[1]

    @property
    def quantized_tokens(self) -> int:
        return self.codes.shape[1]

    def append(self, x_f16) -> None:
        """x_f16: [n_seq, t, d] fp16, t new tokens per sequence."""
        x = np.asarray(x_f16, dtype=np.float16)
        assert x.shape[0] == self.n_seq and x.shape[2] == self.d
        for tok in range(x.shape[1]):
            self.window = np.concatenate([self.window, x[:, tok:tok + 1]], axis=1)
            if self.window.shape[1] == self.R:                          # full: quantize the window, empty it
                flat = self.window.reshape(-1, self.d)
                q = O.quantize(flat, self.s, self.lam, self.g)
                back = O.dequantize(q["codes"], q["scales"], self.s, self.lam, self.g)
                self.codes = np.concatenate([self.codes, q["codes"].reshape(self.n_seq, self.R, -1)], axis=1)
                self.scales = np.concatenate([self.scales, q["scales"].reshape(self.n_seq, self.R, -1)], axis=1)
                self.prefix = np.concatenate([self.prefix, back.reshape(self.n_seq, self.R, self.d)], axis=1)
                self.window = self.window[:, :0]
                self.flushes += 1

    def view(self) -> np.ndarray:
        """What attention reads: [n_seq, tokens, d] fp16 = dequantized prefix, then the window."""
        return np.concatenate([self.prefix, self.window], axis=1)

    def stored_bytes_per_sequence(self) -> int:
        """int4 record bytes of the quantized tokens plus fp16 bytes of the window (the dequantized prefix is a
        cache of the store, not storage)."""
        return self.quantized_tokens * O.record_bytes(self.d, self.g) + self.window.shape[1] * 2 * self.d
