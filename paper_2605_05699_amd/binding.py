"""ctypes binding over libsrft_kv.so: argument marshalling only.

Functions carry the names of the C entry points declared in ``include/srft_kv.h``
and take torch tensors (device memory) where the C side takes device pointers.
Every step of the method runs inside the library's HIP kernels; there is no
fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SRFT_KV_LIB") or os.path.join(_PKG, "libsrft_kv.so")
_lib = None

EXPORTS = [
    "srft_plan_create", "srft_plan_destroy", "srft_kv_quantize", "srft_kv_dequantize",
    "srft_kv_forward_f32", "srft_plan_d", "srft_plan_group_size", "srft_plan_groups",
    "srft_plan_code_bytes", "srft_plan_get_signs", "srft_plan_set_max_workgroups",
    "srft_status_string", "srft_last_hip_error",
    "srft_kv_quantize_batched", "srft_kv_dequantize_batched",
    "srft_kv_channel_absmax", "srft_lambda_from_absmax",
    "srft_cache_create", "srft_cache_destroy", "srft_cache_append", "srft_cache_rebuild_view",
    "srft_cache_tokens", "srft_cache_quantized_tokens",
    "srft_plan_create_bits", "srft_plan_bits", "srft_plan_form", "srft_plan_create_ex",
    "srft_scores_workspace_bytes", "srft_kv_scores", "srft_kv_scores_static", "srft_kv_quantize_butterfly",
    "srft_attend_workspace_bytes", "srft_kv_attend", "srft_decode_attention_workspace_bytes", "srft_kv_decode_attention",
]


class SrftError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().srft_status_string(status).decode()
        if status == -6:
            msg += f" [hipError {lib().srft_last_hip_error()}]"
        super().__init__(f"{where}: {msg} (status {status})")


def lib() -> C.CDLL:
    """Load the library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2605_05699_amd.build` "
            "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i64, u64, ci = C.c_void_p, C.c_int64, C.c_uint64, C.c_int
    L.srft_plan_create.argtypes = [C.POINTER(vp), ci, ci, u64, vp]
    L.srft_plan_create_bits.argtypes = [C.POINTER(vp), ci, ci, ci, u64, vp]
    L.srft_plan_create_ex.argtypes = [C.POINTER(vp), ci, ci, ci, ci, u64, vp]
    L.srft_plan_bits.argtypes = [vp]
    L.srft_plan_form.argtypes = [vp, ci]
    L.srft_plan_destroy.argtypes = [vp]
    L.srft_kv_quantize.argtypes = [vp, vp, i64, vp, vp, vp]
    L.srft_kv_dequantize.argtypes = [vp, vp, vp, i64, vp, vp]
    L.srft_kv_quantize_butterfly.argtypes = [vp, vp, i64, vp, vp, vp]
    L.srft_kv_forward_f32.argtypes = [vp, vp, i64, vp, vp]
    L.srft_cache_create.argtypes = [C.POINTER(vp), vp, ci, ci, i64, ci, vp, vp, vp]
    L.srft_cache_destroy.argtypes = [vp]
    L.srft_cache_append.argtypes = [vp, vp, ci, vp]
    L.srft_cache_rebuild_view.argtypes = [vp, vp]
    L.srft_cache_tokens.argtypes = [vp]
    L.srft_cache_quantized_tokens.argtypes = [vp]
    L.srft_scores_workspace_bytes.argtypes = [vp]
    L.srft_kv_scores.argtypes = [vp, vp, ci, vp, vp, i64, vp, vp, vp]
    L.srft_attend_workspace_bytes.argtypes = [vp]
    L.srft_kv_attend.argtypes = [vp, vp, ci, vp, vp, i64, vp, vp, vp]
    L.srft_decode_attention_workspace_bytes.argtypes = [vp, vp, ci, i64]
    L.srft_kv_decode_attention.argtypes = [vp, vp, vp, ci, vp, vp, vp, vp, i64, C.c_float, vp, vp, vp]
    L.srft_kv_scores_static.argtypes = [vp, vp, ci, vp, vp, i64, vp, vp]
    L.srft_kv_channel_absmax.argtypes = [vp, vp, i64, vp, vp]
    L.srft_lambda_from_absmax.argtypes = [vp, ci, vp]
    L.srft_kv_quantize_batched.argtypes = [vp, vp, vp, vp, vp, ci, vp]
    L.srft_kv_dequantize_batched.argtypes = [vp, vp, vp, vp, vp, ci, vp]
    for name in ("srft_plan_d", "srft_plan_group_size", "srft_plan_groups", "srft_plan_code_bytes"):
        getattr(L, name).argtypes = [vp]
    L.srft_plan_get_signs.argtypes = [vp, vp]
    L.srft_plan_set_max_workgroups.argtypes = [vp, ci]
    L.srft_status_string.argtypes = [ci]
    L.srft_status_string.restype = C.c_char_p
    L.srft_last_hip_error.argtypes = []
    for name in EXPORTS:
        if name != "srft_status_string":
            getattr(L, name).restype = ci
    L.srft_scores_workspace_bytes.restype = i64
    L.srft_attend_workspace_bytes.restype = i64
    L.srft_decode_attention_workspace_bytes.restype = i64
    L.srft_cache_tokens.restype = i64
    L.srft_cache_quantized_tokens.restype = i64
    _lib = L
    return L


def _check(status: int, where: str) -> None:
    if status != 0:
        raise SrftError(status, where)


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dev_ptr(t: torch.Tensor, dtype, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous {dtype} tensor")
    return t.data_ptr()


# ---------------------------------------------------------------------------- C entry points
TRANSFORMS = {"dft": 0, "hadamard": 1}


def srft_plan_create(d: int, group_size: int, sign_seed: int, lam=None, bits: int = 4, transform: str = "dft") -> int:
    """Returns the opaque plan handle.  ``lam``: d positive floats (host) or None for all ones."""
    handle = C.c_void_p()
    lam_ptr = None
    if lam is not None:
        lam_arr = np.ascontiguousarray(np.asarray(lam, dtype=np.float32))
        if lam_arr.shape != (d,):
            raise ValueError("lambda must have d entries")
        lam_ptr = lam_arr.ctypes.data_as(C.c_void_p)
    if transform != "dft":
        _check(lib().srft_plan_create_ex(C.byref(handle), d, group_size, bits, TRANSFORMS[transform],
                                         sign_seed & (2 ** 64 - 1), lam_ptr), "srft_plan_create_ex")
    elif bits == 4:
        _check(lib().srft_plan_create(C.byref(handle), d, group_size, sign_seed & (2 ** 64 - 1), lam_ptr),
               "srft_plan_create")
    else:
        _check(lib().srft_plan_create_bits(C.byref(handle), d, group_size, bits, sign_seed & (2 ** 64 - 1), lam_ptr),
               "srft_plan_create_bits")
    return handle.value


def srft_plan_destroy(plan: int) -> None:
    _check(lib().srft_plan_destroy(plan), "srft_plan_destroy")


def srft_kv_quantize(plan: int, x: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor, stream=None) -> None:
    n = x.shape[0]
    _check(lib().srft_kv_quantize(plan, _dev_ptr(x, torch.float16, "x"), n,
                                  _dev_ptr(codes, torch.uint8, "codes"),
                                  _dev_ptr(scales, torch.float32, "scales"), _stream_handle(stream)),
           "srft_kv_quantize")


def srft_kv_quantize_butterfly(plan: int, x: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor, stream=None) -> None:
    """The write path with the transform as vector-ALU FFT butterflies (d = 128, g = 32, 4-bit): the comparison form."""
    _check(lib().srft_kv_quantize_butterfly(plan, _dev_ptr(x, torch.float16, "x"), x.shape[0],
                                            _dev_ptr(codes, torch.uint8, "codes"), _dev_ptr(scales, torch.float32, "scales"),
                                            _stream_handle(stream)), "srft_kv_quantize_butterfly")


def srft_kv_dequantize(plan: int, codes: torch.Tensor, scales: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    n = codes.shape[0]
    _check(lib().srft_kv_dequantize(plan, _dev_ptr(codes, torch.uint8, "codes"),
                                    _dev_ptr(scales, torch.float32, "scales"), n,
                                    _dev_ptr(out, torch.float16, "out"), _stream_handle(stream)),
           "srft_kv_dequantize")


class BatchTable:
    """Host arrays for one batched call: plan handles, device addresses, vector counts.  Marshalling only.

    Built once and reused by a decode loop whose buffers do not move; ``set_counts`` changes the number of
    vectors per entry between calls.  The tensors are kept alive by the table.
    """

    def __init__(self, plans, big, codes, scales, n_vec=None):
        """big: the fp16 tensors (x on the write path, out on the read path), one per plan."""
        k = len(plans)
        if not (len(big) == len(codes) == len(scales) == k):
            raise ValueError("one tensor of each kind per plan")
        self.count = k
        self._keep = (list(big), list(codes), list(scales))
        self.plans = (C.c_void_p * k)(*[int(h) for h in plans])
        self.big = (C.c_void_p * k)(*[_dev_ptr(t, torch.float16, "x/out") for t in big])
        self.codes = (C.c_void_p * k)(*[_dev_ptr(t, torch.uint8, "codes") for t in codes])
        self.scales = (C.c_void_p * k)(*[_dev_ptr(t, torch.float32, "scales") for t in scales])
        self.n_vec = (C.c_int64 * k)()
        self.set_counts([t.shape[0] for t in big] if n_vec is None else n_vec)

    def set_counts(self, n_vec) -> None:
        if len(n_vec) != self.count:
            raise ValueError("one count per plan")
        big, codes, scales = self._keep
        for i, n in enumerate(n_vec):
            if n > min(big[i].shape[0], codes[i].shape[0], scales[i].shape[0]):
                raise ValueError(f"entry {i}: {n} vectors exceed the buffers")
            self.n_vec[i] = int(n)


def srft_kv_quantize_batched(table: BatchTable, stream=None) -> None:
    _check(lib().srft_kv_quantize_batched(table.plans, table.big, table.n_vec, table.codes, table.scales,
                                          table.count, _stream_handle(stream)), "srft_kv_quantize_batched")


def srft_kv_dequantize_batched(table: BatchTable, stream=None) -> None:
    _check(lib().srft_kv_dequantize_batched(table.plans, table.codes, table.scales, table.n_vec, table.big,
                                            table.count, _stream_handle(stream)), "srft_kv_dequantize_batched")


def srft_kv_forward_f32(plan: int, x: torch.Tensor, w: torch.Tensor, stream=None) -> None:
    _check(lib().srft_kv_forward_f32(plan, _dev_ptr(x, torch.float16, "x"), x.shape[0],
                                     _dev_ptr(w, torch.float32, "w"), _stream_handle(stream)),
           "srft_kv_forward_f32")


def srft_kv_scores(plan: int, q: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor, scores: torch.Tensor,
                   workspace: torch.Tensor, stream=None) -> None:
    """scores [n_q, n_keys] fp32 <- inner products of q [n_q, d] with the keys stored as (codes, scales)."""
    if workspace.numel() * workspace.element_size() < lib().srft_scores_workspace_bytes(plan):
        raise ValueError("workspace too small")
    if scores.shape != (q.shape[0], codes.shape[0]):
        raise ValueError("scores must be [n_q, n_keys]")
    _check(lib().srft_kv_scores(plan, _dev_ptr(q, torch.float16, "q"), q.shape[0], _dev_ptr(codes, torch.uint8, "codes"),
                                _dev_ptr(scales, torch.float32, "scales"), codes.shape[0],
                                _dev_ptr(scores, torch.float32, "scores"), workspace.data_ptr(),
                                _stream_handle(stream)), "srft_kv_scores")


def srft_kv_scores_static(plan: int, q: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor, scores: torch.Tensor,
                          stream=None) -> None:
    """srft_kv_scores with the library's static workspace: nothing is allocated and no workspace is passed."""
    if scores.shape != (q.shape[0], codes.shape[0]):
        raise ValueError("scores must be [n_q, n_keys]")
    _check(lib().srft_kv_scores_static(plan, _dev_ptr(q, torch.float16, "q"), q.shape[0],
                                       _dev_ptr(codes, torch.uint8, "codes"), _dev_ptr(scales, torch.float32, "scales"),
                                       codes.shape[0], _dev_ptr(scores, torch.float32, "scores"),
                                       _stream_handle(stream)), "srft_kv_scores_static")


def srft_kv_attend(plan: int, weights: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor, out: torch.Tensor,
                   workspace: torch.Tensor, stream=None) -> None:
    """out [n_q, d] fp32 <- weights [n_q, n_keys] fp32 times the values stored as (codes, scales)."""
    if workspace.numel() * workspace.element_size() < lib().srft_attend_workspace_bytes(plan):
        raise ValueError("workspace too small")
    if weights.shape[1] != codes.shape[0] or out.shape[0] != weights.shape[0]:
        raise ValueError("weights must be [n_q, n_keys], out [n_q, d]")
    _check(lib().srft_kv_attend(plan, _dev_ptr(weights, torch.float32, "weights"), weights.shape[0],
                                _dev_ptr(codes, torch.uint8, "codes"), _dev_ptr(scales, torch.float32, "scales"),
                                codes.shape[0], _dev_ptr(out, torch.float32, "out"), workspace.data_ptr(),
                                _stream_handle(stream)), "srft_kv_attend")


def srft_kv_decode_attention(plan_k: int, plan_v: int, q: torch.Tensor, k_codes: torch.Tensor, k_scales: torch.Tensor,
                             v_codes: torch.Tensor, v_scales: torch.Tensor, softmax_scale: float, out: torch.Tensor,
                             workspace: torch.Tensor, stream=None) -> None:
    """out [n_q, d] fp32 <- softmax(softmax_scale * q K^T) V over the two stored records."""
    n_q, n_keys = q.shape[0], k_codes.shape[0]
    if workspace.numel() * workspace.element_size() < lib().srft_decode_attention_workspace_bytes(plan_k, plan_v, n_q, n_keys):
        raise ValueError("workspace too small")
    if v_codes.shape[0] != n_keys:
        raise ValueError("keys and values must be as many")
    _check(lib().srft_kv_decode_attention(plan_k, plan_v, _dev_ptr(q, torch.float16, "q"), n_q,
                                          _dev_ptr(k_codes, torch.uint8, "k_codes"), _dev_ptr(k_scales, torch.float32, "k_scales"),
                                          _dev_ptr(v_codes, torch.uint8, "v_codes"), _dev_ptr(v_scales, torch.float32, "v_scales"),
                                          n_keys, float(softmax_scale), _dev_ptr(out, torch.float32, "out"),
                                          workspace.data_ptr(), _stream_handle(stream)), "srft_kv_decode_attention")


def srft_kv_channel_absmax(plan: int, x: torch.Tensor, amax: torch.Tensor, stream=None) -> None:
    """amax (d fp32 on the device, >= 0) becomes max(amax, per-channel abs-max of the transform of x)."""
    if amax.numel() != lib().srft_plan_d(plan):
        raise ValueError("amax must have d entries")
    _check(lib().srft_kv_channel_absmax(plan, _dev_ptr(x, torch.float16, "x"), x.shape[0],
                                        _dev_ptr(amax, torch.float32, "amax"), _stream_handle(stream)),
           "srft_kv_channel_absmax")


def srft_lambda_from_absmax(amax) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(amax, dtype=np.float32))
    lam = np.empty_like(a)
    _check(lib().srft_lambda_from_absmax(a.ctypes.data_as(C.c_void_p), a.size, lam.ctypes.data_as(C.c_void_p)),
           "srft_lambda_from_absmax")
    return lam


def srft_plan_get_signs(plan: int) -> np.ndarray:
    d = lib().srft_plan_d(plan)
    out = np.empty(d, dtype=np.int8)
    _check(lib().srft_plan_get_signs(plan, out.ctypes.data_as(C.c_void_p)), "srft_plan_get_signs")
    return out


def srft_plan_set_max_workgroups(plan: int, n: int) -> None:
    _check(lib().srft_plan_set_max_workgroups(plan, n), "srft_plan_set_max_workgroups")


class Cache:
    """The library's cache manager over torch-owned buffers (marshalling only): per plan an int4 store, its scales
    and the fp16 view, each paged as [capacity / R][n_seq][R][...]."""

    def __init__(self, plans, n_seq: int, capacity_tokens: int, residual_tokens: int = 16, device="cuda"):
        self.plans = list(plans)
        d, G = self.plans[0].d, self.plans[0].groups
        self.n_seq, self.R, self.capacity, self.d = n_seq, residual_tokens, capacity_tokens, d
        if capacity_tokens < 1 or residual_tokens < 1 or capacity_tokens % residual_tokens:
            raise ValueError("capacity must be a positive multiple of the residual window")
        pages = capacity_tokens // residual_tokens
        k = len(self.plans)
        cb = self.plans[0].code_bytes
        self.codes = [torch.zeros(pages, n_seq, residual_tokens, cb, dtype=torch.uint8, device=device) for _ in range(k)]
        self.scales = [torch.zeros(pages, n_seq, residual_tokens, G, dtype=torch.float32, device=device) for _ in range(k)]
        self.view = [torch.zeros(pages, n_seq, residual_tokens, d, dtype=torch.float16, device=device) for _ in range(k)]
        handle = C.c_void_p()
        _check(lib().srft_cache_create(
            C.byref(handle), (C.c_void_p * k)(*[int(p.handle) for p in self.plans]), k, n_seq, capacity_tokens,
            residual_tokens, (C.c_void_p * k)(*[t.data_ptr() for t in self.codes]),
            (C.c_void_p * k)(*[t.data_ptr() for t in self.scales]),
            (C.c_void_p * k)(*[t.data_ptr() for t in self.view])), "srft_cache_create")
        self.handle = handle.value

    def append(self, new, stream=None) -> None:
        """new: one [n_seq, t, d] fp16 device tensor per plan (all with the same t)."""
        k = len(self.plans)
        if len(new) != k:
            raise ValueError("one tensor of new tokens per plan")
        t = new[0].shape[1]
        for x in new:
            if x.shape != (self.n_seq, t, self.d):
                raise ValueError("new tokens must be [n_seq, t, d]")
        ptrs = (C.c_void_p * k)(*[_dev_ptr(x, torch.float16, "new") if t else 0 for x in new])
        _check(lib().srft_cache_append(self.handle, ptrs, t, _stream_handle(stream)), "srft_cache_append")

    def prepare(self, new):
        """Pointer table for tensors that will be appended again and again from the same addresses (a decode
        loop with static buffers): pass it to ``append_prepared``."""
        t = new[0].shape[1]
        for x in new:
            if x.shape != (self.n_seq, t, self.d):
                raise ValueError("new tokens must be [n_seq, t, d]")
        return (C.c_void_p * len(new))(*[_dev_ptr(x, torch.float16, "new") for x in new]), t, list(new)

    def append_prepared(self, prepared, stream=None) -> None:
        _check(lib().srft_cache_append(self.handle, prepared[0], prepared[1], _stream_handle(stream)),
               "srft_cache_append")

    def rebuild_view(self, stream=None) -> None:
        _check(lib().srft_cache_rebuild_view(self.handle, _stream_handle(stream)), "srft_cache_rebuild_view")

    @property
    def tokens(self) -> int:
        return lib().srft_cache_tokens(self.handle)

    @property
    def quantized_tokens(self) -> int:
        return lib().srft_cache_quantized_tokens(self.handle)

    def close(self) -> None:
        if self.handle:
            _check(lib().srft_cache_destroy(self.handle), "srft_cache_destroy")
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---------------------------------------------------------------------------- convenience wrapper
class Plan:
    """One (layer, K|V) plan.  Allocates outputs with torch when none are passed; computes nothing itself."""

    def __init__(self, d: int, group_size: int = 32, sign_seed: int = 0, lam=None, bits: int = 4,
                 transform: str = "dft"):
        self.handle = srft_plan_create(d, group_size, sign_seed, lam, bits, transform)
        self.d, self.g, self.bits = d, group_size, bits
        self.groups = lib().srft_plan_groups(self.handle)
        self.code_bytes = lib().srft_plan_code_bytes(self.handle)

    def close(self) -> None:
        if self.handle:
            srft_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def signs(self) -> np.ndarray:
        return srft_plan_get_signs(self.handle)

    def quantize(self, x, codes=None, scales=None, stream=None):
        n = x.shape[0]
        if codes is None:
            codes = torch.empty(n, self.code_bytes, dtype=torch.uint8, device=x.device)
        if scales is None:
            scales = torch.empty(n, self.groups, dtype=torch.float32, device=x.device)
        srft_kv_quantize(self.handle, x, codes, scales, stream)
        return codes, scales

    def dequantize(self, codes, scales, out=None, stream=None):
        if out is None:
            out = torch.empty(codes.shape[0], self.d, dtype=torch.float16, device=codes.device)
        srft_kv_dequantize(self.handle, codes, scales, out, stream)
        return out

    def scores(self, q, codes, scales, out=None, workspace=None, stream=None):
        if out is None:
            out = torch.empty(q.shape[0], codes.shape[0], dtype=torch.float32, device=q.device)
        if workspace is None:
            workspace = torch.empty(lib().srft_scores_workspace_bytes(self.handle), dtype=torch.uint8, device=q.device)
        srft_kv_scores(self.handle, q, codes, scales, out, workspace, stream)
        return out

    def channel_absmax(self, x, amax=None, stream=None):
        if amax is None:
            amax = torch.zeros(self.d, dtype=torch.float32, device=x.device)
        srft_kv_channel_absmax(self.handle, x, amax, stream)
        return amax

    def forward_f32(self, x, w=None, stream=None):
        if w is None:
            w = torch.empty(x.shape[0], self.d, dtype=torch.float32, device=x.device)
        srft_kv_forward_f32(self.handle, x, w, stream)
        return w
