"""Host-side checks that need no GPU: the library loads, exports what the header declares,
and rejects bad arguments before touching HIP."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2605_05699_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2605_05699_amd import build
        build.build()
    return binding.lib()


def declared_functions(header="srft_kv.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(srft_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert "srft_plan_create" in names and "srft_kv_quantize" in names and "srft_kv_dequantize" in names
    for name in names:
        assert hasattr(L, name), f"{name} declared in srft_kv.h but not exported"
    from paper_2605_05699_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_measurement_library_exports_its_header_and_nothing_of_it_is_in_the_product(L):
    from paper_2605_05699_amd import measure
    M = measure.lib()
    names = declared_functions("srft_measure.h")
    assert sorted(measure.EXPORTS) == names
    for name in names:
        assert hasattr(M, name), f"{name} declared in srft_measure.h but not exported"
        assert not hasattr(L, name), f"{name} is a measurement aid and must not be in libsrft_kv.so"
    # argument checks precede HIP: byte counts are multiples of 16, not both zero; either may be zero
    assert M.srft_stream_copy(None, None, 24, None) == -7
    assert M.srft_stream_copy(None, None, 32, None) == -1
    assert M.srft_stream_copy(None, None, 0, None) == 0
    for rb, wb in ((0, 0), (-16, 16), (16, -16), (24, 16), (16, 8)):
        assert M.srft_stream_mix(None, None, 4, rb, wb, 0, 0, None) == -7, (rb, wb)
    assert M.srft_stream_mix(None, None, -1, 16, 16, 0, 0, None) == -7
    assert M.srft_stream_mix(None, None, 0, 16, 0, 0, 0, None) == 0          # no tiles: nothing to do
    assert M.srft_stream_mix(None, None, 4, 16, 0, 0, 1, None) == -1         # read-only is a valid shape; pointers are not
    assert M.srft_stream_mix(None, None, 4, 0, 16, 0, 0, None) == -1


def test_the_library_reads_no_environment_variables():
    """Kernel choice depends on the plan alone: no getenv anywhere in the product sources."""
    import glob
    for path in glob.glob(os.path.join(ROOT, "paper_2605_05699_amd", "csrc", "**", "*.h*"), recursive=True):
        assert "getenv" not in open(path).read(), path


def test_status_strings(L):
    for code in range(0, -12, -1):
        assert L.srft_status_string(code)
    known = {L.srft_status_string(code) for code in range(0, -11, -1)}
    assert len(known) == 11 and L.srft_status_string(-11) not in known     # -10 is the last defined status
    assert L.srft_status_string(0) == b"ok"


def test_plan_create_rejects_bad_arguments_before_any_hip_call(L):
    h = C.c_void_p()
    lam = (C.c_float * 256)(*([1.0] * 256))
    assert L.srft_plan_create(None, 128, 32, 0, None) == -1
    for d in (0, 2, 16, 31, 100, 130, 288, 512, -128):
        assert L.srft_plan_create(C.byref(h), d, 32, 0, None) == -2, d
        assert h.value is None
    for g in (0, 8, 33, 48, 96, 256, -32):
        assert L.srft_plan_create(C.byref(h), 128, g, 0, None) == -3, g
    for bits in (0, 3, 6, 16, -4):
        assert L.srft_plan_create_bits(C.byref(h), 128, 32, bits, 0, None) == -9, bits
    assert L.srft_plan_create_bits(C.byref(h), 100, 32, 8, 0, None) == -2
    assert L.srft_plan_bits(None) == -1
    assert L.srft_plan_create_ex(C.byref(h), 128, 32, 4, 7, 0, None) == -10
    assert L.srft_plan_create_ex(C.byref(h), 96, 32, 4, 1, 0, None) == -2      # Hadamard needs a power of two
    for bad in (0.0, -1.0, float("nan"), float("inf")):
        lam[17] = bad
        assert L.srft_plan_create(C.byref(h), 128, 32, 0, lam) == -4, bad
    lam[17] = 1.0
    lam[3] = 1e-3
    lam[4] = 1e3            # ratio 1e6 > 2^16
    assert L.srft_plan_create(C.byref(h), 128, 32, 0, lam) == -4


def test_null_plan_and_size_errors(L):
    assert L.srft_kv_quantize(None, None, 1, None, None, None) == -1
    assert L.srft_kv_dequantize(None, None, None, 1, None, None) == -1
    assert L.srft_kv_forward_f32(None, None, 1, None, None) == -1
    assert L.srft_plan_d(None) == -1
    assert L.srft_plan_destroy(None) == 0
    # lambda from the calibration statistic: host only
    amax = (C.c_float * 4)(2.0, 0.0, 1e-9, 0.5)
    lam = (C.c_float * 4)()
    assert L.srft_lambda_from_absmax(amax, 4, lam) == 0
    assert list(lam) == [0.5, 2.0 ** 15, 2.0 ** 15, 2.0]
    zero = (C.c_float * 4)()
    assert L.srft_lambda_from_absmax(zero, 4, lam) == 0 and list(lam) == [1.0] * 4
    assert L.srft_lambda_from_absmax(None, 4, lam) == -1 and L.srft_lambda_from_absmax(amax, 0, lam) == -2
    amax[1] = -1.0
    assert L.srft_lambda_from_absmax(amax, 4, lam) == -4
    amax[1] = float("nan")
    assert L.srft_lambda_from_absmax(amax, 4, lam) == -4
    assert L.srft_kv_channel_absmax(None, None, 1, None, None) == -1
    assert L.srft_kv_scores(None, None, 1, None, None, 1, None, None, None) == -1
    assert L.srft_scores_workspace_bytes(None) == -1
    # cache manager: argument checks need no GPU (and no plan: a NULL plan entry is caught first)
    h = C.c_void_p()
    one = (C.c_void_p * 1)(None)
    assert L.srft_cache_create(None, one, 1, 1, 16, 16, one, one, one) == -1
    assert L.srft_cache_create(C.byref(h), None, 1, 1, 16, 16, one, one, one) == -1
    for bad in ((0, 1, 16, 16), (1, 0, 16, 16), (1, 1, 16, 0), (1, 1, 8, 16), (1, 1, 24, 16), (1, 1, 0, 16)):
        assert L.srft_cache_create(C.byref(h), one, bad[0], bad[1], bad[2], bad[3], one, one, one) == -7, bad
    assert L.srft_cache_create(C.byref(h), one, 1, 1, 16, 16, one, one, one) == -1 and h.value is None
    assert L.srft_cache_destroy(None) == 0
    assert L.srft_cache_append(None, None, 1, None) == -1 and L.srft_cache_rebuild_view(None, None) == -1
    assert L.srft_cache_tokens(None) == -1 and L.srft_cache_quantized_tokens(None) == -1
    # batched calls: an empty list is a no-op, a negative count or a missing array is an error
    one = (C.c_void_p * 1)(None)
    n1 = (C.c_int64 * 1)(5)
    for fn in (L.srft_kv_quantize_batched, L.srft_kv_dequantize_batched):
        assert fn(None, None, None, None, None, 0, None) == 0
        assert fn(None, None, None, None, None, -3, None) == -7
        assert fn(None, None, None, None, None, 1, None) == -1
        assert fn(one, one, n1, one, one, 1, None) == -1          # entry 0 has no plan


def test_workload_table_matches_the_stated_shapes():
    from paper_2605_05699_amd import workloads as W
    w = W.WORKLOADS
    assert w["tiny"].total_vectors == 512
    assert w["qwen2.5-1.5b-4k"].total_vectors == 458_752
    assert w["gemma3-1b-4k"].total_vectors == 212_992
    assert w["decode-d96"].append_vectors_per_plan * w["decode-d96"].n_plans == 32_768
    assert w["decode-d96"].vectors_per_plan == 4_194_304
    assert w["llama3-70b-128k"].vectors_per_plan == 1_048_576
    assert w["llama3-70b-128k"].total_vectors == 167_772_160
    # generators are deterministic and plan-specific
    a = W.make_kv(w["tiny"], 0)
    b = W.make_kv(w["tiny"], 0)
    c = W.make_kv(w["tiny"], 1)
    assert a.shape == (256, 128) and bool((a == b).all()) and not bool((a == c).all())
    seed, lam, gain = W.plan_constants(w["tiny"], 0)
    assert lam.shape == (128,) and (lam > 0).all() and int((gain == 20).sum()) == 4
    assert np.isclose(float(a.float().std()), float(np.sqrt((gain ** 2).mean())), rtol=0.1)
