"""The C-ABI library loads, exports every declared symbol, and rejects bad
arguments before touching a GPU.  No compute call is made here."""
import ctypes
import os
import re

import pytest

from paper_2605_08134_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB_PATH):
        from paper_2605_08134_amd import build
        build.build_library(verbose=False)
    return B.lib()


def _declared():
    names = set()
    for h in ("dare.h", "dare_kernels.h", "dare_model.h"):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(dare_[a-z0-9_]+)\s*\(", text))
    return names


def test_every_declared_symbol_is_exported(L):
    declared = _declared()
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None


def test_bench_library_exports_what_its_header_declares(L):
    text = open(os.path.join(ROOT, "include", "dare_bench.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(dare_[a-z0-9_]+)\s*\(", text))
    assert declared == set(B.BENCH_EXPORTS)
    for name in declared:
        assert getattr(B.bench_lib(), name) is not None
        assert not hasattr(L, name)          # benchmark aids stay out of the product library


def test_version(L):
    assert re.fullmatch(r"\d+\.\d+", B.dare_version())


def _cfg(**kw):
    base = dict(struct_size=ctypes.sizeof(B.DareConfig), hidden=256, n_heads=4, head_dim=64,
                max_batch=1, max_seq=128, dtype=B.DARE_F32, score_head=0, device=0, flags=0)
    base.update(kw)
    return B.DareConfig(**base)


@pytest.mark.parametrize("kw,want", [
    (dict(struct_size=8), B.DARE_ERR_INVALID_ARG),
    (dict(hidden=255), B.DARE_ERR_INVALID_ARG),
    (dict(dtype=7), B.DARE_ERR_INVALID_ARG),
    (dict(flags=1), B.DARE_ERR_INVALID_ARG),
    (dict(max_seq=0), B.DARE_ERR_INVALID_ARG),
    (dict(score_head=2), B.DARE_ERR_UNSUPPORTED),
    (dict(hidden=96, n_heads=3, head_dim=32), B.DARE_ERR_UNSUPPORTED),
    (dict(hidden=320, n_heads=5, head_dim=64, max_batch=1 << 15, max_seq=1 << 15), B.DARE_ERR_UNSUPPORTED),
])
def test_create_rejects_bad_config(L, kw, want):
    ctx = ctypes.c_void_p(1234)
    fake = 0x1000  # never dereferenced: the checks come first
    st = L.dare_create(ctypes.byref(_cfg(**kw)), fake, fake, fake, fake, None, ctypes.byref(ctx))
    assert st == want
    assert not ctx.value
    assert L.dare_last_error(None)


def test_create_rejects_null_pointers(L):
    ctx = ctypes.c_void_p()
    assert L.dare_create(None, 1, 1, 1, 1, None, ctypes.byref(ctx)) == B.DARE_ERR_INVALID_ARG
    assert L.dare_create(ctypes.byref(_cfg()), None, 1, 1, 1, None, ctypes.byref(ctx)) == B.DARE_ERR_INVALID_ARG
    assert L.dare_create(ctypes.byref(_cfg()), 1, 1, 1, 1, None, None) == B.DARE_ERR_INVALID_ARG


def test_step_and_destroy_null_context(L):
    assert L.dare_layer_step(None, 0, 0.0, 1, 1, *([None] * 11)) == B.DARE_ERR_INVALID_ARG
    assert L.dare_destroy(None) == B.DARE_OK


def test_kernel_entry_points_reject_bad_arguments(L):
    f = 0x1000
    arr = (ctypes.c_void_p * 3)(f, None, None)
    assert L.dare_k_gemm(B.DARE_BF16, None, 64, f, 64, 64, 1, None, None, arr, 64, 64, None, 0, 1, 0, None) == B.DARE_ERR_INVALID_ARG
    assert L.dare_k_gemm(B.DARE_BF16, f, 32, f, 64, 64, 1, None, None, arr, 64, 64, None, 0, 1, 0, None) == B.DARE_ERR_INVALID_ARG
    assert L.dare_k_gemm(B.DARE_BF16, f, 96, f, 64, 96, 1, None, None, arr, 64, 64, None, 0, 1, 0, None) == B.DARE_ERR_UNSUPPORTED
    assert L.dare_k_gemm(5, f, 64, f, 64, 64, 1, None, None, arr, 64, 64, None, 0, 1, 0, None) == B.DARE_ERR_INVALID_ARG
    assert L.dare_k_gemm(B.DARE_BF16, f, 64, f, 128, 64, 1, None, None, arr, 64, 48, None, 0, 1, 0, None) == B.DARE_ERR_INVALID_ARG
    assert L.dare_k_score(f, 64, 64, 1, 0, f, 4, float("nan"), 0, None, f, None) == B.DARE_ERR_INVALID_ARG
    assert L.dare_k_score(f, 32, 64, 1, 0, f, 4, 0.1, 0, None, f, None) == B.DARE_ERR_INVALID_ARG
    assert L.dare_k_score(f, 64, 64, 2, 8, f, 4, 0.1, 0, None, f, None) == B.DARE_ERR_INVALID_ARG
    arr0 = (ctypes.c_void_p * 3)(None, None, None)
    assert L.dare_k_gemm(B.DARE_BF16, f, 256, f, 64, 256, 8, None, None, arr0, 64, 64, f, 64, 3, 512, None) == B.DARE_ERR_UNSUPPORTED
    assert L.dare_k_gemm(B.DARE_BF16, f, 256, f, 64, 256, 8, None, None, arr0, 64, 64, f, 64, 2, 100, None) == B.DARE_ERR_INVALID_ARG
    assert L.dare_k_compact(None, 1, 8, f, f, f, None) == B.DARE_ERR_INVALID_ARG
    assert L.dare_k_attention(B.DARE_BF16, f, f, f, f, 1, 8, 2, 96, None, None, None, 0, None) == B.DARE_ERR_UNSUPPORTED
    assert L.dare_k_attention(B.DARE_BF16, f, f, f, f, 1, 8, 2, 64, f, None, None, 0, None) == B.DARE_ERR_INVALID_ARG
    assert L.dare_k_copy_rows(f, f, 4, 24, None, None, None) == B.DARE_ERR_INVALID_ARG
    assert L.dare_k_pack_weight(B.DARE_F32, f, 8, 8, f, 4, None) == B.DARE_ERR_INVALID_ARG


def test_allocate_quantiles_host_function_matches_oracle(L):
    import numpy as np
    from oracle import dare_oracle as orc
    s = np.random.Generator(np.random.PCG64(4)).random(32) * 0.3
    for phi_bar, eps in ((0.3, 0.05), (0.9, 1e-3), (0.5, 10.0)):
        got = np.array(B.dare_allocate_quantiles(s, phi_bar, eps))
        assert np.allclose(got, orc.allocate_quantiles(s, phi_bar, eps), rtol=1e-12, atol=1e-15)
    for bad in ((0.3, 0.0), (1.5, 0.1), (-0.1, 0.1)):
        with pytest.raises(B.DareError):
            B.dare_allocate_quantiles(s, *bad)


def test_policy_mode_host_function_matches_oracle(L):
    from oracle import dare_oracle as orc
    for mode in (1, 2, 3):
        for layer in (0, 9, 10, 31):
            for step in range(5):
                for skip, every in ((0, 0), (10, 0), (0, 2), (10, 3)):
                    assert B.dare_policy_mode(mode, layer, step, skip, every) == \
                        orc.policy_mode(mode, layer, step, skip, every)
