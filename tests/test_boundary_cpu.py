"""Host-side checks of the C-ABI boundary that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2603_08982_amd as sv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return sv.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "svgear.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(svgear_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    declared = _declared_symbols()
    assert set(declared) == set(sv.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_version_and_error_state(lib):
    assert lib.svgear_version() >= 1
    assert lib.svgear_last_hip_error() == 0


def test_kmeans_list_threshold_sets_and_queries(lib):
    lib.svgear_kmeans_list_threshold.restype = ctypes.c_int
    lib.svgear_kmeans_list_threshold.argtypes = [ctypes.c_int]
    default = lib.svgear_kmeans_list_threshold(0)
    assert default == 400
    assert lib.svgear_kmeans_list_threshold(7) == default
    assert lib.svgear_kmeans_list_threshold(-3) == 7      # query only
    assert lib.svgear_kmeans_list_threshold(default) == 7
    assert lib.svgear_kmeans_list_threshold(0) == default


def test_workspace_queries_are_monotone(lib):
    a = lib.svgear_kmeans_workspace(1, 1, 4096, 64, 32)
    b = lib.svgear_kmeans_workspace(1, 40, 75600, 128, 500)
    assert 0 < a < b
    assert lib.svgear_kmeans_workspace(0, 1, 10, 64, 2) == 0
    assert lib.svgear_permute_workspace(1, 1, 4096, 64) > 0
    assert lib.svgear_probe_route_workspace(1, 1, 4096, 64, 32, 64) >= 32 * 64 * 4
    assert lib.svgear_sparse_attn_comp_workspace(1, 40, 75600, 75600, 128, 100, 500) > 40 * 500 * 128 * 4


def test_invalid_arguments_are_rejected_on_the_host(lib):
    st = (ctypes.c_int64 * 3)(1, 1, 1)
    # null pointers
    assert lib.svgear_kmeans(None, None, 0, 1, 1, 16, 0, 64, st, 2, 1, None, None, None, None, None, 0, None) == -1
    assert lib.svgear_unpermute(None, None, 0, 1, 1, 16, 64, None, st, None) == -1
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: argument checks come first
    big = ctypes.c_size_t(1 << 40)
    # C > N - n_tail
    assert lib.svgear_kmeans(fake, None, 0, 1, 1, 16, 0, 64, (ctypes.c_int64 * 3)(1024, 1024, 64), 17, 1,
                             fake, None, fake, fake, fake, big, None) == -1
    # d not in {64,128}
    assert lib.svgear_kmeans(fake, None, 0, 1, 1, 16, 0, 32, (ctypes.c_int64 * 3)(512, 512, 32), 2, 1,
                             fake, None, fake, fake, fake, big, None) == -1
    # bad dtype
    assert lib.svgear_kmeans(fake, None, 7, 1, 1, 16, 0, 64, (ctypes.c_int64 * 3)(1024, 1024, 64), 2, 1,
                             fake, None, fake, fake, fake, big, None) == -1
    # workspace too small
    assert lib.svgear_kmeans(fake, None, 0, 1, 1, 16, 0, 64, (ctypes.c_int64 * 3)(1024, 1024, 64), 2, 1,
                             fake, None, fake, fake, fake, ctypes.c_size_t(8), None) == -2
    # negative budget
    assert lib.svgear_probe_route(fake, fake, fake, fake, fake, 0, fake, fake, 1, 1, 16, 16, 64, 2, 2, -5, 0.125, 0,
                                  fake, fake, fake, fake, fake, fake, big, None) == -1
    # unknown flag bit
    assert lib.svgear_probe_route(fake, fake, fake, fake, fake, 0, fake, fake, 1, 1, 16, 16, 64, 2, 2, 5, 0.125, 64,
                                  fake, fake, fake, fake, fake, fake, big, None) == -1
    # misaligned token pointer
    odd = ctypes.c_void_p(0x1004)
    assert lib.svgear_sparse_attn_comp(odd, fake, fake, 1, fake, fake, fake, fake, fake, fake, fake, 1, 1, 16, 16, 64,
                                       2, 2, 0.125, fake, None, fake, big, None) == -1


def test_argument_checks_of_the_variant_entry_points(lib):
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: argument checks come first
    big = ctypes.c_size_t(1 << 40)
    st = (ctypes.c_int64 * 3)(128 * 16, 128 * 16, 128)
    F = ctypes.c_float
    # adaptive budgets: p outside (0, 1], the per-row flag, a missing output
    for p in (0.0, -1.0, 1.5, float("nan")):
        assert lib.svgear_probe_route_top_p(fake, fake, fake, fake, fake, 1, fake, fake, 1, 1, 16, 16, 128, 2, 2, F(p),
                                            F(0.1), 0, fake, fake, fake, fake, fake, fake, fake, big, None) == -1
    assert lib.svgear_probe_route_top_p(fake, fake, fake, fake, fake, 1, fake, fake, 1, 1, 16, 16, 128, 2, 2, F(0.5),
                                        F(0.1), 2, fake, fake, fake, fake, fake, fake, fake, big, None) == -1
    assert lib.svgear_probe_route_top_p(fake, fake, fake, fake, fake, 1, fake, fake, 1, 1, 16, 16, 128, 2, 2, F(0.5),
                                        F(0.1), 0, fake, fake, fake, fake, fake, None, fake, big, None) == -1
    # row movement alone: no tensors, a null permutation
    src = (ctypes.c_void_p * 1)(0x1000)
    sst = ((ctypes.c_int64 * 3) * 1)((128 * 16, 128 * 16, 128))
    assert lib.svgear_permute_rows(fake, 1, 1, 16, 0, src, sst, src, 1, 128, None) == -1
    assert lib.svgear_permute_rows(None, 1, 1, 16, 1, src, sst, src, 1, 128, None) == -1
    # token-order attention: missing permutation, rows that are not 16-byte aligned, stride_n < d
    args_tail = (1, 1, 16, 16, 128, 2, 2, F(0.1))
    assert lib.svgear_sparse_attn_comp_token_order(fake, st, fake, fake, 1, fake, fake, fake, fake, fake, fake, fake,
                                                   None, *args_tail, fake, st, None, fake, big, None) == -1
    bad = (ctypes.c_int64 * 3)(129 * 16, 129 * 16, 129)
    assert lib.svgear_sparse_attn_comp_token_order(fake, st, fake, fake, 1, fake, fake, fake, fake, fake, fake, fake,
                                                   fake, *args_tail, fake, bad, None, fake, big, None) == -1
    short = (ctypes.c_int64 * 3)(64 * 16, 64 * 16, 64)
    assert lib.svgear_sparse_attn_comp_token_order(fake, short, fake, fake, 1, fake, fake, fake, fake, fake, fake,
                                                   fake, fake, *args_tail, fake, st, None, fake, big, None) == -1
    # more key clusters than the bf16 kernels' LDS tables hold: refused before anything is launched
    assert lib.svgear_sparse_attn_comp(fake, fake, fake, 1, fake, fake, fake, fake, fake, fake, fake, 1, 1, 4096, 4096,
                                       128, 2, 3000, F(0.1), fake, None, fake, big, None) == -4
    # the two-stage form exists for bf16, d = 128 only
    assert lib.svgear_sparse_attn_two_stage(fake, fake, fake, 0, fake, fake, fake, fake, fake, fake, fake, 1, 1, 16, 16,
                                            128, 2, 2, F(0.1), fake, None, fake, big, None) == -4


def test_product_has_no_cpu_fallback():
    import torch

    x = torch.zeros(1, 1, 16, 64)
    c = torch.zeros(1, 1, 2, 64)
    with pytest.raises(sv.SvgearError):
        sv.kmeans(x, c, 1)


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2603_08982_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("no CPU", ""), f


def test_static_scratch_entry_point_rejects_on_the_host(lib):
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: argument checks come first
    assert lib.svgear_permute_static_capacity() == 8 << 20
    # needs more scratch than the library's fixed array holds
    assert lib.svgear_permute_workspace(1, 40, 75600, 1500) > lib.svgear_permute_static_capacity()
    assert lib.svgear_permute_static(fake, 1, 40, 75600, 0, 1500, fake, fake, 0, None, None, None, 1, 128, None) == -2
    # non-positive sizes
    assert lib.svgear_permute_static(fake, 0, 1, 16, 0, 2, fake, fake, 0, None, None, None, 1, 128, None) == -1
