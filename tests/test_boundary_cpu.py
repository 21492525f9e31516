"""CPU-only checks of the C-ABI boundary: the library loads, exports what
include/thi.h declares, and rejects bad arguments on the host before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2605_25655_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2605_25655_amd import build
        build.build(verbose=False)
    return binding.load_library()


def declared_symbols(header="thi.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(thi_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    from paper_2605_25655_amd import binding
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTED_SYMBOLS)
    for n in names:
        assert hasattr(lib, n), n


def test_probe_header_symbols_live_in_their_own_library(lib):
    """The benchmark's measurement probes are declared in include/thi_probe.h and exported by libthi_probe.so,
    not by the product library."""
    from paper_2605_25655_amd import binding
    names = declared_symbols("thi_probe.h")
    assert set(names) == set(binding.PROBE_SYMBOLS) and names
    assert os.path.exists(binding.probe_library_path())
    probe = binding.load_probe_library()
    for n in names:
        assert hasattr(probe, n), n
        assert not hasattr(lib, n), f"{n} must not be exported by libthi.so"


def test_version_and_status_strings(lib):
    assert lib.thi_version() >= 100
    assert lib.thi_status_string(0) == b"THI_OK"
    for s in range(1, 7):
        assert lib.thi_status_string(s).startswith(b"THI_ERR_")
    assert lib.thi_status_string(77) == b"THI_ERR_UNKNOWN"


def test_workspace_bytes_is_pure_and_monotone(lib):
    f = lib.thi_workspace_bytes
    assert f(9, 1, 8, 8) == 0 and f(0, 0, 8, 8) == 0 and f(1, 1, -1, 8) == 0
    a = f(1, 1, 4096, 4096)
    assert a > 0 and a == f(1, 1, 4096, 4096)
    assert f(1, 32, 4096, 4096) >= a
    mlp1, mlp2 = f(2, 32, 4096, 11008), f(2, 2048, 4096, 11008)
    assert mlp2 - mlp1 >= (2048 - 32) * 11008 * 2      # h buffer grows with M*I


def test_decode_workspace_is_small_and_gemm_needs_the_larger_one(lib):
    """Up to 32 tokens a workspace holds the status words and hand-over slots only (plus h for the MLP);
    the GEMM kernels' 256 MiB of partial tiles are added above, or while those kernels are forced -- and
    a forced GEMM call on a decode-sized workspace is refused on the host."""
    f = lib.thi_workspace_bytes
    small = f(1, 32, 4096, 4096)
    assert small < 20 << 20
    assert f(2, 32, 4096, 11008) == small + 32 * 11008 * 2
    assert f(1, 33, 4096, 4096) >= small + (256 << 20)
    buf = ctypes.create_string_buffer(1 << 12)
    p = ctypes.c_void_p((ctypes.addressof(buf) + 255) // 256 * 256)
    null = ctypes.c_void_p(0)
    prev = lib.thi_set_kernel_family(2)
    try:
        assert f(1, 32, 4096, 4096) >= small + (256 << 20)
        assert lib.thi_linear(p, p, p, 32, 4096, 4096, p, small, null) == 4
    finally:
        lib.thi_set_kernel_family(prev)
    # attention's workspace starts behind the other calls' status words and slots
    assert lib.thi_attention_workspace_bytes(1, 32, 32, 128, 4096) > small - 32 * 4096 * 0


def test_workspace_status_validates(lib):
    null = ctypes.c_void_p(0)
    buf = ctypes.create_string_buffer(1 << 12)
    p = ctypes.c_void_p((ctypes.addressof(buf) + 255) // 256 * 256)
    assert lib.thi_workspace_status(null, 1 << 30, null) == 1
    assert lib.thi_workspace_status(ctypes.c_void_p(p.value + 4), 1 << 30, null) == 3
    assert lib.thi_workspace_status(p, 1024, null) == 4
    assert lib.thi_status_string(6).startswith(b"THI_ERR_TIMEOUT")
    assert lib.thi_debug_handover(0, 0) == 0


def test_argument_errors_return_codes_without_launching(lib):
    buf = ctypes.create_string_buffer(1 << 12)
    base = ctypes.addressof(buf)
    p = ctypes.c_void_p((base + 255) // 256 * 256)
    odd = ctypes.c_void_p(p.value + 2)
    big = 1 << 40
    null = ctypes.c_void_p(0)
    # NULL pointers
    assert lib.thi_linear(null, p, p, 1, 8, 8, p, big, null) == 1
    assert lib.thi_rmsnorm_qkv(p, null, 1e-6, p, p, 1, 8, 8, p, big, null) == 1
    assert lib.thi_swiglu_mlp(p, p, null, p, p, 1, 8, 8, p, big, null) == 1
    assert lib.thi_linear(p, p, p, 1, 8, 8, null, big, null) == 1
    # shapes
    assert lib.thi_linear(p, p, p, 0, 8, 8, p, big, null) == 2
    assert lib.thi_linear(p, p, p, 1, 8, 12, p, big, null) == 2
    assert lib.thi_swiglu_mlp(p, p, p, p, p, 1, 8, 20, p, big, null) == 2
    assert lib.thi_swiglu_mlp(p, p, p, p, p, 1, 4, 8, p, big, null) == 2
    # alignment
    assert lib.thi_linear(odd, p, p, 1, 8, 8, p, big, null) == 3
    assert lib.thi_linear(p, p, p, 1, 8, 8, odd, big, null) == 3
    # workspace too small
    assert lib.thi_linear(p, p, p, 1, 8, 8, p, 1024, null) == 4
    assert lib.thi_workspace_init(null, 1 << 20, null) == 1
    assert lib.thi_workspace_init(p, 16, null) == 4
    # the fused variants and decode attention validate the same way
    assert lib.thi_linear_residual(p, p, null, p, 1, 8, 8, p, big, null) == 1
    assert lib.thi_linear_residual(p, p, odd, p, 1, 8, 8, p, big, null) == 3
    assert lib.thi_rmsnorm_swiglu_mlp(p, null, 1e-6, p, p, p, null, p, 1, 8, 8, p, big, null) == 1
    assert lib.thi_rmsnorm_swiglu_mlp(p, p, 1e-6, p, p, p, null, p, 1, 8, 12, p, big, null) == 2
    assert lib.thi_decode_attention(p, p, p, null, 1.0, p, 1, 2, 2, 128, 8, p, big, null) == 1
    assert lib.thi_decode_attention(p, p, p, p, 1.0, p, 1, 3, 2, 128, 8, p, big, null) == 2       # Hq % Hkv
    assert lib.thi_decode_attention(p, p, p, p, 1.0, p, 1, 2, 2, 96, 8, p, big, null) == 2        # head size
    assert lib.thi_decode_attention(odd, p, p, p, 1.0, p, 1, 2, 2, 128, 8, p, big, null) == 3
    assert lib.thi_decode_attention(p, p, p, p, 1.0, p, 1, 2, 2, 128, 8, p, 16, null) == 4
    assert lib.thi_attention_workspace_bytes(2, 8, 2, 128, 1000) >= 2 * 8 * 130 * 4
    assert lib.thi_attention_workspace_bytes(2, 8, 3, 128, 1000) == 0
    assert lib.thi_query_kernel_family(0, 8, 8, 0) == 0 and lib.thi_query_kernel_family(4096, 4096, 4096, 0) == 2


def test_kernel_family_switch_roundtrip(lib):
    prev = lib.thi_set_kernel_family(1)
    assert lib.thi_set_kernel_family(prev) == 1
