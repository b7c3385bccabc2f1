"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments on the host before touching a device (no compute is launched here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "spectre.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2502_18394_amd import build
    path = os.path.join(ROOT, "paper_2502_18394_amd", "libspectre_hip.so")
    if not os.path.exists(path):
        build.build()
    L = ctypes.CDLL(path)
    L.spectre_last_error.restype = ctypes.c_char_p
    for n in ("spectre_mix_workspace_bytes", "spectre_prefix_bytes", "spectre_gate_workspace_bytes"):
        getattr(L, n).restype = ctypes.c_size_t
    return L


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spectre_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_four_named_entry_points():
    names = declared_functions()
    for n in ("spectre_mix_forward", "spectre_gate", "spectre_prefix_update", "spectre_prefix_readout"):
        assert n in names


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), f"{n} declared in spectre.h but not exported"


def test_version_and_supported_lengths(lib):
    assert lib.spectre_version() >= 100
    for n in (2, 4, 128, 196, 256, 512, 1024, 4096, 8192, 32768, 131072, 49, 360):
        assert lib.spectre_length_supported(n, 64) == 1, n
    # any other length up to 65536 goes through a padded power-of-two convolution
    for n in (1, 11, 26, 197, 1022, 1031, 3 * 4096, 65535, 65536):
        assert lib.spectre_length_supported(n, 64) == 1, n
    # 3 * 32768 = 24 * 4096 has a four-step plan with an odd factor; 5 * 32768 = 40 * 4096 has none
    assert lib.spectre_length_supported(3 * 32768, 64) == 1
    for n in (0, -4, 65537, 5 * 32768, 262144):
        assert lib.spectre_length_supported(n, 64) == 0, n
    assert lib.spectre_length_supported(1024, 48) == 0


def test_workspace_queries(lib):
    assert lib.spectre_mix_workspace_bytes(1, 131072, 32, 64, 1) > 32 * 131072 * 8
    assert lib.spectre_mix_workspace_bytes(256, 196, 12, 64, 0) == 256          # slab path needs no scratch
    assert lib.spectre_mix_workspace_bytes(1, 5 * 32768, 1, 64, 0) == 0         # unsupported
    # L=11: padded length 256; gate planes + scratch + two staging tensors of one pseudo-head
    assert lib.spectre_mix_workspace_bytes(1, 11, 1, 64, 0) == 256 * 8 + 256 * 32 * 8 + 11 * 32 * 8 + 256 * 32 * 8
    F = 32768 // 2 + 1
    assert lib.spectre_prefix_bytes(8, 32, 64, 32768, 0) == 8 * 32 * F * 64 * 8
    assert lib.spectre_prefix_bytes(8, 32, 64, 32768, 1) == 8 * 32 * 32768 * 64 * 4
    assert lib.spectre_prefix_bytes(8, 32, 64, 32768, 3) == 8 * 32 * 64 * 8
    assert lib.spectre_prefix_bytes(8, 32, 64, 32768, 4) == 32768 * 8
    assert lib.spectre_prefix_bytes(8, 32, 64, 1000, 0) == 0
    assert lib.spectre_prefix_bytes(8, 32, 64, 32768, 9) == 0


def test_bad_arguments_fail_on_the_host(lib):
    fake = ctypes.c_void_p(4096)      # never dereferenced: every call below fails validation first
    rc = lib.spectre_mix_forward(None, fake, fake, 1, 1024, 1, 64, 0, fake, ctypes.c_size_t(1 << 30), None)
    assert rc == 1 and b"null" in lib.spectre_last_error()
    rc = lib.spectre_mix_forward(fake, fake, ctypes.c_void_p(1 << 40), 1, 0, 1, 64, 0, fake, ctypes.c_size_t(1 << 30), None)
    assert rc == 1
    rc = lib.spectre_mix_forward(fake, fake, fake, 1, 1024, 1, 64, 0, fake, ctypes.c_size_t(1 << 30), None)
    assert rc == 1 and b"overlap" in lib.spectre_last_error()
    far = ctypes.c_void_p(1 << 40)
    rc = lib.spectre_mix_forward(fake, fake, far, 1, 5 * 32768, 1, 64, 0, fake, ctypes.c_size_t(1 << 30), None)
    assert rc == 2                                                                # unsupported length
    rc = lib.spectre_mix_forward(fake, fake, far, 1, 1024, 1, 32, 0, fake, ctypes.c_size_t(1 << 30), None)
    assert rc == 2                                                                # unsupported d
    rc = lib.spectre_mix_forward(fake, fake, far, 1, 1024, 1, 64, 7, fake, ctypes.c_size_t(1 << 30), None)
    assert rc == 1                                                                # bad dtype
    rc = lib.spectre_mix_forward(fake, fake, far, 1, 1024, 1, 64, 0, fake, ctypes.c_size_t(16), None)
    assert rc == 3 and b"workspace" in lib.spectre_last_error()
    rc = lib.spectre_mix_forward(fake, fake, far, 1, 1024, 1, 64, 0, ctypes.c_void_p(4097), ctypes.c_size_t(1 << 30), None)
    assert rc == 1 and b"aligned" in lib.spectre_last_error()
    rc = lib.spectre_gate(fake, 0, 0, ctypes.c_double(1.0), None, 1, 8, 1, ctypes.c_longlong(0), fake, fake,
                          ctypes.c_size_t(1 << 20), None)
    assert rc == 1
    rc = lib.spectre_prefix_init(None, None)
    assert rc == 1
    rc = lib.spectre_prefix_readout(None, fake, 0, fake, 0, fake, ctypes.c_size_t(1 << 20), None)
    assert rc == 1


def test_options_and_prepare_argument_checks(lib):
    """The tuning switches are host-side state: defaults, set, restore, bad values - no device needed.  spectre_prepare
    rejects bad sizes and unsupported (n, d) before it touches a device."""
    lib.spectre_get_option.restype = ctypes.c_long
    defaults = {0: 2, 1: 204, 2: 1, 3: 1, 4: 1, 5: 0, 6: 0}
    for which, val in defaults.items():
        assert lib.spectre_get_option(which) == val
    assert lib.spectre_set_option(0, ctypes.c_long(1)) == 0 and lib.spectre_get_option(0) == 1
    assert lib.spectre_set_option(2, ctypes.c_long(0)) == 0 and lib.spectre_get_option(2) == 0
    assert lib.spectre_mix_workspace_bytes(1, 4096, 8, 64, 1) > 256            # three-kernel route now needs scratch
    assert lib.spectre_set_option(1, ctypes.c_long(12)) == 0
    small = lib.spectre_mix_workspace_bytes(1, 8192, 32, 64, 1)
    for which in defaults:
        assert lib.spectre_set_option(which, ctypes.c_long(-1)) == 0
        assert lib.spectre_get_option(which) == defaults[which]
    assert lib.spectre_mix_workspace_bytes(1, 4096, 8, 64, 1) == 256
    assert small < lib.spectre_mix_workspace_bytes(1, 8192, 32, 64, 1)
    assert lib.spectre_set_option(0, ctypes.c_long(3)) == 1 and lib.spectre_get_option(0) == 2
    assert lib.spectre_set_option(9, ctypes.c_long(1)) == 1 and lib.spectre_get_option(9) == -1
    assert lib.spectre_prepare(0, 64) == 1
    assert lib.spectre_prepare(1024, 32) == 2
    assert lib.spectre_prepare(5 * 32768, 64) == 2 and b"length" in lib.spectre_last_error()
    fake, far = ctypes.c_void_p(4096), ctypes.c_void_p(1 << 40)
    rc = lib.spectre_mix_forward_ex(fake, fake, far, 1, 1024, 1, 64, 0, ctypes.c_uint(6), fake, ctypes.c_size_t(1 << 30), None)
    assert rc == 1 and b"flag" in lib.spectre_last_error()


def test_static_scratch_entry_point_rejects_what_does_not_fit(lib):
    lib.spectre_mix_static_bytes.restype = ctypes.c_size_t
    assert lib.spectre_mix_static_bytes() == 98 << 20
    fake, far = ctypes.c_void_p(4096), ctypes.c_void_p(1 << 40)
    # a length without a four-step plan, a batch whose gate planes exceed the array, a bad dtype, overlap, d
    assert lib.spectre_mix_forward_static(fake, fake, far, 1, 1000, 1, 64, 0, None) == 2
    assert lib.spectre_mix_forward_static(fake, fake, far, 2, 131072, 32, 64, 1, None) == 2
    assert b"exceeds" in lib.spectre_last_error()
    assert lib.spectre_mix_forward_static(fake, fake, far, 1, 1024, 1, 64, 5, None) == 1
    assert lib.spectre_mix_forward_static(fake, fake, fake, 1, 1024, 1, 64, 0, None) == 1
    assert lib.spectre_mix_forward_static(fake, fake, far, 1, 1024, 1, 32, 0, None) == 2
    assert lib.spectre_mix_forward_static(None, fake, far, 1, 1024, 1, 64, 0, None) == 1


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    from paper_2502_18394_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError):
        binding.lib()


def _plan_rule(n):
    """The documented rule, written out independently: in-LDS kernel for 2-3-5-7-smooth n <= 2048; four-step
    for n = N1 * N2, N1 in {256, 4096}, N2 <= 32 of the form {1,3,5,7} * 2^a; else padded convolution up to 65536."""
    if n < 1:
        return False
    m = n
    for p in (2, 3, 5, 7):
        while m % p == 0:
            m //= p
    if m == 1 and 2 <= n <= 2048:
        return True
    for n1 in (256, 4096):
        if n % n1 == 0:
            n2 = n // n1
            odd = n2
            while odd % 2 == 0:
                odd //= 2
            if n2 <= 32 and odd in (1, 3, 5, 7):
                return True
    return n <= 65536


def test_supported_lengths_follow_the_documented_rule(lib):
    for n in list(range(-2, 9000)) + list(range(65000, 66000)) + [k * 4096 for k in range(1, 40)] + [131072, 131073]:
        assert bool(lib.spectre_length_supported(n, 64)) == _plan_rule(n), n
        assert lib.spectre_length_supported(n, 32) == 0


def test_workspace_sizes_are_consistent(lib):
    """Every supported length reports a workspace; four-step lengths need the expanded gate plus scratch that never
    exceeds the memory-side-cache budget by more than one head."""
    for L in (256, 768, 4096, 12288, 32768, 98304, 131072):
        for BH in (1, 8, 32, 256):
            ws = lib.spectre_mix_workspace_bytes(1, L, BH, 64, 1)
            per_head = L * 32 * 8
            if (BH * L <= 65536 and L <= 2048) or L == 4096:
                assert ws == 256                       # one launch with the data in LDS, no scratch
                continue
            gate = BH * L * 8
            assert gate + per_head <= ws <= gate + max(per_head, 204 << 20) + 1024, (L, BH, ws)
    assert lib.spectre_wrm_apply_workspace_bytes(1, 131072, 32, 64, 17) == 256 + 2 * 32 * 512 * 64 * 4
    assert lib.spectre_wrm_apply_workspace_bytes(1, 131072, 32, 64, 8) == 256
    assert lib.spectre_wrm_apply_workspace_bytes(1, 100, 1, 64, 3) == 0          # 8 does not divide 100
