"""Host-only checks of the C ABI: the library loads, exports every declared
symbol, and rejects bad arguments before touching any device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2510_21956_amd as la
    if not os.path.exists(la.library_path()):
        from paper_2510_21956_amd import build
        build.build_library()
    return la.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "la.h")).read()
    return sorted(set(re.findall(r"LA_API[^;(]*?\b(la_[a-z_]+)\s*\(", text)))


def test_exports_match_header(lib):
    names = declared_symbols()
    import paper_2510_21956_amd as la
    assert names == sorted(la.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_strings(lib):
    import paper_2510_21956_amd as la
    assert la.la_version() >= 100
    assert la.la_status_string(0) == "LA_OK"
    for code in range(1, 8):
        assert la.la_status_string(code).startswith("LA_ERR_")
    assert la.la_status_string(99) == "unknown la_status"


def test_workspace_bytes(lib):
    import paper_2510_21956_amd as la
    assert la.la_workspace_bytes(4, 16, 4096, 64, la.LA_F32, 1, 0) > 0
    assert la.la_workspace_bytes(4, 16, 4096, 64, la.LA_F32, 1, 1) > \
        la.la_workspace_bytes(4, 16, 4096, 64, la.LA_F32, 1, 0)
    assert la.la_workspace_bytes(4, 16, 4096, 48, la.LA_F32, 1, 0) == 0      # unsupported D
    assert la.la_workspace_bytes(4, 16, 4096, 256, la.LA_F32, 1, 1) > 0
    assert la.la_workspace_bytes(0, 16, 4096, 64, la.LA_F32, 1, 0) == 0      # bad shape
    assert la.la_workspace_bytes(1, 1, 1, 64, 7, 1, 0) == 0                  # bad dtype
    # size limits: B*H*N*D < 2^40 elements, B*H < 2^31 / 4096
    assert la.la_workspace_bytes(1, 1, 2 ** 31 - 1, 128, la.LA_F32, 1, 0) > 0
    assert la.la_workspace_bytes(64, 64, 2 ** 21, 128, la.LA_F32, 1, 0) == 0   # 2^40 elements
    assert la.la_workspace_bytes(1024, 1024, 64, 64, la.LA_F32, 1, 0) == 0     # too many slices
    # a backward pass that recomputes O and g needs room for them and for the forward pass
    assert la.la_workspace_bytes(4, 16, 4096, 64, la.LA_F32, 1, 2) >= \
        la.la_workspace_bytes(4, 16, 4096, 64, la.LA_F32, 1, 1) + \
        la.la_workspace_bytes(4, 16, 4096, 64, la.LA_F32, 1, 0) + 4 * 16 * 4096 * (64 * 4 + 4)
    # the test hook changes the plan, hence the sizes; 0, 0 restores the automatic plan
    auto = la.la_workspace_bytes(4, 16, 4096, 64, la.LA_F32, 1, 0)
    la.la_debug_override(64, 0)
    assert la.la_workspace_bytes(4, 16, 4096, 64, la.LA_F32, 1, 0) > auto
    la.la_debug_override(0, 1)
    assert la.la_saved_state_bytes(4, 16, 4096, 64, la.LA_F32, 1) == 0
    la.la_debug_override(0, 0)
    assert la.la_workspace_bytes(4, 16, 4096, 64, la.LA_F32, 1, 0) == auto
    # slices x segments must fit the launch grid
    la.la_debug_override(64, 0)
    assert la.la_workspace_bytes(1, 4096, 2 ** 26, 16, la.LA_F32, 1, 0) == 0
    la.la_debug_override(0, 0)
    # the hand-over buffer: present for the matrix-core head sizes, absent otherwise
    assert la.la_saved_state_bytes(4, 16, 4096, 64, la.LA_F32, 1) > 0
    assert la.la_saved_state_bytes(4, 16, 4096, 128, la.LA_BF16, 0) > 0
    assert la.la_saved_state_bytes(4, 16, 4096, 16, la.LA_F32, 1) == 0
    assert la.la_saved_state_bytes(4, 16, 4096, 48, la.LA_F32, 1) == 0


def test_argument_checks_precede_any_launch(lib):
    """Bad arguments are rejected on the host: these calls must return an error
    code without a GPU being present."""
    vp = ctypes.c_void_p
    fake = vp(0x1000)  # never dereferenced: validation fails first
    # NULL pointer
    rc = lib.la_forward(vp(0), fake, fake, fake, fake, 1, 1, 64, 16, 1.0, 0.5, 1, 0, fake, 1 << 20,
                        vp(0))
    assert rc == 1
    # bad shape
    rc = lib.la_forward(fake, fake, fake, fake, fake, 1, 1, 0, 16, 1.0, 0.5, 1, 0, fake, 1 << 20,
                        vp(0))
    assert rc == 2
    # unsupported D
    rc = lib.la_forward(fake, fake, fake, fake, fake, 1, 1, 64, 20, 1.0, 0.5, 1, 0, fake, 1 << 20,
                        vp(0))
    assert rc == 3
    # misaligned
    rc = lib.la_forward(vp(0x1004), fake, fake, fake, fake, 1, 1, 64, 16, 1.0, 0.5, 1, 0, fake,
                        1 << 20, vp(0))
    assert rc == 4
    # workspace too small
    rc = lib.la_forward(fake, fake, fake, fake, fake, 4, 16, 4096, 64, 1.0, 0.5, 1, 0, fake, 16,
                        vp(0))
    assert rc == 5
    rc = lib.la_backward(fake, fake, fake, fake, fake, fake, fake, fake, vp(0), 1, 1, 64, 16, 1.0,
                         0.5, 1, 0, fake, 1 << 20, vp(0))
    assert rc == 1
    # overlapping buffers (distinct 1 MiB-spaced fakes; O on top of Q, then dK on top of dQ)
    f = [vp(0x10000000 + k * (1 << 20)) for k in range(12)]
    rc = lib.la_forward(f[0], f[1], f[2], f[0], f[4], 1, 1, 64, 16, 1.0, 0.5, 1, 0, f[5], 1 << 20,
                        vp(0))
    assert rc == 7
    rc = lib.la_backward(f[0], f[1], f[2], f[3], f[4], f[5], f[6], f[6], f[8], 1, 1, 64, 16, 1.0,
                         0.5, 1, 0, f[9], 1 << 20, vp(0))
    assert rc == 7
    # a workspace that overlaps an input
    rc = lib.la_forward(f[0], f[1], f[2], f[3], f[4], 1, 1, 64, 16, 1.0, 0.5, 1, 0, f[1], 1 << 20,
                        vp(0))
    assert rc == 7
    rc = lib.la_backward(fake, fake, fake, fake, fake, fake, fake, fake, fake, 4, 16, 4096, 64,
                         1.0, 0.5, 1, 0, fake, 16, vp(0))
    assert rc == 5


def test_header_is_plain_c(tmp_path):
    """include/la.h is a C header: it must compile as C and as C++ on its own."""
    import shutil
    import subprocess
    hdr = os.path.join(ROOT, "include", "la.h")
    for cc, lang in (("gcc", "c"), ("g++", "c++")):
        if shutil.which(cc) is None:
            pytest.skip("%s not available" % cc)
        subprocess.run([cc, "-fsyntax-only", "-Wall", "-Werror", "-x", lang, hdr], check=True)
