"""The C-ABI library builds for gfx950, loads without a GPU and exports every
symbol that include/svg2.h declares (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "svg2.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2505_18875_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.load_library()


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(svg2_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_five_entry_points():
    names = _declared()
    for n in ("svg2_kmeans", "svg2_permute", "svg2_select_topp", "svg2_sparse_attn", "svg2_forward"):
        assert n in names


def test_library_exports_every_declared_symbol(lib):
    from paper_2505_18875_amd import binding
    names = _declared()
    assert sorted(binding.EXPORTS) == names
    for n in names:
        assert hasattr(lib, n), n
    assert lib.svg2_version() >= 100
    assert lib.svg2_last_error() == b""


def test_workspace_queries_and_validation_run_on_the_host(lib):
    # size queries never touch the GPU
    assert lib.svg2_forward_workspace_size(1, 40, 75600, 128, 100, 500) > 3 * 40 * 75600 * 128 * 2
    assert lib.svg2_kmeans_workspace_size(1, 40, 75600, 128, 500) >= 256
    assert lib.svg2_permute_workspace_size(40, 75600, 500) >= 256
    assert lib.svg2_select_topp_workspace_size(40, 100, 500) >= 40 * 100 * 500 * 4
    assert lib.svg2_sparse_attn_workspace_size(1, 40, 75600, 128, 100, 500) >= 256
    # invalid arguments are rejected before anything is launched (no GPU needed)
    vp = ctypes.c_void_p
    one = vp(256)
    rc = lib.svg2_kmeans(one, 7, 1, 16, 64, 4, 1, one, one, one, one, None, one, 1 << 20, None)
    assert rc == 2 and b"dtype" in lib.svg2_last_error()
    rc = lib.svg2_kmeans(one, 0, 1, 16, 96, 4, 1, one, one, one, one, None, one, 1 << 20, None)
    assert rc == 2 and b"head dimension" in lib.svg2_last_error()
    rc = lib.svg2_kmeans(one, 0, 1, 16, 64, 17, 1, one, one, one, one, None, one, 1 << 20, None)
    assert rc == 1 and b"C = 17" in lib.svg2_last_error()
    rc = lib.svg2_kmeans(one, 0, 1, 16, 64, 4, 0, one, one, one, one, None, one, 1 << 20, None)
    assert rc == 1 and b"iters" in lib.svg2_last_error()
    rc = lib.svg2_kmeans(None, 0, 1, 16, 64, 4, 1, one, one, one, one, None, one, 1 << 20, None)
    assert rc == 1
    rc = lib.svg2_kmeans(one, 0, 1, 16, 64, 4, 1, one, one, one, one, None, one, 16, None)
    assert rc == 3 and b"workspace" in lib.svg2_last_error()
    rc = lib.svg2_select_topp(one, one, None, one, 1, 4, 4, 64, 1.5, one, one, None, None, one, 1 << 20, None)
    assert rc == 1 and b"top_p" in lib.svg2_last_error()
    rc = lib.svg2_permute(one, 1, 16, 5000, one, one, None, 0, None, None, 0, 0, one, 1 << 20, None)
    assert rc == 1
    # the entry point that allocates nothing rejects sizes beyond its built-in scratch before it touches the GPU
    rc = lib.svg2_permute_noalloc(one, 40, 75600, 4096, one, one, None, 0, None, None, 0, 0, None)
    assert rc == 3 and b"scratch" in lib.svg2_last_error()
    rc = lib.svg2_sparse_attn(one, one, one, 1, 1, 16, 128, 1, 1, one, one, one, one, None, 0.0, one, None, one,
                              1 << 20, None)
    assert rc == 1 and b"alias" in lib.svg2_last_error()
    rc = lib.svg2_forward(one, one, one, 1, 1, 16, 128, 1, 1, 0.9, 0, one, one, vp(512), None, one, 1 << 30, None)
    assert rc == 1 and b"iters" in lib.svg2_last_error()
    rc = lib.svg2_forward(one, one, one, 1, 40000, 64, 128, 1, 1, 0.9, 1, one, one, vp(512), None, one, 1 << 30, None)
    assert rc == 1 and b"32767" in lib.svg2_last_error()
    # a head of 2^31 bytes or more cannot be addressed by the attention kernels' 32-bit row offsets
    rc = lib.svg2_sparse_attn(one, one, one, 0, 1, 1 << 22, 128, 1, 1, one, one, one, one, None, 0.0, vp(512), None,
                              one, 1 << 20, None)
    assert rc == 1 and b"2^31" in lib.svg2_last_error()
    rc = lib.svg2_forward(one, one, one, 1, 1, 1 << 23, 128, 1, 1, 0.9, 1, one, one, vp(512), None, one, 1 << 30, None)
    assert rc == 1 and b"2^31" in lib.svg2_last_error()


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_2505_18875_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(FileNotFoundError):
        binding.load_library()
