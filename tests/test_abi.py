"""The C-ABI library loads and exports every symbol include/efcp.h declares.
No compute call is made here (no GPU in this tier)."""
import ctypes
import os
import re

import pytest

from paper_2306_06098_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "efcp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(efcp_[a-z_]+)\s*\(", text)))


def test_header_declares_the_documented_entry_points():
    syms = _declared_symbols()
    for must in ("efcp_create", "efcp_step", "efcp_destroy", "efcp_workspace_bytes"):
        assert must in syms
    assert set(syms) == set(binding.EXPORTS)


def test_library_exports_every_declared_symbol():
    assert os.path.exists(binding.LIB_PATH), "build libefcp.so first (python -m paper_2306_06098_amd.build)"
    lib = ctypes.CDLL(binding.LIB_PATH)
    for s in _declared_symbols():
        assert hasattr(lib, s), f"libefcp.so does not export {s}"


def test_binding_signatures_cover_all_exports():
    lib = binding.load_library()
    for s in binding.EXPORTS:
        assert getattr(lib, s).argtypes is not None


def test_null_context_is_rejected_without_a_gpu():
    lib = binding.load_library()
    assert lib.efcp_destroy(None) == binding.EFCP_OK
    assert lib.efcp_step(None, None, None, None) == binding.EFCP_EINVAL
    assert lib.efcp_last_error(None) == b"null context"


def test_options_structure_matches_the_header():
    """struct efcp_options: int32 fields in the order the header declares them."""
    text = open(os.path.join(ROOT, "include", "efcp.h")).read()
    body = re.search(r"typedef struct efcp_options \{(.*?)\} efcp_options;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"int32_t\s+(\w+)\s*;", body)
    assert fields == [f[0] for f in binding.Options._fields_]
    assert ctypes.sizeof(binding.Options) == 4 * len(fields) == 20
    lib = binding.load_library()
    assert lib.efcp_create_opts(None, 10, 1, 1, 1.0, None, None, 0) == binding.EFCP_EINVAL


def test_row_length_arithmetic_matches_the_oracle(oracle_mod):
    """efcp_row_length is host arithmetic only (no device needed): global Top-k keeps k, block-wise
    Top-k keeps k per block of 16,384 and the same share, rounded up, of a ragged last block -- the
    rule the oracle implements independently."""
    lib = binding.load_library()
    B = binding.TOPK_BLOCK
    assert lib.efcp_row_length(1000, 10, 0) == 10
    assert lib.efcp_row_length(1000, 1001, 0) == 0                       # k > d
    assert lib.efcp_row_length(1000, 0, 0) == 0
    assert lib.efcp_row_length(10 * B, 164, B) == 1640
    assert lib.efcp_row_length(1000, 10, 4096) == 0                      # unsupported block size
    assert lib.efcp_row_length(1000, B + 1, B) == 0                      # more than a block holds
    ob = oracle_mod._load().eo_block_row_length
    for d in (1, 3, B - 1, B, B + 1, 272_474, 110_000_000, 2 ** 31 - 1):
        for kb in (1, 7, 164, 4099, B):
            assert lib.efcp_row_length(d, kb, B) == ob(d, B, kb), (d, kb)
    # a null context is refused by every new entry point too
    assert lib.efcp_step_ex(None, None, 0, None, None, 0.0, 0.0, None) == binding.EFCP_EINVAL
    assert lib.efcp_apply(None, None, None, None) == binding.EFCP_EINVAL
    assert lib.efcp_state_bytes(None) == 0


def test_header_is_plain_c(tmp_path):
    """include/efcp.h is a C header: it must compile as C99 and as C++11 with nothing but itself."""
    import shutil
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "efcp.h"\nint main(void) { efcp_options o = {0, 0, 0, 0, 0}; (void)o; '
                   'return efcp_destroy(0) == EFCP_OK ? 0 : 1; }\n')
    inc = os.path.join(ROOT, "include")
    if shutil.which("gcc"):
        subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                        "-I", inc, str(src)], check=True)
    if shutil.which("g++"):
        subprocess.run(["g++", "-std=c++11", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                        "-x", "c++", "-I", inc, str(src)], check=True)


def test_default_slice_width_invariants():
    """The automatic d-slice width (host arithmetic): a multiple of 64 in [1024, 16384]; either the
    widest slice, with less than 2 % of the places of its rounds of 256 empty, or slices that fit
    the same number of rounds as the widest would need and leave less than one slice per
    workgroup of slack; never more slices per workgroup than the SP kernel has room for; the
    values the GPU tests and the design notes quote."""
    lib = binding.load_library()
    import numpy as np
    rng = np.random.default_rng(5)
    ds = [1, 3, 1023, 1024, 5_000, 65_536, 272_474, 4_194_304, 4_194_305, 11_200_000, 21_100_000, 110_000_000,
          340_000_000, 2 ** 31 - 1] + [int(x) for x in np.exp(rng.uniform(0, np.log(2.0 ** 31 - 1), 400))]
    for d in ds:
        w = lib.efcp_default_slice_width(d, 0)
        assert 1024 <= w <= 16384 and w % 64 == 0, (d, w)
        n = -(-d // w)
        widest = -(-d // 16384)
        rounds = -(-widest // 256)
        if w == 16384:
            assert (rounds * 256 - widest) * 50 < rounds * 256 or d <= 1024 * 256 // 1, (d, w)
        else:
            assert n <= rounds * 256 or w == 1024, (d, w, n)
            assert rounds * 256 - n < 256 or w == 1024, (d, w, n)
        assert -(-(-(-n // 8)) // 32) <= 512
        assert lib.efcp_default_slice_width(d, binding.TOPK_BLOCK) == 16384
    for d, want in [(5_000, 1024), (272_474, 1280), (11_200_000, 14_592), (4_194_304, 16_384), (4_194_305, 8_256),
                    (21_100_000, 13_760), (110_000_000, 15_936), (340_000_000, 16_384)]:
        assert lib.efcp_default_slice_width(d, 0) == want
    assert lib.efcp_default_slice_width(0, 0) == 0 and lib.efcp_default_slice_width(2 ** 31, 0) == 0
    assert lib.efcp_default_slice_width(1000, 4096) == 0
