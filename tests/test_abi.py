"""Host-side checks of the C ABI (no GPU): the built library loads and exports every function that
include/hispec.h declares, the Python binding lists the same names, and argument checks that need no
device work return the documented error codes."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "hispec.h")
LIB = os.path.join(ROOT, "paper_2510_01336_amd", "libhispec.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+)?[A-Za-z_][A-Za-z_0-9]*\s*\*?\s*\b((?:ee|kv)_[a-z_0-9]+)\s*\(", text, flags=re.M)
    return sorted(set(names))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} is missing: run `python paper_2510_01336_amd/build.py` (hipcc cross-compiles without a GPU)")
    import torch  # noqa: F401  (brings the HIP runtime the library links against into the process)
    return ctypes.CDLL(LIB)


def test_header_declares_the_five_calls_of_the_path():
    names = declared_functions()
    for required in ("ee_model_load", "ee_draft", "ee_verify_intermediate", "ee_verify_full", "kv_rollback"):
        assert required in names


def test_library_exports_every_declared_function(lib):
    missing = [n for n in declared_functions() if not hasattr(lib, n)]
    assert not missing, missing


def test_binding_lists_the_same_names():
    import paper_2510_01336_amd as hs
    assert sorted(hs.EXPORTED_SYMBOLS) == declared_functions()
    for n in hs.EXPORTED_SYMBOLS:
        assert callable(getattr(hs, n)), n


def test_config_checks_need_no_device(lib):
    import paper_2510_01336_amd as hs
    import synth
    lib.ee_model_bytes.restype = ctypes.c_size_t
    lib.ee_last_error.restype = ctypes.c_char_p
    good = hs.make_config(synth.tiny_config())
    assert lib.ee_model_bytes(ctypes.byref(good)) > 0
    bad = hs.make_config(synth.tiny_config())
    bad.exit_inter = bad.exit_draft            # exits must be strictly increasing
    assert lib.ee_model_bytes(ctypes.byref(bad)) == 0
    assert b"L_d" in lib.ee_last_error()
    # the 8B-shaped bf16 model: 16.06 GB of weights in the library's layout (bf16, padded tiles)
    big = hs.make_config(synth.llama8b_config())
    n = lib.ee_model_bytes(ctypes.byref(big))
    params = 32 * 218103808 + 2 * 128256 * 4096
    assert 2 * params <= n <= 2 * params * 1.01
    # null / misaligned arenas are refused before any device work
    out = ctypes.c_void_p()
    assert lib.ee_model_load(ctypes.byref(good), None, 0, 0, None, ctypes.byref(out)) == -1


def test_config_checks_of_the_optional_model_parts(lib):
    """Low-rank exit heads (App. I) and further verifier exits: shape rules and their cost in bytes, no device."""
    import paper_2510_01336_amd as hs
    import synth
    lib.ee_model_bytes.restype = ctypes.c_size_t
    lib.ee_last_error.restype = ctypes.c_char_p
    plain = lib.ee_model_bytes(ctypes.byref(hs.make_config(synth.llama8b_config())))
    heads = lib.ee_model_bytes(ctypes.byref(hs.make_config(synth.llama8b_config(head_rank=1024))))
    # two exits x (A: 1024 x 4096, B: 4096 x 1024) in bf16 = 33.6 MB plus gains and alignment: under 2 % of the model
    assert 2 * 2 * 2 * 1024 * 4096 <= heads - plain <= 2 * 2 * 2 * 1024 * 4096 + 65536
    bad = hs.make_config(synth.llama8b_config())
    bad.head_rank = 40                                   # bf16 models need a multiple of 32
    assert lib.ee_model_bytes(ctypes.byref(bad)) == 0 and b"head_rank" in lib.ee_last_error()
    chain = hs.make_config(synth.llama8b_config(exit_extra=(20, 24)))
    assert (chain.n_extra_exits, list(chain.extra_exits)[:2]) == (2, [20, 24])
    assert lib.ee_model_bytes(ctypes.byref(chain)) == plain     # exits add no weights
    for extra in ((16,), (24, 20), (32,)):               # not above L_i, not increasing, not below L_f
        bad = hs.make_config(synth.llama8b_config())
        bad.n_extra_exits = len(extra)
        for i, e in enumerate(extra):
            bad.extra_exits[i] = e
        assert lib.ee_model_bytes(ctypes.byref(bad)) == 0 and b"verifier exits" in lib.ee_last_error()


def test_gemm_form_selector_checks_its_argument(lib):
    """The tuning entry point that forces the narrow-projection GEMM form: host state only, no device."""
    lib.ee_last_error.restype = ctypes.c_char_p
    for ok in (0, 4, 8, 16, 104, 108, -1):
        assert lib.ee_debug_gemm_row_blocks(ok) == 0, ok
    for bad in (1, 12, 32, 100, -2, 1001):
        assert lib.ee_debug_gemm_row_blocks(bad) == -1, bad
        assert b"row_tiles" in lib.ee_last_error()
    assert lib.ee_debug_gemm_row_blocks(-1) == 0


def test_attention_split_selector_checks_its_argument(lib):
    lib.ee_last_error.restype = ctypes.c_char_p
    for ok in (2, 1, 17, 0):
        assert lib.ee_debug_attention_split_pages(ok) == 0, ok
    assert lib.ee_debug_attention_split_pages(-3) == -1 and b"pages per split" in lib.ee_last_error()
    assert lib.ee_debug_attention_split_pages(0) == 0


def test_read_floor_checks_its_arguments(lib):
    """Bad arguments are refused before any device call."""
    lib.ee_last_error.restype = ctypes.c_char_p
    f = lib.ee_debug_read_floor
    f.restype = ctypes.c_int
    f.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_size_t), ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_float),
                  ctypes.c_void_p]
    sizes = (ctypes.c_size_t * 2)(4096, 4096)
    out = (ctypes.c_float * 2)()
    assert f(None, sizes, 2, 1, out, None) == -1 and b"read floor" in lib.ee_last_error()
    assert f(ctypes.c_void_p(256), sizes, 0, 1, out, None) == -1
    assert f(ctypes.c_void_p(256), sizes, 17, 1, out, None) == -1
    assert f(ctypes.c_void_p(256), sizes, 2, 0, out, None) == -1
    assert f(ctypes.c_void_p(264), sizes, 2, 1, out, None) == -1          # not 16-byte aligned
    odd = (ctypes.c_size_t * 2)(4096, 100)
    assert f(ctypes.c_void_p(256), odd, 2, 1, out, None) == -1 and b"multiple of 16" in lib.ee_last_error()
