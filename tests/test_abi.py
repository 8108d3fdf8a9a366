"""CPU checks of the C-ABI library: it loads, exports every symbol the header declares, and rejects bad
arguments before touching the GPU (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "lite_attn.h")
# the sanitizer run (test_sanitizers.py) points this suite at its own build of the library's host side
LIB = os.environ.get("LITE_ATTN_TEST_LIB") or os.path.join(ROOT, "paper_2511_11062_amd", "liblite_attn.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    return ctypes.CDLL(LIB)


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lite_attn_[a-z_]+)\s*\(", text)))


def test_header_declares_the_named_entry_points():
    names = declared_functions()
    for n in ("lite_attn_init_mask", "lite_attn_fwd", "lite_attn_skip_stats"):
        assert n in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_bad_arguments_are_rejected_on_the_host(lib):
    from paper_2511_11062_amd import lite_attn as la
    ok = dict(batch=1, heads=2, seqlen=256)
    h = ctypes.c_void_p()
    assert lib.lite_attn_init_mask(None, ctypes.byref(h)) == -1
    def rc(**kw):
        args = dict(ok); args.update(kw)
        strides = args.pop("strides", (args["heads"] * args["seqlen"] * 128, args["seqlen"] * 128, 128))
        d = la.Desc(args["batch"], args["heads"], args["seqlen"], args.get("head_dim", 128), args.get("tile_q", 128),
                    args.get("tile_k", 128), strides[0], strides[1], strides[2], args.get("ps", 0), args.get("pl", 0),
                    args.get("flags", 0), args.get("max_steps", 4))
        return lib.lite_attn_init_mask(ctypes.byref(d), ctypes.byref(h))
    assert rc(batch=0) == -1 and rc(seqlen=0) == -1 and rc(max_steps=0) == -1 and rc(flags=4) == -1
    assert rc(strides=(0, 100, 128)) == -1            # stride not a multiple of 8 elements
    assert rc(strides=(65536, 0, 128)) == -1          # two heads on top of each other
    assert rc(pl=10, ps=250) == -1                    # protected range past the end
    assert rc(head_dim=64) == -3 and rc(tile_q=64) == -3 and rc(tile_k=176) == -3
    assert rc(seqlen=128 * 70000) == -3
    assert h.value is None
    # calls on a null handle
    assert lib.lite_attn_fwd(None, None, None, None, None, ctypes.c_float(-1.0), 0) == -1
    assert lib.lite_attn_skip_stats(None, 0, None) == -1
    assert lib.lite_attn_mask_words(None) == 0
    lib.lite_attn_free_mask(None)
    # contexts
    assert lib.lite_attn_ctx_create(None) == -1
    assert lib.lite_attn_ctx_set_stream(None, None) == -1
    ok_desc = la.Desc(1, 2, 256, 128, 128, 128, 2 * 256 * 128, 256 * 128, 128, 0, 0, 0, 4)
    assert lib.lite_attn_init_mask_shared(ctypes.byref(ok_desc), None, ctypes.byref(h)) == -1
    assert lib.lite_attn_ctx_free(None) == 0
    lib.lite_attn_strerror.restype = ctypes.c_char_p
    assert b"step" in lib.lite_attn_strerror(-2) and b"shared" in lib.lite_attn_strerror(-6)


def test_allocation_free_entry_point_rejects_on_the_host(lib):
    """lite_attn_fwd_static checks its arguments and the scratch limit before it touches a device."""
    from paper_2511_11062_amd import lite_attn as la
    if not hasattr(lib, "lite_attn_fwd_static"):
        pytest.skip("host-only sanitizer build: the entry point lives beside its device array")
    f = lib.lite_attn_fwd_static
    f.argtypes = [ctypes.c_void_p] * 4 + [ctypes.POINTER(la.Desc), ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p]
    small = la.make_desc(1, 2, 300, max_steps=1)
    a = 4096                                                          # never dereferenced: every case fails earlier
    assert f(a, a, a, a, None, a, -1.0, None) == -1
    assert f(None, a, a, a, ctypes.byref(small), a, -1.0, None) == -1
    assert f(a, a, a, a + 8, ctypes.byref(small), a, -1.0, None) == -1           # out not 16-byte aligned
    assert f(a, a, a, a, ctypes.byref(small), None, -1.0, None) == -1
    assert f(a, a, a, a, ctypes.byref(small), a + 4, -1.0, None) == -1           # mask not 8-byte aligned
    assert f(a, a, a, a, ctypes.byref(small), a, 0.5, None) == -1
    assert f(a, a, a, a, ctypes.byref(la.make_desc(1, 2, 300, head_dim=64, strides=(2 * 300 * 64, 300 * 64, 64))), a,
             -1.0, None) == -3
    # the Wan-14B-like layer needs 0.77 GB of scratch: more than the static array holds
    assert f(a, a, a, a, ctypes.byref(la.make_desc(1, 40, 75600)), a, -1.0, None) == -7
    text = open(HEADER).read()
    assert re.search(r"#define\s+LITE_ATTN_STATIC_SCRATCH_BYTES\s+\(128u << 20\)", text)
    lib.lite_attn_strerror.restype = ctypes.c_char_p
    assert b"static" in lib.lite_attn_strerror(-7)


def test_binding_flag_constants_match_the_header():
    """The Python binding repeats the desc.flags values of the header."""
    text = open(HEADER).read()
    defines = dict(re.findall(r"#define\s+(LITE_ATTN_[A-Z_]+)\s+(\d+)", text))
    src = open(os.path.join(ROOT, "paper_2511_11062_amd", "lite_attn.py")).read()
    consts = dict(re.findall(r"^(LITE_ATTN_[A-Z_]+)\s*=\s*(\d+)", src, flags=re.M))
    assert consts and consts == {k: v for k, v in defines.items() if k in consts}
    assert set(consts) == {"LITE_ATTN_PV_SKIP_IMMEDIATE", "LITE_ATTN_ORDER_DIAGONAL_FIRST"}
