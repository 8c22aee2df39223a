"""The C-ABI library loads and exports every function the headers under include/ declare.  CPU only:
nothing here calls into the GPU."""

import ctypes
import glob
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
LIB = os.path.join(ROOT, "paper_2508_18736_amd", "libsiso.so")


def declared_functions(headers=None):
    text = "\n".join(open(h).read() for h in (headers or HEADERS))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(siso_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_four_named_calls():
    names = declared_functions([os.path.join(ROOT, "include", "siso.h")])
    for must in ("siso_create", "siso_lookup", "siso_update", "siso_merge"):
        assert must in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        from paper_2508_18736_amd import build
        build.build(verbose=False)
    lib = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in siso.h but not exported"


def test_binding_covers_every_declared_symbol():
    if not os.path.exists(LIB):
        from paper_2508_18736_amd import build
        build.build(verbose=False)
    from paper_2508_18736_amd import siso
    assert sorted(siso.SYMBOLS) == declared_functions()


def test_argument_errors_without_touching_the_gpu():
    """NULL handles and NULL out-pointers are rejected before any HIP call."""
    if not os.path.exists(LIB):
        from paper_2508_18736_amd import build
        build.build(verbose=False)
    from paper_2508_18736_amd import siso
    lib = siso._lib
    assert lib.siso_create(768, 10, None) == siso.EINVAL
    h = ctypes.c_void_p()
    assert lib.siso_create(0, 10, ctypes.byref(h)) == siso.EINVAL
    assert lib.siso_create(5000, 10, ctypes.byref(h)) == siso.EINVAL
    assert lib.siso_create(768, 0, ctypes.byref(h)) == siso.EINVAL
    assert lib.siso_create_ex(768, 10, 7, ctypes.byref(h)) == siso.EINVAL
    assert lib.siso_lookup(None, None, 0, 0.5, None, None, None) == siso.EINVAL
    assert lib.siso_update(None, None, None, 0) == siso.EINVAL
    assert lib.siso_merge(None, 0.5, None, 0) == siso.EINVAL
    assert lib.siso_count(None) == siso.EINVAL
    lib.siso_destroy(None)
