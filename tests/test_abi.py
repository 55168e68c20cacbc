"""CPU-side checks of the boundary: the shared library loads, exports every entry point that
include/pag.h declares, its structs have the layout the Python binding assumes, and argument errors
are reported without touching a GPU."""
import ctypes as C
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pag.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2603_06660_amd import binding, build
    if not os.path.exists(binding.library_path()):
        build.build()
    return binding.load_library()


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pag_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_entry_point_is_exported(lib):
    from paper_2603_06660_amd import EXPORTED_SYMBOLS
    names = _declared()
    assert "pag_build" in names and "pag_search" in names and "pag_insert" in names
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(EXPORTED_SYMBOLS) == names


def test_struct_layouts_match_the_header(tmp_path):
    from paper_2603_06660_amd import binding
    src = tmp_path / "sizes.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "pag.h"\nint main(void){printf("%zu %zu %zu %zu %zu %zu %zu\\n",'
                   'sizeof(pag_params),sizeof(pag_arrays),sizeof(pag_counters),offsetof(pag_params,stream),'
                   'offsetof(pag_arrays,entry),offsetof(pag_counters,last_build_ms),offsetof(pag_counters,relinked_batches));return 0;}\n')
    exe = tmp_path / "sizes"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    got = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    want = [C.sizeof(binding._Params), C.sizeof(binding._Arrays), C.sizeof(binding._Counters),
            binding._Params.stream.offset, binding._Arrays.entry.offset, binding._Counters.last_build_ms.offset,
            binding._Counters.relinked_batches.offset]
    assert got == want


def test_constants_match_the_header():
    """Flags, metrics and error codes of the binding are the header's."""
    from paper_2603_06660_amd import binding
    text = open(HEADER).read()
    flags = {k: int(v) for k, v in re.findall(r"#define\s+PAG_(FLAG_[A-Z0-9_]+)\s+(\d+)u", text)}
    assert len(flags) >= 6
    for name, value in flags.items():
        assert getattr(binding, name) == value, name
    assert sorted(flags.values()) == [1 << i for i in range(len(flags))]     # distinct single bits, none skipped


def test_argument_errors_need_no_gpu(lib):
    """Null handles and null pointers are rejected before any HIP call."""
    lib.pag_last_error.restype = C.c_char_p
    assert lib.pag_search(None, None, C.c_uint64(1), C.c_uint32(1), C.c_uint32(1), None, None) == -1
    assert b"null" in lib.pag_last_error()
    assert lib.pag_insert(None, None, C.c_uint64(1)) == -1
    assert lib.pag_set_search_options(None, C.c_uint32(0), C.c_uint32(0)) == -1
    assert lib.pag_build(None, C.c_uint64(0), C.c_uint32(8), None, None) == -1
    h = C.c_void_p()
    assert lib.pag_build(None, C.c_uint64(0), C.c_uint32(8), None, C.byref(h)) == -1      # params null
    assert lib.pag_free(None) == 0
    s = C.c_void_p()
    assert lib.pag_searcher_create(None, None, C.byref(s)) == -1 and not s.value
    assert lib.pag_searcher_search(None, None, C.c_uint64(1), C.c_uint32(1), C.c_uint32(1), None, None) == -1
    assert lib.pag_searcher_free(None) == 0
    assert lib.pag_search_static(None, None, C.c_uint64(1), C.c_uint32(1), C.c_uint32(1), None, None) == -1
    assert b"null" in lib.pag_last_error()
    assert lib.pag_insertion_candidates(None, None, C.c_uint64(1), None, None, None, None, None, None) == -1


def test_missing_library_is_an_error(monkeypatch):
    """There is no CPU fallback: without the built library the binding refuses to work."""
    from paper_2603_06660_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libpag_hip.so")
    with pytest.raises(binding.PagError):
        binding.load_library()


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_product_never_imports_the_oracle():
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_2603_06660_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f), errors="ignore").read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2603_06660_amd" not in text and "libpag_hip" not in text
