"""The built C-ABI library loads and exports every function include/msched.h declares.
No compute call is made here (no GPU needed)."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "msched.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(msched_[a-z_]+)\s*\(", text)))


def test_header_declares_the_three_named_calls():
    names = _declared_functions()
    for must in ("msched_plan", "msched_migrate", "msched_pagetable_query"):
        assert must in names


def test_library_exports_every_declared_symbol():
    import paper_2512_24637_amd as pkg
    lib = pkg.load_library()
    names = _declared_functions()
    assert set(names) == set(pkg.EXPORTED_SYMBOLS)
    for n in names:
        assert getattr(lib, n) is not None
    assert lib.msched_strerror(-4).decode().startswith("first command")


def test_struct_layouts_match_the_header():
    import ctypes as C
    from paper_2512_24637_amd import binding as b
    assert C.sizeof(b._Rule) == 48
    assert C.sizeof(b._TimelineEntry) == 8
    assert C.sizeof(b._Plan) == 72
    assert C.sizeof(b._Config) == 56
