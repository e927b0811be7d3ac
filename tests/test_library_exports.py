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
    assert C.sizeof(b._ProfileBatch) == 56


def test_create_refuses_bad_configurations_before_touching_the_gpu():
    """Argument checks of msched_create come before its first HIP call, so they can run anywhere."""
    import ctypes as C
    import numpy as np
    import paper_2512_24637_amd as pkg
    from paper_2512_24637_amd import binding as b
    lib = pkg.load_library()
    buf = np.zeros(1 << 16, np.uint8)
    ptr = buf.ctypes.data & ~0xF
    good = dict(page_shift=12, n_frames=4, n_virtual_pages=8, hbm_pool=ptr, host_store=ptr, n_host_slots=8,
                host_slot=None, stream=None)
    bad = [dict(page_shift=5), dict(page_shift=31), dict(n_frames=0), dict(n_virtual_pages=0),
           dict(n_virtual_pages=0xFFFFFFFF), dict(hbm_pool=None), dict(host_store=None),
           dict(hbm_pool=ptr + 8), dict(n_host_slots=7)]
    for change in bad:
        cfg = b._Config(**{**good, **change})
        h = C.c_void_p()
        assert lib.msched_create(C.byref(cfg), C.byref(h)) == -1, change
        assert not h.value
    slot = np.arange(8, dtype=np.uint32)
    slot[3] = 9                                             # slot beyond the backing store
    cfg = b._Config(**{**good, "host_slot": slot.ctypes.data})
    h = C.c_void_p()
    assert lib.msched_create(C.byref(cfg), C.byref(h)) == -2
    slot = np.arange(8, dtype=np.uint32)
    slot[5] = 2                                             # two pages on one backing slot
    cfg = b._Config(**{**good, "host_slot": slot.ctypes.data})
    assert lib.msched_create(C.byref(cfg), C.byref(h)) == -1 and not h.value
    assert lib.msched_create(None, C.byref(h)) == -1
    for fn in (lib.msched_destroy, lib.msched_last_hip_error):
        fn(None)
    assert lib.msched_plan(None, None, 0, None) == -1
    assert lib.msched_migrate(None, None) == -1
    assert lib.msched_pagetable_query(None, None, 0, None) == -1
    assert lib.msched_pagetable_query_static(None, None, 0, None) == -1


def test_bench_refuses_more_than_one_gpu():
    """Every box has one GPU: the benchmark says so instead of starting ranks."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], cwd=root,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stdout or "1 GPU" in r.stdout or "single" in r.stdout.lower()
