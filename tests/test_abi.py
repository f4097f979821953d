"""CPU-only checks of the boundary: the shared library loads, exports every entry point the
public header declares, and rejects bad configurations without touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "louver.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lvr_[a-z_0-9]+)\s*\(", text)))


@pytest.fixture(scope="module")
def L():
    import paper_2605_06763_amd as L
    if not os.path.exists(L.binding.LIB_PATH):
        from paper_2605_06763_amd.build import build_library
        build_library()
    return L


def test_header_and_library_agree(L):
    names = _declared()
    assert len(names) >= 12
    lib = L.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/louver.h but not exported"
    assert sorted(L.EXPORTS) == names
    for n in names:
        if n not in ("lvr_strerror", "lvr_last_hip_error", "lvr_arena_bytes"):
            assert callable(getattr(L, n)), f"binding lacks {n}"


def test_config_struct_matches_header(L):
    """Field order of the ctypes mirror equals the header's struct (argument marshalling only
    works if both sides agree on the layout)."""
    text = open(os.path.join(ROOT, "include", "louver.h")).read()
    body = re.search(r"typedef struct lvr_config \{(.*?)\} lvr_config;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b(?:int32_t|uint32_t|int64_t|uint64_t|float)\s+([a-z_]+)\s*;", body)
    assert fields == [f for f, _ in L.lvr_config._fields_]
    body = re.search(r"typedef struct lvr_stats \{(.*?)\} lvr_stats;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b(?:int32_t|uint32_t|int64_t|uint64_t|float)\s+([a-z_]+)\s*;", body)
    assert fields == [f for f, _ in L.lvr_stats._fields_]


def test_bad_configs_are_rejected_on_the_host(L):
    ok = dict(batch=1, n_q_heads=32, n_kv_heads=8, capacity=1024)
    assert L.lvr_arena_bytes(L.make_config(**ok)) > 2 * 8 * 1024 * 128 * 2
    for bad in (dict(ok, head_dim=64), dict(ok, n_q_heads=30), dict(ok, group_size=3), dict(ok, n_subspaces=32),
                dict(ok, buffer_size=100), dict(ok, capacity=0), dict(ok, n_q_heads=24, n_kv_heads=8),
                dict(ok, kv_dtype=7), dict(ok, reservoir_size=257), dict(ok, reservoir_size=-1), dict(ok, flags=16),
                dict(ok, flags=1 << 31), dict(ok, index_dtype=4)):
        cfg = L.make_config(**bad)
        assert L.lvr_arena_bytes(cfg) == 0
        h = C.c_void_p()
        assert L.lib().lvr_create(C.byref(cfg), C.byref(h)) < 0 and not h.value
    assert L.lib().lvr_strerror(L.LVR_E_OVERFLOW).decode().startswith("a retrieved set")
    assert L.lib().lvr_strerror(-99).decode() == "unknown error"
    # NULL handles are refused, not dereferenced
    assert L.lib().lvr_query(None, None, None, None, None, 0, None) == L.LVR_E_INVALID
    assert L.lib().lvr_destroy(None) == L.LVR_E_INVALID


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2605_06763_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower().replace("threshold oracle", ""), f


def test_header_is_plain_c(tmp_path):
    """include/louver.h is the C ABI: it must compile as C99 (and as C++) on its own, with no
    HIP or torch types in any signature."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "louver.h"\nint main(void) { lvr_config c; lvr_stats s; (void)c; (void)s; '
                   'return lvr_strerror(0) == 0; }\n')
    inc = os.path.join(ROOT, "include")
    for cmd in (["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror"], ["g++", "-std=c++17", "-x", "c++", "-Wall", "-Werror"]):
        r = subprocess.run(cmd + ["-I", inc, "-c", str(src), "-o", str(tmp_path / "o.o")], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, "louver.h")).read(), flags=re.S)   # declarations only
    assert "hipStream_t" not in text and "torch" not in text and "at::" not in text and "#include <hip" not in text


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; any other --gpus value ends with a message and a non-zero status
    before anything touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
