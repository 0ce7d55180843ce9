"""The C-ABI library loads and exports every symbol the header declares; host
paths that need no device behave as documented (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mi_shmem.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(shmem_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2511_15076_amd as sh
    names = declared_symbols()
    assert len(names) >= 28
    lib = ctypes.CDLL(sh.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(sh.EXPORTS)          # the binding covers the header, name for name


def test_uninitialised_calls_fail_cleanly():
    import paper_2511_15076_amd as sh
    assert sh.n_pes() == 0
    assert sh.malloc(64) is None and sh.ptr(4096, 0) is None
    assert sh.scratch_bytes(0) == 0 and sh.scratch_bytes(8) % 256 == 0
    assert sh.scratch_bytes(64) > sh.scratch_bytes(8)
    for call in (lambda: sh.put(0, 0, 0, 8, 0), lambda: sh.quiet(), lambda: sh.barrier_all(),
                 lambda: sh.finalize(), lambda: sh.op_batch(0, 1, 1, 1), lambda: sh.free(256),
                 lambda: sh.amo_batch(0, 0, 1, 0, 0, 0, 0, 0, 1, 1), lambda: sh.stream_sync()):
        with pytest.raises(sh.ShmemError) as e:
            call()
        assert e.value.status == sh.ERR_NOT_INIT
    assert "not initialised" in sh.strerror(sh.ERR_NOT_INIT)
    assert sh.strerror(12345) == "unknown status"


def test_init_argument_checks_need_no_device():
    import paper_2511_15076_amd as sh
    for args, status in [((0, 4096, 256, 256), sh.ERR_INVALID_ARG), ((2, 0, 256, 256), sh.ERR_INVALID_ARG),
                         ((2, 4096, 0, 256), sh.ERR_INVALID_ARG), ((2, 4097, 256, 256), sh.ERR_ALIGN),
                         ((2, 4096, 264, 256), sh.ERR_ALIGN), ((2, 4096, 256, 8), sh.ERR_ALIGN)]:
        with pytest.raises(sh.ShmemError) as e:
            sh.init(*args)
        assert e.value.status == status, args
    assert sh.n_pes() == 0


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2511_15076_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower().replace("no cpu fallback", ""), f


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_refers_only_to_functions_it_defines():
    # every function bench.py calls by bare name exists (a lost helper must not wait for a GPU run)
    import ast
    import builtins
    import os
    src = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "bench.py")).read()
    tree = ast.parse(src)
    defined = {n.name for n in ast.walk(tree) if isinstance(n, ast.FunctionDef)}
    called = {n.func.id for n in ast.walk(tree) if isinstance(n, ast.Call) and isinstance(n.func, ast.Name)}
    local = {n.id for n in ast.walk(tree) if isinstance(n, ast.Name) and isinstance(n.ctx, ast.Store)}
    missing = {c for c in called if c not in defined and c not in local and not hasattr(builtins, c)}
    assert not missing, missing


def test_binding_loads_torch_before_the_library():
    # torch ships its own HIP runtime; the library must bind to that copy whatever the caller imports first
    import subprocess
    import sys
    code = ("import sys; sys.path.insert(0, %r)\n"
            "assert 'torch' not in sys.modules\n"
            "import paper_2511_15076_amd\n"
            "assert 'torch' in sys.modules\n"
            "maps = open('/proc/self/maps').read()\n"
            "paths = {l.split()[-1] for l in maps.splitlines() if 'libamdhip64' in l}\n"
            "assert len(paths) == 1, paths\n") % (ROOT,)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]


def test_public_header_is_plain_c_and_cpp(tmp_path):
    # the boundary is a C ABI: the header must compile as C11 and as C++17, warnings being errors
    import subprocess
    (tmp_path / "c.c").write_text('#include "mi_shmem.h"\nint main(void) { return sizeof(shmem_bfs_stats) == 0; }\n')
    (tmp_path / "cpp.cpp").write_text('#include "mi_shmem.h"\nint main() { shmem_pe_team t = {0, 1, 1, 0, 0}; return (int)t.start; }\n')
    inc = os.path.join(ROOT, "include")
    for cmd in (["gcc", "-std=c11", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc, str(tmp_path / "c.c")],
                ["g++", "-std=c++17", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc, str(tmp_path / "cpp.cpp")]):
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]


def test_public_headers_stand_alone():
    """include/ is what a user of the library installs: no header there may reach outside it, and the device API
    header must hold real code (the library's own kernels are built on the same files)."""
    import re
    inc = os.path.join(ROOT, "include")
    for name in sorted(os.listdir(inc)):
        text = open(os.path.join(inc, name)).read()
        for target in re.findall(r'#include\s+"([^"]+)"', text):
            assert "/" not in target and os.path.exists(os.path.join(inc, target)), f"{name} includes {target}"
    dev = open(os.path.join(inc, "mi_shmemx.hpp")).read()
    assert "__device__" in dev and "barrier_all" in dev and "copy(" in dev
    # and the library's sources take those primitives from include/, not from a private copy
    csrc = os.path.join(ROOT, "paper_2511_15076_amd", "csrc")
    assert not os.path.exists(os.path.join(csrc, "shmemx.hpp")) and not os.path.exists(os.path.join(csrc, "gin.hpp"))
