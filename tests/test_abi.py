"""The C-ABI library loads without a GPU and exports every symbol the public header declares."""
import ctypes
import os
import re

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2502_01941_amd import build, shotkv
    if not os.path.exists(shotkv.LIB_PATH):
        build.build(force=True)
    return shotkv.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "shotkv.h")).read()
    return re.findall(r"SHOTKV_API\s+[\w\s\*]+?\b(shotkv_\w+)\s*\(", text)


def test_header_symbols_are_exported(lib):
    from paper_2502_01941_amd import shotkv
    names = _declared_symbols()
    assert len(names) >= 8 and set(names) == set(shotkv.EXPORTS)
    for name in names:
        assert hasattr(lib, name), name


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 (and as C++) on its own, with no other include."""
    import shutil
    import subprocess
    header = os.path.join(ROOT, "include", "shotkv.h")
    for cc, std, lang in (("gcc", "-std=c99", "c"), ("g++", "-std=c++17", "c++")):
        if shutil.which(cc) is None:
            pytest.skip(f"{cc} not installed")
        r = subprocess.run([cc, std, "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", lang, header],
                           capture_output=True, text=True, timeout=120)
        assert r.returncode == 0, r.stderr
    # a C translation unit that takes the address of every declared function links against the library's names
    src = tmp_path / "use.c"
    names = _declared_symbols()
    src.write_text('#include "shotkv.h"\n' + "void* table[] = {" + ", ".join(f"(void*){n}" for n in names) + "};\n")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-Wno-pedantic", "-I", os.path.join(ROOT, "include"),
                        "-c", str(src), "-o", str(tmp_path / "use.o")], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr


def test_host_only_entry_points(lib):
    from paper_2502_01941_amd import shotkv
    assert lib.shotkv_abi_version() == 3
    assert lib.shotkv_strerror(0) == b"ok"
    assert b"workspace" in lib.shotkv_strerror(-3)
    n = shotkv.prefill_workspace_bytes(32, 8, 128, 32, torch.bfloat16, 4, 32768, 160)
    assert 0 < n < (1 << 30)
    assert shotkv.prefill_workspace_bytes(32, 8, 128, 32, torch.bfloat16, 8, 32768, 160) > n
    cfg = shotkv._config(32, 8, 96, 32, torch.bfloat16, 0.1, 0)          # head_dim 96 is unsupported
    assert lib.shotkv_prefill_workspace_bytes(ctypes.byref(cfg), 1, 1000, 4) == 0
    cfg = shotkv._config(32, 8, 128, 32, torch.bfloat16, 0.1, 0)
    assert lib.shotkv_prefill_workspace_bytes(ctypes.byref(cfg), 1, 1000, 5000) == 0   # too many shots
    assert lib.shotkv_decode_workspace_bytes(ctypes.byref(cfg), 16, 4096, 1025) > 0


def test_null_arguments_are_rejected_before_any_launch(lib):
    from paper_2502_01941_amd import shotkv
    cfg = shotkv._config(32, 8, 128, 32, torch.bfloat16, 0.1, 0)
    rc = lib.shotkv_prefill_scores(ctypes.byref(cfg), 1, 1000, 4, None, None, None, None, None, None, 0, None)
    assert rc == -1
    rc = lib.shotkv_decode_step(ctypes.byref(cfg), 1, None, 0, None, None, None, None, None, None, None,
                                None, 0, None)
    assert rc == -1


def test_missing_library_fails_loudly_and_package_never_imports_the_oracle():
    """There is no CPU fallback: without the built library the binding raises, in a fresh interpreter; and
    nothing in the product package refers to the oracle."""
    import subprocess
    import sys
    code = ("import sys; sys.path.insert(0, %r)\n"
            "from paper_2502_01941_amd import shotkv\n"
            "try:\n    shotkv.load_library()\nexcept shotkv.ShotKVError as e:\n    print('RAISED', e)\n"
            "assert 'oracle' not in sys.modules and 'oracle.shotkv_oracle' not in sys.modules\n") % ROOT
    env = dict(os.environ, SHOTKV_LIBRARY="/nonexistent/libshotkv.so")
    out = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr
    assert "RAISED" in out.stdout and "not found" in out.stdout
    pkg = os.path.join(ROOT, "paper_2502_01941_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "oracle/" not in text, f
