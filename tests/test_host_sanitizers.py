"""Host code under sanitizers (CPU only): the C-ABI layer's argument validation, plan selection
and launch wrappers built with AddressSanitizer + UndefinedBehaviorSanitizer on the host side
(device code as usual) and driven through the whole host test file; the C oracle built with
gcc's sanitizers and driven through a slice of its pins.  Each runs in a child process whose
LD_PRELOAD puts the sanitizer runtime first (whatever was preloaded before stays after it)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(preload, code, timeout=600):
    env = dict(os.environ)
    env["LD_PRELOAD"] = preload + ((":" + env["LD_PRELOAD"]) if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:halt_on_error=1:alloc_dealloc_mismatch=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    return subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True,
                          timeout=timeout)


def test_api_layer_host_code_under_asan_and_ubsan():
    from paper_2307_14995_amd import build
    rt = build.sanitizer_runtime()
    if not rt or not os.path.exists(rt):
        pytest.skip("the compiler ships no shared AddressSanitizer runtime")
    lib = build.build_sanitized()
    code = (
        "import sys\n"
        "import paper_2307_14995_amd.binding as b\n"
        f"b._LIB_PATH = {lib!r}\n"
        "import pytest\n"
        "sys.exit(pytest.main(['-x', '-q', 'tests/test_abi_host.py', '-p', 'no:cacheprovider',\n"
        "                      '-k', 'not bench_refuses and not does_not_import']))\n"
    )
    r = _run(rt, code)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "passed" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_oracle_under_asan_and_ubsan(tmp_path):
    src = os.path.join(ROOT, "oracle", "ltn_oracle.c")
    lib = str(tmp_path / "libltn_oracle_san.so")
    rt = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(rt):
        pytest.skip("gcc ships no shared AddressSanitizer runtime")
    subprocess.run(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-fno-fast-math",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                    "-o", lib, src, "-lm"], check=True)
    code = (
        "import sys\n"
        "import oracle.ltn_oracle as o\n"
        f"o._LIB = {lib!r}\n"
        "o.build = lambda force=False: o._LIB\n"
        "import pytest\n"
        "sys.exit(pytest.main(['-x', '-q', 'tests/test_oracle_pins.py', 'tests/test_oracle_pins_prologue.py',\n"
        "                      '-p', 'no:cacheprovider']))\n"
    )
    r = _run(os.path.realpath(rt), code)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "passed" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
