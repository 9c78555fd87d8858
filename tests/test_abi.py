"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the
header declares, sizes its workspace sensibly and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2602_10378_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "sdkde.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sdkde_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = P.load()
    names = _declared_functions()
    assert {"sdkde_score", "sdkde_debias", "sdkde_eval", "sdkde_eval_laplace", "sdkde_workspace_bytes"} <= set(names)
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in sdkde.h but not exported by libsdkde.so"


def test_binding_exposes_the_same_names():
    for name in _declared_functions():
        assert hasattr(P, name), f"binding lacks {name}"


def test_status_strings():
    assert P.sdkde_status_string(0) == "ok"
    for code in range(1, 5):
        assert P.sdkde_status_string(code) not in ("ok", "unknown status")
    assert P.sdkde_status_string(99) == "unknown status"


def test_workspace_bytes_scales_and_validates():
    small = P.sdkde_workspace_bytes(4096, 1024, 16)
    big = P.sdkde_workspace_bytes(1048576, 131072, 16)
    assert 0 < small < big < 4 << 30
    # padded operands alone: xs + xt (n_pad * dp floats each)
    assert big >= 2 * 1048576 * 16 * 4
    assert P.sdkde_workspace_bytes(1000, 0, 3) > 0
    for bad in ((0, 1, 16), (10, -1, 16), (10, 1, 0)):
        with pytest.raises(P.SdkdeError) as e:
            P.sdkde_workspace_bytes(*bad)
        assert e.value.status == 1
    with pytest.raises(P.SdkdeError) as e:
        P.sdkde_workspace_bytes(10, 1, 129)
    assert e.value.status == 2
    for bad_flags in (7, 128, 16 | 4, 32 | 5):
        with pytest.raises(P.SdkdeError) as e:
            P.sdkde_workspace_bytes(10, 1, 16, flags=bad_flags)
        assert e.value.status == 2
    assert P.sdkde_workspace_bytes(10, 1, 16, flags=P.SDKDE_FLAG_MAX_SHIFT | P.SDKDE_PREC_FP16X2) > 0
    # the symmetric score keeps one partial per group of sample blocks: more workspace where it takes effect
    sym = P.sdkde_workspace_bytes(1048576, 131072, 16, flags=P.SDKDE_FLAG_SYMMETRIC)
    assert big < sym < 6 << 30
    assert P.sdkde_workspace_bytes(1048576, 131072, 64, flags=P.SDKDE_FLAG_SYMMETRIC) == \
        P.sdkde_workspace_bytes(1048576, 131072, 64)


def test_null_and_invalid_arguments_are_rejected_without_a_device():
    lib = P.load()
    null = ctypes.c_void_p(None)
    fake = ctypes.c_void_p(4096)          # never dereferenced: every call below fails validation first
    assert lib.sdkde_score(null, 10, null, 10, 16, 1.0, fake, fake, 1 << 20, 0, null) == 1
    assert lib.sdkde_score(fake, 10, null, 7, 16, 1.0, fake, fake, 1 << 20, 0, null) == 1      # NULL points need m == n
    assert lib.sdkde_score(fake, 10, null, 10, 16, float("inf"), fake, fake, 1 << 20, 0, null) == 1
    assert lib.sdkde_score(fake, 10, null, 10, 16, 1.0, fake, null, 0, 0, null) == 3
    assert lib.sdkde_score(fake, 10, null, 10, 16, 1.0, fake, ctypes.c_void_p(4100), 1 << 30, 0, null) == 3   # misaligned
    assert lib.sdkde_score(fake, 10, null, 10, 16, 1.0, fake, fake, 16, 0, null) == 3           # too small
    assert lib.sdkde_debias(null, fake, 10, 16, 1.0, fake, null) == 1
    assert lib.sdkde_debias(fake, fake, 0, 16, 1.0, fake, null) == 0                            # n = 0: no-op
    assert lib.sdkde_eval(fake, 10, fake, 5, 16, 1.0, null, null, fake, 1 << 20, 0, null) == 1  # no output
    assert lib.sdkde_eval(fake, 10, fake, 0, 16, 1.0, null, null, fake, 1 << 20, 0, null) == 0  # m = 0: no-op
    assert lib.sdkde_eval_laplace(fake, 10, fake, 5, 300, 1.0, fake, fake, 1 << 20, 0, null) == 2
    count, total = ctypes.c_int(), ctypes.c_float()
    assert lib.sdkde_profile_summary(5, ctypes.byref(count), ctypes.byref(total)) == 1


def test_product_package_never_references_the_oracle():
    pkg = os.path.join(ROOT, "paper_2602_10378_amd")
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".h")):
                assert "oracle" not in open(os.path.join(dirpath, name)).read(), f"{name} mentions the oracle"


def test_bench_refuses_more_than_one_gpu():
    """bench.py is single-GPU by design: asking for more must end with a message, before any GPU work."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for extra_env, args in (({}, ["--gpus", "2"]), ({"WORLD_SIZE": "2"}, [])):
        env = dict(os.environ, **extra_env)
        proc = subprocess.run([sys.executable, os.path.join(root, "bench.py"), *args], env=env, capture_output=True, text=True,
                              timeout=120)
        assert proc.returncode != 0
        assert "single-GPU" in (proc.stderr + proc.stdout)


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """include/sdkde.h must compile as C (no C++ or HIP in the interface) and a C program that takes the
    address of every entry point must link against the built library (no GPU call is made)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    P.load()
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    header = open(os.path.join(root, "include", "sdkde.h")).read()
    names = sorted(set(re.findall(r"\b(sdkde_[a-z_]+)\s*\(", header)))
    lines = ['#include "sdkde.h"', "#include <stdio.h>", "typedef void (*fn_t)(void);", "int main(void)", "{",
             f"    fn_t table[{len(names)}];", "    size_t bytes = 0;", "    int rc;"]
    lines += [f"    table[{k}] = (fn_t)&{name};" for k, name in enumerate(names)]
    lines += ["    rc = sdkde_workspace_bytes(4096, 1024, 16, SDKDE_PREC_FP32, &bytes);",
              '    printf("%d %lu %s %d\\n", rc, (unsigned long)bytes, sdkde_status_string(rc), table[0] != 0);',
              "    return rc;", "}", ""]
    src = tmp_path / "use_sdkde.c"
    src.write_text("\n".join(lines))
    libdir = os.path.join(root, "paper_2602_10378_amd")
    exe = tmp_path / "use_sdkde"
    proc = subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(root, "include"), str(src),
                           "-o", str(exe), "-L", libdir, "-lsdkde", f"-Wl,-rpath,{libdir}"], capture_output=True, text=True)
    assert proc.returncode == 0, proc.stderr
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True, timeout=60).stdout.split()
    assert out[0] == "0" and int(out[1]) == P.sdkde_workspace_bytes(4096, 1024, 16) and out[2] == "ok" and out[3] == "1"
