"""The C ABI's host side (argument checks, workspace plan, launch dispatch) built with
AddressSanitizer and UndefinedBehaviorSanitizer and exercised without a GPU.  Only the two
translation units that hold host logic are instrumented; the kernels' objects are linked as built."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.timeout(1500)
def test_argument_layer_under_address_and_ub_sanitizers(tmp_path):
    from paper_1805_10032_amd import build
    build.build(verbose=False, force=False)          # objects of the kernel translation units (reused when fresh)
    hipcc = build._hipcc()
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    objs = []
    for src in ("zeno_capi.hip", "zeno_layer.hip"):
        obj = str(tmp_path / src.replace(".hip", ".o"))
        subprocess.run([hipcc, *build.HIPCC_FLAGS, *san, "-c", os.path.join(build.CSRC, src), "-o", obj],
                       check=True, capture_output=True, text=True)
        objs.append(obj)
    for src, suffix, _flags in build.SOURCES:
        if src not in ("zeno_capi.hip", "zeno_layer.hip"):
            objs.append(os.path.join(build.OBJ_DIR, src.replace(".hip", suffix + ".o")))
    main_obj = str(tmp_path / "host_checks.o")
    subprocess.run([hipcc, "-x", "c++", "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                    "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"),
                    "-c", os.path.join(ROOT, "tests", "sanitize", "host_checks.cpp"), "-o", main_obj],
                   check=True, capture_output=True, text=True)
    exe = str(tmp_path / "host_checks")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                    "-o", exe, main_obj, *objs], check=True, capture_output=True, text=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "host checks passed" in res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr
