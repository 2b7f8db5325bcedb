"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer: the C oracle, the C ABI's argument
handling and the model / selector are compiled with gcc's sanitizers (the device side replaced by
tests/native/stub_device.cpp, whose launches fail with hipErrorNoDevice) into one host program,
tests/native/sanitize_host.cpp, which must run clean.  Also: on a machine without a visible GPU the real
library reports ATB_ERR_HIP from its launch calls instead of crashing."""
import os
import shutil
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NATIVE = os.path.join(ROOT, "tests", "native")
CSRC = os.path.join(ROOT, "paper_2511_16041_amd", "csrc")
ROCM_INC = "/opt/rocm/include"


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir(ROCM_INC), reason="needs g++ and the HIP headers")
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_host")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan",
           "-fno-omit-frame-pointer", "-g", "-O1"]
    obj_c = str(tmp_path / "oracle.o")
    subprocess.run(["gcc", "-std=c99", "-fopenmp", "-ffp-contract=off", "-c", os.path.join(ROOT, "oracle", "atb_oracle.c"),
                    "-o", obj_c] + san, check=True)
    cmd = ["g++", "-std=c++17", "-fopenmp", "-D__HIP_PLATFORM_AMD__", "-I", ROCM_INC, "-I", os.path.join(ROOT, "include"),
           "-I", CSRC, "-Wno-deprecated-declarations",
           os.path.join(NATIVE, "sanitize_host.cpp"), os.path.join(NATIVE, "stub_device.cpp"),
           os.path.join(CSRC, "atb_api.cpp"), os.path.join(CSRC, "atb_model.cpp"), obj_c, "-o", exe, "-lm"] + san
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2", ATB_LOG="1")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=120)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out
    assert "sanitize_host: ok" in r.stdout
    assert "AddressSanitizer" not in out and "runtime error" not in out, out
    assert "atb_gemm_create: M=3000 N=5000 K=4104" in r.stderr          # the ATB_LOG=1 plan dump


def test_launch_without_a_device_returns_hip_error():
    """A child process that sees no GPU (none exists, or all are hidden) builds a plan and launches it:
    every launching entry point must come back with ATB_ERR_HIP and leave the process alive."""
    code = textwrap.dedent("""
        import ctypes, sys
        sys.path.insert(0, %r)
        import paper_2511_16041_amd as atb
        L = atb.lib()
        buf = ctypes.create_string_buffer(1 << 16)
        base = (ctypes.addressof(buf) + 255) & ~255
        vp = ctypes.c_void_p
        for tiles in ((256, 256, 64, 256), (32, 64, 64, 64)):          # a persistent-grid instance and a plain one
            h = vp()
            assert L.atb_gemm_create(ctypes.byref(h), 256, 256, 256, *tiles) == 0
            st = L.atb_gemm_run(h, vp(base), vp(base), vp(base), None)
            assert st == 5, st
            assert L.atb_last_hip_error() != 0
            L.atb_gemm_destroy(h)
        assert L.atb_bfp16_quantize(vp(base), 8, vp(base), 1, 8, None) == 5
        assert L.atb_mfma_probe(vp(base), None, 1, 1, 1, 16, None, None) == 5
        print("no-device ok")
    """ % ROOT)
    env = dict(os.environ, HIP_VISIBLE_DEVICES="", ROCR_VISIBLE_DEVICES="", CUDA_VISIBLE_DEVICES="")
    r = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "no-device ok" in r.stdout, r.stdout + r.stderr
