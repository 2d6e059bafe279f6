"""The CPU-side code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU involved):
the oracle's C source against all of its pins, and the host half of the C ABI (argument validation and dispatch of
api.hip, built with g++ against stand-in launchers) against the ABI tests.  Each runs in a child interpreter with the
sanitizer runtime preloaded; a report from either sanitizer makes the child fail."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]


def _runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True, check=True).stdout.strip()
    if not os.path.isabs(path):
        pytest.skip(f"{name} is not installed")
    return path


def _child_env(extra):
    env = dict(os.environ)
    preload = [_runtime("libasan.so"), _runtime("libubsan.so")]
    if env.get("LD_PRELOAD"):
        preload.append(env["LD_PRELOAD"])          # whatever is preloaded already stays, behind the sanitizer runtime
    env["LD_PRELOAD"] = ":".join(preload)
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["PYTHONPATH"] = ROOT + os.pathsep + env.get("PYTHONPATH", "")
    env.update(extra)
    return env


def _run_pytest(files, env, timeout=600):
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files]
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=timeout)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "runtime error" not in tail and "AddressSanitizer" not in tail, tail
    return tail


def test_oracle_pins_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    lib = str(tmp_path / "libogq_oracle_san.so")
    subprocess.run(["gcc", *SAN, "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                    os.path.join(ROOT, "oracle", "ogq_oracle.c"), "-o", lib, "-lm"], check=True)
    files = sorted(glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py")))
    assert len(files) >= 7
    tail = _run_pytest(files, _child_env({"OGQ_ORACLE_LIBRARY": lib, "OMP_NUM_THREADS": "4"}))
    assert " passed" in tail


def test_abi_validation_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    hip_include = "/opt/rocm/include"
    if not os.path.isdir(os.path.join(hip_include, "hip")):
        pytest.skip("HIP headers not found")
    lib = str(tmp_path / "libogq_host_san.so")
    csrc = os.path.join(ROOT, "paper_2002_11082_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", *SAN, "-D__HIP_PLATFORM_AMD__", "-I" + hip_include,
                    "-I" + os.path.join(ROOT, "include"), "-I" + csrc, "-shared", "-fPIC", "-x", "c++",
                    os.path.join(csrc, "api.hip"), os.path.join(ROOT, "tests", "host_stubs", "launch_stubs.cpp"),
                    "-o", lib], check=True)
    env = _child_env({"OGQ_LIBRARY": lib})
    tail = _run_pytest([os.path.join(ROOT, "tests", "test_abi.py")], env)
    assert " passed" in tail
    # a launch the runtime refuses comes back as OGQ_ERR_LAUNCH with the runtime's code, for every entry point
    probe = (
        "import ctypes, paper_2002_11082_amd as ogq\n"
        "A = 0x10000\n"
        "for scheme, bits, d in ((ogq.BINGRAD_B, 1, 2048), (ogq.ORQ, 2, 2048), (ogq.ORQ, 3, 4096), (ogq.ORQ_PAPER, 2, 32768),\n"
        "                        (ogq.EVEN, 2, 64), (ogq.LINEAR, 3, 512), (ogq.BINGRAD_PB, 1, 8192)):\n"
        "    p = ogq.make_params(d, bits, scheme)\n"
        "    assert ogq.ogq_quantize_raw(A, 100000, p, A, A) == -8\n"
        "    assert ogq.lib().ogq_last_hip_error() != 0\n"
        "    assert ogq.ogq_dequantize_average_raw([A, A], [A, A], 100000, p, A) == -8\n"
        "assert ogq.lib().ogq_probe_read(A, 64, A, None) == -8 and ogq.lib().ogq_probe_copy(A, A, 64, None) == -8\n"
        "print('refused launches reported')\n")
    res = subprocess.run([sys.executable, "-c", probe], cwd=ROOT, env=env, capture_output=True, text=True, timeout=120)
    assert res.returncode == 0 and "refused launches reported" in res.stdout, res.stdout + res.stderr
