"""The CPU builds stay clean under AddressSanitizer and UndefinedBehaviorSanitizer.

* the C oracle is rebuilt with ``-fsanitize=address,undefined`` and its pin
  files are run against that build (through ``PIPESGD_ORACLE_LIB``);
* the host-only part of the library (size rules, bucket planner, segment
  tables, timing models: ``csrc/pipesgd_host.cpp``, which has no device code)
  is built the same way and driven through its edge cases.

The sanitizer runtimes are loaded in front of the (uninstrumented) interpreter
in a child process.  To show that they are really watching, the same harness is
first pointed at a copy of the oracle with a planted one-element heap overrun
and must report it.
"""
import os
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_SRC = os.path.join(ROOT, "oracle", "pipesgd_oracle.c")
HOST_SRC = os.path.join(ROOT, "paper_1811_03619_amd", "csrc", "pipesgd_host.cpp")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
PIN_FILES = ["test_oracle_codec.py", "test_oracle_ring.py", "test_oracle_update.py", "test_oracle_bucket.py",
             "test_oracle_direct.py", "test_oracle_hd.py", "test_golden.py"]


def runtime(name, compiler="gcc"):
    path = subprocess.check_output([compiler, f"-print-file-name={name}"], text=True).strip()
    if not os.path.isabs(path):
        pytest.skip(f"{name} is not installed")
    return path


def sanitized_env(**extra):
    env = dict(os.environ)
    pre = [runtime("libasan.so"), runtime("libubsan.so")]
    if env.get("LD_PRELOAD"):
        pre.append(env["LD_PRELOAD"])                 # whatever is preloaded already stays, behind the runtimes
    env["LD_PRELOAD"] = ":".join(pre)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=87"    # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "halt_on_error=1:exitcode=88:print_stacktrace=1"
    env.update(extra)
    return env


def build_oracle(src, out):
    subprocess.check_call(["gcc", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math", "-mfma",
                           *SAN, src, "-o", out, "-lm"])


def run_pins(lib, files, tmp_path):
    # -s: the child's pytest must not take over file descriptor 2, where the sanitizers report
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-s", "-p", "no:cacheprovider", *[os.path.join(ROOT, "tests", f) for f in files]]
    return subprocess.run(cmd, cwd=ROOT, env=sanitized_env(PIPESGD_ORACLE_LIB=lib), stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True, timeout=900)


def test_the_harness_notices_a_planted_overrun(tmp_path):
    text = open(ORACLE_SRC).read()
    good = "R->tmp = (float *)malloc((R->ce + 1) * sizeof(float));"
    assert text.count(good) == 1
    bad = tmp_path / "overrun.c"
    # the scratch vector of the ring is one element short of a block, and the block is written in full
    bad.write_text(text.replace(good, "R->tmp = (float *)malloc((R->ce - 1) * sizeof(float));"))
    lib = str(tmp_path / "liboverrun.so")
    build_oracle(str(bad), lib)
    res = run_pins(lib, ["test_oracle_ring.py"], tmp_path)
    assert res.returncode != 0 and "AddressSanitizer" in res.stdout, res.stdout[-2000:]


def test_oracle_pins_pass_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "liboracle_san.so")
    build_oracle(ORACLE_SRC, lib)
    res = run_pins(lib, PIN_FILES, tmp_path)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "passed" in res.stdout and "Sanitizer" not in res.stdout and "runtime error" not in res.stdout, res.stdout[-4000:]


HOST_DRIVER = textwrap.dedent(r'''
    import ctypes as C, sys
    L = C.CDLL(sys.argv[1])
    u64, i32, dbl = C.c_uint64, C.c_int, C.c_double

    class Bucket(C.Structure):
        _fields_ = [("start", u64), ("n", u64)]

    class Segment(C.Structure):
        _fields_ = [("tensor", C.c_void_p), ("packed", C.c_void_p), ("numel", u64), ("first_tile", u64)]

    L.pipesgd_chunk_elems.restype = u64; L.pipesgd_chunk_elems.argtypes = [u64, i32]
    L.pipesgd_payload_bytes.restype = u64; L.pipesgd_payload_bytes.argtypes = [i32, u64]
    L.pipesgd_num_scales.restype = u64; L.pipesgd_num_scales.argtypes = [i32, u64]
    L.pipesgd_placement_offset.restype = u64; L.pipesgd_placement_offset.argtypes = [i32, i32, i32]
    L.pipesgd_workspace_bytes.argtypes = [i32, i32, u64, i32, C.POINTER(u64)]
    L.pipesgd_bucket_plan.argtypes = [C.POINTER(u64), u64, u64, C.POINTER(Bucket), u64, C.POINTER(u64), C.POINTER(u64)]
    L.pipesgd_segments_prepare.argtypes = [C.POINTER(Segment), u64, C.POINTER(u64)]
    L.pipesgd_strerror.restype = C.c_char_p
    L.pipesgd_model_ring_comm_time.restype = dbl
    L.pipesgd_model_ring_comm_time.argtypes = [i32, dbl, dbl, dbl, dbl, dbl, i32]
    for name, k in (("pipesgd_model_sync_time", 4), ("pipesgd_model_pipe_ideal_time", 5), ("pipesgd_model_pipe_time", 4),
                    ("pipesgd_model_scaling_efficiency", 3)):
        getattr(L, name).restype = dbl; getattr(L, name).argtypes = [dbl] * k

    big = 2 ** 64 - 1
    for n in (0, 1, 4095, 4096, 4097, 60965224, 2 ** 40, big // 8):
        for p in (-1, 0, 1, 3, 4, 16, 2 ** 31 - 1):
            L.pipesgd_chunk_elems(n, p)
        for mode in (-1, 0, 1, 2, 3):
            L.pipesgd_payload_bytes(mode, n); L.pipesgd_num_scales(mode, n)
            out = (u64 * 3)()
            for sched in (-1, 0, 1, 2, 3, 4):
                for p in (0, 1, 2, 4):
                    L.pipesgd_workspace_bytes(sched, mode, n, p, out)
    for kind in range(-2, 13):
        for p in range(0, 18):
            for r in range(-1, p + 1):
                assert L.pipesgd_placement_offset(kind, r, p) < 4096
    for err in range(-9, 3):
        assert L.pipesgd_strerror(err)
    # planner: exactly-sized output tables, so a write past either end is an overrun the sanitizer sees
    cases = [[], [1], [4096] * 7, [10, 20, 5000, 3, 2000000, 7, 1 << 20, 1], [1 << 20] * 70, [3] * 5000]
    for numels in cases:
        for cap in (1, 4096, 1 << 20, 1 << 40):
            for max_b in (0, 1, 2, 64, 5000):
                nt = len(numels)
                arr = (u64 * nt)(*numels)
                out_b = (Bucket * max_b)()
                out_o = (u64 * nt)()
                npk = u64()
                rc = L.pipesgd_bucket_plan(arr, nt, cap, out_b, max_b, out_o, C.byref(npk))
                assert rc == -4 or 1 <= rc <= max_b, (rc, max_b)
    assert L.pipesgd_bucket_plan(None, 0, 10, (Bucket * 1)(), 1, (u64 * 1)(), C.byref(u64())) == 1
    for num in (0, 1, 7, 300):
        tab = (Segment * num)()
        for i in range(num):
            tab[i].tensor, tab[i].packed, tab[i].numel = 0x1000 + 4 * i, 0x100000 + 4 * i, (i * 977) % 9000
        total = u64()
        assert L.pipesgd_segments_prepare(tab, num, C.byref(total)) == 0
    for p in (-3, 0, 1, 4, 1000):
        for seg in (-1, 0, 1, 9):
            L.pipesgd_model_ring_comm_time(p, 1e9, 1e-6, 1e-9, 1e-10, 1e-5, seg)
    L.pipesgd_model_sync_time(1e3, 1.0, 2.0, 3.0); L.pipesgd_model_pipe_ideal_time(1e3, 0.0, 1.0, 2.0, 3.0)
    L.pipesgd_model_pipe_time(1e3, 1.0, 2.0, 3.0); L.pipesgd_model_scaling_efficiency(0.0, 0.0, 0.0)
    print("host driver ok")
''')


def test_host_only_library_code_is_clean_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "libpipesgd_host_san.so")
    subprocess.check_call(["g++", "-std=c++17", "-fPIC", "-shared", *SAN, "-I", os.path.join(ROOT, "include"),
                           HOST_SRC, "-o", lib])
    driver = tmp_path / "drive_host.py"
    driver.write_text(HOST_DRIVER)
    env = sanitized_env()
    env["LD_PRELOAD"] = ":".join([runtime("libasan.so"), runtime("libubsan.so"), runtime("libstdc++.so", "g++")] +
                                 ([os.environ["LD_PRELOAD"]] if os.environ.get("LD_PRELOAD") else []))
    res = subprocess.run([sys.executable, str(driver), lib], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                         text=True, timeout=600)
    assert res.returncode == 0 and "host driver ok" in res.stdout, res.stdout[-4000:]
    assert "Sanitizer" not in res.stdout and "runtime error" not in res.stdout, res.stdout[-4000:]
