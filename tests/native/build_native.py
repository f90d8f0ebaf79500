"""Builds tests/native/native_parity (hipcc; links libpipesgd.so and the C oracle)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
BIN = os.path.join(HERE, "native_parity")


def build(force: bool = True) -> str:
    src = os.path.join(HERE, "native_parity.cpp")
    lib_dir, orc_dir = os.path.join(ROOT, "paper_1811_03619_amd"), os.path.join(ROOT, "oracle")
    deps = [src, os.path.join(lib_dir, "libpipesgd.so"), os.path.join(orc_dir, "libpipesgd_oracle.so")]
    if not force and os.path.exists(BIN) and all(os.path.getmtime(d) <= os.path.getmtime(BIN) for d in deps):
        return BIN
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O1", "-std=c++17", "-x", "c++", src, "-I", os.path.join(ROOT, "include"),
           "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include",
           "-L", lib_dir, "-lpipesgd", "-L", orc_dir, "-lpipesgd_oracle", "-L", "/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_1811_03619_amd:$ORIGIN/../../oracle:/opt/rocm/lib", "-o", BIN]
    subprocess.check_call(cmd)
    return BIN


if __name__ == "__main__":
    print(build())
