"""The C ABI without Python or PyTorch in between: a small HIP host program
(tests/native/native_parity.cpp) allocates device memory itself, calls
libpipesgd.so and compares every output byte with the C oracle it links."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))


def test_native_program_matches_the_oracle(orc):
    sys.path.insert(0, os.path.join(HERE, "native"))
    try:
        import build_native
    finally:
        sys.path.pop(0)
    from paper_1811_03619_amd import binding as B
    B.lib()                                            # the library exists (built beforehand)
    exe = build_native.build(force=False)              # compiles only if no current binary is there
    print(f"running {exe}", flush=True)
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    print(res.stdout, flush=True)
    assert res.returncode == 0, res.stdout
    assert "native parity ok" in res.stdout
