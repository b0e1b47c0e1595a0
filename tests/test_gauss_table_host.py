"""Host-only check of the compile-time normal-distribution table the bf16 row kernels read GELU and GELU' from
(csrc/common.hip.h): the constexpr evaluation is compiled with the host compiler, every entry is printed, and each
must be the fp32 rounding of the oracle's double-precision value (Phi(z) - 1/2 and z phi(z) at each of the 2304 bf16
magnitudes in [2^-14, 16)), up to one unit in the last place where the double value sits on a rounding boundary."""
import os
import re
import subprocess

import numpy as np
import pytest

from oracle import fdl_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "paper_2509_14279_amd", "csrc", "common.hip.h")


def test_compile_time_table_matches_the_oracle(tmp_path):
    text = open(HEADER).read()
    a = text.index("namespace ctmath {")
    b = text.index("__device__ const GaussTableData g_gauss_table")
    prog = ("#include <cstdint>\n#include <cstdio>\n" + text[a:b] +
            "int main() { static constexpr GaussTableData t = make_gauss_table();\n"
            "  for (int i = 0; i < kGaussEntries; i++) std::printf(\"%a %a %a\\n\", (double)t.h[i], (double)t.pair[2 * i], (double)t.pair[2 * i + 1]);\n"
            "  return 0; }\n")
    src = tmp_path / "table.cpp"
    src.write_text(prog)
    exe = tmp_path / "table"
    r = subprocess.run(["g++", "-std=c++17", "-O0", "-fconstexpr-ops-limit=2000000000", "-fconstexpr-loop-limit=10000000",
                        str(src), "-o", str(exe)], capture_output=True, text=True)
    if r.returncode != 0:
        pytest.fail("host compile of the table failed:\n" + r.stderr[-2000:])
    out = subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split()
    vals = np.array([float.fromhex(v) for v in out]).reshape(-1, 3)
    assert vals.shape[0] == 0x417f - 0x3880 + 1 == 2304
    bits = (np.arange(0x3880, 0x417f + 1, dtype=np.uint32) << 16)
    z = bits.view(np.float32).astype(np.float64)
    assert z[0] == 2.0 ** -14 and z[-1] < 16.0 and z[-1] > 15.9
    H = O.Phi(z) - 0.5
    Q = z * O.phi(z)
    assert np.array_equal(vals[:, 0], vals[:, 1])                      # the two layouts hold the same H
    for got, ref in ((vals[:, 0], H), (vals[:, 2], Q)):
        want = ref.astype(np.float32).astype(np.float64)
        ulp = np.spacing(np.maximum(np.abs(want), 2.0 ** -126).astype(np.float32)).astype(np.float64)
        assert np.all(np.abs(got - want) <= ulp), np.abs(got - want).max()
        assert np.mean(got == want) > 0.995                             # essentially all entries are the exact rounding
        assert np.all(np.abs(got - ref) <= 0.51 * ulp + 1e-12 * np.abs(ref))
