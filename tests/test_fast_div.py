"""The launch-time multipliers that replace division instructions in the kernels (work
hand-out of the tile kernel, the causal rule's row index modulo the rows per head): the host
side of the same header function, compiled for the host alone, must agree with the division
operator for every divisor and dividend the kernels can meet."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(os.path.dirname(HERE), "paper_2505_14201_amd", "csrc")

PROGRAM = r"""
#include <cstdio>
#include <cstdint>
#include "flashd_common.h"
int main() {
    unsigned long long checked = 0, bad = 0;
    auto check = [&](uint32_t d, uint32_t n) {
        const flashd::FastDiv f = flashd::make_fast_div(d);
        ++checked;
        if (flashd::fast_div(n, f) != n / d) {
            if (bad < 5) std::printf("d=%u n=%u got %u\n", d, n, flashd::fast_div(n, f));
            ++bad;
        }
    };
    for (uint32_t d = 1; d <= 2000; ++d)
        for (uint32_t n = 0; n < 40000; ++n) check(d, n);
    uint64_t s = 88172645463325252ull;
    auto rnd = [&]() { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return s; };
    for (int i = 0; i < 20000000; ++i) {
        const uint32_t d = 1 + (uint32_t)(rnd() % 1073741824ull);        // up to 2^30
        check(d, (uint32_t)(rnd() & 0x7fffffffull));
    }
    const uint32_t edge[] = {1u, 2u, 3u, 7u, 128u, 65535u, 65536u, 1000000000u, 0x3fffffffu,
                             0x40000000u, 0x7fffffffu};
    for (uint32_t d : edge)
        for (uint32_t n : {0u, 1u, d - 1, d, d + 1, 2 * d - 1, 2 * d, 0x7ffffffeu, 0x7fffffffu,
                           0xffffffffu})
            check(d, n);
    std::printf("%llu checked, %llu bad\n", checked, bad);
    return bad != 0;
}
"""


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc to compile the header")
def test_fast_div_agrees_with_division(tmp_path):
    src = tmp_path / "fast_div_check.cpp"
    exe = tmp_path / "fast_div_check"
    src.write_text(PROGRAM)
    subprocess.run(["hipcc", "-x", "hip", "--cuda-host-only", "-O2", "-std=c++17", "-I", CSRC,
                    "-o", str(exe), str(src)], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stdout + out.stderr
    assert out.stdout.strip().endswith("0 bad"), out.stdout
