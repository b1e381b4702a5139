"""Host check of the multiply-high division the conv kernels use for tile and pixel decoding:
the same header compiled with g++ and compared with the machine's division over every small
divisor, the divisors the networks use, random 31-bit pairs and the extreme operands."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = r'''
#include <cstdio>
#include <cstdlib>
#include "fastdiv.hpp"
using namespace relay;
static int check(uint32_t n, uint32_t d) {
  const uint32_t q = fast_div(n, make_fastdiv(d));
  if (q != n / d) { std::printf("n=%u d=%u got %u want %u\n", n, d, q, n / d); return 1; }
  return 0;
}
int main() {
  const uint32_t top = 0x7fffffffu;
  int bad = 0;
  for (uint32_t d = 1; d <= 4096 && !bad; ++d) {
    for (uint32_t n = 0; n < 20000; ++n) bad |= check(n, d);
    for (uint32_t k = 0; k < 64; ++k) { bad |= check(top - k, d); bad |= check(k * d, d); bad |= check(k * d + d - 1, d); }
    const uint32_t qmax = top / d;
    bad |= check(qmax * d, d); bad |= check(qmax * d - 1, d); if (qmax * (uint64_t)d + d - 1 <= top) bad |= check(qmax * d + d - 1, d);
  }
  const uint32_t special[] = {7*7, 14*14, 28*28, 56*56, 112*112, 224*224, 784, 392, 196, 98, 49, 25, 13, 3136, 12544,
                              0x3fffffffu, 0x40000000u, 0x40000001u, 0x7ffffffeu, 0x7fffffffu, 65535u, 65536u, 65537u};
  for (uint32_t d : special) for (uint32_t k = 0; k < 200000 && !bad; ++k) { bad |= check(k * 10007u % top, d); bad |= check(top - k, d); }
  uint64_t s = 88172645463325252ull;
  for (int i = 0; i < 5000000 && !bad; ++i) {
    s ^= s << 13; s ^= s >> 7; s ^= s << 17;
    const uint32_t n = (uint32_t)(s >> 33), d = (uint32_t)((s & 0x7fffffffu) >> (s >> 59)) | 1u;
    bad |= check(n, d); bad |= check(n, d + 1);
  }
  return bad;
}
'''


def test_fastdiv_matches_integer_division(tmp_path):
    src = tmp_path / "fd.cpp"
    src.write_text(SRC)
    exe = tmp_path / "fd"
    subprocess.run(["g++", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "paper_1904_08368_amd", "csrc"), str(src), "-o", str(exe)],
                   check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout[-400:]
