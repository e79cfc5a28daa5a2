"""The multiply-high division the kernels use for tile and pixel numbers (csrc/bsp_fastdiv.h),
compiled for the host: exact for every dividend x with x * d < 2^32, which is the condition the
launchers check before a launch; beyond it wrong quotients exist, so the checks are needed."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PROGRAM = r"""
#include <cstdio>
#include <cstdint>
#include "bsp_fastdiv.h"
int main() {
  // divisors: all small ones, then a spread up to 2^20 (tiles per image, pixels per row, pitches)
  uint64_t checked = 0, wrong_inside = 0, wrong_beyond = 0;
  for (uint32_t d = 1; d <= (1u << 20); d = d < 4096 ? d + 1 : d + d / 7 + 1) {
    const FastDiv f = make_fastdiv(d);
    const uint64_t limit = ((1ull << 32) - 1) / d;  // largest x with x * d < 2^32
    // every dividend for small ranges, otherwise the multiples of d and their neighbours
    // (where a quotient changes) and the end of the range
    if (limit <= 70000) {
      for (uint64_t x = 0; x <= limit; ++x, ++checked) wrong_inside += fdiv_host((uint32_t)x, f) != x / d;
    } else {
      const uint64_t step = limit / d / 3000 + 1;
      for (uint64_t q = 0; q * d <= limit; q += step)
        for (int64_t e = -2; e <= 2; ++e) {
          const int64_t x = (int64_t)(q * d) + e;
          if (x < 0 || (uint64_t)x > limit) continue;
          ++checked;
          wrong_inside += fdiv_host((uint32_t)x, f) != (uint64_t)x / d;
        }
      for (uint64_t x = limit - 5000; x <= limit; ++x, ++checked) wrong_inside += fdiv_host((uint32_t)x, f) != x / d;
    }
    // beyond the limit the quotient may be off by one: count, to show the bound matters
    if (d > 1)
      for (uint64_t x = 0xFFFFFFFFull - 5000; x <= 0xFFFFFFFFull; ++x) wrong_beyond += fdiv_host((uint32_t)x, f) != x / d;
  }
  // the case that prompted the launcher's check: 131072 tiles per image, the last three tiles
  const FastDiv f = make_fastdiv(131072);
  int known = 0;
  for (uint32_t x = 131069; x <= 131071; ++x) known += fdiv_host(x, f) != x / 131072;
  printf("%llu %llu %llu %d\n", (unsigned long long)checked, (unsigned long long)wrong_inside,
         (unsigned long long)wrong_beyond, known);
  return 0;
}
"""


def test_fastdiv_is_exact_inside_the_checked_range(tmp_path):
    src = tmp_path / "fd.cpp"
    src.write_text(PROGRAM)
    exe = tmp_path / "fd"
    subprocess.run(["g++", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "paper_2407_09453_amd", "csrc"),
                    str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    checked, wrong_inside, wrong_beyond, known = (int(v) for v in out)
    assert checked > 10_000_000
    assert wrong_inside == 0
    assert wrong_beyond > 0          # without the launchers' checks wrong tile numbers would occur
    assert known == 3                # x = 131069..131071 with d = 131072: x * d >= 2^32, all three wrong


def test_launchers_state_the_condition():
    """Every source that builds a divider also bounds its dividends (a 2^32 comparison nearby)."""
    csrc = os.path.join(ROOT, "paper_2407_09453_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if not name.endswith((".hip", ".cpp")):
            continue
        text = open(os.path.join(csrc, name)).read()
        if "make_fastdiv(" in text:
            assert "1ll << 32" in text, f"{name} builds dividers but never bounds a dividend"
