"""The host packer under AddressSanitizer + UBSan (host code only, no GPU):
pack.cpp is compiled with g++ into a small driver that packs and unpacks
random TW / TVW masks, ragged sizes included, and checks the round trip."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r"""
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>
#include "packed.h"
int main() {
  std::mt19937 rng(7);
  int fails = 0;
  for (int it = 0; it < 60; ++it) {
    const int K = 1 + rng() % 150, N = 1 + rng() % 300;
    const int G = (int[]){32, 64, 128}[rng() % 3];
    const int pattern = it % 2;
    std::vector<uint16_t> B((size_t)K * N);
    for (auto& b : B) b = (uint16_t)rng();
    std::vector<uint8_t> tm((size_t)K * N, 0), mask((size_t)K * N, 0);
    std::vector<int> cols;
    for (int n = 0; n < N; ++n) if (rng() % 10 < 8) cols.push_back(n);
    for (size_t i = 0; i < cols.size(); i += G) {
      std::vector<int> rows;
      for (int k = 0; k < K; ++k) if (rng() % 10 < 5) rows.push_back(k);
      for (size_t j = i; j < cols.size() && j < i + G; ++j) {
        for (int k : rows) tm[(size_t)k * N + cols[j]] = 1;
        if (!pattern) { for (int k : rows) mask[(size_t)k * N + cols[j]] = 1; continue; }
        for (size_t g = 0; g < rows.size(); g += 4) {          // keep up to 2 of each group
          int kept = 0;
          for (size_t p = g; p < rows.size() && p < g + 4; ++p)
            if (kept < 2 && rng() % 2) { mask[(size_t)rows[p] * N + cols[j]] = 1; ++kept; }
        }
      }
    }
    tw_handle_s h;
    tw_status st = twg::pack_host(B.data(), mask.data(), pattern ? tm.data() : nullptr, K, N, G, pattern, &h);
    if (st != TW_OK) { std::printf("pack failed %d at it %d\n", (int)st, it); ++fails; continue; }
    std::vector<uint16_t> Bm((size_t)K * N); std::vector<uint8_t> m2((size_t)K * N);
    twg::unpack_host(&h, Bm.data(), m2.data());
    for (size_t i = 0; i < mask.size(); ++i) {
      if (m2[i] != mask[i] || Bm[i] != (mask[i] ? B[i] : 0)) { ++fails; std::printf("round trip mismatch it %d\n", it); break; }
    }
  }
  std::printf("done fails=%d\n", fails);
  return fails ? 1 : 0;
}
"""


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_packer_round_trip_under_asan_ubsan(tmp_path):
    src = tmp_path / "driver.cpp"
    src.write_text(DRIVER)
    exe = tmp_path / "driver"
    csrc = os.path.join(ROOT, "paper_2402_10876_amd", "csrc")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-I", csrc, "-I", os.path.join(ROOT, "include"), str(src), os.path.join(csrc, "pack.cpp"), "-o", str(exe)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1")
    env.pop("LD_PRELOAD", None)      # a preloaded library would have to come after the ASan runtime
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, (r.stdout + r.stderr)[-2000:]
    assert "fails=0" in r.stdout
