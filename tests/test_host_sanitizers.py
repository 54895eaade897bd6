"""The host-only sources (planner, partition) rebuilt with AddressSanitizer + UBSan and driven
through a sweep of plans, explicit tables, tile tables, migration plans and partitions.  CPU only."""
import os
import shutil
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2510_00606_amd", "csrc")

DRIVER = textwrap.dedent(r"""
    #include <cstdio>
    #include <cstdlib>
    #include <vector>
    #include "plan_internal.h"
    // the library's ew_plan_free also releases device tables; plans here are never uploaded
    extern "C" void ew_plan_free(ew_plan_t *p) { delete p; }
    #define REQUIRE(c) do { if (!(c)) { std::printf("FAILED %s line %d\n", #c, __LINE__); return 1; } } while (0)
    static int check(ew_plan_t *p, uint64_t numel) {
      const ew_seg_t *s = ew_plan_segs(p);
      uint64_t sum = 0;
      for (uint64_t i = 0; i < ew_plan_num_segs(p); ++i) sum += s[i].len;
      REQUIRE(sum == numel && ew_plan_numel(p) == numel);
      for (int which = 0; which < 2; ++which)
        for (uint32_t te : {1u, 64u, 1024u})
          for (uint32_t al : {0u, 32u}) {
            uint64_t total = 0;
            REQUIRE(ew_plan_tiles(p, which, te, al, 0, 0, nullptr, &total) == EW_OK);
            std::vector<ew_tile_t> t(total);
            if (total) REQUIRE(ew_plan_tiles(p, which, te, al, 0, total, t.data(), nullptr) == EW_OK);
            uint64_t tsum = 0;
            for (auto &x : t) tsum += x.len;
            REQUIRE(tsum == (which ? numel : ew_plan_stage_len(p)));
          }
      ew_plan_free(p);
      return 0;
    }
    // the multiply-and-shift division of the tile decoder against the machine's own, on every divisor
    // up to 4096, divisors around every power of two, and dividends around multiples of the divisor
    static int check_div() {
      std::vector<uint32_t> ds;
      for (uint32_t d = 1; d <= 4096; ++d) ds.push_back(d);
      for (uint32_t b = 12; b < 32; ++b)
        for (int o = -2; o <= 2; ++o) ds.push_back((uint32_t)((1ull << b) + o));
      ds.push_back(0xffffffffu); ds.push_back(0xfffffffeu); ds.push_back(0x80000001u); ds.push_back(2654435761u);
      uint64_t x = 88172645463325252ull;
      for (uint32_t d : ds) {
        uint32_t magic; uint8_t s1, s2;
        ew::div_invariant_setup(d, magic, s1, s2);
        std::vector<uint32_t> ns = {0u, 1u, d - 1, d, d + 1, 0x7fffffffu, 0x80000000u, 0xffffffffu, 0xfffffffeu};
        for (unsigned long long k : {2ull, 3ull, 1000ull, 65535ull, 65536ull, (unsigned long long)(0xffffffffu / d)})
          for (int o = -1; o <= 1; ++o) ns.push_back((uint32_t)(k * d + o));
        for (int i = 0; i < 64; ++i) { x ^= x << 13; x ^= x >> 7; x ^= x << 17; ns.push_back((uint32_t)x); ns.push_back((uint32_t)(x >> 40)); }
        for (uint32_t n : ns) REQUIRE(ew::div_by_invariant(n, magic, s1, s2) == n / d);
      }
      return 0;
    }
    int main() {
      if (check_div()) return 1;
      for (uint32_t Do = 1; Do <= 6; ++Do)
        for (uint32_t Dn = 1; Dn <= 6; ++Dn)
          for (uint64_t mask = 1; mask < (1ull << Do); ++mask)
            for (uint64_t N : {0ull, 1ull, 9ull, 1000ull, 4099ull})
              for (uint64_t C : {1ull, 8ull, 100ull, 5000ull}) {
                ew_plan_t *p = nullptr;
                const int rc = ew_plan(Do, Dn, mask, N, C, &p);
                if (rc == EW_EUNRECOVERABLE) continue;
                REQUIRE(rc == EW_OK);
                if (check(p, N)) return 1;
              }
      ew_plan_t *p = nullptr;
      REQUIRE(ew_plan(64, 64, ~0ull, 1 << 20, 4096, &p) == EW_OK);
      if (check(p, 1 << 20)) return 1;
      const uint64_t src[] = {0, 100, 364, 1000, 1000, 4099}, dst[] = {0, 264, 500, 777};
      for (uint32_t a = 0; a < 2; ++a)
        for (uint32_t D : {1u, 3u, 8u, 32u})
          for (uint64_t mv = 0; mv <= 5; ++mv) {
            REQUIRE(ew_plan_migrate(a, D, 5, src, 3, dst, mv, &p) == EW_OK);
            if (check(p, 4099 + 777)) return 1;
          }
      const uint32_t L = 9, P = 4;
      std::vector<double> t(P * L * L), mem(L * L), cap(P, 5.0);
      for (uint32_t q = 0; q < P; ++q)
        for (uint32_t x = 0; x < L; ++x)
          for (uint32_t y = 0; y < L; ++y) { t[(q * L + x) * L + y] = (y + 1.0 - x) * (q + 1); mem[x * L + y] = y + 1.0 - x; }
      uint32_t bounds[P - 1]; double cost = 0;
      REQUIRE(ew_partition_layers(L, P, t.data(), mem.data(), cap.data(), bounds, &cost) == EW_OK);
      cap.assign(P, 1.0);
      REQUIRE(ew_partition_layers(L, P, t.data(), mem.data(), cap.data(), bounds, &cost) == EW_EINFEASIBLE);
      std::printf("sanitized sweep ok\n");
      return 0;
    }
""")


def test_planner_under_asan_ubsan(tmp_path):
    gxx = shutil.which("g++") or shutil.which("clang++")
    if not gxx:
        pytest.skip("no host C++ compiler")
    drv = tmp_path / "driver.cpp"
    drv.write_text(DRIVER)
    exe = tmp_path / "driver"
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, str(drv), os.path.join(CSRC, "plan.cpp"),
           os.path.join(CSRC, "partition.cpp"), "-o", str(exe), "-pthread"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1", LD_PRELOAD="")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=600)
    sys.stdout.write(r.stdout[-2000:])
    sys.stderr.write(r.stderr[-4000:])
    assert r.returncode == 0 and "sanitized sweep ok" in r.stdout
