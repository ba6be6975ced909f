"""The host-side plan, placement and bookkeeping (csrc/plan.cpp) built with AddressSanitizer and
UndefinedBehaviorSanitizer and driven over two thousand random cases, the plan in both modes: any out-of-bounds access, signed overflow or
other undefined behaviour aborts the run.  Host code only; no GPU, no HIP call."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r'''
#include <cstdio>
#include <cstdint>
#include <vector>
#include "feplb.h"
namespace feplb { void set_error(const char* fmt, ...) { (void)fmt; } }   // host.cpp's, without HIP
int main() {
  uint64_t s = 12345;
  auto rnd = [&](uint64_t m) { s = s * 6364136223846793005ull + 1442695040888963407ull; return (s >> 33) % m; };
  for (int it = 0; it < 2000; ++it) {
    const int P = 1 + (int)rnd(8), per = 1 + (int)rnd(32), E = P * per;
    std::vector<int32_t> owner(E), slots(P);
    std::vector<int64_t> n(E), before(P), after(P);
    std::vector<uint8_t> dyn(E);
    for (int e = 0; e < E; ++e) { owner[e] = e / per; n[e] = rnd(4) ? (int64_t)rnd(5000) : 0; dyn[e] = (uint8_t)rnd(2); }
    for (int r = 0; r < P; ++r) slots[r] = (int32_t)rnd(9);
    std::vector<feplb_move> moves(E + 1);
    int32_t nm = -1, chosen = -1;
    for (int mode = 0; mode < 2; ++mode) {
      const int32_t rc = feplb_plan(P, E, owner.data(), n.data(), dyn.data(), slots.data(), (int64_t)rnd(200), mode, -1,
                                    moves.data(), (int32_t)moves.size(), &nm, before.data(), after.data(), &chosen);
      if (rc != 0) { std::printf("rc %d in case %d\n", rc, it); return 1; }
      int64_t a = 0, b = 0;
      for (int r = 0; r < P; ++r) { a += after[r]; b += before[r]; }
      if (a != b || nm < 0 || nm > E) { std::printf("bad result in case %d\n", it); return 2; }
    }
    // a move table that is too small must be refused, not overrun
    int32_t rc = feplb_plan(P, E, owner.data(), n.data(), dyn.data(), slots.data(), 0, 0, -1, moves.data(), 0, &nm,
                            before.data(), after.data(), &chosen);
    if (rc != 0 && rc != FEPLB_ECAPACITY) { std::printf("rc %d with an empty move table\n", rc); return 3; }
    // macro level: history, placement (random current map, limit with and without slack), marking, bookkeeping
    std::vector<int64_t> hist(E, 0);
    for (int u = 0; u < 3; ++u) {
      for (int e = 0; e < E; ++e) n[e] = rnd(4) ? (int64_t)rnd(200000) : 0;
      if (feplb_history_update(E, hist.data(), n.data(), (int32_t)rnd(8)) != 0) return 4;
    }
    std::vector<int32_t> cur(E), out(E), home(E);
    for (int e = 0; e < E; ++e) cur[e] = (int32_t)rnd(P);
    int32_t moved = -1;
    if (feplb_place(P, E, hist.data(), per + (int32_t)rnd(3), cur.data(), out.data(), before.data(), after.data(), &moved) != 0) return 5;
    int64_t a2 = 0, b2 = 0;
    for (int r = 0; r < P; ++r) { a2 += after[r]; b2 += before[r]; }
    if (a2 != b2 || moved < 0 || moved > E) { std::printf("bad placement in case %d\n", it); return 6; }
    if (feplb_place(P, E, hist.data(), per - 1, cur.data(), out.data(), nullptr, nullptr, nullptr) != FEPLB_ESHAPE) return 7;
    if (feplb_mark_dynamic(P, E, out.data(), hist.data(), (int32_t)rnd(per + 2), dyn.data()) != 0) return 8;
    if (feplb_plan(P, E, out.data(), n.data(), dyn.data(), slots.data(), 0, 0, -1, moves.data(), (int32_t)moves.size(), &nm,
                   before.data(), after.data(), &chosen) != 0) return 9;
    if (feplb_apply_moves(P, E, out.data(), moves.data(), nm, home.data()) != 0) return 10;
    std::vector<double> v(P);
    for (int r = 0; r < P; ++r) v[r] = (double)after[r];
    double st = -1.0;
    if (feplb_straggler(P, v.data(), &st) != 0 || st < 0.0) return 11;
  }
  std::puts("ok");
  return 0;
}
'''


def test_plan_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    (tmp_path / "drv.cpp").write_text(DRIVER)
    exe = tmp_path / "plan_san"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROOT, "paper_2604_19654_amd", "csrc"),
           os.path.join(ROOT, "paper_2604_19654_amd", "csrc", "plan.cpp"), str(tmp_path / "drv.cpp"), "-o", str(exe)]
    built = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    if built.returncode != 0 and "sanitize" in built.stderr and "cannot find" in built.stderr:
        pytest.skip("sanitizer runtime libraries are not installed")
    assert built.returncode == 0, built.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0 and r.stdout.strip() == "ok", r.stdout + r.stderr[-3000:]
