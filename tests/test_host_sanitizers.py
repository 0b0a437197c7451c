"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer: the C oracle (all three decoder
routines), the C++ batch former and the request queue's frame allocator, each through a small native driver.
CPU only."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def run(cmd, **kw):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)  # the sanitizer runtime must come first in the library list
    return subprocess.run(cmd, capture_output=True, text=True, env=env, **kw)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "san_oracle")
    r = run(["gcc", "-std=c11", *SAN, "-fopenmp", os.path.join(ROOT, "tests", "native", "sanitize_host.c"),
             os.path.join(ROOT, "oracle", "aed_oracle.c"), "-lm", "-o", exe])
    assert r.returncode == 0, r.stderr
    r = run([exe])
    assert r.returncode == 0, r.stdout + r.stderr
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_batch_former_under_asan_ubsan(tmp_path):
    src = tmp_path / "drv.cpp"
    src.write_text(r'''
#include <cstdio>
#include <vector>
#include "include/aed_batching.h"
int main() {
    std::vector<int32_t> in, out;
    unsigned s = 3;
    for (int i = 0; i < 1000; ++i) { s = s * 1664525u + 1013904223u; in.push_back(1 + (s >> 8) % 500); s = s * 1664525u + 1013904223u; out.push_back(1 + (s >> 8) % 256); }
    aed_bucketing* b = nullptr;
    if (aed_bucketing_estimate(in.data(), out.data(), 1000, 30, 2, &b) != 0) return 2;
    std::vector<int32_t> iu(30), ou(60), sizes(60), batch_of(1000), bucket_of_batch(1000);
    aed_bucketing_bounds(b, iu.data(), ou.data());
    if (aed_bucketing_batch_sizes(b, 4500, 128, sizes.data()) != 0) return 3;
    int32_t nb = 0;
    for (int mode = 0; mode < 2; ++mode)
        if (aed_bucketing_form_batches(b, in.data(), out.data(), 1000, mode, sizes.data(), batch_of.data(), bucket_of_batch.data(), &nb) != 0) return 4;
    int32_t kept = 0;
    for (int i = 0; i < 1000; ++i) kept += batch_of[i] >= 0;
    std::vector<int32_t> avail(60, 0); avail[59] = 1;
    if (aed_bucket_select(1, 2, avail.data(), 60) != 59) return 5;
    if (aed_bucketing_allocate(b, 100000, 1, 1) != -1) return 6;
    if (aed_bucketing_estimate(in.data(), out.data(), 0, 30, 2, &b) == 0) return 7;
    std::printf("batches %d kept %d\n", nb, kept);
    aed_bucketing_free(b);
    return kept == 1000 ? 0 : 8;
}
''')
    exe = str(tmp_path / "san_batching")
    r = run(["g++", "-std=c++17", *SAN, "-I", ROOT, str(src),
             os.path.join(ROOT, "paper_2503_05931_amd", "csrc", "batching.cpp"), "-o", exe])
    assert r.returncode == 0, r.stderr
    r = run([exe])
    assert r.returncode == 0, r.stdout + r.stderr
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_frame_allocator_under_asan_ubsan(tmp_path):
    """The request queue's frame allocator against a brute-force occupancy map: random takes and gives,
    no overlap, first fit, and one whole interval again once everything is given back."""
    src = tmp_path / "frames.cpp"
    src.write_text(r'''
#include <cstdio>
#include <vector>
#include "paper_2503_05931_amd/csrc/frame_space.h"
int main() {
    const int total = 1000;
    aed::FrameSpace fs(total);
    std::vector<char> used(total, 0);
    std::vector<std::pair<int, int>> held;
    unsigned s = 7;
    auto rnd = [&](unsigned m) { s = s * 1664525u + 1013904223u; return (s >> 8) % m; };
    for (int it = 0; it < 20000; ++it) {
        if (held.empty() || rnd(100) < 55) {
            const int n = 1 + (int)rnd(rnd(4) == 0 ? 400 : 60);
            int want = -1;                       // brute force: lowest start of a free run of n
            for (int a = 0, run = 0; a < total; ++a) {
                run = used[a] ? 0 : run + 1;
                if (run == n) { want = a - n + 1; break; }
            }
            const int got = fs.take(n);
            if (got != want) { std::printf("take(%d) = %d, brute force says %d\\n", n, got, want); return 2; }
            if (got >= 0) {
                for (int a = got; a < got + n; ++a) { if (used[a]) return 3; used[a] = 1; }
                held.push_back({got, n});
            }
        } else {
            const size_t k = rnd((unsigned)held.size());
            for (int a = held[k].first; a < held[k].first + held[k].second; ++a) used[a] = 0;
            fs.give(held[k].first, held[k].second);
            held.erase(held.begin() + k);
        }
        // the free list is sorted, merged, and equals the occupancy map
        int free_total = 0, prev_end = -1;
        for (auto& r : fs.free_runs()) {
            if (r.second < 1 || r.first <= prev_end) return 4;   // empty run, or touching / overlapping its neighbour
            for (int a = r.first; a < r.first + r.second; ++a) if (used[a]) return 5;
            prev_end = r.first + r.second;
            free_total += r.second;
        }
        int want_free = 0;
        for (int a = 0; a < total; ++a) want_free += !used[a];
        if (free_total != want_free) return 6;
    }
    for (auto& h : held) fs.give(h.first, h.second);
    if (fs.free_runs().size() != 1 || fs.free_runs()[0].first != 0 || fs.free_runs()[0].second != total) return 7;
    if (fs.take(total) != 0 || fs.take(1) != -1) return 8;
    std::printf("ok\\n");
    return 0;
}
''')
    exe = str(tmp_path / "san_frames")
    r = run(["g++", "-std=c++17", *SAN, "-I", ROOT, str(src), "-o", exe])
    assert r.returncode == 0, r.stderr
    r = run([exe])
    assert r.returncode == 0, r.stdout + r.stderr
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr
