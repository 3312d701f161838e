"""Host logic of the tiled kernel: the closed-form bound on the padded-input
extent of a tile must never be below the exact extent (it sizes the LDS
allocation).  Compiled with g++ from the library's own header, no GPU."""
import os
import subprocess
import textwrap

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_extent_bound_covers_exact_extent(tmp_path):
    src = tmp_path / "geom.cpp"
    src.write_text(textwrap.dedent(r"""
        #include "tile_geometry.h"
        #include <cstdio>
        #include <cstdlib>
        using namespace ebs;
        int main() {
            unsigned s = 12345u;
            auto rnd = [&](int lo, int hi) { s = s * 1664525u + 1013904223u; return lo + (int)((s >> 8) % (unsigned)(hi - lo + 1)); };
            long long worst_slack = 0; int checked = 0;
            for (int it = 0; it < 20000; ++it) {
                int H = rnd(1, 20), W = rnd(1, 20), R = rnd(1, 5), S = rnd(1, 5), st = rnd(1, 3);
                int pad = rnd(0, (R < S ? R : S) - 1);
                if (H + 2 * pad < R || W + 2 * pad < S) continue;
                int OH = (H + 2 * pad - R) / st + 1, OW = (W + 2 * pad - S) / st + 1;
                int N = rnd(1, 6);
                if (pad > 1) continue;
                TileGeom g{H, W, R, S, st, pad, OH, OW, 1};
                long long total = (long long)N * OH * OW;
                int tps[] = {1, 2, 3, 64, 128, 256, 512, 1024};
                for (int tp : tps) {
                    long long eff = tp < total ? tp : total;
                    long long bound = g.extent_bound(eff);
                    for (long long t0 = 0; t0 < total; t0 += tp) {
                        long long t1 = t0 + tp - 1; if (t1 > total - 1) t1 = total - 1;
                        long long ex = g.extent(t0, t1);
                        if (ex > bound || ex < 1) { printf("FAIL H%d W%d R%d S%d st%d pad%d N%d tp%d t0=%lld ex=%lld bound=%lld\n", H, W, R, S, st, pad, N, tp, t0, ex, bound); return 1; }
                        if (bound - ex > worst_slack) worst_slack = bound - ex;
                        ++checked;
                    }
                    // base() must be non-decreasing
                }
                for (long long t = 1; t < total; ++t) if (g.base(t) < g.base(t - 1)) { printf("FAIL monotone\n"); return 1; }
            }
            printf("ok checked=%d worst_slack=%lld\n", checked, worst_slack);
            return 0;
        }
    """))
    exe = tmp_path / "geom"
    subprocess.run(["g++", "-O1", "-std=c++17", "-I", os.path.join(ROOT, "paper_2003_07577_amd", "csrc"),
                    str(src), "-o", str(exe)], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.startswith("ok")


def test_fastdiv_matches_integer_division(tmp_path):
    src = tmp_path / "fd.cpp"
    src.write_text(textwrap.dedent(r"""
        #include "fastdiv.h"
        #include <cstdio>
        using namespace ebs;
        int main() {
            unsigned s = 99u;
            auto rnd = [&]() { s = s * 1664525u + 1013904223u; return s; };
            unsigned ds[] = {1, 2, 3, 5, 7, 9, 16, 30, 49, 56, 58, 81, 116, 3136, 3364, 65535, 65536, 65537, 1000003, 0x3fffffff, 0x7fffffff};
            for (unsigned d : ds) {
                FastDiv f = make_fastdiv(d);
                unsigned xs[] = {0, 1, d - 1, d, d + 1, 2 * d - 1, 2 * d, 0x7fffffffu, 0x7ffffffeu, 0x40000000u};
                for (unsigned x : xs) { if (x > 0x7fffffffu) continue; if (fd_div_host(x, f) != x / d) { printf("FAIL d=%u x=%u\n", d, x); return 1; } }
                for (int i = 0; i < 200000; ++i) { unsigned x = rnd() & 0x7fffffffu; if (fd_div_host(x, f) != x / d) { printf("FAIL d=%u x=%u\n", d, x); return 1; } }
            }
            for (int i = 0; i < 20000; ++i) {
                unsigned d = (rnd() & 0x7fffffffu) >> (rnd() % 31); if (d == 0) d = 1;
                FastDiv f = make_fastdiv(d);
                for (int j = 0; j < 100; ++j) { unsigned x = rnd() & 0x7fffffffu; if (fd_div_host(x, f) != x / d) { printf("FAIL d=%u x=%u\n", d, x); return 1; } }
                unsigned q = 0x7fffffffu / d; unsigned edge[] = {q * d, q * d - 1, (q ? (q - 1) * d : 0)};
                for (unsigned x : edge) { if (x > 0x7fffffffu) continue; if (fd_div_host(x, f) != x / d) { printf("FAIL d=%u x=%u\n", d, x); return 1; } }
            }
            printf("ok\n");
            return 0;
        }
    """))
    exe = tmp_path / "fd"
    subprocess.run(["g++", "-O1", "-std=c++17", "-I", os.path.join(ROOT, "paper_2003_07577_amd", "csrc"),
                    str(src), "-o", str(exe)], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.startswith("ok"), r.stdout + r.stderr
