"""The host scheduler under AddressSanitizer + UBSan (host code only: plain g++, no GPU, no HIP).
A small C++ driver is compiled together with the scheduler sources and hammers ss_schedule /
ss_schedule_failures / ss_plan_free with random groups and every flag combination, checking the plan
invariants (each query exactly once, offsets monotone, caps in range) in C++ as well."""
import os
import shutil
import subprocess
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2305_13144_amd", "csrc")

DRIVER = textwrap.dedent(r"""
    #include <cstdint>
    #include <cstdio>
    #include <cstdlib>
    #include <vector>
    #include "ss.h"
    static uint64_t s = 88172645463325252ull;
    static uint32_t rnd() { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return (uint32_t)(s >> 11); }
    static void check(const ss_plan* p, int n, const ss_policy& pol) {
        if (p->n != n) { std::printf("bad n\n"); std::exit(2); }
        std::vector<int> seen(n, 0);
        if (p->mb_offsets[0] != 0 || p->mb_offsets[p->n_mb] != n) { std::printf("bad offsets\n"); std::exit(2); }
        for (int k = 0; k < p->n_mb; ++k) {
            if (p->mb_offsets[k + 1] <= p->mb_offsets[k]) { std::printf("empty micro-batch\n"); std::exit(2); }
            if (p->mb_cap[k] < 1 || p->mb_cap[k] > pol.base_len) { std::printf("bad cap\n"); std::exit(2); }
        }
        for (int i = 0; i < n; ++i) {
            int q = p->query_idx[i];
            if (q < 0 || q >= n || seen[q]++) { std::printf("not a permutation\n"); std::exit(2); }
        }
    }
    int main() {
        const uint32_t flagsets[] = {0, SS_SORT, SS_SORT | SS_FCR, SS_SORT | SS_BIN, SS_SORT | SS_BIN | SS_FCR,
                                     SS_SORT | SS_FCR | SS_VBS, SS_SORT | SS_BIN | SS_FCR | SS_VBS | SS_COMPACT};
        for (int trial = 0; trial < 3000; ++trial) {
            int n = 1 + rnd() % 400;
            ss_policy pol;
            pol.flags = flagsets[rnd() % 7];
            pol.base_batch = 1 + rnd() % 20;
            pol.max_batch = pol.base_batch + rnd() % 300;
            pol.base_len = 1 + rnd() % 1100;
            pol.vbs_rule = rnd() % 2;
            int bin = (pol.flags & SS_BIN) ? 1 + rnd() % 100 : (int)(rnd() % 2) * (1 + rnd() % 100);
            std::vector<int32_t> pred(n);
            for (auto& v : pred) v = 1 + rnd() % (pol.base_len * 2 + 3);
            ss_plan* p = nullptr;
            if (ss_schedule(pred.data(), n, bin, &pol, &p) != SS_OK) { std::printf("schedule: %s\n", ss_last_error()); return 3; }
            check(p, n, pol);
            ss_plan_free(p);
            std::vector<int32_t> failed;
            for (int i = 0; i < n; ++i) if (rnd() % 4 == 0) failed.push_back(i);
            if (ss_schedule_failures(pred.data(), n, failed.data(), (int)failed.size(), bin, &pol, &p) != SS_OK) return 4;
            if (p->n != (int)failed.size()) return 5;
            ss_plan_free(p);
        }
        // error paths must not leak or touch the output
        ss_plan* p = nullptr;
        ss_policy bad = {SS_BIN, 16, 512, 256, 0};
        int32_t one = 5;
        if (ss_schedule(&one, 1, 50, &bad, &p) != SS_EINVAL || p != nullptr) return 6;
        std::printf("ok\n");
        return 0;
    }
""")


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_scheduler_under_asan_ubsan(tmp_path):
    drv = tmp_path / "driver.cpp"
    drv.write_text(DRIVER)
    exe = tmp_path / "driver"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-I", os.path.join(ROOT, "include"), str(drv), os.path.join(CSRC, "ss_sched.cpp"),
           os.path.join(CSRC, "ss_common.cpp"), "-o", str(exe)]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.strip() == "ok"


PLAN_DRIVER = textwrap.dedent(r"""
    #include <cstdio>
    #include <cstdlib>
    #include "ss_plan.h"
    // Every plan the projection planner can return for 1..n_max rows must fit the partial-sum buffer the engine
    // sizes with gemm_partial_rows_bound (the kernels write [ksplit][rows][N] floats into it).
    int main() {
        const int dims[] = {64, 256, 512, 1024, 2048, 4096, 5120, 8192};
        const int ffns[] = {16, 512, 688, 4096, 11008, 13824, 28672};
        const int row_grid[] = {1, 15, 16, 17, 33, 63, 64, 65, 127, 128, 129, 163, 255, 256, 257, 511, 512, 640, 641,
                                1023, 1024, 1025, 2311, 2312, 2313, 4642, 4643, 4644, 8191, 8192, 10880, 10881, 32703,
                                32704, 32705, 100000, 1048576};
        const int cus[] = {64, 256, 304};
        long checked = 0;
        const int modes[] = {0, 1, 2, 4, 5, 6, 8, 9, 10, 12, 13, 14};   // every mode the library accepts
        for (int mode : modes) {
            ss::set_gemm_mode(mode);
            for (int cu : cus)
                for (int d : dims)
                    for (int F : ffns) {
                        const int Fp = (F + 63) / 64 * 64;
                        struct { int N, Kp, epi; bool sliced_only; } mats[] = {
                            {3 * d, d, ss::EPI_PARTIAL, false}, {d, d, ss::EPI_PARTIAL, false},
                            {2 * F, d, ss::EPI_SWIGLU, true}, {d, Fp, ss::EPI_PARTIAL, false}};
                        for (auto& m : mats)
                            for (int n_max : row_grid) {
                                const size_t cap = ss::gemm_partial_rows_bound(m.N, n_max, m.sliced_only);
                                for (int n : row_grid) {
                                    if (n > n_max) break;
                                    const ss::GemmPlan p = ss::gemm_plan(m.N, m.Kp, n, m.epi, cu);
                                    if (p.ksplit < 1 || p.ksplit > 8) { std::printf("bad ksplit\n"); return 2; }
                                    // what the launchers assume of a plan
                                    const int KB = m.Kp / 32;
                                    bool ok = KB / p.ksplit >= 1 && (p.ksplit & (p.ksplit - 1)) == 0;
                                    if (p.sweep_gn > 0) {        // sweep kernel: at most 8 units per workgroup, 4 with 4 waves
                                        const int nbw = ss::sweep_nbw(m.epi, n);
                                        const int units = (m.N / 16 + nbw - 1) / nbw;
                                        const int per = (units + p.sweep_gn - 1) / p.sweep_gn;
                                        ok = ok && n <= ss::kSweepMaxRows && per >= 1 && per <= 8;
                                        ok = ok && (p.sweep_p == 8 || (p.sweep_p == 4 && per <= 4));
                                        ok = ok && (p.sweep_kh == 1 || (p.sweep_kh == 2 && p.sweep_p == 4 && n > 96));
                                        ok = ok && (m.epi != ss::EPI_SWIGLU || p.ksplit == 1);
                                    } else if (n <= 64) {        // skinny kernel
                                        ok = ok && (p.nb == 2 || p.nb == 4) && (p.kd == 2 || p.kd == 4);
                                        ok = ok && (m.epi != ss::EPI_SWIGLU || p.ksplit == 1);
                                    } else {                     // tiled kernel
                                        ok = ok && (p.kp == 1 || (p.kp == 2 && p.ksplit == 1)) && (p.tms == 4 || p.tms == 8);
                                        ok = ok && p.ksplit <= 4 && (p.tms == 4 || n >= ss::kTiledTallFrom);
                                        ok = ok && ((mode & 8) == 0 || p.tms == 4);
                                    }
                                    if (!ok) {
                                        std::printf("plan breaks a launcher's assumption: mode %d N %d Kp %d rows %d cu %d: "
                                                    "ksplit %d nb %d kd %d kp %d sweep %d/%d/%d tms %d\n", mode, m.N, m.Kp, n,
                                                    cu, p.ksplit, p.nb, p.kd, p.kp, p.sweep_p, p.sweep_gn, p.sweep_kh, p.tms);
                                        return 7;
                                    }
                                    if (m.sliced_only && p.ksplit == 1) continue;
                                    if ((size_t)p.ksplit * (size_t)n > cap) {
                                        std::printf("overflow: N %d Kp %d rows %d (n_max %d) ksplit %d > %zu rows\n", m.N,
                                                    m.Kp, n, n_max, p.ksplit, cap);
                                        return 3;
                                    }
                                    ++checked;
                                }
                            }
                    }
        }
        // dense sweep of the row count on the shapes the advisor's replay found overflowing
        ss::set_gemm_mode(0);
        for (int n_max = 1; n_max <= 12000; n_max += 7) {
            const size_t c1 = ss::gemm_partial_rows_bound(1024, n_max), c2 = ss::gemm_partial_rows_bound(2 * 512, n_max, true);
            for (int n = 1; n <= n_max; n += 13) {
                if ((size_t)ss::gemm_plan(1024, 4096, n, ss::EPI_PARTIAL, 256).ksplit * n > c1) return 4;
                if ((size_t)ss::gemm_plan(1024, 1024, n, ss::EPI_PARTIAL, 256).ksplit * n > c1) return 5;
                const ss::GemmPlan g = ss::gemm_plan(2 * 512, 4096, n, ss::EPI_SWIGLU, 256);
                if (g.ksplit > 1 && (size_t)g.ksplit * n > c2) return 6;
            }
        }
        std::printf("ok %ld\n", checked);
        return 0;
    }
""")


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_projection_plans_fit_their_partial_sum_buffers(tmp_path):
    drv = tmp_path / "plan_driver.cpp"
    drv.write_text(PLAN_DRIVER)
    exe = tmp_path / "plan_driver"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-I", CSRC, str(drv), os.path.join(CSRC, "ss_plan.cpp"), "-o", str(exe)]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.startswith("ok ")
