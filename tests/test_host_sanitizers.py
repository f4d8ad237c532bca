"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the library's
planner (cs_params_init, the only non-trivial host logic) and the reference's C loops, each
driven by a small C/C++ program built here with gcc."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1")

PLANNER = r"""
#include <stdio.h>
#include "csketch.h"
int main() {
    struct { unsigned r, c; unsigned long long seed; long long d; } cases[] = {
        {5, 1u << 15, 190304489ull, 1 << 20}, {15, 180000, 1, 6500000}, {1, 1, 0, 0}, {7, 40, 3, 784},
        {5, 1u << 12, 9, 300001}, {3, 64, 3, 2000003}, {5, 1u << 20, 7, 5000000}, {1, 1u << 31, 5, 4096},
        {15, 1u << 6, 11, 70001}};
    for (auto& k : cases) {
        cs_params p;
        if (cs_params_init(&p, k.r, k.c, k.seed, k.d) != CS_OK) return 1;
        for (unsigned j = 0; j < k.r; ++j)
            if (p.visit[j].K > CS_MAX_VISITS || p.plan[j].D < 1 || p.plan[j].Dw < 1) return 2;
    }
    cs_params q;
    if (cs_params_init(&q, 4, 16, 1, 0) != CS_EINVAL) return 3;          /* even r */
    if (cs_params_init(&q, 5, 0, 1, 0) != CS_EINVAL) return 4;
    if (cs_params_init(0, 5, 16, 1, 0) != CS_EINVAL) return 5;
    if (cs_params_init(&q, 5, 16, 1, -1) != CS_EINVAL) return 6;
    return 0;
}
"""

ORACLE = r"""
#include <stdint.h>
#include <stdlib.h>
void cso_derive_params(uint64_t, int, uint64_t*, uint64_t*, uint64_t*, uint64_t*);
void cso_hash(int, uint32_t, const uint64_t*, const uint64_t*, const uint64_t*, const uint64_t*,
              const int64_t*, int64_t, uint32_t*, int8_t*);
void cso_accumulate_f32(int, uint32_t, const uint64_t*, const uint64_t*, const uint64_t*, const uint64_t*,
                        double*, const float*, int64_t, int64_t, double);
void cso_estimate(int, uint32_t, const uint64_t*, const uint64_t*, const uint64_t*, const uint64_t*,
                  const double*, int64_t, int64_t, double*);
int main(void) {
    enum { R = 7, C = 40, D = 784 };
    uint64_t a[R], b[R], as[R], bs[R];
    cso_derive_params(12345, R, a, b, as, bs);
    float* g = malloc(D * sizeof *g);
    for (int i = 0; i < D; ++i) g[i] = (float)(i % 7) - 3.0f;
    double* T = calloc(R * C, sizeof *T);
    double* est = malloc(D * sizeof *est);
    int64_t idx[3] = {0, D - 1, ((int64_t)1 << 61) - 2};
    uint32_t bucket[R * 3]; int8_t sign[R * 3];
    cso_hash(R, C, a, b, as, bs, idx, 3, bucket, sign);
    for (int t = 0; t < R * 3; ++t) if (bucket[t] >= C || (sign[t] != 1 && sign[t] != -1)) return 1;
    cso_accumulate_f32(R, C, a, b, as, bs, T, g, D, ((int64_t)1 << 61) - D, 0.5);
    cso_estimate(R, C, a, b, as, bs, T, D, ((int64_t)1 << 61) - D, est);
    free(g); free(T); free(est);
    return 0;
}
"""


def _build_and_run(tmp_path, name, source, compiler, extra):
    src = tmp_path / name
    src.write_text(source)
    exe = tmp_path / (name + ".bin")
    subprocess.check_call([compiler, *SAN, "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src), *extra])
    done = subprocess.run([str(exe)], env=ENV, capture_output=True, text=True)
    assert done.returncode == 0, done.stderr[-2000:]


def test_planner_under_sanitizers(tmp_path):
    _build_and_run(tmp_path, "planner.cpp", PLANNER, "g++",
                   ["-std=c++17", os.path.join(ROOT, "paper_1903_04488_amd", "csrc", "cs_host.cpp")])


def test_reference_loops_under_sanitizers(tmp_path):
    _build_and_run(tmp_path, "oracle_driver.c", ORACLE, "gcc",
                   [os.path.join(ROOT, "oracle", "cs_oracle.c"), "-lm"])
