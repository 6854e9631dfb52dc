"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the evaluator
translation unit (no HIP calls in it) and the C oracle, each built with g++/gcc and run
as a small native program.  GPU sanitizers are not available on this machine."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-g", "-O1"]
# verify_asan_link_order=0: tolerate libraries the environment preloads ahead of the ASan runtime
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")


def _run(cmd, **kw):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert p.returncode == 0, "%s\n%s" % (" ".join(cmd), p.stdout)
    return p.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_evaluator_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanity")
    _run(["g++", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"),
          "-I", os.path.join(ROOT, "paper_2601_02311_amd", "csrc"),
          os.path.join(ROOT, "paper_2601_02311_amd", "csrc", "ps_cost.cpp"),
          os.path.join(ROOT, "tests", "native", "host_sanity.cpp"), "-o", exe])
    assert "host sanity ok" in _run([exe], env=ENV)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no host compiler")
def test_oracle_under_asan_ubsan(tmp_path):
    src = tmp_path / "drv.c"
    src.write_text(r'''
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "step.c"
int main(void)
{
    enum { N = 4, n = 1031 };
    uint16_t *g[N]; const void *gp[N];
    for (int r = 0; r < N; ++r) {
        g[r] = malloc(n * 2);
        for (int e = 0; e < n; ++e) g[r][e] = (uint16_t)(0x3a00 + ((e * 31 + r * 7) & 0xff) + ((e & 1) << 15));
        gp[r] = g[r];
    }
    float *th = malloc(n * 4), *m = calloc(n, 4), *v = calloc(n, 4), *acc = malloc(n * 4);
    uint16_t *p = malloc(n * 2);
    for (int e = 0; e < n; ++e) th[e] = 0.01f * (float)(e % 17 - 8);
    oracle_scalars s;
    for (uint64_t t = 1; t <= 3; ++t) {
        oracle_derive_scalars(1e-4, 0.9, 0.999, 1e-8, 0.01, t, N, 0.0, 0.0, &s);
        oracle_step_f32(gp, N, 0, &s, th, m, v, p, 0, 0, n);
        oracle_step_f32(gp, N, 2, &s, th, m, v, p, 1, 0, n);   /* the same bits read as binary16 */
    }
    oracle_accumulate(gp, N, 0, acc, 1, 0, n);
    oracle_accumulate(gp, N, 0, acc, 0, 3, n - 3);
    double ss = oracle_mean_sumsq(gp, N, 0, 0.25f, acc, 0, n), out[2];
    oracle_diff_sumsq(g[0], g[1], 0, 0, n, out);
    uint64_t c = oracle_checksum((const uint64_t *)th, n / 2, 5);
    double *t64 = malloc(n * 8), *m64 = malloc(n * 8), *v64 = malloc(n * 8);
    oracle_step_f64(gp, N, 0, 1e-4, 0.9, 0.999, 1e-8, 0.01, 4, 0.0, 0.0, th, m, v, t64, m64, v64, 0, n);
    uint16_t edge[6]; float fe[6] = {3.4e38f, -3.4e38f, 1e-45f, -0.0f, 1.0f, 65504.0f};
    oracle_bf16_rne_array(fe, edge, 6);
    oracle_f16_rne_array(fe, edge, 6);
    printf("oracle ok %g %g %llu %g %u\n", ss, out[0], (unsigned long long)c, t64[7], edge[0]);
    for (int r = 0; r < N; ++r) free(g[r]);
    free(th); free(m); free(v); free(acc); free(p); free(t64); free(m64); free(v64);
    return !(ss > 0 && oracle_clip_coef(ss, 0, 1e-9) < 1.0);
}
''')
    exe = str(tmp_path / "oracle_sanity")
    _run(["gcc", "-std=c11", *SAN, "-ffp-contract=off", "-I", os.path.join(ROOT, "oracle"), str(src),
          "-o", exe, "-lm"])
    assert "oracle ok" in _run([exe], env=ENV)
