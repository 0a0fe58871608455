"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU code involved): the C oracle and the
library's host packer are compiled with gcc -fsanitize=address,undefined together with a small driver that runs every
entry point on small, odd-sized inputs; any out-of-bounds access, leak or undefined operation fails the run."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r"""
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "lordba.h"

int lordba_oracle_pack(const int8_t*, int64_t, int64_t, uint32_t*);
void lordba_oracle_unpack(const uint32_t*, int64_t, int64_t, int8_t*);
int lordba_oracle_sign_f64(const double*, int64_t, int8_t*);
int lordba_oracle_forward(const uint16_t*, const int8_t*, const int8_t*, const uint16_t*, const uint16_t*, const uint16_t*,
                          const uint16_t*, double*, int64_t, int64_t, int64_t, int64_t, int);
int lordba_oracle_forward_packed(const uint16_t*, const uint32_t*, const uint32_t*, const uint16_t*, const uint16_t*, const uint16_t*,
                                 const uint16_t*, double*, int64_t, int64_t, int64_t, int64_t, int);
int lordba_oracle_forward_multi(const uint16_t*, const int8_t*, const int8_t*, const uint16_t*, const uint16_t*, const uint16_t*,
                                const uint16_t*, double*, int64_t, int64_t, int64_t, int64_t, int64_t, int);
int lordba_oracle_forward_batched(const uint16_t*, const int8_t*, const int8_t*, const uint16_t*, const uint16_t*, const uint16_t*,
                                  const int32_t*, const uint16_t*, double*, int64_t, int64_t, int64_t, int64_t, int64_t);
int lordba_oracle_rank_intermediate(const uint16_t*, const int8_t*, const uint16_t*, double*, int64_t, int64_t, int64_t);
int lordba_oracle_backward(const uint16_t*, const uint16_t*, const int8_t*, const int8_t*, const uint16_t*, const uint16_t*,
                           const uint16_t*, const float*, const float*, double, const uint16_t*, double*, double*, double*, double*,
                           double*, double*, int64_t, int64_t, int64_t, int64_t);
int lordba_oracle_backward_multi(const uint16_t*, const uint16_t*, const int8_t*, const int8_t*, const uint16_t*, const uint16_t*,
                                 const uint16_t*, const float*, const float*, double, const uint16_t*, double*, double*, double*,
                                 double*, double*, double*, int64_t, int64_t, int64_t, int64_t, int64_t);

static uint32_t state = 12345u;
static uint32_t rnd(void) { state = state * 1664525u + 1013904223u; return state >> 8; }
static uint16_t half(void) { return (uint16_t)(((rnd() & 1u) << 15) | ((10u + rnd() % 8u) << 10) | (rnd() & 0x3ffu)); }  /* finite, normal */
#define NEW(T, n) ((T*)malloc(sizeof(T) * (size_t)((n) > 0 ? (n) : 1)))

int main(void) {
    const int64_t shapes[][4] = {{5, 37, 29, 3}, {1, 1, 1, 1}, {4, 64, 96, 8}, {0, 8, 8, 2}, {3, 33, 65, 7}};   /* T, d_in, d_out, r */
    for (unsigned c = 0; c < sizeof(shapes) / sizeof(shapes[0]); ++c) {
        const int64_t T = shapes[c][0], d_in = shapes[c][1], d_out = shapes[c][2], r = shapes[c][3], ell = 3, nad = 2;
        int8_t *sA = NEW(int8_t, nad * r * d_in), *sB = NEW(int8_t, nad * d_out * r);
        for (int64_t i = 0; i < nad * r * d_in; ++i) sA[i] = (rnd() & 1) ? 1 : -1;
        for (int64_t i = 0; i < nad * d_out * r; ++i) sB[i] = (rnd() & 1) ? 1 : -1;
        uint16_t *x = NEW(uint16_t, T * d_in), *g = NEW(uint16_t, T * d_out), *yb = NEW(uint16_t, T * d_out), *dxb = NEW(uint16_t, T * d_in);
        uint16_t *si = NEW(uint16_t, ell * d_in), *sr = NEW(uint16_t, ell * r), *so = NEW(uint16_t, ell * d_out);
        for (int64_t i = 0; i < T * d_in; ++i) { x[i] = half(); dxb[i] = half(); }
        for (int64_t i = 0; i < T * d_out; ++i) { g[i] = half(); yb[i] = half(); }
        for (int64_t i = 0; i < ell * d_in; ++i) si[i] = half();
        for (int64_t i = 0; i < ell * r; ++i) sr[i] = half();
        for (int64_t i = 0; i < ell * d_out; ++i) so[i] = half();
        float *lA = NEW(float, r * d_in), *lB = NEW(float, d_out * r);
        for (int64_t i = 0; i < r * d_in; ++i) lA[i] = sA[i] * 0.01f * (float)(1 + rnd() % 7);
        for (int64_t i = 0; i < d_out * r; ++i) lB[i] = sB[i] * 0.01f * (float)(1 + rnd() % 7);
        int32_t* ids = NEW(int32_t, T);
        for (int64_t t = 0; t < T; ++t) ids[t] = (int32_t)(rnd() % 4) - 1;     /* -1 .. 2: also out of range */
        double *y = NEW(double, T * d_out), *dx = NEW(double, T * d_in), *tt = NEW(double, T * r);
        double *dsi = NEW(double, ell * d_in), *dsr = NEW(double, ell * r), *dso = NEW(double, ell * d_out);
        double *dlA = NEW(double, r * d_in), *dlB = NEW(double, d_out * r);
        /* the library's host packer against the oracle's, both directions, all variants */
        const size_t wA = lordba_packed_words(r, d_in), wB = lordba_packed_words(d_out, r);
        uint32_t *pA = NEW(uint32_t, wA), *pB = NEW(uint32_t, wB), *qA = NEW(uint32_t, wA), *qB = NEW(uint32_t, wB);
        if (lordba_pack_signs(sA, sB, pA, pB, d_in, d_out, r) != LORDBA_OK) return 10;
        if (lordba_oracle_pack(sA, r, d_in, qA) || lordba_oracle_pack(sB, d_out, r, qB)) return 11;
        if (memcmp(pA, qA, wA * 4) || memcmp(pB, qB, wB * 4)) return 12;
        if (lordba_pack_signs_f32(lA, lB, qA, qB, d_in, d_out, r) != LORDBA_OK || memcmp(pA, qA, wA * 4) || memcmp(pB, qB, wB * 4)) return 13;
        int8_t *uA = NEW(int8_t, r * d_in), *uB = NEW(int8_t, d_out * r);
        if (lordba_unpack_signs(pA, pB, uA, uB, d_in, d_out, r) != LORDBA_OK || memcmp(uA, sA, (size_t)(r * d_in)) || memcmp(uB, sB, (size_t)(d_out * r))) return 14;
        lordba_oracle_unpack(qA, r, d_in, uA);
        if (memcmp(uA, sA, (size_t)(r * d_in))) return 15;
        /* every oracle entry point */
        if (lordba_oracle_forward(x, sA, sB, si, sr, so, yb, y, T, d_in, d_out, r, 3)) return 20;
        if (lordba_oracle_forward_packed(x, pA, pB, si, sr, so, yb, y, T, d_in, d_out, r, 1)) return 21;
        if (lordba_oracle_forward_multi(x, sA, sB, si, sr, so, yb, y, T, d_in, d_out, r, ell, 2)) return 22;
        if (lordba_oracle_forward_batched(x, sA, sB, si, sr, so, ids, yb, y, T, d_in, d_out, r, nad)) return 23;
        if (lordba_oracle_rank_intermediate(x, sA, si, tt, T, d_in, r)) return 24;
        if (lordba_oracle_backward(x, g, sA, sB, si, sr, so, lA, lB, 100.0, dxb, dx, dsi, dsr, dso, dlA, dlB, T, d_in, d_out, r)) return 25;
        if (lordba_oracle_backward(x, g, sA, sB, si, sr, so, lA, lB, 100.0, NULL, dx, dsi, dsr, dso, dlA, dlB, T, d_in, d_out, r)) return 26;
        if (lordba_oracle_backward_multi(x, g, sA, sB, si, sr, so, lA, lB, 7.0, dxb, dx, dsi, dsr, dso, dlA, dlB, T, d_in, d_out, r, ell)) return 27;
        free(sA); free(sB); free(x); free(g); free(yb); free(dxb); free(si); free(sr); free(so); free(lA); free(lB); free(ids);
        free(y); free(dx); free(tt); free(dsi); free(dsr); free(dso); free(dlA); free(dlB); free(pA); free(pB); free(qA); free(qB);
        free(uA); free(uB);
    }
    /* argument errors of the host packer: bad values, bad dimensions */
    int8_t bad[4] = {1, -1, 0, 1};
    uint32_t w[2];
    if (lordba_pack_signs(bad, bad, w, w + 1, 4, 4, 1) != LORDBA_ERR_VALUE) return 30;
    if (lordba_pack_signs(bad, bad, w, w + 1, 0, 4, 1) != LORDBA_ERR_DIM) return 31;
    puts("sanitized run ok");
    return 0;
}
"""


@pytest.mark.skipif(sys.platform != "linux", reason="gcc sanitizers")
def test_oracle_and_host_packer_under_asan_and_ubsan(tmp_path):
    drv = tmp_path / "driver.c"
    drv.write_text(DRIVER)
    exe = tmp_path / "driver"
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-O1", "-g"]
    inc = ["-I", os.path.join(ROOT, "include")]
    objs = []
    for cc, src, std in (("gcc", str(drv), "-std=c11"), ("gcc", os.path.join(ROOT, "oracle", "lordba_oracle.c"), "-std=c11"),
                         ("g++", os.path.join(ROOT, "paper_2605_24058_amd", "csrc", "lordba_pack.cpp"), "-std=c++17")):
        obj = tmp_path / (os.path.basename(src) + ".o")
        subprocess.check_call([cc, std, "-ffp-contract=off", "-Wall"] + san + inc + ["-c", src, "-o", str(obj)])
        objs.append(str(obj))
    subprocess.check_call(["g++"] + san + objs + ["-o", str(exe), "-lm", "-lpthread"])
    # (verify_asan_link_order=0: the environment may preload other libraries, which is none of this test's business)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert p.returncode == 0 and "sanitized run ok" in p.stdout, (p.returncode, p.stdout[-2000:], p.stderr[-4000:])
