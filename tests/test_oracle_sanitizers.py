"""The C oracles under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU): a small driver links
oracle/*.c built with -fsanitize=address,undefined, runs seeded cases with exactly sized heap buffers (so that an
index one past a tail is caught), and must finish without a report and with the values of the normal build."""
import os
import subprocess
import sys

import numpy as np
import pytest

from oracle import hlstm_oracle as horc
from oracle import lstm_oracle as orc
from paper_1901_10997_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r"""
#include <stdio.h>
#include <stdlib.h>
int lstm_oracle_forward(int L, int ndir, int D0, int H, int T, int B, const float *const *Wx, const unsigned char *const *Mx,
                        const float *const *Wh, const unsigned char *const *Mh, const float *const *bias, const float *x,
                        const float *h0, const float *c0, double *y, double *hT, double *cT, int nthreads);
int hlstm_oracle_forward(int L, int ndir, int D0, int H, int G, int T, int B, const float *const *W1x,
                         const unsigned char *const *M1x, const float *const *W1h, const unsigned char *const *M1h,
                         const float *const *b1, const float *const *W2, const unsigned char *const *M2,
                         const float *const *b2, const float *x, const float *h0, const float *c0, double *y, double *hT,
                         double *cT, int nthreads);
static void *rd(FILE *f, size_t bytes) { void *p = malloc(bytes ? bytes : 1); if (bytes && fread(p, 1, bytes, f) != bytes) exit(3); return p; }
int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 2;
    int hdr[9];   /* L ndir D0 H G T B masked state */
    if (fread(hdr, sizeof(int), 9, f) != 9) return 3;
    const int L = hdr[0], nd = hdr[1], D0 = hdr[2], H = hdr[3], G = hdr[4], T = hdr[5], B = hdr[6], masked = hdr[7], state = hdr[8];
    const int n = L * nd;
    const float **a = calloc((size_t)n * 5, sizeof(void *));
    const unsigned char **m = calloc((size_t)n * 3, sizeof(void *));
    for (int l = 0; l < L; ++l)
        for (int d = 0; d < nd; ++d) {
            const int i = l * nd + d, D = l == 0 ? D0 : nd * H;
            if (G == 0) {
                a[i] = rd(f, (size_t)4 * H * D * 4);          if (masked) m[i] = rd(f, (size_t)4 * H * D);
                a[n + i] = rd(f, (size_t)4 * H * H * 4);      if (masked) m[n + i] = rd(f, (size_t)4 * H * H);
                a[2 * n + i] = rd(f, (size_t)4 * H * 4);
            } else {
                a[i] = rd(f, (size_t)4 * G * D * 4);          if (masked) m[i] = rd(f, (size_t)4 * G * D);
                a[n + i] = rd(f, (size_t)4 * G * H * 4);      if (masked) m[n + i] = rd(f, (size_t)4 * G * H);
                a[2 * n + i] = rd(f, (size_t)4 * G * 4);
                a[3 * n + i] = rd(f, (size_t)4 * H * G * 4);  if (masked) m[2 * n + i] = rd(f, (size_t)4 * H * G);
                a[4 * n + i] = rd(f, (size_t)4 * H * 4);
            }
        }
    float *x = rd(f, (size_t)T * B * D0 * 4);
    float *h0 = state ? rd(f, (size_t)n * B * H * 4) : NULL, *c0 = state ? rd(f, (size_t)n * B * H * 4) : NULL;
    fclose(f);
    const size_t ny = (size_t)T * B * nd * H, ns = (size_t)n * B * H;
    double *y = malloc((ny ? ny : 1) * 8), *hT = malloc((ns ? ns : 1) * 8), *cT = malloc((ns ? ns : 1) * 8);
    int rc;
    if (G == 0) rc = lstm_oracle_forward(L, nd, D0, H, T, B, a, m, a + n, m + n, a + 2 * n, x, h0, c0, y, hT, cT, 2);
    else rc = hlstm_oracle_forward(L, nd, D0, H, G, T, B, a, m, a + n, m + n, a + 2 * n, a + 3 * n, m + 2 * n, a + 4 * n, x, h0, c0, y, hT, cT, 2);
    if (rc != 0) return 4;
    FILE *o = fopen(argv[2], "wb");
    fwrite(y, 8, ny, o); fwrite(hT, 8, ns, o); fwrite(cT, 8, ns, o);
    fclose(o);
    for (int i = 0; i < 5 * n; ++i) free((void *)a[i]);
    for (int i = 0; i < 3 * n; ++i) free((void *)m[i]);
    free(a); free(m); free(x); free(h0); free(c0); free(y); free(hT); free(cT);
    return 0;
}
"""


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    d = tmp_path_factory.mktemp("asan")
    src = d / "driver.c"
    src.write_text(DRIVER)
    exe = d / "driver"
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-static-libasan", str(src), os.path.join(ROOT, "oracle", "lstm_oracle.c"),
           os.path.join(ROOT, "oracle", "hlstm_oracle.c"), "-o", str(exe), "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        pytest.skip("no sanitizer runtime for the host compiler here: " + r.stderr[-300:])
    return exe, d


def _write(path, w, case):
    G = w.gate_hidden
    masked = 1 if w.keep is not None else 0
    with open(path, "wb") as f:
        f.write(np.array([w.layers, w.ndir, w.input_dim, w.hidden, G, w.T, w.B, masked, 0 if case.h0 is None else 1],
                         np.int32).tobytes())
        for l in range(w.layers):
            for d in range(w.ndir):
                p = case.weights[(l, d)]
                names = (("W1x", "M1x"), ("W1h", "M1h"), ("b1", None), ("W2", "M2"), ("b2", None)) if G else \
                        (("Wx", "Mx"), ("Wh", "Mh"), ("b", None))
                for wn, mn in names:
                    f.write(np.ascontiguousarray(p[wn], np.float32).tobytes())
                    if mn and masked:
                        f.write(np.ascontiguousarray(p[mn], np.uint8).tobytes())
        f.write(np.ascontiguousarray(case.x, np.float32).tobytes())
        if case.h0 is not None:
            f.write(np.ascontiguousarray(case.h0, np.float32).tobytes())
            f.write(np.ascontiguousarray(case.c0, np.float32).tobytes())


@pytest.mark.parametrize("spec", [
    # layers, bidirectional, D0, H, G, T, B, keep, random state
    (1, False, 5, 3, 0, 4, 2, None, False),
    (2, True, 7, 5, 0, 3, 3, 0.5, True),
    (3, False, 1, 1, 0, 1, 1, 0.9, True),
    (2, False, 6, 9, 0, 0, 2, None, False),       # no timesteps
    (1, False, 5, 4, 3, 4, 2, None, False),
    (2, True, 6, 5, 7, 3, 2, 0.5, True),
])
def test_oracles_run_clean_under_asan_and_ubsan(driver, spec):
    exe, d = driver
    L, bidir, D0, H, G, T, Bn, keep, rs = spec
    w = inputs.Workload(60, "asan", L, bidir, D0, H, T, Bn, "f32", 0.4, keep, "uniform", G)
    case = inputs.make_case(w, 0, random_state=rs)
    inp, out = d / "in.bin", d / "out.bin"
    _write(inp, w, case)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([str(exe), str(inp), str(out)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stderr[-2000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-2000:]
    ref = (horc if G else orc).forward_case(case)
    got = np.frombuffer(open(out, "rb").read(), np.float64)
    want = np.concatenate([a.ravel() for a in ref])
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)
