"""Host-side sanitizer run of the CPU oracle (AddressSanitizer + UBSan; no GPU code involved)."""
import os

import oracle

def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    """Build the oracle as a standalone program with -fsanitize=address,undefined (host code only) and run
    one small step with ragged sizes: no out-of-bounds access, no undefined behaviour."""
    import subprocess
    import sys
    src = os.path.join(os.path.dirname(oracle.__file__), "apms_oracle.c")
    main_c = tmp_path / "main.c"
    main_c.write_text(r'''
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
int apms_oracle_compress(int, int64_t, int32_t, int64_t, const float*, const float*, float*, uint32_t*, float*, float*, float);
int apms_oracle_server_reduce(int, int64_t, int32_t, int64_t, const uint32_t*, const float*, const float*, float*, uint32_t*, float*, float*);
int apms_oracle_apply(int, int64_t, int32_t, int64_t, const uint32_t*, const float*, const float*, const float*, float*, float*, float, float);
int apms_oracle_warmup_step(int64_t, int32_t, float*, float*, float*, const float*, float, float, float, float, int64_t);
int apms_oracle_freeze(int64_t, int32_t, const float*, float*, float*, float*);
int apms_oracle_widen_g16(int, int64_t, const uint16_t*, float*);
int main(void) {
    const int64_t L = 96, C = 3, d = L * C; const int32_t n = 3;
    float *m = calloc(n * d, 4), *g = calloc(n * d, 4), *e = calloc(n * d, 4), *sc = calloc(n * C, 4);
    float *se = calloc(d, 4), *ssc = calloc(C, 4), *v = calloc(d, 4), *x = calloc(d, 4);
    uint32_t *p = calloc(n * d / 32, 4), *sp = calloc(d / 32, 4);
    uint16_t *h = calloc(n * d, 2);
    for (int64_t j = 0; j < n * d; ++j) { h[j] = (uint16_t)(j * 2654435761u >> 16); }
    apms_oracle_widen_g16(2, n * d, h, g);
    for (int64_t j = 0; j < n * d; ++j) if (!(g[j] == g[j]) || g[j] > 1e30f || g[j] < -1e30f) g[j] = 0.5f;
    for (int64_t j = 0; j < d; ++j) v[j] = 1e-6f + (float)j;
    for (int t = 1; t <= 2; ++t) apms_oracle_warmup_step(d, n, x, m, v, g, 1e-3f, 0.9f, 0.999f, 1e-8f, t);
    apms_oracle_freeze(d, n, m, m, e, se);
    for (int t = 0; t < 3; ++t) {
        apms_oracle_compress(0, d, n, L, m, g, e, p, sc, NULL, 0.9f);
        apms_oracle_server_reduce(0, d, n, L, p, sc, NULL, se, sp, ssc, NULL);
        apms_oracle_apply(0, d, n, L, sp, ssc, NULL, v, x, m, 1e-4f, 1e-8f);
    }
    printf("ok %g\n", (double)x[d - 1]);
    free(m); free(g); free(e); free(sc); free(se); free(ssc); free(v); free(x); free(p); free(sp); free(h);
    return 0;
}
''')
    exe = tmp_path / "oracle_san"
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-ffp-contract=off", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-o", str(exe), str(main_c), src, "-lm"])
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60,
                         env={**os.environ, "ASAN_OPTIONS": "detect_leaks=1:verify_asan_link_order=0"})
    assert out.returncode == 0 and out.stdout.startswith("ok"), out.stderr[-2000:]
