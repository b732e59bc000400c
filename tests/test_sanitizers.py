"""Memory-safety check of the CPU oracle under AddressSanitizer + UBSan (host code only, no GPU).

The oracle is what every parity claim rests on; an out-of-bounds read in it could make two wrong
results agree.  It is rebuilt here as a small executable with -fsanitize=address,undefined and run on
ragged sizes, every mantissa width and a damaged container.
"""
import os
import subprocess
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = textwrap.dedent(r"""
    #include <stdio.h>
    #include <stdlib.h>
    #include <string.h>
    #include "neuzip_oracle.h"
    static uint32_t rng = 12345;
    static uint32_t next(void) { rng = rng * 1664525u + 1013904223u; return rng >> 8; }
    int main(void) {
        const uint64_t sizes[] = {0, 1, 7, 8, 127, 4095, 4096, 4097, 70001};
        const int ks[] = {7, 3, 1, 0};
        for (unsigned si = 0; si < sizeof sizes / sizeof *sizes; si++) {
            uint64_t n = sizes[si];
            uint16_t *w = malloc((n + 1) * 2), *back = malloc((n + 1) * 2), *want = malloc((n + 1) * 2);
            for (uint64_t i = 0; i < n; i++)   /* narrow exponent range with a few outliers */
                w[i] = (uint16_t)(((next() & 1) << 15) | ((118 + next() % 6 + (next() % 97 == 0) * (next() % 100)) << 7) | (next() & 0x7F));
            for (int ki = 0; ki < 4; ki++) {
                uint64_t cap = nzo_compress_bound(n, ks[ki]), len = 0;
                uint8_t *blob = malloc(cap);
                if (nzo_compress(w, n, ks[ki], blob, cap, &len, 3) != NZO_OK) return 1;
                uint8_t *exact = malloc(len ? len : 1);         /* exact-size copy: overreads trip ASan */
                memcpy(exact, blob, len);
                if (nzo_decompress(exact, len, back, n, 2) != NZO_OK) return 2;
                nzo_truncate(w, n, ks[ki], want);
                if (memcmp(back, want, n * 2) != 0) return 3;
                if (len > 700) {                                  /* damaged payload must not crash */
                    exact[len / 2] ^= 0x40; exact[len / 2 + 3] ^= 0x11;
                    (void)nzo_decompress(exact, len, back, n, 1);
                }
                if (len > 64) (void)nzo_decompress(exact, len - 16, back, n, 1);
                free(exact); free(blob);
            }
            free(w); free(back); free(want);
        }
        puts("sanitized oracle ok");
        return 0;
    }
""")


def test_oracle_under_asan_and_ubsan(tmp_path):
    src = tmp_path / "driver.c"
    src.write_text(DRIVER)
    exe = tmp_path / "oracle_asan"
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-static-libasan", "-pthread", "-I", os.path.join(ROOT, "oracle"),
           str(src), os.path.join(ROOT, "oracle", "neuzip_oracle.c"), "-lm", "-o", str(exe)]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "asan" in built.stderr.lower():
        pytest.skip("sanitizer runtime not available: " + built.stderr[-200:])
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "sanitized oracle ok" in run.stdout
