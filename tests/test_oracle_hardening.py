"""Checks that guard the checker itself: the frozen rounding draws, and the C oracle run
under AddressSanitizer + UndefinedBehaviorSanitizer on the host (no GPU involved)."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLD = os.path.join(ROOT, "tests", "golden", "uniform24.txt")


def test_uniform24_matches_frozen_draws(oracle):
    """The counter hash behind the rounding draws may not move unnoticed: every stored draw
    (written by tests/golden/make_uniform24.py from the oracle alone) is reproduced."""
    n = 0
    with open(GOLD) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            seed, stream, row, col, draw = (int(t) for t in line.split())
            assert oracle.uniform24(seed, stream, row, col) == draw, (seed, stream, row, col)
            assert 0 <= draw < 2 ** 24
            n += 1
    assert n >= 300


def test_quantizer_uses_the_frozen_draws(oracle):
    """Ties the packed bits to the frozen draws: a row whose normalised values sit at k / 2^24
    exactly gets bit = [draw < k]."""
    import numpy as np
    d, rows = 96, 3
    seed, stream = 20230301, 7
    rng = np.random.default_rng(5)
    k = rng.integers(1, 2 ** 24 - 1, size=(rows, d))
    k[:, 0], k[:, 1] = 0, 2 ** 24                      # pin min = 0 and max = 1: scale = 1 exactly
    x = (k.astype(np.float64) / 2.0 ** 24).astype(np.float32)
    assert np.array_equal(x.astype(np.float64) * 2 ** 24, k)          # exactly representable
    packed, scale, zero = oracle.quantize_1bit(x, d, rows, seed, stream)
    assert (scale == 1.0).all() and (zero == 0.0).all()
    for i in range(rows):
        for c in range(d):
            bit = (int(packed[i, c // 64]) >> (c % 64)) & 1
            assert bit == (1 if oracle.uniform24(seed, stream, i, c) < k[i, c] else 0), (i, c)


DRIVER = r"""
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
/* the oracle's translation unit, compiled with the sanitizers */
#include "sylvie_oracle.c"

int main(void)
{
    enum { N = 37, D = 131, W = (D + 63) / 64, NDST = 11 };
    float *x = malloc(sizeof(float) * N * D), *out = malloc(sizeof(float) * N * D);
    float *J = calloc((size_t)NDST * D, sizeof(float));
    uint64_t *packed = malloc(sizeof(uint64_t) * N * W);
    float scale[N], zero[N];
    int32_t idx[N], dst[N];
    for (int i = 0; i < N * D; ++i) x[i] = (float)((i * 2654435761u) % 1000) / 37.0f - 11.0f;
    for (int i = 0; i < N; ++i) { idx[i] = (i * 7) % N; dst[i] = (i * 5) % NDST; }
    for (int c = 0; c < D; ++c) x[3 * D + c] = 2.5f;          /* constant row */
    orc_quantize_1bit(x, D, D, idx, 0, N, 99u, 3u, 0, packed, scale, zero);
    orc_dequantize_1bit_fwd(packed, scale, zero, N, D, out, D, 0);
    orc_dequantize_1bit_bwd(packed, scale, zero, N, D, J, D, dst);
    for (int i = 0; i < N; ++i)
        for (int c = 0; c < D; ++c) {
            const float v = out[i * D + c];
            if (!(v == zero[i] || v == zero[i] + scale[i])) { puts("level"); return 1; }
        }
    /* aggregation on a ring with self loops */
    int64_t rowptr[N + 1];
    int32_t col[3 * N];
    float w[3 * N];
    for (int v = 0; v < N; ++v) {
        rowptr[v] = 3 * v;
        col[3 * v] = (v + N - 1) % N; col[3 * v + 1] = v; col[3 * v + 2] = (v + 1) % N;
        w[3 * v] = w[3 * v + 1] = w[3 * v + 2] = 1.0f / 3.0f;
    }
    rowptr[N] = 3 * N;
    float *Z = malloc(sizeof(float) * N * D), *S = malloc(sizeof(float) * N * D);
    float *dX = malloc(sizeof(float) * N * D), *Sb = malloc(sizeof(float) * N * D);
    orc_aggregate_fwd(rowptr, col, w, N, x, D, D, Z, D, S, D);
    if (orc_aggregate_bwd(rowptr, col, w, N, N, out, D, D, dX, D, Sb, D) != 0) { puts("bwd"); return 1; }
    /* b-bit round trip */
    for (int bits = 2; bits <= 8; bits *= 2) {
        const int64_t wb = orc_words_per_row_bits(D, bits);
        uint64_t *pw = malloc(sizeof(uint64_t) * N * (size_t)wb);
        orc_quantize_bbit(x, D, D, idx, 0, N, bits, 5u, 1u, 0, pw, scale, zero);
        orc_dequantize_bbit_fwd(pw, scale, zero, N, D, bits, out, D, 0);
        free(pw);
    }
    free(x); free(out); free(J); free(packed); free(Z); free(S); free(dX); free(Sb);
    puts("sanitized oracle ok");
    return 0;
}
"""


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    """Compiles oracle/sylvie_oracle.c with -fsanitize=address,undefined (host only) together
    with a small driver that walks the quantizer, both dequantizers, both aggregations and the
    b-bit round trip on ragged sizes; any out-of-bounds access, leak or undefined operation
    makes the run fail."""
    src = tmp_path / "driver.c"
    src.write_text(DRIVER)
    exe = tmp_path / "driver"
    cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-I", os.path.join(ROOT, "oracle"), "-o", str(exe), str(src), "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, OMP_NUM_THREADS="2",
               ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "sanitized oracle ok" in r.stdout
