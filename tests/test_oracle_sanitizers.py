"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the C source is built a second time
with -fsanitize=address,undefined into a small program of its own, which runs the hand-worked two-sub-quantiser
example and one small end-to-end search (train, encode, list building order, search, brute force) and exits
non-zero on any report."""
import os
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = textwrap.dedent(r"""
    #include <stdint.h>
    #include <stdio.h>
    #include <stdlib.h>
    #include <string.h>
    void oracle_assign(const float*, int64_t, int, int64_t, const float*, int64_t, int32_t*, float*);
    void oracle_assign_among(const float*, int64_t, int, int64_t, const float*, const int32_t*, int, int32_t*, float*);
    void oracle_kmeans(const float*, int64_t, int, int64_t, int64_t, int, const int64_t*, float*, double*);
    void oracle_encode(const float*, int64_t, int, const float*, int64_t, const float*, int, int, int32_t*, uint8_t*);
    void oracle_lut(const float*, int64_t, int, const float*, int, int, float*);
    void oracle_search(const float*, int64_t, int, const float*, int64_t, const float*, int, int, const int64_t*,
                       const uint8_t*, const int64_t*, int, int, float*, int64_t*, int32_t*, int64_t*);
    void oracle_brute_force_knn(const float*, int64_t, int, const float*, int64_t, int, float*, int64_t*);
    void oracle_decode(const uint8_t*, int64_t, const float*, int, int, int, float*);

    static unsigned long long state = 88172645463325252ull;
    static float rnd(void) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return (float)((state >> 11) % 2001) / 1000.f - 1.f; }

    int main(void) {
        /* the worked example: d = 4, M = 2, four centres per sub-quantiser */
        const float pq2[2 * 4 * 2] = {0, 0, 1, 1, 3, 2, -2, 2, 0, 0, 0, -1, 2, -1, 3, 1};
        const float q2[4] = {1, 2, 0, -1};
        float lut2[8];
        oracle_lut(q2, 1, 4, pq2, 2, 4, lut2);
        const float want[8] = {5, 1, 4, 9, 1, 0, 4, 13};
        for (int i = 0; i < 8; ++i) if (lut2[i] != want[i]) { printf("table entry %d: %g\n", i, lut2[i]); return 2; }
        /* a small index end to end */
        enum { N = 600, D = 8, NLIST = 7, M = 4, KSUB = 256, NQ = 5, K = 6, NPROBE = 3 };
        float *x = malloc(sizeof(float) * N * D), *q = malloc(sizeof(float) * NQ * D);
        for (int i = 0; i < N * D; ++i) x[i] = rnd();
        for (int i = 0; i < NQ * D; ++i) q[i] = rnd();
        int64_t init[KSUB];
        for (int i = 0; i < KSUB; ++i) init[i] = (int64_t)i * 2;
        float *coarse = malloc(sizeof(float) * NLIST * D), *pq = malloc(sizeof(float) * M * KSUB * (D / M));
        double inertia[3];
        oracle_kmeans(x, N, D, D, NLIST, 3, init, coarse, inertia);
        for (int m = 0; m < M; ++m) oracle_kmeans(x + m * (D / M), N, D / M, D, KSUB, 2, init, pq + m * KSUB * (D / M), NULL);
        int32_t *lists = malloc(sizeof(int32_t) * N);
        uint8_t *codes = malloc((size_t)N * M);
        oracle_encode(x, N, D, coarse, NLIST, pq, M, KSUB, lists, codes);
        /* group into lists (ascending id inside a list) */
        int64_t off[NLIST + 1] = {0}, fill[NLIST] = {0};
        for (int i = 0; i < N; ++i) off[lists[i] + 1]++;
        for (int l = 0; l < NLIST; ++l) off[l + 1] += off[l];
        uint8_t *lc = malloc((size_t)N * M);
        int64_t *ids = malloc(sizeof(int64_t) * N);
        for (int i = 0; i < N; ++i) { const int64_t p = off[lists[i]] + fill[lists[i]]++; memcpy(lc + p * M, codes + (size_t)i * M, M); ids[p] = i; }
        float od[NQ * K]; int64_t oi[NQ * K]; int32_t probes[NQ * NPROBE]; int64_t scanned[NQ];
        oracle_search(q, NQ, D, coarse, NLIST, pq, M, KSUB, off, lc, ids, NPROBE, K, od, oi, probes, scanned);
        for (int i = 0; i < NQ * K; ++i) if (oi[i] < -1 || oi[i] >= N) { printf("id out of range\n"); return 3; }
        float bd[NQ * K]; int64_t bi[NQ * K];
        oracle_brute_force_knn(x, N, D, q, NQ, K, bd, bi);
        int32_t cand[N * 2], among[N];
        for (int i = 0; i < N; ++i) { cand[2 * i] = lists[i]; cand[2 * i + 1] = (lists[i] + 1) % NLIST; }
        oracle_assign_among(x, N, D, D, coarse, cand, 2, among, NULL);
        for (int i = 0; i < N; ++i) if (among[i] != lists[i]) { printf("restricted assignment differs at row %d\n", i); return 4; }
        float *dec = malloc(sizeof(float) * N * D);
        oracle_decode(lc, N, pq, M, KSUB, D / M, dec);
        free(x); free(q); free(coarse); free(pq); free(lists); free(codes); free(lc); free(ids); free(dec);
        printf("sanitized oracle run ok\n");
        return 0;
    }
""")


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    src = os.path.join(ROOT, "oracle", "ivfpq_oracle.c")
    drv = tmp_path / "driver.c"
    drv.write_text(DRIVER)
    exe = tmp_path / "oracle_san"
    cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fopenmp", "-o", str(exe), str(drv), src, "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "asan" in (built.stderr or "").lower() and "cannot find" in built.stderr.lower():
        pytest.skip("the sanitizer runtime is not installed")
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    env.pop("LD_PRELOAD", None)
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "sanitized oracle run ok" in run.stdout
