/* Host-logic fuzz of the C ABI without a GPU: random (including absurd) sizes through the configuration
 * chooser and the workspace queries, random configuration specs through the spec parser, random text
 * through the tune-cache reader.  Every call must return (a status, not a crash); built by the test
 * suite against the in-tree library, and by hand with the address and undefined-behaviour sanitizers. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "tgemm.h"
static unsigned long long st = 88172645463325252ull;
static unsigned long long rnd(void) { st ^= st << 13; st ^= st >> 7; st ^= st << 17; return st; }
int main(void) {
    char buf[256];
    static const long long dims[] = {0, 1, 3, 4, 7, 16, 31, 32, 33, 63, 64, 65, 100, 127, 128, 129, 255, 256, 257, 1000, 1024, 1536, 4000, 4096, 8192, 65536, 2147483647LL, 2147483648LL, -1};
    const int nd = sizeof dims / sizeof dims[0];
    long ok = 0, bad = 0;
    for (int i = 0; i < 40000; ++i) {
        long long b = dims[rnd() % nd], m = dims[rnd() % nd], n = dims[rnd() % nd], k = dims[rnd() % nd];
        if (rnd() % 4) b = 1;
        /* both math modes, with and without a (never dereferenced) workspace: split-K, tail splits and the
           cut-ahead piece kernels only become candidates with one */
        if (i % 1000 == 0) {
            (void)tg_set_math((i / 1000) % 2 ? TG_MATH_BF16_PIECES : TG_MATH_FP32_MFMA);
            (void)tg_set_workspace((i / 2000) % 2 ? (void *)0x10000 : NULL, (i / 2000) % 2 ? ((size_t)1 << (20 + (i / 4000) % 16)) : 0);
        }
        tg_status s = tg_get_config(b, m, n, k, buf, sizeof buf);
        if (s == TG_OK) ++ok; else ++bad;
        (void)tg_workspace_bytes(b, m, n, k);
        (void)tg_strided_workspace_bytes(m, n, k, (long long)(rnd() % 5), (long long)(rnd() % 5));
        if (i % 16 == 0) {
            double lb, model;
            const int count = tg_num_candidates(b, m, n, k);
            if (count > 0) (void)tg_candidate(b, m, n, k, (int)(rnd() % (unsigned)count), buf, sizeof buf, &lb, &model);
        }
    }
    (void)tg_set_math(TG_MATH_FP32_MFMA);
    /* spec grammar */
    const char *pieces[] = {"t128x128x16_w64x64", "d64x64x32_w32x32", "wave32", "p128x128x16_w64x64", "nope", "", ":", ":s", ":s4", ":g0", ":g8", ":o17", ":o2", ":p3", ":p99", ":x1", ":s99999999999", "::", ":s-1", ":s4:s2",
                            ":t1x2", ":t3x6", ":t0x2", ":t2x1", ":t9999x9999", ":tx", ":t3x", ":t3x6x2", "e128x256x32_w64x128_x6", "c128x256x32_w64x128_x9"};
    const int np = sizeof pieces / sizeof pieces[0];
    for (int i = 0; i < 20000; ++i) {
        char spec[256] = "";
        int parts = 1 + rnd() % 4;
        for (int j = 0; j < parts; ++j) strncat(spec, pieces[rnd() % np], sizeof spec - strlen(spec) - 1);
        tg_status s = tg_force_config(spec);
        if (s == TG_OK) {
            (void)tg_get_config(1, 1024, 1024, 1024, buf, sizeof buf);
            (void)tg_get_config(1 + (long long)(rnd() % 3), 3072, 3072, 3072, buf, sizeof buf);
            (void)tg_get_config(1, 1 + (long long)(rnd() % 300), 4 * (1 + (long long)(rnd() % 100)), 1 + (long long)(rnd() % 3000), buf, sizeof buf);
        }
    }
    tg_force_config(NULL);
    (void)tg_set_workspace(NULL, 0);
    /* cache files */
    const char *path = "tg_fuzz_cache.txt";
    for (int i = 0; i < 300; ++i) {
        FILE *f = fopen(path, "w");
        if (!f) return 2;
        const int ver = 3 + (int)(rnd() % 2);
        if (rnd() % 8) fprintf(f, "tgemm-tune-cache %d gfx950\n", ver); else fprintf(f, "garbage %llu\n", rnd());
        int lines = rnd() % 6;
        for (int j = 0; j < lines; ++j) {
            switch (rnd() % 4) {
                case 0: fprintf(f, "1 1024 1024 1024 1 t128x128x16_w64x64 1 4 0 0 20.5\n"); break;
                case 1: fprintf(f, "%lld %lld %lld %lld %d %s %d %d %d %d %f\n", (long long)rnd() % 9, (long long)rnd() % 5000, (long long)rnd() % 5000, (long long)rnd() % 5000,
                                (int)(rnd() % 4), pieces[rnd() % 5], (int)(rnd() % 40) - 4, (int)(rnd() % 40) - 4, (int)(rnd() % 20) - 2, (int)(rnd() % 20) - 2, 1.0); break;
                case 2: fprintf(f, "1 3072 3072 3072 %d t128x256x32_w64x128_acc2 1 8 0 0 %d %d 440.0\n", (int)(rnd() % 8), (int)(rnd() % 30) - 2, (int)(rnd() % 20) - 2); break;
                default: fprintf(f, "%0200llu x y z\n", rnd()); break;
            }
        }
        fclose(f);
        (void)tg_load_tune_cache(path);
        (void)tg_get_config(1, 1024, 1024, 1024, buf, sizeof buf);
        (void)tg_set_workspace(i % 2 ? (void *)0x10000 : NULL, i % 2 ? (size_t)1 << 30 : 0);
        (void)tg_get_config(1, 3072, 3072, 3072, buf, sizeof buf);
        if (i % 50 == 0) { (void)tg_save_tune_cache("tg_fuzz_saved.txt"); tg_clear_tune_cache(); }
    }
    tg_clear_tune_cache();
    (void)tg_set_workspace(NULL, 0);
    printf("fuzz: ok (%ld configs chosen, %ld rejected)\n", ok, bad);
    return 0;
}
