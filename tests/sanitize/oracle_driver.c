/* Host-only driver for the sanitizer build of the C oracle: reads one case written by
 * tests/test_sanitizers.py (sizes, block table, kv_lens, then q / K / V as raw 16-bit patterns),
 * runs the oracle on every request and prints a checksum. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int pat_oracle_decode_attention(int B, int Hq, int Hkv, int d, int P, int dtype, const int32_t *bt,
                                int W, const int32_t *kv_lens, int num_pages, const uint16_t *q,
                                const uint16_t *k, const uint16_t *v, int64_t sp, int64_t st,
                                int64_t sh, double scale, const int32_t *req_ids, int n_out,
                                double *out, double *lse, int nthreads);

int main(int argc, char **argv)
{
    if (argc != 2) return 2;
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 2;
    int32_t h[12];
    if (fread(h, 4, 12, f) != 12) return 2;
    const int B = h[0], W = h[1], P = h[2], pages = h[3], Hq = h[4], Hkv = h[5], d = h[6], dtype = h[7];
    const int64_t sp = h[8], st = h[9], sh = h[10];
    const int want_rc = h[11];
    int32_t *bt = malloc(sizeof(int32_t) * (size_t)B * W), *kv = malloc(sizeof(int32_t) * (size_t)B);
    const size_t pool = (size_t)pages * P * Hkv * d, nq = (size_t)B * Hq * d;
    uint16_t *q = malloc(2 * nq), *k = malloc(2 * pool), *v = malloc(2 * pool);
    if (fread(bt, 4, (size_t)B * W, f) != (size_t)B * W || fread(kv, 4, B, f) != (size_t)B ||
        fread(q, 2, nq, f) != nq || fread(k, 2, pool, f) != pool || fread(v, 2, pool, f) != pool)
        return 2;
    fclose(f);
    double *out = malloc(sizeof(double) * nq), *lse = malloc(sizeof(double) * (size_t)B * Hq);
    const int rc = pat_oracle_decode_attention(B, Hq, Hkv, d, P, dtype, bt, W, kv, pages, q, k, v, sp, st,
                                               sh, 0.088388347648318, NULL, B, out, lse, 2);
    if (rc != want_rc) { fprintf(stderr, "oracle rc %d, expected %d\n", rc, want_rc); return 1; }
    double s = 0;
    if (rc == 0) for (size_t i = 0; i < nq; ++i) s += out[i];
    printf("ok %.6f\n", s);
    free(bt); free(kv); free(q); free(k); free(v); free(out); free(lse);
    return 0;
}
