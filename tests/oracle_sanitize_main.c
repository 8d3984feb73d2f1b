/*
 * Driver for a sanitised build of the CPU checker (test infrastructure only).
 * tests/test_oracle_sanitized.py compiles this file, which includes the checker's one
 * source file, with -fsanitize=address,undefined and runs it: every exported function is
 * called on small shapes that reach its edge cases (partitions of one row, odd and even n,
 * key lengths 0, past n and negative, padded rows left out, single rows of one head, empty
 * batch).  Any report of the sanitisers ends the run with a non-zero status.  The checksum
 * it prints must equal that of the same driver built without sanitisers.
 */
#include <stdio.h>

#include "../oracle/attn_oracle.c"

static uint64_t lcg_state = 0x9E3779B97F4A7C15ull;
static double next_unit(void)
{
    lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(lcg_state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}
static uint64_t fnv(uint64_t h, const void *p, size_t bytes)
{
    const unsigned char *c = p;
    for (size_t i = 0; i < bytes; ++i) { h ^= c[i]; h *= 1099511628211ull; }
    return h;
}

int main(void)
{
    uint64_t h = 1469598103934665603ull;
    const int shapes[][6] = { /* batch, n, d_model, heads, d_k, p */
        {1, 7, 5, 1, 3, 7}, {2, 12, 6, 2, 5, 3}, {3, 16, 8, 2, 4, 4}, {1, 9, 9, 3, 3, 1}, {0, 4, 4, 1, 4, 2}};
    for (size_t s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s) {
        orc_cfg c = {shapes[s][0], shapes[s][1], shapes[s][2], shapes[s][3], shapes[s][4], shapes[s][5], 0.37, 0};
        const int B = c.batch, n = c.n, D = c.d_model, HD = c.n_heads * c.d_k;
        double *X = malloc(sizeof(double) * (size_t)(B * n * D + 1));
        double *W[3];
        for (int i = 0; i < B * n * D; ++i) X[i] = next_unit();
        for (int m = 0; m < 3; ++m) {
            W[m] = malloc(sizeof(double) * (size_t)D * HD);
            for (int i = 0; i < D * HD; ++i) W[m][i] = next_unit() * 0.5;
        }
        double *out = malloc(sizeof(double) * (size_t)(B * n * HD + 1));
        double *wts = malloc(sizeof(double) * (size_t)(B * c.n_heads * n * n + 1));
        int32_t lens[3] = {0, n + 5, -2};
        if (n > 2) lens[2] = n / 2 + 1;
        for (int scheme = 0; scheme < 3; ++scheme)
            for (int variant = 0; variant < 3; ++variant)
                for (int with_lens = 0; with_lens < 2; ++with_lens)
                    for (int rows_too = 0; rows_too < 2; ++rows_too) {
                        c.skip_padded_rows = rows_too;
                        const int32_t *lp = with_lens ? lens : NULL;
                        int rc = attn_oracle_forward(&c, X, W[0], W[1], W[2], scheme, lp, variant, out, wts);
                        h = fnv(h, &rc, sizeof(rc));
                        if (rc == 0) {
                            h = fnv(h, out, sizeof(double) * (size_t)(B * n * HD));
                            h = fnv(h, wts, sizeof(double) * (size_t)(B * c.n_heads * n * n));
                        }
                        orc_counts cnt;
                        rc = attn_oracle_counts(&c, scheme, lp, &cnt);
                        h = fnv(h, &rc, sizeof(rc));
                        if (rc == 0) h = fnv(h, &cnt.tiles_executed, sizeof(cnt.tiles_executed));
                        if (B > 0) {
                            int32_t rows[3] = {0, n - 1, n / 2};
                            double hr[3 * 8];
                            rc = attn_oracle_head_rows(&c, X, W[0], W[1], W[2], scheme, lp, B - 1, c.n_heads - 1, 3,
                                                       rows, hr);
                            h = fnv(h, &rc, sizeof(rc));
                            if (rc == 0) h = fnv(h, hr, sizeof(double) * 3 * (size_t)c.d_k);
                        }
                    }
        /* q = k = v on the unprojected inputs (needs d_model = heads * d_k) */
        if (D == HD) {
            int rc = attn_oracle_forward(&c, X, NULL, NULL, NULL, ORC_SYMMETRIC, NULL, ORC_SKIP, out, NULL);
            h = fnv(h, &rc, sizeof(rc));
            if (rc == 0) h = fnv(h, out, sizeof(double) * (size_t)(B * n * HD));
        }
        /* argument errors must come back as codes */
        c.p = n > 1 ? n - 1 : 2;
        int rc = attn_oracle_forward(&c, X, W[0], W[1], W[2], ORC_FULL, NULL, ORC_PLAIN, out, NULL);
        h = fnv(h, &rc, sizeof(rc));
        rc = attn_oracle_forward(NULL, X, W[0], W[1], W[2], ORC_FULL, NULL, ORC_PLAIN, out, NULL);
        h = fnv(h, &rc, sizeof(rc));
        free(X); free(out); free(wts);
        for (int m = 0; m < 3; ++m) free(W[m]);
    }
    for (int n = 1; n <= 17; ++n)
        for (int m = 1; m <= n; ++m)
            for (int algo = 0; algo <= 3; ++algo) {
                int64_t cy = attn_oracle_ring_cycles(n, m, algo);
                h = fnv(h, &cy, sizeof(cy));
            }
    int t = attn_oracle_num_threads();
    printf("threads %d\nchecksum %016llx\n", t, (unsigned long long)h);
    return 0;
}
