/*
 * CPU checker for multi-head self-attention with redundancy skipping.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain float64 statement of
 * what the GPU library must compute.  It is used by the tests, by the smoke
 * check and by the CPU-baseline leg of the benchmark; the product never calls
 * it.  It shares no code, header, table or helper with the GPU path.
 *
 * What it follows (Yu & Fujita, "Parallel Scheduling Self-attention Mechanism"):
 *   Sec. 3.1, Eq. (1)  phase 1:  w'_ij = sum_l q_i[l] * k_j[l]
 *   Sec. 3.1, Eq. (2)  phase 2:  w_ij  = exp(w'_ij) / sum_j exp(w'_ij)
 *   Sec. 3.1, Eq. (3)  phase 3:  y_i   = sum_j w_ij * v_j      (sum over the n vectors)
 *   Sec. 3.1           q, k, v are linear projections of the inputs x; several
 *                      heads are independent sets of projection matrices.
 *   Sec. 4.1, Eq. (4)  q = k = v  =>  w'_ij = w'_ji ; only phase 1 can reuse it.
 *   Sec. 4.2           which of each symmetric pair is computed (diagonal groups),
 *                      and the even-n trade-off that computes one diagonal twice.
 *   Sec. 5.1           masked attention: only the n(n+1)/2 weights with j <= i matter,
 *                      in all three phases; practice writes -inf into the others.
 *
 * The skipping is exact, so the result is the plain definition with a mask.
 * Readings of points the paper leaves open:
 *   - a `scale` factor multiplies w'_ij (scale = 1 is Eq. (1) literally);
 *   - the row maximum is subtracted before exp (same value, no overflow);
 *   - key lengths: pair (i,j) of batch item b is allowed only if j < len[b]
 *     (every query row is still produced); a row with no allowed pair gives zeros;
 *     with `skip_padded_rows` the padded vectors are left out as queries as well:
 *     a pair also needs i < len[b], so rows i >= len[b] are zeros (the paper has no
 *     padding; this is Sec. 5.1's rule, "what is masked is not computed", applied to
 *     both sides of a pair);
 *   - in the q = k = v scheme the shared vectors are z = x.Wq (or x itself when
 *     Wq is NULL and d_model = n_heads * d_k).
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py and
 * tests/test_oracle_counts.py (library special cases, closed forms, hand-worked
 * examples, the cycle counts printed in Tables 1 and 2).  The cycle count of the
 * symmetric schedule (Algorithm 2) is not modelled: parity unpinned, and unused.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_FULL = 0, ORC_SYMMETRIC = 1, ORC_CAUSAL = 2 };
enum { ORC_PLAIN = 0, ORC_NOSKIP = 1, ORC_SKIP = 2 };

typedef struct {
    int32_t batch, n, d_model, n_heads, d_k, p;
    double scale;
    int32_t skip_padded_rows;     /* with key lengths: rows i >= len take part in no pair */
} orc_cfg;

typedef struct {
    uint64_t pairs_full;          /* B*H*n*n, per phase */
    uint64_t pairs_needed[3];     /* fewest pairs each phase must touch */
    uint64_t pairs_scheduled[3];  /* pairs the paper's schedule touches (differs: Sec. 4.2, even n) */
    uint64_t tiles_full;          /* B*H*P*P logical tiles of (n/P) x (n/P) pairs */
    uint64_t tiles_executed;      /* logical tiles holding at least one scheduled pair */
    uint64_t pairs_executed;      /* tiles_executed * (n/P)^2 */
} orc_counts;

static int allowed(int scheme, int i, int j, int len, int rows_too)
{
    if (j >= len) return 0;                        /* key padding */
    if (rows_too && i >= len) return 0;            /* query padding, when asked for */
    if (scheme == ORC_CAUSAL && j > i) return 0;   /* Sec. 5.1: main diagonal and below */
    return 1;
}

/* Sec. 4.2: the computed element of each symmetric pair.  Group g joins the
 * g-th farthest upper diagonal (g elements) with the g-th nearest lower diagonal
 * (n-g elements): together the circulant diagonal (i-j) mod n = g.  Groups
 * 0..h' are computed; for even n the diagonal n/2 is computed in full although
 * it holds both halves of its pairs. */
static int sym_computed(int i, int j, int n)
{
    int g = ((i - j) % n + n) % n;
    return g <= n / 2;
}

/* Sec. 3.1: out[i][l] = sum_c x_i[c] * W[c][h*d_k + l], c ascending. */
static void project_head(const orc_cfg *c, const double *X, const double *W,
                         int b, int h, int row_lo, int row_hi, double *out)
{
    const int D = c->d_model, d = c->d_k, HD = c->n_heads * c->d_k;
#pragma omp parallel for schedule(static)
    for (int i = row_lo; i < row_hi; ++i) {
        const double *x = X + ((size_t)b * c->n + i) * D;
        double *o = out + (size_t)i * d;
        for (int l = 0; l < d; ++l) o[l] = 0.0;
        if (W == NULL) {                           /* z = x (q = k = v scheme without projection) */
            for (int l = 0; l < d; ++l) o[l] = x[h * d + l];
            continue;
        }
        for (int cc = 0; cc < D; ++cc) {
            const double xv = x[cc];
            const double *w = W + (size_t)cc * HD + (size_t)h * d;
            for (int l = 0; l < d; ++l) o[l] += xv * w[l];
        }
    }
}

static double dot(const double *a, const double *b, int d)
{
    double s = 0.0;
    for (int l = 0; l < d; ++l) s += a[l] * b[l];
    return s;
}

/* One output row from its score row s[0..n): Eq. (2) then Eq. (3), j ascending.
 * `use[j]` says whether pair j takes part; entries that do not are never read
 * (PLAIN, SKIP) or are read as -inf (NOSKIP, what practice does, Sec. 5.1). */
static void row_softmax_pv(const double *s, const unsigned char *use, int n, int d,
                           const double *v, int variant, double *y, double *wrow)
{
    double M = -INFINITY;
    for (int j = 0; j < n; ++j)
        if (use[j] && s[j] > M) M = s[j];
    for (int l = 0; l < d; ++l) y[l] = 0.0;
    if (wrow) for (int j = 0; j < n; ++j) wrow[j] = 0.0;
    if (M == -INFINITY) return;                    /* no allowed pair: zeros */
    double L = 0.0;
    for (int j = 0; j < n; ++j) {
        if (use[j]) L += exp(s[j] - M);
        else if (variant == ORC_NOSKIP) L += exp(-INFINITY - M);
    }
    for (int j = 0; j < n; ++j) {
        double w;
        if (use[j]) w = exp(s[j] - M) / L;
        else if (variant == ORC_NOSKIP) w = exp(-INFINITY - M) / L;
        else continue;
        if (wrow) wrow[j] = w;
        const double *vj = v + (size_t)j * d;
        for (int l = 0; l < d; ++l) y[l] += w * vj[l];
    }
}

static int check_cfg(const orc_cfg *c, int scheme, const int32_t *lens)
{
    if (!c) return 1;
    if (c->batch < 0 || c->n < 0 || c->d_model <= 0 || c->n_heads <= 0 || c->d_k <= 0 || c->p <= 0) return 1;
    if (scheme < 0 || scheme > 2) return 1;
    if (c->n % c->p != 0) return 2;                /* abstract: n divisible by the number of PEs */
    if (scheme == ORC_SYMMETRIC && lens) return 3;
    return 0;
}

/*
 * Whole forward pass.  Host pointers, row-major:
 *   X [B][n][D], Wq/Wk/Wv [D][H*d_k], lens [B] or NULL, out [B][n][H*d_k],
 *   weights (optional) [B][H][n][n] receives w_ij (0 where not allowed).
 * variant: ORC_PLAIN  the definition, touching allowed pairs only;
 *          ORC_NOSKIP every pair computed, disallowed ones set to -inf afterwards;
 *          ORC_SKIP   disallowed pairs never touched and, for q = k = v, only the
 *                     selected element of each symmetric pair computed, the other copied.
 * Returns 0, or 1 bad argument, 2 n not divisible by p, 3 unsupported, 4 no memory.
 */
int attn_oracle_forward(const orc_cfg *c, const double *X, const double *Wq, const double *Wk,
                        const double *Wv, int scheme, const int32_t *lens, int variant,
                        double *out, double *weights)
{
    int rc = check_cfg(c, scheme, lens);
    if (rc) return rc;
    if (!X || !out) return 1;
    if (scheme != ORC_SYMMETRIC && (!Wq || !Wk || !Wv)) return 1;
    const int n = c->n, d = c->d_k, H = c->n_heads, HD = H * d;
    if (scheme == ORC_SYMMETRIC && !Wq && c->d_model != HD) return 1;
    if (n == 0 || c->batch == 0) return 0;

    double *q = malloc(sizeof(double) * (size_t)n * d);
    double *k = malloc(sizeof(double) * (size_t)n * d);
    double *v = malloc(sizeof(double) * (size_t)n * d);
    double *S = NULL;                              /* full score matrix, q = k = v variants only */
    if (scheme == ORC_SYMMETRIC) S = malloc(sizeof(double) * (size_t)n * n);
    if (!q || !k || !v || (scheme == ORC_SYMMETRIC && !S)) { free(q); free(k); free(v); free(S); return 4; }

    for (int b = 0; b < c->batch; ++b) {
        const int len = lens ? (lens[b] < n ? lens[b] : n) : n;
        for (int h = 0; h < H; ++h) {
            project_head(c, X, Wq, b, h, 0, n, q);
            if (scheme == ORC_SYMMETRIC) {
                memcpy(k, q, sizeof(double) * (size_t)n * d);
                memcpy(v, q, sizeof(double) * (size_t)n * d);
            } else {
                project_head(c, X, Wk, b, h, 0, n, k);
                project_head(c, X, Wv, b, h, 0, n, v);
            }
            if (scheme == ORC_SYMMETRIC && variant == ORC_SKIP) {
                /* Sec. 4.1: compute one of (w'_ij, w'_ji), reuse it as the other. */
#pragma omp parallel for schedule(static)
                for (int i = 0; i < n; ++i)
                    for (int j = 0; j < n; ++j)
                        if (sym_computed(i, j, n))
                            S[(size_t)i * n + j] = c->scale * dot(q + (size_t)i * d, k + (size_t)j * d, d);
#pragma omp parallel for schedule(static)
                for (int i = 0; i < n; ++i)
                    for (int j = 0; j < n; ++j)
                        if (!sym_computed(i, j, n))
                            S[(size_t)i * n + j] = S[(size_t)j * n + i];
            }
#pragma omp parallel
            {
                double *s = malloc(sizeof(double) * (size_t)n);
                unsigned char *use = malloc((size_t)n);
                double *y = malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 4)
                for (int i = 0; i < n; ++i) {
                    for (int j = 0; j < n; ++j) {
                        use[j] = (unsigned char)allowed(scheme, i, j, len, c->skip_padded_rows);
                        if (scheme == ORC_SYMMETRIC && variant == ORC_SKIP)
                            s[j] = S[(size_t)i * n + j];
                        else if (use[j] || variant == ORC_NOSKIP)
                            s[j] = c->scale * dot(q + (size_t)i * d, k + (size_t)j * d, d);  /* Eq. (1) */
                        else
                            s[j] = 0.0;            /* never read */
                    }
                    double *wrow = weights ? weights + (((size_t)b * H + h) * n + i) * n : NULL;
                    row_softmax_pv(s, use, n, d, v, variant, y, wrow);
                    double *o = out + ((size_t)b * n + i) * HD + (size_t)h * d;
                    for (int l = 0; l < d; ++l) o[l] = y[l];
                }
                free(s); free(use); free(y);
            }
        }
    }
    free(q); free(k); free(v); free(S);
    return 0;
}

/*
 * Selected output rows of one (batch item, head): rows[r] in [0,n), out [nrows][d_k].
 * Same definition as attn_oracle_forward (PLAIN); lets a large workload be checked
 * on sampled rows.  K and V of the head are projected in full, q only where needed.
 */
int attn_oracle_head_rows(const orc_cfg *c, const double *X, const double *Wq, const double *Wk,
                          const double *Wv, int scheme, const int32_t *lens, int b, int h,
                          int nrows, const int32_t *rows, double *out)
{
    int rc = check_cfg(c, scheme, lens);
    if (rc) return rc;
    if (!X || !out || !rows || nrows < 0) return 1;
    if (b < 0 || b >= c->batch || h < 0 || h >= c->n_heads) return 1;
    if (scheme != ORC_SYMMETRIC && (!Wq || !Wk || !Wv)) return 1;
    const int n = c->n, d = c->d_k;
    if (scheme == ORC_SYMMETRIC && !Wq && c->d_model != c->n_heads * d) return 1;
    for (int r = 0; r < nrows; ++r) if (rows[r] < 0 || rows[r] >= n) return 1;
    const int len = lens ? (lens[b] < n ? lens[b] : n) : n;

    double *q = malloc(sizeof(double) * (size_t)n * d);
    double *k = malloc(sizeof(double) * (size_t)n * d);
    double *v = malloc(sizeof(double) * (size_t)n * d);
    if (!q || !k || !v) { free(q); free(k); free(v); return 4; }
    if (scheme == ORC_SYMMETRIC) {
        project_head(c, X, Wq, b, h, 0, n, q);
        memcpy(k, q, sizeof(double) * (size_t)n * d);
        memcpy(v, q, sizeof(double) * (size_t)n * d);
    } else {
        for (int r = 0; r < nrows; ++r) project_head(c, X, Wq, b, h, rows[r], rows[r] + 1, q);
        project_head(c, X, Wk, b, h, 0, n, k);
        project_head(c, X, Wv, b, h, 0, n, v);
    }
#pragma omp parallel
    {
        double *s = malloc(sizeof(double) * (size_t)n);
        unsigned char *use = malloc((size_t)n);
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < nrows; ++r) {
            const int i = rows[r];
            for (int j = 0; j < n; ++j) {
                use[j] = (unsigned char)allowed(scheme, i, j, len, c->skip_padded_rows);
                s[j] = use[j] ? c->scale * dot(q + (size_t)i * d, k + (size_t)j * d, d) : 0.0;
            }
            row_softmax_pv(s, use, n, d, v, ORC_PLAIN, out + (size_t)r * d, NULL);
        }
        free(s); free(use);
    }
    free(q); free(k); free(v);
    return 0;
}

/*
 * Pair and tile counts, by enumerating the predicate (no closed form is used
 * here; the tests compare the result with the paper's closed forms).
 *   needed    : fewest pairs per phase.  FULL n^2 each (Sec. 3.2).  q = k = v:
 *               phase 1 one per unordered pair, phases 2 and 3 all (Sec. 4.1).
 *               Masked: allowed pairs in every phase (Sec. 5.1).
 *   scheduled : pairs the paper's schedule computes; differs only for q = k = v with
 *               even n, where the middle diagonal is computed in full (Sec. 4.2).
 *   tiles     : the same rules applied to the P x P matrix of (n/P)-square tiles; a
 *               tile is executed if it holds at least one scheduled pair (FULL,
 *               masked) or is selected by the diagonal-group rule on tiles (q = k = v).
 */
int attn_oracle_counts(const orc_cfg *c, int scheme, const int32_t *lens, orc_counts *out)
{
    int rc = check_cfg(c, scheme, lens);
    if (rc) return rc;
    if (!out) return 1;
    memset(out, 0, sizeof(*out));
    const int n = c->n, P = c->p, H = c->n_heads;
    const int bsz = n / P;
    unsigned char *tile = malloc((size_t)P * P);
    if (!tile) return 4;
    for (int b = 0; b < c->batch; ++b) {
        const int len = lens ? (lens[b] < n ? lens[b] : n) : n;
        uint64_t need[3] = {0, 0, 0}, sched[3] = {0, 0, 0}, tiles = 0;
        memset(tile, 0, (size_t)P * P);
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                if (!allowed(scheme, i, j, len, c->skip_padded_rows)) continue;
                if (scheme == ORC_SYMMETRIC) {
                    if (i >= j) need[0]++;          /* one per unordered pair */
                    if (sym_computed(i, j, n)) sched[0]++;
                } else {
                    need[0]++; sched[0]++;
                    tile[(size_t)(i / bsz) * P + j / bsz] = 1;
                }
                need[1]++; need[2]++; sched[1]++; sched[2]++;
            }
        for (int I = 0; I < P; ++I)
            for (int J = 0; J < P; ++J) {
                if (scheme == ORC_SYMMETRIC) tiles += (uint64_t)sym_computed(I, J, P);
                else tiles += tile[(size_t)I * P + J];
            }
        for (int ph = 0; ph < 3; ++ph) {
            out->pairs_needed[ph] += need[ph] * (uint64_t)H;
            out->pairs_scheduled[ph] += sched[ph] * (uint64_t)H;
        }
        out->tiles_executed += tiles * (uint64_t)H;
        out->pairs_full += (uint64_t)n * n * H;
        out->tiles_full += (uint64_t)P * P * H;
    }
    out->pairs_executed = out->tiles_executed * (uint64_t)bsz * bsz;
    free(tile);
    return 0;
}

/*
 * Cycle count of the paper's ring schedules with n = d vectors on m PEs: the
 * number of iterations of the loops around the parallel `for all PEs` body,
 * every phase included (phase 2 is two passes: accumulate, then divide).
 *   algo 1 (Algorithm 1): phases 1 and 3 run n rows, each (n/m)*n cycles.
 *   algo 3 (Algorithm 3): phases 1 and 3 run the row groups h = 0..h' (row n-h packed
 *          with row h, Sec. 5.2) plus, for even n, one more stage for row n/2; phase 2
 *          keeps all n*n slots (the accepted ~50% utilisation).
 * Returns -1 for arguments outside the model (m must divide n; algo 2 is not modelled).
 */
int64_t attn_oracle_ring_cycles(int n, int m, int algo)
{
    if (n <= 0 || m <= 0 || n % m != 0) return -1;
    int64_t stage = (int64_t)(n / m) * n;          /* loops i in [1,n/m], j in [1,n] */
    int64_t cycles = 0;
    if (algo == 1) {
        for (int h = 1; h <= n; ++h) cycles += stage;          /* phase 1 */
        cycles += stage + stage;                                /* phase 2, two passes */
        for (int h = 1; h <= n; ++h) cycles += stage;          /* phase 3 */
        return cycles;
    }
    if (algo == 3) {
        int hp = (n % 2) ? (n - 1) / 2 : n / 2 - 1;
        for (int ph = 0; ph < 2; ++ph) {                        /* phases 1 and 3 */
            for (int h = 0; h <= hp; ++h) cycles += stage;
            if (n % 2 == 0) cycles += stage;                    /* row n/2 alone */
        }
        cycles += stage + stage;                                /* phase 2 */
        return cycles;
    }
    return -1;
}

int attn_oracle_num_threads(void)
{
    int t = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        t = omp_get_num_threads();
    }
#endif
    return t;
}
