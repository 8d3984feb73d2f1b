/*
 * attnring - multi-head self-attention with redundant-computation skipping
 * for AMD MI355X (gfx950).  C ABI of libattnring.so.
 *
 * The library computes, for every batch item and head (Yu & Fujita, "Parallel
 * Scheduling Self-attention Mechanism: Generalization and Optimization"):
 *
 *     q_i = x_i.Wq,  k_j = x_j.Wk,  v_j = x_j.Wv            (Sec. 3.1, projections)
 *     w'_ij = scale * sum_l q_i[l] k_j[l]                    (Sec. 3.1, Eq. (1), phase 1)
 *     w_ij  = exp(w'_ij) / sum_j exp(w'_ij)                  (Sec. 3.1, Eq. (2), phase 2)
 *     y_i   = sum_j w_ij v_j                                 (Sec. 3.1, Eq. (3), phase 3)
 *
 * and never computes the pairs (i,j) that the chosen application scheme makes
 * irrelevant to y: for masked self-attention the pairs above the main diagonal,
 * in all three phases (Sec. 5.1); for q = k = v one element of every symmetric
 * pair of phase 1 (Sec. 4.1, Eq. (4); selection rule of Sec. 4.2).  Each
 * workgroup plays one or more of the paper's ring PEs: a PE owns n/P query
 * vectors (the abstract requires n divisible by P) and meets the key/value
 * blocks in ring order, own block first.
 *
 * Conventions
 *   - Every function returns attn_status (except attn_last_error, attn_destroy).
 *     No exception crosses the boundary; nothing is printed.
 *   - X, Wq, Wk, Wv, out and the key-length array are DEVICE pointers on the
 *     HIP device that was current at attn_init.  The caller owns them; they must
 *     stay valid until the stream has finished the call.  The library owns the
 *     context and its workspace (projected q, k, v, counters).
 *   - Layout, all row-major and dense: X [batch][n][d_model]; Wq, Wk, Wv
 *     [d_model][n_heads*d_k] (q = x.W, head h uses columns h*d_k ..); out
 *     [batch][n][n_heads*d_k]; elements are float or bfloat16 per cfg.dtype;
 *     accumulation is always float.
 *   - attn_forward only enqueues work on the given stream and does not wait for it, with one
 *     exception: the first call on a context that needs a workspace attn_init did not allocate
 *     allocates it with hipMalloc, which synchronises the device.  That is the float workspace when
 *     a context whose shape fits the matrix-core kernels is given unaligned pointers, and the
 *     workspace of ATTN_SCHEME_SYMMETRIC (score matrix on the float path, partial row states on the
 *     matrix-core path).  Every later call with the same kind of work only enqueues.
 *     One context serves one call at a time (calls on it are ordered by the caller).
 *   - bfloat16 storage: the matrix-core kernels (d_k 64 or 128, d_model a multiple of 8) contract
 *     bfloat16 operands in the projection and keep the projected q, k, v and the exponentials in half
 *     precision (same matrix-core rate, three more significand bits; values beyond its range
 *     saturate), with float accumulation throughout; out is rounded once to bfloat16.
 */
#ifndef ATTNRING_H
#define ATTNRING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct attn_ctx attn_ctx; /* opaque, owned by the library */

typedef enum {
    ATTN_OK = 0,
    ATTN_ERR_INVALID = 1,     /* NULL pointer, unknown enum value, non-positive size */
    ATTN_ERR_SHAPE = 2,       /* n not divisible by p; sizes that overflow 32-bit indices */
    ATTN_ERR_UNSUPPORTED = 3, /* combination the library does not implement (see attn_init) */
    ATTN_ERR_ALLOC = 4,       /* device or host allocation failed */
    ATTN_ERR_DEVICE = 5       /* a HIP call failed; text in attn_last_error */
} attn_status;

typedef enum {
    ATTN_SCHEME_FULL = 0,      /* original definition: every pair (Sec. 3, Algorithm 1) */
    ATTN_SCHEME_SYMMETRIC = 1, /* q = k = v: phase-1 symmetric reuse (Sec. 4, Algorithm 2) */
    ATTN_SCHEME_CAUSAL = 2     /* masked: pairs j <= i only, all phases (Sec. 5, Algorithm 3) */
} attn_scheme;

typedef enum { ATTN_F32 = 0, ATTN_BF16 = 1 } attn_dtype;

/* Debug flag: same kernels, but every tile is visited and redundant pairs are
 * given weight zero by writing -inf into their scores (the practice Sec. 5.1
 * describes).  Outputs must equal those of the skipping run bit for bit. */
enum { ATTN_FLAG_NO_SKIP = 1u,
       /* Workgroup shape of the bf16 matrix-core path for d_k = 64, normally 128 query rows
        * (4 wavefronts): WIDE asks for 256 rows (8 wavefronts), NARROW for 128.  d_k = 128
        * always takes 256 rows.  Results obey the same bars. */
       ATTN_FLAG_WIDE_TILES = 2u,
       ATTN_FLAG_NARROW_TILES = 4u,
       /* With key lengths: the padded vectors are left out as queries too.  A pair (i, j) of
        * batch item b then also needs i < len[b]; rows i >= len[b] of `out` are written as zeros,
        * their q rows are not projected, and the counts are those of the len x len problems.
        * (Sec. 5.1's rule - what is masked is not computed - applied to both sides of a pair.)
        * No effect without key lengths. */
       ATTN_FLAG_SKIP_PADDED_ROWS = 8u,
       /* Matrix-core path: the query vectors are projected inside the attention kernel, by each
        * wavefront for its own rows, and never leave the registers; the projection kernel computes
        * k and v only.  (Sec. 3.1 / 4.1: the inputs of a row block are loaded once and used for all
        * phases.)  Needs d_model a multiple of 64 and 16-byte aligned weights, else it has no effect;
        * no effect on ATTN_SCHEME_SYMMETRIC and on the float path.  Results obey the same bars. */
       ATTN_FLAG_FUSE_Q_PROJECTION = 16u };

typedef struct {
    int32_t batch;     /* >= 1 */
    int32_t n;         /* vectors per batch item, >= 1 */
    int32_t d_model;   /* length of an input vector x */
    int32_t n_heads;
    int32_t d_k;       /* length of q, k and v of one head */
    int32_t p;         /* ring partitions (the paper's m PEs); n % p == 0 */
    int32_t dtype;     /* attn_dtype of X, W and out */
    float scale;       /* multiplies w'_ij; 0 selects 1/sqrt(d_k); 1 is Eq. (1) as printed */
    uint32_t flags;    /* ATTN_FLAG_* */
} attn_config;

typedef struct {
    uint64_t pairs_full;          /* batch*heads*n*n: pairs per phase in the original definition */
    uint64_t pairs_needed[3];     /* fewest pairs phases 1..3 must touch (closed forms of Sec. 3.2, 4.1, 5.1; host) */
    uint64_t pairs_scheduled[3];  /* pairs the paper's schedule touches; differs from needed only for
                                     q = k = v with even n: n(n+2)/2 (Sec. 4.2, item 4) */
    uint64_t tiles_full;          /* batch*heads*p*p logical tiles of (n/p)^2 pairs */
    uint64_t tiles_executed;      /* logical tiles the last attn_forward worked on; COUNTED ON THE DEVICE */
    uint64_t pairs_executed;      /* tiles_executed * (n/p)^2 */
    uint64_t phys_tiles_executed; /* score blocks of phys_br x phys_bc pairs the kernels issued; device-counted */
    int32_t phys_br, phys_bc;
    uint64_t proj_gemms;          /* 3; q = k = v scheme: 1 on the float path (0 when X is used unprojected),
                                     2 on the matrix-core path (z = x.Wq produced in two layouts) */
} attn_stats_t;

typedef struct {
    int32_t calls;            /* attn_forward calls timed since profiling was switched on */
    float ms_prepare;         /* average per call: kernels ahead of the projection (weight re-layout on the
                                 fallback path), 0 when there is none */
    float ms_projection;      /* average per call: q/k/v projection kernel(s) */
    float ms_attention;       /* average per call: score/softmax/weighted-sum kernel(s) */
} attn_profile_t;

/*
 * Create a context for one problem shape on the current HIP device and allocate
 * its workspace.  Errors: INVALID (NULL, sizes < 1, unknown dtype or flag),
 * SHAPE (n % p != 0, or batch*n*n_heads*d_k does not fit 31 bits),
 * UNSUPPORTED (d_k above 256), ALLOC, DEVICE.
 * On error *out_ctx is NULL and attn_last_error(NULL) describes the failure.
 */
attn_status attn_init(const attn_config* cfg, attn_ctx** out_ctx);

/*
 * Key padding (not in the paper; batch items are independent): lens_dev is a
 * device array of `batch` int32, or NULL to clear.  Pair (i,j) of item b then
 * needs j < lens_dev[b] besides the scheme's own rule; every query row is still
 * produced and a row with no allowed pair is all zeros.  The pointer is borrowed
 * until it is replaced; the array is read by each attn_forward.  Not accepted
 * together with ATTN_SCHEME_SYMMETRIC (attn_forward then returns UNSUPPORTED).
 */
attn_status attn_set_key_lengths(attn_ctx* ctx, const int32_t* lens_dev);

/*
 * Enqueue one forward pass on `hip_stream` (a hipStream_t, NULL = default
 * stream): projections, scores, softmax and weighted sum, skipping what `scheme`
 * makes redundant (Sec. 3-5; see the head of this file).  For
 * ATTN_SCHEME_SYMMETRIC the shared vectors are z = x.Wq; Wk and Wv are ignored
 * (may be NULL); Wq == NULL means z = x and needs d_model == n_heads*d_k.  On the
 * matrix-core path (bfloat16, d_k 64 or 128, Wq given) every 128 x 128 score tile is
 * computed once and used for both of its row blocks (Sec. 4.1, Eq. (4)), the scores stay
 * on chip and 128 (d_k + 2) floats of partial row state per use go through device memory;
 * elsewhere one score matrix per (batch, head) does.  Either workspace is bounded by
 * 1 GiB; a shape beyond it on both paths is refused (UNSUPPORTED).
 * Errors: INVALID (NULL ctx/X/out, NULL weights where needed, bad scheme),
 * UNSUPPORTED, ALLOC, DEVICE (launch failure).
 */
attn_status attn_forward(attn_ctx* ctx, const void* X, const void* Wq, const void* Wk,
                         const void* Wv, int32_t scheme, void* out, void* hip_stream);

/*
 * attn_forward on sequences of different lengths stored back to back, without padding (not in
 * the paper, which has one sequence; batch items are independent, and a vector past an item's
 * length would be in no allowed pair under Sec. 5.1's rule applied to padding).
 * row_offsets_dev: device array of batch + 1 int32, non-decreasing, row_offsets_dev[0] = 0: item b
 * is rows row_offsets_dev[b] .. row_offsets_dev[b + 1] - 1 of X and of out, both
 * [row_offsets_dev[batch]][...] row-major; its length must not exceed the context's n (a longer
 * item is cut at n: its later rows take no part and their rows of out are left as they were).
 * Pair (i, j) of item b needs i, j below the item's length besides the scheme's own rule; only
 * rows that exist are projected, walked and written, and attn_stats afterwards reports the
 * counts for these lengths (pairs with both i and j below the length).  The array is read by the
 * kernels of the call only.  Key lengths set with attn_set_key_lengths are not used by this call.
 * Only on the matrix-core path (bfloat16, d_k 64 or 128, d_model a multiple of 8, X 16-byte and
 * out 8-byte aligned) and for ATTN_SCHEME_FULL and ATTN_SCHEME_CAUSAL: anything else returns
 * UNSUPPORTED, and so does a context created with ATTN_FLAG_NO_SKIP.  ATTN_FLAG_FUSE_Q_PROJECTION
 * is ignored.  Other errors as for attn_forward.
 */
attn_status attn_forward_packed(attn_ctx* ctx, const int32_t* row_offsets_dev, const void* X,
                                const void* Wq, const void* Wk, const void* Wv, int32_t scheme,
                                void* out, void* hip_stream);

/*
 * Wait for the stream of the last attn_forward and report its executed-versus-full
 * counts.  The closed-form fields are evaluated on the host with the key lengths that
 * call ran with (they are copied back for that: the array it was given must still be
 * valid); the *_executed fields are what the kernels counted.
 */
attn_status attn_stats(attn_ctx* ctx, attn_stats_t* out);

/*
 * Kernel timing with HIP events recorded on the launch stream around each
 * kernel group of every later attn_forward.  enable != 0 starts (and resets)
 * the record, 0 stops it.  attn_profile_read waits for the stream and returns
 * per-call averages.  At most 4096 calls are kept per record; later calls are
 * not timed.
 */
attn_status attn_profile(attn_ctx* ctx, int32_t enable);
attn_status attn_profile_read(attn_ctx* ctx, attn_profile_t* out);

/*
 * attn_forward without any allocation, for callers that cannot allocate: code under HIP graph
 * capture, serving loops and harnesses that forbid hipMalloc.  No context: the configuration and the
 * key lengths (device array of `batch` int32, or NULL) come with the call; X, Wq, Wk, Wv, out and
 * hip_stream are as for attn_forward.  The workspace (counter slots, projected q, k, v) is a fixed
 * array of ATTN_STATIC_SCRATCH_MIB MiB of device memory that belongs to the loaded library; every GPU
 * the library is used on holds its copy until the process ends.  The call makes no hipMalloc, hipFree
 * or other allocating call and does not wait for the stream.
 * Takes only what the matrix-core kernels take with the weights read in place: bfloat16, d_k 64 or
 * 128, d_model a multiple of 64, n_heads*d_k a multiple of 128, X and weights 16-byte aligned, schemes
 * FULL and CAUSAL; anything else, and any shape whose workspace
 *     130 KiB + 3 * batch * roundup(n, 256) * n_heads * d_k * 2 bytes
 * exceeds the array, returns UNSUPPORTED with the size needed in attn_last_error(NULL).
 * All calls on one GPU share that GPU's array, which keeps what the last call left: the call clears
 * what must start at zero (counter slots, the rows past n) itself, and two calls that overlap in time
 * on one GPU - on different streams or from different threads - race.  Calls on one stream, or
 * otherwise ordered by the caller, are fine.  Results obey the same bars as attn_forward's.
 */
#define ATTN_STATIC_SCRATCH_MIB 64
attn_status attn_forward_static(const attn_config* cfg, const int32_t* lens_dev, const void* X,
                                const void* Wq, const void* Wk, const void* Wv, int32_t scheme, void* out,
                                void* hip_stream);

/* Text of the last failure on this context (ctx == NULL: of the last failed
 * attn_init on this thread).  Never NULL; valid until the next call. */
const char* attn_last_error(const attn_ctx* ctx);

/* Free the workspace and the context.  NULL is accepted.  The caller must have
 * synchronised the stream of the last attn_forward. */
void attn_destroy(attn_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* ATTNRING_H */
