// Host side of libattnring.so: the C ABI declared in include/attnring.h.
// Validation, workspace, choice of kernel path, launches, counters, timing.
#include "../../include/attnring.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "mfma_common.h"

using namespace attnring;

struct attn_ctx {
    attn_config cfg;
    int device;
    int b, Npad;
    float scale;
    bool mfma_shape;  // shape and dtype fit the bf16 MFMA kernels
    // bf16 MFMA workspace
    h16_t *qb, *kb, *vtb;  // projected q, k, v^T, half precision
    bf16_t* wt;
    // generic float workspace (allocated on first use)
    float *qf, *kf, *vf;
    float* scores;  // q = k = v scheme, float path: one n x n score matrix per (batch, head)
    float* sym_work;  // q = k = v scheme, matrix-core path: partial row states (allocated on first use)
    unsigned long long* counters;
    const int32_t* lens;
    int32_t* packed_lens;  // [batch]: the lengths a packed call derives from its row offsets
    // last forward
    const int32_t* last_lens;  // the key lengths that call ran with
    bool last_rows_too;
    hipStream_t last_stream;
    int last_scheme;
    int last_proj_gemms;
    int last_phys;
    bool have_forward;
    // timing
    bool prof_on;
    int prof_calls;
    std::vector<unsigned char> prof_prepared;  // per recorded call: a kernel ran before the projection
    std::vector<hipEvent_t> events;  // 4 per timed call
    char err[512];
};

// Workspace of attn_forward_static: counter slots, then q, k and v^T of one call, in device memory
// that belongs to the loaded library (one copy per GPU, held until the process ends) instead of
// coming from hipMalloc.  In host code this name only stands for the symbol; its address on a
// device comes from hipGetSymbolAddress (static_scratch_on_current_device).
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)ATTN_STATIC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_init_err[512] = "";
constexpr int MAX_PROFILE_CALLS = 4096;
constexpr size_t MAX_SCORE_BYTES = (size_t)1 << 30;

attn_status fail(attn_ctx* ctx, attn_status st, const char* fmt, const char* detail = "")
{
    char* dst = ctx ? ctx->err : g_init_err;
    snprintf(dst, 512, fmt, detail);
    return st;
}

attn_status hip_fail(attn_ctx* ctx, const char* what, hipError_t e)
{
    char* dst = ctx ? ctx->err : g_init_err;
    snprintf(dst, 512, "%s: %s", what, hipGetErrorString(e));
    return e == hipErrorOutOfMemory ? ATTN_ERR_ALLOC : ATTN_ERR_DEVICE;
}

void free_all(attn_ctx* c)
{
    void* ptrs[] = {c->qb, c->kb, c->vtb, c->wt, c->qf, c->kf, c->vf, c->scores, c->sym_work, c->counters, c->packed_lens};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    for (hipEvent_t e : c->events) (void)hipEventDestroy(e);
    c->events.clear();
}

Problem make_problem(const attn_ctx* c, int scheme)
{
    Problem pb;
    pb.B = c->cfg.batch; pb.N = c->cfg.n; pb.D = c->cfg.d_model; pb.H = c->cfg.n_heads; pb.d = c->cfg.d_k;
    pb.P = c->cfg.p; pb.b = c->b; pb.Npad = c->Npad; pb.scale = c->scale; pb.scheme = scheme;
    pb.noskip = (c->cfg.flags & ATTN_FLAG_NO_SKIP) != 0;
    pb.skip_rows = (c->cfg.flags & ATTN_FLAG_SKIP_PADDED_ROWS) != 0 && c->lens != nullptr;
    pb.no_q = scheme == ATTN_SCHEME_SYMMETRIC;
    pb.is_bf16 = c->cfg.dtype == ATTN_BF16;
    pb.lens = c->lens;
    pb.row0 = nullptr;
    pb.counters = c->counters;
    return pb;
}

__global__ __launch_bounds__(1024) void zero_counters_kernel(unsigned long long* c)
{
    for (int w = 0; w < CNT_WORDS; ++w) c[(size_t)threadIdx.x * CNT_SLOT_WORDS + w] = 0ull;  // CNT_SLOTS threads
    if (threadIdx.x < CNT_WORDS) c[CNT_TOTALS + threadIdx.x] = 0ull;
}

// totals[w] = sum over the slots; one workgroup of CNT_SLOTS threads
__global__ __launch_bounds__(1024) void sum_counters_kernel(unsigned long long* c)
{
    __shared__ unsigned long long part[CNT_WORDS][16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int w = 0; w < CNT_WORDS; ++w) {
        unsigned long long v = c[(size_t)threadIdx.x * CNT_SLOT_WORDS + w];
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
        if (lane == 0) part[w][wave] = v;
    }
    __syncthreads();
    if (threadIdx.x < CNT_WORDS) {
        unsigned long long v = 0;
        for (int i = 0; i < CNT_SLOTS / 64; ++i) v += part[threadIdx.x][i];
        c[CNT_TOTALS + threadIdx.x] = v;
    }
}

// Packed layout: item b holds rows row0[b] .. row0[b + 1] - 1; its length, kept inside 0 .. n.
__global__ __launch_bounds__(256) void lens_from_offsets_kernel(const int32_t* __restrict__ row0,
                                                                int32_t* __restrict__ lens, int B, int N)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    const int len = row0[b + 1] - row0[b];
    lens[b] = len < 0 ? 0 : (len > N ? N : len);
}

attn_status ensure_generic_workspace(attn_ctx* c)
{
    if (c->qf && c->kf && c->vf) return ATTN_OK;
    const size_t bytes = (size_t)c->cfg.batch * c->cfg.n_heads * c->cfg.n * c->cfg.d_k * sizeof(float);
    float** dst[3] = {&c->qf, &c->kf, &c->vf};
    for (auto p : dst) {
        if (*p) continue;
        hipError_t e = hipMalloc((void**)p, bytes);
        if (e != hipSuccess) {
            // all three or none: a later call must not find a partial workspace
            for (auto r : dst) {
                if (*r) (void)hipFree(*r);
                *r = nullptr;
            }
            return hip_fail(c, "hipMalloc(float q/k/v workspace)", e);
        }
    }
    return ATTN_OK;
}

bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// sum over batch items of f(len_b), key lengths copied from the device when set
template <typename F>
attn_status sum_over_lengths(attn_ctx* c, F f, unsigned long long* out)
{
    const int B = c->cfg.batch, N = c->cfg.n;
    std::vector<int32_t> lens((size_t)B, N);
    if (c->last_lens) {
        hipError_t e = hipMemcpy(lens.data(), c->last_lens, sizeof(int32_t) * (size_t)B, hipMemcpyDeviceToHost);
        if (e != hipSuccess) return hip_fail(c, "hipMemcpy(key lengths)", e);
    }
    unsigned long long s = 0;
    for (int b = 0; b < B; ++b) {
        long long L = lens[(size_t)b];
        L = L < 0 ? 0 : (L > N ? N : L);
        s += f((unsigned long long)L);
    }
    *out = s;
    return ATTN_OK;
}

long long padded_rows(int n) { return ((long long)n + 255) / 256 * 256; }  // row pitch of the projected q, k, v

float effective_scale(const attn_config* cfg)
{
    return cfg->scale == 0.f ? 1.f / std::sqrt((float)cfg->d_k) : cfg->scale;
}

// Shape and dtype fit the matrix-core kernels.
bool matrix_core_shape(const attn_config* cfg)
{
    return cfg->dtype == ATTN_BF16 && (cfg->d_k == 64 || cfg->d_k == 128) && cfg->d_model % 8 == 0 &&
           effective_scale(cfg) > 0.f;
}

// The checks every entry point that takes a configuration starts with.
attn_status validate_config(const attn_config* cfg)
{
    if (cfg->batch < 1 || cfg->n < 1 || cfg->d_model < 1 || cfg->n_heads < 1 || cfg->d_k < 1 || cfg->p < 1)
        return fail(nullptr, ATTN_ERR_INVALID, "attn config: every size must be >= 1%s");
    if (cfg->dtype != ATTN_F32 && cfg->dtype != ATTN_BF16)
        return fail(nullptr, ATTN_ERR_INVALID, "attn config: unknown dtype%s");
    if (cfg->flags & ~(uint32_t)(ATTN_FLAG_NO_SKIP | ATTN_FLAG_WIDE_TILES | ATTN_FLAG_NARROW_TILES |
                                 ATTN_FLAG_SKIP_PADDED_ROWS | ATTN_FLAG_FUSE_Q_PROJECTION))
        return fail(nullptr, ATTN_ERR_INVALID, "attn config: unknown flag%s");
    if ((cfg->flags & ATTN_FLAG_WIDE_TILES) && (cfg->flags & ATTN_FLAG_NARROW_TILES))
        return fail(nullptr, ATTN_ERR_INVALID, "attn config: WIDE_TILES and NARROW_TILES exclude each other%s");
    if (!(cfg->scale == cfg->scale) || std::isinf(cfg->scale))
        return fail(nullptr, ATTN_ERR_INVALID, "attn config: scale is not finite%s");
    if (cfg->n % cfg->p != 0)
        return fail(nullptr, ATTN_ERR_SHAPE, "attn config: n must be divisible by p (ring partitions)%s");
    const long long Npad = ((long long)cfg->n + 255) / 256 * 256;
    const long long hd = (long long)cfg->n_heads * cfg->d_k;
    const long long limit = 0x7fffffffLL;
    if ((long long)cfg->batch * Npad * hd > limit || (long long)cfg->batch * cfg->n * cfg->d_model > limit ||
        3 * hd * cfg->d_model > limit || (long long)cfg->p * cfg->p > limit)
        return fail(nullptr, ATTN_ERR_SHAPE, "attn config: problem too large for 32-bit element indices%s");
    if (cfg->d_k > 256)
        return fail(nullptr, ATTN_ERR_UNSUPPORTED, "attn config: d_k above 256 is not implemented%s");
    return ATTN_OK;
}

// Address of `scratch` on the current device: asked for once per device, with that device
// current (every GPU holds its own copy of the array at its own address), and kept.
constexpr int MAX_DEVICES = 64;
unsigned char* g_scratch_ptr[MAX_DEVICES] = {};
std::mutex g_scratch_mutex;

attn_status static_scratch_on_current_device(unsigned char** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(nullptr, "hipGetDevice", e);
    if (dev < 0 || dev >= MAX_DEVICES) return fail(nullptr, ATTN_ERR_UNSUPPORTED, "device index beyond 63%s");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(nullptr, "hipGetSymbolAddress(scratch)", e);
        g_scratch_ptr[dev] = (unsigned char*)p;
    }
    *out = g_scratch_ptr[dev];
    return ATTN_OK;
}

// Rows n .. Npad-1 of q and k, and the key slots of v^T that belong to them, of every (batch, head):
// the kernels take them to be zero.  Grid (batch * heads, 3).
__global__ __launch_bounds__(256) void clear_pad_rows_kernel(int N, int Npad, int d, h16_t* __restrict__ q,
                                                             h16_t* __restrict__ k, h16_t* __restrict__ vt)
{
    const size_t head = (size_t)blockIdx.x * Npad * d;
    if (blockIdx.y < 2) {
        h16_t* dst = (blockIdx.y == 0 ? q : k) + head + (size_t)N * d;
        const int count = (Npad - N) * d;
        for (int e = threadIdx.x; e < count; e += blockDim.x) dst[e] = 0;
    } else {
        // v^T: [64-key block][d][64 slots]; slot (s & 48) | vt_slot16(s & 15) holds key s of the block,
        // and the permutation is its own inverse
        const int first = (N >> 6) * 64 * d;
        const int count = Npad * d - first;
        for (int e = threadIdx.x; e < count; e += blockDim.x) {
            const int pos = first + e;
            const int blk = pos / (64 * d), slot = pos & 63;
            const int key = blk * 64 + ((slot & 48) | vt_slot16(slot & 15));
            if (key >= N) vt[head + pos] = 0;
        }
    }
}

size_t round_up_256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

extern "C" {

attn_status attn_init(const attn_config* cfg, attn_ctx** out_ctx)
{
    if (out_ctx) *out_ctx = nullptr;
    if (!cfg || !out_ctx) return fail(nullptr, ATTN_ERR_INVALID, "attn_init: NULL argument%s");
    attn_status vst = validate_config(cfg);
    if (vst != ATTN_OK) return vst;
    const long long Npad = padded_rows(cfg->n);
    const long long hd = (long long)cfg->n_heads * cfg->d_k;

    attn_ctx* c = new (std::nothrow) attn_ctx();
    if (!c) return fail(nullptr, ATTN_ERR_ALLOC, "attn_init: out of host memory%s");
    c->cfg = *cfg;
    c->b = cfg->n / cfg->p;
    c->Npad = (int)Npad;
    c->scale = effective_scale(cfg);
    c->err[0] = 0;
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) { attn_status st = hip_fail(nullptr, "hipGetDevice", e); delete c; return st; }

    c->mfma_shape = matrix_core_shape(cfg);
    e = hipMalloc((void**)&c->counters, sizeof(unsigned long long) * CNT_BUFFER_WORDS);
    if (e == hipSuccess) e = hipMemset(c->counters, 0, sizeof(unsigned long long) * CNT_BUFFER_WORDS);
    if (e == hipSuccess) e = hipMalloc((void**)&c->packed_lens, sizeof(int32_t) * (size_t)(cfg->batch > 0 ? cfg->batch : 1));
    if (e == hipSuccess && c->mfma_shape) {
        const size_t qkv = (size_t)cfg->batch * c->Npad * hd * sizeof(h16_t);
        h16_t** dst[3] = {&c->qb, &c->kb, &c->vtb};
        for (auto p : dst) {
            if (e == hipSuccess) e = hipMalloc((void**)p, qkv);
            if (e == hipSuccess) e = hipMemset(*p, 0, qkv);  // rows past n stay zero for good
        }
        if (e == hipSuccess) e = hipMalloc((void**)&c->wt, (size_t)3 * hd * cfg->d_model * sizeof(bf16_t));
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        attn_status st = hip_fail(nullptr, "attn_init: workspace", e);
        free_all(c);
        delete c;
        return st;
    }
    if (!c->mfma_shape) {
        attn_status st = ensure_generic_workspace(c);
        if (st != ATTN_OK) {
            snprintf(g_init_err, sizeof(g_init_err), "%s", c->err);
            free_all(c);
            delete c;
            return st;
        }
    }
    *out_ctx = c;
    return ATTN_OK;
}

attn_status attn_set_key_lengths(attn_ctx* ctx, const int32_t* lens_dev)
{
    if (!ctx) return fail(nullptr, ATTN_ERR_INVALID, "attn_set_key_lengths: NULL context%s");
    ctx->lens = lens_dev;
    return ATTN_OK;
}

// attn_forward (row0 == NULL) and attn_forward_packed (row0: device, the items' first rows)
static attn_status forward_on(attn_ctx* ctx, const int32_t* row0, const void* X, const void* Wq, const void* Wk,
                              const void* Wv, int32_t scheme, void* out, void* hip_stream)
{
    if (!ctx) return fail(nullptr, ATTN_ERR_INVALID, "attn_forward: NULL context%s");
    if (!X || !out) return fail(ctx, ATTN_ERR_INVALID, "attn_forward: X and out must not be NULL%s");
    if (scheme != ATTN_SCHEME_FULL && scheme != ATTN_SCHEME_SYMMETRIC && scheme != ATTN_SCHEME_CAUSAL)
        return fail(ctx, ATTN_ERR_INVALID, "attn_forward: unknown scheme%s");
    const attn_config& cf = ctx->cfg;
    const int hd = cf.n_heads * cf.d_k;
    if (scheme == ATTN_SCHEME_SYMMETRIC) {
        if (row0) return fail(ctx, ATTN_ERR_UNSUPPORTED, "attn_forward_packed: the q=k=v scheme takes no lengths%s");
        if (ctx->lens) return fail(ctx, ATTN_ERR_UNSUPPORTED, "attn_forward: key lengths with the q=k=v scheme%s");
        if (!Wq && cf.d_model != hd)
            return fail(ctx, ATTN_ERR_INVALID, "attn_forward: Wq == NULL needs d_model == n_heads*d_k%s");
        if (cf.d_k > 256) return fail(ctx, ATTN_ERR_UNSUPPORTED, "attn_forward: q=k=v scheme with d_k above 256%s");
    } else if (!Wq || !Wk || !Wv) {
        return fail(ctx, ATTN_ERR_INVALID, "attn_forward: Wq, Wk and Wv must not be NULL%s");
    }
    hipStream_t s = (hipStream_t)hip_stream;
    Problem pb = make_problem(ctx, scheme);
    if (row0) {  // the items' lengths are their key lengths, and no row past them exists
        pb.lens = ctx->packed_lens;
        pb.row0 = row0;
        pb.skip_rows = true;
    }
    hipError_t e;

    hipEvent_t* ev = nullptr;
    if (ctx->prof_on && ctx->prof_calls < MAX_PROFILE_CALLS) {
        const size_t need = (size_t)(ctx->prof_calls + 1) * 4;
        while (ctx->events.size() < need) {
            hipEvent_t n;
            e = hipEventCreate(&n);
            if (e != hipSuccess) return hip_fail(ctx, "hipEventCreate", e);
            ctx->events.push_back(n);
        }
        ev = &ctx->events[(size_t)ctx->prof_calls * 4];
    }
#define MARK(i_)                                                              \
    if (ev) {                                                                 \
        e = hipEventRecord(ev[i_], s);                                        \
        if (e != hipSuccess) return hip_fail(ctx, "hipEventRecord", e);       \
    }
#define CHECK(what_)                                                          \
    if (e != hipSuccess) return hip_fail(ctx, what_, e);

    MARK(0);
    bool prepared = false;  // whether event 1 of this call gets recorded

    // The q = k = v scheme runs on the matrix cores when z is a projection (Wq given) and the
    // partial row states fit the workspace bound.
    const bool sym = scheme == ATTN_SCHEME_SYMMETRIC;
    const bool sym_fits = sym && Wq != nullptr && sym_pair_workspace_floats(pb) * sizeof(float) <= MAX_SCORE_BYTES;
    const bool use_mfma = ctx->mfma_shape && (!sym || sym_fits) && aligned_to(X, 16) && aligned_to(out, 8) &&
                          aligned_to(Wq, 2) && (sym || (aligned_to(Wk, 2) && aligned_to(Wv, 2)));
    if (row0 && (cf.flags & ATTN_FLAG_NO_SKIP))
        return fail(ctx, ATTN_ERR_UNSUPPORTED, "attn_forward_packed: not with ATTN_FLAG_NO_SKIP%s");
    if (row0 && !use_mfma)
        return fail(ctx, ATTN_ERR_UNSUPPORTED,
                    "attn_forward_packed: needs the matrix-core path (bfloat16, d_k 64 or 128, d_model a multiple "
                    "of 8, X 16-byte and out 8-byte aligned)%s");
    if (row0) {
        hipLaunchKernelGGL(lens_from_offsets_kernel, dim3((cf.batch + 255) / 256), dim3(256), 0, s, row0,
                           ctx->packed_lens, cf.batch, cf.n);
        e = hipGetLastError();
        CHECK("launch lens_from_offsets");
    }
    if (sym && use_mfma) { Wk = Wq; Wv = Wq; }  // one set of vectors in all three roles (Sec. 4.1)
    if (sym && use_mfma && !ctx->sym_work) {
        e = hipMalloc((void**)&ctx->sym_work, sym_pair_workspace_floats(pb) * sizeof(float));
        if (e != hipSuccess) return hip_fail(ctx, "hipMalloc(partial row states)", e);
    }
    if (!use_mfma) {  // the matrix-core path clears the counters in its first kernel
        hipLaunchKernelGGL(zero_counters_kernel, dim3(1), dim3(CNT_SLOTS), 0, s, ctx->counters);
        e = hipGetLastError();
        CHECK("launch zero_counters");
    }
    if (use_mfma) {
        // the first kernel of the call clears the counter slots: the projection itself when it reads
        // the weights in place, else the weight re-layout
        if (!proj_reads_weights_in_place(pb, (const bf16_t*)Wq, (const bf16_t*)Wk, (const bf16_t*)Wv)) {
            e = launch_transpose_w(pb, (const bf16_t*)Wq, (const bf16_t*)Wk, (const bf16_t*)Wv, ctx->wt, s);
            CHECK("launch transpose_w");
            MARK(1);
            prepared = true;
        }
        // queries projected inside the attention kernel: when asked for and the weights are read in place
        const bool fuse_q = !sym && !row0 && (cf.flags & ATTN_FLAG_FUSE_Q_PROJECTION) != 0 &&
                            proj_reads_weights_in_place(pb, (const bf16_t*)Wq, (const bf16_t*)Wk, (const bf16_t*)Wv);
        if (fuse_q) pb.no_q = true;
        e = launch_proj_mfma(pb, (const bf16_t*)X, (const bf16_t*)Wq, (const bf16_t*)Wk, (const bf16_t*)Wv, ctx->wt,
                             ctx->qb, ctx->kb, ctx->vtb, s);
        CHECK("launch proj_mfma");
        MARK(2);
        if (sym) {
            e = launch_sym_pair(pb, ctx->kb, ctx->vtb, ctx->sym_work, (bf16_t*)out, s);
            CHECK("launch q=k=v attention (mfma)");
            ctx->last_proj_gemms = 2;  // z = x.Wq, produced in the k and in the v^T layout
        } else {
            // d_k = 64: 128-row workgroups of 4 wavefronts, three of them per CU; d_k = 128: 256 rows, 8 wavefronts
            int waves = cf.d_k == 128 ? 8 : 4;
            if (cf.d_k == 64 && (cf.flags & ATTN_FLAG_WIDE_TILES)) waves = 8;
            e = launch_attn_pipe(pb, ctx->qb, ctx->kb, ctx->vtb, (bf16_t*)out, waves, s,
                                 fuse_q ? (const bf16_t*)X : nullptr, fuse_q ? (const bf16_t*)Wq : nullptr);
            CHECK("launch attention (mfma)");
            ctx->last_proj_gemms = 3;
        }
        MARK(3);
        ctx->last_phys = MFMA_BLOCK;
    } else {
        attn_status st = ensure_generic_workspace(ctx);
        if (st != ATTN_OK) return st;
        MARK(1);
        prepared = true;
        if (scheme == ATTN_SCHEME_SYMMETRIC) {
            const size_t bytes = (size_t)cf.batch * cf.n_heads * cf.n * cf.n * sizeof(float);
            if (bytes > MAX_SCORE_BYTES)
                return fail(ctx, ATTN_ERR_UNSUPPORTED, "attn_forward: q=k=v score scratch would exceed 1 GiB%s");
            if (!ctx->scores) {
                e = hipMalloc((void**)&ctx->scores, bytes);
                CHECK("hipMalloc(score scratch)");
            }
            if (Wq) e = launch_proj_generic(pb, X, Wq, ctx->qf, s);
            else e = launch_copy_heads_generic(pb, X, ctx->qf, s);
            CHECK("launch projection (q=k=v)");
            MARK(2);
            e = launch_sym_generic(pb, ctx->qf, ctx->scores, out, s);
            CHECK("launch q=k=v attention");
            ctx->last_proj_gemms = Wq ? 1 : 0;
        } else {
            e = launch_proj_generic(pb, X, Wq, ctx->qf, s);
            if (e == hipSuccess) e = launch_proj_generic(pb, X, Wk, ctx->kf, s);
            if (e == hipSuccess) e = launch_proj_generic(pb, X, Wv, ctx->vf, s);
            CHECK("launch projection");
            MARK(2);
            e = launch_attn_generic(pb, ctx->qf, ctx->kf, ctx->vf, out, s);
            CHECK("launch attention");
            ctx->last_proj_gemms = 3;
        }
        MARK(3);
        ctx->last_phys = ctx->b;
    }
#undef MARK
#undef CHECK
    if (ev) {
        if (ctx->prof_prepared.size() <= (size_t)ctx->prof_calls) ctx->prof_prepared.resize((size_t)ctx->prof_calls + 1);
        ctx->prof_prepared[(size_t)ctx->prof_calls] = prepared ? 1 : 0;
        ctx->prof_calls += 1;
    }
    ctx->last_stream = s;
    ctx->last_lens = pb.lens;
    ctx->last_rows_too = pb.skip_rows;
    ctx->last_scheme = scheme;
    ctx->have_forward = true;
    return ATTN_OK;
}

attn_status attn_forward(attn_ctx* ctx, const void* X, const void* Wq, const void* Wk, const void* Wv,
                         int32_t scheme, void* out, void* hip_stream)
{
    return forward_on(ctx, nullptr, X, Wq, Wk, Wv, scheme, out, hip_stream);
}

attn_status attn_forward_packed(attn_ctx* ctx, const int32_t* row_offsets_dev, const void* X, const void* Wq,
                                const void* Wk, const void* Wv, int32_t scheme, void* out, void* hip_stream)
{
    if (!ctx) return fail(nullptr, ATTN_ERR_INVALID, "attn_forward_packed: NULL context%s");
    if (!row_offsets_dev) return fail(ctx, ATTN_ERR_INVALID, "attn_forward_packed: NULL row offsets%s");
    return forward_on(ctx, row_offsets_dev, X, Wq, Wk, Wv, scheme, out, hip_stream);
}

attn_status attn_forward_static(const attn_config* cfg, const int32_t* lens_dev, const void* X, const void* Wq,
                                const void* Wk, const void* Wv, int32_t scheme, void* out, void* hip_stream)
{
    if (!cfg) return fail(nullptr, ATTN_ERR_INVALID, "attn_forward_static: NULL configuration%s");
    attn_status st = validate_config(cfg);
    if (st != ATTN_OK) return st;
    if (!X || !out || !Wq || !Wk || !Wv)
        return fail(nullptr, ATTN_ERR_INVALID, "attn_forward_static: X, Wq, Wk, Wv and out must not be NULL%s");
    if (scheme != ATTN_SCHEME_FULL && scheme != ATTN_SCHEME_CAUSAL)
        return fail(nullptr, ATTN_ERR_UNSUPPORTED, "attn_forward_static: FULL and CAUSAL schemes only%s");

    // the matrix-core path with the weights read in place: the one path whose whole workspace is
    // the counters and the projected q, k, v
    Problem pb;
    pb.B = cfg->batch; pb.N = cfg->n; pb.D = cfg->d_model; pb.H = cfg->n_heads; pb.d = cfg->d_k;
    pb.P = cfg->p; pb.b = cfg->n / cfg->p; pb.Npad = (int)padded_rows(cfg->n); pb.scale = effective_scale(cfg);
    pb.scheme = scheme;
    pb.noskip = (cfg->flags & ATTN_FLAG_NO_SKIP) != 0;
    pb.skip_rows = (cfg->flags & ATTN_FLAG_SKIP_PADDED_ROWS) != 0 && lens_dev != nullptr;
    pb.no_q = false;
    pb.is_bf16 = true;
    pb.lens = lens_dev;
    pb.row0 = nullptr;
    if (!matrix_core_shape(cfg) || !aligned_to(X, 16) || !aligned_to(out, 8) ||
        !proj_reads_weights_in_place(pb, (const bf16_t*)Wq, (const bf16_t*)Wk, (const bf16_t*)Wv))
        return fail(nullptr, ATTN_ERR_UNSUPPORTED,
                    "attn_forward_static: needs bfloat16, d_k 64 or 128, d_model a multiple of 64, n_heads*d_k a "
                    "multiple of 128, 16-byte aligned X and weights%s");
    const size_t cnt_bytes = round_up_256(sizeof(unsigned long long) * CNT_BUFFER_WORDS);
    const size_t qkv = round_up_256((size_t)pb.B * pb.Npad * pb.H * pb.d * sizeof(h16_t));
    if (cnt_bytes + 3 * qkv > STATIC_SCRATCH_BYTES) {
        char msg[256];
        snprintf(msg, sizeof(msg),
                 "attn_forward_static: this shape needs %zu bytes of workspace, beyond the fixed %d MiB; use "
                 "attn_init / attn_forward", cnt_bytes + 3 * qkv, (int)ATTN_STATIC_SCRATCH_MIB);
        return fail(nullptr, ATTN_ERR_UNSUPPORTED, "%s", msg);
    }
    unsigned char* base = nullptr;
    st = static_scratch_on_current_device(&base);
    if (st != ATTN_OK) return st;
    pb.counters = (unsigned long long*)base;
    h16_t* q = (h16_t*)(base + cnt_bytes);
    h16_t* k = (h16_t*)(base + cnt_bytes + qkv);
    h16_t* vt = (h16_t*)(base + cnt_bytes + 2 * qkv);

    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e;
    if (pb.Npad > pb.N) {  // whatever an earlier call left in the rows past n
        hipLaunchKernelGGL(clear_pad_rows_kernel, dim3(pb.B * pb.H, 3), dim3(256), 0, s, pb.N, pb.Npad, pb.d, q, k, vt);
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(nullptr, "launch clear_pad_rows", e);
    }
    e = launch_proj_mfma(pb, (const bf16_t*)X, (const bf16_t*)Wq, (const bf16_t*)Wk, (const bf16_t*)Wv, nullptr, q, k,
                         vt, s);
    if (e != hipSuccess) return hip_fail(nullptr, "launch proj_mfma", e);
    int waves = cfg->d_k == 128 ? 8 : 4;
    if (cfg->d_k == 64 && (cfg->flags & ATTN_FLAG_WIDE_TILES)) waves = 8;
    e = launch_attn_pipe(pb, q, k, vt, (bf16_t*)out, waves, s);
    if (e != hipSuccess) return hip_fail(nullptr, "launch attention (mfma)", e);
    return ATTN_OK;
}

attn_status attn_stats(attn_ctx* ctx, attn_stats_t* out)
{
    if (!ctx) return fail(nullptr, ATTN_ERR_INVALID, "attn_stats: NULL context%s");
    if (!out) return fail(ctx, ATTN_ERR_INVALID, "attn_stats: NULL output%s");
    if (!ctx->have_forward) return fail(ctx, ATTN_ERR_INVALID, "attn_stats: no attn_forward has run%s");
    hipLaunchKernelGGL(sum_counters_kernel, dim3(1), dim3(CNT_SLOTS), 0, ctx->last_stream, ctx->counters);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(ctx, "launch sum_counters", e);
    e = hipStreamSynchronize(ctx->last_stream);
    if (e != hipSuccess) return hip_fail(ctx, "hipStreamSynchronize", e);
    unsigned long long cnt[CNT_WORDS];
    e = hipMemcpy(cnt, ctx->counters + CNT_TOTALS, sizeof(cnt), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(ctx, "hipMemcpy(counters)", e);

    const attn_config& cf = ctx->cfg;
    const unsigned long long n = (unsigned long long)cf.n, H = (unsigned long long)cf.n_heads;
    const unsigned long long B = (unsigned long long)cf.batch, P = (unsigned long long)cf.p;
    memset(out, 0, sizeof(*out));
    out->pairs_full = B * H * n * n;
    out->tiles_full = B * H * P * P;
    attn_status st = ATTN_OK;
    unsigned long long per_head_sum = 0;
    const bool rows_too = ctx->last_rows_too;
    switch (ctx->last_scheme) {
    case ATTN_SCHEME_FULL:  // Sec. 3.2: n^2 per phase; with key padding n*len
        st = sum_over_lengths(ctx, [n, rows_too](unsigned long long L) { return (rows_too ? L : n) * L; },
                              &per_head_sum);
        for (int ph = 0; ph < 3; ++ph) out->pairs_needed[ph] = out->pairs_scheduled[ph] = H * per_head_sum;
        break;
    case ATTN_SCHEME_SYMMETRIC:  // Sec. 4.1 / 4.2: phase 1 n(n+1)/2 needed, n(n+2)/2 scheduled for even n
        out->pairs_needed[0] = B * H * (n * (n + 1) / 2);
        out->pairs_scheduled[0] = B * H * ((n % 2) ? n * (n + 1) / 2 : n * (n + 2) / 2);
        for (int ph = 1; ph < 3; ++ph) out->pairs_needed[ph] = out->pairs_scheduled[ph] = B * H * n * n;
        break;
    default:  // Sec. 5.1: n(n+1)/2 in all phases; with key padding sum_i min(i+1, len)
        st = sum_over_lengths(
            ctx, [n, rows_too](unsigned long long L) { return L * (L + 1) / 2 + (rows_too ? 0ull : (n - L) * L); },
            &per_head_sum);
        for (int ph = 0; ph < 3; ++ph) out->pairs_needed[ph] = out->pairs_scheduled[ph] = H * per_head_sum;
        break;
    }
    if (st != ATTN_OK) return st;
    out->tiles_executed = cnt[CNT_LOGICAL];
    out->pairs_executed = cnt[CNT_LOGICAL] * (unsigned long long)ctx->b * (unsigned long long)ctx->b;
    out->phys_tiles_executed = cnt[CNT_PHYS];
    out->phys_br = out->phys_bc = ctx->last_phys;
    out->proj_gemms = (unsigned long long)ctx->last_proj_gemms;
    return ATTN_OK;
}

attn_status attn_profile(attn_ctx* ctx, int32_t enable)
{
    if (!ctx) return fail(nullptr, ATTN_ERR_INVALID, "attn_profile: NULL context%s");
    if (enable && ctx->have_forward) {
        hipError_t e = hipStreamSynchronize(ctx->last_stream);  // events of the old record may be reused
        if (e != hipSuccess) return hip_fail(ctx, "hipStreamSynchronize", e);
    }
    ctx->prof_on = enable != 0;
    if (enable) ctx->prof_calls = 0;
    return ATTN_OK;
}

attn_status attn_profile_read(attn_ctx* ctx, attn_profile_t* out)
{
    if (!ctx) return fail(nullptr, ATTN_ERR_INVALID, "attn_profile_read: NULL context%s");
    if (!out) return fail(ctx, ATTN_ERR_INVALID, "attn_profile_read: NULL output%s");
    memset(out, 0, sizeof(*out));
    if (ctx->prof_calls == 0) return ATTN_OK;
    hipError_t e = hipStreamSynchronize(ctx->last_stream);
    if (e != hipSuccess) return hip_fail(ctx, "hipStreamSynchronize", e);
    double sum[3] = {0, 0, 0};
    for (int c = 0; c < ctx->prof_calls; ++c) {
        const bool prepared = ctx->prof_prepared[(size_t)c] != 0;
        for (int k = prepared ? 0 : 1; k < 3; ++k) {
            float ms = 0.f;
            const int from = (k == 1 && !prepared) ? 0 : k;  // no kernel before the projection: it starts at event 0
            e = hipEventElapsedTime(&ms, ctx->events[(size_t)c * 4 + from], ctx->events[(size_t)c * 4 + k + 1]);
            if (e != hipSuccess) return hip_fail(ctx, "hipEventElapsedTime", e);
            sum[k] += ms;
        }
    }
    out->calls = ctx->prof_calls;
    out->ms_prepare = (float)(sum[0] / ctx->prof_calls);
    out->ms_projection = (float)(sum[1] / ctx->prof_calls);
    out->ms_attention = (float)(sum[2] / ctx->prof_calls);
    return ATTN_OK;
}

const char* attn_last_error(const attn_ctx* ctx) { return ctx ? ctx->err : g_init_err; }

void attn_destroy(attn_ctx* ctx)
{
    if (!ctx) return;
    free_all(ctx);
    delete ctx;
}

}  // extern "C"
