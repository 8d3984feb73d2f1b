// Float-compute kernels for every shape the MFMA path does not take: f32
// storage, head sizes other than 64/128, and the q = k = v scheme.
//
// Mapping of the paper's ring onto the GPU: workgroup I is PE I.  It owns the
// n/P query rows [I*b, (I+1)*b) (abstract: n divisible by the number of PEs)
// and meets the key/value blocks in ring order J = I, I-1, ..., wrapping
// (the order in which PE l holds block (l - j) mod m in Algorithm 1).  Blocks
// that hold no needed pair are never touched: above the diagonal for masked
// attention (Sec. 5.1), past the key length for padded batches.
#include "common.h"

namespace attnring {
namespace {

__device__ __forceinline__ float load_as_float(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_as_float(const bf16_t* p, size_t i)
{
    return __uint_as_float(((unsigned)p[i]) << 16);
}
__device__ __forceinline__ void store_from_float(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_from_float(bf16_t* p, size_t i, float v)
{
    unsigned u = __float_as_uint(v);
    u += 0x7fffu + ((u >> 16) & 1u);  // round to nearest even (inputs are finite)
    p[i] = (bf16_t)(u >> 16);
}

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}
__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

// ---------------------------------------------------------------------------
// Projection (Sec. 3.1): out[b][h][i][l] = sum_c X[b][i][c] * W[c][h*d + l].
// 64 x 64 output tile per workgroup, 16-deep slices through LDS, 4 x 4 per thread.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void proj_generic_kernel(int M, int N, int D, int H, int d, const T* __restrict__ X,
                                                           const T* __restrict__ W, float* __restrict__ out)
{
    __shared__ float As[16][64 + 4];
    __shared__ float Bs[16][64 + 4];
    const int HD = H * d;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int row0 = blockIdx.y * 64, col0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < D; k0 += 16) {
        for (int e = tid; e < 64 * 16; e += 256) {
            int r = e >> 4, kk = e & 15;
            int gr = row0 + r, gk = k0 + kk;
            As[kk][r] = (gr < M && gk < D) ? load_as_float(X, (size_t)gr * D + gk) : 0.f;
        }
        for (int e = tid; e < 16 * 64; e += 256) {
            int kk = e >> 6, c = e & 63;
            int gk = k0 + kk, gc = col0 + c;
            Bs[kk][c] = (gk < D && gc < HD) ? load_as_float(W, (size_t)gk * HD + gc) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], bv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { a[u] = As[kk][ty * 4 + u]; bv[u] = Bs[kk][tx * 4 + u]; }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int w = 0; w < 4; ++w) acc[u][w] = fmaf(a[u], bv[w], acc[u][w]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        int gr = row0 + ty * 4 + u;
        if (gr >= M) continue;
        int bb = gr / N, i = gr - bb * N;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            int gc = col0 + tx * 4 + w;
            if (gc >= HD) continue;
            int h = gc / d, l = gc - h * d;
            out[(((size_t)bb * H + h) * N + i) * d + l] = acc[u][w];
        }
    }
}

// z = x split into heads, for the q = k = v scheme without a projection matrix.
template <typename T>
__global__ void copy_heads_kernel(int total, int N, int H, int d, const T* __restrict__ X, float* __restrict__ out)
{
    int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    int l = e % d, t = e / d;
    int h = t % H, bi = t / H;  // bi = b*N + i
    int bb = bi / N, i = bi - bb * N;
    out[(((size_t)bb * H + h) * N + i) * d + l] = load_as_float(X, (size_t)e);
}

// ---------------------------------------------------------------------------
// Online row state of phases 2 and 3 (Eq. (2), Eq. (3)) for one query row held
// by one wavefront: running maximum m, running sum l of exp(s - m), and the
// un-normalised output o (lane L holds columns L, L+64, ...).
// ---------------------------------------------------------------------------
enum { MAX_ACC = 4 };  // d_k <= 256

struct RowState {
    float m, l;
    float o[MAX_ACC];
};

// Fold up to 64 keys (one per lane) into the row state.  `s` is the lane's score,
// `ok` whether its pair takes part; keys jbase .. jbase+cnt-1 of head `vh`.
__device__ __forceinline__ void fold_chunk(RowState& st, float s, bool ok, int jbase, int cnt,
                                           const float* __restrict__ vh, int d, int lane)
{
    s = ok ? s : -INFINITY;
    const float m_new = fmaxf(st.m, wave_max(s));
    if (m_new == -INFINITY) return;  // nothing allowed so far (uniform over the wave)
    const float alpha = expf(st.m - m_new);
    const float p = ok ? expf(s - m_new) : 0.f;
    st.l = st.l * alpha + wave_sum(p);
    st.m = m_new;
#pragma unroll
    for (int a = 0; a < MAX_ACC; ++a) st.o[a] *= alpha;
    for (int jj = 0; jj < cnt; ++jj) {
        const float pj = __shfl(p, jj, 64);
        const float* vr = vh + (size_t)(jbase + jj) * d;
#pragma unroll
        for (int a = 0; a < MAX_ACC; ++a) {
            int col = lane + 64 * a;
            if (col < d) st.o[a] = fmaf(pj, vr[col], st.o[a]);
        }
    }
}

template <typename T>
__device__ __forceinline__ void store_row(const RowState& st, T* out, size_t base, int d, int lane)
{
    const float inv = st.l > 0.f ? 1.f / st.l : 0.f;  // a row with no allowed pair is zero
#pragma unroll
    for (int a = 0; a < MAX_ACC; ++a) {
        int col = lane + 64 * a;
        if (col < d) store_from_float(out, base + col, st.o[a] * inv);
    }
}

// len: key length of the batch item; rlen: the same limit for query rows when padded rows are left
// out, else n.
__device__ __forceinline__ bool pair_allowed(int scheme, int i, int j, int len, int rlen)
{
    return j < len && i < rlen && (scheme != SCHEME_CAUSAL || j <= i);
}
// A b x b tile holds a needed pair iff its first row's pair with its first key is allowed.
__device__ __forceinline__ bool tile_needed(int scheme, int I, int J, int b, int len, int rlen)
{
    return J * b < len && I * b < rlen && (scheme != SCHEME_CAUSAL || J <= I);
}

// ---------------------------------------------------------------------------
// Fused phases 1-3 for FULL and CAUSAL.  Grid (P, H, B); 4 wavefronts per PE,
// row r of the PE goes to wavefront r % 4.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_generic_kernel(Problem pb, const float* __restrict__ q,
                                                           const float* __restrict__ k,
                                                           const float* __restrict__ v, T* __restrict__ out)
{
    const int I = blockIdx.x, h = blockIdx.y, bb = blockIdx.z;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int N = pb.N, d = pb.d, b = pb.b, P = pb.P;
    int len = N;
    if (pb.lens) { len = pb.lens[bb]; len = len < 0 ? 0 : (len > N ? N : len); }
    const int rlen = pb.skip_rows ? len : N;
    const size_t head = ((size_t)bb * pb.H + h) * (size_t)N * d;
    const float* qh = q + head;
    const float* kh = k + head;
    const float* vh = v + head;

    if (threadIdx.x == 0) {  // tiles this PE works on (the same for each of its rows)
        unsigned long long tiles = 0;
        for (int t = 0; t < P; ++t) {
            int J = I - t; if (J < 0) J += P;
            if (pb.noskip || tile_needed(pb.scheme, I, J, b, len, rlen)) ++tiles;
        }
        count_add(pb.counters, (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x, tiles, tiles);
    }

    for (int r = wave; r < b; r += 4) {
        const int i = I * b + r;
        const float* qr = qh + (size_t)i * d;
        RowState st;
        st.m = -INFINITY; st.l = 0.f;
#pragma unroll
        for (int a = 0; a < MAX_ACC; ++a) st.o[a] = 0.f;
        for (int t = 0; t < P; ++t) {  // ring order, own block first
            int J = I - t; if (J < 0) J += P;
            if (!pb.noskip && !tile_needed(pb.scheme, I, J, b, len, rlen)) continue;  // redundant tile: skipped
            for (int c0 = 0; c0 < b; c0 += 64) {
                const int cnt = (b - c0) < 64 ? (b - c0) : 64;
                const int j = J * b + c0 + lane;
                const bool valid = lane < cnt;
                float s = 0.f;
                if (valid) {
                    const float* kr = kh + (size_t)j * d;
                    for (int l = 0; l < d; ++l) s = fmaf(qr[l], kr[l], s);  // Eq. (1)
                    s *= pb.scale;
                }
                fold_chunk(st, s, valid && pair_allowed(pb.scheme, i, j, len, rlen), J * b + c0, cnt, vh, d, lane);
            }
        }
        store_row(st, out, ((size_t)bb * N + i) * ((size_t)pb.H * d) + (size_t)h * d, d, lane);
    }
}

// ---------------------------------------------------------------------------
// q = k = v scheme (Sec. 4).  Phase 1 on tiles: PE I computes the tiles on the
// circulant tile diagonals (I - J) mod P = 0 .. floor(P/2) (Sec. 4.2 applied to
// the P x P tile matrix; for even P the middle diagonal is computed by both of
// its owners, the paper's balance trade-off) and stores each score also at its
// mirrored position, which is the reuse of w'_ij as w'_ji (Eq. (4)).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void sym_scores_kernel(Problem pb, const float* __restrict__ z,
                                                         float* __restrict__ scores)
{
    const int I = blockIdx.x, h = blockIdx.y, bb = blockIdx.z;
    const int N = pb.N, d = pb.d, b = pb.b, P = pb.P;
    const size_t bh = (size_t)bb * pb.H + h;
    const float* zh = z + bh * (size_t)N * d;
    float* S = scores + bh * (size_t)N * N;
    const int gmax = pb.noskip ? P - 1 : P / 2;
    for (int g = 0; g <= gmax; ++g) {
        int J = I - g; if (J < 0) J += P;
        const bool mirror = !pb.noskip && g != 0 && !(P % 2 == 0 && g == P / 2);
        for (int e = threadIdx.x; e < b * b; e += 256) {
            const int i = I * b + e / b, j = J * b + e % b;
            const float* zi = zh + (size_t)i * d;
            const float* zj = zh + (size_t)j * d;
            float s = 0.f;
            for (int l = 0; l < d; ++l) s = fmaf(zi[l], zj[l], s);
            s *= pb.scale;
            S[(size_t)i * N + j] = s;
            if (mirror) S[(size_t)j * N + i] = s;
        }
    }
    if (threadIdx.x == 0) {
        count_add(pb.counters, (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x,
                  (unsigned long long)(gmax + 1), (unsigned long long)(gmax + 1));
    }
}

// Phases 2 and 3 of the q = k = v scheme: unchanged from the original definition
// (Sec. 4.1), reading the stored scores.  One wavefront per row.
template <typename T>
__global__ __launch_bounds__(256) void sym_softmax_pv_kernel(Problem pb, const float* __restrict__ z,
                                                             const float* __restrict__ scores, T* __restrict__ out)
{
    const int h = blockIdx.y, bb = blockIdx.z;
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int N = pb.N, d = pb.d;
    if (i >= N) return;
    const size_t bh = (size_t)bb * pb.H + h;
    const float* vh = z + bh * (size_t)N * d;
    const float* Srow = scores + bh * (size_t)N * N + (size_t)i * N;
    RowState st;
    st.m = -INFINITY; st.l = 0.f;
#pragma unroll
    for (int a = 0; a < MAX_ACC; ++a) st.o[a] = 0.f;
    for (int j0 = 0; j0 < N; j0 += 64) {
        const int cnt = (N - j0) < 64 ? (N - j0) : 64;
        const bool valid = lane < cnt;
        const float s = valid ? Srow[j0 + lane] : 0.f;
        fold_chunk(st, s, valid, j0, cnt, vh, d, lane);
    }
    store_row(st, out, ((size_t)bb * N + i) * ((size_t)pb.H * d) + (size_t)h * d, d, lane);
}

}  // namespace

hipError_t launch_proj_generic(const Problem& pb, const void* X, const void* W, float* out, hipStream_t s)
{
    const int M = pb.B * pb.N, HD = pb.H * pb.d;
    dim3 grid((HD + 63) / 64, (M + 63) / 64);
    if (pb.is_bf16)
        hipLaunchKernelGGL(proj_generic_kernel<bf16_t>, grid, dim3(256), 0, s, M, pb.N, pb.D, pb.H, pb.d,
                           (const bf16_t*)X, (const bf16_t*)W, out);
    else
        hipLaunchKernelGGL(proj_generic_kernel<float>, grid, dim3(256), 0, s, M, pb.N, pb.D, pb.H, pb.d,
                           (const float*)X, (const float*)W, out);
    return hipGetLastError();
}

hipError_t launch_copy_heads_generic(const Problem& pb, const void* X, float* out, hipStream_t s)
{
    const int total = pb.B * pb.N * pb.H * pb.d;
    dim3 grid((total + 255) / 256);
    if (pb.is_bf16)
        hipLaunchKernelGGL(copy_heads_kernel<bf16_t>, grid, dim3(256), 0, s, total, pb.N, pb.H, pb.d,
                           (const bf16_t*)X, out);
    else
        hipLaunchKernelGGL(copy_heads_kernel<float>, grid, dim3(256), 0, s, total, pb.N, pb.H, pb.d,
                           (const float*)X, out);
    return hipGetLastError();
}

hipError_t launch_attn_generic(const Problem& pb, const float* q, const float* k, const float* v, void* out,
                               hipStream_t s)
{
    dim3 grid(pb.P, pb.H, pb.B);
    if (pb.is_bf16)
        hipLaunchKernelGGL(attn_generic_kernel<bf16_t>, grid, dim3(256), 0, s, pb, q, k, v, (bf16_t*)out);
    else
        hipLaunchKernelGGL(attn_generic_kernel<float>, grid, dim3(256), 0, s, pb, q, k, v, (float*)out);
    return hipGetLastError();
}

hipError_t launch_sym_generic(const Problem& pb, const float* z, float* scores, void* out, hipStream_t s)
{
    hipLaunchKernelGGL(sym_scores_kernel, dim3(pb.P, pb.H, pb.B), dim3(256), 0, s, pb, z, scores);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 grid((pb.N + 3) / 4, pb.H, pb.B);
    if (pb.is_bf16)
        hipLaunchKernelGGL(sym_softmax_pv_kernel<bf16_t>, grid, dim3(256), 0, s, pb, z, scores, (bf16_t*)out);
    else
        hipLaunchKernelGGL(sym_softmax_pv_kernel<float>, grid, dim3(256), 0, s, pb, z, scores, (float*)out);
    return hipGetLastError();
}

}  // namespace attnring
