// q/k/v projections (Sec. 3.1: q, k, v are linear maps of the inputs x by three
// learned matrices; one set per head) as ONE bf16 MFMA GEMM over the stacked
// output columns [q | k | v], fp32 accumulation, rounded once to half precision and
// written straight into the layouts the attention kernel streams:
//   q, k : [B][H][Npad][d]            (row = vector, d contiguous)
//   v^T  : [B][H][Npad/64][d][64]     (per 64-key block, key contiguous, and the
//                                      keys of each 16-group in MFMA operand order)
// The weights arrive as [D][H*d] (q = x.W), i.e. contiguous along the output
// columns, while an MFMA operand register wants 8 consecutive values of the
// contraction index.  The main kernel leaves them where they are and turns them
// while reading LDS (ds_read_b64_tr_b16); the fallback kernel for shapes and
// alignments that kernel does not take has a small kernel lay them out as
// W^T [3*H*d][D] first.
#include "mfma_common.h"

namespace attnring {
namespace {

// ---------------------------------------------------------------------------
// W^T: 64 x 64 tiles through LDS; grid (HD/64, ceil(D/64), 3).  Workgroup
// (0,0,0) also clears the counter slots of the call (every forward pass runs
// this kernel first).
// ---------------------------------------------------------------------------
__device__ __forceinline__ void clear_counters(unsigned long long* counters)
{
    if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0) {
        for (int sl = threadIdx.x; sl < CNT_SLOTS; sl += blockDim.x)
            for (int w = 0; w < CNT_WORDS; ++w) counters[(size_t)sl * CNT_SLOT_WORDS + w] = 0ull;
        if (threadIdx.x < CNT_WORDS) counters[CNT_TOTALS + threadIdx.x] = 0ull;
    }
}

__global__ __launch_bounds__(256) void transpose_w_kernel(int D, int HD, const bf16_t* __restrict__ Wq,
                                                          const bf16_t* __restrict__ Wk,
                                                          const bf16_t* __restrict__ Wv, bf16_t* __restrict__ Wt,
                                                          unsigned long long* counters)
{
    __shared__ bf16_t tile[64][64 + 2];
    clear_counters(counters);
    const bf16_t* W = blockIdx.z == 0 ? Wq : (blockIdx.z == 1 ? Wk : Wv);
    bf16_t* dst = Wt + (size_t)blockIdx.z * HD * D;
    const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int r = ty; r < 64; r += 4) {
        const int gr = r0 + r;
        tile[r][tx] = gr < D ? W[(size_t)gr * HD + c0 + tx] : (bf16_t)0;
    }
    __syncthreads();
    for (int c = ty; c < 64; c += 4) {
        const int gk = r0 + tx;
        if (gk < D) dst[(size_t)(c0 + c) * D + gk] = tile[tx][c];
    }
}

// The same for 16-byte aligned weights (D is a multiple of 8): 16 bytes per lane in and out.
__global__ __launch_bounds__(256) void transpose_w16_kernel(int D, int HD, const bf16_t* __restrict__ Wq,
                                                            const bf16_t* __restrict__ Wk,
                                                            const bf16_t* __restrict__ Wv, bf16_t* __restrict__ Wt,
                                                            unsigned long long* counters)
{
    constexpr int PITCH = 64 + 8;  // elements; keeps 16-byte alignment of the rows
    __shared__ __attribute__((aligned(16))) bf16_t tile[64 * PITCH];
    clear_counters(counters);
    const bf16_t* W = blockIdx.z == 0 ? Wq : (blockIdx.z == 1 ? Wk : Wv);
    bf16_t* dst = Wt + (size_t)blockIdx.z * HD * D;
    const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int c = threadIdx.x + 256 * u;
        const int row = c >> 3, cc = c & 7;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (r0 + row < D) v = *(const u32x4*)(W + (size_t)(r0 + row) * HD + c0 + 8 * cc);
        *(u32x4*)(tile + row * PITCH + 8 * cc) = v;
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int c = threadIdx.x + 256 * u;
        const int n = c >> 3, kc = c & 7;
        if (r0 + 8 * kc >= D) continue;
        u32x4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned lo = tile[(8 * kc + 2 * j) * PITCH + n], hi = tile[(8 * kc + 2 * j + 1) * PITCH + n];
            v[j] = lo | (hi << 16);
        }
        *(u32x4*)(dst + (size_t)(c0 + n) * D + r0 + 8 * kc) = v;
    }
}

// ---------------------------------------------------------------------------
// Fallback GEMM (any d_model, any alignment), on transposed weights:
// C = A . B^T with both operands k-contiguous.  Square BT x BT tile per
// workgroup, 2 x 2 wavefronts, 32x32x16 MFMA blocks, 64-deep k slices double
// buffered in LDS.  The "x side" rows are vectors (with the per-batch row pitch
// Npad; rows past n read the last real row and are not stored), the "w side"
// rows are output columns of [q | k | v].
// For q and k tiles the w side is the A operand, so a lane ends up with four
// consecutive output columns of one vector (8-byte store into [..][d]); for v
// tiles the x side is the A operand, so a lane holds four consecutive vectors of
// one column (8-byte store into the transposed layout).
// ---------------------------------------------------------------------------
constexpr int BK = 64;
constexpr int ROWB = BK * 2 + 16;  // LDS bytes per tile row (padded)

// Tile order.  Workgroup ids are dealt round-robin to the 8 XCDs, so each XCD is
// given a contiguous run of tile numbers; within the run, tiles are walked in
// groups of GROUP_W weight tiles by all x tiles, weight tile fastest, so that the
// ~32 tiles in flight on one XCD form a 4 x 8 patch that shares its operand
// slices in that XCD's L2 instead of fetching 32 different x slices.
constexpr int GROUP_W = 4;
__device__ __forceinline__ void tile_of(int id, int tiles_x, int tiles_w, int& tw, int& tx, int group_w = GROUP_W)
{
    const int width = group_w * tiles_x;
    const int grp = id / width;
    const int first_w = grp * group_w;
    const int gsz = min(tiles_w - first_w, group_w);
    const int local = id - grp * width;
    tx = local / gsz;
    tw = first_w + (local - tx * gsz);
}
// With key lengths some k and v tiles return at once, and an XCD keeps the run of tiles it was
// given: the order above would hand some XCDs q tiles only and others the short batch items.
// Both tile indices are therefore permuted, so that every run holds q, k and v tiles in equal
// parts (groups of three column tiles, dealt round-robin over the three matrices) and x tiles
// from all over the batch (a multiplier that is coprime to their number).
__device__ __forceinline__ void spread_tiles(int tiles_x, int tiles_w, int& tw, int& tx, int n_matrices = 3)
{
    const int per_matrix = tiles_w / n_matrices;
    tw = (tw % n_matrices) * per_matrix + tw / n_matrices;
    int mult = tiles_x / 8 + 1;
    while (true) {  // the next number coprime to tiles_x
        int a = mult, b = tiles_x;
        while (b) { const int r = a % b; a = b; b = r; }
        if (a == 1) break;
        ++mult;
    }
    tx = (int)(((long long)tx * mult) % tiles_x);
}

// Whether every row of the x tile that starts at flattened row x0 (Npad rows per batch item, a
// multiple of the tile height) lies at or past the key length of its batch item.
__device__ __forceinline__ bool past_key_length(const int* __restrict__ lens, int x0, int Npad, int N)
{
    const int bb = x0 / Npad;
    int len = lens[bb];
    len = len < 0 ? 0 : (len > N ? N : len);
    return x0 - bb * Npad >= len;
}

template <int BT>
__global__ __launch_bounds__(256) void proj_mfma_kernel(int Bsz, int N, int Npad, int D, int H, int d,
                                                        const bf16_t* __restrict__ X,
                                                        const bf16_t* __restrict__ Wt, h16_t* __restrict__ qo,
                                                        h16_t* __restrict__ ko, h16_t* __restrict__ vto,
                                                        int tiles_x, int tiles_w, float qscale, const int* __restrict__ lens, bool skip_q_rows, bool no_q,
                                                        const int* __restrict__ row0)
{
    constexpr int WT = BT / 2;          // wavefront tile edge
    constexpr int NB = WT / 32;         // MFMA blocks per edge
    constexpr int NCH = BT * 8 / 256;   // 16-byte chunks per thread and side
    constexpr int SIDE = BT * ROWB;
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * 2 * SIDE];

    const int tid = threadIdx.x;
    const int lane = tid & 63, ln = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wc = wave & 1;
    const int HD = H * d;

    const int n_tiles = tiles_x * tiles_w;
    const int per_xcd = gridDim.x >> 3;
    const int tile_id = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile_id >= n_tiles) return;
    int tw, tx_;
    tile_of(tile_id, tiles_x, tiles_w, tw, tx_);
    const int x0 = tx_ * BT;   // first x-side row (padded vector index)
    const int w0 = tw * BT;    // first stacked output column
    const bool is_v = w0 >= 2 * HD;
    // Keys past the key length of their batch item are in no allowed pair (Sec. 5.1 applied to
    // padding): their k and v rows are not computed.  (q rows are: every query row has an output.)
    // With padded rows left out as queries too, the same holds for their q rows.
    if (lens != nullptr && (w0 >= HD || skip_q_rows) && past_key_length(lens, x0, Npad, N)) return;
    if (no_q && w0 < HD) return;  // q = k = v scheme: the shared vectors are wanted as k and v^T only

    // per-thread source rows: chunk ch = tid + 256*u -> row ch/8, k-chunk ch%8
    const int kc = tid & 7;
    unsigned xoff[NCH], woff[NCH];
#pragma unroll
    for (int u = 0; u < NCH; ++u) {
        const int row = (tid >> 3) + 32 * u;
        const int xr = x0 + row;
        const int bb = xr / Npad;
        xoff[u] = source_row(row0, Bsz, N, bb, xr - bb * Npad) * (unsigned)D;
        woff[u] = (unsigned)(w0 + row) * (unsigned)D;
    }

    f32x16 acc[NB][NB];
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    u32x4 xreg[NCH], wreg[NCH];
    auto issue_loads = [&](int k0) {
        const int kk = k0 + kc * 8;
        const bool in = kk < D;  // D is a multiple of 8
#pragma unroll
        for (int u = 0; u < NCH; ++u) {
            u32x4 z = {0u, 0u, 0u, 0u};
            xreg[u] = in ? *(const u32x4*)(X + (size_t)xoff[u] + kk) : z;
            wreg[u] = in ? *(const u32x4*)(Wt + (size_t)woff[u] + kk) : z;
        }
    };
    // A operand side first, then B operand side
    auto stage_store = [&](int buf) {
        unsigned char* base = lds + buf * 2 * SIDE;
        unsigned char* xs = base + (is_v ? 0 : SIDE);
        unsigned char* ws = base + (is_v ? SIDE : 0);
#pragma unroll
        for (int u = 0; u < NCH; ++u) {
            const int row = (tid >> 3) + 32 * u;
            *(u32x4*)(xs + row * ROWB + kc * 16) = xreg[u];
            *(u32x4*)(ws + row * ROWB + kc * 16) = wreg[u];
        }
    };

    const int nk = (D + BK - 1) / BK;
    issue_loads(0);
    stage_store(0);
    __syncthreads();
    for (int it = 0; it < nk; ++it) {
        if (it + 1 < nk) issue_loads((it + 1) * BK);
        const unsigned char* as = lds + (it & 1) * 2 * SIDE + (wr * WT + ln) * ROWB + g * 16;
        const unsigned char* bs = lds + (it & 1) * 2 * SIDE + SIDE + (wc * WT + ln) * ROWB + g * 16;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            u32x4 af[NB], bf[NB];
#pragma unroll
            for (int a = 0; a < NB; ++a) af[a] = *(const u32x4*)(as + a * 32 * ROWB + ks * 32);
#pragma unroll
            for (int b = 0; b < NB; ++b) bf[b] = *(const u32x4*)(bs + b * 32 * ROWB + ks * 32);
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int b = 0; b < NB; ++b) acc[a][b] = mfma32(af[a], bf[b], acc[a][b]);
        }
        if (it + 1 < nk) stage_store((it + 1) & 1);
        __syncthreads();
    }

    // Epilogue.  acc[a][b][r]: A-side row wr*WT + 32a + acc_row(r,g), B-side row wc*WT + 32b + ln.
    if (!is_v) {
        // A side = output columns (4 consecutive per register quad), B side = vectors.
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int xr = x0 + wc * WT + 32 * b + ln;
            const int bb = xr / Npad;
            const int i = xr - bb * Npad;
            if (i >= N) continue;
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int col = w0 + wr * WT + 32 * a + 8 * r4 + 4 * g;  // stacked column of register 4*r4
                    const int which = col >= HD ? 1 : 0;
                    const int cc = col - which * HD;
                    const int h = cc / d, l = cc - h * d;
                    h16_t* dst = (which ? ko : qo) + (((size_t)bb * H + h) * Npad + i) * d + l;
                    const float qs = which ? 1.f : qscale;  // q is stored pre-multiplied (see launch_proj_mfma)
                    u32x2 w;
                    w[0] = pack_f16_sat(acc[a][b][4 * r4 + 0] * qs, acc[a][b][4 * r4 + 1] * qs);
                    w[1] = pack_f16_sat(acc[a][b][4 * r4 + 2] * qs, acc[a][b][4 * r4 + 3] * qs);
                    *(u32x2*)dst = w;
                }
        }
    } else {
        // A side = vectors (4 consecutive per register quad), B side = output columns of v.
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int cc = w0 - 2 * HD + wc * WT + 32 * b + ln;
            const int h = cc / d, l = cc - h * d;
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int xr = x0 + wr * WT + 32 * a + 8 * r4 + 4 * g;  // vector of register 4*r4
                    const int bb = xr / Npad;
                    const int i = xr - bb * Npad;
                    if (i >= N) continue;
                    const int blk = i >> 6, r64 = i & 63;
                    const int slot = (r64 & 48) | vt_slot16(r64 & 15);
                    h16_t* dst = vto + ((((size_t)bb * H + h) * (Npad >> 6) + blk) * d + l) * 64 + slot;
                    u32x2 w;
                    w[0] = pack_f16_sat(acc[a][b][4 * r4 + 0], acc[a][b][4 * r4 + 1]);
                    w[1] = pack_f16_sat(acc[a][b][4 * r4 + 2], acc[a][b][4 * r4 + 3]);
                    *(u32x2*)dst = w;
                }
        }
    }
}

// ---------------------------------------------------------------------------
// The GEMM for d_model a multiple of 64 and 16-byte aligned weights, with the operands
// copied from global memory straight into LDS (buffer_load ... lds, 16 bytes per lane) and
// the weights taken in the caller's layout.
//
// A request for 64 KiB of operands takes longer to come back than the MFMAs of one
// 64-deep slice take to run, so two slices have to be in flight, and LDS cannot hold
// three 64-deep stages of a 256 x 256 tile.  The two sides are kept in rings of their own:
//   x side   three units of BT rows x 128 bytes (64 k of a vector: a whole slice).  The vector
//            cache works by 128-byte lines, and a request that takes 64 bytes from each of 16
//            rows costs it twice the lines of one that takes 8 whole ones.  A unit is free when
//            its slice is done; its 16-byte chunks are XOR-swizzled with bits 1..3 of the row
//            index (128-bit operand reads of 16 consecutive rows fall on distinct banks).
//   weights  four slots of 32 k-rows x BT columns (half a slice) as they lie in memory, read
//            with the transposing LDS read (see the offset table in the kernel).  A slot is
//            free half a slice after its first read.
// Every request has at least one slice period to land.  WR x WC wavefronts share a BT x BT tile.
// ---------------------------------------------------------------------------
template <int BT, int WR, int WC>
__global__ __launch_bounds__(64 * WR * WC, (WR * WC) / 4 * (BT == 256 ? 1 : 2))
void proj_dma_kernel(int Bsz, int N, int Npad, int D, int H, int d, const bf16_t* __restrict__ X,
                     const bf16_t* __restrict__ Wq, const bf16_t* __restrict__ Wk, const bf16_t* __restrict__ Wv,
                     h16_t* __restrict__ qo, h16_t* __restrict__ ko, h16_t* __restrict__ vto, int tiles_x,
                     int tiles_w, float qscale, const int* __restrict__ lens, bool skip_q_rows, bool no_q,
                     const int* __restrict__ row0, unsigned long long* __restrict__ counters)
{
    constexpr int NW = WR * WC;
    constexpr int TA = BT / WR, TB = BT / WC;    // wavefront tile: TA rows of the A side, TB of the B side
    constexpr int NA = TA / 32, NBK = TB / 32;   // MFMA blocks per edge
    constexpr int XU = BT * 128;                 // bytes of one x unit: BT rows x 64 k
    constexpr int NXU = 3;
    constexpr int WROWB = BT * 2;                // bytes of one k-row of the weight side in a slot
    constexpr int WS = 32 * WROWB;               // bytes of one weight slot: 32 k-rows
    constexpr int NWS = 4;
    constexpr int W_BASE = NXU * XU;
    constexpr int XPW = (BT / 8) / NW;           // x pieces (1 KiB: 8 rows x 128 bytes) per wavefront and slice
    constexpr int WPW = (WS / 1024) / NW;        // weight pieces (1 KiB) per wavefront and half slice
    static_assert(XPW == 4 && WPW == 2, "the request schedule below deals 4 + 2 + 2 requests per slice");
    constexpr int WCPR = WROWB / 16;             // 16-byte chunks of a weight k-row
    constexpr int WRPP = 64 / WCPR;              // k-rows per 1 KiB piece
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NXU * XU + NWS * WS];
    clear_counters(counters);  // this is the first kernel of a forward pass on this path

    const int tid = threadIdx.x;
    const int lane = tid & 63, ln = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave / WC, wc = wave % WC;
    const int HD = H * d;

    const int n_tiles = tiles_x * tiles_w;
    const int per_xcd = gridDim.x >> 3;
    const int tile_id = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile_id >= n_tiles) return;
    int tw, tx_;
    // no_q (the queries are not wanted: q = k = v scheme, or projected by the attention kernel): the
    // grid holds the k and v column tiles only
    tile_of(tile_id, tiles_x, tiles_w, tw, tx_, lens != nullptr ? (no_q ? 2 : 3) : GROUP_W);
    if (lens != nullptr) spread_tiles(tiles_x, tiles_w, tw, tx_, no_q ? 2 : 3);
    const int x0 = tx_ * BT, w0 = tw * BT + (no_q ? HD : 0);
    const bool is_v = w0 >= 2 * HD;
    // Keys past the key length of their batch item are in no allowed pair (Sec. 5.1 applied to
    // padding): their k and v rows are not computed.  (q rows are: every query row has an output.)
    // With padded rows left out as queries too, the same holds for their q rows.
    if (lens != nullptr && (w0 >= HD || skip_q_rows) && past_key_length(lens, x0, Npad, N)) return;

    // The weights stay in the caller's layout, W[k][column]: this tile's columns of the one matrix
    // it lies in.
    const int which = w0 / HD;
    const bf16_t* Wm = (which == 0 ? Wq : (which == 1 ? Wk : Wv)) + (w0 - which * HD);

    // Source byte offsets of this lane for its pieces.  32 bits hold them (attn_init bounds the
    // element counts), which lets a request take a uniform 64-bit base and this offset.
    //   x side: rows are vectors, 128 bytes (64 k) each; piece m = wave + NW*u holds rows
    //           8m..8m+7; the lane lands at row 8m + lane/8, chunk position lane%8;
    //   w side: rows are k, BT columns each; piece m holds k-rows m*WRPP..; the lane lands at
    //           k-row m*WRPP + lane/WCPR, chunk position lane%WCPR.
    // Either way it fetches the chunk that the swizzle of its row puts at that position.
    unsigned xoff[XPW], woff[WPW];
#pragma unroll
    for (int u = 0; u < XPW; ++u) {
        const int row = (wave + NW * u) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);
        const int xr = x0 + row;
        const int bb = xr / Npad;
        xoff[u] = 2u * (source_row(row0, Bsz, N, bb, xr - bb * Npad) * (unsigned)D + c * 8);
    }
#pragma unroll
    for (int u = 0; u < WPW; ++u) {
        const int kr = (wave + NW * u) * WRPP + lane / WCPR;
        const int wc16 = (lane % WCPR) ^ (4 * (kr & 3));
        woff[u] = 2u * ((unsigned)kr * (unsigned)HD + wc16 * 8);
    }
    // Buffer addressing: descriptor base + the lane's 32-bit offset + a scalar offset for the
    // slice, so that a request costs no vector instruction for its address.
    const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)X, 0, -1, 0x00020000);
    const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)Wm, 0, -1, 0x00020000);
    // piece u of the x side of the slice that starts at k0, into unit `unit`
    auto req_x = [&](int u, int k0, int unit) {
        unsigned char* dst = lds + unit * XU + (wave + NW * u) * 1024;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(x_rsrc, (__attribute__((address_space(3))) void*)dst, 16,
                                                 (int)xoff[u], (int)(2u * (unsigned)k0), 0, 0);
    };
    // piece u of half h of the weight side of the slice that starts at k0, into slot `slot`
    auto req_w = [&](int u, int k0, int h, int slot) {
        unsigned char* dst = lds + W_BASE + slot * WS + (wave + NW * u) * 1024;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rsrc, (__attribute__((address_space(3))) void*)dst, 16,
                                                 (int)woff[u], (int)(2u * (unsigned)(k0 + 32 * h) * (unsigned)HD), 0, 0);
    };

    // LDS byte offsets of this lane's operand reads, from the unit / slot base, for the first
    // 32-row block of the wavefront's share of each side.
    //   x side: 128 bits = 8 k of row ln, chunk 2*ks + g of the four k-steps of a slice; 2*ks has no
    //           bit in common with g, so the offset for k-step ks is the one for k-step 0 XOR 32*ks.
    //   w side: stored k-major, read with the transposing 64-bit LDS read: 16 lanes hand in the
    //           addresses of a 4 (k) x 16 (columns) patch, four columns each, and lane i gets
    //           column i of the patch, its four k values.  Lanes 16..31 take the next 16 columns,
    //           the upper half of the wavefront the upper 8 k of the k-step; two reads (4 k each)
    //           make one operand.  k-rows are BT*2 bytes apart, a multiple of the 256 bytes the
    //           banks span, and LDS serves 32 lanes (two patches, 4 k x 32 columns) at a time, so
    //           the chunks of k-row k are XOR-ed with 4*(k%4): the four 64-byte runs then fall on
    //           different banks.  That XOR reaches bits 2 and 3 of the chunk index, which is also
    //           where the 32-column block number sits: one table per block.
    const int x_row0 = is_v ? wr * TA : wc * TB;  // first x row / first w column of this wavefront
    const int w_col0 = is_v ? wc * TB : wr * TA;
    constexpr int NWB = NA > NBK ? NA : NBK;  // 32-column blocks of the weight side of a wavefront
    int wfo[NWB];  // w side: k-step 0, first read; the others lie whole k-rows further (same k % 4)
    const int xfo0 = (x_row0 + ln) * 128 + ((g ^ ((ln >> 1) & 7)) << 4);  // x_row0 is a multiple of 32
#pragma unroll
    for (int blk = 0; blk < NWB; ++blk) {
        const int i16 = lane & 15;
        const int k = 8 * g + (i16 >> 2);
        const int col = w_col0 + 32 * blk + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
        wfo[blk] = k * WROWB + (((col >> 3) ^ (4 * (k & 3))) << 4) + ((col & 7) << 1);
    }

    f32x16 acc[NA][NBK];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int b = 0; b < NBK; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // One k-step = the MFMAs of 16 k values on fragments that are already in registers.  Behind
    // the first MFMAs go, two at a time, the reads of the fragments of the following k-step (order
    // a0, b0.., a1..: what its first MFMAs need comes first); nd requests (numbers q0 .. q0+nd-1 of
    // a slice) are spread over the MFMAs: a wavefront that sends all requests of a slice in one run
    // issues no MFMA meanwhile, and since all wavefronts do so at the same point the matrix pipe
    // would drain.  The order is pinned with scheduling fences; the group-barrier solver drops its
    // pattern as soon as memory requests are part of it.
    u32x4 af[2][NA], bf[2][NBK];
    // ks4: k-step of the slice, 0..3
    auto x_frag = [&](const unsigned char* unit_base, int ks4, int blk) -> u32x4 {
        return *(const u32x4*)(unit_base + (xfo0 ^ (32 * ks4)) + blk * 4096);
    };
    // The transposing reads are written out by hand: as a builtin, the compiler takes them to
    // alias the copies into LDS that are still in flight and makes each of them wait for all of
    // those (vmcnt(0)), which is the prefetch gone.  It does not count hand-written requests, so
    // every k-step starts with its own wait for the LDS reads of the one before.
    const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)lds;
    auto w_frag = [&](const unsigned char* slot_base, int ks, int blk) -> u32x4 {
        const unsigned addr = lds_addr + (unsigned)(slot_base - lds) + (unsigned)wfo[blk];
        u32x2 lo, hi;
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "n"(16 * ks * WROWB));
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(addr), "n"((16 * ks + 4) * WROWB));
        return u32x4{lo[0], lo[1], hi[0], hi[1]};
    };
    // fragment number r of a k-step, in the order a0, b0.., a1..; the weights are the A side of q and
    // k tiles and the B side of v tiles
    // hs: half slice 0 / 1 of x unit `unit` and weight slot `slot`; ks: k-step 0 / 1 of the half slice
    auto read_frag = [&](auto is_v_, u32x4 (&fa)[NA], u32x4 (&fb)[NBK], int r, const unsigned char* unit_base,
                         const unsigned char* slot_base, int hs, int ks) {
        constexpr bool IS_V = decltype(is_v_)::value;
        if (r == 0 || r > NBK) {
            const int a = r == 0 ? 0 : r - NBK;
            fa[a] = IS_V ? x_frag(unit_base, 2 * hs + ks, a) : w_frag(slot_base, ks, a);
        } else {
            fb[r - 1] = IS_V ? w_frag(slot_base, ks, r - 1) : x_frag(unit_base, 2 * hs + ks, r - 1);
        }
    };
    auto load_frags = [&](auto is_v_, u32x4 (&fa)[NA], u32x4 (&fb)[NBK], int unit, int slot, int hs, int ks) {
#pragma unroll
        for (int r = 0; r < NA + NBK; ++r)
            read_frag(is_v_, fa, fb, r, lds + unit * XU, lds + W_BASE + slot * WS, hs, ks);
    };
    // `reqs(i)`, i = 0 .. ND-1: the requests that go out behind the MFMAs of this k-step
    auto kstep = [&](auto is_v_, const u32x4 (&fa)[NA], const u32x4 (&fb)[NBK], u32x4 (&na)[NA], u32x4 (&nb)[NBK],
                     int unit, int slot, int hs, int ks, auto nd_, auto&& reqs) {
        constexpr int ND = decltype(nd_)::value;
        constexpr int NRD = NA + NBK, NMF = NA * NBK;
        static_assert(NRD % 2 == 0 && NRD / 2 <= NMF, "read pairs fit behind the MFMAs of a k-step");
        static_assert(ND <= NMF, "at most one request per MFMA");
        const unsigned char* unit_base = lds + unit * XU;
        const unsigned char* slot_base = lds + W_BASE + slot * WS;
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the fragments of this k-step are in
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int b = 0; b < NBK; ++b) {
                acc[a][b] = mfma32(fa[a], fb[b], acc[a][b]);
                const int m = a * NBK + b + 1;  // MFMAs issued so far
                if (m <= NRD / 2) {
                    read_frag(is_v_, na, nb, 2 * m - 2, unit_base, slot_base, hs, ks);
                    read_frag(is_v_, na, nb, 2 * m - 1, unit_base, slot_base, hs, ks);
                }
                if (ND > 0 && (m * ND) % NMF == 0) reqs(m * ND / NMF - 1);
                __builtin_amdgcn_sched_barrier(0);
            }
    };
    constexpr std::integral_constant<int, 0> no_req{};
    constexpr std::integral_constant<int, 1> one_req{};
    constexpr std::integral_constant<int, 2> two_req{};

    // Slice j: x in unit ux, its two weight half slices in slots wa and wa+1.  A k-step runs the
    // MFMAs of fragments that are in registers and reads those of the next k-step.  The barrier
    // of a half slice sits before its second k-step, whose fragments are in registers by then:
    // behind the first barrier (A) slot wa is free, behind the second (B) slot wa+1 and unit ux,
    // and the matrix pipe has work on both sides of either.  Each k-step sends two requests for
    // what has just become free, the weight piece first:
    //     step 1   weights (j+1, half 1) piece 1  -> slot wa+3      x (j+2) piece 0 -> unit ux+2
    //     step 2   weights (j+2, half 0) piece 0  -> slot wa        x (j+2) piece 1
    //     step 3   weights (j+2, half 0) piece 1  -> slot wa        x (j+2) piece 2
    //     step 4   weights (j+2, half 1) piece 0  -> slot wa+1      x (j+2) piece 3
    // Loads return in order.  Barrier B wants x (j+1) and the first weight half of slice j+1 in,
    // whose last piece went out in step 4 of slice j-1: the six requests of steps 1-3 may be in
    // flight.  Barrier A wants the second weight half of slice j in, whose last piece went out
    // first in step 1 of slice j-1: nine requests may be in flight.  VAR: 2 if slice j+2 exists,
    // 1 if slice j+1 is the last, 0 if slice j is.
    auto slice = [&](auto is_v_, auto var_, int j, int& ux, int& wa) {
        constexpr int VAR = decltype(var_)::value;
        constexpr bool E1 = VAR >= 1, E2 = VAR == 2;
        const int ux1 = ux == NXU - 1 ? 0 : ux + 1, ux2 = ux1 == NXU - 1 ? 0 : ux1 + 1;
        const int wb = (wa + 1) & 3, wc = (wa + 2) & 3, wd = (wa + 3) & 3;
        const int k1 = (j + 1) * 64, k2 = (j + 2) * 64;
        kstep(is_v_, af[0], bf[0], af[1], bf[1], ux, wa, 0, 1, std::integral_constant<int, (E1 ? 1 : 0) + (E2 ? 1 : 0)>{},
              [&](int i) {
                  if (E1 && i == 0) req_w(1, k1, 1, wd);
                  else req_x(0, k2, ux2);
              });
        __builtin_amdgcn_s_waitcnt(0x0070 | (8 * (E1 ? 1 : 0) + (E2 ? 1 : 0)));  // lgkmcnt(0), see above
        __builtin_amdgcn_s_barrier();
        kstep(is_v_, af[1], bf[1], af[0], bf[0], ux, wb, 1, 0, std::integral_constant<int, E2 ? 2 : 0>{}, [&](int i) {
            if (i == 0) req_w(0, k2, 0, wa);
            else req_x(1, k2, ux2);
        });
        kstep(is_v_, af[0], bf[0], af[1], bf[1], ux, wb, 1, 1, std::integral_constant<int, E2 ? 2 : 0>{}, [&](int i) {
            if (i == 0) req_w(1, k2, 0, wa);
            else req_x(2, k2, ux2);
        });
        __builtin_amdgcn_s_waitcnt(0x0070 | ((E1 ? 1 : 0) + 5 * (E2 ? 1 : 0)));
        __builtin_amdgcn_s_barrier();
        // reads ahead into slice j+1
        kstep(is_v_, af[1], bf[1], af[0], bf[0], ux1, wc, 0, 0, std::integral_constant<int, E2 ? 2 : 0>{}, [&](int i) {
            if (i == 0) req_w(0, k2, 1, wb);
            else req_x(3, k2, ux2);
        });
        ux = ux1;
        wa = wc;
    };

    // Prologue: slice 0 whole, and of slice 1 what steps 2-4 of a slice before slice 0 would
    // have sent (its last weight piece follows in step 1 of slice 0).
    const int ns = D / 64;
    req_w(0, 0, 0, 0);
    req_w(1, 0, 0, 0);
#pragma unroll
    for (int u = 0; u < XPW; ++u) req_x(u, 0, 0);
    req_w(0, 0, 1, 1);
    req_w(1, 0, 1, 1);
    if (ns > 1) {
        req_x(0, 64, 1);
        req_w(0, 64, 0, 2);
        req_x(1, 64, 1);
        req_w(1, 64, 0, 2);
        req_x(2, 64, 1);
        req_w(0, 64, 1, 3);
        req_x(3, 64, 1);
        __builtin_amdgcn_s_waitcnt(0x0F70 | 7);  // loads return in order: slice 0 has landed
    } else {
        __builtin_amdgcn_s_waitcnt(0x0F70);
    }
    __builtin_amdgcn_s_barrier();
    auto all_slices = [&](auto is_v_) {
        load_frags(is_v_, af[0], bf[0], 0, 0, 0, 0);
        int ux = 0, wa = 0;
        int j = 0;
#pragma nounroll
        for (; j + 2 < ns; ++j) slice(is_v_, two_req, j, ux, wa);
#pragma nounroll
        for (; j + 1 < ns; ++j) slice(is_v_, one_req, j, ux, wa);
#pragma nounroll
        for (; j < ns; ++j) slice(is_v_, no_req, j, ux, wa);
    };
    if (is_v) all_slices(std::true_type{});
    else all_slices(std::false_type{});
    __builtin_amdgcn_s_waitcnt(0x0070);  // the fragments read ahead for a slice that does not exist are dropped
    __builtin_amdgcn_s_barrier();

    // Epilogue.  acc[a][b][r]: A-side row wr*TA + 32a + acc_row(r,g), B-side row wc*TB + 32b + ln.
    // A lane owns 8-byte runs whose neighbours in memory sit in other lanes' later registers, so
    // storing them directly would touch 64 cache lines per instruction.  The tile is staged in LDS
    // (free by now) in the order of the output arrays and leaves in 16-byte pieces, a full KiB of
    // consecutive addresses per wavefront and instruction.  Staged rows are XOR-swizzled by 16-byte
    // chunk like the operand tiles, which keeps both the 8-byte writes and the 16-byte reads spread
    // over the banks.
    constexpr int NT = 64 * NW;
    constexpr int UNITS = BT * BT / 8;  // 16-byte pieces of the tile
    const int dsh = d == 128 ? 7 : 6;   // d is 64 or 128 on this path
    const int bb = x0 / Npad;           // Npad is a multiple of BT: one batch element per tile
    const int i0 = x0 - bb * Npad;
    if (!is_v) {
        // q and k: [head][vector][d], a staged row is one vector's d values of one head.
        const int which = w0 >= HD ? 1 : 0;
        const float qs = which ? 1.f : qscale;  // q is stored pre-multiplied (see launch_proj_mfma)
        const int cmask = (d >> 3) - 1, rowb = 2 * d;
#pragma unroll
        for (int b = 0; b < NBK; ++b) {
            const int v = wc * TB + 32 * b + ln;
#pragma unroll
            for (int a = 0; a < NA; ++a)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int ct = wr * TA + 32 * a + 8 * r4;  // tile column of register 4*r4 in half 0
                    const int hc = ct >> dsh, c = (ct & (d - 1)) >> 3;
                    u32x2 w;
                    w[0] = pack_f16_sat(acc[a][b][4 * r4 + 0] * qs, acc[a][b][4 * r4 + 1] * qs);
                    w[1] = pack_f16_sat(acc[a][b][4 * r4 + 2] * qs, acc[a][b][4 * r4 + 3] * qs);
                    *(u32x2*)(lds + (hc * BT + v) * rowb + ((c ^ (v & cmask)) << 4) + 8 * g) = w;
                }
        }
        __syncthreads();
        h16_t* base = (which ? ko : qo) + ((size_t)bb * H + ((w0 - which * HD) >> dsh)) * Npad * d;
#pragma unroll 4
        for (int e0 = tid; e0 < UNITS; e0 += NT) {
            const int hv = e0 >> (dsh - 3);  // head-in-tile * BT + vector
            const int c = e0 & cmask;
            const int hc = hv / BT, v = hv - hc * BT;
            if (i0 + v >= N) continue;  // rows past n stay zero
            const u32x4 val = *(const u32x4*)(lds + hv * rowb + ((c ^ (v & cmask)) << 4));
            *(u32x4*)(base + ((size_t)hc * Npad + i0 + v) * d + c * 8) = val;
        }
    } else {
        // v transposed: [head][64-key block][d][64 key slots], a staged row is the 64 slots of one
        // column; vectors past n are staged as zeros.
#pragma unroll
        for (int b = 0; b < NBK; ++b) {
            const int cl = wc * TB + 32 * b + ln;
            const int hc = cl >> dsh, l = cl & (d - 1);
#pragma unroll
            for (int a = 0; a < NA; ++a)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int vl = wr * TA + 32 * a + 8 * r4 + 4 * g;  // vector of register 4*r4
                    const int vb = vl >> 6, r64 = vl & 63;
                    const int slot = (r64 & 48) | vt_slot16(r64 & 15);
                    const int left = N - (i0 + vl);
                    u32x2 w;
                    w[0] = pack_f16_sat(left > 0 ? acc[a][b][4 * r4 + 0] : 0.f, left > 1 ? acc[a][b][4 * r4 + 1] : 0.f);
                    w[1] = pack_f16_sat(left > 2 ? acc[a][b][4 * r4 + 2] : 0.f, left > 3 ? acc[a][b][4 * r4 + 3] : 0.f);
                    *(u32x2*)(lds + ((hc * (BT / 64) + vb) * d + l) * 128 + (((slot >> 3) ^ (l & 7)) << 4) +
                              2 * (slot & 7)) = w;
                }
        }
        __syncthreads();
        const int h0 = (w0 - 2 * HD) >> dsh;
#pragma unroll 4
        for (int e0 = tid; e0 < UNITS; e0 += NT) {
            const int ul = e0 >> 3;  // (head-in-tile * blocks + block) * d + column
            const int c = e0 & 7;
            const int u = ul >> dsh, l = ul & (d - 1);
            const int hc = u / (BT / 64), vb = u - hc * (BT / 64);
            const int blk = (i0 >> 6) + vb;
            if (blk * 64 >= N) continue;  // blocks past n stay zero
            const u32x4 val = *(const u32x4*)(lds + ul * 128 + ((c ^ (l & 7)) << 4));
            *(u32x4*)(vto + ((((size_t)bb * H + h0 + hc) * (Npad >> 6) + blk) * d + l) * 64 + c * 8) = val;
        }
    }
}

// The stored q carries the score scale and the change to base-2 exponentials:
// q' = q * scale * log2(e), applied to the fp32 accumulator before the one rounding to
// half precision, so that the attention kernels get base-2 scores straight out of the MFMA.
inline float q_prescale(const Problem& pb) { return pb.scale * 1.4426950408889634f; }

template <int BT, int WR, int WC>
hipError_t launch_dma(const Problem& pb, const bf16_t* X, const bf16_t* Wq, const bf16_t* Wk, const bf16_t* Wv,
                      h16_t* q, h16_t* k, h16_t* vt, hipStream_t s)
{
    const float qscale = q_prescale(pb);
    const int tiles_x = pb.B * pb.Npad / BT;
    const int tiles_w = (pb.no_q ? 2 : 3) * pb.H * pb.d / BT;
    const int grid = ((tiles_x * tiles_w + 7) / 8) * 8;
    hipLaunchKernelGGL((proj_dma_kernel<BT, WR, WC>), dim3(grid), dim3(64 * WR * WC), 0, s, pb.B, pb.N, pb.Npad, pb.D,
                       pb.H, pb.d, X, Wq, Wk, Wv, q, k, vt, tiles_x, tiles_w, qscale, pb.noskip ? nullptr : pb.lens,
                       pb.skip_rows, pb.no_q, pb.row0, pb.counters);
    return hipGetLastError();
}

template <int BT>
hipError_t launch_bt(const Problem& pb, const bf16_t* X, const bf16_t* Wt, h16_t* q, h16_t* k, h16_t* vt,
                     hipStream_t s)
{
    const float qscale = q_prescale(pb);
    const int tiles_x = pb.B * pb.Npad / BT;
    const int tiles_w = 3 * pb.H * pb.d / BT;
    const int grid = ((tiles_x * tiles_w + 7) / 8) * 8;
    hipLaunchKernelGGL(proj_mfma_kernel<BT>, dim3(grid), dim3(256), 0, s, pb.B, pb.N, pb.Npad, pb.D, pb.H, pb.d, X, Wt,
                       q, k, vt, tiles_x, tiles_w, qscale, pb.noskip ? nullptr : pb.lens, pb.skip_rows, pb.no_q, pb.row0);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_transpose_w(const Problem& pb, const bf16_t* Wq, const bf16_t* Wk, const bf16_t* Wv, bf16_t* Wt,
                              hipStream_t s)
{
    const int HD = pb.H * pb.d;
    const dim3 grid(HD / 64, (pb.D + 63) / 64, 3);
    const bool aligned16 = ((reinterpret_cast<uintptr_t>(Wq) | reinterpret_cast<uintptr_t>(Wk) |
                             reinterpret_cast<uintptr_t>(Wv) | reinterpret_cast<uintptr_t>(Wt)) & 15) == 0 &&
                           pb.D % 8 == 0;
    if (aligned16)
        hipLaunchKernelGGL(transpose_w16_kernel, grid, dim3(256), 0, s, pb.D, HD, Wq, Wk, Wv, Wt, pb.counters);
    else
        hipLaunchKernelGGL(transpose_w_kernel, grid, dim3(256), 0, s, pb.D, HD, Wq, Wk, Wv, Wt, pb.counters);
    return hipGetLastError();
}

// Whether the projection reads the weights where the caller has them (no W^T, no re-layout
// kernel): d_model in whole 64-deep slices, and 16-byte aligned weights for the 16-byte copies.
bool proj_reads_weights_in_place(const Problem& pb, const bf16_t* Wq, const bf16_t* Wk, const bf16_t* Wv)
{
    const int HD = pb.H * pb.d;
    const bool aligned16 = ((reinterpret_cast<uintptr_t>(Wq) | reinterpret_cast<uintptr_t>(Wk) |
                             reinterpret_cast<uintptr_t>(Wv)) & 15) == 0;
    return pb.D % 64 == 0 && HD % 128 == 0 && aligned16;
}

hipError_t launch_proj_mfma(const Problem& pb, const bf16_t* X, const bf16_t* Wq, const bf16_t* Wk,
                            const bf16_t* Wv, const bf16_t* Wt, h16_t* q, h16_t* k, h16_t* vt, hipStream_t s)
{
    // Largest square tile that divides the per-matrix column count (so a tile never
    // mixes q, k and v columns) and still gives every CU a few tiles.
    const int HD = pb.H * pb.d;
    const long rows = (long)pb.B * pb.Npad;
    const bool big = HD % 256 == 0 && rows % 256 == 0 && (rows / 256) * ((pb.no_q ? 2L : 3L) * HD / 256) >= 512;
    if (proj_reads_weights_in_place(pb, Wq, Wk, Wv)) {  // operands go straight to LDS
        if (big) return launch_dma<256, 2, 4>(pb, X, Wq, Wk, Wv, q, k, vt, s);
        return launch_dma<128, 2, 2>(pb, X, Wq, Wk, Wv, q, k, vt, s);
    }
    if (HD % 128 == 0) return launch_bt<128>(pb, X, Wt, q, k, vt, s);
    return launch_bt<64>(pb, X, Wt, q, k, vt, s);
}

}  // namespace attnring
