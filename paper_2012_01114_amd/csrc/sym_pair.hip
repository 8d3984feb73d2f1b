// The q = k = v scheme (Sec. 4) on the matrix cores, with the reuse kept on chip.
//
// Eq. (4): with one set of vectors z in all three roles, w'_ij = w'_ji, so phase 1 needs one
// element of every symmetric pair; phases 2 and 3 do not share it (Sec. 4.1).  Here the unit of
// reuse is a 128 x 128 score tile.  Workgroup (A, B), A >= B, computes S_AB = z_A . z_B^T once with
// MFMAs and uses it twice:
//     as it stands      for the rows of A against the keys of B   (phases 2 and 3 of row block A)
//     transposed        for the rows of B against the keys of A   (phases 2 and 3 of row block B)
// The transposition goes through LDS: the tile is stored as fp32 while the first use runs from
// registers, and read back in the accumulator layout of the other orientation, so the second use
// runs the very code of the first.  Each use yields a partial row state (m, l, O) over 128 keys;
// the T = n/128 partial states of a row block (one per key tile, whichever workgroup made them) are
// merged by a second kernel.  The scores never leave the chip; what does is 128 (d + 2) floats per
// use.  Tiles on the diagonal (A == B) are used once.
//
// The paper's selection rule (Sec. 4.2: circulant diagonals 0 .. floor(P/2) of the P x P matrix of
// (n/P)-row tiles, the middle one computed by both owners when P is even) fixes WHICH element of a
// pair a ring of P processing elements computes.  On 128-row tiles every unordered pair of tiles
// is simply computed once; the count of logical tiles the rule selects is taken on the device over
// the regions the kernel covers (each position of the P x P matrix lies in exactly one use).
//
// Both operands of the score MFMAs are the same half-precision z (the scale is applied to the
// fp32 scores), so S_AB and S_BA^T are equal bit for bit, as Eq. (4) has it; with every tile
// computed in its own orientation instead (the debug mode) the outputs are the same bits.
#include "attn_common.h"

namespace attnring {
namespace {

constexpr int ST = 128;           // rows and keys of a score tile
constexpr int SPITCH = ST + 4;    // floats per row of the staged tile: 16 lanes x 16 bytes meet 64 banks once

template <int DK>
struct Sym {
    static constexpr int NKS = DK / 16, NDB = DK / 32;
    static constexpr int KROWB = DK * 2;             // bytes of a key row in LDS
    static constexpr int K_BYTES = ST * KROWB;       // K tile: 128 keys
    static constexpr int V_TILE = DK * 64 * 2;       // one 64-key block of V^T
    static constexpr int V_BYTES = 2 * V_TILE;
    static constexpr int S_BYTES = ST * SPITCH * 4;
    static constexpr int LDS_BYTES = K_BYTES + V_BYTES + S_BYTES;
};

// z rows [row0, row0 + 128) of one head as a K tile: rows of KROWB bytes, 16-byte chunks swizzled.
template <int DK>
__device__ __forceinline__ void load_k_tile(unsigned char* dst, const h16_t* kh, int row0, int tid)
{
    constexpr int CPR = DK / 8;
    const u32x4* src = (const u32x4*)(kh + (size_t)row0 * DK);
#pragma unroll
    for (int c = tid; c < ST * CPR; c += 256) {
        const int row = c / CPR, p = c % CPR;
        *(u32x4*)(dst + row * (DK * 2) + swz<DK * 2>(p, row) * 16) = src[c];
    }
}
// V^T of the same rows: two 64-key blocks of [DK][64], rows of 128 bytes, chunks swizzled.
template <int DK>
__device__ __forceinline__ void load_vt_tile(unsigned char* dst, const h16_t* vth, int row0, int tid)
{
    const u32x4* src = (const u32x4*)(vth + (size_t)(row0 >> 6) * DK * 64);
#pragma unroll
    for (int c = tid; c < 2 * DK * 8; c += 256) {
        const int row = c >> 3, p = c & 7;  // row: block * DK + column of v
        *(u32x4*)(dst + row * 128 + swz<128>(p, row % DK) * 16) = src[c];
    }
}

// Phases 2 and 3 (Eq. (2), (3)) of 32 rows (one per lane pair) over the 128 keys of a tile whose
// scores S[kb][r] are in accumulator layout (key kb * 32 + acc_row(r, g)); keys at or past
// `keys_left` are not there.  V^T of the tile in LDS at vt.  Writes the partial state.
template <int DK>
__device__ __forceinline__ void softmax_pv_store(f32x16 (&S)[4], int keys_left, const unsigned char* vt, int ln, int g,
                                                 bool row_live, float* __restrict__ pm, float* __restrict__ pl,
                                                 float* __restrict__ po)
{
    constexpr int NDB = DK / 32;
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = kb * 32 + acc_row(r, g);
            S[kb][r] = key < keys_left ? S[kb][r] : -INFINITY;
            mx = fmaxf(mx, S[kb][r]);
        }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float ref = mx > -INFINITY ? mx : 0.f;
    float l = 0.f;
    f32x16 O[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) O[db][e] = 0.f;
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
        u32x4 P[2];
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float p0 = __builtin_amdgcn_exp2f(S[kb][8 * hf + 2 * w] - ref);
                const float p1 = __builtin_amdgcn_exp2f(S[kb][8 * hf + 2 * w + 1] - ref);
                P[hf][w] = pack_f16(p0, p1);
                l += p0 + p1;
            }
        const unsigned char* blk = vt + (kb >> 1) * (DK * 128);
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                const int row = db * 32 + ln;
                const int chunk = swz<128>(2 * hf + g, row) ^ (4 * (kb & 1));
                const u32x4 vf = *(const u32x4*)(blk + row * 128 + chunk * 16);
                O[db] = mfma32h(vf, P[hf], O[db]);
            }
    }
    l += __shfl_xor(l, 32, 64);
    if (row_live) {
        if (g == 0) { *pm = mx; *pl = l; }
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                f32x4 v = {O[db][4 * r4 + 0], O[db][4 * r4 + 1], O[db][4 * r4 + 2], O[db][4 * r4 + 3]};
                *(f32x4*)(po + db * 32 + 8 * r4 + 4 * g) = v;
            }
    }
}

// Grid: (pairs, batch * heads).  all_ordered: every ordered pair of tiles computed in its own
// orientation, nothing reused (the debug mode); else the unordered pairs A >= B.
template <int DK>
__global__ __launch_bounds__(256) void sym_pair_kernel(Problem pb, CountCfg cc, const h16_t* __restrict__ z,
                                                       const h16_t* __restrict__ zt, float* __restrict__ part_m,
                                                       float* __restrict__ part_l, float* __restrict__ part_o,
                                                       int T, bool all_ordered, float c2)
{
    typedef Sym<DK> Y;
    constexpr int NKS = Y::NKS;
    __shared__ __attribute__((aligned(16))) unsigned char lds[Y::LDS_BYTES];
    unsigned char* kt = lds;
    unsigned char* vt = lds + Y::K_BYTES;
    float* sc = (float*)(lds + Y::K_BYTES + Y::V_BYTES);

    const int tid = threadIdx.x, lane = tid & 63, ln = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int bh = blockIdx.y;
    int A, B;
    if (all_ordered) {
        A = blockIdx.x / T;
        B = blockIdx.x - A * T;
    } else {
        A = (int)((sqrtf(8.f * (float)blockIdx.x + 1.f) - 1.f) * 0.5f);
        while (A * (A + 1) / 2 > (int)blockIdx.x) --A;
        while ((A + 1) * (A + 2) / 2 <= (int)blockIdx.x) ++A;
        B = blockIdx.x - A * (A + 1) / 2;
    }
    const int N = pb.N, Npad = pb.Npad;
    const h16_t* zh = z + (size_t)bh * Npad * DK;
    const h16_t* zth = zt + (size_t)bh * Npad * DK;
    const bool twice = !all_ordered && A != B;

    // ---- counts: logical tiles the selection rule picks, over the regions this workgroup covers ----
    {
        unsigned long long cnt = 0;
        const int ia0 = (int)cdiv_b(A * ST, cc), ia1 = (int)cdiv_b(min((A + 1) * ST, N), cc);
        const int ib0 = (int)cdiv_b(B * ST, cc), ib1 = (int)cdiv_b(min((B + 1) * ST, N), cc);
        const int na = ia1 - ia0, nb = ib1 - ib0, P = pb.P;
        for (int e = tid; e < na * nb; e += 256) {
            const int I = ia0 + e / nb, J = ib0 + e % nb;
            const int gd = ((I - J) % P + P) % P, gt = ((J - I) % P + P) % P;
            cnt += (all_ordered || 2 * gd <= P) ? 1u : 0u;          // region (A, B)
            if (twice) cnt += (2 * gt <= P) ? 1u : 0u;              // region (B, A), met transposed
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
        // 32 x 32 score blocks issued: the key blocks that hold a key, for a wavefront that holds a row
        unsigned phys = 0;
        if (A * ST + wave * 32 < N) phys = (unsigned)min(4, (N - B * ST + 31) / 32);
        if (lane == 0) count_add(pb.counters, (unsigned)(blockIdx.y * gridDim.x + blockIdx.x) * 4u + wave, cnt, phys);
    }

    // ---- phase 1 (Eq. (1)), once: S^T = z_B . z_A^T, the wavefront's 32 rows of A against 128 keys of B ----
    load_k_tile<DK>(kt, zh, B * ST, tid);
    load_vt_tile<DK>(vt, zth, B * ST, tid);
    const int ia = A * ST + wave * 32 + ln;  // this lane's row of A
    u32x4 qf[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[ks] = *(const u32x4*)(zh + (size_t)ia * DK + ks * 16 + g * 8);
    __syncthreads();
    f32x16 S[4];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
#pragma unroll
        for (int e = 0; e < 16; ++e) S[kb][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const int row = kb * 32 + ln;
            const u32x4 kf = *(const u32x4*)(kt + row * Y::KROWB + swz<Y::KROWB>(2 * ks + g, row) * 16);
            S[kb] = mfma32h(kf, qf[ks], S[kb]);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) S[kb][e] *= c2;  // scale and base-2 exponent, on the fp32 score
        if (twice) {
            // staged for the other orientation: sc[key of B][row of A]
#pragma unroll
            for (int e = 0; e < 16; ++e) sc[(kb * 32 + acc_row(e, g)) * SPITCH + wave * 32 + ln] = S[kb][e];
        }
    }
    {
        const size_t slot = (((size_t)bh * T + A) * T + B) * ST + wave * 32 + ln;
        softmax_pv_store<DK>(S, N - B * ST, vt, ln, g, ia < N, part_m + slot, part_l + slot, part_o + slot * DK);
    }
    if (!twice) return;

    // ---- the same scores, transposed: the wavefront's 32 rows of B against the 128 keys of A ----
    __syncthreads();  // the staged tile is complete, V^T of B no longer needed
    load_vt_tile<DK>(vt, zth, A * ST, tid);
    const int jb_row = wave * 32 + ln;  // this lane's row of B within the tile
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const f32x4 v = *(const f32x4*)(sc + jb_row * SPITCH + kb * 32 + 8 * r4 + 4 * g);
            S[kb][4 * r4 + 0] = v[0]; S[kb][4 * r4 + 1] = v[1]; S[kb][4 * r4 + 2] = v[2]; S[kb][4 * r4 + 3] = v[3];
        }
    __syncthreads();
    {
        const size_t slot = (((size_t)bh * T + B) * T + A) * ST + wave * 32 + ln;
        softmax_pv_store<DK>(S, N - A * ST, vt, ln, g, B * ST + jb_row < N, part_m + slot, part_l + slot,
                             part_o + slot * DK);
    }
}

// y_i = sum over the key tiles of a row of 2^(m_t - M) O_t / sum 2^(m_t - M) l_t, M the largest m_t.
// Grid (T, batch * heads); four rows at a time, a lane per output column.
template <int DK>
__global__ __launch_bounds__(256) void sym_merge_kernel(Problem pb, const float* __restrict__ part_m,
                                                        const float* __restrict__ part_l,
                                                        const float* __restrict__ part_o, bf16_t* __restrict__ out, int T)
{
    const int A = blockIdx.x, bh = blockIdx.y;
    const int bb = bh / pb.H, h = bh - bb * pb.H;
    const int lane = threadIdx.x & 63, sub = threadIdx.x >> 6;
    for (int r0 = 0; r0 < ST; r0 += 4) {
        const int row = r0 + sub, i = A * ST + row;
        if (i >= pb.N) continue;
        const size_t base = (((size_t)bh * T + A) * T) * ST + row;
        float M = -INFINITY;
        for (int t = 0; t < T; ++t) M = fmaxf(M, part_m[base + (size_t)t * ST]);
        float L = 0.f, acc[DK / 64];
#pragma unroll
        for (int u = 0; u < DK / 64; ++u) acc[u] = 0.f;
        for (int t = 0; t < T; ++t) {
            const float m = part_m[base + (size_t)t * ST];
            const float w = m > -INFINITY ? __builtin_amdgcn_exp2f(m - M) : 0.f;
            L += w * part_l[base + (size_t)t * ST];
#pragma unroll
            for (int u = 0; u < DK / 64; ++u) acc[u] += w * part_o[(base + (size_t)t * ST) * DK + lane + 64 * u];
        }
        const float inv = L > 0.f ? 1.f / L : 0.f;
        bf16_t* o = out + ((size_t)bb * pb.N + i) * ((size_t)pb.H * DK) + (size_t)h * DK;
#pragma unroll
        for (int u = 0; u < DK / 64; ++u) {
            unsigned v = __float_as_uint(acc[u] * inv);
            v += 0x7fffu + ((v >> 16) & 1u);  // round to nearest even; the value is finite
            o[lane + 64 * u] = (bf16_t)(v >> 16);
        }
    }
}

}  // namespace

size_t sym_pair_workspace_floats(const Problem& pb)
{
    const size_t T = (size_t)(pb.N + ST - 1) / ST;
    return (size_t)pb.B * pb.H * T * T * ST * (size_t)(pb.d + 2);
}

// z: [B][H][Npad][d] half precision; zt: the same vectors in the transposed layout of the
// attention kernels; work: sym_pair_workspace_floats(pb) floats.
hipError_t launch_sym_pair(const Problem& pb, const h16_t* z, const h16_t* zt, float* work, bf16_t* out, hipStream_t s)
{
    const int T = (pb.N + ST - 1) / ST;
    const size_t rows = (size_t)pb.B * pb.H * T * T * ST;
    float* part_m = work;
    float* part_l = work + rows;
    float* part_o = work + 2 * rows;
    CountCfg cc;
    cc.b = pb.b;
    cc.b_shift = -1;
    for (int sft = 0; sft < 31; ++sft)
        if ((1 << sft) == pb.b) cc.b_shift = sft;
    const float c2 = pb.scale * 1.4426950408889634f;
    const dim3 grid(pb.noskip ? T * T : T * (T + 1) / 2, pb.B * pb.H);
    if (pb.d == 64) {
        hipLaunchKernelGGL(sym_pair_kernel<64>, grid, dim3(256), 0, s, pb, cc, z, zt, part_m, part_l, part_o, T, pb.noskip, c2);
        hipLaunchKernelGGL(sym_merge_kernel<64>, dim3(T, pb.B * pb.H), dim3(256), 0, s, pb, part_m, part_l, part_o, out, T);
    } else if (pb.d == 128) {
        hipLaunchKernelGGL(sym_pair_kernel<128>, grid, dim3(256), 0, s, pb, cc, z, zt, part_m, part_l, part_o, T, pb.noskip, c2);
        hipLaunchKernelGGL(sym_merge_kernel<128>, dim3(T, pb.B * pb.H), dim3(256), 0, s, pb, part_m, part_l, part_o, out, T);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace attnring
