// Fused phases 1-3 (Sec. 3.1, Eq. (1)-(3)) on the bf16 matrix cores of gfx950,
// for the FULL and the masked scheme, with redundant score blocks never issued
// (Sec. 5.1: masked pairs are excluded from all three phases).
//
// Ring mapping.  A wavefront owns 32 consecutive query rows (one or several of
// the paper's PEs, which own n/P rows each); four wavefronts form a workgroup of
// 128 rows.  The workgroup meets the 64-key blocks of its head in ring order,
// starting with the block at its own diagonal and walking down, wrapping round
// for the FULL scheme; blocks with no needed pair are left out of the walk.
// Masked scheme: workgroup x handles row tiles T-1-x and x, the packing of row
// n-i with row i that equalises the work per PE (Sec. 5.2).
//
// Data path per key block: K[64][d] and V^T[d][64] are staged through LDS
// (double buffered, one barrier per block).  Scores are computed transposed,
// S^T = K.Q^T, so that a lane holds 16 keys of ONE query per 32x32 block: the
// row maximum and row sum of the online softmax need one cross-lane exchange,
// and the exponentials, converted to bf16, are already in B-operand layout for
// O^T += V^T.P^T.
#include "mfma_common.h"

namespace attnring {
namespace {

constexpr int BR = 128;  // query rows per workgroup tile
constexpr int BC = 64;   // keys per staged block
constexpr int NTHREADS = 256;

template <int DK>
struct Lds {
    static constexpr int KS = DK * 2 + 16;  // bytes per key row (padded: conflict-free b128 reads)
    static constexpr int VS = BC * 2 + 16;  // bytes per V^T row
    static constexpr int K_BYTES = BC * KS;
    static constexpr int V_BYTES = DK * VS;
    static constexpr int STAGE = K_BYTES + V_BYTES;
};

struct CountCfg {
    int b;        // rows per logical PE
    int b_shift;  // log2(b), or -1 when b is not a power of two
};

// ceil(x / b): the number of multiples of b in [0, x)
__device__ __forceinline__ unsigned cdiv_b(unsigned x, const CountCfg& cc)
{
    const unsigned y = x + (unsigned)cc.b - 1u;
    return cc.b_shift >= 0 ? (y >> cc.b_shift) : y / (unsigned)cc.b;
}

template <int DK, bool CAUSAL>
__global__ __launch_bounds__(NTHREADS, 2) void attn_mfma_kernel(Problem pb, CountCfg cc, const bf16_t* __restrict__ q,
                                                                const bf16_t* __restrict__ k,
                                                                const bf16_t* __restrict__ vt,
                                                                bf16_t* __restrict__ out, int n_qtiles, int per_head,
                                                                int n_work)
{
    typedef Lds<DK> L;
    constexpr int NKS = DK / 16;  // k-steps of the score product
    constexpr int NDB = DK / 32;  // 32-row blocks of O^T
    constexpr int KCH = BC * DK * 2 / 16 / NTHREADS;  // 16-byte chunks per thread, K block
    constexpr int VCH = KCH;                          // V^T block has the same size
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * L::STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63, ln = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // Consecutive workgroup ids go to different XCDs; give each XCD a contiguous
    // run of work items so that the workgroups of one head share an L2.
    const int per_xcd = gridDim.x >> 3;
    const int work = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (work >= n_work) return;
    const int bh = work / per_head;
    const int x = work - bh * per_head;
    const int bb = bh / pb.H, h = bh - bb * pb.H;

    const int N = pb.N, Npad = pb.Npad;
    int len = N;
    if (pb.lens) { len = pb.lens[bb]; len = len < 0 ? 0 : (len > N ? N : len); }
    const int nkt_all = Npad / BC;
    const float c2 = pb.scale * 1.4426950408889634f;  // scores are taken to base 2

    const bf16_t* qh = q + (size_t)bh * Npad * DK;
    const unsigned char* kh = (const unsigned char*)(k + (size_t)bh * Npad * DK);
    const unsigned char* vh = (const unsigned char*)(vt + (size_t)bh * Npad * DK);

    unsigned cnt_logical = 0;  // per lane
    unsigned cnt_phys = 0;     // per wave (lane 0 adds)

    const int n_pass = CAUSAL ? 2 : 1;
    for (int pass = 0; pass < n_pass; ++pass) {
        int I;
        if (CAUSAL) {
            I = pass == 0 ? n_qtiles - 1 - x : x;
            if (pass == 1 && x == n_qtiles - 1 - x) break;
        } else {
            I = x;
        }
        const int i0w = I * BR + wave * 32;  // first row of this wavefront
        const int i = i0w + ln;              // this lane's query row
        const bool wave_active = i0w < N;

        // Key blocks that hold a needed pair: J = 0 .. nJ-1.
        int nJ = (len + BC - 1) / BC;
        if (CAUSAL) nJ = nJ < 2 * I + 2 ? nJ : 2 * I + 2;
        const int nT = pb.noskip ? nkt_all : nJ;
        const int modJ = nT;
        int Js = 2 * I + 1;
        if (Js > nT - 1) Js = nT - 1;

        f32x16 O[NDB];
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) O[db][r] = 0.f;
        float m_run = -INFINITY, l_run = 0.f;

        if (nT > 0) {
            // Q rows of this wavefront as B operand (rows >= N of the workspace are zero).
            u32x4 qf[NKS];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                qf[ks] = *(const u32x4*)(qh + (size_t)i * DK + ks * 16 + g * 8);

            const bool row_anchor = i < N && (cc.b_shift >= 0 ? (i & (cc.b - 1)) == 0 : (i % cc.b) == 0);
            const unsigned nr_anchor = cdiv_b(min(i0w + 32, N), cc) - cdiv_b(min(i0w, N), cc);

            u32x4 kreg[KCH], vreg[VCH];
            auto issue_loads = [&](int J) {
                const unsigned char* ksrc = kh + (size_t)J * (BC * DK * 2);
                const unsigned char* vsrc = vh + (size_t)J * (BC * DK * 2);
#pragma unroll
                for (int u = 0; u < KCH; ++u) kreg[u] = *(const u32x4*)(ksrc + (size_t)(tid + u * NTHREADS) * 16);
#pragma unroll
                for (int u = 0; u < VCH; ++u) vreg[u] = *(const u32x4*)(vsrc + (size_t)(tid + u * NTHREADS) * 16);
            };
            auto stage_store = [&](int buf) {
                unsigned char* kd = lds + buf * L::STAGE;
                unsigned char* vd = kd + L::K_BYTES;
#pragma unroll
                for (int u = 0; u < KCH; ++u) {
                    const int ch = tid + u * NTHREADS;
                    const int row = ch / (DK / 8), col = ch % (DK / 8);
                    *(u32x4*)(kd + row * L::KS + col * 16) = kreg[u];
                }
#pragma unroll
                for (int u = 0; u < VCH; ++u) {
                    const int ch = tid + u * NTHREADS;
                    const int row = ch / (BC / 8), col = ch % (BC / 8);
                    *(u32x4*)(vd + row * L::VS + col * 16) = vreg[u];
                }
            };

            issue_loads(Js);
            stage_store(0);
            __syncthreads();

            for (int t = 0; t < nT; ++t) {
                int J = Js - t;
                if (J < 0) J += modJ;
                if (t + 1 < nT) {
                    int Jn = J - 1;
                    if (Jn < 0) Jn += modJ;
                    issue_loads(Jn);
                }
                const unsigned char* kl = lds + (t & 1) * L::STAGE;
                const unsigned char* vl = kl + L::K_BYTES;

                // Which of the two 32-key score blocks this wavefront issues.
                const int kb0 = J * BC;
                bool need[2], edge[2];
#pragma unroll
                for (int jb = 0; jb < 2; ++jb) {
                    const int kb = kb0 + 32 * jb;
                    need[jb] = wave_active && (pb.noskip || (kb < len && (!CAUSAL || kb <= i0w)));
                    edge[jb] = pb.noskip || kb + 32 > len || (CAUSAL && kb + 31 > i0w);
                }
                if (need[0] || need[1]) {
                    f32x16 S[2];
#pragma unroll
                    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) S[jb][r] = 0.f;
                    // phase 1 (Eq. (1)): S^T[key][query] = sum_l k[key][l] q[query][l]
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks) {
#pragma unroll
                        for (int jb = 0; jb < 2; ++jb) {
                            if (need[jb]) {
                                const u32x4 kf = *(const u32x4*)(kl + (32 * jb + ln) * L::KS + (2 * ks + g) * 16);
                                S[jb] = mfma32(kf, qf[ks], S[jb]);
                            }
                        }
                    }
                    // counting and element mask on blocks that touch the diagonal or the key length
                    float mx = -INFINITY;
#pragma unroll
                    for (int jb = 0; jb < 2; ++jb) {
                        if (!need[jb]) continue;
                        const int kb = kb0 + 32 * jb;
                        cnt_phys += 1;
                        if (edge[jb] || i0w + 32 > N || kb + 32 > N) {
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int j = kb + acc_row(r, g);
                                const bool ok = j < len && (!CAUSAL || j <= i);
                                if (edge[jb]) S[jb][r] = ok ? S[jb][r] : -INFINITY;
                                const bool col_anchor = cc.b_shift >= 0 ? (j & (cc.b - 1)) == 0 : (j % cc.b) == 0;
                                cnt_logical += (row_anchor && col_anchor && j < N && (ok || pb.noskip)) ? 1u : 0u;
                            }
                        } else if (lane == 0) {
                            cnt_logical += nr_anchor * (cdiv_b(kb + 32, cc) - cdiv_b(kb, cc));
                        }
#pragma unroll
                        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[jb][r]);
                    }
                    // phase 2 (Eq. (2)), online: running maximum and sum per query row
                    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                    const float m_new = fmaxf(m_run, mx * c2);
                    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                    const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
                    m_run = m_new;
                    float psum = 0.f;
                    u32x4 pf[4];
#pragma unroll
                    for (int jb = 0; jb < 2; ++jb) {
                        if (need[jb]) {
                            float p[16];
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                p[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[jb][r], c2, -m_safe));
                                psum += p[r];
                            }
#pragma unroll
                            for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                                for (int w = 0; w < 4; ++w)
                                    pf[2 * jb + hf][w] = pack_bf16(p[8 * hf + 2 * w], p[8 * hf + 2 * w + 1]);
                        }
                    }
                    l_run = l_run * alpha + psum;
#pragma unroll
                    for (int db = 0; db < NDB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) O[db][r] *= alpha;
                    // phase 3 (Eq. (3)): O^T[col][query] += sum_key V^T[col][key] P^T[key][query]
#pragma unroll
                    for (int jb = 0; jb < 2; ++jb) {
                        if (need[jb]) {
#pragma unroll
                            for (int hf = 0; hf < 2; ++hf) {
                                const int ch = 2 * jb + hf;
#pragma unroll
                                for (int db = 0; db < NDB; ++db) {
                                    const u32x4 vf = *(const u32x4*)(vl + (32 * db + ln) * L::VS + (2 * ch + g) * 16);
                                    O[db] = mfma32(vf, pf[ch], O[db]);
                                }
                            }
                        }
                    }
                }
                if (t + 1 < nT) stage_store((t + 1) & 1);
                __syncthreads();
            }
        }

        // y_i = O_i / l_i ; a row with no allowed pair is zero.
        const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
        if (i < N) {
            const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
            bf16_t* orow = out + ((size_t)bb * N + i) * ((size_t)pb.H * DK) + (size_t)h * DK;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    u32x2 w;
                    w[0] = pack_bf16(O[db][4 * r4 + 0] * inv, O[db][4 * r4 + 1] * inv);
                    w[1] = pack_bf16(O[db][4 * r4 + 2] * inv, O[db][4 * r4 + 3] * inv);
                    *(u32x2*)(orow + 32 * db + 8 * r4 + 4 * g) = w;
                }
        }
    }

    // one atomic per wavefront
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt_logical += __shfl_xor(cnt_logical, o, 64);
    if (lane == 0) {
        if (cnt_logical) atomicAdd(&pb.counters[CNT_LOGICAL], (unsigned long long)cnt_logical);
        if (cnt_phys) atomicAdd(&pb.counters[CNT_PHYS], (unsigned long long)cnt_phys);
    }
}

}  // namespace

hipError_t launch_attn_mfma(const Problem& pb, const bf16_t* q, const bf16_t* k, const bf16_t* vt, bf16_t* out,
                            hipStream_t s)
{
    const bool causal = pb.scheme == SCHEME_CAUSAL;
    const int n_qtiles = (pb.N + BR - 1) / BR;
    const int per_head = causal ? (n_qtiles + 1) / 2 : n_qtiles;
    const int n_work = pb.B * pb.H * per_head;
    const int grid = ((n_work + 7) / 8) * 8;
    CountCfg cc;
    cc.b = pb.b;
    cc.b_shift = -1;
    for (int sft = 0; sft < 31; ++sft)
        if ((1 << sft) == pb.b) cc.b_shift = sft;
#define ATTN_LAUNCH(DK_, C_)                                                                                       \
    hipLaunchKernelGGL((attn_mfma_kernel<DK_, C_>), dim3(grid), dim3(NTHREADS), 0, s, pb, cc, q, k, vt, out, \
                       n_qtiles, per_head, n_work)
    if (pb.d == 64) {
        if (causal) ATTN_LAUNCH(64, true); else ATTN_LAUNCH(64, false);
    } else if (pb.d == 128) {
        if (causal) ATTN_LAUNCH(128, true); else ATTN_LAUNCH(128, false);
    } else {
        return hipErrorInvalidValue;
    }
#undef ATTN_LAUNCH
    return hipGetLastError();
}

}  // namespace attnring
