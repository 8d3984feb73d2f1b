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
// Data path per key block: K[64][d] and V^T[d][64] go from global memory
// straight into LDS (global_load_lds, 16 bytes per lane), double buffered, one
// barrier per block.  LDS rows are unpadded; the 16-byte chunks of a row are
// XOR-swizzled with the row index so that the 128-bit operand reads of 16
// consecutive rows hit 16 different bank groups.  Scores are computed
// transposed, S^T = K.Q^T, so that a lane holds 16 keys of ONE query per 32x32
// block: the row maximum and row sum of the online softmax need one cross-lane
// exchange, and the exponentials, converted to bf16, are already in B-operand
// layout for O^T += V^T.P^T.
#include "attn_common.h"

namespace attnring {
namespace {

constexpr int BR = 128;  // query rows per workgroup tile
constexpr int NTHREADS = 256;

template <int DK, bool CAUSAL>
struct Tile {
    static constexpr int NKS = DK / 16;         // k-steps of the score product
    static constexpr int NDB = DK / 32;         // 32-row blocks of O^T
    static constexpr int KROWB = DK * 2;        // bytes per key row in LDS
    static constexpr int K_BYTES = BC * KROWB;  // 8 or 16 KiB
    static constexpr int V_BYTES = DK * BC * 2; // same size
    static constexpr int STAGE = K_BYTES + V_BYTES;

    // Everything one wavefront carries along a row tile.
    struct State {
        f32x16 O[NDB];
        float m_run, l_run;
    };

    // One 32-key score block of the staged tile, all three phases.
    // MASK = false: every pair of the 32 x 32 block is allowed (no test at all).
    // MASK = true : pairs are tested one by one (diagonal, key length, debug mode).
    // The running maximum is only raised when a row's scores exceed it by more than
    // 2^RAISE; until then exponentials may reach 2^RAISE, which fp32 sums and bf16
    // operands hold without loss, and the 16*NDB accumulator rescales are skipped.
    static constexpr float RAISE = 8.f;
    template <bool MASK>
    static __device__ __forceinline__ void block(State& st, const u32x4 (&qf)[NKS], const unsigned char* kl,
                                                 const int (&koff)[NKS], const int (&voff)[4], int jb, float c2,
                                                 int kb, int i, int g, int len)
    {
        // operand reads of phase 1: all K fragments of the block at once
        u32x4 kf[NKS], vf[2][NDB];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) kf[ks] = *(const u32x4*)(kl + koff[ks] + jb * 32 * KROWB);
        __builtin_amdgcn_sched_barrier(0);
        // phase 1 (Eq. (1)): S^T[key][query] = sum_l k[key][l] q[query][l]
        f32x16 S;
#pragma unroll
        for (int r = 0; r < 16; ++r) S[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) S = mfma32(kf[ks], qf[ks], S);
        __builtin_amdgcn_sched_barrier(0);
        // operand reads of phase 3, issued now so that they land during the softmax
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int db = 0; db < NDB; ++db)
                vf[hf][db] = *(const u32x4*)(kl + voff[2 * jb + hf] + db * 32 * (BC * 2));
        __builtin_amdgcn_sched_barrier(0);
        if (MASK) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int j = kb + acc_row(r, g);
                const bool ok = j < len && (!CAUSAL || j <= i);
                S[r] = ok ? S[r] : -INFINITY;
            }
        }
        // phase 2 (Eq. (2)), online: running maximum and sum per query row
        // The running maximum is the reference of the exponentials.  It is raised only when a
        // row's scores exceed it by more than 2^RAISE; that is rare after the first blocks, so the
        // common path has no cross-lane exchange, no accumulator rescale and one exp per pair.
        float mxl = S[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mxl = fmaxf(mxl, S[r]);
        if (__builtin_amdgcn_ballot_w64(mxl * c2 > st.m_run + RAISE) != 0ull) {
            const float mx = fmaxf(mxl, __shfl_xor(mxl, 32, 64)) * c2;  // both halves of a row agree
            const float m_new = mx > st.m_run + RAISE ? mx : st.m_run;
            const float m_ref = (MASK && m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(st.m_run - m_ref);
            st.m_run = m_new;
            st.l_run *= alpha;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) st.O[db][r] *= alpha;
        }
        const float m_use = (MASK && st.m_run == -INFINITY) ? 0.f : st.m_run;
        float psum = 0.f;
        u32x4 pf[2];
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[8 * hf + 2 * w], c2, -m_use));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[8 * hf + 2 * w + 1], c2, -m_use));
                psum += p0 + p1;
                pf[hf][w] = pack_bf16(p0, p1);
            }
        st.l_run += psum;
        __builtin_amdgcn_sched_barrier(0);
        // phase 3 (Eq. (3)): O^T[col][query] += sum_key V^T[col][key] P^T[key][query]
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int db = 0; db < NDB; ++db) st.O[db] = mfma32(vf[hf][db], pf[hf], st.O[db]);
    }
};

template <int DK, bool CAUSAL>
__global__ __launch_bounds__(NTHREADS, 2) void attn_mfma_kernel(Problem pb, CountCfg cc, const bf16_t* __restrict__ q,
                                                                const bf16_t* __restrict__ k,
                                                                const bf16_t* __restrict__ vt,
                                                                bf16_t* __restrict__ out, int n_qtiles, int per_head,
                                                                int n_work)
{
    typedef Tile<DK, CAUSAL> T;
    constexpr int NKS = T::NKS, NDB = T::NDB;
    constexpr int KPIECES = T::K_BYTES / 1024 / 4;  // 1 KiB pieces per wavefront
    constexpr int VPIECES = T::V_BYTES / 1024 / 4;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * T::STAGE];

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

    // Swizzled LDS byte offsets of this lane's operand reads within a stage (the second
    // 32-key block of a tile lies 32 key rows higher).
    int koff[NKS], voff[4];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) koff[ks] = ln * T::KROWB + swz<T::KROWB>(2 * ks + g, ln) * 16;
#pragma unroll
    for (int ch = 0; ch < 4; ++ch) voff[ch] = T::K_BYTES + ln * (BC * 2) + swz<BC * 2>(2 * ch + g, ln) * 16;

    const unsigned k_lane_off = dma_lane_offset<T::KROWB>(wave, lane);
    const unsigned v_lane_off = dma_lane_offset<BC * 2>(wave, lane);

    unsigned cnt_edge = 0;      // logical tiles found lane by lane in edge blocks
    unsigned cnt_interior = 0;  // logical tiles of fully allowed blocks (wave-uniform)
    unsigned cnt_phys = 0;      // 32 x 32 score blocks issued (wave-uniform)

    const int n_pass = CAUSAL ? 2 : 1;
#pragma nounroll
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

        // The walk over key blocks.  Needed blocks are J = 0 .. nJ-1.
        //   masked scheme: J = Js, Js-1, .., 0 (own diagonal block first);
        //   FULL: the block cut by the key length first (if any), then the whole
        //         blocks in ring order from the own block.
        // In debug mode the blocks with no needed pair are walked first; they change nothing.
        int nJ = (len + BC - 1) / BC;
        if (CAUSAL) nJ = nJ < 2 * I + 2 ? nJ : 2 * I + 2;
        const int n_dead = pb.noskip ? nkt_all - nJ : 0;
        const int nT = nJ + n_dead;
        const int has_cut = (!CAUSAL && (len % BC) != 0) ? 1 : 0;
        const int n_ring = nJ - has_cut;                      // FULL: whole blocks
        const int Js = CAUSAL ? nJ - 1 : (2 * I + 1 < n_ring ? 2 * I + 1 : n_ring - 1);
        auto block_of_step = [&](int t) -> int {
            if (t < n_dead) return nkt_all - 1 - t;
            t -= n_dead;
            if (CAUSAL) return Js - t;
            if (t < has_cut) return nJ - 1;
            int J = Js - (t - has_cut);
            return J < 0 ? J + n_ring : J;
        };
        // Steps this wavefront takes through the general code; the rest are blocks in
        // which every pair is allowed.
        int n_gen;
        if (pb.noskip || !wave_active) {
            n_gen = nT;
        } else if (CAUSAL) {
            int j_int = (i0w + 1) / BC - 1;                  // last block entirely at or below row i0w
            const int j_len = len / BC - 1;                  // last block entirely below the key length
            j_int = j_int < j_len ? j_int : j_len;
            n_gen = Js - j_int;
            n_gen = n_gen < 0 ? 0 : (n_gen > nT ? nT : n_gen);
        } else {
            n_gen = has_cut;
        }

        typename T::State st;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.O[db][r] = 0.f;
        st.m_run = -INFINITY;
        st.l_run = 0.f;

        if (nT > 0) {
            // Q rows of this wavefront as B operand (rows >= n of the workspace are zero).
            u32x4 qf[NKS];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) qf[ks] = *(const u32x4*)(qh + (size_t)i * DK + ks * 16 + g * 8);

            const bool row_anchor = i < N && is_multiple(i, cc);
            const unsigned nr_anchor = cdiv_b(min(i0w + 32, N), cc) - cdiv_b(min(i0w, N), cc);

            auto issue_loads = [&](int J, int buf) {
                unsigned char* base = lds + buf * T::STAGE;
                dma_pieces<KPIECES>(kh + (size_t)J * T::K_BYTES, base, k_lane_off, wave, 4);
                dma_pieces<VPIECES>(vh + (size_t)J * T::V_BYTES, base + T::K_BYTES, v_lane_off, wave, 4);
            };

            issue_loads(block_of_step(0), 0);
            __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the LDS writes of this wavefront have landed
            __syncthreads();

            // ---- general steps: blocks may be skipped or masked pair by pair ----
            int t = 0;
#pragma nounroll
            for (; t < n_gen; ++t) {
                const int J = block_of_step(t);
                if (t + 1 < nT) issue_loads(block_of_step(t + 1), (t + 1) & 1);
                const unsigned char* kl = lds + (t & 1) * T::STAGE;
                if (wave_active) {
#pragma unroll
                    for (int jb = 0; jb < 2; ++jb) {
                        const int kb = J * BC + 32 * jb;
                        const bool need = pb.noskip || (kb < len && (!CAUSAL || kb <= i0w));
                        if (need) {  // otherwise: redundant block, never issued
                            const bool edge = pb.noskip || kb + 32 > len || (CAUSAL && kb + 31 > i0w);
                            cnt_phys += 1;
                            if (edge) T::template block<true>(st, qf, kl, koff, voff, jb, c2, kb, i, g, len);
                            else T::template block<false>(st, qf, kl, koff, voff, jb, c2, kb, i, g, len);
                            if (edge || i0w + 32 > N) {
                                // logical tiles whose first pair lies in this block and is allowed:
                                // each such pair is seen by the lane that holds it in the accumulator
                                if (row_anchor) {
                                    const int jend = min(kb + 32, N);
#pragma nounroll
                                    for (int j = (int)cdiv_b(kb, cc) * cc.b; j < jend; j += cc.b) {
                                        const bool mine = (((j - kb) >> 2) & 1) == g;
                                        const bool ok = j < len && (!CAUSAL || j <= i);
                                        cnt_edge += (mine && (ok || pb.noskip)) ? 1u : 0u;
                                    }
                                }
                            } else {
                                cnt_interior += nr_anchor * (cdiv_b(kb + 32, cc) - cdiv_b(kb, cc));
                            }
                        }
                    }
                }
                __builtin_amdgcn_s_waitcnt(0x0F70);  // the next block is in LDS before anyone reads it
                __syncthreads();
            }
            // ---- the rest: every pair allowed; no test, no branch ----
            if (t < nT) {
                // These steps cover a contiguous range of whole blocks; count their tiles from the range.
                const int j_hi = block_of_step(t);
                const int j_lo = CAUSAL ? 0 : 0;
                const int n_fast = nT - t;
                cnt_phys += 2u * (unsigned)n_fast;
                const int k_hi = CAUSAL ? (j_hi + 1) * BC : n_ring * BC;
                cnt_interior += nr_anchor * (cdiv_b(k_hi, cc) - cdiv_b(j_lo * BC, cc));
            }
#pragma nounroll
            for (; t < nT; ++t) {
                const int J = block_of_step(t);
                if (t + 1 < nT) issue_loads(block_of_step(t + 1), (t + 1) & 1);
                const unsigned char* kl = lds + (t & 1) * T::STAGE;
                T::template block<false>(st, qf, kl, koff, voff, 0, c2, J * BC, i, g, len);
                T::template block<false>(st, qf, kl, koff, voff, 1, c2, J * BC + 32, i, g, len);
                __builtin_amdgcn_s_waitcnt(0x0F70);
                __syncthreads();
            }
        }

        // y_i = O_i / l_i ; a row with no allowed pair is zero.
        const float l_tot = st.l_run + __shfl_xor(st.l_run, 32, 64);
        if (i < N) {
            const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
            bf16_t* orow = out + ((size_t)bb * N + i) * ((size_t)pb.H * DK) + (size_t)h * DK;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    u32x2 w;
                    w[0] = pack_bf16(st.O[db][4 * r4 + 0] * inv, st.O[db][4 * r4 + 1] * inv);
                    w[1] = pack_bf16(st.O[db][4 * r4 + 2] * inv, st.O[db][4 * r4 + 3] * inv);
                    *(u32x2*)(orow + 32 * db + 8 * r4 + 4 * g) = w;
                }
        }
    }

    // one atomic per wavefront
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt_edge += __shfl_xor(cnt_edge, o, 64);
    if (lane == 0) {
        const unsigned long long logical = (unsigned long long)cnt_edge + cnt_interior;
        if (logical) atomicAdd(&pb.counters[CNT_LOGICAL], logical);
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
