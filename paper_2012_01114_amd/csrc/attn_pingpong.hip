// Fused phases 1-3 (Sec. 3.1, Eq. (1)-(3)) for long sequences: the same
// arithmetic, ring walk and skipping rules as attn_mfma.hip, scheduled so that
// the matrix cores and the vector ALUs of a SIMD work at the same time.
//
// A workgroup owns 256 query rows and has 8 wavefronts in two groups of four;
// hardware places wavefront w and w+4 on the same SIMD.  Time is cut into
// slots that end in a workgroup barrier.  In every slot one group is in its
// VECTOR phase (online softmax of its current 32-key block: phase 2, Eq. (2))
// while the other is in its MATRIX phase (O^T += V^T.P^T of that block, phase 3,
// Eq. (3), then S^T = K.Q^T of the next block, phase 1, Eq. (1)); the next slot
// they swap.  The operands of a matrix phase are read from LDS during the
// preceding vector phase, so a matrix phase is MFMA instructions only.
//
// K / V^T tiles of 64 keys go from global memory straight into a ring of three
// LDS stages (global_load_lds); tile u is requested when tile u-3 has been read
// for the last time and awaited two slots before its first use.
#include "attn_common.h"

namespace attnring {
namespace {

constexpr int PP_BR = 256;     // query rows per workgroup
constexpr int PP_THREADS = 512;
constexpr int PP_STAGES = 3;

template <int DK, bool CAUSAL>
struct PP {
    static constexpr int NKS = DK / 16;
    static constexpr int NDB = DK / 32;
    static constexpr int KROWB = DK * 2;
    static constexpr int K_BYTES = BC * KROWB;
    static constexpr int V_BYTES = DK * BC * 2;
    static constexpr int STAGE = K_BYTES + V_BYTES;
    static constexpr int PPW = STAGE / 1024 / 8;  // 1 KiB pieces per wavefront and tile
    static constexpr float RAISE = 8.f;           // see attn_mfma.hip: lazy raise of the running maximum

    struct State {
        f32x16 O[NDB];
        f32x16 S;        // scores of the block whose vector phase comes next
        u32x4 pf[2];     // its exponentials (bf16, B-operand layout) once that phase is done
        u32x4 vf[2][NDB];  // V^T operands of the coming matrix phase
        float m_run, l_run;
    };

    // vector phase of block n: fetch the V^T operands of the matrix phase that follows, then softmax
    template <bool MASK>
    static __device__ __forceinline__ void vector_phase(State& st, const unsigned char* lds, int v_stage,
                                                        bool have_cur, int jb_cur, const int (&voff)[4], float c2,
                                                        int kb, int i, int g, int len)
    {
        if (have_cur) {
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                for (int db = 0; db < NDB; ++db)
                    st.vf[hf][db] =
                        *(const u32x4*)(lds + v_stage + voff[2 * jb_cur + hf] + db * 32 * (BC * 2));
        }
        if (!have_cur) return;
        f32x16 S = st.S;
        if (MASK) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int j = kb + acc_row(r, g);
                const bool ok = j < len && (!CAUSAL || j <= i);
                S[r] = ok ? S[r] : -INFINITY;
            }
        }
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
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[8 * hf + 2 * w], c2, -m_use));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(S[8 * hf + 2 * w + 1], c2, -m_use));
                psum += p0 + p1;
                st.pf[hf][w] = pack_bf16(p0, p1);
            }
        st.l_run += psum;
    }

    // matrix phase: phase 3 of the current block, phase 1 of the next one (whose K operands
    // are read from LDS while the phase-3 MFMAs run)
    static __device__ __forceinline__ void matrix_phase(State& st, const u32x4 (&qf)[NKS], const unsigned char* lds,
                                                        int k_stage, int jb_next, const int (&koff)[NKS],
                                                        bool have_cur, bool have_next)
    {
        u32x4 kf[NKS];
        if (have_next) {
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                kf[ks] = *(const u32x4*)(lds + k_stage + koff[ks] + jb_next * 32 * KROWB);
        }
        if (have_cur) {
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                for (int db = 0; db < NDB; ++db) st.O[db] = mfma32(st.vf[hf][db], st.pf[hf], st.O[db]);
        }
        if (have_next) {
            f32x16 S;
#pragma unroll
            for (int r = 0; r < 16; ++r) S[r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) S = mfma32(kf[ks], qf[ks], S);
            st.S = S;
        }
    }
};

template <int DK, bool CAUSAL>
__global__ __launch_bounds__(PP_THREADS, 2) void attn_pp_kernel(Problem pb, CountCfg cc, const bf16_t* __restrict__ q,
                                                                const bf16_t* __restrict__ k,
                                                                const bf16_t* __restrict__ vt,
                                                                bf16_t* __restrict__ out, int n_qtiles, int per_head,
                                                                int n_work)
{
    typedef PP<DK, CAUSAL> T;
    constexpr int NKS = T::NKS, NDB = T::NDB;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[PP_STAGES * T::STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63, ln = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2;  // 0: vector phase in even slots, 1: in odd slots

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
    const float c2 = pb.scale * 1.4426950408889634f;

    const bf16_t* qh = q + (size_t)bh * Npad * DK;
    const unsigned char* kh = (const unsigned char*)(k + (size_t)bh * Npad * DK);
    const unsigned char* vh = (const unsigned char*)(vt + (size_t)bh * Npad * DK);

    int koff[NKS], voff[4];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) koff[ks] = ln * T::KROWB + swz<T::KROWB>(2 * ks + g, ln) * 16;
#pragma unroll
    for (int ch = 0; ch < 4; ++ch) voff[ch] = T::K_BYTES + ln * (BC * 2) + swz<BC * 2>(2 * ch + g, ln) * 16;

    const unsigned k_lane_off = dma_lane_offset<T::KROWB>(wave, lane);
    const unsigned v_lane_off = dma_lane_offset<BC * 2>(wave, lane);

    unsigned cnt_edge = 0, cnt_interior = 0, cnt_phys = 0;

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
        const int i0w = I * PP_BR + wave * 32;
        const int i = i0w + ln;
        const bool wave_active = i0w < N;

        // The walk over key tiles: as in attn_mfma.hip, for a 256-row tile.
        int nJ = (len + BC - 1) / BC;
        if (CAUSAL) nJ = nJ < 4 * I + 4 ? nJ : 4 * I + 4;
        const int n_dead = pb.noskip ? nkt_all - nJ : 0;
        const int nT = nJ + n_dead;
        const int has_cut = (!CAUSAL && (len % BC) != 0) ? 1 : 0;
        const int n_ring = nJ - has_cut;
        const int Js = CAUSAL ? nJ - 1 : (4 * I + 3 < n_ring ? 4 * I + 3 : n_ring - 1);
        auto tile_of_step = [&](int t) -> int {
            if (t < n_dead) return nkt_all - 1 - t;
            t -= n_dead;
            if (CAUSAL) return Js - t;
            if (t < has_cut) return nJ - 1;
            int J = Js - (t - has_cut);
            return J < 0 ? J + n_ring : J;
        };
        int n_gen;  // leading tiles this wavefront takes through the general code
        if (pb.noskip || !wave_active) {
            n_gen = nT;
        } else if (CAUSAL) {
            int j_int = (i0w + 1) / BC - 1;
            const int j_len = len / BC - 1;
            j_int = j_int < j_len ? j_int : j_len;
            n_gen = Js - j_int;
            n_gen = n_gen < 0 ? 0 : (n_gen > nT ? nT : n_gen);
        } else {
            n_gen = has_cut;
        }
        const int NBLK = 2 * nT;   // 32-key blocks, two per tile, in walk order
        const int nb_gen = 2 * n_gen;

        typename T::State st;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.O[db][r] = 0.f;
        st.m_run = -INFINITY;
        st.l_run = 0.f;

        if (nT > 0) {
            u32x4 qf[NKS];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) qf[ks] = *(const u32x4*)(qh + (size_t)i * DK + ks * 16 + g * 8);
            const bool row_anchor = i < N && is_multiple(i, cc);
            const unsigned nr_anchor = cdiv_b(min(i0w + 32, N), cc) - cdiv_b(min(i0w, N), cc);

            auto issue_tile = [&](int u) {
                const int J = tile_of_step(u);
                unsigned char* base = lds + (u % PP_STAGES) * T::STAGE;
                // 8 wavefronts: pieces wave, wave+8, ... of K then of V^T
                dma_pieces<T::K_BYTES / 1024 / 8>(kh + (size_t)J * T::K_BYTES, base, k_lane_off, wave, 8);
                dma_pieces<T::V_BYTES / 1024 / 8>(vh + (size_t)J * T::V_BYTES, base + T::K_BYTES, v_lane_off, wave, 8);
            };
            // End of slot tau: await what the next slots need, meet, then request a new tile.
            //   tile u (u >= 2) is requested at the start of slot 4u-7 (its stage held tile u-3, read
            //   for the last time in slot 4u-9) and awaited at the end of slot 4u-3 (first read: 4u-2).
            auto slot_end = [&](int tau) {
                if ((tau & 3) == 1) {
                    const int u = (tau + 3) >> 2;
                    if (u >= 2 && u < nT) {
                        if (u + 1 < nT) __builtin_amdgcn_s_waitcnt(0x0F70 | T::PPW);  // newest request may stay in flight
                        else __builtin_amdgcn_s_waitcnt(0x0F70);
                    }
                }
                // a bare barrier: the fence of __syncthreads() would also wait for the tile requests in flight
                __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wavefront's LDS reads are done
                __builtin_amdgcn_s_barrier();
                const int sigma = tau + 1;
                if ((sigma & 3) == 1) {
                    const int u = (sigma + 7) >> 2;
                    if (u < nT) issue_tile(u);
                }
            };
            // block n of the walk: key offset and what this wavefront does with it
            auto block_info = [&](int n, int& kb, bool& need, bool& edge) {
                const int J = tile_of_step(n >> 1);
                kb = J * BC + 32 * (n & 1);
                need = wave_active && n < NBLK && (pb.noskip || (kb < len && (!CAUSAL || kb <= i0w)));
                edge = pb.noskip || kb + 32 > len || (CAUSAL && kb + 31 > i0w);
            };
            auto stage_of = [&](int n) -> int { return ((n >> 1) % PP_STAGES) * T::STAGE; };

            issue_tile(0);
            if (nT > 1) issue_tile(1);
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();

            // phase 1 of block 0, outside the rotation (group 1 does it in slot 0)
            {
                int kb; bool need, edge;
                block_info(0, kb, need, edge);
                T::matrix_phase(st, qf, lds, stage_of(0), 0, koff, false, need);
            }
            if (grp == 1) slot_end(0);

            int n = 0;
            // ---- general iterations: blocks may be skipped or masked pair by pair ----
            auto general_iter = [&](int nn) {
                int kb, kbn; bool need, edge, needn, edgen;
                block_info(nn, kb, need, edge);
                block_info(nn + 1, kbn, needn, edgen);
                if (need) {
                    cnt_phys += 1;
                    if (edge || i0w + 32 > N) {
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
                if (edge) T::template vector_phase<true>(st, lds, stage_of(nn), need, nn & 1, voff, c2, kb, i, g, len);
                else T::template vector_phase<false>(st, lds, stage_of(nn), need, nn & 1, voff, c2, kb, i, g, len);
                slot_end(2 * nn + grp);
                T::matrix_phase(st, qf, lds, stage_of(nn + 1), (nn + 1) & 1, koff, need, needn);
                slot_end(2 * nn + 1 + grp);
            };
            const int n_lead = nb_gen < NBLK ? nb_gen : NBLK;
#pragma nounroll
            for (; n < n_lead; ++n) general_iter(n);
            // ---- steady state: every pair allowed, next block exists ----
            if (n < NBLK) {
                const int n_fast_blocks = NBLK - n;
                cnt_phys += (unsigned)n_fast_blocks;
                const int k_hi = CAUSAL ? (tile_of_step(n >> 1) + 1) * BC : n_ring * BC;
                cnt_interior += nr_anchor * (cdiv_b(k_hi, cc) - cdiv_b(0, cc));
            }
#pragma nounroll
            for (; n + 1 < NBLK; ++n) {
                const int kb = tile_of_step(n >> 1) * BC + 32 * (n & 1);
                T::template vector_phase<false>(st, lds, stage_of(n), true, n & 1, voff, c2, kb, i, g, len);
                slot_end(2 * n + grp);
                T::matrix_phase(st, qf, lds, stage_of(n + 1), (n + 1) & 1, koff, true, true);
                slot_end(2 * n + 1 + grp);
            }
            if (n < NBLK) {  // last block: nothing follows
                const int kb = tile_of_step(n >> 1) * BC + 32 * (n & 1);
                T::template vector_phase<false>(st, lds, stage_of(n), true, n & 1, voff, c2, kb, i, g, len);
                slot_end(2 * n + grp);
                T::matrix_phase(st, qf, lds, 0, 0, koff, true, false);
                slot_end(2 * n + 1 + grp);
                ++n;
            }
            if (grp == 0) slot_end(2 * NBLK);
        }

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

#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt_edge += __shfl_xor(cnt_edge, o, 64);
    if (lane == 0) {
        const unsigned long long logical = (unsigned long long)cnt_edge + cnt_interior;
        if (logical) atomicAdd(&pb.counters[CNT_LOGICAL], logical);
        if (cnt_phys) atomicAdd(&pb.counters[CNT_PHYS], (unsigned long long)cnt_phys);
    }
}

}  // namespace

hipError_t launch_attn_pingpong(const Problem& pb, const bf16_t* q, const bf16_t* k, const bf16_t* vt, bf16_t* out,
                                hipStream_t s)
{
    const bool causal = pb.scheme == SCHEME_CAUSAL;
    const int n_qtiles = (pb.N + PP_BR - 1) / PP_BR;
    const int per_head = causal ? (n_qtiles + 1) / 2 : n_qtiles;
    const int n_work = pb.B * pb.H * per_head;
    const int grid = ((n_work + 7) / 8) * 8;
    CountCfg cc;
    cc.b = pb.b;
    cc.b_shift = -1;
    for (int sft = 0; sft < 31; ++sft)
        if ((1 << sft) == pb.b) cc.b_shift = sft;
#define ATTN_LAUNCH(DK_, C_)                                                                                    \
    hipLaunchKernelGGL((attn_pp_kernel<DK_, C_>), dim3(grid), dim3(PP_THREADS), 0, s, pb, cc, q, k, vt, out, \
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
