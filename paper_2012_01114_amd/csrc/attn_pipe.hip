// Fused phases 1-3 (Sec. 3.1, Eq. (1)-(3)) on the 16-bit matrix cores of gfx950,
// FULL and masked scheme, scheduled so that the two wavefronts that share a SIMD
// keep its matrix cores and its vector ALUs busy at the same time.
//
// Ring mapping.  A wavefront owns 32 consecutive query rows (one or several of
// the paper's PEs, which own n/P rows each); WAVES wavefronts form a workgroup.
// The workgroup meets the 64-key tiles of its head in ring order, starting with
// the tile at its own diagonal and walking down, wrapping round for the FULL
// scheme; tiles with no needed pair are not in the walk, and a wavefront joins
// the walk at the first 32-key block that holds a pair it needs (Sec. 5.1:
// masked pairs are left out of all three phases).  Masked scheme: workgroup x
// handles row tiles T-1-x and x, the packing of row n-i with row i that
// equalises the work per PE (Sec. 5.2).
//
// Schedule.  The walk is cut into 32-key blocks; for block n a wavefront runs
//     E(n)  vector ALUs :  pair tests of an edge block, P(n) = exp2(S(n) - ref), row sums
//                          (phase 2, Eq. (2)); between the exponentials it requests from
//                          LDS the fragments M(n) will take: K of block n+1, V^T of block n
//     M(n)  matrix cores:  S(n+1) = K(n+1).Q^T (phase 1 of the next block, Eq. (1)),
//                          O += V(n)^T.P(n)^T (phase 3, Eq. (3)); the copy requests for a
//                          later tile go out behind single MFMAs
// in the order E(n), M(n), E(n+1), ...  A workgroup of eight wavefronts has two
// groups of four; wavefronts w and w+4 share a SIMD.  Group 0 meets the per-tile
// workgroup barrier in front of E(2t), group 1 between E(2t) and M(2t): after
// every barrier one group is in a vector phase while the other is in a matrix
// phase, and they stay half an iteration apart.  Scores are computed transposed
// (S^T = K.Q^T): a lane holds 16 keys of ONE query per 32x32 block, the
// exponentials, rounded to half precision, are already in B-operand layout for
// O^T += V^T.P^T, and a row needs no cross-lane traffic on the common path.
//
// Online softmax with a lazily raised reference.  q arrives pre-multiplied by
// scale*log2(e) and the score MFMAs start from minus the row's reference, so the
// MFMA yields the base-2 exponent itself and an exponential costs one v_exp_f32;
// row sums are plain fp32 additions (dot instructions stall on the matrix pipe).
// The reference is raised only when a score exceeds it by more than 2^RAISE (rare
// after the first blocks); until then exponentials may reach 2^RAISE, which fp32
// sums and half-precision operands hold without loss.  Raising rescales the row at the head of E(n), when everything computed
// with the old reference has been added to O.
//
// K[64][d] and V^T[d][64] tiles go from global memory straight into a ring of
// LDS stages (buffer_load ... lds, 16 bytes per lane) two to three tiles ahead of
// their use; one workgroup barrier per tile.  LDS rows are unpadded; their 16-byte chunks are
// XOR-swizzled with the row index (conflict-free 128-bit reads).
#include <type_traits>

#include "attn_common.h"

namespace attnring {
namespace {

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>)
template <int N, class F, int I = 0>
__device__ __forceinline__ void static_for_q(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for_q<N, F, I + 1>(static_cast<F&&>(f));
    }
}

constexpr float PIPE_RAISE = 8.f;  // slack of the lazy reference, in base-2 exponent units
// A lane's 16 exponentials of a block add up to more than this only if one of them is above
// 2^PIPE_RAISE, and as long as they do not, none is above 2^12, far inside half precision.
constexpr float PIPE_SUM_LIMIT = 4096.f;

template <int DK, int WAVES, bool CAUSAL>
struct Pipe {
    static constexpr int NKS = DK / 16;         // k-steps of the score product
    static constexpr int NDB = DK / 32;         // 32-row blocks of O^T
    static constexpr int KROWB = DK * 2;        // bytes per key row in LDS
    static constexpr int K_BYTES = BC * KROWB;  // 8 or 16 KiB
    static constexpr int V_BYTES = DK * BC * 2;
    static constexpr int STAGE = K_BYTES + V_BYTES;
    static constexpr int BR = 32 * WAVES;       // rows per workgroup
    static constexpr int KPIECES = K_BYTES / 1024 / WAVES;  // 1 KiB copy pieces per wavefront and tile
    static constexpr int VPIECES = V_BYTES / 1024 / WAVES;
    static constexpr int PPW = KPIECES + VPIECES;
    // LDS ring, in 64-key tiles.  Three stages let three 4-wavefront workgroups of d_k = 64 share a
    // CU (three wavefronts per SIMD); otherwise five stages (all 160 KiB at d_k = 128) and two
    // wavefronts per SIMD.
    static constexpr int STAGES = (DK == 64 && WAVES == 4) ? 3 : 5;
    static constexpr int OCC = (DK == 64 && WAVES == 4) ? 3 : 2;
    // With five stages a wavefront in the walk does not request a tile right behind the barrier
    // that frees its stage but spreads its pieces over the matrix phases up to the next barrier.
    static constexpr bool SPREAD = STAGES >= 5;
    // Fold the reference into the score accumulator: saves a subtraction per pair, costs 16 registers
    // (168 in all for the 4-wavefront d_k = 64 kernel, just what three wavefronts per SIMD allow).
    static constexpr bool USE_CNEG = true;

    struct Row {
        f32x16 O[NDB];  // O^T, un-normalised
        f32x16 S;       // base-2 scores, minus the reference, of the block whose phase 2 comes next
        f32x16 Cneg;    // minus the reference: the C operand the score MFMAs start from
        u32x4 P[2];     // exponentials of the current block, half precision, B-operand layout
        float thr;      // RAISE once the row has a reference, -inf before
        float mref;     // the reference (0 before the row has one)
        float l;        // this lane's part of the row sum
    };
    struct Frags {
        u32x4 kf[NKS];     // K of block n+1
        u32x4 vf[2][NDB];  // V^T of block n: keys 0..15 and 16..31 of the block
    };

    static __device__ __forceinline__ f32x16 zero16()
    {
        f32x16 z;
#pragma unroll
        for (int e = 0; e < 16; ++e) z[e] = 0.f;
        return z;
    }
    static __device__ __forceinline__ float max16(const f32x16& S)
    {
        float m0 = fmaxf(fmaxf(S[0], S[1]), S[2]), m1 = fmaxf(fmaxf(S[3], S[4]), S[5]);
        float m2 = fmaxf(fmaxf(S[6], S[7]), S[8]), m3 = fmaxf(fmaxf(S[9], S[10]), S[11]);
        float m4 = fmaxf(fmaxf(S[12], S[13]), S[14]);
        m0 = fmaxf(fmaxf(m0, m1), m2);
        m3 = fmaxf(fmaxf(m3, m4), S[15]);
        return fmaxf(m0, m3);
    }
    // Pair test of an edge block: key kb + acc_row(e, g) against the lane's last allowed key.
    static __device__ __forceinline__ void mask_block(f32x16& S, int lim)
    {
#pragma unroll
        for (int e = 0; e < 16; ++e) S[e] = (8 * (e >> 2) + (e & 3)) <= lim ? S[e] : -INFINITY;
    }
    // The chunk of k-step ks is chunk 2*ks + g XOR-ed with row bits, and 2*ks has no bit in
    // common with g: the lane's byte address for k-step ks is its address for k-step 0 XOR 32*ks
    // (32-key blocks start at multiples of 256 bytes).  ka0: LDS byte offset for k-step 0.
    static __device__ __forceinline__ u32x4 read_k1(const unsigned char* lds, unsigned ka0, int ks)
    {
        return *(const u32x4*)(lds + (ka0 ^ (unsigned)(32 * ks)));
    }
    static __device__ __forceinline__ void read_k(Frags& fr, const unsigned char* lds, unsigned ka0)
    {
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) fr.kf[ks] = read_k1(lds, ka0, ks);
    }
    // Phase 1 (Eq. (1)) of one block from the K fragments in fr; the accumulator starts at minus
    // the row's reference, so the result is the exponent phase 2 needs.
    // `between(m)` runs behind MFMA m of the phase (a copy request, or nothing).
    template <class F>
    static __device__ __forceinline__ f32x16 scores(const Row& r, const Frags& fr, const u32x4 (&qf)[NKS], F&& between)
    {
        f32x16 S;
        if constexpr (USE_CNEG) {
            // D and C in different registers: written with the builtin, the compiler copies the 16
            // registers of C first and accumulates in place.
            asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %3" : "=&v"(S) : "v"(fr.kf[0]), "v"(qf[0]), "v"(r.Cneg));
        } else {
            S = mfma32h(fr.kf[0], qf[0], zero16());
        }
        between(0);
#pragma unroll
        for (int ks = 1; ks < NKS; ++ks) {
            S = mfma32h(fr.kf[ks], qf[ks], S);
            between(ks);
        }
        return S;
    }
    // Phase 3 (Eq. (3)) of one block from the V^T fragments in fr and the row's exponentials.
    template <class F>
    static __device__ __forceinline__ void weighted_sum(Row& r, const Frags& fr, F&& between)
    {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                r.O[db] = mfma32h(fr.vf[hf][db], r.P[hf], r.O[db]);
                between(NKS + hf * NDB + db);
            }
    }

    // A score beyond the slack (or the first finite score of a row): move the reference to the
    // row's largest score and rescale what the row has accumulated.  Returns what the reference
    // went up by; the scores at hand were computed against the old reference.
    static __device__ __forceinline__ float raise_reference(Row& r, float mxl)
    {
        asm volatile("" ::: "memory");  // keeps this rare path a branch of its own
        const float mx = fmaxf(mxl, __shfl_xor(mxl, 32, 64));  // both halves of a row agree
        const bool raise = mx > r.thr;
        const bool started = r.thr > -INFINITY;
        const float delta = raise ? mx : 0.f;
        const float alpha = (raise && started) ? __builtin_amdgcn_exp2f(-delta) : 1.f;
        r.mref = raise ? r.mref + delta : r.mref;
        r.thr = raise ? PIPE_RAISE : r.thr;
        r.l *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) r.O[db][e] *= alpha;
        if (USE_CNEG) {
            // the scores at hand were taken against the old reference
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                r.Cneg[e] = -r.mref;
                r.S[e] -= delta;
            }
        }
        return delta;
    }

    // Phase 2 (Eq. (2)) of the block in r.S; the row sum is normalised at the very end.
    // SHIFT: the scores still refer to a reference that was `delta` lower.
    // `between(p)` runs behind score pair p (0..7): the LDS requests for the matrix phase.
    // Returns the sum of the lane's 16 exponentials, which the caller adds to r.l.
    template <bool SHIFT, class F>
    static __device__ __forceinline__ float exponentials(Row& r, float delta, F&& between)
    {
        // The row sum is taken with plain additions of the unrounded exponentials.  A v_dot2c on
        // the rounded pairs would be half the instructions, but dot instructions do not run beside
        // the matrix pipe: each one waits until the MFMAs in flight on its SIMD have drained, from
        // whichever wavefront they are, which serialises the vector phase with the matrix phase
        // of the wavefront it shares the SIMD with (measured: an MFMA followed by one v_dot2c
        // takes 51 cycles instead of 32; exponentials, conversions, max and fma add 1-3).
        float psum0 = 0.f, psum1 = 0.f;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float s0 = r.S[8 * hf + 2 * w], s1 = r.S[8 * hf + 2 * w + 1];
                const float p0 = __builtin_amdgcn_exp2f(SHIFT ? s0 - delta : s0);
                const float p1 = __builtin_amdgcn_exp2f(SHIFT ? s1 - delta : s1);
                r.P[hf][w] = pack_f16(p0, p1);
                psum0 += p0;
                psum1 += p1;
                between(4 * hf + w);
            }
        return psum0 + psum1;
    }
};

// q' = (x.Wq) * qscale for the 32 rows of a wavefront (lane L: row L % 32), as B operands of the score
// MFMAs: qf[ks] holds 8 consecutive columns 16 ks + 8 (L / 32) ...  All wavefronts of the workgroup
// call it together (same head): the weight columns of the head go through LDS in slices of 64 rows
// of Wq, two buffers at wbuf (2 * 64 * d_k * 2 bytes), one barrier per slice; what a slice needs from
// global memory (its part of Wq, the lane's 128 bytes of x) is requested four slices ahead.
//   Q^T [d_k x 32 rows] += Wq_h^T [d_k x 16] . x^T [16 x 32 rows]   per k-step, bf16 MFMA, fp32 sums:
//   A operand: a column of Wq (one l) along 8 consecutive k - read from the k-major LDS slice with
//              the transposing 64-bit read (16 lanes hand in a 4 k x 16 columns patch, lane i gets
//              column i); rows of 128 bytes (d_k = 64) have their chunks XOR-ed with 4*((k>>1)&1),
//              rows of 256 bytes with 4*(k&3), so the four k-rows of a patch meet different banks;
//   B operand: 16 bytes of the lane's own row of x, straight from global memory.
// xrow: the lane's row of x; wh: Wq at the first column of the head, row pitch hd; d_model % 64 == 0.
template <int DK, int WAVES>
__device__ __forceinline__ void project_queries(u32x4 (&qf)[DK / 16], const bf16_t* __restrict__ xrow,
                                                const bf16_t* __restrict__ wh, int d_model, int hd, float qscale,
                                                unsigned char* wbuf, int tid, int lane)
{
    constexpr int NDB = DK / 32, NKS = DK / 16;
    constexpr int SLK = 64, KSS = SLK / 16;  // rows of Wq and k-steps per slice
    constexpr int WROWB = DK * 2, CPRW = DK / 8, NCH = SLK * CPRW, NT = 64 * WAVES;
    constexpr int PER = (NCH + NT - 1) / NT;  // 16-byte chunks of a slice per thread
    constexpr int SLICE = SLK * WROWB;
    constexpr int AHEAD = 4;
    // Everything below depends on the lane only.  Taken from opaque copies of the thread and lane
    // numbers it is computed here, in every pass; otherwise the compiler hoists two dozen addresses
    // out of the pass loop and keeps them in scratch memory during the walk.
    asm volatile("" : "+v"(tid), "+v"(lane));
    const int g = lane >> 5;
    auto wswz = [](int kr) { return DK == 64 ? 4 * ((kr >> 1) & 1) : 4 * (kr & 3); };
    f32x16 qa[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) qa[db][e] = 0.f;
    // this lane's address of the transposing reads: k-step 0 of a slice, first read; the k-steps of a
    // slice lie 16 rows apart, which leaves the swizzle alone
    const unsigned lds_w = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)wbuf;
    unsigned wfo[NDB];
    {
        const int i16 = lane & 15;
        const int kr = 8 * g + (i16 >> 2);
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
            const int col = db * 32 + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
            wfo[db] = (unsigned)(kr * WROWB + (((col >> 3) ^ wswz(kr)) << 4) + ((col & 7) << 1));
        }
    }
    u32x4 wreg[AHEAD][PER], xreg[AHEAD][KSS];
    auto fetch = [&](int sl, auto set_) {
        constexpr int SET = decltype(set_)::value;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int c = tid + NT * u;
            if (c < NCH) wreg[SET][u] = *(const u32x4*)(wh + (size_t)(SLK * sl + c / CPRW) * hd + (c % CPRW) * 8);
        }
#pragma unroll
        for (int ks = 0; ks < KSS; ++ks) xreg[SET][ks] = *(const u32x4*)(xrow + SLK * sl + 16 * ks + 8 * g);
    };
    auto stage = [&](int buf, auto set_) {
        constexpr int SET = decltype(set_)::value;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int c = tid + NT * u;
            if (c < NCH) {
                const int kr = c / CPRW, p = c % CPRW;
                *(u32x4*)(wbuf + buf * SLICE + kr * WROWB + ((p ^ wswz(kr)) << 4)) = wreg[SET][u];
            }
        }
    };
    const int ns = d_model / SLK;
    // slice sl: Wq part in LDS buffer sl & 1 (staged during slice sl - 1), x in register set sl % AHEAD
    auto slice = [&](int sl, auto set_) {
        constexpr int SET = decltype(set_)::value;
        if (sl >= ns) return;
        const unsigned base = lds_w + (unsigned)((sl & 1) * SLICE);
        // the fragments of GRP k-steps are requested in one run and awaited once
        constexpr int GRP = KSS / 2;
#pragma unroll
        for (int k0 = 0; k0 < KSS; k0 += GRP) {
            u32x4 af[GRP][NDB];
#pragma unroll
            for (int kk = 0; kk < GRP; ++kk)
#pragma unroll
                for (int db = 0; db < NDB; ++db) {
                    u32x2 lo, hi;
                    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2"
                                 : "=v"(lo)
                                 : "v"(base + wfo[db]), "n"(16 * (k0 + kk) * WROWB));
                    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2"
                                 : "=v"(hi)
                                 : "v"(base + wfo[db]), "n"((16 * (k0 + kk) + 4) * WROWB));
                    af[kk][db] = u32x4{lo[0], lo[1], hi[0], hi[1]};
                }
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_waitcnt(0xC07F);  // the compiler does not count hand-written LDS reads
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kk = 0; kk < GRP; ++kk)
#pragma unroll
                for (int db = 0; db < NDB; ++db) qa[db] = mfma32(af[kk][db], xreg[SET][k0 + kk], qa[db]);
        }
        // the other buffer was last read in slice sl - 1, which every wavefront has left
        if (sl + 1 < ns) stage((sl + 1) & 1, std::integral_constant<int, (SET + 1) % AHEAD>{});
        if (sl + AHEAD < ns) fetch(sl + AHEAD, set_);
        __syncthreads();
    };
    static_for_q<AHEAD>([&](auto j_) { if (decltype(j_)::value < ns) fetch(decltype(j_)::value, j_); });
    stage(0, std::integral_constant<int, 0>{});
    __syncthreads();
#pragma nounroll
    for (int sl = 0; sl < ns; sl += AHEAD)
        static_for_q<AHEAD>([&](auto j_) { slice(sl + decltype(j_)::value, j_); });
    // Accumulator layout -> operand layout.  For k-step ks the lane holds, of the 16 columns,
    // {4g .. 4g+3} and {8+4g .. 8+4g+3}; the operand wants {8g .. 8g+7}: the halves of the wavefront
    // exchange one group of four.
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
        const int db = ks >> 1, hh = ks & 1;
        unsigned w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            w[j] = pack_f16_sat(qa[db][8 * hh + 2 * j] * qscale, qa[db][8 * hh + 2 * j + 1] * qscale);
        const unsigned s0 = g ? w[0] : w[2], s1 = g ? w[1] : w[3];
        const unsigned r0 = __shfl_xor(s0, 32, 64), r1 = __shfl_xor(s1, 32, 64);
        qf[ks] = g ? u32x4{r0, r1, w[2], w[3]} : u32x4{w[0], w[1], r0, r1};
    }
}

// FUSEQ: the query vectors are not read from the workspace but projected here, q = x.Wq (Sec. 3.1),
// by each wavefront for its own 32 rows in the prologue of a pass, and stay in registers: the
// inputs of the row block are loaded once and used for all three phases (the aim of Sec. 3.1 and
// 4.1), and the projection kernel in front computes k and v only.
template <int DK, int WAVES, bool CAUSAL, bool FUSEQ>
__global__ __launch_bounds__(64 * WAVES)
__attribute__((amdgpu_waves_per_eu(Pipe<DK, WAVES, CAUSAL>::OCC, Pipe<DK, WAVES, CAUSAL>::OCC)))
void attn_pipe_kernel(Problem pb, CountCfg cc, const h16_t* __restrict__ q, const h16_t* __restrict__ k,
                      const h16_t* __restrict__ vt, bf16_t* __restrict__ out, int n_qtiles, int per_head, int n_work,
                      const bf16_t* __restrict__ X, const bf16_t* __restrict__ Wq, float qscale, int single)
{
    typedef Pipe<DK, WAVES, CAUSAL> T;
    constexpr int NKS = T::NKS, NDB = T::NDB, BR = T::BR;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[T::STAGES * T::STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63, ln = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = WAVES == 8 ? (wave >> 2) : 0;  // which side of the workgroup barrier E(2t) lies on

    // Consecutive workgroup ids go to different XCDs; give each XCD a contiguous
    // run of work items so that the workgroups of one head share an L2.
    const int per_xcd = gridDim.x >> 3;
    int bh, x;
    if (CAUSAL && single) {
        // Masked scheme on a launch too small to give every CU several row-tile pairs: one row tile
        // per workgroup (x is the tile itself), all of them resident at once, three to a CU.  The
        // tiles of an XCD's heads, heaviest first, are dealt over its 32 CUs in rows that run forth
        // and back, so that the three tiles that meet on a CU weigh about the same everywhere
        // (workgroup j of an XCD is taken to land on CU j % 32; if it does not, nothing breaks).
        const int j = blockIdx.x >> 3;
        const int r = j >> 5, c = j & 31;
        const int row_len = min(32, per_xcd - (r << 5));
        const int p = (r << 5) + ((r & 1) ? row_len - 1 - c : c);
        const int nh = per_xcd / per_head;  // whole heads per XCD (the launcher sees to it)
        bh = (blockIdx.x & 7) * nh + p % nh;
        x = per_head - 1 - p / nh;
    } else {
        const int work = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
        if (work >= n_work) return;
        bh = work / per_head;
        x = work - bh * per_head;
        if (pb.skip_rows && ((pb.B * pb.H) & 7) == 0) {
            // With the padded rows left out the batch items differ in work by the square of their
            // lengths, and a run of heads is a run of whole items: an XCD takes every eighth head
            // instead, its share of every item.  (Measured at batch 32 x 2048 rows, lengths 64 .. 2048:
            // 0.524 -> 0.511 ms per call, packed layout 0.523 -> 0.498 ms.  With every query row
            // computed the items differ less and the same change gains nothing over a run of a
            // hundred calls: the kernel gets 6 % faster and the GEMM beside it as much slower - the
            // chip holds a power limit, and time follows the energy of a call, not its idle gaps.)
            const int j = (blockIdx.x >> 3) / per_head;  // head number within the XCD
            x = (blockIdx.x >> 3) - j * per_head;
            bh = j * 8 + (blockIdx.x & 7);
        }
    }
    const int bb = bh / pb.H, h = bh - bb * pb.H;

    const int N = pb.N, Npad = pb.Npad;
    int len = N;
    if (pb.lens) { len = pb.lens[bb]; len = len < 0 ? 0 : (len > N ? N : len); }
    const int rlen = pb.skip_rows ? len : N;  // query rows at or past it take part in no pair
    // Rows of `out`: n per batch item, or, in the packed layout, the item's own vectors and nothing
    // after them (the rows that follow belong to the next item and are not to be written).
    const size_t out_row0 = pb.row0 ? (size_t)pb.row0[bb] : (size_t)bb * N;
    const int n_out = pb.row0 ? rlen : N;
    const int nkt_all = Npad / BC;

    const h16_t* qh = q + (size_t)bh * Npad * DK;
    const unsigned char* kh = (const unsigned char*)(k + (size_t)bh * Npad * DK);
    const unsigned char* vh = (const unsigned char*)(vt + (size_t)bh * Npad * DK);

    // Swizzled LDS byte offsets of this lane's operand reads: K rows relative to the first row of
    // a 32-key block, V^T relative to the stage for the lower 32 keys of a tile (the upper 32 keys
    // lie 4 chunks further, which under the XOR swizzle is the offset XOR 64).
    int voff[2];
    const int koff0 = ln * T::KROWB + swz<T::KROWB>(g, ln) * 16;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) voff[hf] = T::K_BYTES + ln * (BC * 2) + swz<BC * 2>(2 * hf + g, ln) * 16;

    const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)kh, 0, -1, 0x00020000);
    const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)vh, 0, -1, 0x00020000);
    const unsigned k_lane_off = dma_lane_offset<T::KROWB>(wave, lane);
    const unsigned v_lane_off = dma_lane_offset<BC * 2>(wave, lane);

    unsigned long long cnt_logical = 0;  // per lane; summed over the wavefront at the end
    unsigned cnt_phys = 0;               // wave-uniform

    // Masked scheme: workgroup x takes row tiles T-1-x and x (Sec. 5.2).  With padded rows left
    // out, T counts the row tiles that hold a row below the key length, so that the pairing
    // balances the rows that are there; the row tiles past them only have zeros written, by two
    // more passes with no walk.
    const bool repair = CAUSAL && pb.skip_rows && !pb.noskip;
    const int n_live = repair ? (rlen + BR - 1) / BR : n_qtiles;
    const int n_pass = (CAUSAL && !single) ? (repair ? 4 : 2) : 1;
#pragma nounroll
    for (int pass = 0; pass < n_pass; ++pass) {
        int I;
        bool zeros_only = false;
        if (CAUSAL && single) {
            I = x;
        } else if (CAUSAL) {
            if (pass < 2) {
                I = pass == 0 ? n_live - 1 - x : x;
                // no such pair; the lower tile of a pair is a pass of its own only below the upper one
                if (n_live - 1 - x < x || (pass == 1 && x == n_live - 1 - x)) continue;
            } else {
                I = n_live + (pass - 2) * per_head + x;
                if (I >= n_qtiles || pb.row0) continue;  // packed layout: no such rows in `out`
                zeros_only = true;
            }
        } else {
            I = x;
        }
        const int i0w = I * BR + wave * 32;  // first row of this wavefront
        const int i = i0w + ln;              // this lane's query row
        const bool wave_active = i0w < (pb.noskip ? N : rlen);
        const bool cut_rows = rlen < i0w + 32;  // some of this wavefront's rows are left out: test every pair

        // The walk over 64-key tiles.  Needed tiles are J = 0 .. nJ-1.
        //   masked scheme: J = Js, Js-1, .., 0 (own diagonal tile first);
        //   FULL: the tile cut by the key length first (if any), then the whole
        //         tiles in ring order from the own tile.
        // In debug mode the tiles with no needed pair are walked first; they change nothing.
        // Inside a tile the upper 32 keys come first, so key offsets fall along the masked walk.
        int nJ = (len + BC - 1) / BC;
        if (CAUSAL) nJ = nJ < (I + 1) * (BR / BC) ? nJ : (I + 1) * (BR / BC);
        if (zeros_only) nJ = 0;
        const int n_dead = pb.noskip ? nkt_all - nJ : 0;
        const int nT = nJ + n_dead;
        const int has_cut = (!CAUSAL && (len % BC) != 0) ? 1 : 0;
        const int n_ring = nJ - has_cut;  // FULL: whole tiles
        const int Jown = (I + 1) * (BR / BC) - 1;
        const int Js = CAUSAL ? nJ - 1 : (Jown < n_ring ? Jown : n_ring - 1);
        auto tile_of_step = [&](int t) -> int {
            if (t < n_dead) return nkt_all - 1 - t;
            t -= n_dead;
            if (CAUSAL) return Js - t;
            if (t < has_cut) return nJ - 1;
            int J = Js - (t - has_cut);
            return J < 0 ? J + n_ring : J;
        };
        const int NB = 2 * nT;  // 32-key blocks of the walk
        auto key_of_block = [&](int n) -> int { return tile_of_step(n >> 1) * BC + 32 * (1 - (n & 1)); };
        auto block_needed = [&](int kb) -> bool { return pb.noskip || (kb < len && (!CAUSAL || kb <= i0w)); };
        auto block_is_edge = [&](int kb) -> bool {
            return pb.noskip || cut_rows || kb + 32 > len || (CAUSAL && kb + 31 > i0w);
        };
        // The blocks a wavefront leaves out lie at the head of the walk, its edge blocks follow,
        // the rest are blocks in which every pair is allowed.
        int n_first = 0;
        if (!wave_active) n_first = NB;
        while (n_first < NB && !block_needed(key_of_block(n_first))) ++n_first;
        int n_edge_end = n_first;
        while (n_edge_end < NB && block_is_edge(key_of_block(n_edge_end))) ++n_edge_end;

        // ---- counts: logical tiles whose first pair is allowed ----
        if (n_first < NB) {
            cnt_phys += (unsigned)(NB - n_first);
            const int rcnt = pb.noskip ? N : rlen;  // rows that anchor counted tiles
            const unsigned nr_anchor = cdiv_b(min(i0w + 32, rcnt), cc) - cdiv_b(min(i0w, rcnt), cc);
            if (pb.noskip) {
                if (lane == 0) cnt_logical += (unsigned long long)nr_anchor * cdiv_b(N, cc);
            } else {
                // whole blocks below the diagonal block and below the key length: every pair allowed
                int k_int = (len >> 5) << 5;
                if (CAUSAL) k_int = k_int < i0w ? k_int : i0w;
                if (k_int < 0) k_int = 0;
                if (lane == 0) cnt_logical += (unsigned long long)nr_anchor * cdiv_b(k_int, cc);
                // the rest (diagonal block, block cut by the key length): pair by pair
                const int k_end = CAUSAL ? (len < i0w + 32 ? len : i0w + 32) : len;
                if (g == 0 && i < rlen && is_multiple(i, cc)) {
#pragma nounroll
                    for (int j = (int)cdiv_b(k_int, cc) * cc.b; j < k_end; j += cc.b)
                        cnt_logical += (!CAUSAL || j <= i) ? 1u : 0u;
                }
            }
        }

        typename T::Row r;
#pragma unroll
        for (int db = 0; db < NDB; ++db) r.O[db] = T::zero16();
        r.S = T::zero16();
        r.Cneg = T::zero16();
        r.P[0] = r.P[1] = u32x4{0u, 0u, 0u, 0u};
        r.thr = -INFINITY;
        r.mref = 0.f;
        r.l = 0.f;

        if (nT > 0) {
            // Q rows of this wavefront as B operands (rows >= n of the workspace are zero).
            u32x4 qf[NKS];
            if constexpr (!FUSEQ) {
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) qf[ks] = *(const u32x4*)(qh + (size_t)i * DK + ks * 16 + g * 8);
            }

            // Piece c (K pieces first) of the tile with K at byte ksoff and V^T at byte vsoff of the
            // head, into the stage at LDS byte `stage`.  A buffer load: descriptor base, the lane's
            // offset inside its piece, a scalar offset for tile and piece; no vector instruction.
            auto issue_piece = [&](int c, int ksoff, int vsoff, unsigned stage) {
                if (c < T::KPIECES) {
                    const int m = wave + c * WAVES;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        k_rsrc, (__attribute__((address_space(3))) void*)(lds + stage + m * 1024), 16,
                        (int)k_lane_off, ksoff + m * 1024, 0, 0);
                } else {
                    const int m = wave + (c - T::KPIECES) * WAVES;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        v_rsrc, (__attribute__((address_space(3))) void*)(lds + stage + T::K_BYTES + m * 1024), 16,
                        (int)v_lane_off, vsoff + m * 1024, 0, 0);
                }
            };
            auto issue_tile = [&](int u) {
                const int J = tile_of_step(u);
                const unsigned stage = (unsigned)(u % T::STAGES) * T::STAGE;
#pragma unroll
                for (int c = 0; c < T::PPW; ++c) issue_piece(c, J * T::K_BYTES, J * T::V_BYTES, stage);
            };
            // A tile whose pieces this wavefront still has to request (SPREAD): set by the barrier
            // that frees the stage, worked off by the two matrix phases that follow it.
            // LDS byte offsets of the stages of the walk's current tile and of the one after it,
            // kept by increments
            constexpr unsigned RING = T::STAGES * T::STAGE;
            unsigned stg = 0, stg_n = 0;
            bool req_on = false;
            int req_k = 0, req_v = 0;
            unsigned req_stage = 0;
            // Start of tile t: tiles t and t+1 are in LDS, every wavefront is done with tile t-1,
            // whose stage takes tile t+STAGES-1 (`defer`: by and by, see above).
            auto tile_sync = [&](int t, bool defer) {
                // tiles t+2 .. t+STAGES-2 may stay in flight, as far as the walk has them
                const int ahead = nT - 2 - t;
                if (T::STAGES > 4 && ahead >= 2) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * T::PPW));
                else if (T::STAGES > 3 && ahead >= 1) __builtin_amdgcn_s_waitcnt(0x0F70 | T::PPW);
                else __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
                __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0): this wavefront's LDS reads are done
                __builtin_amdgcn_s_barrier();
                const int u = t + T::STAGES - 1;
                if (u < nT) {
                    if (T::SPREAD && defer) {
                        const int J = tile_of_step(u);
                        req_on = true;
                        req_k = J * T::K_BYTES;
                        req_v = J * T::V_BYTES;
                        req_stage = stg == 0 ? RING - T::STAGE : stg - T::STAGE;  // the stage tile t-1 has left
                    } else {
                        issue_tile(u);
                    }
                }
            };
            // prologue of the ring: the first STAGES-1 tiles requested, tiles 0 and 1 awaited
            {
                const int pre = nT < T::STAGES - 1 ? nT : T::STAGES - 1;
                for (int u = 0; u < pre; ++u) issue_tile(u);
                // the last stage of the ring is free until the first barrier: the weight slices of
                // the query projection pass through it while the first tiles are on their way
                if constexpr (FUSEQ)
                    project_queries<DK, WAVES>(qf, X + ((size_t)bb * N + (i < N ? i : N - 1)) * pb.D, Wq + (size_t)h * DK,
                                               pb.D, pb.H * DK, qscale, lds + (T::STAGES - 1) * T::STAGE, tid, lane);
                tile_sync(0, false);
            }
            // The barrier of tile t (t >= 1) lies in front of E(2t) for group 0 and between E(2t) and
            // M(2t) for group 1.  A wavefront that joins the walk at block n_first first passes the
            // barriers that lie in front of E(n_first).
            int next_sync = 1;
            {
                const int upto = grp == 0 ? (n_first >> 1) : ((n_first - 1) >> 1);  // n_first == 0: none
                for (; next_sync <= upto && next_sync < nT; ++next_sync) tile_sync(next_sync, false);
            }

            if (n_first < NB) {
                typename T::Frags fr;
                int t = n_first >> 1;
                stg = (unsigned)(t % T::STAGES) * T::STAGE;
                stg_n = stg + T::STAGE == RING ? 0u : stg + T::STAGE;
                // scores of the first block, outside the rotation
                {
                    T::read_k(fr, lds, stg + (1 - (n_first & 1)) * 32 * T::KROWB + koff0);
                    r.S = T::scores(r, fr, qf, [](int) {});
                }
                int lim_base = len - 1;  // the lane's last allowed key
                if (CAUSAL) lim_base = lim_base < i ? lim_base : i;
                if (i >= rlen) lim_base = -1;  // a row that is left out has no allowed key
                const bool live = lim_base >= 0;
                bool fresh = true;  // a live row may still be without a reference
                lim_base -= 4 * g;

                // E(n) for the upper (UPPER = 1: first block of a tile) or lower 32 keys of tile t
                auto phase_e = [&](auto upper, bool masked, int J) {
                    constexpr int UPPER = decltype(upper)::value;
                    if (masked) T::mask_block(r.S, lim_base - (J * BC + 32 * UPPER));
                    if (fresh) {
                        // Some row that has an allowed key is still without a reference: the largest
                        // score of its first block with a finite one becomes it.
                        const float mxl = T::USE_CNEG ? T::max16(r.S) : T::max16(r.S) - r.mref;
                        if (__builtin_amdgcn_ballot_w64(mxl > r.thr) != 0ull) T::raise_reference(r, mxl);
                        fresh = __builtin_amdgcn_ballot_w64(live && !(r.thr > -INFINITY)) != 0ull;
                    }
                    // The LDS requests for M(n) go out between the exponentials, a quarter of them
                    // behind every second pair: K of the next block (the lower half of this tile or
                    // the upper half of the next tile), which M(n) takes first, and V^T of this block.
                    // In one run they queue up behind those of the other wavefronts and hold this one.
                    const unsigned ka0 = (UPPER ? stg : stg_n + 32 * T::KROWB) + koff0;
                    const unsigned char* vstage = lds + stg;
                    const int voff0 = voff[0] ^ (64 * UPPER), voff1 = voff[1] ^ (64 * UPPER);
                    auto reads = [&](int p) {
                        if ((p & 1) == 0) return;
                        const int q = p >> 1;  // 0..3
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int u = 0; u < NKS / 4; ++u) fr.kf[q * (NKS / 4) + u] = T::read_k1(lds, ka0, q * (NKS / 4) + u);
#pragma unroll
                        for (int u = 0; u < (2 * NDB) / 4; ++u) {
                            const int e = q * ((2 * NDB) / 4) + u, hf = e / NDB, db = e % NDB;
                            fr.vf[hf][db] = *(const u32x4*)(vstage + (hf ? voff1 : voff0) + db * 32 * (BC * 2));
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    };
                    float bsum;
                    if constexpr (!T::USE_CNEG) bsum = T::template exponentials<true>(r, r.mref, reads);
                    else bsum = T::template exponentials<false>(r, 0.f, reads);
                    // The reference follows the scores lazily, and what tells that it has fallen too
                    // far behind is the sum the phase forms anyway: no row maximum in the common case.
                    // Then the reference goes up to the row's largest score of this block and the
                    // exponentials of the block are taken again; O and l do not hold this block yet.
                    if (__builtin_amdgcn_ballot_w64(bsum > PIPE_SUM_LIMIT) != 0ull) {
                        const float mxl = T::USE_CNEG ? T::max16(r.S) : T::max16(r.S) - r.mref;
                        T::raise_reference(r, mxl);
                        if constexpr (!T::USE_CNEG) bsum = T::template exponentials<true>(r, r.mref, [](int) {});
                        else bsum = T::template exponentials<false>(r, 0.f, [](int) {});
                    }
                    r.l += bsum;
                    // The weights are wanted here: without a use at this point the compiler sinks the
                    // exponentials into the matrix phase, down to the block of their first MFMA.
                    asm volatile("" : "+v"(r.P[0]), "+v"(r.P[1]), "+v"(r.l));
                };
                // M(n).  HALF: 0 / 1 for the first / second matrix phase behind a tile's barrier, which
                // request the first / second half of the pending tile's pieces, each behind an
                // MFMA of its own (a run of requests stalls on the queue of the address unit, and
                // every wavefront of the workgroup would issue its run at the same moment); -1: none.
                auto phase_m = [&](auto half) {
                    constexpr int HALF = decltype(half)::value;
                    constexpr int NMF = NKS + 2 * NDB;
                    constexpr int PER = T::PPW / 2;
                    auto between = [&](int m) {
                        if constexpr (HALF >= 0 && T::SPREAD) {
#pragma unroll
                            for (int j = 0; j < PER; ++j)
                                if (m == 1 + j * (NMF / PER)) {
                                    __builtin_amdgcn_sched_barrier(0);
                                    if (req_on) issue_piece(HALF * PER + j, req_k, req_v, req_stage);
                                    __builtin_amdgcn_sched_barrier(0);
                                }
                        }
                    };
                    __builtin_amdgcn_sched_barrier(0);  // the vector phase stays in front of the matrix phase
                    __builtin_amdgcn_s_setprio(1);
                    r.S = T::scores(r, fr, qf, between);  // first, so that E(n+1) finds them done; after
                                                          // the last block: of stale keys, unused
                    T::weighted_sum(r, fr, between);
                    __builtin_amdgcn_s_setprio(0);
                    if (HALF == 1) req_on = false;
                };
                const std::integral_constant<int, 0> first_m{};
                const std::integral_constant<int, 1> second_m{};
                const std::integral_constant<int, -1> plain_m{};
                auto next_tile = [&]() {
                    ++t;
                    stg = stg_n;
                    stg_n = stg_n + T::STAGE == RING ? 0u : stg_n + T::STAGE;
                };
                // tiles [t, t_end): both blocks of each, with the group's barrier position
                auto run_tiles = [&](int t_end, bool masked) {
#pragma nounroll
                    while (t < t_end) {
                        const int J = masked ? tile_of_step(t) : 0;
                        if (grp == 0 && t >= next_sync) { tile_sync(t, true); ++next_sync; }
                        phase_e(std::integral_constant<int, 1>{}, masked, J);
                        if (grp == 1 && t >= next_sync) { tile_sync(t, true); ++next_sync; }
                        phase_m(first_m);
                        phase_e(std::integral_constant<int, 0>{}, masked, J);
                        phase_m(second_m);
                        next_tile();
                    }
                };
                // a walk that starts with the lower block of a tile
                if (n_first & 1) {
                    const bool masked = n_first < n_edge_end;
                    phase_e(std::integral_constant<int, 0>{}, masked, masked ? tile_of_step(t) : 0);
                    phase_m(plain_m);
                    next_tile();
                }
                const int t_edge_end = (n_edge_end + 1) >> 1;  // tiles that hold an edge block: pair tests
                run_tiles(t_edge_end < nT ? t_edge_end : nT, true);
                run_tiles(nT, false);
            }
            // keep the ring going to its end (wavefronts that never joined the walk)
            for (; next_sync < nT; ++next_sync) tile_sync(next_sync, false);
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();  // the next pass refills the stages
        }

        // y_i = O_i / l_i ; a row with no allowed pair is zero.  A lane owns 8-byte runs of 32 rows,
        // so the wavefront's 32 x d_k tile goes through LDS (the ring is idle between passes; rows
        // swizzled by 16-byte chunk as everywhere) and leaves as whole 16-byte pieces, four or eight
        // full rows per store instruction.
        {
            constexpr int CPR = DK / 8;  // 16-byte chunks per row
            const float l_tot = r.l + __shfl_xor(r.l, 32, 64);
            const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
            unsigned char* stage = lds + wave * (32 * DK * 2);
            // The addresses below depend on the lane only.  Computed from an opaque copy of the lane
            // number they stay here; otherwise the compiler hoists them out of the pass loop, spills
            // them, and reloads them one by one between the stores, and every reload then waits
            // (vmcnt) until the store before it has been acknowledged by memory.
            int le = lane;
            asm volatile("" : "+v"(le));
            const int ln_e = le & 31, g_e = le >> 5;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    u32x2 w;
                    w[0] = pack_bf16(r.O[db][4 * r4 + 0] * inv, r.O[db][4 * r4 + 1] * inv);
                    w[1] = pack_bf16(r.O[db][4 * r4 + 2] * inv, r.O[db][4 * r4 + 3] * inv);
                    const int c = 4 * db + r4;
                    *(u32x2*)(stage + ln_e * (DK * 2) + ((c ^ (ln_e & (CPR - 1))) << 4) + 8 * g_e) = w;
                }
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): only this wavefront reads what it wrote
            bf16_t* obase = out + (out_row0 + i0w) * ((size_t)pb.H * DK) + (size_t)h * DK;
#pragma unroll
            for (int it = 0; it < 32 * CPR / 64; ++it) {
                const int row = it * (64 / CPR) + le / CPR, c = le % CPR;
                const u32x4 v = *(const u32x4*)(stage + row * (DK * 2) + ((c ^ (row & (CPR - 1))) << 4));
                if (i0w + row < n_out) *(u32x4*)(obase + (size_t)row * ((size_t)pb.H * DK) + c * 8) = v;
            }
            if (pass + 1 < n_pass) {
                // the next pass refills the ring: every wavefront has to be done with its staging first
                __builtin_amdgcn_s_waitcnt(0xC07F);
                __builtin_amdgcn_s_barrier();
            }
        }
    }

    // one atomic per wavefront
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt_logical += __shfl_xor(cnt_logical, o, 64);
    if (lane == 0) {
        count_add(pb.counters, blockIdx.x, cnt_logical, cnt_phys);
    }
}

}  // namespace

hipError_t launch_attn_pipe(const Problem& pb, const h16_t* q, const h16_t* k, const h16_t* vt, bf16_t* out,
                            int waves, hipStream_t s, const bf16_t* X, const bf16_t* Wq)
{
    const bool causal = pb.scheme == SCHEME_CAUSAL;
    const bool fuse = X != nullptr && Wq != nullptr;  // queries projected inside the kernel
    const float qscale = pb.scale * 1.4426950408889634f;
    const int br = 32 * waves;
    const int n_qtiles = (pb.N + br - 1) / br;
    // One row tile per workgroup instead of a pair when the pairs would not give every CU four
    // workgroups (and the heads divide evenly over the eight XCDs, padded rows are not left out).
    // Measured, 128-row workgroups: batch 8, n 1024, 12 heads 39.5 -> 32 us, batch 2 27 -> 23 us,
    // even at 768 pairs; with 256-row workgroups the pairing stays ahead (d_k = 128, 512 pairs: +5 %).
    const bool single = causal && waves == 4 && !pb.skip_rows && (pb.B * pb.H) % 8 == 0 &&
                        (long)pb.B * pb.H * ((n_qtiles + 1) / 2) < 4L * 256;
    const int per_head = (causal && !single) ? (n_qtiles + 1) / 2 : n_qtiles;
    const int n_work = pb.B * pb.H * per_head;
    const int grid = ((n_work + 7) / 8) * 8;
    CountCfg cc;
    cc.b = pb.b;
    cc.b_shift = -1;
    for (int sft = 0; sft < 31; ++sft)
        if ((1 << sft) == pb.b) cc.b_shift = sft;
#define ATTN_LAUNCH(DK_, W_, C_, F_)                                                                                    \
    hipLaunchKernelGGL((attn_pipe_kernel<DK_, W_, C_, F_>), dim3(grid), dim3(64 * W_), 0, s, pb, cc, q, k, vt, out, \
                       n_qtiles, per_head, n_work, X, Wq, qscale, single ? 1 : 0)
#define ATTN_PICK(DK_, W_)                                                                  \
    do {                                                                                    \
        if (causal) { if (fuse) ATTN_LAUNCH(DK_, W_, true, true); else ATTN_LAUNCH(DK_, W_, true, false); }   \
        else { if (fuse) ATTN_LAUNCH(DK_, W_, false, true); else ATTN_LAUNCH(DK_, W_, false, false); }        \
    } while (0)
    if (pb.d == 64 && waves == 4) ATTN_PICK(64, 4);
    else if (pb.d == 64 && waves == 8) ATTN_PICK(64, 8);
    else if (pb.d == 128 && waves == 8) ATTN_PICK(128, 8);
    else return hipErrorInvalidValue;
#undef ATTN_PICK
#undef ATTN_LAUNCH
    return hipGetLastError();
}

}  // namespace attnring
