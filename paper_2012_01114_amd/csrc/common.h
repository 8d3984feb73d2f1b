// Internal declarations shared by the translation units of libattnring.so.
// Nothing here is part of the public C ABI (see include/attnring.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace attnring {

typedef unsigned short bf16_t;  // raw bfloat16 bits: the caller's X, W and out
typedef unsigned short h16_t;   // raw half-precision bits: the projected q, k, v between the kernels

enum { SCHEME_FULL = 0, SCHEME_SYMMETRIC = 1, SCHEME_CAUSAL = 2 };

// Everything a kernel launcher needs to know about one forward call.
struct Problem {
    int B, N, D, H, d;   // batch, vectors, d_model, heads, d_k
    int P, b;            // ring partitions and rows per partition (b = N / P)
    int Npad;            // row pitch of the projected bf16 q/k/v (multiple of 256)
    float scale;         // multiplies the raw scores
    int scheme;
    bool noskip;         // debug: visit every tile, mask with -inf
    bool skip_rows;      // with key lengths: rows i >= len take part in no pair and give zeros
    bool no_q;           // the projection kernel leaves q out (q = k = v scheme; queries projected by the attention kernel)
    bool is_bf16;        // storage type of X, W, out
    const int* lens;     // device, [B] or nullptr
    const int* row0;     // packed layout of x and out: device, [B + 1] first rows of the batch items; else nullptr
    unsigned long long* counters;  // device: CNT_SLOTS slots of (logical tiles, physical score blocks), then totals
};

// Device counters written by the attention kernels.  Adds to one address from thousands of
// wavefronts serialise in L2, so the kernels add into one of CNT_SLOTS slots, each on a cache
// line of its own, chosen by work item; a one-workgroup kernel sums the slots into the totals
// (the two words that follow the slots) when the counts are asked for.
enum { CNT_LOGICAL = 0, CNT_PHYS = 1, CNT_WORDS = 2 };
enum { CNT_SLOTS = 1024, CNT_SLOT_WORDS = 16, CNT_TOTALS = CNT_SLOTS * CNT_SLOT_WORDS,
       CNT_BUFFER_WORDS = CNT_TOTALS + CNT_WORDS };
__device__ __forceinline__ void count_add(unsigned long long* counters, unsigned item, unsigned long long logical,
                                          unsigned long long phys)
{
    unsigned long long* slot = counters + (size_t)(item & (CNT_SLOTS - 1)) * CNT_SLOT_WORDS;
    if (logical) atomicAdd(&slot[CNT_LOGICAL], logical);
    if (phys) atomicAdd(&slot[CNT_PHYS], phys);
}

// Row of the caller's x (and out) that holds vector i of batch item bb.  Padded layout: every item
// has N rows.  Packed layout: item bb has rows row0[bb] .. row0[bb + 1] - 1 and nothing follows its
// last vector; a vector at or past its length is in no allowed pair, and a read for it (whole tiles
// are fetched) is pointed at a row that exists.
__device__ __forceinline__ unsigned source_row(const int* __restrict__ row0, int Bsz, int N, int bb, int i)
{
    if (row0 == nullptr) return (unsigned)(bb * N + (i < N ? i : N - 1));
    const int first = row0[bb], len = row0[bb + 1] - first, total = row0[Bsz];
    i = i < len ? i : len - 1;
    int r = first + (i < 0 ? 0 : i);
    r = r < total ? r : total - 1;
    return (unsigned)(r < 0 ? 0 : r);
}

// ---- generic float-compute path (any shape, f32 or bf16 storage) ----------
// q/k/v workspace: float [B][H][N][d].
hipError_t launch_proj_generic(const Problem& pb, const void* X, const void* W, float* out, hipStream_t s);
hipError_t launch_copy_heads_generic(const Problem& pb, const void* X, float* out, hipStream_t s);
hipError_t launch_attn_generic(const Problem& pb, const float* q, const float* k, const float* v,
                               void* out, hipStream_t s);
hipError_t launch_sym_generic(const Problem& pb, const float* z, float* scores, void* out, hipStream_t s);

// ---- matrix-core path (bf16 storage, d_k 64 or 128, FULL and CAUSAL) --------
// The projection contracts bf16 operands; q, k, v leave it in half precision (fp32 accumulators
// rounded once to an 11-bit significand instead of bfloat16's 8: with bfloat16 there, the roundings
// of q, k and v alone reach 1.5e-2 on outputs of size 2, three quarters of the 2e-2 allowed) and the
// attention kernel contracts half-precision operands, at the same matrix-core rate.
// q, k: [B][H][Npad][d]; vt: [B][H][Npad/64][d][64] with the keys of every 16-group stored in MFMA
// operand order.  Wt: [3][H*d][D], transposed weights, needed only when the projection cannot read
// the weights in place (launch_transpose_w fills it, and is then the first kernel of the call).
hipError_t launch_transpose_w(const Problem& pb, const bf16_t* Wq, const bf16_t* Wk, const bf16_t* Wv,
                              bf16_t* Wt, hipStream_t s);
bool proj_reads_weights_in_place(const Problem& pb, const bf16_t* Wq, const bf16_t* Wk, const bf16_t* Wv);
hipError_t launch_proj_mfma(const Problem& pb, const bf16_t* X, const bf16_t* Wq, const bf16_t* Wk,
                            const bf16_t* Wv, const bf16_t* Wt, h16_t* q, h16_t* k, h16_t* vt, hipStream_t s);
// Fused phases 1-3 with redundant blocks left out; `waves` wavefronts of 32 rows per workgroup:
// 4 or 8 for d_k = 64, 8 for d_k = 128.
// X and Wq given: the kernel projects its queries itself (q is not read).
hipError_t launch_attn_pipe(const Problem& pb, const h16_t* q, const h16_t* k, const h16_t* vt,
                            bf16_t* out, int waves, hipStream_t s, const bf16_t* X = nullptr,
                            const bf16_t* Wq = nullptr);
// q = k = v scheme on the matrix cores: every 128 x 128 score tile computed once and used for both
// of its row blocks, partial row states merged by a second kernel.  z, zt: the shared vectors in
// the k and v^T layouts above; work: sym_pair_workspace_floats(pb) floats.
size_t sym_pair_workspace_floats(const Problem& pb);
hipError_t launch_sym_pair(const Problem& pb, const h16_t* z, const h16_t* zt, float* work, bf16_t* out, hipStream_t s);
// Physical score-block edge of the MFMA attention kernels (phys_br = phys_bc).
enum { MFMA_BLOCK = 32 };

}  // namespace attnring
