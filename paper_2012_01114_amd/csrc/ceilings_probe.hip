// Ceilings of the units the fused attention kernel keeps busy, measured one by one and together:
// matrix cores (32x32x16 half-precision MFMAs), vector ALUs (the per-pair work of the online softmax,
// Eq. (2): subtraction, exp2, conversion to half precision, row-sum addition) and LDS fragment reads
// (one 16-byte-per-lane read per MFMA, as the kernel issues them).  Built into libattnprobe.so, not
// into the product library; instrumentation only.
//
// A "group" is what one wavefront does per 32 x 32 score block at d_k = 128: 16 MFMAs, with the
// vector work of 8 score pairs per lane (16 at d_k = 64 density) and 16 fragment reads spread
// between them.  Operands are either constants or hashed half-precision values in (-2, 2): the
// power the matrix cores draw, and with it the clock the chip holds, depends on the data.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

enum { UNIT_MFMA = 1, UNIT_VALU = 2, UNIT_LDS = 4 };

__device__ __forceinline__ unsigned pack_f16(float a, float b)
{
    f32x2 v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, f16x2));
}
__device__ __forceinline__ unsigned hashed_half2(unsigned& h)
{
    h = h * 1664525u + 1013904223u;
    return (h & 0x83ff83ffu) | 0x38003800u;  // sign, exponent of 0.5 .. 2, random significand
}

// PAIRS2: score pairs per two MFMAs (1: d_k = 128 density, 2: d_k = 64 density)
template <int UNITS, int PAIRS2>
__global__ __launch_bounds__(256) void probe_kernel(float* out, long long* cycles, int iters, int random_operands)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[65536];
    f32x16 acc[8];
    for (int a = 0; a < 8; ++a)
        for (int e = 0; e < 16; ++e) acc[a][e] = 0.f;
    unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u;
    u32x4 A, B;
    for (int j = 0; j < 4; ++j) {
        A[j] = random_operands ? hashed_half2(h) : 0x3c003c00u;
        B[j] = random_operands ? hashed_half2(h) : 0x3c003c00u;
    }
    for (int i = threadIdx.x; i < 65536 / 4; i += blockDim.x) {
        unsigned g = (i + blockIdx.x * 977u) * 2654435761u;
        ((unsigned*)lds)[i] = random_operands ? hashed_half2(g) : 0x3c003c00u;
    }
    __syncthreads();
    float s[16];
    for (int e = 0; e < 16; ++e) s[e] = 0.01f * (e + 1) + threadIdx.x * 1e-3f;
    float ref = 0.03f, sum0 = 0.f, sum1 = 0.f;
    unsigned P[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    u32x4 fr[16];
    for (int m = 0; m < 16; ++m) fr[m] = A;
    const unsigned la = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)lds +
                        (threadIdx.x & 63) * 16 + (threadIdx.x >> 6) * 8192;
    const long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            __builtin_amdgcn_sched_barrier(0);
            if (UNITS & UNIT_LDS) {  // the fragment of this MFMA was requested 15 requests ago
                __builtin_amdgcn_s_waitcnt(0xC07F | (15 << 8));
                __builtin_amdgcn_sched_barrier(0);
            }
            if (UNITS & UNIT_MFMA)
                acc[m & 7] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                    __builtin_bit_cast(f16x8, (UNITS & UNIT_LDS) ? fr[m] : A), __builtin_bit_cast(f16x8, B), acc[m & 7], 0, 0, 0);
            if (UNITS & UNIT_LDS)
                asm volatile("ds_read_b128 %0, %1 offset:%2" : "+v"(fr[m]) : "v"(la), "n"((m & 7) * 1024));
            if (UNITS & UNIT_VALU) {
#pragma unroll
                for (int p = (m * PAIRS2) / 2; p < ((m + 1) * PAIRS2) / 2; ++p) {
                    const int e = p % 8;
                    const float p0 = __builtin_amdgcn_exp2f(s[2 * e] - ref), p1 = __builtin_amdgcn_exp2f(s[2 * e + 1] - ref);
                    P[e] = pack_f16(p0, p1);
                    sum0 += p0;
                    sum1 += p1;
                    s[2 * e] += 1e-3f;  // keeps the iterations distinct
                }
                asm volatile("" : "+v"(sum0), "+v"(sum1));
            }
        }
        asm volatile("" ::"v"(P[0]), "v"(P[1]), "v"(P[2]), "v"(P[3]), "v"(P[4]), "v"(P[5]), "v"(P[6]), "v"(P[7]));
    }
    const long long t1 = __builtin_readcyclecounter();
    __builtin_amdgcn_s_waitcnt(0xC07F);
    float r = sum0 + sum1;
    for (int m = 0; m < 16; ++m) r += __uint_as_float(fr[m][0]);
    for (int a = 0; a < 8; ++a) r += acc[a][0];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
    if (threadIdx.x == 0) cycles[blockIdx.x] = t1 - t0;
}

template <int UNITS, int PAIRS2>
int run(int waves_per_simd, int iters, int random_operands, double* ns_per_group, double* cycles_per_group)
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 5;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 5;
    const int nblk = cus * waves_per_simd;  // 256 threads = one wavefront per SIMD and workgroup
    float* out = nullptr;
    long long* cyc = nullptr;
    if (hipMalloc((void**)&out, sizeof(float) * nblk * 256) != hipSuccess) return 4;
    if (hipMalloc((void**)&cyc, sizeof(long long) * nblk) != hipSuccess) { (void)hipFree(out); return 4; }
    hipEvent_t e0, e1;
    int rc = 0;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) rc = 5;
    if (!rc) {
        hipLaunchKernelGGL((probe_kernel<UNITS, PAIRS2>), dim3(nblk), dim3(256), 0, 0, out, cyc, 10, random_operands);
        (void)hipEventRecord(e0, 0);
        hipLaunchKernelGGL((probe_kernel<UNITS, PAIRS2>), dim3(nblk), dim3(256), 0, 0, out, cyc, iters, random_operands);
        (void)hipEventRecord(e1, 0);
        if (hipDeviceSynchronize() != hipSuccess) rc = 5;
    }
    if (!rc) {
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        long long* h = new long long[nblk];
        (void)hipMemcpy(h, cyc, sizeof(long long) * nblk, hipMemcpyDeviceToHost);
        double avg = 0;
        for (int i = 0; i < nblk; ++i) avg += (double)h[i];
        delete[] h;
        // per SIMD: waves_per_simd wavefronts share it, each doing `iters` groups in the measured time
        *ns_per_group = (double)ms * 1e6 / iters / waves_per_simd;
        *cycles_per_group = avg / nblk / iters / waves_per_simd;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipFree(out);
    (void)hipFree(cyc);
    return rc;
}

// The instruction stream of one 32 x 32 block of the attention walk at d_k = 64, without any memory
// behind it (no copies into LDS, no barrier): a vector phase (16 exponentials per lane, their packing
// and their row sums, the check of the block sum) and a matrix phase (the 4-MFMA score chain of the
// next block, whose accumulator starts at minus the reference, and the 4 weighted-sum MFMAs), in
// the order of the kernel (DEFERRED 0) or with the weighted sum of the block before issued between
// the exponentials (DEFERRED 1); READS adds the 8 LDS fragment reads of a block.  Operands random.
template <int DEFERRED, int READS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3)))
void block_kernel(float* out, long long* cycles, int iters, float seed)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[32768];
    unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u;
    for (int i = threadIdx.x; i < 32768 / 4; i += blockDim.x) ((unsigned*)lds)[i] = hashed_half2(h);
    __syncthreads();
    u32x4 qf[4], kf[4], vf[4];
    for (int j = 0; j < 4; ++j)
        for (int c = 0; c < 4; ++c) { qf[j][c] = hashed_half2(h); kf[j][c] = hashed_half2(h); vf[j][c] = hashed_half2(h); }
    f32x16 O[2], S, Cneg;
    for (int e = 0; e < 16; ++e) { O[0][e] = O[1][e] = 0.f; S[e] = seed * e; Cneg[e] = -seed; }
    u32x4 P[2][2];
    for (int a = 0; a < 2; ++a)
        for (int b = 0; b < 2; ++b) P[a][b] = u32x4{0u, 0u, 0u, 0u};
    float l = 0.f;
    const unsigned char* lane_lds = lds + (threadIdx.x & 63) * 16 + (threadIdx.x >> 6) * 8192;
    auto mf = [](u32x4 a, u32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    };
    const long long t0 = __builtin_readcyclecounter();
#pragma nounroll
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int set = DEFERRED ? half : 0, prev = DEFERRED ? 1 - half : 0;
            float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                if (DEFERRED && (p & 1) == 0) {
                    __builtin_amdgcn_sched_barrier(0);
                    const int e = p >> 1;
                    O[e & 1] = mf(vf[e], P[prev][e >> 1], O[e & 1]);
                    __builtin_amdgcn_sched_barrier(0);
                }
                const float p0 = __builtin_amdgcn_exp2f(S[2 * p] * 1e-3f), p1 = __builtin_amdgcn_exp2f(S[2 * p + 1] * 1e-3f);
                P[set][p >> 2][p & 3] = pack_f16(p0, p1);
                ps0 += p0;
                ps1 += p1;
                if (READS && (p & 1)) {
                    __builtin_amdgcn_sched_barrier(0);
                    const int q = p >> 1;
                    kf[q] = *(const u32x4*)(lane_lds + q * 1024);
                    vf[q] = *(const u32x4*)(lane_lds + 4096 + q * 1024);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            const float bs = ps0 + ps1;
            if (__builtin_amdgcn_ballot_w64(bs > 1e30f) != 0ull) {
                for (int e = 0; e < 16; ++e) { O[0][e] *= 0.5f; O[1][e] *= 0.5f; }
            }
            l += bs;
            asm volatile("" : "+v"(P[set][0]), "+v"(P[set][1]), "+v"(l));
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(1);
            asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %3" : "=&v"(S) : "v"(kf[0]), "v"(qf[0]), "v"(Cneg));
            for (int ks = 1; ks < 4; ++ks) S = mf(kf[ks], qf[ks], S);
            if (!DEFERRED)
                for (int e = 0; e < 4; ++e) O[e & 1] = mf(vf[e], P[0][e >> 1], O[e & 1]);
            __builtin_amdgcn_s_setprio(0);
        }
    }
    const long long t1 = __builtin_readcyclecounter();
    float r = l;
    for (int e = 0; e < 16; ++e) r += O[0][e] + O[1][e] + S[e];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
    if (threadIdx.x == 0) cycles[blockIdx.x] = t1 - t0;
}

template <int DEFERRED, int READS>
int run_block(int waves_per_simd, int iters, double* ns_per_block, double* cycles_per_block)
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 5;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 5;
    const int nblk = cus * waves_per_simd;
    float* out = nullptr;
    long long* cyc = nullptr;
    if (hipMalloc((void**)&out, sizeof(float) * nblk * 256) != hipSuccess) return 4;
    if (hipMalloc((void**)&cyc, sizeof(long long) * nblk) != hipSuccess) { (void)hipFree(out); return 4; }
    hipEvent_t e0, e1;
    int rc = 0;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) rc = 5;
    if (!rc) {
        hipLaunchKernelGGL((block_kernel<DEFERRED, READS>), dim3(nblk), dim3(256), 0, 0, out, cyc, 10, 0.01f);
        (void)hipEventRecord(e0, 0);
        hipLaunchKernelGGL((block_kernel<DEFERRED, READS>), dim3(nblk), dim3(256), 0, 0, out, cyc, iters, 0.01f);
        (void)hipEventRecord(e1, 0);
        if (hipDeviceSynchronize() != hipSuccess) rc = 5;
    }
    if (!rc) {
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        long long* hcyc = new long long[nblk];
        (void)hipMemcpy(hcyc, cyc, sizeof(long long) * nblk, hipMemcpyDeviceToHost);
        double avg = 0;
        for (int i = 0; i < nblk; ++i) avg += (double)hcyc[i];
        delete[] hcyc;
        // per SIMD: its wavefronts each do 2 * iters blocks in the measured time
        *ns_per_block = (double)ms * 1e6 / (2.0 * iters) / waves_per_simd;
        *cycles_per_block = avg / nblk / (2.0 * iters);   // of one wavefront
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipFree(out);
    (void)hipFree(cyc);
    return rc;
}

}  // namespace

// One block of the d_k = 64 walk as a wavefront issues it, nothing behind it: deferred 0 / 1 (see
// block_kernel), lds_reads 0 / 1, waves_per_simd 1..3.  Results: nanoseconds per block and SIMD,
// shader cycles per block of one wavefront.  Returns as attn_probe_run.
extern "C" int attn_probe_block(int deferred, int lds_reads, int waves_per_simd, int iters, double* ns_per_block,
                                double* cycles_per_block)
{
    if (deferred < 0 || deferred > 1 || lds_reads < 0 || lds_reads > 1 || waves_per_simd < 1 || waves_per_simd > 3 ||
        iters < 1 || !ns_per_block || !cycles_per_block)
        return 1;
    if (deferred)
        return lds_reads ? run_block<1, 1>(waves_per_simd, iters, ns_per_block, cycles_per_block)
                         : run_block<1, 0>(waves_per_simd, iters, ns_per_block, cycles_per_block);
    return lds_reads ? run_block<0, 1>(waves_per_simd, iters, ns_per_block, cycles_per_block)
                     : run_block<0, 0>(waves_per_simd, iters, ns_per_block, cycles_per_block);
}

// units: bit 0 MFMAs, bit 1 softmax vector work, bit 2 LDS fragment reads; density: 1 = 8 pairs per
// group (d_k = 128), 2 = 16 pairs (d_k = 64); waves_per_simd 1..3.  Results per 16-MFMA group and
// SIMD: nanoseconds (HIP events) and shader cycles (cycle counter inside the kernel).
// Returns 0, 1 for a bad argument, 4 / 5 for an allocation / device failure.
extern "C" int attn_probe_run(int units, int density, int waves_per_simd, int iters, int random_operands,
                              double* ns_per_group, double* cycles_per_group)
{
    if (units < 1 || units > 7 || (density != 1 && density != 2) || waves_per_simd < 1 || waves_per_simd > 3 || iters < 1 ||
        !ns_per_group || !cycles_per_group)
        return 1;
#define CASE(U_)                                                                                       \
    case U_:                                                                                           \
        return density == 1 ? run<U_, 1>(waves_per_simd, iters, random_operands, ns_per_group, cycles_per_group) \
                            : run<U_, 2>(waves_per_simd, iters, random_operands, ns_per_group, cycles_per_group);
    switch (units) {
        CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7)
    }
#undef CASE
    return 1;
}
