// Prefill kernel: Y[m, n] = sum_k X[m, k] * d[n, k/32] * (q[n, k] - 2^(bits-1))
//
// Exact products: code tiles are unpacked to the small integers (q - z) in the activations' 16-bit
// float type (|q - z| <= 8 is exact in bf16 and fp16) and staged in LDS next to the matching X
// columns; one 16x16x32 MFMA runs per (16 m, 16 n, block of 32 k); the fp16 block scale d[n, block]
// multiplies that block's partial sum in fp32 on the way into the accumulators.  The scale is never
// rounded into a 16-bit weight, so only fp32 summation rounds (rel-L2 ~1e-7).  The price is one fp32
// FMA per 32 MFMA multiply-adds: the vector ALU is busy for as long as the matrix pipe.
//
// Workgroup = 4 wavefronts, tile = 64 n (4 row tiles of the blob, one unit per wavefront and chunk)
// x MT m with MT = 64*A (A = 5: all 300 prefill rows in one workgroup, so every weight is unpacked
// once).  Wavefront w owns m-tiles [w*A, (w+1)*A) x all 64 n: A*4 accumulator tiles.  Its rows of X
// are private, so X goes global -> registers in MFMA layout (two 32-k steps ahead) and only the
// unpacked weights pass through LDS, double-buffered per 256-k chunk: one barrier per chunk.
// A batched launch runs a list of matrices in one grid (a lone 4096-row matrix fills 64 of 256 CUs).
#include <hip/hip_runtime.h>
#include "aq_layout.h"
#include "aq_kernels.h"
#include "aq_codec.h"

namespace {

using namespace aqdev;
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));

constexpr int GM_WAVES = 4;
constexpr int GM_THREADS = GM_WAVES * 64;
constexpr int GM_NT = 64;                          // n per workgroup
constexpr int W_ROW = AQ_CHUNK_K * 2 + 16;         // LDS row stride of the W chunk tile: 528 B

// words of one block -> 16 registers, each a pair of exact (q - z) in fp16 or bf16
template <int BITS, bool XBF>
__device__ __forceinline__ void unpack_exact(const uint32_t* w, const typename Codec<BITS>::Magic& magic,
                                             uint32_t (&o)[16])
{
    uint32_t a[16];
    Codec<BITS>::unpack(w, magic, a);              // fp16 pairs (magic + q)
    const float z = (float)(1 << (BITS - 1));
#pragma unroll
    for (int p = 0; p < 16; ++p) {
        const _Float16 k = (_Float16)(Codec<BITS>::offset(p) + z);
        const uint32_t ap = a[p];
        const half2v h = __builtin_bit_cast(half2v, ap) - half2v{k, k};      // exact: small integers
        if (XBF) {
            const float lo = (float)h.x, hi = (float)h.y;                    // bf16 = upper half of the fp32
            o[p] = (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xFFFF0000u);
        } else {
            o[p] = __builtin_bit_cast(uint32_t, h);
        }
    }
}

template <bool XBF>
__device__ __forceinline__ float4v mfma16(const u32x4& a, const u32x4& b, const float4v& c)
{
    if (XBF)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a), __builtin_bit_cast(bf8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

#define AQ_FIND_GEMM_TASK(t, wg)                                                  \
    AqGemmTask t;                                                                 \
    int wg = blockIdx.x;                                                          \
    if (count == 0) {                                                             \
        t = single;                                                               \
    } else {                                                                      \
        int lo = 0, hi = count - 1;                                               \
        while (lo < hi) {                                                         \
            int mid = (lo + hi + 1) >> 1;                                         \
            if (tasks[mid].wg_begin <= wg) lo = mid; else hi = mid - 1;           \
        }                                                                         \
        t = tasks[lo];                                                            \
        wg -= t.wg_begin;                                                         \
    }                                                                             \
    if (wg >= t.wg_count) return

// BITS_T == 0: the tasks' bit-widths differ, branch per workgroup
template <int BITS_T, bool XBF, int A>
__global__ __launch_bounds__(GM_THREADS) void qgemm_kernel(const AqGemmTask* __restrict__ tasks, int count,
                                                           AqGemmTask single)
{
    extern __shared__ __align__(16) uint8_t smem[];
    AQ_FIND_GEMM_TASK(t, wg);
    if (BITS_T == 2 || (BITS_T == 0 && t.bits == 2)) {
        constexpr int BITS = 2;
#include "aq_gemm_body.inc"
    } else if (BITS_T == 3 || (BITS_T == 0 && t.bits == 3)) {
        constexpr int BITS = 3;
#include "aq_gemm_body.inc"
    } else {
        constexpr int BITS = 4;
#include "aq_gemm_body.inc"
    }
}

template <int BITS_T, bool XBF>
void launch_a(int A, dim3 grid, size_t lds, hipStream_t s, const AqGemmTask* tasks, int count, const AqGemmTask& single)
{
    dim3 block(GM_THREADS);
    switch (A) {
        case 1: hipLaunchKernelGGL((qgemm_kernel<BITS_T, XBF, 1>), grid, block, lds, s, tasks, count, single); break;
        case 2: hipLaunchKernelGGL((qgemm_kernel<BITS_T, XBF, 2>), grid, block, lds, s, tasks, count, single); break;
        case 3: hipLaunchKernelGGL((qgemm_kernel<BITS_T, XBF, 3>), grid, block, lds, s, tasks, count, single); break;
        default: hipLaunchKernelGGL((qgemm_kernel<BITS_T, XBF, 5>), grid, block, lds, s, tasks, count, single); break;
    }
}

}  // namespace

// m-tiles (16 rows) per wavefront for M rows of activations: the workgroup covers 64*A rows
int aqk_gemm_mtiles(int64_t M)
{
    if (M <= 64) return 1;
    if (M <= 128) return 2;
    if (M <= 192) return 3;
    return 5;
}

int aqk_gemm_wg_count(int64_t N, int64_t M, int A, int* slabs)
{
    const int sl = (int)(aq_num_groups(N) * 2);
    if (slabs) *slabs = sl;
    return sl * (int)((M + 64 * A - 1) / (64 * A));
}

size_t aqk_gemm_workspace(int64_t, int64_t, int64_t, int) { return 0; }

// bits == 0: mixed bit-widths; x_dtype is common to all tasks of a launch
hipError_t aqk_gemm(const AqGemmTask* tasks_dev, int count, const AqGemmTask& single, int bits, int x_dtype, int A,
                    int total_wgs, hipStream_t s)
{
    const size_t lds = 2 * ((size_t)GM_NT * W_ROW + GM_NT * 8 * sizeof(float));     // two chunk buffers
    const dim3 grid((unsigned)total_wgs);
    const bool bf = (x_dtype == 2);
#define AQ_GO(B)                                                                     \
    do {                                                                             \
        if (bf) launch_a<B, true>(A, grid, lds, s, tasks_dev, count, single);        \
        else launch_a<B, false>(A, grid, lds, s, tasks_dev, count, single);          \
    } while (0)
    if (bits == 2) AQ_GO(2);
    else if (bits == 3) AQ_GO(3);
    else if (bits == 4) AQ_GO(4);
    else AQ_GO(0);
#undef AQ_GO
    return hipGetLastError();
}
