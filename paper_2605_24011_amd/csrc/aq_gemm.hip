// Prefill kernel: Y[m, n] = sum_k X[m, k] * d[n, k/32] * (q[n, k] - 2^(bits-1))
//
// Exact products: code tiles are unpacked to the small integers (q - z) in the activations' 16-bit
// float type (|q - z| <= 8 is exact in bf16 and fp16) and staged in LDS next to the matching X
// columns; one 16x16x32 MFMA runs per (16 m, 16 n, block of 32 k); the fp16 block scale d[n, block]
// multiplies that block's partial sum in fp32 on the way into the accumulators.  The scale is never
// rounded into a 16-bit weight, so only fp32 summation rounds (rel-L2 ~1e-7).  The price is one fp32
// FMA per 32 MFMA multiply-adds: the vector ALU is busy for as long as the matrix pipe.
//
// Workgroup = 8 wavefronts, tile = 128 n (one row group of the blob: one unit per wavefront and chunk)
// x up to 384 m (A = 3 m-tiles per wavefront: all 300 prefill rows in one workgroup, so every weight
// is unpacked once).  The wavefronts split m only: each owns 2 or 3 m-tiles x all 128 n, 16 or 24
// accumulator tiles.  Its rows of X are private, so X goes global -> registers (two 32-k steps ahead)
// and only the unpacked weights pass through LDS, double-buffered per 256-k chunk: one barrier per
// chunk.  Splitting n across wavefronts instead would make several wavefronts request the same X;
// hits or not, the CU's L1 path delivers 64 bytes per clock and was the measured limit of that shape.
// A lane of an MFMA A operand holds 16 bytes of ONE row, and neighbouring lanes hold different rows:
// read from a row-major X that is 64 cache lines per load instruction.  So a small pre-pass re-tiles X
// once per product list into operand order (retile_kernel) and the main kernel's loads are 1 KiB
// contiguous.  A batched launch runs a list of matrices in one grid (a lone 4096-row matrix gives only
// 32 workgroups for 256 CUs).
#include "aq_gemm_kernel.h"

namespace {

// X[M][ldx] (16-bit elements) -> Xt in operand order.  Thread e handles the 16-byte piece j = e % (K/8)
// of row e / (K/8): reads run along the rows of X, rows in [M, 16*ceil(M/16)) are written as zeros.
__global__ __launch_bounds__(256) void retile_kernel(const AqRetileTask* __restrict__ tasks, int count,
                                                     AqRetileTask single, uint8_t* __restrict__ workspace)
{
    AqRetileTask t;
    if (count == 0) t = single; else t = tasks[blockIdx.y];
    if ((int)blockIdx.x >= t.blocks) return;
    const int pieces = t.K >> 3;                               // 16-byte pieces per row
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row = e / pieces;
    const int j = (int)(e - row * pieces);
    const int64_t mpad = (t.M + 15) & ~(int64_t)15;
    if (row >= mpad) return;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (row < t.M) v = *as_global<u32x4>(t.X + row * t.ldx + (int64_t)j * 8);
    const int64_t mtile = row >> 4;
    const int c = (int)(row & 15), step = j >> 2, g = j & 3;
    const int64_t ksteps = t.K >> 5;
    u32x4* dst = reinterpret_cast<u32x4*>(workspace + t.xt_offset);
    dst[(mtile * ksteps + step) * 64 + g * 16 + c] = v;
    if (j == 0) reinterpret_cast<int32_t*>(workspace + t.xt_offset + mpad * t.K * 2)[row] = 0;       // rowexp
}

// bf16 X[M][ldx] -> binary16 Xt with one power-of-two factor per row.  One workgroup per padded row:
// pass 1 finds the row's largest magnitude, pass 2 scales, converts (round to nearest even) and scatters
// the 16-byte pieces into operand order; rowexp[row] = the exponent the product kernel adds back.
__global__ __launch_bounds__(256) void retile_convert_kernel(const AqRetileTask* __restrict__ tasks, int count,
                                                             AqRetileTask single, uint8_t* __restrict__ workspace)
{
    __shared__ uint32_t wave_max[4];
    AqRetileTask t;
    if (count == 0) t = single; else t = tasks[blockIdx.y];
    const int64_t row = blockIdx.x;
    const int64_t mpad = (t.M + 15) & ~(int64_t)15;
    if (row >= mpad) return;                                   // uniform per workgroup
    const int pieces = t.K >> 3, tid = threadIdx.x;
    const int64_t ksteps = t.K >> 5;
    u32x4* dst = reinterpret_cast<u32x4*>(workspace + t.xt_offset);
    int32_t* rowexp = reinterpret_cast<int32_t*>(workspace + t.xt_offset + mpad * t.K * 2);
    const int64_t base = ((row >> 4) * ksteps) * 64 + (row & 15);
    if (row >= t.M) {
        for (int j = tid; j < pieces; j += 256) dst[base + (int64_t)(j >> 2) * 64 + (j & 3) * 16] = u32x4{0u, 0u, 0u, 0u};
        if (tid == 0) rowexp[row] = 0;
        return;
    }
    const AQ_GLOBAL u32x4* src = as_global<u32x4>(t.X + row * t.ldx);
    uint32_t mx = 0;                                           // bf16 magnitudes order like unsigned integers
    for (int j = tid; j < pieces; j += 256) {
        const u32x4 v = src[j];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t lo = v[i] & 0x7FFFu, hi = (v[i] >> 16) & 0x7FFFu;
            mx = lo > mx ? lo : mx;
            mx = hi > mx ? hi : mx;
        }
    }
    for (int o = 32; o >= 1; o >>= 1) {
        const uint32_t other = (uint32_t)__shfl_xor((int)mx, o);
        mx = other > mx ? other : mx;
    }
    if ((tid & 63) == 0) wave_max[tid >> 6] = mx;
    __syncthreads();
    mx = wave_max[0];
#pragma unroll
    for (int i = 1; i < 4; ++i) mx = wave_max[i] > mx ? wave_max[i] : mx;
    int shift = 0;                                             // x * 2^shift has its largest magnitude in [2^14, 2^15)
    if (mx != 0) {
        const int field = (int)(mx >> 7);                      // biased exponent; 0 = bf16 subnormal, 255 = inf / NaN
        shift = 14 - ((field ? field : 1) - 127);
    }
    for (int j = tid; j < pieces; j += 256) {
        const u32x4 v = src[j];
        u32x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float lo = ldexpf(__uint_as_float(v[i] << 16), shift);
            const float hi = ldexpf(__uint_as_float(v[i] & 0xFFFF0000u), shift);
            const half2v h = {(_Float16)lo, (_Float16)hi};
            o[i] = __builtin_bit_cast(uint32_t, h);
        }
        dst[base + (int64_t)(j >> 2) * 64 + (j & 3) * 16] = o;
    }
    if (tid == 0) rowexp[row] = -shift;
}

}  // namespace

// Shape of the wavefront grid for M rows of activations.  mtiles = most m-tiles (16 rows) per wavefront;
// nsplit = wavefronts side by side along n (the 8 wavefronts form an (8 / nsplit) x nsplit grid): when M has
// fewer m-tiles than wavefronts the spare ones take a share of the 128 n instead of idling.
int aqk_gemm_mtiles(int64_t M, int64_t groups)
{
    const int most = M <= 128 ? 1 : M <= 256 ? 2 : 3;       // all rows of X in one workgroup: weights unpacked once
    // A launch with few 128-row groups (a lone matrix) would leave most of the 256 CUs idle: split m over more
    // workgroups (each unpacks the weights again) while that adds workgroups the chip has room for.
    int best = most;
    int64_t best_wgs = groups * ((M + GM_WAVES * 16 * most - 1) / (GM_WAVES * 16 * most));
    for (int a = most - 1; a >= 1 && best_wgs < 192; --a) {
        const int64_t wgs = groups * ((M + GM_WAVES * 16 * a - 1) / (GM_WAVES * 16 * a));
        if (wgs > best_wgs && wgs <= 320) { best = a; best_wgs = wgs; }
    }
    return best;
}

int aqk_gemm_nsplit(int64_t M)
{
    if (M <= 16) return 8;
    if (M <= 32) return 4;
    if (M <= 64) return 2;
    return 1;
}

int aqk_gemm_wg_count(int64_t N, int64_t M, int A, int nsplit, int* slabs)
{
    const int sl = (int)aq_num_groups(N);
    if (slabs) *slabs = sl;
    const int64_t rows = (int64_t)(GM_WAVES / nsplit) * 16 * A;
    return sl * (int)((M + rows - 1) / rows);
}

// Xt (2 bytes per element, rows padded to 16) followed by rowexp (one int32 per padded row), rounded up to 1 KiB
size_t aqk_retile_bytes(int64_t M, int64_t K)
{
    const int64_t mpad = ((M + 15) / 16) * 16;
    return (size_t)(mpad * K * 2 + ((mpad * 4 + 1023) / 1024) * 1024);
}

int aqk_retile_blocks(int64_t M, int64_t K, int convert)
{
    const int64_t mpad = ((M + 15) / 16) * 16;
    return convert ? (int)mpad : (int)((mpad * (K / 8) + 255) / 256);
}

hipError_t aqk_retile(const AqRetileTask* tasks_dev, int count, const AqRetileTask& single, int max_blocks,
                      int convert, void* workspace, hipStream_t s)
{
    const dim3 grid((unsigned)max_blocks, (unsigned)(count == 0 ? 1 : count));
    if (convert)
        hipLaunchKernelGGL(retile_convert_kernel, grid, dim3(256), 0, s, tasks_dev, count, single,
                           static_cast<uint8_t*>(workspace));
    else
        hipLaunchKernelGGL(retile_kernel, grid, dim3(256), 0, s, tasks_dev, count, single, static_cast<uint8_t*>(workspace));
    return hipGetLastError();
}

// bits == 0: mixed bit-widths; x_dtype, the wavefront grid and the mode are common to all tasks of a launch
hipError_t aqk_gemm(const AqGemmTask* tasks_dev, int count, const AqGemmTask& single, int bits, int x_dtype, int A,
                    int nsplit, int fast, int total_wgs, const void* workspace, hipStream_t s)
{
    const size_t lds = gm_lds_bytes(0);
    const dim3 grid((unsigned)total_wgs);
    const bool bf = (x_dtype == 2) && !fast;         // the fp16-weight mode reads binary16 activations from Xt
    const uint8_t* ws = static_cast<const uint8_t*>(workspace);
#define AQ_GO(B)                                                                                     \
    do {                                                                                             \
        if (fast) launch_a<B, false, true, 0>(A, nsplit, grid, lds, s, tasks_dev, count, single, ws);   \
        else if (bf) launch_a<B, true, false, 0>(A, nsplit, grid, lds, s, tasks_dev, count, single, ws); \
        else launch_a<B, false, false, 0>(A, nsplit, grid, lds, s, tasks_dev, count, single, ws);       \
    } while (0)
    if (bits == 2) AQ_GO(2);
    else if (bits == 3) AQ_GO(3);
    else if (bits == 4) AQ_GO(4);
    else AQ_GO(0);
#undef AQ_GO
    return hipGetLastError();
}
