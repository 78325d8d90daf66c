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

// X[M][ldx] (16-bit elements) -> Xt in operand order: Xt[m-tile][32-k step][lane (g, c)] = the 16 bytes
// X[16 m-tile + c][32 step + 8g .. + 8].  One wavefront writes whole 1 KiB fragments (contiguous, coalesced stores) and
// reads, per fragment, 64 bytes of each of the tile's 16 rows; its four fragments are four consecutive steps, so the
// 16 rows' reads cover whole 256-byte runs.  A workgroup = one m-tile x 16 steps.  Rows in [M, 16 ceil(M/16)) are
// written as zeros.
// Rows [16 mtile, 16 mtile + 16) of Y, columns of share `part` of `parts`, = 0: folded into the re-tiling launch of a
// lone product whose workgroups add their parts of K into Y.
struct AqZeroY {
    float* Y;           // null: nothing to clear
    int64_t M, N, ldy;
};
__device__ __forceinline__ void zero_y_share(const AqZeroY& z, int64_t mtile, int part, int parts)
{
    if (!z.Y) return;
    const int64_t per = (z.N + parts - 1) / parts, n0 = part * per, n1 = n0 + per < z.N ? n0 + per : z.N;
    for (int r = 0; r < 16; ++r) {
        const int64_t m = mtile * 16 + r;
        if (m >= z.M) break;
        for (int64_t n = n0 + threadIdx.x; n < n1; n += 256) z.Y[m * z.ldy + n] = 0.f;
    }
}

constexpr int RT_STEPS = 4;                                    // steps per wavefront
__global__ __launch_bounds__(256) void retile_kernel(const AqRetileTask* __restrict__ tasks, int count,
                                                     AqRetileTask single, uint8_t* __restrict__ workspace, AqZeroY zero)
{
    AqRetileTask t;
    if (count == 0) t = single; else t = tasks[blockIdx.y];
    if ((int)blockIdx.x >= t.blocks) return;
    const int ksteps = t.K >> 5;
    const int per_tile = (ksteps + 4 * RT_STEPS - 1) / (4 * RT_STEPS);       // workgroups per m-tile
    const int64_t mtile = blockIdx.x / per_tile;
    zero_y_share(zero, mtile, blockIdx.x % per_tile, per_tile);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
    const int step0 = ((blockIdx.x % per_tile) * 4 + wave) * RT_STEPS;
    const int64_t row = mtile * 16 + c;
    const int64_t mpad = (t.M + 15) & ~(int64_t)15;
    u32x4 v[RT_STEPS];
#pragma unroll
    for (int s = 0; s < RT_STEPS; ++s) {
        v[s] = u32x4{0u, 0u, 0u, 0u};
        if (row < t.M && step0 + s < ksteps) v[s] = *as_global<u32x4>(t.X + row * t.ldx + (int64_t)(step0 + s) * 32 + g * 8);
    }
    u32x4* dst = reinterpret_cast<u32x4*>(workspace + t.xt_offset) + (mtile * ksteps + step0) * 64 + lane;
#pragma unroll
    for (int s = 0; s < RT_STEPS; ++s)
        if (step0 + s < ksteps) dst[s * 64] = v[s];
    if (step0 == 0 && g == 0) reinterpret_cast<int32_t*>(workspace + t.xt_offset + mpad * t.K * 2)[row] = 0;       // rowexp
}

// bf16 X[M][ldx] -> binary16 Xt with one power-of-two factor per row.  A workgroup = one m-tile (16 rows) x one of
// gridDim.z slices of its steps (one slice in a list; a lone product cuts the steps into slices so that more than
// ceil(M / 16) compute units take part): pass 1 finds every row's largest magnitude (wavefront w takes rows 4w .. 4w+3,
// reading along the rows, the four rows' loads in flight together), pass 2 walks the slice's fragments as retile_kernel
// does (second read of the tile: from L2), scales, converts (round to nearest even) and stores whole fragments;
// rowexp[row] = the exponent the product kernel adds back.
__global__ __launch_bounds__(256) void retile_convert_kernel(const AqRetileTask* __restrict__ tasks, int count,
                                                             AqRetileTask single, uint8_t* __restrict__ workspace,
                                                             AqZeroY zero)
{
    __shared__ int row_shift[16];
    AqRetileTask t;
    if (count == 0) t = single; else t = tasks[blockIdx.y];
    const int64_t mtile = blockIdx.x;
    const int64_t mpad = (t.M + 15) & ~(int64_t)15;
    if (mtile * 16 >= mpad) return;                            // uniform per workgroup
    const int slice = blockIdx.z, slices = gridDim.z;
    zero_y_share(zero, mtile, slice, slices);
    const int pieces = t.K >> 3, ksteps = t.K >> 5;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4, c = lane & 15;
    int32_t* rowexp = reinterpret_cast<int32_t*>(workspace + t.xt_offset + mpad * t.K * 2);
    // pass 1: bf16 magnitudes order like unsigned integers
    {
        uint32_t mx[4] = {0u, 0u, 0u, 0u};
#pragma unroll 4
        for (int j = lane; j < pieces; j += 64) {
            u32x4 v[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t row = mtile * 16 + wave * 4 + r;
                v[r] = u32x4{0u, 0u, 0u, 0u};
                if (row < t.M) v[r] = as_global<u32x4>(t.X + row * t.ldx)[j];
            }
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t lo = v[r][i] & 0x7FFFu, hi = (v[r][i] >> 16) & 0x7FFFu;
                    mx[r] = lo > mx[r] ? lo : mx[r];
                    mx[r] = hi > mx[r] ? hi : mx[r];
                }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            uint32_t m = mx[r];
            for (int o = 32; o >= 1; o >>= 1) {
                const uint32_t other = (uint32_t)__shfl_xor((int)m, o);
                m = other > m ? other : m;
            }
            if (lane == 0) {
                int shift = 0;                                 // x * 2^shift has its largest magnitude in [2^14, 2^15)
                if (m != 0) {
                    const int field = (int)(m >> 7);           // biased exponent; 0 = bf16 subnormal, 255 = inf / NaN
                    shift = 14 - ((field ? field : 1) - 127);
                }
                row_shift[wave * 4 + r] = shift;
                if (slice == 0) rowexp[mtile * 16 + wave * 4 + r] = -shift;      // padded rows: 0
            }
        }
    }
    __syncthreads();
    // pass 2
    const int64_t row = mtile * 16 + c;
    const int shift = row_shift[c];
    u32x4* dst = reinterpret_cast<u32x4*>(workspace + t.xt_offset) + mtile * ksteps * 64 + lane;
    const int groups = (ksteps + 4 * RT_STEPS - 1) / (4 * RT_STEPS);          // runs of 16 steps (4 wavefronts x RT_STEPS)
    const int gper = (groups + slices - 1) / slices;
    const int gend = (slice + 1) * gper < groups ? (slice + 1) * gper : groups;
    for (int gi = slice * gper; gi < gend; ++gi) {
        const int step0 = (gi * 4 + wave) * RT_STEPS;
        u32x4 v[RT_STEPS];
#pragma unroll
        for (int s = 0; s < RT_STEPS; ++s) {
            v[s] = u32x4{0u, 0u, 0u, 0u};
            if (row < t.M && step0 + s < ksteps) v[s] = *as_global<u32x4>(t.X + row * t.ldx + (int64_t)(step0 + s) * 32 + g * 8);
        }
#pragma unroll
        for (int s = 0; s < RT_STEPS; ++s) {
            u32x4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float lo = ldexpf(__uint_as_float(v[s][i] << 16), shift);
                const float hi = ldexpf(__uint_as_float(v[s][i] & 0xFFFF0000u), shift);
                const half2v h = {(_Float16)lo, (_Float16)hi};
                o[i] = __builtin_bit_cast(uint32_t, h);
            }
            if (step0 + s < ksteps) dst[(int64_t)(step0 + s) * 64] = o;
        }
    }
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

// workgroups of a re-tiling task: one per m-tile (converting), one per m-tile and 16 steps of 32 k (plain)
int aqk_retile_blocks(int64_t M, int64_t K, int convert)
{
    const int64_t mtiles = (M + 15) / 16, ksteps = K / 32;
    return convert ? (int)mtiles : (int)(mtiles * ((ksteps + 15) / 16));
}

hipError_t aqk_retile(const AqRetileTask* tasks_dev, int count, const AqRetileTask& single, int max_blocks,
                      int convert, void* workspace, hipStream_t s, float* zero_Y, int64_t zero_N, int64_t zero_ldy)
{
    AqZeroY zero = {nullptr, 0, 0, 0};
    if (zero_Y && count == 0) zero = AqZeroY{zero_Y, single.M, zero_N, zero_ldy};
    if (convert) {
        // a lone product: the steps of an m-tile in slices of at least 16, up to 8 of them
        const int runs = count == 0 ? (int)((single.K / 32 + 4 * RT_STEPS - 1) / (4 * RT_STEPS)) : 1;
        const dim3 grid((unsigned)max_blocks, (unsigned)(count == 0 ? 1 : count), (unsigned)(runs < 8 ? runs : 8));
        hipLaunchKernelGGL(retile_convert_kernel, grid, dim3(256), 0, s, tasks_dev, count, single,
                           static_cast<uint8_t*>(workspace), zero);
    } else {
        const dim3 grid((unsigned)max_blocks, (unsigned)(count == 0 ? 1 : count));
        hipLaunchKernelGGL(retile_kernel, grid, dim3(256), 0, s, tasks_dev, count, single, static_cast<uint8_t*>(workspace),
                           zero);
    }
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
