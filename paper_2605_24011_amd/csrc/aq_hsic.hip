// HSIC-based tensor sensitivity (Section 4.1, Eq. 5) from the empirical estimator of Eq. 2 (Section 3, "HSIC") with RBF kernels:
//     HSIC(A, B) = (K - 1)^-2 tr(K_A C K_B C),   [K_A]_ij = exp(-gamma_A ||a_i - a_j||^2),   C = I - (1/K) 1 1^T.
//
// The dense part is the Gram matrix A A^T of K samples x d features (2 K^2 d flop): fp32 on the matrix cores
// (V_MFMA_F32_32X32X2_F32), one 128 x 128 tile of the K x K result per workgroup, 4 wavefronts of 64 x 64 each,
// A staged through a double-buffered LDS 32 features at a time.  The kernel value follows in the epilogue from the squared norms:
// ||a_i - a_j||^2 = r_i + r_j - 2 a_i.a_j (clamped at 0).  The kernel is translation invariant, and that identity
// cancels badly when the samples share a large offset (r far above the distances): every sample is therefore taken
// relative to sample 0, a_i - a_0, in the squared norms and in the staging of the product alike (no extra pass, no
// extra memory).  Everything after that is O(K^2) streaming in fp64:
// with a_i, b_i the row sums of K_A, K_B,
//     tr(K_A C K_B C) = sum_ij [K_A]_ij [K_B]_ij - (2/K) sum_i a_i b_i + (1/K^2) (sum_i a_i)(sum_i b_i),
// (C K_A C written out), so the centering matrix is never formed and no K x K product is needed.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "aq_kernels.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int GT = 128;            // tile of the Gram matrix per workgroup
#ifndef AQ_GRAM_KC
#define AQ_GRAM_KC 32
#endif
#ifndef AQ_GRAM_WGS
#define AQ_GRAM_WGS 2
#endif
constexpr int KC = AQ_GRAM_KC;     // features per LDS stage: 32 = 128 bytes of a row, one cache line
constexpr int LPR = KC / 4;        // lanes that share a row's stage (one quad each)
constexpr int NH = GT * LPR / 256; // row groups a thread copies per block and stage
constexpr int LROW = KC + 1;       // LDS row stride in floats: 33 keeps the 32 rows of an operand read on 32 banks
constexpr int GSTAGE = 2 * GT * LROW;            // floats of one stage: the row block's rows, then the column block's
constexpr size_t GRAM_LDS = 2 * GSTAGE * sizeof(float);     // two stages

// Barrier for LDS traffic only: __syncthreads() would also wait for the global loads of the stage after next, which
// are meant to stay in flight across it.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// r[i] = sum_k (A[i][k] - A[0][k])^2, one wavefront per row
__global__ __launch_bounds__(256) void sqnorm_kernel(const float* __restrict__ A, int64_t K, int64_t d, int64_t lda,
                                                     float* __restrict__ r)
{
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= K) return;
    const int lane = threadIdx.x & 63;
    float s = 0.f;
    for (int64_t k = lane; k < d; k += 64) {
        const float v = A[row * lda + k] - A[k];
        s = fmaf(v, v, s);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) r[row] = s;
}

// G[i][j] = exp(-gamma * max(0, r_i + r_j - 2 a_i.a_j)) for the 128 x 128 tile (blockIdx.y, blockIdx.x).  The matrix
// is symmetric: only tiles on or above the diagonal are computed, and each writes its mirror image as well.
//
// Pipeline, one barrier per stage of 32 features: during stage s the registers that hold stage s + 1 (requested a
// whole stage earlier) go to the LDS buffer that stage s - 1 was read from, stage s + 2 is requested into a second
// set of registers, and stage s is multiplied out of the other buffer.  Eight lanes read the 128 contiguous bytes
// of a row's stage.
//
// SPLIT: the features are cut into gridDim.y slices of `per` stages; every workgroup adds its slice's raw dot products
// into G (zeroed beforehand, upper tiles only) with fp32 atomics, and gram_finish_kernel turns the sums into kernel
// values afterwards.  Used when the tile count fits the GPU's workgroup slots badly (528 tiles on 512 slots: the last
// 16 would run alone for as long as all the others together took).
template <bool SPLIT>
__global__ __launch_bounds__(256, AQ_GRAM_WGS) void gram_rbf_kernel(const float* __restrict__ A, int64_t K, int64_t d, int64_t lda,
                                                          const float* __restrict__ r, float gamma, float* __restrict__ G,
                                                          int per)
{
    extern __shared__ __align__(16) float gl[];              // [2 stages][i rows, j rows][GT][LROW]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = wave >> 1, wj = wave & 1;                 // this wavefront's 64 x 64 quadrant
    // blockIdx.x counts the tiles on or above the diagonal row by row: no workgroup is launched for the others
    const int tiles = (int)((K + GT - 1) / GT);
    int by = 0, bx = (int)blockIdx.x;
    while (bx >= tiles - by) { bx -= tiles - by; ++by; }
    bx += by;
    const int64_t i0 = (int64_t)by * GT, j0 = (int64_t)bx * GT;
    const bool mirror = bx != by;

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // staging: thread t copies features 4 * (t % 8) .. + 3 of rows t / 8 + 32 h (h = 0 .. 3) of both blocks: per stage
    // 8 quads = 16 pairs of floats, written to LDS one pair per group of four MFMAs so that the writes of stage s + 1
    // sit between the MFMAs of stage s (a lone wavefront on its SIMD has nobody else to cover them)
    const int srow = tid / LPR, sk = (tid % LPR) * 4;
    const bool vec = (lda & 3) == 0;                         // rows start 16-byte aligned: whole quads in one load
    f32x4 nxA[NH][2], nxB[NH][2];                            // [row group][i / j block], two stages in flight
    f32x4 rfA, rfB;                                          // sample 0's quad of the same stages: the common shift
    // No lane-dependent branches around the loads (a join after a divergent branch makes the compiler wait for every
    // load in flight): rows beyond K re-read row K - 1 (their results are never stored), and the choice between whole
    // quads and guarded single elements (last stage of a d that is not a multiple of 32, unaligned rows) is uniform.
    auto fetch = [&](f32x4 (&nx)[NH][2], f32x4& rf, int64_t k0) {
        const int64_t k = k0 + sk;
        const float* p[NH][2];
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                const int64_t row = (blk ? j0 : i0) + srow + (GT / NH) * h;
                p[h][blk] = A + (row < K ? row : K - 1) * lda;
            }
        if (vec && k0 + KC <= d) {
#pragma unroll
            for (int h = 0; h < NH; ++h)
#pragma unroll
                for (int blk = 0; blk < 2; ++blk) nx[h][blk] = *reinterpret_cast<const f32x4*>(p[h][blk] + k);
            rf = *reinterpret_cast<const f32x4*>(A + k);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float x = A[k + e < d ? k + e : 0];
                rf[e] = k + e < d ? x : 0.f;
            }
#pragma unroll
            for (int h = 0; h < NH; ++h)
#pragma unroll
                for (int blk = 0; blk < 2; ++blk) {
                    f32x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float x = p[h][blk][k + e < d ? k + e : 0];
                        v[e] = k + e < d ? x : 0.f;
                    }
                    nx[h][blk] = v;
                }
        }
    };
    auto stash_piece = [&](float* buf, const f32x4 (&nx)[NH][2], const f32x4& rf, int g) {    // g = 0 .. KC / 2 - 1 = 4 NH - 1
        const int h = g >> 2, blk = (g >> 1) & 1, e = 2 * (g & 1);
        float* dst = buf + (blk * GT + srow + (GT / NH) * h) * LROW + sk + e;
        dst[0] = nx[h][blk][e] - rf[e];
        dst[1] = nx[h][blk][e + 1] - rf[e + 1];
    };
    // operand layout of the 32x32x2 MFMA: lane l supplies A[row l % 32][k l / 32] and B[k l / 32][column l % 32]
    const int lr = lane & 31, lk = lane >> 5;
    const int64_t all_stages = (d + KC - 1) / KC;
    const int64_t first = SPLIT ? (int64_t)blockIdx.y * per : 0;           // this workgroup's stages: first .. first + stages - 1
    const int64_t stages = SPLIT ? (all_stages - first < per ? all_stages - first : per) : all_stages;
    if (stages <= 0) return;                                                // uniform
    // one stage: `cur` holds stage s + 1 (requested a stage ago) and goes to the other LDS buffer piece by piece,
    // `nxt` receives stage s + 2, stage s is multiplied out of its buffer
    auto stage = [&](int64_t s, const f32x4 (&cur)[NH][2], const f32x4& rcur, f32x4 (&nxt)[NH][2], f32x4& rnxt) {
        const float* buf = gl + (s & 1) * GSTAGE;
        float* other = gl + ((s + 1) & 1) * GSTAGE;          // read last during stage s - 1, before the barrier
        const bool more = s + 1 < stages;
        if (s + 2 < stages) fetch(nxt, rnxt, (first + s + 2) * KC);
        const float* ti = buf + (wi * 64 + lr) * LROW + lk;
        const float* tj = buf + (GT + wj * 64 + lr) * LROW + lk;
        // operands of feature pair kk + 2 are requested before the four MFMAs of pair kk
        float fa[2][2], fb[2][2];
#pragma unroll
        for (int a = 0; a < 2; ++a) { fa[0][a] = ti[a * 32 * LROW]; fb[0][a] = tj[a * 32 * LROW]; }
#pragma unroll
        for (int kk = 0; kk < KC; kk += 2) {
            const int cb = (kk >> 1) & 1;
            if (kk + 2 < KC) {
#pragma unroll
                for (int a = 0; a < 2; ++a) { fa[cb ^ 1][a] = ti[a * 32 * LROW + kk + 2]; fb[cb ^ 1][a] = tj[a * 32 * LROW + kk + 2]; }
            }
            if (more) stash_piece(other, cur, rcur, kk >> 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[cb][a], fb[cb][b], acc[a][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        lds_barrier();                                       // stage s read by everyone, stage s + 1 in place
    };
    fetch(nxB, rfB, first * KC);
#pragma unroll
    for (int g = 0; g < KC / 2; ++g) stash_piece(gl, nxB, rfB, g);
    if (stages > 1) fetch(nxA, rfA, (first + 1) * KC);
    lds_barrier();
    for (int64_t s = 0; s < stages; s += 2) {
        stage(s, nxA, rfA, nxB, rfB);
        if (s + 1 < stages) stage(s + 1, nxB, rfB, nxA, rfA);
    }

    // result layout: register v of lane l is row 8 * (v / 4) + 4 * (l / 32) + v % 4, column l % 32 of the 32 x 32 tile
    const int lc = lane & 31, lh = lane >> 5;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int64_t j = j0 + wj * 64 + b * 32 + lc;
            const float rj = j < K ? r[j] : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t i = i0 + wi * 64 + a * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                if (i < K && j < K) {
                    if (SPLIT) {
                        unsafeAtomicAdd(&G[i * K + j], acc[a][b][v]);
                    } else {
                        const float d2 = fmaxf(r[i] + rj - 2.f * acc[a][b][v], 0.f);
                        const float gv = i == j ? 1.f : __expf(-gamma * d2);
                        G[i * K + j] = gv;
                        if (mirror) G[j * K + i] = gv;
                    }
                }
            }
        }
}

// SPLIT path, before: zero the tiles on or above the diagonal.  After: G[i][j] holds a_i.a_j there; write the kernel
// value and its mirror image.  One workgroup per tile (the same linear tile index), rows of 128 contiguous floats.
template <bool FINISH>
__global__ __launch_bounds__(256) void gram_tile_pass_kernel(int64_t K, const float* __restrict__ r, float gamma,
                                                             float* __restrict__ G)
{
    const int tiles = (int)((K + GT - 1) / GT);
    int by = 0, bx = (int)blockIdx.x;
    while (bx >= tiles - by) { bx -= tiles - by; ++by; }
    bx += by;
    const int64_t i0 = (int64_t)by * GT, j0 = (int64_t)bx * GT;
    const int64_t j = j0 + (threadIdx.x & 127);
    if (j >= K) return;
    const float rj = FINISH ? r[j] : 0.f;
    for (int64_t i = i0 + (threadIdx.x >> 7); i < i0 + GT && i < K; i += 2) {
        if (!FINISH) { G[i * K + j] = 0.f; continue; }
        const float d2 = fmaxf(r[i] + rj - 2.f * G[i * K + j], 0.f);
        const float gv = i == j ? 1.f : __expf(-gamma * d2);
        G[i * K + j] = gv;
        if (bx != by) G[j * K + i] = gv;
    }
}

// rs[i] = sum_j G[i][j] in fp64, one wavefront per row
__global__ __launch_bounds__(256) void rowsum_kernel(const float* __restrict__ G, int64_t K, double* __restrict__ rs)
{
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= K) return;
    const int lane = threadIdx.x & 63;
    double s = 0.0;
    for (int64_t j = lane; j < K; j += 64) s += (double)G[row * K + j];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) rs[row] = s;
}

// acc[0] += sum_ij GA_ij GB_ij (this workgroup's share); workgroup 0 also adds acc[1] = sum a_i b_i, acc[2] = sum a_i,
// acc[3] = sum b_i.  acc is zeroed by the caller.
__global__ __launch_bounds__(256) void pair_kernel(const float* __restrict__ GA, const float* __restrict__ GB, int64_t K,
                                                   const double* __restrict__ ra, const double* __restrict__ rb,
                                                   double* __restrict__ acc)
{
    __shared__ double part[4][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n = K * K;
    double s = 0.0, sab = 0.0, sa = 0.0, sb = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * 256 + tid; e < n; e += (int64_t)gridDim.x * 256)
        s += (double)GA[e] * (double)GB[e];
    if (blockIdx.x == 0)
        for (int64_t i = tid; i < K; i += 256) {
            sab += ra[i] * rb[i];
            sa += ra[i];
            sb += rb[i];
        }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        s += __shfl_xor(s, o, 64);
        sab += __shfl_xor(sab, o, 64);
        sa += __shfl_xor(sa, o, 64);
        sb += __shfl_xor(sb, o, 64);
    }
    if (lane == 0) { part[wave][0] = s; part[wave][1] = sab; part[wave][2] = sa; part[wave][3] = sb; }
    __syncthreads();
    if (tid < 4) {
        const double t = part[0][tid] + part[1][tid] + part[2][tid] + part[3][tid];
        if (tid == 0 || blockIdx.x == 0) atomicAdd(acc + tid, t);
    }
}

__global__ void zero_kernel(double* p, int n)
{
    if ((int)threadIdx.x < n) p[threadIdx.x] = 0.0;
}

// out[0] = HSIC from acc; with two pairs: out[0] = HSIC(X, Z), out[1] = HSIC(Z, Y), out[2] = -alpha out[0] + beta out[1]
__global__ void finish_kernel(const double* acc, int pairs, int64_t K, double alpha, double beta, double* out)
{
    if (threadIdx.x != 0) return;
    const double k = (double)K, km1 = (double)(K - 1);
    double h[2] = {0.0, 0.0};
    for (int p = 0; p < pairs; ++p) {
        const double* a = acc + 4 * p;
        h[p] = (a[0] - 2.0 / k * a[1] + a[2] * a[3] / (k * k)) / (km1 * km1);
        out[p] = h[p];
    }
    if (pairs == 2) out[2] = -alpha * h[0] + beta * h[1];
}

}  // namespace

// G (K x K floats) = RBF Gram matrix of the K rows of A; sq = K floats of scratch (the squared norms)
hipError_t aqk_rbf_gram(const float* A, int64_t K, int64_t d, int64_t lda, float gamma, float* G, float* sq, hipStream_t s)
{
    hipLaunchKernelGGL(sqnorm_kernel, dim3((unsigned)((K + 3) / 4)), dim3(256), 0, s, A, K, d, lda, sq);
    const int64_t t = (K + GT - 1) / GT, ntiles = t * (t + 1) / 2, stages = (d + KC - 1) / KC;
    // slices of the feature range: the count (1, 2 or 4) that needs the fewest rounds of workgroups, a round being
    // AQ_GRAM_WGS workgroups on every compute unit; a slice keeps at least 16 stages
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return hipErrorInvalidDevice;
    const int64_t slots = (int64_t)cus * AQ_GRAM_WGS;
    int split = 1;
    double best = (double)((ntiles + slots - 1) / slots);
    for (int c = 2; c <= 4; c *= 2) {
        if (stages / c < 16) break;
        const double rounds = (double)((ntiles * c + slots - 1) / slots) / c * 1.03;      // + the two extra passes over G
        if (rounds < best * 0.9) { best = rounds; split = c; }
    }
    const dim3 grid((unsigned)ntiles, (unsigned)split);
    if (split == 1) {
        auto k = gram_rbf_kernel<false>;
        (void)aqk_allow_lds(reinterpret_cast<const void*>(k), GRAM_LDS);
        hipLaunchKernelGGL(k, grid, dim3(256), GRAM_LDS, s, A, K, d, lda, sq, gamma, G, 0);
    } else {
        auto k = gram_rbf_kernel<true>;
        (void)aqk_allow_lds(reinterpret_cast<const void*>(k), GRAM_LDS);
        hipLaunchKernelGGL(gram_tile_pass_kernel<false>, dim3((unsigned)ntiles), dim3(256), 0, s, K, sq, gamma, G);
        hipLaunchKernelGGL(k, grid, dim3(256), GRAM_LDS, s, A, K, d, lda, sq, gamma, G, (int)((stages + split - 1) / split));
        hipLaunchKernelGGL(gram_tile_pass_kernel<true>, dim3((unsigned)ntiles), dim3(256), 0, s, K, sq, gamma, G);
    }
    return hipGetLastError();
}

hipError_t aqk_rowsum(const float* G, int64_t K, double* rs, hipStream_t s)
{
    hipLaunchKernelGGL(rowsum_kernel, dim3((unsigned)((K + 3) / 4)), dim3(256), 0, s, G, K, rs);
    return hipGetLastError();
}

hipError_t aqk_zero_f64(double* p, int n, hipStream_t s)
{
    if (n < 1 || n > 64) return hipErrorInvalidValue;
    hipLaunchKernelGGL(zero_kernel, dim3(1), dim3(64), 0, s, p, n);
    return hipGetLastError();
}

// acc (4 doubles, zeroed) += the four sums of one pair of Gram matrices
hipError_t aqk_hsic_pair(const float* GA, const float* GB, int64_t K, const double* ra, const double* rb, double* acc,
                         hipStream_t s)
{
    int64_t blocks = (K * K + 256 * 8 - 1) / (256 * 8);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(pair_kernel, dim3((unsigned)blocks), dim3(256), 0, s, GA, GB, K, ra, rb, acc);
    return hipGetLastError();
}

hipError_t aqk_hsic_finish(const double* acc, int pairs, int64_t K, double alpha, double beta, double* out, hipStream_t s)
{
    if (pairs != 1 && pairs != 2) return hipErrorInvalidValue;
    hipLaunchKernelGGL(finish_kernel, dim3(1), dim3(64), 0, s, acc, pairs, K, alpha, beta, out);
    return hipGetLastError();
}
