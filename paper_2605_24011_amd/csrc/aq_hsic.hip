// HSIC-based tensor sensitivity (Section 4.1, Eq. 5) from the empirical estimator of Eq. 4 with RBF kernels:
//     HSIC(A, B) = (K - 1)^-2 tr(K_A C K_B C),   [K_A]_ij = exp(-gamma_A ||a_i - a_j||^2),   C = I - (1/K) 1 1^T.
//
// The dense part is the Gram matrix A A^T of K samples x d features (2 K^2 d flop): fp32 on the matrix cores
// (V_MFMA_F32_32X32X2_F32), one 128 x 128 tile of the K x K result per workgroup, 4 wavefronts of 64 x 64 each,
// A staged through a double-buffered LDS 32 features at a time.  The kernel value follows in the epilogue from the squared norms:
// ||a_i - a_j||^2 = r_i + r_j - 2 a_i.a_j (clamped at 0).  Everything after that is O(K^2) streaming in fp64:
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
constexpr int KC = 32;             // features per LDS stage: 128 bytes of a row, one cache line
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

// r[i] = sum_k A[i][k]^2, one wavefront per row
__global__ __launch_bounds__(256) void sqnorm_kernel(const float* __restrict__ A, int64_t K, int64_t d, int64_t lda,
                                                     float* __restrict__ r)
{
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= K) return;
    const int lane = threadIdx.x & 63;
    float s = 0.f;
    for (int64_t k = lane; k < d; k += 64) {
        const float v = A[row * lda + k];
        s = fmaf(v, v, s);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) r[row] = s;
}

// G[i][j] = exp(-gamma * max(0, r_i + r_j - 2 a_i.a_j)) for the 128 x 128 tile (blockIdx.y, blockIdx.x).  The matrix
// is symmetric: only tiles on or above the diagonal are computed, and each writes its mirror image as well.
//
// Pipeline, one barrier per stage of 32 features: at the top of stage s the registers hold stage s + 1 (requested a
// whole stage earlier); they go to the LDS buffer that stage s - 1 was read from, stage s + 2 is requested, then
// stage s is multiplied out of the other buffer.  Eight lanes read the 128 contiguous bytes of a row's stage.
__global__ __launch_bounds__(256, 2) void gram_rbf_kernel(const float* __restrict__ A, int64_t K, int64_t d, int64_t lda,
                                                          const float* __restrict__ r, float gamma, float* __restrict__ G)
{
    extern __shared__ __align__(16) float gl[];              // [2 stages][i rows, j rows][GT][LROW]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wi = wave >> 1, wj = wave & 1;                 // this wavefront's 64 x 64 quadrant
    if (blockIdx.x < blockIdx.y) return;                     // below the diagonal: the mirror tile writes it
    const int64_t i0 = (int64_t)blockIdx.y * GT, j0 = (int64_t)blockIdx.x * GT;
    const bool mirror = blockIdx.x != blockIdx.y;

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // staging: thread t copies features 4 * (t % 8) .. + 3 of rows t / 8 + 32 h (h = 0 .. 3) of both blocks
    const int srow = tid >> 3, sk = (tid & 7) * 4;
    const bool vec = (lda & 3) == 0;                         // rows start 16-byte aligned: whole quads in one load
    f32x4 nx[4][2];                                          // [row group][i / j block]
    auto fetch = [&](int64_t k0) {
        const int64_t k = k0 + sk;
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            const int rr = srow + 32 * h;
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                const int64_t row = (blk ? j0 : i0) + rr;
                if (row < K && vec && k + 3 < d) {
                    nx[h][blk] = *reinterpret_cast<const f32x4*>(A + row * lda + k);
                } else {
                    f32x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (row < K && k + e < d) ? A[row * lda + k + e] : 0.f;
                    nx[h][blk] = v;
                }
            }
        }
    };
    auto stash = [&](float* buf) {
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            const int rr = srow + 32 * h;
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
#pragma unroll
                for (int e = 0; e < 4; ++e) buf[(blk * GT + rr) * LROW + sk + e] = nx[h][blk][e];
        }
    };
    // operand layout of the 32x32x2 MFMA: lane l supplies A[row l % 32][k l / 32] and B[k l / 32][column l % 32]
    const int lr = lane & 31, lk = lane >> 5;
    const int64_t stages = (d + KC - 1) / KC;
    fetch(0);
    stash(gl);
    if (stages > 1) fetch(KC);
    lds_barrier();
    for (int64_t s = 0; s < stages; ++s) {
        const float* cur = gl + (s & 1) * GSTAGE;
        if (s + 1 < stages) {
            stash(gl + ((s + 1) & 1) * GSTAGE);              // read last during stage s - 1, before the barrier
            if (s + 2 < stages) fetch((s + 2) * KC);
        }
        const float* ti = cur + (wi * 64 + lr) * LROW + lk;
        const float* tj = cur + (GT + wj * 64 + lr) * LROW + lk;
#pragma unroll
        for (int kk = 0; kk < KC; kk += 2) {
            float fa[2], fb[2];
#pragma unroll
            for (int a = 0; a < 2; ++a) fa[a] = ti[a * 32 * LROW + kk];
#pragma unroll
            for (int b = 0; b < 2; ++b) fb[b] = tj[b * 32 * LROW + kk];
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a], fb[b], acc[a][b], 0, 0, 0);
        }
        lds_barrier();                                       // stage s read by everyone, stage s + 1 in place
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
                    const float d2 = fmaxf(r[i] + rj - 2.f * acc[a][b][v], 0.f);
                    const float gv = i == j ? 1.f : __expf(-gamma * d2);
                    G[i * K + j] = gv;
                    if (mirror) G[j * K + i] = gv;
                }
            }
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
    const unsigned tiles = (unsigned)((K + GT - 1) / GT);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gram_rbf_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)GRAM_LDS);
    hipLaunchKernelGGL(gram_rbf_kernel, dim3(tiles, tiles), dim3(256), GRAM_LDS, s, A, K, d, lda, sq, gamma, G);
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
