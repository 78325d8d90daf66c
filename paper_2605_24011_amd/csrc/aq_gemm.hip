// Prefill kernel: Y[m, n] = sum_k X[m, k] * d[n, k/32] * (q[n, k] - 2^(bits-1))
//
// Per 256-k chunk a workgroup unpacks its weight units to exact small integers (q - z) in the
// activations' 16-bit float type (|q - z| <= 8 is exact in bf16 and fp16), stages them and the
// matching X columns in LDS, and runs one 16x16x32 MFMA per (16 m, 16 n, block of 32 k).  The
// fp16 block scale d[n, block] multiplies that block's partial sum in fp32 on the way into the
// accumulators, so every product is exact (the scale is never rounded into a 16-bit weight) and
// only fp32 summation rounds.
//
// Tile: 64 n (4 row tiles of the blob, one per wavefront) x MT m (MT = 80: 4 tiles cover M = 300
// with 256 workgroups on a 4096-row matrix); each wavefront keeps MT/16 accumulators.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "aq_layout.h"
#include "aq_kernels.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int NT = 64;                 // n per workgroup
constexpr int MT = 80;                 // m per workgroup
constexpr int MTILES = MT / 16;
constexpr int ROW_BYTES = AQ_CHUNK_K * 2 + 16;   // LDS row stride (256 k of 16-bit + pad)
constexpr int THREADS = 256;

// element e (0..31) of a block from its words, as an integer code
template <int BITS>
__device__ inline int code_of(const uint32_t* w, int e) { return (int)aq_block_get(w, BITS, e); }

// (q - z) for two codes as a packed pair of 16-bit floats of type XBF ? bf16 : fp16
template <bool XBF>
__device__ inline uint32_t pack_pair(int v0, int v1)
{
    if (XBF) {
        uint32_t f0 = __float_as_uint((float)v0), f1 = __float_as_uint((float)v1);   // exact, low 16 bits zero
        return (f0 >> 16) | (f1 & 0xFFFF0000u);
    } else {
        __half h0 = __int2half_rn(v0), h1 = __int2half_rn(v1);
        return (uint32_t)__half_as_ushort(h0) | ((uint32_t)__half_as_ushort(h1) << 16);
    }
}

template <int BITS> struct Words { static constexpr int N = 2 * BITS; };

template <int BITS>
__device__ inline void load_words(const uint8_t* unit, int lane, uint32_t* w)
{
#pragma unroll
    for (int wi = 0; wi < 2 * BITS; ++wi)
        w[wi] = *reinterpret_cast<const uint32_t*>(unit + aq_word_offset(BITS, lane, wi));
}

template <bool XBF>
__device__ inline float4v mfma16(const u32x4& a, const u32x4& b, const float4v& c)
{
    if (XBF)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a), __builtin_bit_cast(bf8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

template <int BITS, bool XBF>
__global__ __launch_bounds__(THREADS) void qgemm_kernel(const uint8_t* __restrict__ blob, int64_t N, int K,
                                                        const uint16_t* __restrict__ X, int64_t M, int64_t ldx,
                                                        float* __restrict__ Y, int64_t ldy)
{
    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t* Wl = smem;                                   // NT rows x ROW_BYTES
    uint8_t* Xl = smem + NT * ROW_BYTES;                  // MT rows x ROW_BYTES
    float* Sl = reinterpret_cast<float*>(smem + (NT + MT) * ROW_BYTES);   // NT x 8 scales

    constexpr int UNIT = 512 * BITS + 256;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, c = lane & 15;
    const int nch = (int)aq_num_chunks(K);
    const int64_t ntile4 = blockIdx.x;                    // which 64-row slab
    const int64_t group = ntile4 >> 1;
    const int til = (int)(ntile4 & 1) * 4 + wave;         // this wavefront's tile inside the group
    const int64_t m0 = (int64_t)blockIdx.y * MT;
    const int z = 1 << (BITS - 1);

    float4v acc[MTILES];
#pragma unroll
    for (int mt = 0; mt < MTILES; ++mt) acc[mt] = float4v{0.f, 0.f, 0.f, 0.f};

    for (int ch = 0; ch < nch; ++ch) {
        // ---- weights: unit -> integers -> LDS row (wave*16 + c), blocks 2g, 2g+1 ----
        const uint8_t* unit = blob + aq_unit_index(group, ch, til, nch) * UNIT;
        uint32_t w[2 * BITS];
        load_words<BITS>(unit, lane, w);
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            uint32_t out[16];
#pragma unroll
            for (int t = 0; t < 16; ++t)
                out[t] = pack_pair<XBF>(code_of<BITS>(w + blk * BITS, 2 * t) - z,
                                        code_of<BITS>(w + blk * BITS, 2 * t + 1) - z);
            uint8_t* dst = Wl + (wave * 16 + c) * ROW_BYTES + (2 * g + blk) * 64;
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                *reinterpret_cast<u32x4*>(dst + 16 * q4) =
                    u32x4{out[4 * q4], out[4 * q4 + 1], out[4 * q4 + 2], out[4 * q4 + 3]};
        }
        if (c < 8) {
            u32x2 sv = *reinterpret_cast<const u32x2*>(unit + 512 * BITS + (g * 8 + c) * 8);
            const half4v d4 = __builtin_bit_cast(half4v, sv);      // scales of rows 4g .. 4g+3, block c
            Sl[(wave * 16 + 4 * g + 0) * 8 + c] = (float)d4.x;
            Sl[(wave * 16 + 4 * g + 1) * 8 + c] = (float)d4.y;
            Sl[(wave * 16 + 4 * g + 2) * 8 + c] = (float)d4.z;
            Sl[(wave * 16 + 4 * g + 3) * 8 + c] = (float)d4.w;
        }
        // ---- activations: rows m0..m0+MT, columns ch*256..+256 (zero outside M x K) ----
        for (int v = tid; v < MT * 32; v += THREADS) {
            int mr = v >> 5, kv = (v & 31) * 8;
            int64_t m = m0 + mr;
            int k = ch * AQ_CHUNK_K + kv;
            u32x4 val = {0u, 0u, 0u, 0u};
            if (m < M && k < K) val = *reinterpret_cast<const u32x4*>(X + m * ldx + k);
            *reinterpret_cast<u32x4*>(Xl + mr * ROW_BYTES + kv * 2) = val;
        }
        __syncthreads();
        // ---- MFMA: A = X (16 m x 32 k), B = W (32 k x 16 n), per block ----
#pragma unroll
        for (int b = 0; b < AQ_CHUNK_BLOCKS; ++b) {
            const u32x4 bw = *reinterpret_cast<const u32x4*>(Wl + (wave * 16 + c) * ROW_BYTES + b * 64 + g * 16);
            const float s = Sl[(wave * 16 + c) * 8 + b];
#pragma unroll
            for (int mt = 0; mt < MTILES; ++mt) {
                const u32x4 ax = *reinterpret_cast<const u32x4*>(Xl + (mt * 16 + c) * ROW_BYTES + b * 64 + g * 16);
                float4v d = mfma16<XBF>(ax, bw, float4v{0.f, 0.f, 0.f, 0.f});
                acc[mt][0] = fmaf(d[0], s, acc[mt][0]);
                acc[mt][1] = fmaf(d[1], s, acc[mt][1]);
                acc[mt][2] = fmaf(d[2], s, acc[mt][2]);
                acc[mt][3] = fmaf(d[3], s, acc[mt][3]);
            }
        }
        __syncthreads();
    }
    // D layout: lane (g, c) holds rows m = 4g + r, column n = c
    const int64_t n = ntile4 * NT + wave * 16 + c;
#pragma unroll
    for (int mt = 0; mt < MTILES; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int64_t m = m0 + mt * 16 + 4 * g + r;
            if (m < M && n < N) Y[m * ldy + n] = acc[mt][r];
        }
}

}  // namespace

size_t aqk_gemm_workspace(int64_t, int64_t, int64_t, int) { return 0; }

hipError_t aqk_gemm(const void* blob, int64_t N, int64_t K, int bits, const void* X, int64_t M, int64_t ldx,
                    int x_dtype, float* Y, int64_t ldy, void*, hipStream_t s)
{
    dim3 grid((unsigned)(aq_num_groups(N) * 2), (unsigned)((M + MT - 1) / MT)), block(THREADS);
    size_t lds = (size_t)(NT + MT) * ROW_BYTES + NT * 8 * sizeof(float);
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    const uint16_t* x = static_cast<const uint16_t*>(X);
    const bool bf = (x_dtype == 2);
    // more than 64 KB of dynamic LDS needs an explicit opt-in, once per kernel
#define AQ_LAUNCH(BITS, BF)                                                                              \
    do {                                                                                                 \
        static bool ready = false;                                                                       \
        if (!ready) {                                                                                    \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&qgemm_kernel<BITS, BF>),   \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);    \
            if (e != hipSuccess) return e;                                                               \
            ready = true;                                                                                \
        }                                                                                                \
        hipLaunchKernelGGL((qgemm_kernel<BITS, BF>), grid, block, lds, s, b, N, (int)K, x, M, ldx, Y, ldy); \
    } while (0)
    if (bits == 2) { if (bf) AQ_LAUNCH(2, true); else AQ_LAUNCH(2, false); }
    else if (bits == 3) { if (bf) AQ_LAUNCH(3, true); else AQ_LAUNCH(3, false); }
    else { if (bf) AQ_LAUNCH(4, true); else AQ_LAUNCH(4, false); }
#undef AQ_LAUNCH
    return hipGetLastError();
}
