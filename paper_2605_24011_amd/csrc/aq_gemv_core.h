// Device pieces of the decode product shared by the kernels that run it (the batched matrix-vector kernels and
// the layer-by-layer decode step): the LDS layout of the staged x, the per-block correction terms, and the
// unit / chunk steps (unpack, 8 MFMAs against the block-diagonal B operand, scale the block sums).
#pragma once
#include <hip/hip_runtime.h>
#include "aq_layout.h"
#include <hip/hip_fp16.h>
#include "aq_kernels.h"
#include "aq_codec.h"

namespace aqdev {

// LDS layout of the staged x.  A block's 32 fp16 are 8 "quads" of 4 (8 bytes: the two B-operand
// registers of one MFMA).  Blocks are stored in pairs, quad by quad, with an 8-byte zero between:
//     entry m of pair p (24 bytes) = [quad m of block 2p][8 zero bytes][quad m of block 2p+1]
// so the 16 bytes at entry m are (x, x, 0, 0) -- the B registers of an even block's lane -- and the
// 16 bytes at entry m + 8 are (0, 0, x, x), those of an odd block's lane: one 16-byte LDS read
// (8-byte aligned) per MFMA, no ALU work to place the zeros.
constexpr int X_ENTRY_BYTES = 24;
constexpr int X_PAIR_BYTES = 8 * X_ENTRY_BYTES;     // 192
__device__ inline int x_lds_offset(int block, int quad)
{
    return (block >> 1) * X_PAIR_BYTES + quad * X_ENTRY_BYTES + (block & 1) * 16;
}

// corr[block] = sum_t (magic_t + z) (x[2t] + x[2t+1]) for the `nblocks` staged blocks: one 2-wide fp16 dot
// product (fp32 accumulate) per pair; the constants are small integers, exact in fp16.
template <int BITS, int THREADS_>
__device__ __forceinline__ void block_corrections(const uint8_t* xl, float* corr, int nblocks)
{
    const float z = (float)(1 << (BITS - 1));
    for (int b = threadIdx.x; b < nblocks; b += THREADS_) {
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const u32x2 v = *reinterpret_cast<const u32x2*>(xl + x_lds_offset(b, q));
            const uint32_t p0 = v.x, p1 = v.y;   // scalars first: bit_cast of a vector element misreads it
            const _Float16 k0 = (_Float16)(Codec<BITS>::offset(2 * q) + z);
            const _Float16 k1 = (_Float16)(Codec<BITS>::offset(2 * q + 1) + z);
            s = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, p0), half2v{k0, k0}, s, false);
            s = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, p1), half2v{k1, k1}, s, false);
        }
        corr[b] = s;
    }
}

__device__ inline float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Stage x into LDS as fp16 and compute corr[] per block.  bf16 input is multiplied by a power of
// two chosen from max|x| so that it lands in fp16's range (bf16 has 8 significant bits, fp16 11:
// the conversion is exact unless an element is > 2^28 times smaller than the largest); the
// returned factor undoes it at the end.
template <int BITS, int THREADS>
__device__ float stage_x(const AqGemvTask& t, uint8_t* xl, float* corr, float* scratch)
{
    const int tid = threadIdx.x;
    const int K = t.K, Kpad = t.nchunks * AQ_CHUNK_K;
    float unscale = 1.0f;
    for (int e = tid; e < t.nchunks * 4 * 8; e += THREADS)           // the zero middles of all entries
        *reinterpret_cast<u32x2*>(xl + e * X_ENTRY_BYTES + 8) = u32x2{0u, 0u};
    if (t.x_dtype == 1) {   // AQ_F16: copy
        for (int i = tid * 8; i < Kpad; i += THREADS * 8) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (i < K) v = *(as_global<u32x4>(t.x + i));
            *reinterpret_cast<u32x2*>(xl + x_lds_offset(i >> 5, (i & 31) >> 2)) = u32x2{v.x, v.y};
            *reinterpret_cast<u32x2*>(xl + x_lds_offset(i >> 5, ((i & 31) >> 2) + 1)) = u32x2{v.z, v.w};
        }
    } else {                // AQ_BF16
        float amax = 0.f;
        for (int i = tid * 8; i < K; i += THREADS * 8) {
            u32x4 v = *(as_global<u32x4>(t.x + i));
            uint32_t ws[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                amax = fmaxf(amax, fabsf(bf16_bits_to_f32(ws[j] & 0xFFFFu)));
                amax = fmaxf(amax, fabsf(bf16_bits_to_f32(ws[j] >> 16)));
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
        if ((tid & 63) == 0) scratch[tid >> 6] = amax;
        __syncthreads();
        amax = fmaxf(fmaxf(scratch[0], scratch[1]), fmaxf(scratch[2], scratch[3]));
        int e = 0;
        if (amax > 0.f && amax < 3.0e38f) {
            e = (int)((__float_as_uint(amax) >> 23) & 0xFF) - 127 - 14;   // amax * 2^-e in [2^14, 2^15)
            e = e < -100 ? -100 : e;
        }
        const float scale = __uint_as_float((uint32_t)(127 - e) << 23);   // 2^-e
        unscale = __uint_as_float((uint32_t)(127 + e) << 23);            // 2^e
        for (int i = tid * 8; i < Kpad; i += THREADS * 8) {
            u32x4 o = {0u, 0u, 0u, 0u};
            if (i < K) {
                u32x4 v = *(as_global<u32x4>(t.x + i));
                uint32_t ws[4] = {v.x, v.y, v.z, v.w}, os[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    __half lo = __float2half_rn(bf16_bits_to_f32(ws[j] & 0xFFFFu) * scale);
                    __half hi = __float2half_rn(bf16_bits_to_f32(ws[j] >> 16) * scale);
                    os[j] = (uint32_t)__half_as_ushort(lo) | ((uint32_t)__half_as_ushort(hi) << 16);
                }
                o.x = os[0]; o.y = os[1]; o.z = os[2]; o.w = os[3];
            }
            *reinterpret_cast<u32x2*>(xl + x_lds_offset(i >> 5, (i & 31) >> 2)) = u32x2{o.x, o.y};
            *reinterpret_cast<u32x2*>(xl + x_lds_offset(i >> 5, ((i & 31) >> 2) + 1)) = u32x2{o.z, o.w};
        }
    }
    __syncthreads();
    block_corrections<BITS, THREADS>(xl, corr, t.nchunks * AQ_CHUNK_BLOCKS);
    __syncthreads();
    return unscale;
}

// One unit (16 rows x 8 blocks): unpack the ring slot, optionally refill it from `next`, run the
// 8 MFMAs against the block-diagonal B and fold the block sums, times their fp16 scales, into the
// tile's running sums (registers; lane (g, c) holds rows 4g .. 4g+3 of block column c).
// RS = words per ring row: Codec<BITS>::WORDS for a ring of one bit-width, 8 for a ring that serves all three.
template <int BITS, bool REFILL, int RS>
__device__ __forceinline__ void unit_step(uint32_t (&raw)[RS], u32x2& sc,
                                          typename Codec<BITS>::Magic& magic, const half8 (&B)[8],
                                          const float4v& negc, const uint8_t* next, int lane, int sc_off,
                                          float (&acc)[4])
{
    // Order the units: this unit's unpack may not start before the tile's previous unit (two units
    // back) has been folded into acc.  Without it the compiler hoists the unpack of every unit in
    // flight to the top of the loop body and holds all of their operands live at once (2-3x the
    // registers).  The empty asm ties the magic constants (inputs of every unpack instruction) to acc.
    Codec<BITS>::fence(magic, acc[0]);
    uint32_t a0[16], a1[16];
    Codec<BITS>::unpack(&raw[0], magic, a0);
    Codec<BITS>::unpack(&raw[BITS], magic, a1);
    const half4v d4 = __builtin_bit_cast(half4v, sc);           // scales of rows 4g .. 4g+3
    if (REFILL) {
        Codec<BITS>::load(next, lane, *reinterpret_cast<uint32_t(*)[Codec<BITS>::WORDS]>(&raw));
        sc = __builtin_nontemporal_load(as_global<u32x2>(next + sc_off));
    }
    float4v D = negc;
#pragma unroll
    for (int m = 0; m < 8; ++m) {
        u32x4 av = {a0[2 * m], a0[2 * m + 1], a1[2 * m], a1[2 * m + 1]};
        D = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, av), B[m], D, 0, 0, 0);
    }
    acc[0] = fmaf(D[0], (float)d4.x, acc[0]);
    acc[1] = fmaf(D[1], (float)d4.y, acc[1]);
    acc[2] = fmaf(D[2], (float)d4.z, acc[2]);
    acc[3] = fmaf(D[3], (float)d4.w, acc[3]);
}

// One chunk for the wavefront's TW tiles: fetch the chunk's B operand from LDS, then one unit per
// tile out of ring slots slot0 .. slot0+TW-1, each refilled from the chunk two ahead.
template <int BITS, int TW, bool REFILL, int RS>
__device__ __forceinline__ void chunk_step(uint32_t (*raw)[RS], u32x2* sc,
                                           typename Codec<BITS>::Magic& magic, const uint8_t* xl,
                                           const float* corr, const uint8_t* zeros, int ch, bool diag,
                                           int c, const uint8_t* refill, int lane, int sc_off, float (*acc)[4])
{
    constexpr int UNIT = 512 * BITS + 256;
    // B: x of block c goes to the k-slots of block c (the low two registers for even c, the high two
    // for odd c) and zeros elsewhere: one 16-byte LDS read per MFMA (see x_lds_offset).
    // Re-read per chunk: that costs LDS reads only, no ALU work, and B never lives across the loop.
    typedef u32x4 u32x4_a8 __attribute__((aligned(8)));
    const uint8_t* bp = diag ? xl + (ch * 4 + (c >> 1)) * X_PAIR_BYTES + (c & 1) * 8 : zeros;
    half8 B[8];
#pragma unroll
    for (int m = 0; m < 8; ++m)
        B[m] = __builtin_bit_cast(half8, *reinterpret_cast<const u32x4_a8*>(bp + m * X_ENTRY_BYTES));
    const float nc = -corr[ch * AQ_CHUNK_BLOCKS + (c & 7)];
    const float4v negc = {nc, nc, nc, nc};
#pragma unroll
    for (int tw = 0; tw < TW; ++tw)
        unit_step<BITS, REFILL>(raw[tw], sc[tw], magic, B, negc, refill + tw * UNIT, lane, sc_off, acc[tw]);
}

}  // namespace aqdev
