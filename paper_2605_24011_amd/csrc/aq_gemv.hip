// Decode kernel: y[n] = sum_k x[k] * d[n, k/32] * (q[n, k] - 2^(bits-1))   (Eq. 1 fused into the product)
//
// HBM-bound by design: each weight is read once (bits/8 + 1/16 bytes) and costs well under one
// vector-ALU instruction, so the load stream, not the ALUs, sets the pace:
//
//  * unpack: one AND-OR per TWO codes.  A 32-bit word of the blob carries the even element of a
//    pair in its low half and the odd element in its high half at the same bit position, so
//    (word & mask) | magic is a pair of fp16 numbers (2^e + q).  A few shifts per word bring all
//    positions under masks that sit inside the fp16 mantissa.
//  * multiply-accumulate: on the matrix cores.  One V_MFMA_F32_16X16X32_F16 takes 16 rows x 32
//    k-slots of weights as A.  Its 32 k-slots are spread over the 8 blocks of a chunk (4 slots
//    per block), and B holds x on a block diagonal: column c of B is x restricted to the slots of
//    block c.  After 8 MFMAs D[row][c] is the complete 32-element sum of block c for that row,
//    one useful number per lane and register, with no cross-lane reduction.
//  * the -2^(bits-1) offset and the magic constants are linear in x: their contribution
//    corr[block] = sum_t (magic_t + z) (x[2t] + x[2t+1]) depends on x only, is computed once per
//    workgroup while x is staged in LDS, and enters as the C operand of the first MFMA.
//  * the fp16 block scale multiplies the finished block sum in fp32 (one mixed-precision FMA per
//    block and row), so every product is exact and only fp32 summation rounds.
//
// Work split: a workgroup of 4 wavefronts owns RT tiles (16 rows each) of one 128-row group and
// the whole K extent; wavefront w takes chunks w, w+4, ...; partial sums meet in LDS at the end.
// A batched launch runs many matrices (each with its own bit-width) in one grid.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <cstdlib>
#include "aq_layout.h"
#include "aq_kernels.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 half4v __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));

constexpr int WAVES = 4;
constexpr int THREADS = WAVES * 64;

// pointers read from a task record are generic; the streams they point to are global memory
#define AQ_GLOBAL __attribute__((address_space(1)))
template <class T> __device__ inline const AQ_GLOBAL T* as_global(const void* p)
{
    return (const AQ_GLOBAL T*)(uintptr_t)p;
}

// (a & mask) | magic must be ONE VALU instruction (V_AND_OR_B32).  gfx950's VOP3 encoding takes no
// literal and a single scalar operand, so with two compile-time constants the compiler falls back
// to an AND and an OR with literals.  `opaque_vgpr` hides the magic's value behind an empty asm
// statement (no instruction is emitted) which pins it in a VGPR; the mask then rides in an SGPR.
// The AND-OR itself stays ordinary C so that the compiler's hazard handling sees a real
// instruction next to the MFMAs.
__device__ inline uint32_t opaque_vgpr(uint32_t v)
{
    asm volatile("" : "+v"(v));
    return v;
}
__device__ inline uint32_t and_or(uint32_t a, uint32_t mask, uint32_t magic) { return (a & mask) | magic; }

// ---- per-bit-width codec: raw words of a lane, magic offsets, unpack to fp16 pairs ----
template <int BITS> struct Codec;

template <> struct Codec<2> {
    static constexpr int WORDS = 4;            // per lane and unit (2 blocks x 2 words)
    __device__ static float offset(int t) {    // magic of pair t, per half-bit position
        const float o[8] = {64.f, 16.f, 64.f, 16.f, 4.f, 64.f, 16.f, 4.f};
        return o[t & 7];
    }
    __device__ static void load(const uint8_t* unit, int lane, uint32_t (&w)[WORDS]) {
        u32x4 v = __builtin_nontemporal_load(as_global<u32x4>(unit) + lane);
        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    }
    // words of one block -> 16 pair registers (fp16x2 = magic + code)
    struct Magic { uint32_t m64, m16, m4; };
    __device__ static Magic magic() {
        return {opaque_vgpr(0x54005400u), opaque_vgpr(0x4C004C00u), opaque_vgpr(0x44004400u)};
    }
    __device__ static void unpack(const uint32_t* w, const Magic& k, uint32_t (&a)[16]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t u0 = w[h], u1 = u0 >> 6, u2 = u0 << 4;
            a[8 * h + 0] = and_or(u2, 0x00300030u, k.m64);
            a[8 * h + 1] = and_or(u2, 0x00C000C0u, k.m16);
            a[8 * h + 2] = and_or(u0, 0x00300030u, k.m64);
            a[8 * h + 3] = and_or(u0, 0x00C000C0u, k.m16);
            a[8 * h + 4] = and_or(u0, 0x03000300u, k.m4);
            a[8 * h + 5] = and_or(u1, 0x00300030u, k.m64);
            a[8 * h + 6] = and_or(u1, 0x00C000C0u, k.m16);
            a[8 * h + 7] = and_or(u1, 0x03000300u, k.m4);
        }
    }
};

template <> struct Codec<4> {
    static constexpr int WORDS = 8;
    __device__ static float offset(int t) { return (t & 1) ? 16.f : 256.f; }
    __device__ static void load(const uint8_t* unit, int lane, uint32_t (&w)[WORDS]) {
        u32x4 v0 = __builtin_nontemporal_load(as_global<u32x4>(unit) + lane);
        u32x4 v1 = __builtin_nontemporal_load(as_global<u32x4>(unit + 1024) + lane);
        w[0] = v0.x; w[1] = v0.y; w[2] = v0.z; w[3] = v0.w;
        w[4] = v1.x; w[5] = v1.y; w[6] = v1.z; w[7] = v1.w;
    }
    struct Magic { uint32_t m256, m16; };
    __device__ static Magic magic() { return {opaque_vgpr(0x5C005C00u), opaque_vgpr(0x4C004C00u)}; }
    __device__ static void unpack(const uint32_t* w, const Magic& k, uint32_t (&a)[16]) {
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            uint32_t u0 = w[h] << 2, u1 = w[h] >> 6;
            a[4 * h + 0] = and_or(u0, 0x003C003Cu, k.m256);
            a[4 * h + 1] = and_or(u0, 0x03C003C0u, k.m16);
            a[4 * h + 2] = and_or(u1, 0x003C003Cu, k.m256);
            a[4 * h + 3] = and_or(u1, 0x03C003C0u, k.m16);
        }
    }
};

template <> struct Codec<3> {
    static constexpr int WORDS = 6;
    __device__ static float offset(int t) {
        const float o[5] = {128.f, 128.f, 16.f, 128.f, 16.f};
        return t < 15 ? o[t % 5] : 16.f;
    }
    __device__ static void load(const uint8_t* unit, int lane, uint32_t (&w)[WORDS]) {
        u32x2 v0 = __builtin_nontemporal_load(as_global<u32x2>(unit) + lane);
        u32x4 v1 = __builtin_nontemporal_load(as_global<u32x4>(unit + 512) + lane);
        w[0] = v0.x; w[1] = v0.y;
        w[2] = v1.x; w[3] = v1.y; w[4] = v1.z; w[5] = v1.w;
    }
    struct Magic { uint32_t m128, m16; };
    __device__ static Magic magic() { return {opaque_vgpr(0x58005800u), opaque_vgpr(0x4C004C00u)}; }
    __device__ static void unpack(const uint32_t* w, const Magic& k, uint32_t (&a)[16]) {
#pragma unroll
        for (int h = 0; h < 3; ++h) {
            uint32_t u0 = w[h], u1 = u0 >> 6, u2 = u0 << 3;
            a[5 * h + 0] = and_or(u2, 0x00380038u, k.m128);
            a[5 * h + 1] = and_or(u0, 0x00380038u, k.m128);
            a[5 * h + 2] = and_or(u0, 0x01C001C0u, k.m16);
            a[5 * h + 3] = and_or(u1, 0x00380038u, k.m128);
            a[5 * h + 4] = and_or(u1, 0x01C001C0u, k.m16);
        }
        // pair 15: bit h of its codes sits in bit 15 of the halves of word h
        uint32_t r = and_or(w[0] >> 9, 0x00400040u, k.m16);
        r = and_or(w[1] >> 8, 0x00800080u, r);
        a[15] = and_or(w[2] >> 7, 0x01000100u, r);
    }
};

__device__ inline float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Stage x into LDS as fp16 and compute corr[] per block.  bf16 input is multiplied by a power of
// two chosen from max|x| so that it lands in fp16's range (bf16 has 8 significant bits, fp16 11:
// the conversion is exact unless an element is > 2^28 times smaller than the largest); the
// returned factor undoes it at the end.
template <int BITS>
__device__ float stage_x(const AqGemvTask& t, uint16_t* xh, float* corr, float* scratch)
{
    const int tid = threadIdx.x;
    const int K = t.K, Kpad = t.nchunks * AQ_CHUNK_K;
    float unscale = 1.0f;
    if (t.x_dtype == 1) {   // AQ_F16: copy
        for (int i = tid * 8; i < Kpad; i += THREADS * 8) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (i < K) v = *(as_global<u32x4>(t.x + i));
            *reinterpret_cast<u32x4*>(xh + i) = v;
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
            *reinterpret_cast<u32x4*>(xh + i) = o;
        }
    }
    __syncthreads();
    // corr[block] = sum_t (magic_t + z) (x[2t] + x[2t+1]): one 2-wide fp16 dot product (fp32
    // accumulate) per pair; the constants are small integers, exact in fp16
    const float z = (float)(1 << (BITS - 1));
    for (int b = tid; b < t.nchunks * AQ_CHUNK_BLOCKS; b += THREADS) {
        const u32x4* xb = reinterpret_cast<const u32x4*>(xh + b * AQ_BLOCK);
        float s = 0.f;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const u32x4 v = xb[q4];
            const uint32_t ws[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const _Float16 k = (_Float16)(Codec<BITS>::offset(4 * q4 + j) + z);
                s = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, ws[j]), half2v{k, k}, s, false);
            }
        }
        corr[b] = s;
    }
    __syncthreads();
    return unscale;
}

#ifndef AQ_GEMV_SCHED_FENCE
#define AQ_GEMV_SCHED_FENCE 1
#endif
// One unit (16 rows x 8 blocks): unpack the ring slot, optionally refill it from `next`, run the
// 8 MFMAs against the block-diagonal B and fold the block sums, times their fp16 scales, into the
// tile's running sums at `sums` (LDS, owned by this lane).
template <int BITS, bool REFILL>
__device__ __forceinline__ void unit_step(uint32_t (&raw)[Codec<BITS>::WORDS], u32x2& sc,
                                          const typename Codec<BITS>::Magic& magic, const half8 (&B)[8],
                                          const float4v& negc, const uint8_t* next, int lane, int sc_off,
                                          float* sums)
{
#if AQ_GEMV_SCHED_FENCE
    // Pin this unit's unpack behind the previous unit's stores: without it the compiler hoists the
    // unpack of every unit in flight to the top of the loop body and holds all of their operands
    // live at once (2-3x the registers).  Other wavefronts on the SIMD fill the MFMA latency.
#pragma unroll
    for (int i = 0; i < Codec<BITS>::WORDS; ++i) asm volatile("" : "+v"(raw[i]) : : "memory");
#endif
    uint32_t a0[16], a1[16];
    Codec<BITS>::unpack(&raw[0], magic, a0);
    Codec<BITS>::unpack(&raw[BITS], magic, a1);
    const half4v d4 = __builtin_bit_cast(half4v, sc);           // scales of rows 4g .. 4g+3
    if (REFILL) {
        Codec<BITS>::load(next, lane, raw);
        sc = __builtin_nontemporal_load(as_global<u32x2>(next + sc_off));
    }
    float o0 = sums[0], o1 = sums[32], o2 = sums[64], o3 = sums[96];   // read early: the MFMAs hide it
    float4v D = negc;
#pragma unroll
    for (int m = 0; m < 8; ++m) {
        u32x4 av = {a0[2 * m], a0[2 * m + 1], a1[2 * m], a1[2 * m + 1]};
        D = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, av), B[m], D, 0, 0, 0);
    }
    sums[0] = fmaf(D[0], (float)d4.x, o0);
    sums[32] = fmaf(D[1], (float)d4.y, o1);
    sums[64] = fmaf(D[2], (float)d4.z, o2);
    sums[96] = fmaf(D[3], (float)d4.w, o3);
}

// DEPTH consecutive units of one chunk starting at tile rt0; slot u is refilled from refill + u*UNIT
template <int BITS, int DEPTH, bool REFILL>
__device__ __forceinline__ void unit_block(uint32_t (&raw)[DEPTH][Codec<BITS>::WORDS], u32x2 (&sc)[DEPTH],
                                           const typename Codec<BITS>::Magic& magic, const half8 (&B)[8],
                                           const float4v& negc, const uint8_t* refill, int lane, int sc_off,
                                           float* sums, int tile_stride)
{
    constexpr int UNIT = 512 * BITS + 256;
#pragma unroll
    for (int u = 0; u < DEPTH; ++u)
        unit_step<BITS, REFILL>(raw[u], sc[u], magic, B, negc, refill + u * UNIT, lane, sc_off,
                                sums + u * tile_stride);
}

#ifndef AQ_GEMV_MIN_WAVES
#define AQ_GEMV_MIN_WAVES 3
#endif
template <int BITS, int RT>
__global__ __launch_bounds__(THREADS, AQ_GEMV_MIN_WAVES) void qgemv_kernel(const AqGemvTask* __restrict__ tasks, int count,
                                                        AqGemvTask single)
{
    extern __shared__ __align__(16) uint8_t smem[];
    constexpr int WORDS = Codec<BITS>::WORDS;
    constexpr int UNIT = 512 * BITS + 256;
    constexpr int DEPTH = RT < 4 ? RT : 4;          // units of loads kept in flight per wavefront

    AqGemvTask t;
    int wg = blockIdx.x;
    if (count == 0) {
        t = single;
    } else {
        int lo = 0, hi = count - 1;          // last task whose first workgroup is <= blockIdx.x
        while (lo < hi) {
            int mid = (lo + hi + 1) >> 1;
            if (tasks[mid].wg_begin <= wg) lo = mid; else hi = mid - 1;
        }
        t = tasks[lo];
        wg -= t.wg_begin;
    }
    if (wg >= t.wg_count) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // uniform: keep it in an SGPR
    const int g = lane >> 4, c = lane & 15;
    const int nch = t.nchunks, Kpad = nch * AQ_CHUNK_K;

    uint16_t* xh = reinterpret_cast<uint16_t*>(smem);                       // Kpad fp16
    float* corr = reinterpret_cast<float*>(smem + Kpad * 2);                // nch * 8
    float* red = reinterpret_cast<float*>(smem + Kpad * 2 + nch * 32);      // WAVES * (RT + 1) * 128
    uint32_t* zeros = reinterpret_cast<uint32_t*>(smem + Kpad * 2 + nch * 32 + WAVES * (RT + 1) * 512);  // 16 words
    if (tid < 16) zeros[tid] = 0u;

    const int subs = AQ_GROUP_TILES / RT;
    const int group = wg / subs, sub = wg % subs;
    const bool diag = (c < 8) && ((c >> 1) == g);
    const bool hi = (c & 1) != 0;

    // Register ring of DEPTH units (raw code words + 4 scales per lane).  The wavefront walks its
    // units in the order (chunk, tile); a slot is refilled with the unit DEPTH positions ahead as
    // soon as its words have been unpacked, so DEPTH - 1 units of loads stay in flight.  The first
    // fill is issued before x is staged, so that it overlaps the workgroup's start-up.
    const uint8_t* gbase = t.blob + ((int64_t)group * nch * AQ_GROUP_TILES + sub * RT) * UNIT;
    const int64_t chunk_stride = (int64_t)AQ_GROUP_TILES * UNIT;
    const int sc_off = 512 * BITS + (g * 8 + (c & 7)) * 8;
    uint32_t raw[DEPTH][WORDS];
    u32x2 sc[DEPTH];
    if (wave < nch) {
        const uint8_t* ub = gbase + wave * chunk_stride;
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            Codec<BITS>::load(ub + u * UNIT, lane, raw[u]);
            sc[u] = __builtin_nontemporal_load(as_global<u32x2>(ub + u * UNIT + sc_off));
        }
    }

    // Per-wavefront partial sums live in LDS (red[wave][tile][r][g*8 + c], read-modify-written by
    // their owner only), so the tile loop needs no accumulator registers.  Lanes c >= 8 hold no
    // useful MFMA column; they update a private dummy block so that no lane ever branches.
    float* mysum;
    int tile_stride;
    {
        float* dummy = red + WAVES * RT * 128;                 // WAVES * 128 floats
        const int idx = g * 8 + (c & 7);
        mysum = (c < 8) ? red + wave * RT * 128 + idx : dummy + wave * 128 + idx;
        tile_stride = (c < 8) ? 128 : 0;
    }
    for (int i = tid; i < WAVES * (RT + 1) * 128; i += THREADS) red[i] = 0.f;

    const float unscale = stage_x<BITS>(t, xh, corr, reinterpret_cast<float*>(zeros + 16));

    const typename Codec<BITS>::Magic magic = Codec<BITS>::magic();

    // The wavefront's units in visiting order: chunk wave, wave + 4, ...; inside a chunk tiles
    // 0 .. RT-1, taken DEPTH at a time ("blocks").  Block j + 1 refills the ring while block j is
    // being consumed.
    constexpr int NBLK = RT / DEPTH;
    const int my_chunks = wave < nch ? (nch - wave + WAVES - 1) / WAVES : 0;
    const int total = my_chunks * NBLK;
#pragma unroll 1
    for (int j = 0; j < total; ++j) {
        const int cj = j / NBLK, rb = j % NBLK;
        // B operand of the chunk: x of block c goes to the k-slots of block c (the low two registers
        // for even c, the high two for odd c); every other slot reads the 64-byte zero region.  It
        // is re-read from LDS for every block of tiles: that costs LDS reads only and keeps its 32
        // registers from living across the loop.
        const int ch = wave + cj * WAVES;
        const uint32_t* xblk = reinterpret_cast<const uint32_t*>(xh + (ch * AQ_CHUNK_BLOCKS + (c & 7)) * AQ_BLOCK);
        const u32x2* blo = reinterpret_cast<const u32x2*>((diag && !hi) ? xblk : zeros);
        const u32x2* bhi = reinterpret_cast<const u32x2*>((diag && hi) ? xblk : zeros);
        half8 B[8];
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            const u32x2 l = blo[m], h = bhi[m];
            B[m] = __builtin_bit_cast(half8, u32x4{l.x, l.y, h.x, h.y});
        }
        const float nc = -corr[ch * AQ_CHUNK_BLOCKS + (c & 7)];
        const float4v negc = {nc, nc, nc, nc};
        float* sums = mysum + rb * DEPTH * tile_stride;
        if (j + 1 < total) {
            const int cn = (j + 1) / NBLK, rn = (j + 1) % NBLK;
            const uint8_t* nb = gbase + (int64_t)(wave + cn * WAVES) * chunk_stride + rn * DEPTH * UNIT;
            unit_block<BITS, DEPTH, true>(raw, sc, magic, B, negc, nb, lane, sc_off, sums, tile_stride);
        } else {
            unit_block<BITS, DEPTH, false>(raw, sc, magic, B, negc, gbase, lane, sc_off, sums, tile_stride);
        }
    }

    __syncthreads();
    if (tid < RT * 16) {
        const int rt = tid >> 4, i = tid & 15, gg = i >> 2, r = i & 3;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            const float* p = red + ((w * RT + rt) * 4 + r) * 32 + gg * 8;
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) s += p[cc];
        }
        const int64_t row = ((int64_t)group * AQ_GROUP_TILES + sub * RT + rt) * AQ_TILE_ROWS + i;
        if (row < t.N) ((AQ_GLOBAL float*)(uintptr_t)t.y)[row] = s * unscale;
    }
}

size_t gemv_lds_bytes(int max_K, int RT)
{
    int nch = (max_K + AQ_CHUNK_K - 1) / AQ_CHUNK_K;
    return (size_t)nch * AQ_CHUNK_K * 2 + (size_t)nch * 32 + (size_t)WAVES * (RT + 1) * 512 + 64 + 16;
}

}  // namespace

int aqk_gemv_tiles_per_wg(int64_t N, bool batched)
{
    if (batched) {
        const char* e = getenv("AQ_BATCH_RT");
        int v = e ? atoi(e) : 8;
        return (v == 1 || v == 2 || v == 4 || v == 8) ? v : 8;
    }
    // a lone matrix: keep at least ~1024 workgroups where the matrix allows it
    int64_t tiles = (N + AQ_TILE_ROWS - 1) / AQ_TILE_ROWS;
    if (tiles >= 8192) return 8;
    if (tiles >= 4096) return 4;
    if (tiles >= 2048) return 2;
    return 1;
}

int aqk_gemv_wg_count(int64_t N, int tiles_per_wg)
{
    return (int)(aq_num_groups(N) * (AQ_GROUP_TILES / tiles_per_wg));
}

template <int RT>
static void launch_bits(int bits, dim3 grid, size_t lds, hipStream_t s, const AqGemvTask* tasks, int count,
                        const AqGemvTask& single)
{
    dim3 block(THREADS);
    if (bits == 2) hipLaunchKernelGGL((qgemv_kernel<2, RT>), grid, block, lds, s, tasks, count, single);
    else if (bits == 3) hipLaunchKernelGGL((qgemv_kernel<3, RT>), grid, block, lds, s, tasks, count, single);
    else hipLaunchKernelGGL((qgemv_kernel<4, RT>), grid, block, lds, s, tasks, count, single);
}

// all tasks of one launch share `bits`
hipError_t aqk_gemv(const AqGemvTask* tasks_dev, int count, const AqGemvTask& single, int bits, int tiles_per_wg,
                    int total_wgs, int max_K, hipStream_t s)
{
    size_t lds = gemv_lds_bytes(max_K, tiles_per_wg);
    dim3 grid((unsigned)total_wgs);
    switch (tiles_per_wg) {
        case 1: launch_bits<1>(bits, grid, lds, s, tasks_dev, count, single); break;
        case 2: launch_bits<2>(bits, grid, lds, s, tasks_dev, count, single); break;
        case 4: launch_bits<4>(bits, grid, lds, s, tasks_dev, count, single); break;
        default: launch_bits<8>(bits, grid, lds, s, tasks_dev, count, single); break;
    }
    return hipGetLastError();
}
