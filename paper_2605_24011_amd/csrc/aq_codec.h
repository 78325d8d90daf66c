// Device-side pieces shared by the decode and prefill kernels: vector typedefs, the address-space
// helper, and the per-bit-width codec that turns a lane's raw code words into fp16 pairs.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aqdev {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 half4v __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));

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
    __device__ static void fence(Magic& k, float& a) {
        asm volatile("" : "+v"(k.m64), "+v"(k.m16), "+v"(k.m4), "+v"(a));
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
    __device__ static void fence(Magic& k, float& a) { asm volatile("" : "+v"(k.m256), "+v"(k.m16), "+v"(a)); }
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
    // Pair t = 8h + s of a block: its upper two bits sit at half-bits 2s, 2s+1 of word h, its lowest bit at half-bit
    // p = 4 (s / 2) + 2h + (s % 2) of word 2.  The lowest bit keeps its position (moved down by 8 when p >= 8) and the
    // upper bits are shifted next to it: the code then occupies mantissa bits b .. b+2, b = p % 8, of a binary16 number
    // whose exponent makes bit b worth one: magic = 2^(10 - b).
    __device__ static constexpr int lowbit(int t) { return (4 * ((t & 7) >> 1) + 2 * (t >> 3) + (t & 1)) & 7; }
    __device__ static float offset(int t) { return (float)(1 << (10 - lowbit(t))); }
    __device__ static void load(const uint8_t* unit, int lane, uint32_t (&w)[WORDS]) {
        u32x2 v0 = __builtin_nontemporal_load(as_global<u32x2>(unit) + lane);
        u32x4 v1 = __builtin_nontemporal_load(as_global<u32x4>(unit + 512) + lane);
        w[0] = v0.x; w[1] = v0.y;
        w[2] = v1.x; w[3] = v1.y; w[4] = v1.z; w[5] = v1.w;
    }
    struct Magic { uint32_t m[8]; };               // m[b] = the pair (2^(10-b), 2^(10-b)) as binary16 bit patterns
    __device__ static Magic magic() {
        Magic k;
#pragma unroll
        for (int b = 0; b < 8; ++b) k.m[b] = opaque_vgpr((uint32_t)(25 - b) * 0x04000400u);
        return k;
    }
    __device__ static void fence(Magic& k, float& a) {
        asm volatile("" : "+v"(k.m[0]), "+v"(k.m[1]), "+v"(k.m[2]), "+v"(k.m[3]), "+v"(k.m[4]), "+v"(k.m[5]), "+v"(k.m[6]),
                     "+v"(k.m[7]), "+v"(a));
    }
    // words of one block (w[0], w[1]: the upper-bit plane, w[2]: the lowest bits) -> 16 pair registers
    __device__ static void unpack(const uint32_t* w, const Magic& k, uint32_t (&a)[16]) {
        const uint32_t l0 = w[2], l8 = w[2] >> 8;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            // shifts of the upper-bit word that bring the field of pair s to bits b+1, b+2: s < 4: 2h + 1 - (s % 2),
            // s >= 4: that minus 8
            const int up = 2 * h + 1;
            const uint32_t e0 = w[h] << up, o0 = up > 1 ? w[h] << (up - 1) : w[h];
            const uint32_t e1 = w[h] >> (8 - up), o1 = w[h] >> (9 - up);
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int t = 8 * h + s, b = lowbit(t);
                const uint32_t hv = s < 4 ? ((s & 1) ? o0 : e0) : ((s & 1) ? o1 : e1);
                const uint32_t lv = s < 4 ? l0 : l8;
                a[t] = and_or(lv, 0x00010001u << b, and_or(hv, 0x00060006u << b, k.m[b]));
            }
        }
    }
};

// words of one block -> 16 registers, each a pair of exact (q - z) in fp16 or bf16 (RAWQ: the codes q themselves)
template <int BITS, bool XBF, bool RAWQ = false>
__device__ __forceinline__ void unpack_exact(const uint32_t* w, const typename Codec<BITS>::Magic& magic,
                                             uint32_t (&o)[16])
{
    uint32_t a[16];
    Codec<BITS>::unpack(w, magic, a);              // fp16 pairs (magic + q)
    const float z = RAWQ ? 0.f : (float)(1 << (BITS - 1));
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

}  // namespace aqdev
