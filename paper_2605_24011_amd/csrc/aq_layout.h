// Device blob layout of one block-quantised matrix (private to this library).
//
// The blob stores the same information as the canonical form of Eq. 1 (codes q and one
// fp16 scale d per block of 32 along K), re-tiled so that the decode kernel can feed the
// matrix cores straight from 128-bit loads:
//
//   tile   = 16 consecutive rows of W            (the M extent of a 16x16x32 MFMA)
//   chunk  = 8 consecutive blocks = 256 k        (one MFMA per pair-slot, see below)
//   unit   = one tile x one chunk = 4096 weights, UNIT_BYTES(bits) = 512*bits + 256 bytes
//   group  = 8 consecutive tiles = 128 rows
//
// Blob = units in the order [group][chunk][tile in group]; rows are padded to a multiple
// of 128 and blocks to a multiple of 8 with zero codes and zero scales.  A 256-byte trailer
// follows the units; its first 32-bit word is the largest |d| of the matrix as a binary16
// bit pattern (0x7C00 and above: an infinity or NaN is present).  The prefill kernel reads
// it to decide whether d * (q - z) can be formed in binary16 without overflow.
//
// Inside a unit, lane l = 16*g + i (g = l / 16, i = l % 16) of a wavefront owns row i of
// the tile and the two blocks 2g, 2g+1 of the chunk.  A block is `bits` 32-bit words; each
// word is two 16-bit halves, the low half carrying the even elements (2t) and the high half
// the odd elements (2t+1) of "pairs" t = 0..15 of the block, so that one AND-OR with a
// constant turns a word into two fp16 numbers (magic + code):
//   bits = 2: word h (0..1) holds pairs t = 8h + s, s = 0..7, code at half-bit 2s
//   bits = 4: word h (0..3) holds pairs t = 4h + s, s = 0..3, code at half-bit 4s
//   bits = 3: two planes.  Words 0, 1 hold the upper two bits of every code (q >> 1) in the 2-bit format above; word 2
//             holds the lowest bits: bit (q & 1) of element 16h + 4n + 2f + o (h, f, o in {0,1}, n in 0..3) sits at
//             bit 16o + 4n + 2h + f, i.e. pair t = 8h + 2n + f has its two low bits at half-bit 4n + 2h + f.  (The decode
//             kernel feeds each plane to the matrix cores as 4-bit fields: `(word >> j) & 0x11111111` must put
//             element (register j = 2h + f, nibble n + 4o) where `(word_h >> 2f) & 0x33333333` puts its upper bits.)
// The lane's 2*bits words are w[blk*bits + h] (blk = 0, 1).
//   code area  : bits == 2: one plane of 16 B per lane (4 words)          -> 1024 B
//                bits == 3: plane A 8 B per lane (words 0,1), plane B 16 B per lane (words 2..5) -> 512 + 1024 B
//                bits == 4: two planes of 16 B per lane (words 0..3, 4..7) -> 2048 B
//   scale area : 256 B after the codes: for lane l with c = l % 16 < 8, g = l / 16:
//                4 fp16 = scales of rows 4g+r (r = 0..3), block c, at byte (g*8 + c)*8 + 2r.
//                (This is the accumulator layout of the MFMA: lane (g, c) holds rows 4g..4g+3
//                of column c.)
#pragma once
#include <stdint.h>

#define AQ_BLOCK 32
#define AQ_TILE_ROWS 16
#define AQ_CHUNK_BLOCKS 8
#define AQ_CHUNK_K (AQ_CHUNK_BLOCKS * AQ_BLOCK)
#define AQ_GROUP_TILES 8
#define AQ_GROUP_ROWS (AQ_GROUP_TILES * AQ_TILE_ROWS)

#if defined(__HIPCC__)
#define AQ_HD __host__ __device__ inline
#else
#define AQ_HD inline
#endif

AQ_HD int64_t aq_unit_bytes(int bits) { return 512 * (int64_t)bits + 256; }
AQ_HD int64_t aq_num_groups(int64_t N) { return (N + AQ_GROUP_ROWS - 1) / AQ_GROUP_ROWS; }
AQ_HD int64_t aq_num_chunks(int64_t K) { return (K + AQ_CHUNK_K - 1) / AQ_CHUNK_K; }
AQ_HD int64_t aq_unit_index(int64_t group, int64_t chunk, int tile_in_group, int64_t nchunks)
{
    return (group * nchunks + chunk) * AQ_GROUP_TILES + tile_in_group;
}
#define AQ_TRAILER_BYTES 256
AQ_HD int64_t aq_trailer_offset(int64_t N, int64_t K, int bits)
{
    return aq_num_groups(N) * aq_num_chunks(K) * AQ_GROUP_TILES * aq_unit_bytes(bits);
}
AQ_HD int64_t aq_blob_bytes(int64_t N, int64_t K, int bits) { return aq_trailer_offset(N, K, bits) + AQ_TRAILER_BYTES; }

// byte offset inside a unit of word `wi` (0 .. 2*bits-1) of lane `l`
AQ_HD int aq_word_offset(int bits, int l, int wi)
{
    if (bits == 2) return l * 16 + wi * 4;
    if (bits == 4) return (wi >> 2) * 1024 + l * 16 + (wi & 3) * 4;
    return wi < 2 ? l * 8 + wi * 4 : 512 + l * 16 + (wi - 2) * 4;   // bits == 3
}
AQ_HD int aq_scale_offset(int bits, int g, int c, int r)
{
    return 512 * bits + (g * 8 + c) * 8 + 2 * r;
}

// ---- two-level variant of the format: w = D_S * a_b * q - M_S * c_b (a_b, c_b 4-bit codes of block b, D_S, M_S
// binary16 numbers of the super-block = the 8 blocks of a row inside one chunk).  Same tiling and the same code
// words as the base format; the unit's 256 bytes of scales are replaced by 192 bytes of parameters:
//   bytes 512*bits + (g*8 + blk)*4 + r   : a | c << 4 of row 4g + r, block blk          (128 bytes)
//   bytes 512*bits + 128 + (g*4 + r)*4   : D (2 bytes), M (2 bytes) of row 4g + r        (64 bytes)
// so that lane (g, c) of the decode kernel reads its 4 rows of block c & 7 as ONE 32-bit word and the 4 rows'
// D, M as one 16-byte vector.  No trailer.
#define AQ2_PARAM_BYTES 192
AQ_HD int64_t aq2_unit_bytes(int bits) { return 512 * (int64_t)bits + AQ2_PARAM_BYTES; }
AQ_HD int64_t aq2_blob_bytes(int64_t N, int64_t K, int bits)
{
    return aq_num_groups(N) * aq_num_chunks(K) * AQ_GROUP_TILES * aq2_unit_bytes(bits);
}
AQ_HD int aq2_sub_offset(int bits, int g, int blk, int r) { return 512 * bits + (g * 8 + blk) * 4 + r; }
AQ_HD int aq2_sup_offset(int bits, int g, int r) { return 512 * bits + 128 + (g * 4 + r) * 4; }

// element e (0..31) of a block given the block's `bits` words
AQ_HD uint32_t aq_block_get(const uint32_t* w, int bits, int e)
{
    int t = e >> 1, sh = (e & 1) * 16;
    if (bits == 2) return (w[t >> 3] >> (sh + 2 * (t & 7))) & 3u;
    if (bits == 4) return (w[t >> 2] >> (sh + 4 * (t & 3))) & 15u;
    // bits == 3: upper two bits in the 2-bit format, lowest bit in word 2
    int h = t >> 3, s = t & 7, n = s >> 1, f = s & 1;
    uint32_t hi = (w[h] >> (sh + 2 * s)) & 3u, lo = (w[2] >> (sh + 4 * n + 2 * h + f)) & 1u;
    return 2u * hi + lo;
}
AQ_HD void aq_block_put(uint32_t* w, int bits, int e, uint32_t q)
{
    int t = e >> 1, sh = (e & 1) * 16;
    if (bits == 2) w[t >> 3] |= q << (sh + 2 * (t & 7));
    else if (bits == 4) w[t >> 2] |= q << (sh + 4 * (t & 3));
    else {
        int h = t >> 3, s = t & 7, n = s >> 1, f = s & 1;
        w[h] |= (q >> 1) << (sh + 2 * s);
        w[2] |= (q & 1u) << (sh + 4 * n + 2 * h + f);
    }
}
