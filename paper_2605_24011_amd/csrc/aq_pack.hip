// Packer (canonical form of Eq. 1 -> device blob) and its two inverses used for parity
// checks: blob -> codes, blob -> dequantised fp32 weights.  None of these is on the timed
// path; they are written for clarity (one thread per lane-slot of a unit).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "aq_layout.h"
#include "aq_kernels.h"

namespace {

// code e of a canonical block: bits [e*bits, e*bits+bits) of the block's little-endian bitstream
__device__ inline uint32_t canon_code(const uint8_t* blk, int bits, int e)
{
    int bit = e * bits, byte = bit >> 3, sh = bit & 7;
    uint32_t v = blk[byte];
    if (sh + bits > 8) v |= (uint32_t)blk[byte + 1] << 8;
    return (v >> sh) & ((1u << bits) - 1u);
}

// one thread per (unit, lane)
__global__ __launch_bounds__(256) void pack_kernel(const uint8_t* __restrict__ codes,
                                                   const uint16_t* __restrict__ scales,
                                                   int64_t N, int64_t K, int bits,
                                                   uint8_t* __restrict__ blob, int64_t n_units,
                                                   uint32_t* __restrict__ trailer, uint64_t remap)
{
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t unit = gid >> 6;
    if (unit >= n_units) return;                   // whole wavefronts leave together: 64 threads per unit
    int l = (int)(gid & 63), g = l >> 4, i = l & 15;
    int64_t nb = K / AQ_BLOCK, nchunks = aq_num_chunks(K);
    int til = (int)(unit % AQ_GROUP_TILES);
    int64_t chunk = (unit / AQ_GROUP_TILES) % nchunks;
    int64_t group = unit / (AQ_GROUP_TILES * nchunks);
    uint8_t* u = blob + unit * aq_unit_bytes(bits);
    int64_t row0 = (group * AQ_GROUP_TILES + til) * AQ_TILE_ROWS;

    // codes: row i of the tile, blocks 2g and 2g+1 of the chunk
    int64_t row = row0 + i;
    for (int blk = 0; blk < 2; ++blk) {
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        int64_t j = chunk * AQ_CHUNK_BLOCKS + 2 * g + blk;
        if (row < N && j < nb) {
            const uint8_t* src = codes + (row * nb + j) * (4 * bits);
            for (int e = 0; e < 32; ++e)
                aq_block_put(w, bits, e, (uint32_t)(remap >> (4 * canon_code(src, bits, e))) & 15u);
        }
        for (int h = 0; h < bits; ++h)
            *reinterpret_cast<uint32_t*>(u + aq_word_offset(bits, l, blk * bits + h)) = w[h];
    }
    // scales: lane (g, c) with c < 8 stores rows 4g..4g+3 of block c
    uint32_t mag = 0;                               // largest |d| bit pattern this thread stored
    if (i < 8) {
        int64_t j = chunk * AQ_CHUNK_BLOCKS + i;
        for (int r = 0; r < 4; ++r) {
            int64_t rr = row0 + 4 * g + r;
            uint16_t s = (rr < N && j < nb) ? scales[rr * nb + j] : (uint16_t)0;
            *reinterpret_cast<uint16_t*>(u + aq_scale_offset(bits, g, i, r)) = s;
            uint32_t m = s & 0x7FFFu;
            mag = m > mag ? m : mag;
        }
    }
    // trailer word 0 = max over the matrix (binary16 magnitudes order like unsigned integers)
    for (int o = 32; o >= 1; o >>= 1) {
        uint32_t other = (uint32_t)__shfl_xor((int)mag, o);
        mag = other > mag ? other : mag;
    }
    if (l == 0 && mag != 0) atomicMax(trailer, mag);
}

__global__ void clear_trailer_kernel(uint32_t* trailer)
{
    if (threadIdx.x < AQ_TRAILER_BYTES / 4) trailer[threadIdx.x] = 0u;
}

// one thread per (row, block): writes 32 codes or 32 dequantised weights.  TABLE (codebook variant): a stored code c
// is reported as (remap >> 4c) & 15 and dequantised as d * table.level[c]
template <bool DEQUANT, bool TABLE = false>
__global__ __launch_bounds__(256) void decode_kernel(const uint8_t* __restrict__ blob, int64_t N, int64_t K,
                                                     int bits, uint8_t* __restrict__ out_codes,
                                                     float* __restrict__ out_w, uint64_t remap, AqCbTable table)
{
    int64_t nb = K / AQ_BLOCK;
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= N * nb) return;
    int64_t row = gid / nb, j = gid % nb;
    int64_t tile = row / AQ_TILE_ROWS;
    int i = (int)(row % AQ_TILE_ROWS);
    int64_t group = tile / AQ_GROUP_TILES;
    int til = (int)(tile % AQ_GROUP_TILES);
    int64_t chunk = j / AQ_CHUNK_BLOCKS;
    int c = (int)(j % AQ_CHUNK_BLOCKS);
    const uint8_t* u = blob + aq_unit_index(group, chunk, til, aq_num_chunks(K)) * aq_unit_bytes(bits);
    int l = 16 * (c >> 1) + i, blk = c & 1;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    for (int h = 0; h < bits; ++h)
        w[h] = *reinterpret_cast<const uint32_t*>(u + aq_word_offset(bits, l, blk * bits + h));
    if (DEQUANT) {
        uint16_t sb = *reinterpret_cast<const uint16_t*>(u + aq_scale_offset(bits, i >> 2, c, i & 3));
        float d = __half2float(__ushort_as_half(sb));
        int z = 1 << (bits - 1);
        for (int e = 0; e < 32; ++e)
            out_w[row * K + j * AQ_BLOCK + e] = TABLE ? d * table.level[aq_block_get(w, bits, e)]
                                                      : d * (float)((int)aq_block_get(w, bits, e) - z);
    } else {
        for (int e = 0; e < 32; ++e) {
            const uint32_t c = aq_block_get(w, bits, e);
            out_codes[row * K + j * AQ_BLOCK + e] = TABLE ? (uint8_t)((remap >> (4 * c)) & 15u) : (uint8_t)c;
        }
    }
}

// ---- two-level variant: same code words, parameters instead of scales (see aq_layout.h) ----
__global__ __launch_bounds__(256) void pack2_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ sub,
                                                    const uint16_t* __restrict__ sup, int64_t N, int64_t K, int bits,
                                                    uint8_t* __restrict__ blob, int64_t n_units)
{
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t unit = gid >> 6;
    if (unit >= n_units) return;
    int l = (int)(gid & 63), g = l >> 4, i = l & 15;
    int64_t nb = K / AQ_BLOCK, nchunks = aq_num_chunks(K);
    int til = (int)(unit % AQ_GROUP_TILES);
    int64_t chunk = (unit / AQ_GROUP_TILES) % nchunks;
    int64_t group = unit / (AQ_GROUP_TILES * nchunks);
    uint8_t* u = blob + unit * aq2_unit_bytes(bits);
    int64_t row0 = (group * AQ_GROUP_TILES + til) * AQ_TILE_ROWS;
    int64_t row = row0 + i;
    for (int blk = 0; blk < 2; ++blk) {
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        int64_t j = chunk * AQ_CHUNK_BLOCKS + 2 * g + blk;
        if (row < N && j < nb) {
            const uint8_t* src = codes + (row * nb + j) * (4 * bits);
            for (int e = 0; e < 32; ++e) aq_block_put(w, bits, e, canon_code(src, bits, e));
        }
        for (int h = 0; h < bits; ++h)
            *reinterpret_cast<uint32_t*>(u + aq_word_offset(bits, l, blk * bits + h)) = w[h];
    }
    // lane (g, i < 8): the codes of rows 4g..4g+3 of block i; lane (g, i in 8..11): D, M of row 4g + i - 8
    if (i < 8) {
        int64_t j = chunk * AQ_CHUNK_BLOCKS + i;
        for (int r = 0; r < 4; ++r) {
            int64_t rr = row0 + 4 * g + r;
            u[aq2_sub_offset(bits, g, i, r)] = (rr < N && j < nb) ? sub[rr * nb + j] : (uint8_t)0;
        }
    } else if (i < 12) {
        int r = i - 8;
        int64_t rr = row0 + 4 * g + r;
        uint16_t D = 0, M = 0;
        if (rr < N) {
            D = sup[(rr * nchunks + chunk) * 2];
            M = sup[(rr * nchunks + chunk) * 2 + 1];
        }
        *reinterpret_cast<uint16_t*>(u + aq2_sup_offset(bits, g, r)) = D;
        *reinterpret_cast<uint16_t*>(u + aq2_sup_offset(bits, g, r) + 2) = M;
    }
}

// one thread per (row, block): 32 codes or 32 dequantised weights, fp32(D a q - M c) with ONE rounding
template <bool DEQUANT>
__global__ __launch_bounds__(256) void decode2_kernel(const uint8_t* __restrict__ blob, int64_t N, int64_t K,
                                                      int bits, uint8_t* __restrict__ out_codes,
                                                      float* __restrict__ out_w)
{
    int64_t nb = K / AQ_BLOCK;
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= N * nb) return;
    int64_t row = gid / nb, j = gid % nb;
    int64_t tile = row / AQ_TILE_ROWS;
    int i = (int)(row % AQ_TILE_ROWS);
    int64_t group = tile / AQ_GROUP_TILES;
    int til = (int)(tile % AQ_GROUP_TILES);
    int64_t chunk = j / AQ_CHUNK_BLOCKS;
    int c = (int)(j % AQ_CHUNK_BLOCKS);
    const uint8_t* u = blob + aq_unit_index(group, chunk, til, aq_num_chunks(K)) * aq2_unit_bytes(bits);
    int l = 16 * (c >> 1) + i, blk = c & 1;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    for (int h = 0; h < bits; ++h)
        w[h] = *reinterpret_cast<const uint32_t*>(u + aq_word_offset(bits, l, blk * bits + h));
    if (DEQUANT) {
        const uint8_t sb = u[aq2_sub_offset(bits, i >> 2, c, i & 3)];
        const float D = __half2float(__ushort_as_half(*reinterpret_cast<const uint16_t*>(u + aq2_sup_offset(bits, i >> 2, i & 3))));
        const float M = __half2float(__ushort_as_half(*reinterpret_cast<const uint16_t*>(u + aq2_sup_offset(bits, i >> 2, i & 3) + 2)));
        const float s = D * (float)(sb & 15), off = M * (float)(sb >> 4);      // both exact in fp32
        for (int e = 0; e < 32; ++e)
            out_w[row * K + j * AQ_BLOCK + e] = fmaf(s, (float)aq_block_get(w, bits, e), -off);
    } else {
        for (int e = 0; e < 32; ++e)
            out_codes[row * K + j * AQ_BLOCK + e] = (uint8_t)aq_block_get(w, bits, e);
    }
}

}  // namespace

hipError_t aqk_pack(const uint8_t* codes, const uint16_t* scales, int64_t N, int64_t K, int bits,
                    void* blob, hipStream_t s)
{
    return aqk_pack_remap(codes, scales, N, K, bits, 0xFEDCBA9876543210ull, blob, s);
}

hipError_t aqk_pack_remap(const uint8_t* codes, const uint16_t* scales, int64_t N, int64_t K, int bits, uint64_t remap,
                          void* blob, hipStream_t s)
{
    int64_t n_units = aq_num_groups(N) * aq_num_chunks(K) * AQ_GROUP_TILES;
    int64_t threads = n_units * 64;
    unsigned grid = (unsigned)((threads + 255) / 256);
    uint32_t* trailer = reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(blob) + aq_trailer_offset(N, K, bits));
    hipLaunchKernelGGL(clear_trailer_kernel, dim3(1), dim3(64), 0, s, trailer);
    hipLaunchKernelGGL(pack_kernel, dim3(grid), dim3(256), 0, s, codes, scales, N, K, bits,
                       static_cast<uint8_t*>(blob), n_units, trailer, remap);
    return hipGetLastError();
}

namespace {

__global__ void write_table_kernel(AqCbTable table, float* dst)
{
    if (threadIdx.x < 16) dst[threadIdx.x] = table.level[threadIdx.x];
}

}  // namespace

hipError_t aqk_cb_write_table(const AqCbTable& table, float* dst, hipStream_t s)
{
    hipLaunchKernelGGL(write_table_kernel, dim3(1), dim3(64), 0, s, table, dst);
    return hipGetLastError();
}

hipError_t aqk_cb_unpack_codes(const void* blob, int64_t N, int64_t K, int bits, uint64_t inverse_remap, uint8_t* out,
                               hipStream_t s)
{
    unsigned grid = (unsigned)((N * (K / AQ_BLOCK) + 255) / 256);
    hipLaunchKernelGGL((decode_kernel<false, true>), dim3(grid), dim3(256), 0, s, static_cast<const uint8_t*>(blob),
                       N, K, bits, out, (float*)nullptr, inverse_remap, AqCbTable{});
    return hipGetLastError();
}

hipError_t aqk_cb_dequant(const void* blob, int64_t N, int64_t K, int bits, const AqCbTable& stored_levels, float* out,
                          hipStream_t s)
{
    unsigned grid = (unsigned)((N * (K / AQ_BLOCK) + 255) / 256);
    hipLaunchKernelGGL((decode_kernel<true, true>), dim3(grid), dim3(256), 0, s, static_cast<const uint8_t*>(blob),
                       N, K, bits, (uint8_t*)nullptr, out, (uint64_t)0, stored_levels);
    return hipGetLastError();
}

hipError_t aqk_unpack_codes(const void* blob, int64_t N, int64_t K, int bits, uint8_t* out, hipStream_t s)
{
    int64_t threads = N * (K / AQ_BLOCK);
    unsigned grid = (unsigned)((threads + 255) / 256);
    hipLaunchKernelGGL((decode_kernel<false, false>), dim3(grid), dim3(256), 0, s, static_cast<const uint8_t*>(blob),
                       N, K, bits, out, (float*)nullptr, (uint64_t)0, AqCbTable{});
    return hipGetLastError();
}

hipError_t aqk_dequant(const void* blob, int64_t N, int64_t K, int bits, float* out, hipStream_t s)
{
    int64_t threads = N * (K / AQ_BLOCK);
    unsigned grid = (unsigned)((threads + 255) / 256);
    hipLaunchKernelGGL((decode_kernel<true, false>), dim3(grid), dim3(256), 0, s, static_cast<const uint8_t*>(blob),
                       N, K, bits, (uint8_t*)nullptr, out, (uint64_t)0, AqCbTable{});
    return hipGetLastError();
}

hipError_t aqk2_pack(const uint8_t* codes, const uint8_t* sub, const uint16_t* sup, int64_t N, int64_t K, int bits,
                     void* blob, hipStream_t s)
{
    int64_t n_units = aq_num_groups(N) * aq_num_chunks(K) * AQ_GROUP_TILES;
    unsigned grid = (unsigned)((n_units * 64 + 255) / 256);
    hipLaunchKernelGGL(pack2_kernel, dim3(grid), dim3(256), 0, s, codes, sub, sup, N, K, bits,
                       static_cast<uint8_t*>(blob), n_units);
    return hipGetLastError();
}

hipError_t aqk2_unpack_codes(const void* blob, int64_t N, int64_t K, int bits, uint8_t* out, hipStream_t s)
{
    unsigned grid = (unsigned)((N * (K / AQ_BLOCK) + 255) / 256);
    hipLaunchKernelGGL(decode2_kernel<false>, dim3(grid), dim3(256), 0, s, static_cast<const uint8_t*>(blob),
                       N, K, bits, out, (float*)nullptr);
    return hipGetLastError();
}

hipError_t aqk2_dequant(const void* blob, int64_t N, int64_t K, int bits, float* out, hipStream_t s)
{
    unsigned grid = (unsigned)((N * (K / AQ_BLOCK) + 255) / 256);
    hipLaunchKernelGGL(decode2_kernel<true>, dim3(grid), dim3(256), 0, s, static_cast<const uint8_t*>(blob),
                       N, K, bits, (uint8_t*)nullptr, out);
    return hipGetLastError();
}
