// Prefill, fp16-weight mode, prefill-sized M: producer and consumer wavefronts.
//
// The shared-role kernel (aq_gemm.hip: 8 wavefronts that all unpack and all multiply) spends the issue slots of the
// wavefronts that feed the matrix pipe on unpacking.  Here the 12 wavefronts of a workgroup split the ROLES:
//   * wavefronts 0-7 (consumers, two per SIMD: one wavefront alone cannot issue 16x16x32 MFMAs back to back fast
//     enough, 1.25 against 1.5 PFLOP/s in the probe) own 2 or 3 m-tiles x all 8 n-tiles each (up to 24 m-tiles =
//     384 rows of X per workgroup; 19 tiles are dealt 3,3,3,2,2,2,2,2, so that every SIMD works through at most 5;
//     96 accumulator registers).  Per 32-k step a consumer reads 8 weight operands from LDS and its activation
//     operands from the re-tiled X in global memory (two steps ahead) and issues 16 or 24 MFMAs; nothing else
//     competes for its issue slots.  The tile count is a compile-time constant of the loop instance it runs.
//   * wavefronts 8-11 (producers, one per SIMD) own 2 of the group's 8 tiles each: load the packed units two chunks
//     ahead, unpack, multiply by the block scale in binary16 (w = d * (q - z)) and write the next chunk's tile to the
//     other LDS buffer.  Their vector-ALU work runs under the consumers' MFMAs.
// One LDS-only barrier per chunk (256 k) orders "next tile written" and "current tile read".
// (Four consumers of 5 m-tiles each, one per SIMD, 8 wavefronts in all: 3.43 ms for the M = 300 pass against 3.25 ms.)
//
// A matrix whose largest scale could overflow binary16 has every scale multiplied by 2^-sh first and the result by
// 2^sh (as in the small-M kernel).  Activations: the re-tiled binary16 copy Xt with one power-of-two factor per
// row (aq_gemm.hip's pre-pass).
#include <hip/hip_runtime.h>
#include <type_traits>
#include "aq_layout.h"
#include "aq_kernels.h"
#include "aq_codec.h"

namespace {

using namespace aqdev;

#ifndef AQ_PC_CONSUMERS
#define AQ_PC_CONSUMERS 8
#define AQ_PC_MT 3
#define AQ_PC_MT_LOW 2
#endif
constexpr int PC_CONSUMERS = AQ_PC_CONSUMERS;
constexpr int PC_THREADS = (PC_CONSUMERS + 4) * 64;
constexpr int PC_MT = AQ_PC_MT;                       // most m-tiles per consumer
#ifndef AQ_PC_MT_LOW
#define AQ_PC_MT_LOW AQ_PC_MT
#endif
#ifndef AQ_PC_NJ
#define AQ_PC_NJ 2
#endif
constexpr int PC_MT_LOW = AQ_PC_MT_LOW;               // the loop instance of a consumer that owns at most this many
constexpr int PC_MBLOCK = PC_CONSUMERS * PC_MT;       // m-tiles per workgroup
constexpr int PC_W_ROW = AQ_CHUNK_K * 2 + 32;         // LDS row stride of the weight tile: 544 B (64 j + 32: conflict-free b128 reads)
constexpr int PC_WBUF = AQ_GROUP_ROWS * PC_W_ROW;     // one chunk's tile: 128 rows

__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Producer: tiles 2p, 2p+1 of the group, all chunks.  Executes nch + 1 barriers.
// FMT 0: the base format, w = fp16(d * (q - z)).  FMT 1: the two-level variant, w = fp16(q * fp16(D a) - fp16(M c))
// (three roundings to 11 bits instead of one: D a and M c have up to 15 significant bits).  FMT 2: the codebook
// variant, w = fp16(d * level[stored code]), the product formed in fp32 and rounded once; the table of 16 levels sits
// in the lanes of the wavefront (lane l holds level[l % 16]) and a lookup is one cross-lane read (DS_BPERMUTE_B32).
template <int BITS, int FMT>
__device__ __forceinline__ void produce(const AqGemmTask& t, int group, int p, int lane, uint8_t* smem, _Float16 down,
                                        const float* __restrict__ cb_table, int ch0, int nloc)
{
    constexpr int WORDS = Codec<BITS>::WORDS;
    constexpr int UNIT = 512 * BITS + (FMT == 1 ? AQ2_PARAM_BYTES : 256);
    const int g = lane >> 4, c = lane & 15;
    // the workgroup's part of K: chunks ch0 .. ch0 + nloc - 1 of the matrix's t.nchunks (all of them unless K is split)
    const int nch = nloc;
    const uint8_t* ubase = t.blob + (((int64_t)group * t.nchunks + ch0) * AQ_GROUP_TILES + 2 * p) * UNIT;
    const int64_t chunk_stride = (int64_t)AQ_GROUP_TILES * UNIT;
    uint32_t raw[2][WORDS];
    uint32_t sc[2][2];                                // FMT 0: scales of row c, blocks 2g and 2g + 1
                                                      // FMT 1: [0] = the (a, c) bytes of those two blocks, [1] = D | M << 16 of row c
    auto load_w = [&](int ch) {
#pragma unroll
        for (int w = 0; w < 2; ++w) {
            const uint8_t* u = ubase + ch * chunk_stride + w * UNIT;
            Codec<BITS>::load(u, lane, raw[w]);
            if (FMT == 1) {
                const AQ_GLOBAL uint8_t* bp = as_global<uint8_t>(u + aq2_sub_offset(BITS, c >> 2, 2 * g, c & 3));
                sc[w][0] = (uint32_t)bp[0] | ((uint32_t)bp[4] << 8);           // next block: 4 bytes on
                sc[w][1] = *as_global<uint32_t>(u + aq2_sup_offset(BITS, c >> 2, c & 3));
            } else {
                const AQ_GLOBAL uint16_t* sp = as_global<uint16_t>(u + 512 * BITS + ((c >> 2) * 8 + 2 * g) * 8 + (c & 3) * 2);
                sc[w][0] = sp[0];
                sc[w][1] = sp[4];
            }
        }
    };
    typename Codec<BITS>::Magic magic = Codec<BITS>::magic();
    int level_bits = 0;                               // FMT 2: this lane's entry of the table
    if (FMT == 2) level_bits = __float_as_int(cb_table[lane & 15]);
    auto unpack_to = [&](uint8_t* buf) {
        const float z = (float)(1 << (BITS - 1));
#pragma unroll
        for (int w = 0; w < 2; ++w)
#pragma unroll
            for (int b2 = 0; b2 < 2; ++b2) {
                if (FMT == 2) {
                    const float df = (float)__builtin_bit_cast(_Float16, (uint16_t)sc[w][b2]);
                    uint8_t* dst = buf + ((2 * p + w) * 16 + c) * PC_W_ROW + (2 * g + b2) * 64;
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        uint32_t o[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int e = 2 * (4 * q4 + i);            // elements e, e + 1 of the block
                            const int c0 = (int)aq_block_get(&raw[w][b2 * BITS], BITS, e);
                            const int c1 = (int)aq_block_get(&raw[w][b2 * BITS], BITS, e + 1);
                            const float l0 = __int_as_float(__builtin_amdgcn_ds_bpermute(c0 << 2, level_bits));
                            const float l1 = __int_as_float(__builtin_amdgcn_ds_bpermute(c1 << 2, level_bits));
                            const half2v h = {(_Float16)(l0 * df), (_Float16)(l1 * df)};
                            o[i] = __builtin_bit_cast(uint32_t, h);
                        }
                        *reinterpret_cast<u32x4*>(dst + 16 * q4) = u32x4{o[0], o[1], o[2], o[3]};
                    }
                    continue;
                }
                uint32_t a[16];
                Codec<BITS>::unpack(&raw[w][b2 * BITS], magic, a);         // fp16 pairs (magic + q)
                _Float16 d, off = (_Float16)0.0f;
                if (FMT == 1) {
                    const uint32_t ac = (sc[w][0] >> (8 * b2)) & 0xFFu, dm = sc[w][1];
                    d = (_Float16)((float)__builtin_bit_cast(_Float16, (uint16_t)(dm & 0xFFFFu)) * (float)(ac & 15u));
                    off = (_Float16)((float)__builtin_bit_cast(_Float16, (uint16_t)(dm >> 16)) * (float)(ac >> 4));
                } else {
                    d = __builtin_bit_cast(_Float16, (uint16_t)sc[w][b2]) * down;
                }
                uint8_t* dst = buf + ((2 * p + w) * 16 + c) * PC_W_ROW + (2 * g + b2) * 64;
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    uint32_t o[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int pidx = 4 * q4 + i;
                        const _Float16 k = (_Float16)(Codec<BITS>::offset(pidx) + (FMT ? 0.f : z));
                        const uint32_t ap = a[pidx];
                        const half2v qz = __builtin_bit_cast(half2v, ap) - half2v{k, k};      // q - z, or q itself
                        const half2v h = FMT ? __builtin_elementwise_fma(qz, half2v{d, d}, half2v{-off, -off}) : qz * half2v{d, d};
                        o[i] = __builtin_bit_cast(uint32_t, h);
                    }
                    *reinterpret_cast<u32x4*>(dst + 16 * q4) = u32x4{o[0], o[1], o[2], o[3]};
                }
            }
    };
    load_w(0);
    unpack_to(smem);
    load_w(nch > 1 ? 1 : 0);
    lds_barrier();                                    // chunk 0 is in buffer 0
#pragma unroll 1
    for (int ch = 0; ch < nch; ++ch) {
        if (ch + 1 < nch) {
            unpack_to(smem + ((ch + 1) & 1) * PC_WBUF);
            load_w(ch + 2 < nch ? ch + 2 : nch - 1);
        }
        lds_barrier();                                // chunk ch + 1 written, chunk ch read
    }
}

// BITS_T == 0: the tasks' bit-widths differ, branch per workgroup.  FMT: see produce().  KSPLIT: the instance for a
// lone product that splits K (the list kernels carry none of its code).
template <int BITS_T, int FMT, bool KSPLIT = false>
__global__ __launch_bounds__(PC_THREADS) void qgemm_pc_kernel(const AqGemmTask* __restrict__ tasks, int count,
                                                              AqGemmTask single, const uint8_t* __restrict__ workspace,
                                                              const float* __restrict__ cb_table)
{
    extern __shared__ __align__(16) uint8_t smem[];
    AqGemmTask t;
    int wg = blockIdx.x;
    if (count == 0) {
        t = single;
    } else {
        int lo = 0, hi = count - 1;
        while (lo < hi) {
            int mid = (lo + hi + 1) >> 1;
            if (tasks[mid].wg_begin <= wg) lo = mid; else hi = mid - 1;
        }
        t = tasks[lo];
        wg -= t.wg_begin;
        if (FMT == 2) cb_table += 16 * lo;            // a list carries one table of 16 levels per task
    }
    if (wg >= t.wg_count) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // a lone matrix may split K over kparts workgroups per (group, m-block): each adds its part into Y (zeroed before)
    const int kparts = KSPLIT && t.pad[1] > 1 ? (int)t.pad[1] : 1;
    const int wg_part = t.wg_count / kparts, kpart = KSPLIT ? wg / wg_part : 0;
    wg -= kpart * wg_part;
    const int group = wg % t.slabs, mblock = wg / t.slabs;
    const int cpp = (t.nchunks + kparts - 1) / kparts;
    const int ch0 = kpart * cpp;
    const int nch = KSPLIT ? (t.nchunks - ch0 < cpp ? t.nchunks - ch0 : cpp) : t.nchunks;      // this workgroup's chunks: ch0 .. ch0 + nch - 1

    // largest scale of the matrix (blob trailer) -> power-of-two shift that keeps d * (q - z) inside binary16
    // (blobs of the two-level variant carry no such word: their D * 15 * (2^bits - 1) must stay inside binary16)
    int sh = 0;
    if (FMT == 0) {
        const uint32_t max_d = *reinterpret_cast<const uint32_t*>(
            t.blob + (int64_t)t.slabs * t.nchunks * AQ_GROUP_TILES * aq_unit_bytes(t.bits));
        const int max_exp = (int)(max_d >> 10) - 15 + (t.bits - 1) + 1;
        sh = max_exp > 15 ? max_exp - 15 : 0;
    }

    if (wave >= PC_CONSUMERS) {
        const _Float16 down = (_Float16)__builtin_ldexpf(1.f, -(sh < 24 ? sh : 24));
        const int p = wave - PC_CONSUMERS;
        if (BITS_T == 2 || (BITS_T == 0 && t.bits == 2)) produce<2, FMT>(t, group, p, lane, smem, down, cb_table, ch0, nch);
        else if (BITS_T == 3 || (BITS_T == 0 && t.bits == 3)) produce<3, FMT>(t, group, p, lane, smem, down, cb_table, ch0, nch);
        else produce<4, FMT>(t, group, p, lane, smem, down, cb_table, ch0, nch);
        return;
    }

    // the consumers' MFMAs go ahead of the producers' vector-ALU work whenever both are ready to issue
    __builtin_amdgcn_s_setprio(3);

    // ---- consumer `wave`: m-tiles mt0 .. mt0 + cnt - 1 (the workgroup's T <= PC_MBLOCK tiles dealt as evenly as they go)
    const int g = lane >> 4, c = lane & 15;
    const int K = t.K, ksteps = K / AQ_BLOCK;
    const int64_t M = t.M;
    const int mtiles16 = (int)((M + 15) >> 4);
    const int per = t.pad[0] ? (int)t.pad[0] : PC_MBLOCK;       // m-tiles per workgroup (fewer than the most for a lone matrix)
    const int wg_first = mblock * per;
    const int T = mtiles16 - wg_first < per ? mtiles16 - wg_first : per;
    const int cnt = T / PC_CONSUMERS + (wave < T % PC_CONSUMERS ? 1 : 0);
    const int mt0 = wg_first + wave * (T / PC_CONSUMERS) + (wave < T % PC_CONSUMERS ? wave : T % PC_CONSUMERS);

    // The loop is compiled for a wavefront that owns PC_MT m-tiles and (PC_MT_LOW < PC_MT) for one that owns fewer: the
    // tile count is a compile-time constant of the instance a wavefront runs (chosen once, no branch in the loop), so a
    // wavefront with fewer tiles issues fewer MFMAs instead of recomputing a tile it does not own.
    auto consume = [&](auto mtc) {
        constexpr int MTC = decltype(mtc)::value;
        // X operands straight from the re-tiled copy Xt[m-tile][step][lane] (1 KiB per load), two steps ahead.  A tile
        // the wavefront does not own re-reads its first tile (or tile 0) and is never stored; a step beyond K re-reads
        // step 0 and is never used: no branches in the loop.
        const AQ_GLOBAL u32x4* xp[MTC];
#pragma unroll
        for (int mt = 0; mt < MTC; ++mt)
            xp[mt] = as_global<u32x4>(workspace + t.xt_offset) + (int64_t)(mt < cnt ? mt0 + mt : 0) * ksteps * 64 + lane;
        u32x4 xr[2][MTC];
        auto load_x = [&](int mt, int step, u32x4& dst) {
            const int st = step < ksteps ? step : 0;
            dst = xp[mt][st * 64];
        };
#pragma unroll
        for (int mt = 0; mt < MTC; ++mt) {
            load_x(mt, ch0 * 8, xr[0][mt]);
            load_x(mt, ch0 * 8 + 1, xr[1][mt]);
        }

        float4v acc[MTC][8];
#pragma unroll
        for (int mt = 0; mt < MTC; ++mt)
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) acc[mt][nt] = float4v{0.f, 0.f, 0.f, 0.f};

        // weight operand of n-tile nt, block blk: lane (g, c) = row nt*16 + c, k = 8g .. 8g+7 of the block
        const int lane_off = c * PC_W_ROW + g * 16;
        // A step is four quarters of 2 n-tiles (2 MTC MFMAs each).  Four weight operands live in registers: the two the
        // current quarter multiplies and the two of the next quarter, requested when the current one starts, so an LDS
        // read has a quarter's MFMAs to arrive.
        constexpr int NJ = AQ_PC_NJ;                      // n-tiles per batch of LDS reads
        constexpr int BPS = 8 / NJ;                       // batches per step
        u32x4 bw[2][NJ];
        lds_barrier();                                    // chunk 0 is in buffer 0
#pragma unroll 1
        for (int ch = 0; ch < nch; ++ch) {
            const uint8_t* cur = smem + (ch & 1) * PC_WBUF + lane_off;
#pragma unroll
            for (int j = 0; j < NJ; ++j) bw[0][j] = *reinterpret_cast<const u32x4*>(cur + j * 16 * PC_W_ROW);
#pragma unroll
            for (int qs = 0; qs < 8 * BPS; ++qs) {        // batches: step qs / BPS, n-tiles NJ * (qs % BPS) .. + NJ - 1
                const int s = qs / BPS, qt = qs % BPS, par = s & 1, set = qs & 1;
                if (qs < 8 * BPS - 1) {
                    const int s2 = (qs + 1) / BPS, q2 = (qs + 1) % BPS;
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        bw[set ^ 1][j] = *reinterpret_cast<const u32x4*>(cur + (NJ * q2 + j) * 16 * PC_W_ROW + s2 * 64);
                }
                __builtin_amdgcn_sched_barrier(0);        // keep the reads up here, ahead of the MFMAs they overlap with
#pragma unroll
                for (int mt = 0; mt < MTC; ++mt) {
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        acc[mt][NJ * qt + j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, xr[par][mt]),
                                                                                      __builtin_bit_cast(half8, bw[set][j]),
                                                                                      acc[mt][NJ * qt + j], 0, 0, 0);
                    // the step's last batch has used this m-tile's activation operand: request step s + 2's (from
                    // L2: as early as possible)
                    if (qt == BPS - 1) {
                        load_x(mt, (ch0 + ch) * 8 + s + 2, xr[par][mt]);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            lds_barrier();                                // chunk ch read, chunk ch + 1 written
        }

        // D[m][n]: lane (g, c) holds rows 4g .. 4g+3 of the m-tile for column c of the n-tile
        AQ_GLOBAL float* Y = (AQ_GLOBAL float*)(uintptr_t)t.Y;
        const int32_t* rowexp = reinterpret_cast<const int32_t*>(workspace + t.xt_offset + (int64_t)mtiles16 * 16 * K * 2);
#pragma unroll
        for (int mt = 0; mt < MTC; ++mt) {
            if (mt < cnt) {
                int e[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) e[r] = rowexp[(mt0 + mt) * 16 + 4 * g + r] + sh;
#pragma unroll
                for (int nt = 0; nt < 8; ++nt) {
                    const int64_t n = (int64_t)group * AQ_GROUP_ROWS + nt * 16 + c;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int64_t m = (int64_t)(mt0 + mt) * 16 + 4 * g + r;
                        if (m < M && n < t.N) {
                            const float v = ldexpf(acc[mt][nt][r], e[r]);
                            if (KSPLIT && kparts > 1) unsafeAtomicAdd((float*)(uintptr_t)(Y + m * t.ldy + n), v);
                            else Y[m * t.ldy + n] = v;
                        }
                    }
                }
            }
        }
    };
    if (cnt <= 1) consume(std::integral_constant<int, 1>{});
    else if (PC_MT_LOW < PC_MT && cnt <= PC_MT_LOW) consume(std::integral_constant<int, PC_MT_LOW>{});
    else consume(std::integral_constant<int, PC_MT>{});
}

}  // namespace


// m-tile slots the consumers of a product's workgroups compute (each runs the loop instance for PC_MT or PC_MT_LOW
// tiles), per 128-row group: against ceil(M / 16) it says how much of the matrix-core work is spent on real rows
int64_t aqk_gemm_pc_tile_slots(int64_t M, int per)
{
    const int64_t tiles = (M + 15) / 16;
    if (per <= 0 || per > PC_MBLOCK) per = PC_MBLOCK;
    int64_t slots = 0;
    for (int64_t first = 0; first < tiles; first += per) {
        const int T = (int)(tiles - first < per ? tiles - first : per);
        for (int w = 0; w < PC_CONSUMERS; ++w) {
            const int cnt = T / PC_CONSUMERS + (w < T % PC_CONSUMERS ? 1 : 0);
            slots += cnt <= 1 ? 1 : (PC_MT_LOW < PC_MT && cnt <= PC_MT_LOW) ? PC_MT_LOW : PC_MT;
        }
    }
    return slots;
}

// m-tiles per workgroup for a launch with `groups` 128-row groups in all: the most (24), unless that leaves most of the
// chip idle (a lone matrix): then 16 or 8, each workgroup unpacking the weights again
int aqk_gemm_pc_tiles_per_wg(int64_t M, int64_t groups)
{
    const int64_t tiles = (M + 15) / 16;
    for (int per = PC_MBLOCK; per > 8; per -= 8)
        if (groups * ((tiles + per - 1) / per) >= 192) return per;
    return 8;
}

// workgroups of a product: 128-row groups of W x blocks of PC_MBLOCK m-tiles of X
int aqk_gemm_pc_wg_count(int64_t N, int64_t M, int per, int* slabs)
{
    const int sl = (int)aq_num_groups(N);
    if (slabs) *slabs = sl;
    if (per <= 0 || per > PC_MBLOCK) per = PC_MBLOCK;
    return sl * (int)(((M + 15) / 16 + per - 1) / per);
}

// bits == 0: mixed bit-widths.  Xt: binary16, the re-tiled layout of the shared-role kernel.
// format: 0 the base format, 1 the two-level variant, 2 the codebook variant (cb_table: DEVICE, 16 floats per task (one
// table for `single`): the level of every stored code).
hipError_t aqk_gemm_pc(const AqGemmTask* tasks_dev, int count, const AqGemmTask& single, int bits, int format,
                       int total_wgs, const void* workspace, hipStream_t s, const float* cb_table)
{
    if (format == 2 && !cb_table) return hipErrorInvalidValue;
    const size_t lds = 2 * (size_t)PC_WBUF;
    const dim3 grid((unsigned)total_wgs), block(PC_THREADS);
    const uint8_t* ws = static_cast<const uint8_t*>(workspace);
    const bool ksplit = count == 0 && format == 0 && bits != 0 && single.pad[1] > 1;      // a lone product that splits K
#define AQ_PC(B)                                                                                                \
    do {                                                                                                        \
        auto k = format == 1 ? qgemm_pc_kernel<B, 1> : ksplit ? qgemm_pc_kernel<B ? B : 2, 0, true> : qgemm_pc_kernel<B, 0>; \
        if (aqk_allow_lds(reinterpret_cast<const void*>(k), lds) != hipSuccess) return hipErrorInvalidValue;    \
        hipLaunchKernelGGL(k, grid, block, lds, s, tasks_dev, count, single, ws, cb_table);                     \
    } while (0)
#define AQ_PC_CB(B)                                                                                             \
    do {                                                                                                        \
        auto k = qgemm_pc_kernel<B, 2>;                                                                         \
        if (aqk_allow_lds(reinterpret_cast<const void*>(k), lds) != hipSuccess) return hipErrorInvalidValue;    \
        hipLaunchKernelGGL(k, grid, block, lds, s, tasks_dev, count, single, ws, cb_table);                     \
    } while (0)
    if (format == 2) {
        if (bits == 2) AQ_PC_CB(2); else if (bits == 3) AQ_PC_CB(3); else if (bits == 4) AQ_PC_CB(4); else AQ_PC_CB(0);
        return hipGetLastError();
    }
    if (bits == 2) AQ_PC(2);
    else if (bits == 3) AQ_PC(3);
    else if (bits == 4) AQ_PC(4);
    else AQ_PC(0);
#undef AQ_PC
#undef AQ_PC_CB
    return hipGetLastError();
}
