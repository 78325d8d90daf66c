// Prefill with exact products, prefill-sized M: producer and consumer wavefronts (the role split of aq_gemm_pc.hip
// with the arithmetic of aq_gemm.hip).
//
// Y[m, n] = sum over blocks of d[n, block] * (sum_k X[m, k] (q[n, k] - z)): per block of 32 k and 16 x 16 tile one MFMA
// on exact small integers (q - z) in the activations' 16-bit type, and the fp16 block scale multiplies that block's
// sum in fp32 on the way into the accumulators; no weight is ever rounded.
//
// In the shared-role kernel (aq_gemm.hip) every wavefront unpacks, multiplies AND scales.  Here the 12 wavefronts of a
// workgroup split the roles:
//   * wavefronts 0-7 (consumers, two per SIMD) own 2 or 3 m-tiles x all 8 n-tiles each (up to 24 m-tiles = 384 rows of
//     X per workgroup; 19 tiles are dealt 3,3,3,2,2,2,2,2).  Per quarter of a 32-k step a consumer reads 2 weight
//     operands and 2 block scales from LDS (one quarter ahead), issues 4 or 6 MFMAs into temporaries and folds them
//     into the accumulators (4 multiply-adds per MFMA); its activation operands come from the re-tiled X in global
//     memory, two steps ahead.  The tile count is a compile-time constant of the loop instance a consumer runs.
//   * wavefronts 8-11 (producers, one per SIMD) own 2 of the group's 8 tiles each: load the packed units two chunks
//     ahead, unpack to (q - z), write the next chunk's tile and its block scales (as fp32) to the other LDS buffer.
// One LDS-only barrier per chunk (256 k) orders "next tile written" and "current tile read".
#include <hip/hip_runtime.h>
#include <type_traits>
#include "aq_layout.h"
#include "aq_kernels.h"
#include "aq_codec.h"

namespace {

using namespace aqdev;
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));

constexpr int PX_CONSUMERS = 8;
constexpr int PX_THREADS = (PX_CONSUMERS + 4) * 64;
constexpr int PX_MT = 3;                              // most m-tiles per consumer
constexpr int PX_MT_LOW = 2;                          // the loop instance of a consumer that owns at most this many
constexpr int PX_MBLOCK = PX_CONSUMERS * PX_MT;       // most m-tiles per workgroup
constexpr int PX_W_ROW = AQ_CHUNK_K * 2 + 32;         // LDS row stride of the weight tile: 544 B (64 j + 32: conflict-free b128 reads)
constexpr int PX_WTILE = AQ_GROUP_ROWS * PX_W_ROW;    // one chunk's tile: 128 rows
constexpr int PX_WBUF = PX_WTILE + AQ_CHUNK_BLOCKS * AQ_GROUP_ROWS * (int)sizeof(float);      // + scales [block][n]

__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <bool XBF>
__device__ __forceinline__ float4v mfma16(const u32x4& a, const u32x4& b, const float4v& c)
{
    if (XBF)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a), __builtin_bit_cast(bf8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

// Producer: tiles 2p, 2p+1 of the group, all chunks.  Executes nch + 1 barriers.
template <int BITS, bool XBF>
__device__ __forceinline__ void produce_exact(const AqGemmTask& t, int group, int p, int lane, uint8_t* smem, int ch0,
                                              int nloc)
{
    constexpr int WORDS = Codec<BITS>::WORDS;
    constexpr int UNIT = 512 * BITS + 256;
    const int g = lane >> 4, c = lane & 15;
    // the workgroup's part of K: chunks ch0 .. ch0 + nloc - 1 of the matrix's t.nchunks (all of them unless K is split)
    const int nch = nloc;
    const uint8_t* ubase = t.blob + (((int64_t)group * t.nchunks + ch0) * AQ_GROUP_TILES + 2 * p) * UNIT;
    const int64_t chunk_stride = (int64_t)AQ_GROUP_TILES * UNIT;
    uint32_t raw[2][WORDS];
    uint32_t sc[2][2];                                // scales of row c, blocks 2g and 2g + 1
    auto load_w = [&](int ch) {
#pragma unroll
        for (int w = 0; w < 2; ++w) {
            const uint8_t* u = ubase + ch * chunk_stride + w * UNIT;
            Codec<BITS>::load(u, lane, raw[w]);
            const AQ_GLOBAL uint16_t* sp = as_global<uint16_t>(u + 512 * BITS + ((c >> 2) * 8 + 2 * g) * 8 + (c & 3) * 2);
            sc[w][0] = sp[0];
            sc[w][1] = sp[4];                         // next block: 8 bytes on
        }
    };
    typename Codec<BITS>::Magic magic = Codec<BITS>::magic();
    auto unpack_to = [&](uint8_t* buf) {
        float* Sl = reinterpret_cast<float*>(buf + PX_WTILE);
#pragma unroll
        for (int w = 0; w < 2; ++w)
#pragma unroll
            for (int b2 = 0; b2 < 2; ++b2) {
                uint32_t o[16];
                unpack_exact<BITS, XBF>(&raw[w][b2 * BITS], magic, o);
                uint8_t* dst = buf + ((2 * p + w) * 16 + c) * PX_W_ROW + (2 * g + b2) * 64;
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    *reinterpret_cast<u32x4*>(dst + 16 * q4) = u32x4{o[4 * q4], o[4 * q4 + 1], o[4 * q4 + 2], o[4 * q4 + 3]};
                Sl[(2 * g + b2) * AQ_GROUP_ROWS + (2 * p + w) * 16 + c] =
                    (float)__builtin_bit_cast(_Float16, (uint16_t)sc[w][b2]);
            }
    };
    load_w(0);
    unpack_to(smem);
    load_w(nch > 1 ? 1 : 0);
    lds_barrier();                                    // chunk 0 is in buffer 0
#pragma unroll 1
    for (int ch = 0; ch < nch; ++ch) {
        if (ch + 1 < nch) {
            unpack_to(smem + ((ch + 1) & 1) * PX_WBUF);
            load_w(ch + 2 < nch ? ch + 2 : nch - 1);
        }
        lds_barrier();                                // chunk ch + 1 written, chunk ch read
    }
}

// BITS_T == 0: the tasks' bit-widths differ, branch per workgroup.  XBF: the activations are bf16.  KSPLIT: the instance
// for a lone product that splits K (the list kernels carry none of its code).
template <int BITS_T, bool XBF, bool KSPLIT = false>
__global__ __launch_bounds__(PX_THREADS) void qgemm_pcx_kernel(const AqGemmTask* __restrict__ tasks, int count,
                                                               AqGemmTask single, const uint8_t* __restrict__ workspace)
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

    if (wave >= PX_CONSUMERS) {
        const int p = wave - PX_CONSUMERS;
        if (BITS_T == 2 || (BITS_T == 0 && t.bits == 2)) produce_exact<2, XBF>(t, group, p, lane, smem, ch0, nch);
        else if (BITS_T == 3 || (BITS_T == 0 && t.bits == 3)) produce_exact<3, XBF>(t, group, p, lane, smem, ch0, nch);
        else produce_exact<4, XBF>(t, group, p, lane, smem, ch0, nch);
        return;
    }

    // the consumers' MFMAs go ahead of the producers' vector-ALU work whenever both are ready to issue
    __builtin_amdgcn_s_setprio(3);

    // ---- consumer `wave`: m-tiles mt0 .. mt0 + cnt - 1 (the workgroup's T <= PX_MBLOCK tiles dealt as evenly as they go)
    const int g = lane >> 4, c = lane & 15;
    const int K = t.K, ksteps = K / AQ_BLOCK;
    const int64_t M = t.M;
    const int mtiles16 = (int)((M + 15) >> 4);
    const int per = t.pad[0] ? (int)t.pad[0] : PX_MBLOCK;       // m-tiles per workgroup (fewer than the most for a lone matrix)
    const int wg_first = mblock * per;
    const int T = mtiles16 - wg_first < per ? mtiles16 - wg_first : per;
    const int cnt = T / PX_CONSUMERS + (wave < T % PX_CONSUMERS ? 1 : 0);
    const int mt0 = wg_first + wave * (T / PX_CONSUMERS) + (wave < T % PX_CONSUMERS ? wave : T % PX_CONSUMERS);

    auto consume = [&](auto mtc) {
        constexpr int MTC = decltype(mtc)::value;
        // X operands straight from the re-tiled copy Xt[m-tile][step][lane] (1 KiB per load), two steps ahead.  A tile
        // the wavefront does not own re-reads its first tile (or tile 0) and is never stored; a step beyond K re-reads
        // step 0 and is never used: no branches in the loop.
        const AQ_GLOBAL u32x4* xp[MTC];
#pragma unroll
        for (int mt = 0; mt < MTC; ++mt)
            xp[mt] = as_global<u32x4>(workspace + t.xt_offset) + (int64_t)(mt < cnt ? mt0 + mt : (cnt ? mt0 : 0)) * ksteps * 64 + lane;
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

        // weight operand of n-tile nt, block blk: lane (g, c) = row nt*16 + c, k = 8g .. 8g+7 of the block; its scale:
        // Sl[blk][nt*16 + c] (D[m][n]: a lane holds rows 4g .. 4g+3 of column c, so one scale serves its four values)
        const int lane_off = c * PX_W_ROW + g * 16;
        u32x4 bw[2][2];
        float sc[2][2];
        const float4v zero = {0.f, 0.f, 0.f, 0.f};
        lds_barrier();                                    // chunk 0 is in buffer 0
#pragma unroll 1
        for (int ch = 0; ch < nch; ++ch) {
            const uint8_t* cur = smem + (ch & 1) * PX_WBUF + lane_off;
            const float* Sl = reinterpret_cast<const float*>(smem + (ch & 1) * PX_WBUF + PX_WTILE) + c;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                bw[0][j] = *reinterpret_cast<const u32x4*>(cur + j * 16 * PX_W_ROW);
                sc[0][j] = Sl[j * 16];
            }
#pragma unroll
            for (int qs = 0; qs < 32; ++qs) {             // quarter-steps: step qs / 4, n-tiles 2 * (qs % 4), + 1
                const int s = qs >> 2, qt = qs & 3, par = s & 1, set = qs & 1;
                if (qs < 31) {
                    const int s2 = (qs + 1) >> 2, q2 = (qs + 1) & 3;
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        bw[set ^ 1][j] = *reinterpret_cast<const u32x4*>(cur + (2 * q2 + j) * 16 * PX_W_ROW + s2 * 64);
                        sc[set ^ 1][j] = Sl[s2 * AQ_GROUP_ROWS + (2 * q2 + j) * 16];
                    }
                }
                __builtin_amdgcn_sched_barrier(0);        // keep the reads up here, ahead of the MFMAs they overlap with
                // MFMAs of m-tile mt + 1 are issued before the products of m-tile mt are folded in: two tiles' temporaries
                // are live at a time, and a multiply-add never waits for the MFMA issued just before it
                float4v D[2][2];
                auto fold = [&](int mt, const float4v (&d)[2]) {
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        float4v& a = acc[mt][2 * qt + j];
                        const float sv = sc[set][j];
                        a[0] = fmaf(d[j][0], sv, a[0]);
                        a[1] = fmaf(d[j][1], sv, a[1]);
                        a[2] = fmaf(d[j][2], sv, a[2]);
                        a[3] = fmaf(d[j][3], sv, a[3]);
                    }
                };
#pragma unroll
                for (int mt = 0; mt < MTC; ++mt) {
#pragma unroll
                    for (int j = 0; j < 2; ++j) D[mt & 1][j] = mfma16<XBF>(xr[par][mt], bw[set][j], zero);
                    // the step's last quarter has used this m-tile's activation operand: request step s + 2's
                    if (qt == 3) load_x(mt, (ch0 + ch) * 8 + s + 2, xr[par][mt]);
                    if (mt > 0) fold(mt - 1, D[(mt - 1) & 1]);
                }
                fold(MTC - 1, D[(MTC - 1) & 1]);
            }
            lds_barrier();                                // chunk ch read, chunk ch + 1 written
        }

        // D[m][n]: lane (g, c) holds rows 4g .. 4g+3 of the m-tile for column c of the n-tile
        AQ_GLOBAL float* Y = (AQ_GLOBAL float*)(uintptr_t)t.Y;
#pragma unroll
        for (int mt = 0; mt < MTC; ++mt) {
            if (mt < cnt) {
#pragma unroll
                for (int nt = 0; nt < 8; ++nt) {
                    const int64_t n = (int64_t)group * AQ_GROUP_ROWS + nt * 16 + c;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int64_t m = (int64_t)(mt0 + mt) * 16 + 4 * g + r;
                        if (m < M && n < t.N) {
                            if (KSPLIT && kparts > 1) unsafeAtomicAdd((float*)(uintptr_t)(Y + m * t.ldy + n), acc[mt][nt][r]);
                            else Y[m * t.ldy + n] = acc[mt][nt][r];
                        }
                    }
                }
            }
        }
    };
    if (cnt <= 1) consume(std::integral_constant<int, 1>{});
    else if (cnt <= PX_MT_LOW) consume(std::integral_constant<int, PX_MT_LOW>{});
    else consume(std::integral_constant<int, PX_MT>{});
}

}  // namespace

// m-tile slots the consumers of a product's workgroups compute, per 128-row group (see aqk_gemm_pc_tile_slots)
int64_t aqk_gemm_pcx_tile_slots(int64_t M, int per)
{
    const int64_t tiles = (M + 15) / 16;
    if (per <= 0 || per > PX_MBLOCK) per = PX_MBLOCK;
    int64_t slots = 0;
    for (int64_t first = 0; first < tiles; first += per) {
        const int T = (int)(tiles - first < per ? tiles - first : per);
        for (int w = 0; w < PX_CONSUMERS; ++w) {
            const int cnt = T / PX_CONSUMERS + (w < T % PX_CONSUMERS ? 1 : 0);
            slots += cnt <= 1 ? 1 : cnt <= PX_MT_LOW ? PX_MT_LOW : PX_MT;
        }
    }
    return slots;
}

// workgroups of a product: 128-row groups of W x blocks of PX_MBLOCK m-tiles of X
int aqk_gemm_pcx_wg_count(int64_t N, int64_t M, int per, int* slabs)
{
    const int sl = (int)aq_num_groups(N);
    if (slabs) *slabs = sl;
    if (per <= 0 || per > PX_MBLOCK) per = PX_MBLOCK;
    return sl * (int)(((M + 15) / 16 + per - 1) / per);
}

// bits == 0: mixed bit-widths.  Xt: the activations as given (binary16 or bf16), the re-tiled layout of aq_gemm.hip.
hipError_t aqk_gemm_pcx(const AqGemmTask* tasks_dev, int count, const AqGemmTask& single, int bits, int x_dtype,
                        int total_wgs, const void* workspace, hipStream_t s)
{
    const size_t lds = 2 * (size_t)PX_WBUF;
    const dim3 grid((unsigned)total_wgs), block(PX_THREADS);
    const uint8_t* ws = static_cast<const uint8_t*>(workspace);
    const bool ksplit = count == 0 && bits != 0 && single.pad[1] > 1;      // a lone product that splits K
#define AQ_PX(B)                                                                                                \
    do {                                                                                                        \
        auto k = ksplit ? (x_dtype == 2 ? qgemm_pcx_kernel<B ? B : 2, true, true> : qgemm_pcx_kernel<B ? B : 2, false, true>) \
                        : (x_dtype == 2 ? qgemm_pcx_kernel<B, true> : qgemm_pcx_kernel<B, false>);              \
        if (aqk_allow_lds(reinterpret_cast<const void*>(k), lds) != hipSuccess) return hipErrorInvalidValue;    \
        hipLaunchKernelGGL(k, grid, block, lds, s, tasks_dev, count, single, ws);                               \
    } while (0)
    if (bits == 2) AQ_PX(2);
    else if (bits == 3) AQ_PX(3);
    else if (bits == 4) AQ_PX(4);
    else AQ_PX(0);
#undef AQ_PX
    return hipGetLastError();
}
