// One stage of the layer-by-layer decode step: y += W f(in) for the matrices of a stage that share their input
// (q/k/v; o; gate/up; down), M = 1.  A decode step through a transformer block is four such stages, each
// depending on the one before; a stage moves only 7-40 MB of weights (1-5 us of HBM time), so a stage is
// latency-bound and the kernel is built to have ALL of its bytes in flight at once:
//
//  * split K: a workgroup owns 128 rows x `part_chunks` chunks (of 256 k) of one matrix; with 2 chunks its
//    4 wavefronts x 2 tiles have every unit they will ever need in their register rings before the first MFMA.
//    Partial sums are added to y with hardware fp32 atomics; y is the residual stream itself for o and
//    down (x += W a), and a zeroed buffer for the others.
//  * what sits between the matrices runs while x is staged into LDS (each workgroup stages only its own
//    k-range): RMSNorm (every workgroup sums x^2 over the whole vector, L2-resident, and applies the norm
//    multipliers), the gate: act(gate) * up, or the copy of the value head a query head reads.  No
//    stand-alone elementwise kernels, no extra launches.
//  * the staged vector is binary16 times a power of two chosen per workgroup from its largest magnitude
//    (11 significant bits; the matrix cores take 16-bit inputs); the arithmetic on the weights is the decode
//    kernel's: exact integers on the matrix cores, block scales in fp32.
//  * vector-memory loads return in order within a wavefront: the input loads are issued BEFORE the weight
//    loads, so staging waits for the (L2-resident) inputs only while the weights stream in behind.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "aq_layout.h"
#include "aq_kernels.h"
#include "aq_codec.h"
#include "aq_gemv_core.h"

namespace {

using namespace aqdev;

constexpr int WAVES = 4;
constexpr int THREADS = WAVES * 64;
constexpr int TW = 2;                                   // tiles per wavefront: a workgroup covers a whole group
constexpr int XL_BYTES = AQ_STAGE_MAX_PART * 4 * X_PAIR_BYTES;

// orders LDS traffic only (a __syncthreads() would also drain the weight loads in flight)
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ float act_fn(int act, float a)
{
    if (act == 0) return a / (1.f + __expf(-a));                                  // SiLU
    const float u = 0.7978845608028654f * (a + 0.044715f * a * a * a);           // tanh form of GELU
    return 0.5f * a * (1.f + tanhf(u));
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

// The first two chunks of an item (workgroup `wg` of task `t`) into this wavefront's ring.
template <int BITS>
__device__ __forceinline__ void ring_fill(const AqStageTask& t, int wg, int wave, int lane, uint32_t (&raw)[2 * TW][8],
                                          u32x2 (&sc)[2 * TW])
{
    constexpr int UNIT = 512 * BITS + 256;
    const int group = wg / t.parts, part = wg % t.parts;
    const int c0 = part * t.part_chunks;
    const int np = (t.nchunks - c0 < t.part_chunks) ? t.nchunks - c0 : t.part_chunks;
    const int g = lane >> 4, c = lane & 15;
    const uint8_t* ubase = t.blob + (((int64_t)group * t.nchunks + c0) * AQ_GROUP_TILES + wave * TW) * UNIT;
    const int64_t chunk_stride = (int64_t)AQ_GROUP_TILES * UNIT;
    const int sc_off = 512 * BITS + (g * 8 + (c & 7)) * 8;
#pragma unroll
    for (int p = 0; p < 2; ++p)
        if (p < np) {
#pragma unroll
            for (int tw = 0; tw < TW; ++tw) {
                const uint8_t* u = ubase + p * chunk_stride + tw * UNIT;
                Codec<BITS>::load(u, lane, *reinterpret_cast<uint32_t(*)[Codec<BITS>::WORDS]>(&raw[p * TW + tw]));
                sc[p * TW + tw] = __builtin_nontemporal_load(as_global<u32x2>(u + sc_off));
            }
        }
}

__global__ __launch_bounds__(THREADS, 3)
void layer_stage_kernel(const AqStageArgs args)
{
    __shared__ __align__(16) uint8_t smem[XL_BYTES + AQ_STAGE_MAX_PART * 32 + 192 + 32];
    // clear the buffer a later stage accumulates into
    for (int i = blockIdx.x * THREADS + threadIdx.x; i < args.zero_count; i += gridDim.x * THREADS)
        args.zero_ptr[i] = 0.f;

    // this workgroup's matrix: the records arrive as kernel arguments, so one round of scalar loads brings all
    // of them (a table in device memory costs a chain of dependent loads before the first weight load)
    int wg = blockIdx.x;
    AqStageTask t = args.task[0];
    if (args.count > 1 && wg >= args.task[1].wg_begin) t = args.task[1];
    if (args.count > 2 && wg >= args.task[2].wg_begin) t = args.task[2];
    wg -= t.wg_begin;
    if (wg >= t.wg_count) return;

    uint32_t raw[2 * TW][8];
    u32x2 sc[2 * TW];
    // keep the input loads (first half of the body) ahead of the weight loads: loads return in order, and an
    // input load issued behind the weights would be waited for as long as for the weights themselves
    if (t.bits == 2) {
        constexpr int BITS = 2;
#include "aq_layer_body_a.inc"
        __builtin_amdgcn_sched_barrier(0);
        ring_fill<BITS>(t, wg, wave, lane, raw, sc);
#include "aq_layer_body_b.inc"
    } else if (t.bits == 3) {
        constexpr int BITS = 3;
#include "aq_layer_body_a.inc"
        __builtin_amdgcn_sched_barrier(0);
        ring_fill<BITS>(t, wg, wave, lane, raw, sc);
#include "aq_layer_body_b.inc"
    } else {
        constexpr int BITS = 4;
#include "aq_layer_body_a.inc"
        __builtin_amdgcn_sched_barrier(0);
        ring_fill<BITS>(t, wg, wave, lane, raw, sc);
#include "aq_layer_body_b.inc"
    }
}

__global__ void fill_zero_kernel(float* p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = 0.f;
}

}  // namespace

hipError_t aqk_layer_stage(const AqStageArgs& args, int total_wgs, hipStream_t s)
{
    if (args.count < 1 || args.count > AQ_STAGE_MAX_TASKS || total_wgs < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(layer_stage_kernel, dim3((unsigned)total_wgs), dim3(THREADS), 0, s, args);
    return hipGetLastError();
}

hipError_t aqk_fill_zero(float* p, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, n);
    return hipGetLastError();
}
