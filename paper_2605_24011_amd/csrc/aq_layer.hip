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
#include <cstddef>
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

__device__ __forceinline__ void ring_fill_any(const AqStageTask& t, int wg, int wave, int lane,
                                              uint32_t (&raw)[2 * TW][8], u32x2 (&sc)[2 * TW])
{
    if (t.bits == 2) ring_fill<2>(t, wg, wave, lane, raw, sc);
    else if (t.bits == 3) ring_fill<3>(t, wg, wave, lane, raw, sc);
    else ring_fill<4>(t, wg, wave, lane, raw, sc);
}

// ---- one launch per stage ------------------------------------------------------------------------------------
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

// ---- one launch per step -------------------------------------------------------------------------------------
// All stages of all layers in one grid whose workgroups are all resident at once: workgroup b runs item b of
// every stage (stages are split into at most gridDim.x items) and the stages are separated by a grid-wide barrier
// (a counter in device memory).  What this buys over one launch per stage: no launch gap, and the weights of the
// NEXT stage's item -- which depend on nothing -- are requested as soon as the ring is free, so they stream in
// while the partial sums of this stage settle, the barrier is crossed and the next input is staged.
//
// The barrier: every thread makes its atomics and stores visible device-wide (release fence), the workgroup meets,
// one thread counts the workgroup in; one thread polls the counter (bounded: after `spin_limit` polls it raises
// the give-up flag, which every other poller also watches), the workgroup meets again and every thread drops its
// stale cache lines (acquire fence) before it reads what other workgroups wrote.  After a give-up no barrier
// waits any more, every workgroup still runs to the end (all addresses are fixed by the plan), and x is
// overwritten with NaN so that the failure cannot pass for a result.
__device__ __forceinline__ void grid_arrive(unsigned* bar)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __builtin_amdgcn_s_barrier();
    if (threadIdx.x == 0) __hip_atomic_fetch_add(bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void grid_wait(unsigned* bar, unsigned target, int spin_limit)
{
    if (threadIdx.x == 0) {
        int spins = 0;
        while (__hip_atomic_load(bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (__hip_atomic_load(bar + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
            if (++spins > spin_limit) {
                __hip_atomic_store(bar + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(2);
        }
    }
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

// Plan records are the same for every lane.  Inside the stage loop the compiler has to assume that the
// atomics and fences may have changed them and would keep them in vector registers (24 per task record); read
// them once per wavefront and move them to scalar registers by hand.
__device__ __forceinline__ int uniform_word(const void* p, int index)
{
    return __builtin_amdgcn_readfirstlane(reinterpret_cast<const int*>(p)[index]);
}

__device__ __forceinline__ const void* uniform_ptr(const void* p, int index)
{
    const uint64_t lo = (uint32_t)uniform_word(p, index), hi = (uint32_t)uniform_word(p, index + 1);
    return reinterpret_cast<const void*>((hi << 32) | lo);
}

static_assert(offsetof(AqStageTask, N) == 32 && offsetof(AqStageTask, eps) == 80, "uniform_task reads by word index");
__device__ __forceinline__ AqStageTask uniform_task(const AqStageTask* p)
{
    AqStageTask t;
    t.blob = static_cast<const uint8_t*>(uniform_ptr(p, 0));
    t.y = static_cast<float*>(const_cast<void*>(uniform_ptr(p, 2)));
    t.in0 = static_cast<const float*>(uniform_ptr(p, 4));
    t.in1 = static_cast<const float*>(uniform_ptr(p, 6));
    t.N = uniform_word(p, 8);
    t.K = uniform_word(p, 9);
    t.bits = uniform_word(p, 10);
    t.nchunks = uniform_word(p, 11);
    t.part_chunks = uniform_word(p, 12);
    t.parts = uniform_word(p, 13);
    t.wg_begin = uniform_word(p, 14);
    t.wg_count = uniform_word(p, 15);
    t.prologue = uniform_word(p, 16);
    t.act = uniform_word(p, 17);
    t.head_dim = uniform_word(p, 18);
    t.rep = uniform_word(p, 19);
    t.eps = __int_as_float(uniform_word(p, 20));
    t.pad0 = 0;
    t.pad1 = 0;
    return t;
}

// index of the task record of workgroup b's item in stage `st` (-1: the stage has fewer items than b + 1)
__device__ __forceinline__ int find_task(const AqStageTask* tasks, const AqStageEntry* st, int b)
{
    const int task_begin = uniform_word(st, 0), task_count = uniform_word(st, 1), total = uniform_word(st, 2);
    if (b >= total) return -1;
    constexpr int WG_BEGIN = offsetof(AqStageTask, wg_begin) / 4;
    int ti = task_begin;
    if (task_count > 1 && b >= uniform_word(tasks + task_begin + 1, WG_BEGIN)) ti = task_begin + 1;
    if (task_count > 2 && b >= uniform_word(tasks + task_begin + 2, WG_BEGIN)) ti = task_begin + 2;
    return ti;
}

__global__ __launch_bounds__(THREADS, 3)
void decode_step_kernel(const AqStageTask* tasks, const AqStageEntry* stages, int nstages,
                        unsigned* bar, float* gateup, int gateup_floats, float* x, int d_model, int spin_limit)
{
    __shared__ __align__(16) uint8_t smem[XL_BYTES + AQ_STAGE_MAX_PART * 32 + 192 + 32];
    const int b = blockIdx.x;
    const unsigned G = gridDim.x;
    const int wave0 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane0 = threadIdx.x & 63;

    uint32_t raw[2 * TW][8] = {};
    u32x2 sc[2 * TW] = {};
    AqStageTask t = {};
    int wg = 0;
    int ti = find_task(tasks, stages, b);
    if (ti >= 0) {
        t = uniform_task(tasks + ti);
        wg = b - t.wg_begin;
        ring_fill_any(t, wg, wave0, lane0, raw, sc);
    }

#pragma unroll 1
    for (int s = 0; s < nstages; ++s) {
        if (s > 0) grid_wait(bar, (unsigned)s * G, spin_limit);
        // find the next item's record now: two dependent reads that are over long before the ring is free
        const int tin = (s + 1 < nstages) ? find_task(tasks, stages + s + 1, b) : -1;
        const bool clears = uniform_word(stages + s, 3) != 0;
        if (ti >= 0) {
            if (t.bits == 2) {
                constexpr int BITS = 2;
#include "aq_layer_body_a.inc"
#include "aq_layer_body_b.inc"
            } else if (t.bits == 3) {
                constexpr int BITS = 3;
#include "aq_layer_body_a.inc"
#include "aq_layer_body_b.inc"
            } else {
                constexpr int BITS = 4;
#include "aq_layer_body_a.inc"
#include "aq_layer_body_b.inc"
            }
        }
        if (clears)
            for (int i = b * THREADS + threadIdx.x; i < gateup_floats; i += (int)G * THREADS) gateup[i] = 0.f;
        // the ring is spent: say so, or the words the bit-width just run does not use stay live through its body
#pragma unroll
        for (int r = 0; r < 2 * TW; ++r) {
#pragma unroll
            for (int w = 0; w < 8; ++w) raw[r][w] = 0u;
            sc[r] = u32x2{0u, 0u};
        }
        grid_arrive(bar);
        ti = tin;
        if (ti >= 0) {
            t = uniform_task(tasks + ti);
            wg = b - t.wg_begin;
            ring_fill_any(t, wg, wave0, lane0, raw, sc);
        }
    }
    // a barrier gave up: the numbers in x mean nothing
    if (b == 0) {
        __builtin_amdgcn_s_barrier();
        if (__hip_atomic_load(bar + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)
            for (int i = threadIdx.x; i < d_model; i += THREADS) x[i] = __uint_as_float(0x7FC00000u);
    }
}

__global__ void fill_zero_kernel(float* p, int64_t n, uint32_t* q, int m)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = 0.f;
    if (blockIdx.x == 0 && (int)threadIdx.x < m) q[threadIdx.x] = 0u;
}

}  // namespace

hipError_t aqk_layer_stage(const AqStageArgs& args, int total_wgs, hipStream_t s)
{
    if (args.count < 1 || args.count > AQ_STAGE_MAX_TASKS || total_wgs < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(layer_stage_kernel, dim3((unsigned)total_wgs), dim3(THREADS), 0, s, args);
    return hipGetLastError();
}

// workgroups of decode_step_kernel that the current device holds at once (0 if it cannot be asked)
int aqk_decode_step_capacity()
{
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_step_kernel, THREADS, 0) != hipSuccess) return 0;
    return cus * per_cu;
}

hipError_t aqk_decode_step(const AqStageTask* tasks_dev, const AqStageEntry* stages_dev, int nstages, int grid,
                           uint32_t* bar, float* gateup, int gateup_floats, float* x, int d_model, int spin_limit,
                           hipStream_t s)
{
    if (nstages < 1 || grid < 1) return hipErrorInvalidValue;
    void* params[] = {(void*)&tasks_dev, (void*)&stages_dev, (void*)&nstages, (void*)&bar, (void*)&gateup,
                      (void*)&gateup_floats, (void*)&x, (void*)&d_model, (void*)&spin_limit};
    // cooperative: the runtime refuses the launch unless every workgroup can be resident at once
    return hipLaunchCooperativeKernel(reinterpret_cast<const void*>(decode_step_kernel), dim3((unsigned)grid),
                                      dim3(THREADS), params, 0, s);
}

// clears p[0 .. n) and the first m (<= 256) words at q
hipError_t aqk_fill_zero(float* p, int64_t n, uint32_t* q, int m, hipStream_t s)
{
    if (n < 0 || m < 0 || m > 256) return hipErrorInvalidValue;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, n, q, m);
    return hipGetLastError();
}
