// Internal launch interface between the C-ABI shim (aq_api.hip) and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <map>
#include <mutex>
#include <utility>

// One decode product y = x W^T as the kernels see it (device-visible, 64 bytes).
struct AqGemvTask {
    const uint8_t* blob;
    const uint16_t* x;
    float* y;
    int64_t N;
    int32_t K;
    int32_t bits;
    int32_t x_dtype;
    int32_t nchunks;    // ceil(K / 256)
    int32_t wg_begin;   // first workgroup of this task inside a batched launch
    int32_t wg_count;
    int64_t pad;
};
static_assert(sizeof(AqGemvTask) == 64, "AqGemvTask must stay 64 bytes");

// A decode product of the non-uniform codebook variant (device-visible, 192 bytes): the base record, then how the
// table reaches the matrix cores.  form 1 (native): the stored nibbles are fp4 bit patterns and alpha scales the
// result; form 0 (planes): coef[S] is the coefficient of the monomial of the code bits in S (coef[0]: the constant
// term); form 2 (signed planes): the top bit of a stored code is the sign and coef[S] expands the magnitude table over
// the lower bits; alpha is 1 for both plane forms.
struct AqCbTask {
    AqGemvTask g;
    float coef[16];
    float alpha;
    int32_t form;
    int32_t pad[14];
};
static_assert(sizeof(AqCbTask) == 192, "AqCbTask must stay 192 bytes");

// Kernels that need more than the default 64 KiB of dynamic LDS must be told so once per device and kernel.  This
// remembers what has been granted, so that the launch path makes the runtime call the first time only.
inline hipError_t aqk_allow_lds(const void* kernel, size_t lds)
{
    if (lds <= 64 * 1024) return hipSuccess;
    static std::mutex mu;
    static std::map<std::pair<int, const void*>, size_t> granted;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    size_t& have = granted[std::make_pair(dev, kernel)];
    if (have >= lds) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) have = lds;
    return e;
}

hipError_t aqk_pack(const uint8_t* codes, const uint16_t* scales, int64_t N, int64_t K, int bits,
                    void* blob, hipStream_t s);
hipError_t aqk_unpack_codes(const void* blob, int64_t N, int64_t K, int bits, uint8_t* out, hipStream_t s);
hipError_t aqk_dequant(const void* blob, int64_t N, int64_t K, int bits, float* out, hipStream_t s);

// Decode launches.  aqk_gemv_shape sets a task's wg_count:
//   batched == true : workgroups of 4 wavefronts x 2 tiles = one 128-row group each
//   batched == false: a lone matrix; bits 2 and 4: one tile per workgroup, its 4 wavefronts split K
void aqk_gemv_shape(AqGemvTask& t, bool batched);
// count == 0: run `single` (shaped with batched == false); else `count` tasks from device memory (shaped with
// batched == true), `total_wgs` workgroups, wg_task (device) = the index of the task of every workgroup.
// bits: the common bit-width of the tasks, 0 if they differ.  max_K: over the tasks.
hipError_t aqk_gemv(const AqGemvTask* tasks_dev, const int32_t* wg_task, int count, const AqGemvTask& single, int bits,
                    int total_wgs, int max_K, hipStream_t s);

// Two-level variant of the format (layout in aq_layout.h): same contracts as the three functions and the decode
// launcher above, other blobs.
// ---- non-uniform codebook variant (aq_gemv_cb.hip; blobs in the base layout) ----
// remap: sixteen nibbles, stored code of canonical code q = (remap >> 4q) & 15 (identity: 0xFEDCBA9876543210)
hipError_t aqk_pack_remap(const uint8_t* codes, const uint16_t* scales, int64_t N, int64_t K, int bits, uint64_t remap,
                          void* blob, hipStream_t s);
struct AqCbTable { float level[16]; };      // level of every STORED code
hipError_t aqk_cb_unpack_codes(const void* blob, int64_t N, int64_t K, int bits, uint64_t inverse_remap, uint8_t* out,
                               hipStream_t s);
hipError_t aqk_cb_dequant(const void* blob, int64_t N, int64_t K, int bits, const AqCbTable& stored_levels, float* out,
                          hipStream_t s);
// the table of a codebook blob (host analysis, aq_api_cb.hip): the level of every STORED code; AQ_* status
int aqk_cb_stored_levels(const float* levels, int bits, AqCbTable* out);
hipError_t aqk_cb_write_table(const AqCbTable& table, float* dst, hipStream_t s);      // 16 floats to device memory
void aqk_cb_gemv_shape(AqCbTask& t);
bool aqk_cb_light(int form, int bits);
hipError_t aqk_cb_gemv(const AqCbTask* tasks_dev, const int32_t* wg_task, int count, const AqCbTask& single, int mode,
                       int total_wgs, int max_K, hipStream_t s);      // mode: 4 * form + bits for a uniform launch; mixed: 1 if aqk_cb_light holds for every task, else 0

hipError_t aqk2_pack(const uint8_t* codes, const uint8_t* sub, const uint16_t* sup, int64_t N, int64_t K, int bits,
                     void* blob, hipStream_t s);
hipError_t aqk2_unpack_codes(const void* blob, int64_t N, int64_t K, int bits, uint8_t* out, hipStream_t s);
hipError_t aqk2_dequant(const void* blob, int64_t N, int64_t K, int bits, float* out, hipStream_t s);
hipError_t aqk2_gemv(const AqGemvTask* tasks_dev, const int32_t* wg_task, int count, const AqGemvTask& single, int bits,
                     int total_wgs, int max_K, hipStream_t s);

// Prefill.  The activations are first re-tiled into the order the matrix cores read them ("Xt"):
//   Xt[m / 16][k / 32][lane = 16*g + c] = the 16 bytes X[16*(m/16) + c][32*(k/32) + 8g .. 8g+7],
// rows beyond M zero, so that a wavefront's A operand of one (m-tile, 32-k step) is 1 KiB contiguous.
// Xt lives in the caller's workspace at `xt_offset`, followed by one int32 per padded row ("rowexp");
// several products may share one Xt.  convert == 0: the elements are copied, rowexp = 0.
// convert == 1 (bf16 input of the fp16-weight mode): row m is multiplied by 2^-rowexp[m], the power of
// two that puts its largest magnitude in [2^14, 2^15), and written as binary16 (exact unless an element
// is more than 2^38 times smaller than the row's largest); the product kernel scales row m of Y back.
struct AqRetileTask {
    const uint16_t* X;
    int64_t M, ldx;
    int64_t xt_offset;  // bytes from the workspace base, multiple of 1024
    int32_t K;
    int32_t blocks;     // workgroups of 256 threads (aqk_retile_blocks)
    int32_t convert;
    int32_t pad;        // small-M layout: m-tiles of the launch (1, 2, 4); else 0
};
static_assert(sizeof(AqRetileTask) == 48, "AqRetileTask must stay 48 bytes");

// One prefill product Y = X W^T as the kernel sees it (device-visible, 96 bytes).
struct AqGemmTask {
    const uint8_t* blob;
    float* Y;
    int64_t N, M, ldy;
    int64_t xt_offset;  // this product's Xt, bytes from the workspace base
    int32_t K;
    int32_t bits;
    int32_t nchunks;    // ceil(K / 256)
    int32_t slabs;      // 128-row groups of W
    int32_t wg_begin;   // first workgroup of this task inside a batched launch
    int32_t wg_count;   // slabs * m-tiles
    int64_t pad[3];
};
static_assert(sizeof(AqGemmTask) == 96, "AqGemmTask must stay 96 bytes");

int aqk_gemm_mtiles(int64_t M, int64_t groups);   // groups = 128-row groups over all products of the launch
int aqk_gemm_nsplit(int64_t M);
int aqk_gemm_wg_count(int64_t N, int64_t M, int A, int nsplit, int* slabs);
size_t aqk_retile_bytes(int64_t M, int64_t K);
int aqk_retile_blocks(int64_t M, int64_t K, int convert);
// count == 0: run `single`; else `count` tasks from device memory; grid = (max_blocks, tasks); every task
// of a launch has the same `convert`.  zero_Y (lone products, count == 0, only): rows [0, single.M) x columns [0, zero_N)
// of that matrix (row stride zero_ldy) are cleared by the same launch
hipError_t aqk_retile(const AqRetileTask* tasks_dev, int count, const AqRetileTask& single, int max_blocks,
                      int convert, void* workspace, hipStream_t s, float* zero_Y = nullptr, int64_t zero_N = 0,
                      int64_t zero_ldy = 0);
// count == 0: run `single`; bits == 0: the tasks' bit-widths differ; x_dtype, A, nsplit and fast are per
// launch.  fast != 0: weights are formed as binary16 d * (q - z) and the activations in Xt are binary16.
hipError_t aqk_gemm(const AqGemmTask* tasks_dev, int count, const AqGemmTask& single, int bits, int x_dtype, int A,
                    int nsplit, int fast, int total_wgs, const void* workspace, hipStream_t s);

// Block-level scale optimisation: fp32 W, F (F may be null = all ones) -> canonical codes + fp16 scales
hipError_t aqk_optimize_scales(const float* W, const float* F, int64_t N, int64_t K, int bits, int rounds,
                               uint8_t* codes, uint16_t* scales, hipStream_t s);

// Prefill for M <= 64 in the fp16-weight mode: streaming kernel, its own X layout ("Xs")
int aqk_small_mtiles(int64_t M);
size_t aqk_small_retile_bytes(int64_t M, int64_t K);
hipError_t aqk_small_retile(const AqRetileTask* tasks_dev, int count, const AqRetileTask& single, int MT, int bf16,
                            void* workspace, hipStream_t s);
hipError_t aqk_gemm_small(const AqGemmTask* tasks_dev, int count, const AqGemmTask& single, int bits, int MT,
                          bool split, int total_wgs, const void* workspace, hipStream_t s);

// Prefill, fp16-weight mode, prefill-sized M: producer / consumer wavefronts (aq_gemm_pc.hip).  Reads the binary16
// Xt + rowexp that aqk_retile writes; a task's wg_count = aqk_gemm_pc_wg_count (128-row groups x blocks of 320 rows).
// per = m-tiles per workgroup (0: the most, 24), carried by a task in pad[0]; both producer / consumer kernels alike.
// pad[1] = kparts (0 or 1: none): K split over that many workgroups per (group, m-block), wg_count multiplied by it, the
// parts ADDED into Y with fp32 atomics (the caller zeroes Y first; two parts give the same sum in either order)
int aqk_gemm_pc_tiles_per_wg(int64_t M, int64_t groups);   // groups = 128-row groups over all products of the launch
int aqk_gemm_pc_wg_count(int64_t N, int64_t M, int per, int* slabs);
int64_t aqk_gemm_pc_tile_slots(int64_t M, int per);
// exact products, producer / consumer wavefronts (aq_gemm_pcx.hip); tasks as for aqk_gemm_pc with the counts below
int64_t aqk_gemm_pcx_tile_slots(int64_t M, int per);
int aqk_gemm_pcx_wg_count(int64_t N, int64_t M, int per, int* slabs);
hipError_t aqk_gemm_pcx(const AqGemmTask* tasks_dev, int count, const AqGemmTask& single, int bits, int x_dtype,
                        int total_wgs, const void* workspace, hipStream_t s);
// exact products for blobs of the two-level variant (aq_gemm2.hip); tasks as for aqk_gemm with nsplit = 1, X re-tiled
// without conversion
hipError_t aqk2_gemm(const AqGemmTask* tasks_dev, int count, const AqGemmTask& single, int x_dtype, int A,
                     int total_wgs, const void* workspace, hipStream_t s);
hipError_t aqk_gemm_pc(const AqGemmTask* tasks_dev, int count, const AqGemmTask& single, int bits, int format,
                       int total_wgs, const void* workspace, hipStream_t s, const float* cb_table = nullptr);

// Layer-by-layer decode step.  One matrix of one stage as the kernel sees it (device-visible, 96 bytes):
// y[n] += sum over the k of a workgroup's part of W[n][k] * f(in)[k], with f chosen by `prologue`:
//   AQ_PRO_PLAIN  f(in)[k] = in0[src(k)], src(k) = ((k / head_dim) / rep) * head_dim + k % head_dim
//                 (rep query heads read one value head; rep = 1: src(k) = k)
//   AQ_PRO_NORM   f(in)[k] = in0[k] / sqrt(mean(in0^2) + eps) * in1[k]         (in0 has K elements)
//   AQ_PRO_GATED  f(in)[k] = act(in0[k]) * in1[k]                              (act 0: SiLU, 1: tanh-GELU)
#define AQ_PRO_PLAIN 0
#define AQ_PRO_NORM  1
#define AQ_PRO_GATED 2
#define AQ_STAGE_MAX_PART 8      // chunks of 256 k per workgroup at most (sets the kernel's LDS)
struct AqStageTask {
    const uint8_t* blob;
    float* y;
    const float* in0;
    const float* in1;
    int32_t N, K;
    int32_t bits, nchunks;
    int32_t part_chunks, parts;   // parts = ceil(nchunks / part_chunks), 1 <= part_chunks <= AQ_STAGE_MAX_PART
    int32_t wg_begin, wg_count;   // wg_count = groups of 128 rows * parts
    int32_t prologue, act;
    int32_t head_dim, rep;
    float eps;
    int32_t pad0;
    int64_t pad1;
};
static_assert(sizeof(AqStageTask) == 96, "AqStageTask must stay 96 bytes");

// One stage = one launch: up to AQ_STAGE_MAX_TASKS matrices that share their input, passed BY VALUE as the
// kernel argument, and a buffer the launch clears (one that a LATER stage accumulates into; zero_count may be 0).
#define AQ_STAGE_MAX_TASKS 3
struct AqStageArgs {
    AqStageTask task[AQ_STAGE_MAX_TASKS];
    float* zero_ptr;
    int32_t zero_count;
    int32_t count;
};
hipError_t aqk_layer_stage(const AqStageArgs& args, int total_wgs, hipStream_t s);

hipError_t aqk_fill_zero(float* p, int64_t n, hipStream_t s);

// HSIC sensitivity (aq_hsic.hip).  aqk_rbf_gram: G (K x K) from the K rows of A, sq = K floats of scratch;
// aqk_rowsum: fp64 row sums of a Gram matrix; aqk_hsic_pair: acc[0..3] (zeroed before) += sum GA.GB, sum a_i b_i,
// sum a_i, sum b_i; aqk_hsic_finish: out[p] = HSIC of pair p from acc + 4 p (and Eq. 5's combination for 2 pairs).
hipError_t aqk_rbf_gram(const float* A, int64_t K, int64_t d, int64_t lda, float gamma, float* G, float* sq, hipStream_t s);
hipError_t aqk_rowsum(const float* G, int64_t K, double* rs, hipStream_t s);
hipError_t aqk_zero_f64(double* p, int n, hipStream_t s);
hipError_t aqk_hsic_pair(const float* GA, const float* GB, int64_t K, const double* ra, const double* rb, double* acc,
                         hipStream_t s);
hipError_t aqk_hsic_finish(const double* acc, int pairs, int64_t K, double alpha, double beta, double* out, hipStream_t s);
