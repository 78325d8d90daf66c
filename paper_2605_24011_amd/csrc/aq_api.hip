// C-ABI shim: host-side argument validation and dispatch.  Nothing here touches the GPU
// before every argument has been checked, so the error paths can be tested on a machine
// without one.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>
#include "../../include/aq.h"
#include "aq_layout.h"
#include "aq_kernels.h"

namespace {

constexpr int64_t AQ_MAX_K = 65536;          // no kernel's LDS or registers grow with K: a bound on index arithmetic
constexpr int64_t AQ_LAYER_MAX_K = 16384;    // the decode step's stage planner (parts of at most 8 chunks, one round of workgroups)
constexpr int64_t AQ_MAX_N = (int64_t)1 << 24;
constexpr int64_t AQ_MAX_M = (int64_t)1 << 20;

// First 64 bytes of a batch plan image; the task records follow in the caller's order.
struct PlanHeader {
    uint32_t magic;
    int32_t count;
    int32_t tiles_per_wg;
    int32_t max_K;
    int32_t bits;            // the common bit-width of all tasks, 0 if they differ
    int32_t total_wgs;
    int32_t format;          // 0: base format, 1: two-level variant
    int32_t reserved[9];
};
static_assert(sizeof(PlanHeader) == 64, "PlanHeader must stay 64 bytes");
constexpr uint32_t PLAN_MAGIC = 0x41515034u;  // "AQP4"

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_matrix(int64_t N, int64_t K, int bits, int block)
{
    if (bits != 2 && bits != 3 && bits != 4) return AQ_EINVAL;
    if (block != AQ_BLOCK) return AQ_EINVAL;
    if (N < 1 || K < 1 || N > AQ_MAX_N || K > AQ_MAX_K) return AQ_EINVAL;
    if (K % AQ_BLOCK != 0) return AQ_EINVAL;
    return AQ_OK;
}

int check_dtype(int dt) { return (dt == AQ_F16 || dt == AQ_BF16) ? AQ_OK : AQ_EDTYPE; }

struct GemmPlanHeader {
    uint32_t magic;
    int32_t count;
    int32_t bits;            // the common bit-width, 0 if the tasks differ
    int32_t x_dtype;
    int32_t mtiles;          // m-tiles per wavefront, from the largest M
    int32_t total_wgs;
    int32_t retile_count;    // distinct activation matrices
    int32_t retile_max_blocks;
    int64_t workspace_bytes;
    int32_t nsplit;          // wavefronts along n, from the largest M
    int32_t fast;            // fp16-weight mode
    int32_t small_mt;        // > 0: the small-M streaming kernel with that many m-tiles (fast mode, M <= 64)
    int32_t pc;              // a producer / consumer kernel (prefill-sized M; fast: aq_gemm_pc.hip, exact: aq_gemm_pcx.hip)
    int32_t format;          // 0: base format, 1: two-level variant (fast: the producer / consumer kernel; exact: aq_gemm2.hip)
    int32_t reserved;
};
static_assert(sizeof(GemmPlanHeader) == 64, "GemmPlanHeader must stay 64 bytes");
constexpr uint32_t GEMM_PLAN_MAGIC = 0x41514735u;  // "AQG5"

int check_gemm(int64_t N, int64_t K, int bits, int block, int64_t M, int64_t ldx, int64_t ldy, int x_dtype,
               const void* packed, const void* X, const void* Y)
{
    int rc = check_matrix(N, K, bits, block);
    if (rc != AQ_OK) return rc;
    if (M < 1 || M > AQ_MAX_M || ldx < K || ldy < N) return AQ_EINVAL;
    if (ldx % 8 != 0) return AQ_EINVAL;      // rows of X must keep 16-byte alignment
    if ((rc = check_dtype(x_dtype)) != AQ_OK) return rc;
    if (!packed || !X || !Y) return AQ_ENULL;
    if (!aligned16(packed) || !aligned16(X) || !aligned16(Y)) return AQ_EALIGN;
    return AQ_OK;
}

AqGemmTask make_gemm_task(const void* packed, int64_t N, int64_t K, int bits, int64_t M, int64_t xt_offset,
                          float* Y, int64_t ldy, int A, int nsplit, int wg_begin)
{
    AqGemmTask t;
    std::memset(&t, 0, sizeof(t));
    t.blob = static_cast<const uint8_t*>(packed);
    t.Y = Y;
    t.N = N; t.M = M; t.ldy = ldy;
    t.xt_offset = xt_offset;
    t.K = (int32_t)K; t.bits = bits; t.nchunks = (int32_t)aq_num_chunks(K);
    int slabs = 0;
    t.wg_begin = wg_begin;
    t.wg_count = aqk_gemm_wg_count(N, M, A, nsplit, &slabs);
    t.slabs = slabs;
    return t;
}

AqRetileTask make_retile_task(const void* X, int64_t M, int64_t K, int64_t ldx, int64_t xt_offset, int convert)
{
    AqRetileTask r;
    std::memset(&r, 0, sizeof(r));
    r.X = static_cast<const uint16_t*>(X);
    r.M = M; r.ldx = ldx; r.xt_offset = xt_offset;
    r.K = (int32_t)K;
    r.convert = convert;
    r.blocks = aqk_retile_blocks(M, K, convert);
    return r;
}

// indices 0 .. count-1 by descending K, ties in the caller's order
template <class KeyFn>
std::vector<int> longest_k_first(int count, KeyFn key)
{
    std::vector<int> order(count);
    for (int i = 0; i < count; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return key(a) > key(b); });
    return order;
}

constexpr int64_t SMALL_M = 64;      // fast-mode products with M up to this run the streaming kernel
// The producer / consumer kernels' consumers compute whole m-tile slots (1, 2 or 3 per wavefront): used when at least 3
// of 4 of them hold real rows.
bool use_pc(int fast, int64_t M, int per = 0)
{
    if (M <= 64) return false;
    return ((M + 15) / 16) * 4 >= (fast ? aqk_gemm_pc_tile_slots(M, per) : aqk_gemm_pcx_tile_slots(M, per)) * 3;
}

AqGemmTask make_pc_task(const void* packed, int64_t N, int64_t K, int bits, int64_t M, int64_t xt_offset, float* Y,
                        int64_t ldy, int wg_begin, int per = 0)
{
    AqGemmTask t;
    std::memset(&t, 0, sizeof(t));
    t.blob = static_cast<const uint8_t*>(packed);
    t.Y = Y;
    t.N = N; t.M = M; t.ldy = ldy;
    t.xt_offset = xt_offset;
    t.K = (int32_t)K; t.bits = bits; t.nchunks = (int32_t)aq_num_chunks(K);
    int slabs = 0;
    t.wg_begin = wg_begin;
    t.wg_count = aqk_gemm_pc_wg_count(N, M, per, &slabs);
    t.slabs = slabs;
    t.pad[0] = per;
    return t;
}

AqGemmTask make_pcx_task(const void* packed, int64_t N, int64_t K, int bits, int64_t M, int64_t xt_offset, float* Y,
                         int64_t ldy, int wg_begin, int per = 0)
{
    AqGemmTask t = make_pc_task(packed, N, K, bits, M, xt_offset, Y, ldy, wg_begin, per);
    int slabs = 0;
    t.wg_count = aqk_gemm_pcx_wg_count(N, M, per, &slabs);
    return t;
}

constexpr int64_t SMALL_M_EXACT = 64;  // exact-mode products with M up to this run it too, weights as two binary16 terms

AqGemmTask make_small_task(const void* packed, int64_t N, int64_t K, int bits, int64_t M, int64_t xt_offset,
                           float* Y, int64_t ldy, int wg_begin)
{
    AqGemmTask t;
    std::memset(&t, 0, sizeof(t));
    t.blob = static_cast<const uint8_t*>(packed);
    t.Y = Y;
    t.N = N; t.M = M; t.ldy = ldy;
    t.xt_offset = xt_offset;
    t.K = (int32_t)K; t.bits = bits; t.nchunks = (int32_t)aq_num_chunks(K);
    t.slabs = (int32_t)aq_num_groups(N);
    t.wg_begin = wg_begin;
    t.wg_count = t.slabs;                 // one workgroup per 128-row group, all rows of X
    return t;
}

AqRetileTask make_small_retile_task(const void* X, int64_t M, int64_t K, int64_t ldx, int64_t xt_offset, int MT)
{
    AqRetileTask r;
    std::memset(&r, 0, sizeof(r));
    r.X = static_cast<const uint16_t*>(X);
    r.M = M; r.ldx = ldx; r.xt_offset = xt_offset;
    r.K = (int32_t)K;
    r.blocks = MT * 16;
    r.pad = MT;
    return r;
}

int check_flags(int flags) { return (flags == AQ_GEMM_EXACT || flags == AQ_GEMM_FAST) ? AQ_OK : AQ_EINVAL; }

AqGemvTask make_task(const void* packed, int64_t N, int64_t K, int bits, const void* x, int dt, float* y)
{
    AqGemvTask t;
    std::memset(&t, 0, sizeof(t));
    t.blob = static_cast<const uint8_t*>(packed);
    t.x = static_cast<const uint16_t*>(x);
    t.y = y;
    t.N = N;
    t.K = (int32_t)K;
    t.bits = bits;
    t.x_dtype = dt;
    t.nchunks = (int32_t)aq_num_chunks(K);
    return t;
}

// Plan image of the layer-by-layer decode step: this header, one DecodeStage per launch, the task records.
struct DecodePlanHeader {
    uint32_t magic;
    int32_t layers;
    int32_t stages;
    int32_t reserved;
    float* qkv;              // cleared at the start of every step
    int64_t qkv_floats;
    float* gateup;           // cleared by the o stage of every layer
    int64_t gateup_floats;
};
static_assert(sizeof(DecodePlanHeader) == 48, "DecodePlanHeader must stay 48 bytes");
struct DecodeStage {
    int32_t task_begin, task_count, total_wgs, clears_gateup;
};
constexpr uint32_t DECODE_MAGIC = 0x41514431u;  // "AQD1"
constexpr int DECODE_TARGET_WGS = 768;          // 256 compute units x 3 resident workgroups

// chunks per workgroup: the fewest (at least 2 when the matrices are deep enough, so that both ring slots of a
// wavefront are in use; at most AQ_STAGE_MAX_PART) for which the whole stage fits the GPU in ONE round of
// workgroups (3 per compute unit): a second, partial round would double the stage's latency
int decode_part_chunks(const int64_t* rows, int matrices, int nchunks)
{
    int p = nchunks < 2 ? nchunks : 2;
    for (; p < AQ_STAGE_MAX_PART && p < nchunks; ++p) {
        int64_t wgs = 0;
        for (int i = 0; i < matrices; ++i) wgs += aq_num_groups(rows[i]) * ((nchunks + p - 1) / p);
        if (wgs <= DECODE_TARGET_WGS) break;
    }
    return p;
}

}  // namespace

// Scratch of aq_qgemm_noalloc: a file-scope device array (every GPU the library runs on holds its own copy until the
// process ends).  In host code the array's name is only a handle: the address kernels and copies can use comes from
// hipGetSymbolAddress, asked for once per device with that device current.
static __device__ __align__(256) unsigned char scratch[AQ_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
void* scratch_ptr[MAX_DEVICES] = {};

int noalloc_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return AQ_ELAUNCH;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return AQ_ELAUNCH;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return AQ_OK;
}

}  // namespace

extern "C" {

const char* aq_status_string(int status)
{
    switch (status) {
        case AQ_OK: return "ok";
        case AQ_EINVAL: return "invalid argument (bits must be 2, 3 or 4; block 32; K a multiple of 32 and <= 65536; sizes >= 1)";
        case AQ_ENULL: return "null pointer";
        case AQ_EALIGN: return "device pointer not 16-byte aligned";
        case AQ_ESIZE: return "buffer too small";
        case AQ_EDTYPE: return "activation dtype must be AQ_F16 or AQ_BF16";
        case AQ_ELAUNCH: return "HIP launch error";
        default: return "unknown status";
    }
}

size_t aq_packed_size(int64_t N, int64_t K, int bits, int block)
{
    if (check_matrix(N, K, bits, block) != AQ_OK) return 0;
    return (size_t)aq_blob_bytes(N, K, bits);
}

int aq_pack_weights(const uint8_t* codes, const uint16_t* scales, int64_t N, int64_t K, int bits, int block,
                    void* packed, size_t packed_bytes, void* stream)
{
    int rc = check_matrix(N, K, bits, block);
    if (rc != AQ_OK) return rc;
    if (!codes || !scales || !packed) return AQ_ENULL;
    if (!aligned16(codes) || !aligned16(scales) || !aligned16(packed)) return AQ_EALIGN;
    if (packed_bytes < (size_t)aq_blob_bytes(N, K, bits)) return AQ_ESIZE;
    return aqk_pack(codes, scales, N, K, bits, packed, static_cast<hipStream_t>(stream)) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

int aq_qgemv(const void* packed, int64_t N, int64_t K, int bits, int block, const void* x, int x_dtype,
             float* y, void* stream)
{
    int rc = check_matrix(N, K, bits, block);
    if (rc != AQ_OK) return rc;
    if ((rc = check_dtype(x_dtype)) != AQ_OK) return rc;
    if (!packed || !x || !y) return AQ_ENULL;
    if (!aligned16(packed) || !aligned16(x) || !aligned16(y)) return AQ_EALIGN;
    AqGemvTask t = make_task(packed, N, K, bits, x, x_dtype, y);
    t.wg_begin = 0;
    aqk_gemv_shape(t, false);
    return aqk_gemv(nullptr, nullptr, 0, t, bits, t.wg_count, (int)K, static_cast<hipStream_t>(stream)) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

// workgroups of the list (both formats use the same launch shape), -1 if a descriptor is invalid
static int64_t gemv_list_wgs(const aq_gemv_desc* descs, int count, int block, int* status)
{
    int64_t wgs = 0;
    for (int i = 0; i < count; ++i) {
        const aq_gemv_desc& d = descs[i];
        int rc = check_matrix(d.N, d.K, d.bits, block);
        if (rc == AQ_OK) rc = check_dtype(d.x_dtype);
        if (rc == AQ_OK && (!d.packed || !d.x || !d.y)) rc = AQ_ENULL;
        if (rc == AQ_OK && (!aligned16(d.packed) || !aligned16(d.x) || !aligned16(d.y))) rc = AQ_EALIGN;
        if (rc != AQ_OK) { if (status) *status = rc; return -1; }
        AqGemvTask t = make_task(d.packed, d.N, d.K, d.bits, d.x, d.x_dtype, d.y);
        aqk_gemv_shape(t, true);
        wgs += t.wg_count;
        if (wgs > 0x3FFFFFFF) { if (status) *status = AQ_EINVAL; return -1; }
    }
    return wgs;
}

static size_t gemv_plan_bytes(int count, int64_t wgs)
{
    return sizeof(PlanHeader) + (size_t)count * sizeof(AqGemvTask) + (((size_t)wgs * 4 + 15) & ~(size_t)15);
}

size_t aq_qgemv_batch_plan_size(const aq_gemv_desc* descs, int count, int block)
{
    if (count < 1 || !descs) return 0;
    const int64_t wgs = gemv_list_wgs(descs, count, block, nullptr);      // one size serves both planners
    if (wgs < 0) return 0;
    return gemv_plan_bytes(count, wgs);
}

static int gemv_plan(const aq_gemv_desc* descs, int count, int block, void* plan_host, size_t plan_bytes, int format)
{
    if (count < 1) return AQ_EINVAL;
    if (!descs || !plan_host) return AQ_ENULL;
    int status = AQ_OK;
    const int64_t wgs = gemv_list_wgs(descs, count, block, &status);
    if (wgs < 0) return status;
    if (plan_bytes < gemv_plan_bytes(count, wgs)) return AQ_ESIZE;
    int max_K = 0;
    for (int i = 0; i < count; ++i)
        if (descs[i].K > max_K) max_K = (int)descs[i].K;
    PlanHeader h;
    std::memset(&h, 0, sizeof(h));
    h.magic = PLAN_MAGIC;
    h.count = count;
    h.tiles_per_wg = 8;
    h.max_K = max_K;
    h.format = format;
    AqGemvTask* tasks = reinterpret_cast<AqGemvTask*>(static_cast<uint8_t*>(plan_host) + sizeof(PlanHeader));
    int32_t* wg_task = reinterpret_cast<int32_t*>(static_cast<uint8_t*>(plan_host) + sizeof(PlanHeader) +
                                                  (size_t)count * sizeof(AqGemvTask));
    int32_t begin = 0;
    h.bits = descs[0].bits;
    // The products of a list are independent, so their workgroups may run in any order.  A workgroup walks the
    // whole K of its rows: those of the longest K go first, so that the launch does not end on a few long ones.
    std::vector<int> order = longest_k_first(count, [&](int i) { return descs[i].K; });
    for (int j = 0; j < count; ++j) {
        const aq_gemv_desc& d = descs[order[j]];
        if (d.bits != descs[0].bits) h.bits = 0;
        AqGemvTask t = make_task(d.packed, d.N, d.K, d.bits, d.x, d.x_dtype, d.y);
        t.wg_begin = begin;
        aqk_gemv_shape(t, true);
        for (int w = 0; w < t.wg_count; ++w) wg_task[begin + w] = j;
        begin += t.wg_count;
        std::memcpy(&tasks[j], &t, sizeof(t));
    }
    h.total_wgs = begin;
    std::memcpy(plan_host, &h, sizeof(h));
    return AQ_OK;
}

int aq_qgemv_batch_plan(const aq_gemv_desc* descs, int count, int block, void* plan_host, size_t plan_bytes)
{
    return gemv_plan(descs, count, block, plan_host, plan_bytes, 0);
}

int aq2_qgemv_batch_plan(const aq_gemv_desc* descs, int count, int block, void* plan_host, size_t plan_bytes)
{
    return gemv_plan(descs, count, block, plan_host, plan_bytes, 1);
}

size_t aq2_packed_size(int64_t N, int64_t K, int bits, int block)
{
    if (check_matrix(N, K, bits, block) != AQ_OK) return 0;
    return (size_t)aq2_blob_bytes(N, K, bits);
}

int aq2_pack_weights(const uint8_t* codes, const uint8_t* sub, const uint16_t* sup, int64_t N, int64_t K, int bits,
                     int block, void* packed, size_t packed_bytes, void* stream)
{
    int rc = check_matrix(N, K, bits, block);
    if (rc != AQ_OK) return rc;
    if (!codes || !sub || !sup || !packed) return AQ_ENULL;
    if (!aligned16(codes) || !aligned16(sub) || !aligned16(sup) || !aligned16(packed)) return AQ_EALIGN;
    if (packed_bytes < (size_t)aq2_blob_bytes(N, K, bits)) return AQ_ESIZE;
    return aqk2_pack(codes, sub, sup, N, K, bits, packed, static_cast<hipStream_t>(stream)) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

int aq2_qgemv(const void* packed, int64_t N, int64_t K, int bits, int block, const void* x, int x_dtype,
              float* y, void* stream)
{
    int rc = check_matrix(N, K, bits, block);
    if (rc != AQ_OK) return rc;
    if ((rc = check_dtype(x_dtype)) != AQ_OK) return rc;
    if (!packed || !x || !y) return AQ_ENULL;
    if (!aligned16(packed) || !aligned16(x) || !aligned16(y)) return AQ_EALIGN;
    AqGemvTask t = make_task(packed, N, K, bits, x, x_dtype, y);
    t.wg_begin = 0;
    aqk_gemv_shape(t, false);
    return aqk2_gemv(nullptr, nullptr, 0, t, bits, t.wg_count, (int)K, static_cast<hipStream_t>(stream)) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

int aq2_unpack_codes(const void* packed, int64_t N, int64_t K, int bits, int block, uint8_t* codes_u8, void* stream)
{
    int rc = check_matrix(N, K, bits, block);
    if (rc != AQ_OK) return rc;
    if (!packed || !codes_u8) return AQ_ENULL;
    if (!aligned16(packed) || !aligned16(codes_u8)) return AQ_EALIGN;
    return aqk2_unpack_codes(packed, N, K, bits, codes_u8, static_cast<hipStream_t>(stream)) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

int aq2_dequant_f32(const void* packed, int64_t N, int64_t K, int bits, int block, float* W, void* stream)
{
    int rc = check_matrix(N, K, bits, block);
    if (rc != AQ_OK) return rc;
    if (!packed || !W) return AQ_ENULL;
    if (!aligned16(packed) || !aligned16(W)) return AQ_EALIGN;
    return aqk2_dequant(packed, N, K, bits, W, static_cast<hipStream_t>(stream)) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

int aq_qgemv_batch(const void* plan_host, const void* plan_dev, void* stream)
{
    if (!plan_host || !plan_dev) return AQ_ENULL;
    if (!aligned16(plan_dev)) return AQ_EALIGN;
    PlanHeader h;
    std::memcpy(&h, plan_host, sizeof(h));
    if (h.magic != PLAN_MAGIC || h.count < 1 || h.total_wgs < 1 || (h.bits != 0 && (h.bits < 2 || h.bits > 4)) ||
        (h.format != 0 && h.format != 1))
        return AQ_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint8_t* dev = static_cast<const uint8_t*>(plan_dev);
    const AqGemvTask* tasks = reinterpret_cast<const AqGemvTask*>(dev + sizeof(PlanHeader));
    AqGemvTask none;
    std::memset(&none, 0, sizeof(none));
    const int32_t* wg_task = reinterpret_cast<const int32_t*>(dev + sizeof(PlanHeader) + (size_t)h.count * sizeof(AqGemvTask));
    if (h.format == 1)
        return aqk2_gemv(tasks, wg_task, h.count, none, h.bits, h.total_wgs, h.max_K, s) == hipSuccess ? AQ_OK : AQ_ELAUNCH;
    return aqk_gemv(tasks, wg_task, h.count, none, h.bits, h.total_wgs, h.max_K, s) == hipSuccess ? AQ_OK : AQ_ELAUNCH;
}

size_t aq_qgemm_workspace_size(int64_t M, int64_t N, int64_t K, int bits)
{
    if (check_matrix(N, K, bits, AQ_BLOCK) != AQ_OK || M < 1 || M > AQ_MAX_M) return 0;
    const size_t a = aqk_retile_bytes(M, K), b = M <= SMALL_M ? aqk_small_retile_bytes(M, K) : 0;
    return a > b ? a : b;      // either mode's layout of X fits
}

static int qgemm_one(const void* packed, int64_t N, int64_t K, int bits, int block, const void* X, int64_t M,
                     int64_t ldx, int x_dtype, float* Y, int64_t ldy, int flags, void* workspace, size_t workspace_bytes,
                     void* stream)
{
    int rc = check_gemm(N, K, bits, block, M, ldx, ldy, x_dtype, packed, X, Y);
    if (rc != AQ_OK) return rc;
    if (!workspace) return AQ_ENULL;
    if (!aligned16(workspace)) return AQ_EALIGN;
    if (workspace_bytes < aq_qgemm_workspace_size(M, N, K, bits)) return AQ_ESIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int fast = flags == AQ_GEMM_FAST, convert = fast && x_dtype == AQ_BF16;
    if (M <= (fast ? SMALL_M : SMALL_M_EXACT)) {
        const int MT = aqk_small_mtiles(M);
        const AqRetileTask r = make_small_retile_task(X, M, K, ldx, 0, MT);
        if (aqk_small_retile(nullptr, 0, r, MT, x_dtype == AQ_BF16, workspace, s) != hipSuccess) return AQ_ELAUNCH;
        const AqGemmTask t = make_small_task(packed, N, K, bits, M, 0, Y, ldy, 0);
        return aqk_gemm_small(nullptr, 0, t, bits, MT, !fast, t.wg_count, workspace, s) == hipSuccess ? AQ_OK : AQ_ELAUNCH;
    }
    const AqRetileTask r = make_retile_task(X, M, K, ldx, 0, convert);
    const int per = aqk_gemm_pc_tiles_per_wg(M, aq_num_groups(N));      // a lone matrix: fewer m-tiles per workgroup
    if (use_pc(fast, M, per)) {
        AqGemmTask t = fast ? make_pc_task(packed, N, K, bits, M, 0, Y, ldy, 0, per)
                            : make_pcx_task(packed, N, K, bits, M, 0, Y, ldy, 0, per);
        // still under half of the chip's compute units: two workgroups per (group, m-block), each half of K, their
        // parts added into Y, which the re-tiling launch clears
        const int kparts = t.wg_count * 2 <= 256 && t.nchunks >= 8 ? 2 : 1;
        if (kparts > 1) {
            t.pad[1] = kparts;
            t.wg_count *= kparts;
        }
        if (aqk_retile(nullptr, 0, r, r.blocks, convert, workspace, s, kparts > 1 ? Y : nullptr, N, ldy) != hipSuccess)
            return AQ_ELAUNCH;
        if (!fast)
            return aqk_gemm_pcx(nullptr, 0, t, bits, x_dtype, t.wg_count, workspace, s) == hipSuccess ? AQ_OK : AQ_ELAUNCH;
        return aqk_gemm_pc(nullptr, 0, t, bits, 0, t.wg_count, workspace, s) == hipSuccess ? AQ_OK : AQ_ELAUNCH;
    }
    if (aqk_retile(nullptr, 0, r, r.blocks, convert, workspace, s) != hipSuccess) return AQ_ELAUNCH;
    const int A = aqk_gemm_mtiles(M, aq_num_groups(N)), nsplit = aqk_gemm_nsplit(M);
    AqGemmTask t = make_gemm_task(packed, N, K, bits, M, 0, Y, ldy, A, nsplit, 0);
    return aqk_gemm(nullptr, 0, t, bits, x_dtype, A, nsplit, fast, t.wg_count, workspace, s) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

int aq_qgemm(const void* packed, int64_t N, int64_t K, int bits, int block, const void* X, int64_t M,
             int64_t ldx, int x_dtype, float* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream)
{
    return qgemm_one(packed, N, K, bits, block, X, M, ldx, x_dtype, Y, ldy, AQ_GEMM_EXACT, workspace, workspace_bytes,
                     stream);
}

int aq_qgemm_fast(const void* packed, int64_t N, int64_t K, int bits, int block, const void* X, int64_t M,
                  int64_t ldx, int x_dtype, float* Y, int64_t ldy, void* workspace, size_t workspace_bytes,
                  void* stream)
{
    return qgemm_one(packed, N, K, bits, block, X, M, ldx, x_dtype, Y, ldy, AQ_GEMM_FAST, workspace, workspace_bytes,
                     stream);
}

int aq_qgemm_noalloc(const void* packed, int64_t N, int64_t K, int bits, int block, const void* X, int64_t M,
                     int64_t ldx, int x_dtype, float* Y, int64_t ldy, void* stream)
{
    int rc = check_gemm(N, K, bits, block, M, ldx, ldy, x_dtype, packed, X, Y);
    if (rc != AQ_OK) return rc;
    if (aq_qgemm_workspace_size(M, N, K, bits) > (size_t)AQ_NOALLOC_SCRATCH_BYTES) return AQ_ESIZE;
    void* ws = nullptr;
    if ((rc = noalloc_scratch(&ws)) != AQ_OK) return rc;
    return qgemm_one(packed, N, K, bits, block, X, M, ldx, x_dtype, Y, ldy, AQ_GEMM_EXACT, ws, AQ_NOALLOC_SCRATCH_BYTES,
                     stream);
}

static int qgemm2_one(const void* packed, int64_t N, int64_t K, int bits, int block, const void* X, int64_t M, int64_t ldx,
                      int x_dtype, float* Y, int64_t ldy, int flags, void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_gemm(N, K, bits, block, M, ldx, ldy, x_dtype, packed, X, Y);
    if (rc != AQ_OK) return rc;
    if (!workspace) return AQ_ENULL;
    if (!aligned16(workspace)) return AQ_EALIGN;
    if (workspace_bytes < aq_qgemm_workspace_size(M, N, K, bits)) return AQ_ESIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int fast = flags == AQ_GEMM_FAST, convert = fast && x_dtype == AQ_BF16;
    const AqRetileTask r = make_retile_task(X, M, K, ldx, 0, convert);
    if (aqk_retile(nullptr, 0, r, r.blocks, convert, workspace, s) != hipSuccess) return AQ_ELAUNCH;
    if (fast) {
        const AqGemmTask t = make_pc_task(packed, N, K, bits, M, 0, Y, ldy, 0);
        return aqk_gemm_pc(nullptr, 0, t, bits, 1, t.wg_count, workspace, s) == hipSuccess ? AQ_OK : AQ_ELAUNCH;
    }
    const int A = aqk_gemm_mtiles(M, aq_num_groups(N));
    const AqGemmTask t = make_gemm_task(packed, N, K, bits, M, 0, Y, ldy, A, 1, 0);
    return aqk2_gemm(nullptr, 0, t, x_dtype, A, t.wg_count, workspace, s) == hipSuccess ? AQ_OK : AQ_ELAUNCH;
}

int aq2_qgemm(const void* packed, int64_t N, int64_t K, int bits, int block, const void* X, int64_t M, int64_t ldx,
              int x_dtype, float* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream)
{
    return qgemm2_one(packed, N, K, bits, block, X, M, ldx, x_dtype, Y, ldy, AQ_GEMM_EXACT, workspace, workspace_bytes, stream);
}

int aq2_qgemm_fast(const void* packed, int64_t N, int64_t K, int bits, int block, const void* X, int64_t M, int64_t ldx,
                   int x_dtype, float* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream)
{
    return qgemm2_one(packed, N, K, bits, block, X, M, ldx, x_dtype, Y, ldy, AQ_GEMM_FAST, workspace, workspace_bytes, stream);
}

// Codebook variant, fp16-weight prefill: the producer / consumer kernel with the table-lookup producer at every M; the
// table (level of every stored code) goes to the last 64 bytes of the workspace first.
size_t aqc_qgemm_workspace_size(int64_t M, int64_t N, int64_t K, int bits)
{
    const size_t base = aq_qgemm_workspace_size(M, N, K, bits);
    return base ? base + 64 : 0;
}

int aqc_qgemm(const void* packed, int64_t N, int64_t K, int bits, int block, const float* levels, const void* X, int64_t M,
              int64_t ldx, int x_dtype, float* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_gemm(N, K, bits, block, M, ldx, ldy, x_dtype, packed, X, Y);
    if (rc != AQ_OK) return rc;
    if (!workspace || !levels) return AQ_ENULL;
    if (!aligned16(workspace)) return AQ_EALIGN;
    const size_t base = aq_qgemm_workspace_size(M, N, K, bits);
    if (workspace_bytes < base + 64) return AQ_ESIZE;
    AqCbTable table;
    if ((rc = aqk_cb_stored_levels(levels, bits, &table)) != AQ_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* table_dev = reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + base);
    if (aqk_cb_write_table(table, table_dev, s) != hipSuccess) return AQ_ELAUNCH;
    const int convert = x_dtype == AQ_BF16;
    const AqRetileTask r = make_retile_task(X, M, K, ldx, 0, convert);
    if (aqk_retile(nullptr, 0, r, r.blocks, convert, workspace, s) != hipSuccess) return AQ_ELAUNCH;
    const AqGemmTask t = make_pc_task(packed, N, K, bits, M, 0, Y, ldy, 0);
    return aqk_gemm_pc(nullptr, 0, t, bits, 2, t.wg_count, workspace, s, table_dev) == hipSuccess ? AQ_OK : AQ_ELAUNCH;
}

// plan image: header, `count` product tasks, then up to `count` re-tiling tasks
size_t aq_qgemm_batch_plan_size(int count)
{
    if (count < 1) return 0;
    return sizeof(GemmPlanHeader) + (size_t)count * (sizeof(AqGemmTask) + sizeof(AqRetileTask));
}

// format 1 (two-level variant): the fp16-weight mode runs the producer / consumer kernel and the exact mode the
// 8-wavefront kernel, both at every M
static int gemm_plan(const aq_gemm_desc* descs, int count, int block, int flags, void* plan_host, size_t plan_bytes,
                     int format)
{
    if (count < 1 || check_flags(flags) != AQ_OK) return AQ_EINVAL;
    if (!descs || !plan_host) return AQ_ENULL;
    if (plan_bytes < aq_qgemm_batch_plan_size(count)) return AQ_ESIZE;
    int64_t max_M = 0;
    for (int i = 0; i < count; ++i) {
        const aq_gemm_desc& d = descs[i];
        int rc = check_gemm(d.N, d.K, d.bits, block, d.M, d.ldx, d.ldy, d.x_dtype, d.packed, d.X, d.Y);
        if (rc != AQ_OK) return rc;
        if (d.x_dtype != descs[0].x_dtype) return AQ_EDTYPE;
        if (d.M > max_M) max_M = d.M;
    }
    GemmPlanHeader h;
    std::memset(&h, 0, sizeof(h));
    h.magic = GEMM_PLAN_MAGIC;
    h.count = count;
    h.bits = descs[0].bits;
    h.x_dtype = descs[0].x_dtype;
    int64_t groups = 0;
    for (int i = 0; i < count; ++i) groups += aq_num_groups(descs[i].N);
    h.mtiles = aqk_gemm_mtiles(max_M, groups);
    h.nsplit = format ? 1 : aqk_gemm_nsplit(max_M);
    h.fast = flags == AQ_GEMM_FAST;
    h.format = format;
    h.small_mt = !format && max_M <= (h.fast ? SMALL_M : SMALL_M_EXACT) ? aqk_small_mtiles(max_M) : 0;
    h.pc = format ? h.fast : 1;                       // format 1: fast -> pc; format 2: always fast, always pc
    for (int i = 0; i < count && !format; ++i) h.pc = h.pc && use_pc(h.fast, descs[i].M);      // every product of the list
    const int convert = h.fast && h.x_dtype == AQ_BF16;
    uint8_t* base = static_cast<uint8_t*>(plan_host);
    uint8_t* tasks = base + sizeof(GemmPlanHeader);
    uint8_t* rtasks = tasks + (size_t)count * sizeof(AqGemmTask);
    // products that read the same activations (same pointer, shape and row stride) share one re-tiled copy
    std::vector<AqRetileTask> rt;
    int64_t begin = 0, ws = 0;
    std::vector<int> order = longest_k_first(count, [&](int i) { return descs[i].K; });   // see aq_qgemv_batch_plan
    for (int j = 0; j < count; ++j) {
        const int i = j;
        const aq_gemm_desc& d = descs[order[j]];
        if (d.bits != descs[0].bits) h.bits = 0;
        int64_t off = -1;
        for (const AqRetileTask& r : rt)
            if (r.X == d.X && r.M == d.M && r.K == d.K && r.ldx == d.ldx) { off = r.xt_offset; break; }
        if (off < 0) {
            off = ws;
            if (h.small_mt) {
                rt.push_back(make_small_retile_task(d.X, d.M, d.K, d.ldx, off, h.small_mt));
                ws += (int64_t)aqk_small_retile_bytes(max_M, d.K);
            } else {
                rt.push_back(make_retile_task(d.X, d.M, d.K, d.ldx, off, convert));
                ws += (int64_t)aqk_retile_bytes(d.M, d.K);
            }
            if (rt.back().blocks > h.retile_max_blocks) h.retile_max_blocks = rt.back().blocks;
        }
        AqGemmTask t = h.small_mt ? make_small_task(d.packed, d.N, d.K, d.bits, d.M, off, d.Y, d.ldy, (int)begin)
                       : (h.pc && !h.fast) ? make_pcx_task(d.packed, d.N, d.K, d.bits, d.M, off, d.Y, d.ldy, (int)begin)
                       : h.pc ? make_pc_task(d.packed, d.N, d.K, d.bits, d.M, off, d.Y, d.ldy, (int)begin)
                                  : make_gemm_task(d.packed, d.N, d.K, d.bits, d.M, off, d.Y, d.ldy, h.mtiles, h.nsplit, (int)begin);
        begin += t.wg_count;
        if (begin > 0x7FFFFFFF) return AQ_EINVAL;
        std::memcpy(tasks + (size_t)i * sizeof(AqGemmTask), &t, sizeof(t));
    }
    std::memset(rtasks, 0, (size_t)count * sizeof(AqRetileTask));
    std::memcpy(rtasks, rt.data(), rt.size() * sizeof(AqRetileTask));
    h.total_wgs = (int32_t)begin;
    h.retile_count = (int32_t)rt.size();
    h.workspace_bytes = ws;
    std::memcpy(plan_host, &h, sizeof(h));
    return AQ_OK;
}

int aq_qgemm_batch_plan(const aq_gemm_desc* descs, int count, int block, int flags, void* plan_host,
                        size_t plan_bytes)
{
    return gemm_plan(descs, count, block, flags, plan_host, plan_bytes, 0);
}

int aq2_qgemm_batch_plan(const aq_gemm_desc* descs, int count, int block, int flags, void* plan_host, size_t plan_bytes)
{
    return gemm_plan(descs, count, block, flags, plan_host, plan_bytes, 1);
}

// Codebook variant: the base plan image (format 2: the fp16-weight producer / consumer kernel at every M) followed by
// one table of 16 floats per task, in the plan's task order (longest K first, ties in the caller's order).
size_t aqc_qgemm_batch_plan_size(int count)
{
    if (count < 1) return 0;
    return aq_qgemm_batch_plan_size(count) + (size_t)count * 64;
}

int aqc_qgemm_batch_plan(const aqc_gemm_desc* descs, int count, int block, void* plan_host, size_t plan_bytes)
{
    if (count < 1) return AQ_EINVAL;
    if (!descs || !plan_host) return AQ_ENULL;
    if (plan_bytes < aqc_qgemm_batch_plan_size(count)) return AQ_ESIZE;
    std::vector<aq_gemm_desc> plain((size_t)count);
    for (int i = 0; i < count; ++i) {
        plain[i] = descs[i].product;
        if (!descs[i].levels) return AQ_ENULL;
    }
    int rc = gemm_plan(plain.data(), count, block, AQ_GEMM_FAST, plan_host, aq_qgemm_batch_plan_size(count), 2);
    if (rc != AQ_OK) return rc;
    std::vector<int> order = longest_k_first(count, [&](int i) { return plain[i].K; });
    uint8_t* tables = static_cast<uint8_t*>(plan_host) + aq_qgemm_batch_plan_size(count);
    for (int j = 0; j < count; ++j) {
        AqCbTable table;
        if ((rc = aqk_cb_stored_levels(descs[order[j]].levels, plain[order[j]].bits, &table)) != AQ_OK) return rc;
        std::memcpy(tables + (size_t)j * 64, table.level, 64);
    }
    return AQ_OK;
}

static bool read_gemm_plan(const void* plan_host, GemmPlanHeader& h)
{
    std::memcpy(&h, plan_host, sizeof(h));
    return h.magic == GEMM_PLAN_MAGIC && h.count >= 1 && h.total_wgs >= 1 && (h.bits == 0 || (h.bits >= 2 && h.bits <= 4)) &&
           check_dtype(h.x_dtype) == AQ_OK && h.retile_count >= 1 && h.retile_count <= h.count &&
           h.retile_max_blocks >= 1 && h.workspace_bytes >= 1024 &&
           (h.nsplit == 1 || ((h.nsplit == 2 || h.nsplit == 4 || h.nsplit == 8) && h.mtiles == 1)) &&
           (h.fast == 0 || h.fast == 1) &&
           (h.small_mt == 0 || h.small_mt == 1 || h.small_mt == 2 || h.small_mt == 4) &&
           (h.pc == 0 || (h.pc == 1 && h.small_mt == 0)) &&
           (h.format == 0 || (h.format == 1 && h.pc == h.fast && h.small_mt == 0) ||
            (h.format == 2 && h.pc == 1 && h.fast == 1 && h.small_mt == 0));
}

size_t aq_qgemm_batch_workspace_size(const void* plan_host)
{
    GemmPlanHeader h;
    if (!plan_host || !read_gemm_plan(plan_host, h)) return 0;
    return (size_t)h.workspace_bytes;
}

int aq_qgemm_batch(const void* plan_host, const void* plan_dev, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!plan_host || !plan_dev || !workspace) return AQ_ENULL;
    if (!aligned16(plan_dev) || !aligned16(workspace)) return AQ_EALIGN;
    GemmPlanHeader h;
    if (!read_gemm_plan(plan_host, h)) return AQ_EINVAL;
    if (workspace_bytes < (size_t)h.workspace_bytes) return AQ_ESIZE;
    const uint8_t* dev = static_cast<const uint8_t*>(plan_dev);
    const AqGemmTask* tasks = reinterpret_cast<const AqGemmTask*>(dev + sizeof(GemmPlanHeader));
    const AqRetileTask* rtasks =
        reinterpret_cast<const AqRetileTask*>(dev + sizeof(GemmPlanHeader) + (size_t)h.count * sizeof(AqGemmTask));
    hipStream_t s = static_cast<hipStream_t>(stream);
    AqRetileTask rnone;
    std::memset(&rnone, 0, sizeof(rnone));
    const int convert = h.fast && h.x_dtype == AQ_BF16;
    AqGemmTask none;
    std::memset(&none, 0, sizeof(none));
    if (h.small_mt) {
        if (aqk_small_retile(rtasks, h.retile_count, rnone, h.small_mt, h.x_dtype == AQ_BF16, workspace, s) != hipSuccess)
            return AQ_ELAUNCH;
        return aqk_gemm_small(tasks, h.count, none, h.bits, h.small_mt, h.fast == 0, h.total_wgs, workspace, s) == hipSuccess
                   ? AQ_OK : AQ_ELAUNCH;
    }
    if (aqk_retile(rtasks, h.retile_count, rnone, h.retile_max_blocks, convert, workspace, s) != hipSuccess)
        return AQ_ELAUNCH;
    if (h.pc && !h.fast)
        return aqk_gemm_pcx(tasks, h.count, none, h.bits, h.x_dtype, h.total_wgs, workspace, s) == hipSuccess ? AQ_OK : AQ_ELAUNCH;
    if (h.pc) {
        // format 2: the tables follow the re-tiling tasks in the plan image
        const float* tables = h.format == 2 ? reinterpret_cast<const float*>(dev + aq_qgemm_batch_plan_size(h.count)) : nullptr;
        return aqk_gemm_pc(tasks, h.count, none, h.bits, h.format, h.total_wgs, workspace, s, tables) == hipSuccess
                   ? AQ_OK : AQ_ELAUNCH;
    }
    if (h.format == 1)
        return aqk2_gemm(tasks, h.count, none, h.x_dtype, h.mtiles, h.total_wgs, workspace, s) == hipSuccess
                   ? AQ_OK : AQ_ELAUNCH;
    return aqk_gemm(tasks, h.count, none, h.bits, h.x_dtype, h.mtiles, h.nsplit, h.fast, h.total_wgs, workspace, s) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

int aq_optimize_scales(const float* W, const float* F, int64_t N, int64_t K, int bits, int block, int rounds,
                       uint8_t* codes, uint16_t* scales, void* stream)
{
    int rc = check_matrix(N, K, bits, block);
    if (rc != AQ_OK) return rc;
    if (rounds < 0 || rounds > AQ_MAX_ROUNDS) return AQ_EINVAL;
    if (N * K > (int64_t)1 << 40) return AQ_EINVAL;
    if (!W || !codes || !scales) return AQ_ENULL;
    if (!aligned16(W) || (F && !aligned16(F)) || !aligned16(codes) || !aligned16(scales)) return AQ_EALIGN;
    return aqk_optimize_scales(W, F, N, K, bits, rounds, codes, scales, static_cast<hipStream_t>(stream)) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

// Host-only: the greedy solver of the layer-balanced allocation problem (Section 4.1, Eq. 6 and "Solver").
int aq_allocate_bits(const double* S, const int64_t* sizes, int L, int J, const int* choices, int n_choices,
                     double avg_bits_budget, int* bits_out)
{
    if (L < 1 || J < 1 || n_choices < 1 || n_choices > 16) return AQ_EINVAL;
    if (!S || !sizes || !choices || !bits_out) return AQ_ENULL;
    for (int c = 0; c < n_choices; ++c)
        if (choices[c] < 1 || choices[c] > 16 || (c && choices[c] <= choices[c - 1])) return AQ_EINVAL;
    double total = 0.0, used = 0.0;
    for (int64_t i = 0; i < (int64_t)L * J; ++i) {
        if (sizes[i] < 1) return AQ_EINVAL;
        total += (double)sizes[i];
        used += (double)choices[0] * (double)sizes[i];
    }
    if (!(avg_bits_budget * total >= used)) return AQ_EINVAL;      // even the cheapest type everywhere is over budget
    std::vector<int> level((size_t)L * J, 0);
    auto eta = [](int b) { return std::ldexp(1.0, -2 * b); };       // per-element squared error of a b-bit type
    auto layer_error = [&](int l, int swap_j, int swap_bits) {      // E_l, tensor swap_j taken at swap_bits
        double e = 0.0;
        for (int j = 0; j < J; ++j) {
            const int b = j == swap_j ? swap_bits : choices[level[(size_t)l * J + j]];
            e += S[(size_t)l * J + j] * eta(b);
        }
        return e;
    };
    for (;;) {
        int best_l = -1, best_j = -1;
        double best_ratio = 0.0, best_dbits = 0.0;
        for (int l = 0; l < L; ++l) {
            const double e_now = layer_error(l, -1, 0);
            for (int j = 0; j < J; ++j) {
                const int lv = level[(size_t)l * J + j];
                if (lv + 1 >= n_choices) continue;
                const double dbits = (double)(choices[lv + 1] - choices[lv]) * (double)sizes[(size_t)l * J + j];
                if (used + dbits > avg_bits_budget * total) continue;
                const double e_new = layer_error(l, j, choices[lv + 1]);
                const double ratio = (e_now * e_now - e_new * e_new) / dbits;
                if (ratio > best_ratio) { best_ratio = ratio; best_l = l; best_j = j; best_dbits = dbits; }
            }
        }
        if (best_l < 0) break;
        ++level[(size_t)best_l * J + best_j];
        used += best_dbits;
    }
    for (int64_t i = 0; i < (int64_t)L * J; ++i) bits_out[i] = choices[level[(size_t)i]];
    return AQ_OK;
}

size_t aq_decode_plan_size(int layers)
{
    if (layers < 1) return 0;
    return sizeof(DecodePlanHeader) + (size_t)layers * (4 * sizeof(DecodeStage) + 7 * sizeof(AqStageTask));
}

size_t aq_decode_workspace_size(const aq_block_shape* shape)
{
    if (!shape || shape->d_ff < 1) return 0;
    return (size_t)2 * (size_t)shape->d_ff * sizeof(float);
}

int aq_decode_plan(const aq_block_shape* shape, const aq_block_desc* blocks, int layers, int block,
                   float* x, float* qkv, void* workspace, size_t workspace_bytes, void* plan_host, size_t plan_bytes)
{
    if (!shape || !blocks || !x || !qkv || !workspace || !plan_host) return AQ_ENULL;
    if (layers < 1 || block != AQ_BLOCK) return AQ_EINVAL;
    const aq_block_shape& sh = *shape;
    if (sh.d_model < 32 || sh.d_ff < 32 || sh.d_model % 32 || sh.d_ff % 32 || sh.d_model > AQ_LAYER_MAX_K || sh.d_ff > AQ_LAYER_MAX_K)
        return AQ_EINVAL;
    if (sh.n_heads < 1 || sh.n_kv_heads < 1 || sh.n_heads % sh.n_kv_heads || sh.head_dim < 8 || sh.head_dim % 8)
        return AQ_EINVAL;
    const int64_t dq = (int64_t)sh.n_heads * sh.head_dim, dkv = (int64_t)sh.n_kv_heads * sh.head_dim;
    if (dq % 32 || dkv % 32 || dq > AQ_LAYER_MAX_K) return AQ_EINVAL;
    if (sh.act != AQ_ACT_SILU && sh.act != AQ_ACT_GELU_TANH) return AQ_EINVAL;
    if (!(sh.eps >= 0.f)) return AQ_EINVAL;
    if (!aligned16(x) || !aligned16(qkv) || !aligned16(workspace)) return AQ_EALIGN;
    if (workspace_bytes < aq_decode_workspace_size(shape) || plan_bytes < aq_decode_plan_size(layers)) return AQ_ESIZE;
    for (int l = 0; l < layers; ++l) {
        for (int j = 0; j < 7; ++j) {
            if (!blocks[l].w[j]) return AQ_ENULL;
            if (!aligned16(blocks[l].w[j])) return AQ_EALIGN;
            if (blocks[l].bits[j] < 2 || blocks[l].bits[j] > 4) return AQ_EINVAL;
        }
        if (!blocks[l].norm_attn || !blocks[l].norm_mlp) return AQ_ENULL;
        if (!aligned16(blocks[l].norm_attn) || !aligned16(blocks[l].norm_mlp)) return AQ_EALIGN;
    }

    float* gate = static_cast<float*>(workspace);
    float* up = gate + sh.d_ff;
    const int64_t per_layer = dq + 2 * dkv;
    DecodePlanHeader h;
    std::memset(&h, 0, sizeof(h));
    h.magic = DECODE_MAGIC;
    h.layers = layers;
    h.stages = 4 * layers;
    h.qkv = qkv;
    h.qkv_floats = per_layer * layers;
    h.gateup = gate;
    h.gateup_floats = 2 * (int64_t)sh.d_ff;
    uint8_t* base = static_cast<uint8_t*>(plan_host);
    DecodeStage* stages = reinterpret_cast<DecodeStage*>(base + sizeof(DecodePlanHeader));
    AqStageTask* tasks = reinterpret_cast<AqStageTask*>(base + sizeof(DecodePlanHeader) + (size_t)h.stages * sizeof(DecodeStage));

    auto make = [&](const aq_block_desc& b, int j, int64_t N, int64_t K, int part, float* y, const float* in0,
                    const float* in1, int prologue, int& wgs) {
        AqStageTask t;
        std::memset(&t, 0, sizeof(t));
        t.blob = static_cast<const uint8_t*>(b.w[j]);
        t.y = y;
        t.in0 = in0;
        t.in1 = in1;
        t.N = (int32_t)N;
        t.K = (int32_t)K;
        t.bits = b.bits[j];
        t.nchunks = (int32_t)aq_num_chunks(K);
        t.part_chunks = part;
        t.parts = (t.nchunks + part - 1) / part;
        t.wg_begin = wgs;
        t.wg_count = (int32_t)(aq_num_groups(N) * t.parts);
        t.prologue = prologue;
        t.act = sh.act;
        t.head_dim = sh.head_dim;
        t.rep = (prologue == AQ_PRO_PLAIN) ? sh.n_heads / sh.n_kv_heads : 1;
        t.eps = sh.eps;
        wgs += t.wg_count;
        return t;
    };

    int nt = 0;
    for (int l = 0; l < layers; ++l) {
        const aq_block_desc& b = blocks[l];
        float* q = qkv + per_layer * l;
        float* k = q + dq;
        float* v = k + dkv;
        DecodeStage* st = stages + 4 * l;
        int wgs = 0;
        // q, k, v from the normalised residual stream
        const int64_t rows_qkv[3] = {dq, dkv, dkv}, rows_o[1] = {sh.d_model}, rows_mlp[2] = {sh.d_ff, sh.d_ff};
        int part = decode_part_chunks(rows_qkv, 3, (int)aq_num_chunks(sh.d_model));
        st[0].task_begin = nt;
        tasks[nt++] = make(b, 0, dq, sh.d_model, part, q, x, b.norm_attn, AQ_PRO_NORM, wgs);
        tasks[nt++] = make(b, 1, dkv, sh.d_model, part, k, x, b.norm_attn, AQ_PRO_NORM, wgs);
        tasks[nt++] = make(b, 2, dkv, sh.d_model, part, v, x, b.norm_attn, AQ_PRO_NORM, wgs);
        st[0].task_count = 3; st[0].total_wgs = wgs; st[0].clears_gateup = 0;
        // x += W_O a, a = the value head of each query head (attention over the one visible key)
        wgs = 0;
        part = decode_part_chunks(rows_o, 1, (int)aq_num_chunks(dq));
        st[1].task_begin = nt;
        tasks[nt++] = make(b, 3, sh.d_model, dq, part, x, v, nullptr, AQ_PRO_PLAIN, wgs);
        st[1].task_count = 1; st[1].total_wgs = wgs; st[1].clears_gateup = 1;
        // gate, up from the normalised residual stream
        wgs = 0;
        part = decode_part_chunks(rows_mlp, 2, (int)aq_num_chunks(sh.d_model));
        st[2].task_begin = nt;
        tasks[nt++] = make(b, 4, sh.d_ff, sh.d_model, part, gate, x, b.norm_mlp, AQ_PRO_NORM, wgs);
        tasks[nt++] = make(b, 5, sh.d_ff, sh.d_model, part, up, x, b.norm_mlp, AQ_PRO_NORM, wgs);
        st[2].task_count = 2; st[2].total_wgs = wgs; st[2].clears_gateup = 0;
        // x += W_down (act(gate) * up)
        wgs = 0;
        part = decode_part_chunks(rows_o, 1, (int)aq_num_chunks(sh.d_ff));
        st[3].task_begin = nt;
        tasks[nt++] = make(b, 6, sh.d_model, sh.d_ff, part, x, gate, up, AQ_PRO_GATED, wgs);
        st[3].task_count = 1; st[3].total_wgs = wgs; st[3].clears_gateup = 0;
    }
    std::memcpy(base, &h, sizeof(h));
    return AQ_OK;
}

int aq_decode_step(const void* plan_host, void* stream)
{
    if (!plan_host) return AQ_ENULL;
    DecodePlanHeader h;
    std::memcpy(&h, plan_host, sizeof(h));
    if (h.magic != DECODE_MAGIC || h.layers < 1 || h.stages != 4 * h.layers) return AQ_EINVAL;
    const uint8_t* hb = static_cast<const uint8_t*>(plan_host);
    const DecodeStage* stages = reinterpret_cast<const DecodeStage*>(hb + sizeof(DecodePlanHeader));
    const AqStageTask* tasks = reinterpret_cast<const AqStageTask*>(
        hb + sizeof(DecodePlanHeader) + (size_t)h.stages * sizeof(DecodeStage));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (aqk_fill_zero(h.qkv, h.qkv_floats, s) != hipSuccess) return AQ_ELAUNCH;
    for (int i = 0; i < h.stages; ++i) {
        const DecodeStage& st = stages[i];
        if (st.task_count < 1 || st.task_count > AQ_STAGE_MAX_TASKS || st.total_wgs < 1) return AQ_EINVAL;
        AqStageArgs args;
        std::memset(&args, 0, sizeof(args));
        for (int j = 0; j < st.task_count; ++j) args.task[j] = tasks[st.task_begin + j];
        args.count = st.task_count;
        args.zero_ptr = st.clears_gateup ? h.gateup : nullptr;
        args.zero_count = st.clears_gateup ? (int)h.gateup_floats : 0;
        if (aqk_layer_stage(args, st.total_wgs, s) != hipSuccess) return AQ_ELAUNCH;
    }
    return AQ_OK;
}

// ---- HSIC sensitivity ----
// workspace layout for `vars` variables: vars Gram matrices (K*K floats each), vars * K floats of squared norms,
// then (8-byte aligned) vars * K doubles of row sums and 8 doubles of accumulators
static size_t hsic_ws_bytes(int64_t K, int vars)
{
    const size_t f = (size_t)vars * (size_t)K * (size_t)K + (size_t)vars * (size_t)K;
    return ((f * sizeof(float) + 15) / 16) * 16 + ((size_t)vars * (size_t)K + 8) * sizeof(double);
}

size_t aq_hsic_workspace_size(int64_t K)
{
    if (K < 2 || K > 65536) return 0;
    return hsic_ws_bytes(K, 3);
}

int aq_rbf_gram(const float* A, int64_t K, int64_t d, int64_t lda, float gamma, float* G, void* workspace,
                size_t workspace_bytes, void* stream)
{
    if (K < 2 || K > 65536 || d < 1 || d > ((int64_t)1 << 24) || lda < d || !(gamma > 0.f)) return AQ_EINVAL;
    if (!A || !G || !workspace) return AQ_ENULL;
    if (!aligned16(A) || !aligned16(G) || !aligned16(workspace)) return AQ_EALIGN;
    if (workspace_bytes < (size_t)K * sizeof(float)) return AQ_ESIZE;
    return aqk_rbf_gram(A, K, d, lda, gamma, G, static_cast<float*>(workspace), static_cast<hipStream_t>(stream)) ==
                   hipSuccess ? AQ_OK : AQ_ELAUNCH;
}

int aq_hsic_sensitivity(const float* X, int64_t dx, int64_t ldx, float gamma_x, const float* Z, int64_t dz, int64_t ldz,
                        float gamma_z, const float* Y, int64_t dy, int64_t ldy, float gamma_y, int64_t K, double alpha,
                        double beta, double* out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (K < 2 || K > 65536) return AQ_EINVAL;
    const int64_t dmax = (int64_t)1 << 24;
    if (dx < 1 || dz < 1 || dy < 1 || dx > dmax || dz > dmax || dy > dmax || ldx < dx || ldz < dz || ldy < dy) return AQ_EINVAL;
    if (!(gamma_x > 0.f) || !(gamma_z > 0.f) || !(gamma_y > 0.f) || !(alpha >= 0.0) || !(beta >= 0.0)) return AQ_EINVAL;
    if (!X || !Z || !Y || !out || !workspace) return AQ_ENULL;
    if (!aligned16(X) || !aligned16(Z) || !aligned16(Y) || !aligned16(out) || !aligned16(workspace)) return AQ_EALIGN;
    if (workspace_bytes < hsic_ws_bytes(K, 3)) return AQ_ESIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* G = static_cast<float*>(workspace);
    float* sq = G + 3 * K * K;
    const size_t f = (size_t)3 * K * K + (size_t)3 * K;
    double* rs = reinterpret_cast<double*>(static_cast<uint8_t*>(workspace) + ((f * sizeof(float) + 15) / 16) * 16);
    double* acc = rs + 3 * K;
    const float* in[3] = {X, Z, Y};
    const int64_t dd[3] = {dx, dz, dy}, ld[3] = {ldx, ldz, ldy};
    const float gm[3] = {gamma_x, gamma_z, gamma_y};
    for (int v = 0; v < 3; ++v) {
        if (aqk_rbf_gram(in[v], K, dd[v], ld[v], gm[v], G + v * K * K, sq + v * K, s) != hipSuccess) return AQ_ELAUNCH;
        if (aqk_rowsum(G + v * K * K, K, rs + v * K, s) != hipSuccess) return AQ_ELAUNCH;
    }
    if (aqk_zero_f64(acc, 8, s) != hipSuccess) return AQ_ELAUNCH;
    if (aqk_hsic_pair(G, G + K * K, K, rs, rs + K, acc, s) != hipSuccess) return AQ_ELAUNCH;                    // (X, Z)
    if (aqk_hsic_pair(G + K * K, G + 2 * K * K, K, rs + K, rs + 2 * K, acc + 4, s) != hipSuccess) return AQ_ELAUNCH;   // (Z, Y)
    return aqk_hsic_finish(acc, 2, K, alpha, beta, out, s) == hipSuccess ? AQ_OK : AQ_ELAUNCH;
}

int aq_unpack_codes(const void* packed, int64_t N, int64_t K, int bits, int block, uint8_t* codes_u8, void* stream)
{
    int rc = check_matrix(N, K, bits, block);
    if (rc != AQ_OK) return rc;
    if (!packed || !codes_u8) return AQ_ENULL;
    if (!aligned16(packed) || !aligned16(codes_u8)) return AQ_EALIGN;
    return aqk_unpack_codes(packed, N, K, bits, codes_u8, static_cast<hipStream_t>(stream)) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

int aq_dequant_f32(const void* packed, int64_t N, int64_t K, int bits, int block, float* W, void* stream)
{
    int rc = check_matrix(N, K, bits, block);
    if (rc != AQ_OK) return rc;
    if (!packed || !W) return AQ_ENULL;
    if (!aligned16(packed) || !aligned16(W)) return AQ_EALIGN;
    return aqk_dequant(packed, N, K, bits, W, static_cast<hipStream_t>(stream)) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

}  // extern "C"
