// C-ABI of the non-uniform codebook variant of the format (aqc_* entry points): host-side validation, the analysis of
// the caller's table (how it reaches the matrix cores, see aq_gemv_cb.hip) and dispatch.  Nothing here touches the GPU
// before every argument has been checked.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>
#include "../../include/aq.h"
#include "aq_layout.h"
#include "aq_kernels.h"

namespace {

constexpr int64_t CB_MAX_K = 65536;                 // the base format's limit (blobs share aq_packed_size)
constexpr int64_t CB_MAX_N = (int64_t)1 << 24;
constexpr uint64_t IDENTITY_REMAP = 0xFEDCBA9876543210ull;
constexpr uint32_t CB_PLAN_MAGIC = 0x41514331u;     // "AQC1"

struct CbPlanHeader {
    uint32_t magic;
    int32_t count;
    int32_t max_K;
    int32_t total_wgs;
    int32_t mode;            // 4 * form + bits if every product of the list has that form and bit-width; mixed lists:
                             // 1 if every product fits the light mixed kernel, else 0
    int32_t reserved[11];
};
static_assert(sizeof(CbPlanHeader) == 64, "CbPlanHeader must stay 64 bytes");

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_matrix(int64_t N, int64_t K, int bits, int block)
{
    if (bits != 2 && bits != 3 && bits != 4) return AQ_EINVAL;
    if (block != AQ_BLOCK) return AQ_EINVAL;
    if (N < 1 || K < 1 || N > CB_MAX_N || K > CB_MAX_K) return AQ_EINVAL;
    if (K % AQ_BLOCK != 0) return AQ_EINVAL;
    return AQ_OK;
}

// the number the 4-bit pattern s e1 e0 m denotes in E2M1
double e2m1(int p)
{
    const int e = (p >> 1) & 3, m = p & 1;
    const double mag = e == 0 ? 0.5 * m : std::ldexp(1.0 + 0.5 * m, e - 1);
    return (p & 8) ? -mag : mag;
}

// What the kernels need to know of a table.
struct CbInfo {
    int form;              // AQC_FORM_PLANES, AQC_FORM_NATIVE (stored nibble = fp4 pattern of its level / alpha) or
                           // AQC_FORM_SIGNED (stored code = sign bit, then the index into the magnitude table)
    uint64_t remap;        // stored code of canonical code q: (remap >> 4q) & 15
    uint64_t inverse;      // canonical code of stored code c
    float coef[16];        // plane forms: coefficient of the monomial of the (magnitude) bits in S; coef[0] the constant term
    float alpha;
    float stored_level[16];// level of every stored code
};

int analyse(const float* levels, int bits, CbInfo& info)
{
    const int n = 1 << bits;
    std::memset(&info, 0, sizeof(info));
    for (int q = 0; q < n; ++q)
        if (!std::isfinite(levels[q])) return AQ_EINVAL;
    info.remap = info.inverse = IDENTITY_REMAP;
    info.alpha = 1.f;
    for (int q = 0; q < n; ++q) info.stored_level[q] = levels[q];
    if (bits == 4) {
        // alpha * E2M1 in some order (each level within float rounding of alpha * value, every pattern used once)?
        double mx = 0.0;
        for (int q = 0; q < 16; ++q) mx = std::max(mx, std::fabs((double)levels[q]));
        const double alpha = mx / 6.0;
        bool ok = alpha > 0.0 && (double)(float)alpha > 0.0;
        int pattern_of[16];
        bool used[16] = {};
        for (int q = 0; q < 16 && ok; ++q) {
            int found = -1;
            for (int p = 0; p < 16 && found < 0; ++p) {
                if (used[p]) continue;
                const double want = alpha * e2m1(p);
                if (std::fabs((double)levels[q] - want) <= std::ldexp(std::fabs(want), -21) &&
                    (want != 0.0 || levels[q] == 0.f))
                    found = p;
            }
            if (found < 0) ok = false;
            else { used[found] = true; pattern_of[q] = found; }
        }
        if (ok) {
            info.form = AQC_FORM_NATIVE;
            info.alpha = (float)alpha;
            info.remap = info.inverse = 0;
            for (int q = 0; q < 16; ++q) {
                info.remap |= (uint64_t)pattern_of[q] << (4 * q);
                info.inverse |= (uint64_t)q << (4 * pattern_of[q]);
                info.stored_level[pattern_of[q]] = levels[q];
            }
            return AQ_OK;
        }
    }
    // Do the levels come in pairs +v, -v (zeros pair with zeros)?  Then the stored code is (sign, index of the magnitude
    // in ascending order) and only the magnitudes are expanded.
    {
        const int half = n / 2;
        bool used[16] = {};
        int pos[8], neg[8], pairs = 0;
        bool ok = true;
        for (int q = 0; q < n && ok; ++q) {
            if (used[q]) continue;
            int r = -1;
            for (int c = q + 1; c < n && r < 0; ++c)
                if (!used[c] && levels[c] == -levels[q]) r = c;
            if (r < 0) { ok = false; break; }
            used[q] = used[r] = true;
            const bool q_is_pos = levels[q] > 0.f || (levels[q] == 0.f && !std::signbit(levels[q]));
            pos[pairs] = q_is_pos ? q : r;
            neg[pairs] = q_is_pos ? r : q;
            ++pairs;
        }
        if (ok && pairs == half) {
            int order[8];
            for (int i = 0; i < half; ++i) order[i] = i;
            std::stable_sort(order, order + half, [&](int a, int b) { return std::fabs(levels[pos[a]]) < std::fabs(levels[pos[b]]); });
            info.form = AQC_FORM_SIGNED;
            info.remap = info.inverse = 0;
            double a[8];
            for (int m = 0; m < half; ++m) {
                const int P = pos[order[m]], Ng = neg[order[m]], sp = m, sn = half | m;
                info.remap |= ((uint64_t)sp << (4 * P)) | ((uint64_t)sn << (4 * Ng));
                info.inverse |= ((uint64_t)P << (4 * sp)) | ((uint64_t)Ng << (4 * sn));
                info.stored_level[sp] = levels[P];
                info.stored_level[sn] = levels[Ng];
                a[m] = std::fabs((double)levels[P]);
            }
            for (int j = 0; j < bits - 1; ++j)
                for (int S = 0; S < half; ++S)
                    if (S & (1 << j)) a[S] -= a[S ^ (1 << j)];
            for (int S = 0; S < half; ++S) info.coef[S] = (float)a[S];
            return AQ_OK;
        }
    }
    // multilinear coefficients: a_S = sum over T inside S of (-1)^(|S| - |T|) L[T]
    double a[16];
    for (int q = 0; q < n; ++q) a[q] = (double)levels[q];
    for (int j = 0; j < bits; ++j)
        for (int S = 0; S < n; ++S)
            if (S & (1 << j)) a[S] -= a[S ^ (1 << j)];
    for (int S = 0; S < n; ++S) info.coef[S] = (float)a[S];
    return AQ_OK;
}

int check_common(const void* packed, int64_t N, int64_t K, int bits, int block, const float* levels)
{
    int rc = check_matrix(N, K, bits, block);
    if (rc != AQ_OK) return rc;
    if (!packed || !levels) return AQ_ENULL;
    if (!aligned16(packed)) return AQ_EALIGN;
    return AQ_OK;
}

int make_cb_task(const void* packed, int64_t N, int64_t K, int bits, int block, const float* levels, const void* x,
                 int x_dtype, float* y, AqCbTask& t)
{
    int rc = check_common(packed, N, K, bits, block, levels);
    if (rc != AQ_OK) return rc;
    if (x_dtype != AQ_F16 && x_dtype != AQ_BF16) return AQ_EDTYPE;
    if (!x || !y) return AQ_ENULL;
    if (!aligned16(x) || !aligned16(y)) return AQ_EALIGN;
    CbInfo info;
    if ((rc = analyse(levels, bits, info)) != AQ_OK) return rc;
    std::memset(&t, 0, sizeof(t));
    t.g.blob = static_cast<const uint8_t*>(packed);
    t.g.x = static_cast<const uint16_t*>(x);
    t.g.y = y;
    t.g.N = N;
    t.g.K = (int32_t)K;
    t.g.bits = bits;
    t.g.x_dtype = x_dtype;
    t.g.nchunks = (int32_t)aq_num_chunks(K);
    std::memcpy(t.coef, info.coef, sizeof(t.coef));
    t.alpha = info.alpha;
    t.form = info.form;
    aqk_cb_gemv_shape(t);
    return AQ_OK;
}

size_t cb_plan_bytes(int count, int64_t wgs)
{
    return sizeof(CbPlanHeader) + (size_t)count * sizeof(AqCbTask) + (((size_t)wgs * 4 + 15) & ~(size_t)15);
}

}  // namespace

int aqk_cb_stored_levels(const float* levels, int bits, AqCbTable* out)
{
    CbInfo info;
    int rc = analyse(levels, bits, info);
    if (rc != AQ_OK) return rc;
    std::memcpy(out->level, info.stored_level, sizeof(out->level));
    return AQ_OK;
}

extern "C" {

int aqc_table_info(const float* levels, int bits, int* form, float* coef)
{
    if (bits != 2 && bits != 3 && bits != 4) return AQ_EINVAL;
    if (!levels) return AQ_ENULL;
    CbInfo info;
    int rc = analyse(levels, bits, info);
    if (rc != AQ_OK) return rc;
    if (form) *form = info.form;
    if (coef) {
        std::memcpy(coef, info.coef, sizeof(info.coef));
        if (info.form == AQC_FORM_NATIVE) coef[0] = info.alpha;
    }
    return AQ_OK;
}

int aqc_pack_weights(const uint8_t* codes, const uint16_t* scales, const float* levels, int64_t N, int64_t K, int bits,
                     int block, void* packed, size_t packed_bytes, void* stream)
{
    int rc = check_common(packed, N, K, bits, block, levels);
    if (rc != AQ_OK) return rc;
    if (!codes || !scales) return AQ_ENULL;
    if (!aligned16(codes) || !aligned16(scales)) return AQ_EALIGN;
    if (packed_bytes < (size_t)aq_blob_bytes(N, K, bits)) return AQ_ESIZE;
    CbInfo info;
    if ((rc = analyse(levels, bits, info)) != AQ_OK) return rc;
    return aqk_pack_remap(codes, scales, N, K, bits, info.remap, packed, static_cast<hipStream_t>(stream)) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

int aqc_unpack_codes(const void* packed, int64_t N, int64_t K, int bits, int block, const float* levels,
                     uint8_t* codes_u8, void* stream)
{
    int rc = check_common(packed, N, K, bits, block, levels);
    if (rc != AQ_OK) return rc;
    if (!codes_u8) return AQ_ENULL;
    CbInfo info;
    if ((rc = analyse(levels, bits, info)) != AQ_OK) return rc;
    return aqk_cb_unpack_codes(packed, N, K, bits, info.inverse, codes_u8, static_cast<hipStream_t>(stream)) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

int aqc_dequant_f32(const void* packed, int64_t N, int64_t K, int bits, int block, const float* levels, float* W,
                    void* stream)
{
    int rc = check_common(packed, N, K, bits, block, levels);
    if (rc != AQ_OK) return rc;
    if (!W) return AQ_ENULL;
    CbInfo info;
    if ((rc = analyse(levels, bits, info)) != AQ_OK) return rc;
    AqCbTable table;
    std::memcpy(table.level, info.stored_level, sizeof(table.level));
    return aqk_cb_dequant(packed, N, K, bits, table, W, static_cast<hipStream_t>(stream)) == hipSuccess ? AQ_OK : AQ_ELAUNCH;
}

int aqc_qgemv(const void* packed, int64_t N, int64_t K, int bits, int block, const float* levels, const void* x,
              int x_dtype, float* y, void* stream)
{
    AqCbTask t;
    int rc = make_cb_task(packed, N, K, bits, block, levels, x, x_dtype, y, t);
    if (rc != AQ_OK) return rc;
    return aqk_cb_gemv(nullptr, nullptr, 0, t, 4 * t.form + bits, t.g.wg_count, (int)K, static_cast<hipStream_t>(stream)) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

size_t aqc_qgemv_batch_plan_size(const aqc_gemv_desc* descs, int count, int block)
{
    if (count < 1 || !descs) return 0;
    int64_t wgs = 0;
    for (int i = 0; i < count; ++i) {
        const aq_gemv_desc& d = descs[i].product;
        if (check_matrix(d.N, d.K, d.bits, block) != AQ_OK) return 0;
        wgs += aq_num_groups(d.N);
        if (wgs > 0x3FFFFFFF) return 0;
    }
    return cb_plan_bytes(count, wgs);
}

int aqc_qgemv_batch_plan(const aqc_gemv_desc* descs, int count, int block, void* plan_host, size_t plan_bytes)
{
    if (count < 1) return AQ_EINVAL;
    if (!descs || !plan_host) return AQ_ENULL;
    std::vector<AqCbTask> tasks((size_t)count);
    std::vector<int> order((size_t)count);
    for (int i = 0; i < count; ++i) order[i] = i;
    // longest K first (ties in the caller's order): workgroups walk the whole K of their rows
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return descs[a].product.K > descs[b].product.K; });
    int64_t wgs = 0;
    int max_K = 0, mode = 0;
    bool light = true;
    for (int j = 0; j < count; ++j) {
        const aqc_gemv_desc& c = descs[order[j]];
        const aq_gemv_desc& d = c.product;
        int rc = make_cb_task(d.packed, d.N, d.K, d.bits, block, c.levels, d.x, d.x_dtype, d.y, tasks[j]);
        if (rc != AQ_OK) return rc;
        tasks[j].g.wg_begin = (int32_t)wgs;
        wgs += tasks[j].g.wg_count;
        if (wgs > 0x3FFFFFFF) return AQ_EINVAL;
        if (d.K > max_K) max_K = (int)d.K;
        const int m = 4 * tasks[j].form + d.bits;
        mode = j == 0 ? m : (mode == m ? m : 0);
        light = light && aqk_cb_light(tasks[j].form, d.bits);
    }
    if (mode == 0 && light) mode = 1;
    if (plan_bytes < cb_plan_bytes(count, wgs)) return AQ_ESIZE;
    CbPlanHeader h;
    std::memset(&h, 0, sizeof(h));
    h.magic = CB_PLAN_MAGIC;
    h.count = count;
    h.max_K = max_K;
    h.total_wgs = (int32_t)wgs;
    h.mode = mode;
    uint8_t* base = static_cast<uint8_t*>(plan_host);
    std::memcpy(base, &h, sizeof(h));
    std::memcpy(base + sizeof(h), tasks.data(), (size_t)count * sizeof(AqCbTask));
    int32_t* wg_task = reinterpret_cast<int32_t*>(base + sizeof(h) + (size_t)count * sizeof(AqCbTask));
    for (int j = 0; j < count; ++j)
        for (int w = 0; w < tasks[j].g.wg_count; ++w) wg_task[tasks[j].g.wg_begin + w] = j;
    return AQ_OK;
}

int aqc_qgemv_batch(const void* plan_host, const void* plan_dev, void* stream)
{
    if (!plan_host || !plan_dev) return AQ_ENULL;
    if (!aligned16(plan_dev)) return AQ_EALIGN;
    CbPlanHeader h;
    std::memcpy(&h, plan_host, sizeof(h));
    if (h.magic != CB_PLAN_MAGIC || h.count < 1 || h.total_wgs < 1 || h.max_K < AQ_BLOCK || h.mode < 0 || h.mode > 12)
        return AQ_EINVAL;
    const uint8_t* dev = static_cast<const uint8_t*>(plan_dev);
    const AqCbTask* tasks = reinterpret_cast<const AqCbTask*>(dev + sizeof(CbPlanHeader));
    const int32_t* wg_task = reinterpret_cast<const int32_t*>(dev + sizeof(CbPlanHeader) + (size_t)h.count * sizeof(AqCbTask));
    AqCbTask none;
    std::memset(&none, 0, sizeof(none));
    return aqk_cb_gemv(tasks, wg_task, h.count, none, h.mode, h.total_wgs, h.max_K, static_cast<hipStream_t>(stream)) == hipSuccess
               ? AQ_OK : AQ_ELAUNCH;
}

}  // extern "C"
