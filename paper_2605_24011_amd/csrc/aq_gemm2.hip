// Prefill with exact products for blobs of the two-level variant of the format, w = D a q - M c (Eq. 1 in its general
// form: a stored scale and a stored zero point per block): the kernel of aq_gemm.hip with FMT = 1.  Per block of 32 k
// and 16 x 16 tile one MFMA gives P[m][n] = sum_k q[n, k] x[m, k] on exact small integers, one more per m-tile and block
// (against an operand of ones) gives X_b[m] = sum_k x[m, k], and the accumulators take
//     (D a)[n, b] * P[m][n] - (M c)[n, b] * X_b[m]
// in fp32; D a and M c are exact there (11 + 4 significant bits).  No weight is ever rounded.
#include "aq_gemm_kernel.h"

// One instantiation per activation type and m-tile count: the bit-width is a branch per workgroup (as in mixed lists
// of the base format) and the wavefronts always split m only (at M <= 64 most of them just unpack their unit).
// x_dtype is common to all tasks of a launch; tasks from make_gemm_task with nsplit = 1, X re-tiled by aqk_retile
// without conversion.
hipError_t aqk2_gemm(const AqGemmTask* tasks_dev, int count, const AqGemmTask& single, int x_dtype, int A,
                     int total_wgs, const void* workspace, hipStream_t s)
{
    const size_t lds = gm_lds_bytes(1);
    const dim3 grid((unsigned)total_wgs), block(GM_THREADS);
    const uint8_t* ws = static_cast<const uint8_t*>(workspace);
#define AQ_GO(XBF, AA)                                                                              \
    do {                                                                                            \
        auto k = qgemm_kernel<0, XBF, AA, 1, false, 1>;                                             \
        if (aqk_allow_lds(reinterpret_cast<const void*>(k), lds) != hipSuccess) return hipErrorInvalidValue; \
        hipLaunchKernelGGL(k, grid, block, lds, s, tasks_dev, count, single, ws);                   \
    } while (0)
    if (x_dtype == 2) {
        if (A == 1) AQ_GO(true, 1); else if (A == 2) AQ_GO(true, 2); else AQ_GO(true, 3);
    } else {
        if (A == 1) AQ_GO(false, 1); else if (A == 2) AQ_GO(false, 2); else AQ_GO(false, 3);
    }
#undef AQ_GO
    return hipGetLastError();
}
