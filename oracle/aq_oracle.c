/*
 * CPU oracle for the block-quantised matmul (TEST INFRASTRUCTURE, not product code).
 *
 * Plain, slow, fp64.  It is the written-out definition of what the GPU library
 * must compute and shares no code, header, table or helper with it.  Only the
 * tests, the smoke check and the bench's cpu_baseline leg may call it.
 *
 * What it follows:
 *   - block format and dequantisation  w_hat = s_b (q - z_b): Eq. 1, Section 3
 *     ("Weight quantization"), with the readings fixed by the workload
 *     definition: blocks of B = 32 consecutive elements along K inside a row of
 *     W[N, K]; codes q in {0..2^b-1}; z_b = 2^(b-1), not stored; s_b = d, one
 *     fp16 value per block; per block the 32 codes form one little-endian
 *     bitstream of 4b bytes (code i occupies stream bits i*b .. i*b+b-1, stream
 *     bit t is bit t%8 of byte t/8);
 *   - nearest-code assignment q = argmin_q |w - s (q - z)|: Eq. 1 (right part);
 *   - one bit-width per matrix, uniform inside it: Section 1 / Section 4.1;
 *   - activations stay at half precision (fp16 or bf16 values, used exactly):
 *     Appendix "Limitations";
 *   - y = x W_hat^T is the ordinary matrix product, summed in ascending k.
 *
 * Pins (tests/test_oracle_pins.py): hand-worked bitstreams, all-pattern fp16 /
 * bf16 conversion against numpy, grid round trip through the Eq. 1 argmin,
 * exact-rational brute force on 8x32, integer matmul special case, the
 * footprint arithmetic of Table 1.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>

/* ---- scalar conversions (IEEE binary16 and bfloat16 bit patterns -> double) ---- */

double aqo_f16_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int m = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);                 /* zero and subnormals: m * 2^-24 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return sign ? -v : v;
}

double aqo_bf16_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 7) & 0xFF;
    int m = h & 0x7F;
    double v;
    if (e == 0)
        v = ldexp((double)m, -133);                /* m/128 * 2^-126 */
    else if (e == 255)
        v = m ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)m / 128.0, e - 127);
    return sign ? -v : v;
}

void aqo_f16_array_to_f64(const uint16_t *h, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = aqo_f16_to_f64(h[i]);
}

void aqo_bf16_array_to_f64(const uint16_t *h, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = aqo_bf16_to_f64(h[i]);
}

/* ---- bitstream <-> codes ---- */

static int stream_bit(const uint8_t *bytes, int64_t t)
{
    return (bytes[t >> 3] >> (t & 7)) & 1;
}

/* stream uint8[N][K/block][block*bits/8]  ->  q uint8[N][K] */
void aqo_unpack(const uint8_t *stream, int64_t N, int64_t K, int bits, int block, uint8_t *q)
{
    int64_t nb = K / block;
    int64_t bpb = (int64_t)block * bits / 8;       /* bytes per block */
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < nb; ++j) {
            const uint8_t *blk = stream + (n * nb + j) * bpb;
            for (int i = 0; i < block; ++i) {
                int code = 0;
                for (int u = 0; u < bits; ++u)
                    code |= stream_bit(blk, (int64_t)i * bits + u) << u;
                q[n * K + j * block + i] = (uint8_t)code;
            }
        }
}

/* q uint8[N][K] -> stream; inverse of aqo_unpack, used by the round-trip pin */
void aqo_pack(const uint8_t *q, int64_t N, int64_t K, int bits, int block, uint8_t *stream)
{
    int64_t nb = K / block;
    int64_t bpb = (int64_t)block * bits / 8;
    for (int64_t t = 0; t < N * nb * bpb; ++t) stream[t] = 0;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < nb; ++j) {
            uint8_t *blk = stream + (n * nb + j) * bpb;
            for (int i = 0; i < block; ++i) {
                int code = q[n * K + j * block + i];
                for (int u = 0; u < bits; ++u) {
                    int64_t t = (int64_t)i * bits + u;
                    blk[t >> 3] |= (uint8_t)(((code >> u) & 1) << (t & 7));
                }
            }
        }
}

/* ---- Eq. 1 ---- */

/* left part: w_hat = s (q - z), z = 2^(bits-1), s = the block's fp16 scale; W double[N][K] */
void aqo_dequant(const uint8_t *stream, const uint16_t *scales, int64_t N, int64_t K,
                 int bits, int block, double *W)
{
    int64_t nb = K / block;
    int64_t bpb = (int64_t)block * bits / 8;
    int z = 1 << (bits - 1);
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < nb; ++j) {
            const uint8_t *blk = stream + (n * nb + j) * bpb;
            double s = aqo_f16_to_f64(scales[n * nb + j]);
            for (int i = 0; i < block; ++i) {
                int code = 0;
                for (int u = 0; u < bits; ++u)
                    code |= stream_bit(blk, (int64_t)i * bits + u) << u;
                W[n * K + j * block + i] = s * (double)(code - z);
            }
        }
}

/* right part: q_i = argmin over the uniform codebook {0..2^bits-1} of |w_i - s (q - z)|;
 * the first minimiser wins a tie */
void aqo_rtn_codes(const double *w, int64_t n, double s, double z, int bits, uint8_t *q)
{
    int levels = 1 << bits;
    for (int64_t i = 0; i < n; ++i) {
        int best = 0;
        double best_err = fabs(w[i] - s * (0.0 - z));
        for (int c = 1; c < levels; ++c) {
            double err = fabs(w[i] - s * ((double)c - z));
            if (err < best_err) { best_err = err; best = c; }
        }
        q[i] = (uint8_t)best;
    }
}

/* ---- the matrix product  Y[M][N] = X[M][K] . W[N][K]^T, ascending k ---- */
void aqo_matmul_nt(const double *X, const double *W, int64_t M, int64_t N, int64_t K, double *Y)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += X[m * K + k] * W[n * K + k];
            Y[m * N + n] = acc;
        }
}

/* ---- whole path: unpack -> dequantise (fp64) -> matmul, activations given as
 *      fp16 (x_is_bf16 = 0) or bf16 (x_is_bf16 = 1) bit patterns.
 *      scratch_W double[N*K], scratch_X double[M*K] are caller-provided. ---- */
void aqo_qmatmul(const uint8_t *stream, const uint16_t *scales, int64_t N, int64_t K,
                 int bits, int block, const uint16_t *X, int64_t M, int x_is_bf16,
                 double *scratch_W, double *scratch_X, double *Y)
{
    aqo_dequant(stream, scales, N, K, bits, block, scratch_W);
    if (x_is_bf16) aqo_bf16_array_to_f64(X, M * K, scratch_X);
    else           aqo_f16_array_to_f64(X, M * K, scratch_X);
    aqo_matmul_nt(scratch_X, scratch_W, M, N, K, Y);
}

/* ---- storage accounting ---- */

/* bytes of the canonical form: per block block*bits/8 code bytes + one 2-byte scale */
int64_t aqo_stored_bytes(int64_t N, int64_t K, int bits, int block)
{
    int64_t nb = K / block;
    return N * nb * ((int64_t)block * bits / 8 + 2);
}

int aqo_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
