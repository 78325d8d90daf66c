/* Runs every exported function of the C oracles on small inputs whose buffers are heap blocks of exactly the
 * documented size, so that AddressSanitizer sees any access outside them and UndefinedBehaviorSanitizer any shift,
 * overflow or conversion the C standard leaves open.  Built and run by tests/test_sanitizers.py with
 *     gcc -fsanitize=address,undefined -fno-sanitize-recover=all
 * Prints "ok" and exits 0 when nothing was reported. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double aqo_f16_to_f64(uint16_t h);
double aqo_bf16_to_f64(uint16_t h);
void aqo_f16_array_to_f64(const uint16_t *h, int64_t n, double *out);
void aqo_bf16_array_to_f64(const uint16_t *h, int64_t n, double *out);
void aqo_unpack(const uint8_t *stream, int64_t N, int64_t K, int bits, int block, uint8_t *q);
void aqo_pack(const uint8_t *q, int64_t N, int64_t K, int bits, int block, uint8_t *stream);
void aqo_dequant(const uint8_t *stream, const uint16_t *scales, int64_t N, int64_t K, int bits, int block, double *W);
void aqo_rtn_codes(const double *w, int64_t n, double s, double z, int bits, uint8_t *q);
void aqo_matmul_nt(const double *X, const double *W, int64_t M, int64_t N, int64_t K, double *Y);
void aqo_qmatmul(const uint8_t *stream, const uint16_t *scales, int64_t N, int64_t K, int bits, int block,
                 const uint16_t *X, int64_t M, int x_is_bf16, double *scratch_W, double *scratch_X, double *Y);
int64_t aqo_stored_bytes(int64_t N, int64_t K, int bits, int block);
int aqo_num_threads(void);
uint16_t aqs_f64_to_f16(double x);
void aqs_optimize(const float *W, const float *F, int64_t N, int64_t K, int bits, int block, int rounds,
                  uint8_t *codes, uint16_t *scales, double *trace);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 32);
}
static double unit(void) { return (rnd() + 0.5) / 4294967296.0 * 2.0 - 1.0; }

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main(void)
{
    /* all 65536 patterns of both 16-bit formats, and the round trip of the binary16 rounding */
    for (uint32_t h = 0; h < 65536; ++h) {
        const double a = aqo_f16_to_f64((uint16_t)h), b = aqo_bf16_to_f64((uint16_t)h);
        if (a == a && !isinf(a)) CHECK(aqs_f64_to_f16(a) == (uint16_t)h || a == 0.0);
        (void)b;
    }
    aqs_f64_to_f16(1e300); aqs_f64_to_f16(-1e-300); aqs_f64_to_f16(NAN); aqs_f64_to_f16(65519.9);

    const int block = 32;
    const int64_t shapes[4][3] = {{1, 32, 1}, {5, 96, 3}, {17, 256, 2}, {3, 1504, 1}};     /* N, K, M */
    for (int si = 0; si < 4; ++si)
        for (int bits = 2; bits <= 4; ++bits) {
            const int64_t N = shapes[si][0], K = shapes[si][1], M = shapes[si][2], nb = K / block;
            const int64_t sbytes = N * nb * (block * bits / 8);
            CHECK(aqo_stored_bytes(N, K, bits, block) == sbytes + 2 * N * nb);
            uint8_t *q = malloc(N * K), *q2 = malloc(N * K), *stream = malloc(sbytes);
            uint16_t *scales = malloc(sizeof(uint16_t) * N * nb), *X = malloc(sizeof(uint16_t) * M * K);
            double *W = malloc(sizeof(double) * N * K), *Xd = malloc(sizeof(double) * M * K), *Y = malloc(sizeof(double) * M * N);
            double *Y2 = malloc(sizeof(double) * M * N);
            for (int64_t i = 0; i < N * K; ++i) q[i] = (uint8_t)(rnd() % (1u << bits));
            for (int64_t i = 0; i < N * nb; ++i) scales[i] = aqs_f64_to_f16(unit() * 0.05);
            for (int64_t i = 0; i < M * K; ++i) X[i] = aqs_f64_to_f16(unit() * 3.0);
            aqo_pack(q, N, K, bits, block, stream);
            aqo_unpack(stream, N, K, bits, block, q2);
            CHECK(memcmp(q, q2, N * K) == 0);
            aqo_dequant(stream, scales, N, K, bits, block, W);
            for (int bf = 0; bf < 2; ++bf) {
                aqo_qmatmul(stream, scales, N, K, bits, block, X, M, bf, W, Xd, Y);
                aqo_matmul_nt(Xd, W, M, N, K, Y2);
                CHECK(memcmp(Y, Y2, sizeof(double) * M * N) == 0);
            }
            aqo_rtn_codes(W, K, 0.01, (double)(1 << (bits - 1)), bits, q2);
            free(q); free(q2); free(stream); free(scales); free(X); free(W); free(Xd); free(Y); free(Y2);
        }

    /* scale optimiser: with and without sensitivities, with and without a trace, zero and constant blocks */
    for (int bits = 2; bits <= 4; ++bits)
        for (int rounds = 0; rounds <= 5; rounds += 5) {
            const int64_t N = 6, K = 160, nb = K / block;
            float *Wf = malloc(sizeof(float) * N * K), *F = malloc(sizeof(float) * N * K);
            uint8_t *codes = malloc(N * K);
            uint16_t *sc = malloc(sizeof(uint16_t) * N * nb);
            double *trace = malloc(sizeof(double) * N * nb * (2 * rounds + 3));
            for (int64_t i = 0; i < N * K; ++i) { Wf[i] = (float)(unit() * 0.02); F[i] = (float)(unit() * unit()) + 1e-6f; }
            for (int i = 0; i < block; ++i) { Wf[i] = 0.f; Wf[block + i] = 0.5f; Wf[2 * block + i] = 1e30f; }
            aqs_optimize(Wf, F, N, K, bits, block, rounds, codes, sc, trace);
            aqs_optimize(Wf, NULL, N, K, bits, block, rounds, codes, sc, NULL);
            for (int64_t i = 0; i < N * K; ++i) CHECK(codes[i] < (1u << bits));
            free(Wf); free(F); free(codes); free(sc); free(trace);
        }
    CHECK(aqo_num_threads() >= 1);
    puts("ok");
    return 0;
}
