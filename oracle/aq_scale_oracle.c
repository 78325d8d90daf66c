/*
 * CPU oracle for the block-level scale optimisation (TEST INFRASTRUCTURE, not product code).
 *
 * Plain, slow, fp64, one block after the other; shares no code, header, table or helper
 * with the GPU library.  Only the tests, the smoke check and the bench's cpu_baseline leg
 * may call it.
 *
 * What it follows (Section 4.2, paragraph "Block-Level Scale Optimization"):
 *   - per-element sensitivity  omega_i = F_ii * sqrt(sigma_b^2 + w_i^2), sigma_b^2 the mean
 *     squared weight of the block (Eq. 10, left);
 *   - objective  Phi_b(s, q) = sum_i omega_i (w_i - s q_i)^2  (Eq. 10, right);
 *   - the two alternating steps of Eq. 11: with s fixed every q_i is the codebook entry
 *     nearest to w_i / s; with q fixed s = sum(omega w q) / sum(omega q^2).
 * Readings where the paragraph is silent (they are the library's too, listed in its design notes):
 *   - codebook Q_n = the integers -2^(bits-1) .. 2^(bits-1)-1, i.e. (stored code - z) of the
 *     block format with its fixed offset z = 2^(bits-1) (Eq. 10 has no offset term);
 *   - start: s = max|w_i| / 2^(bits-1) (the most negative code reaches -max|w|); an all-zero
 *     block keeps s = 0 and every code at zero;
 *   - "a few rounds" is the parameter `rounds`; a round = one assignment + one scale update;
 *     the loop stops early when sum(omega w q) <= 0 or sum(omega q^2) = 0 (nothing to fit);
 *   - a tie between two codebook entries goes to the smaller one (first minimiser);
 *   - the stored scale is d = binary16(round-to-nearest-even(s)), capped at 65504; the stored
 *     codes are one more assignment against d itself, so that (q, d) is what Eq. 1 decodes.
 *
 * Pins (tests/test_scale_oracle_pins.py): a hand-worked equal-magnitude block, rounds = 0
 * against the Eq. 1 argmin of aq_oracle.c, Phi non-increasing along the trace, stationarity
 * of the scale update, exhaustive search over all code vectors of a 4-element block,
 * double -> binary16 rounding against numpy.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

/* double -> binary16 bit pattern, round to nearest, ties to even; |x| >= 65520 -> infinity */
uint16_t aqs_f64_to_f16(double x)
{
    uint16_t sign = (uint16_t)(signbit(x) ? 0x8000u : 0u);
    double a = fabs(x);
    if (isnan(a)) return (uint16_t)(sign | 0x7E00u);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7C00u);          /* rounds to 2^16: overflow */
    if (a < ldexp(1.0, -25)) return sign;                          /* below half the smallest subnormal */
    int e;
    (void)frexp(a, &e);                                            /* a = m 2^e, m in [0.5, 1) */
    int ulp_exp = (e - 1 < -14 ? -14 : e - 1) - 10;                /* exponent of one unit in the last place */
    double scaled = ldexp(a, -ulp_exp);                            /* exact: a in units of the last place */
    double fl = floor(scaled), frac = scaled - fl;
    if (frac > 0.5 || (frac == 0.5 && fmod(fl, 2.0) == 1.0)) fl += 1.0;
    double r = ldexp(fl, ulp_exp);                                 /* the rounded value, exactly representable */
    if (r == 0.0) return sign;
    if (r < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)ldexp(r, 24));      /* subnormal */
    (void)frexp(r, &e);
    uint16_t mant = (uint16_t)(ldexp(r, 11 - e) - 1024.0);         /* 10 fraction bits */
    return (uint16_t)(sign | (uint16_t)((e - 1 + 15) << 10) | mant);
}

static double f16_bits_to_f64(uint16_t h)
{
    int e = (h >> 10) & 31, m = h & 1023;
    double v = e == 0 ? ldexp((double)m, -24) : ldexp(1.0 + m / 1024.0, e - 15);
    return (h & 0x8000u) ? -v : v;
}

/* Eq. 10 right: Phi_b for one block */
static double phi(const double *w, const double *om, const int *q, int B, double s)
{
    double acc = 0.0;
    for (int i = 0; i < B; ++i) { double r = w[i] - s * q[i]; acc += om[i] * r * r; }
    return acc;
}

/* Eq. 11 left: nearest codebook entry to w_i / s, the smaller entry on a tie */
static void assign(const double *w, int B, double s, int qmin, int qmax, int *q)
{
    for (int i = 0; i < B; ++i) {
        double t = w[i] / s;
        int best = qmin;
        double best_err = fabs(t - (double)qmin);
        for (int c = qmin + 1; c <= qmax; ++c) {
            double err = fabs(t - (double)c);
            if (err < best_err) { best_err = err; best = c; }
        }
        q[i] = best;
    }
}

/*
 * W, F: float[N][K] (F may be NULL: F_ii = 1).  Outputs: codes uint8[N][K] = q + z, scales uint16[N][K/block]
 * binary16 bit patterns.  trace (may be NULL): double[N*K/block][2*rounds + 3] holding, per block,
 * Phi after the first assignment, then after each scale update and each re-assignment in turn (entries of
 * rounds not run repeat the last value), and last Phi of the stored pair (d, q).
 */
void aqs_optimize(const float *W, const float *F, int64_t N, int64_t K, int bits, int block, int rounds,
                  uint8_t *codes, uint16_t *scales, double *trace)
{
    const int B = block, z = 1 << (bits - 1), qmin = -z, qmax = z - 1;
    const int64_t nb = K / B;
    double *w = malloc(sizeof(double) * B), *om = malloc(sizeof(double) * B);
    int *q = malloc(sizeof(int) * B);
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < nb; ++j) {
            const float *wp = W + n * K + j * B;
            const float *fp = F ? F + n * K + j * B : 0;
            double *tr = trace ? trace + (n * nb + j) * (2 * rounds + 3) : 0;
            int ntr = 0;
            double sigma2 = 0.0, amax = 0.0;
            for (int i = 0; i < B; ++i) {
                w[i] = (double)wp[i];
                sigma2 += w[i] * w[i];
                if (fabs(w[i]) > amax) amax = fabs(w[i]);
            }
            sigma2 /= (double)B;
            for (int i = 0; i < B; ++i) om[i] = (fp ? (double)fp[i] : 1.0) * sqrt(sigma2 + w[i] * w[i]);   /* Eq. 10 left */
            double s = amax / (double)z;
            for (int i = 0; i < B; ++i) q[i] = 0;
            if (s > 0.0) {
                assign(w, B, s, qmin, qmax, q);
                if (tr) tr[ntr++] = phi(w, om, q, B, s);
                for (int r = 0; r < rounds; ++r) {
                    double num = 0.0, den = 0.0;
                    for (int i = 0; i < B; ++i) { num += om[i] * w[i] * q[i]; den += om[i] * (double)q[i] * (double)q[i]; }
                    if (!(num > 0.0) || !(den > 0.0)) break;
                    s = num / den;                                  /* Eq. 11 right */
                    if (tr) tr[ntr++] = phi(w, om, q, B, s);
                    assign(w, B, s, qmin, qmax, q);                 /* Eq. 11 left */
                    if (tr) tr[ntr++] = phi(w, om, q, B, s);
                }
            }
            uint16_t d_bits = aqs_f64_to_f16(s > 65504.0 ? 65504.0 : s);
            double d = f16_bits_to_f64(d_bits);
            if (d > 0.0) assign(w, B, d, qmin, qmax, q);
            else for (int i = 0; i < B; ++i) q[i] = 0;
            if (tr) {
                double last = ntr ? tr[ntr - 1] : phi(w, om, q, B, 0.0);
                while (ntr < 2 * rounds + 2) tr[ntr++] = last;
                tr[ntr] = phi(w, om, q, B, d);
            }
            scales[n * nb + j] = d_bits;
            for (int i = 0; i < B; ++i) codes[n * K + j * B + i] = (uint8_t)(q[i] + z);
        }
    free(w); free(om); free(q);
}
