/*
 * aq.h -- C ABI of the block-quantised matmul library for AMD MI355X (gfx950).
 *
 * The library multiplies activations by a weight matrix W[N, K] (N output
 * features, K input features, y = x W^T) that is stored in the block
 * quantisation format of Eq. 1 (Section 3, "Weight quantization"), with one
 * bit-width per matrix (Section 1 and Section 4.1: the bit-width varies across
 * matrices and is uniform inside each, so one dense kernel serves a matrix):
 *
 *     w_hat[n, k] = d[n, k/32] * (q[n, k] - 2^(bits-1)),
 *
 *   bits  in {2, 3, 4}         -- the matrix's bit-width (n of Eq. 1's n-bit quantiser)
 *   block =  32                -- B of Eq. 1; blocks run along K inside a row of W
 *   q     in {0 .. 2^bits - 1} -- the codes (uniform codebook Q_n)
 *   d                          -- s_b of Eq. 1, one IEEE binary16 value per block
 *   z_b   = 2^(bits-1)         -- fixed, not stored
 *
 * Canonical ("interchange") form handed to aq_pack_weights:
 *   codes  uint8  [N][K/32][4*bits] : per block one little-endian bitstream; code i
 *          of the block occupies stream bits i*bits .. i*bits+bits-1, stream bit t is
 *          bit (t % 8) of byte (t / 8).  4-bit: two codes per byte, low nibble first;
 *          3-bit: 12 bytes per block, codes straddle bytes; blocks never share a byte.
 *   scales uint16 [N][K/32]         : binary16 bit patterns.
 *
 * Conventions for every entry point
 *   - Pointers marked DEVICE are device (HBM) addresses, 16-byte aligned; pointers
 *     marked HOST are ordinary host memory.  The caller owns every buffer; the library
 *     allocates and frees no DEVICE memory and keeps no state between calls (the plan
 *     builders and aq_allocate_bits use temporary host memory, std::vector, while they run).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work on it and never synchronise.
 *   - Return value: AQ_OK (0) or a negative AQ_E* code.  Arguments are validated on
 *     the host before anything is launched; on error nothing has been enqueued.
 *   - Activations are half precision (Appendix "Limitations": weight-only quantisation,
 *     activations stay at half precision): AQ_F16 or AQ_BF16 bit patterns.  Outputs are
 *     fp32.  Accumulation is fp32.
 */
#ifndef AQ_H
#define AQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AQ_OK        0
#define AQ_EINVAL   (-1)  /* bits not in {2,3,4}; block != 32; N, K or M < 1; K % 32 != 0; K > 65536; ld too small; count < 1; unknown flags */
#define AQ_ENULL    (-2)  /* a required pointer is NULL */
#define AQ_EALIGN   (-3)  /* a device pointer is not 16-byte aligned */
#define AQ_ESIZE    (-4)  /* a caller-provided buffer is too small */
#define AQ_EDTYPE   (-5)  /* activation dtype is neither AQ_F16 nor AQ_BF16 */
#define AQ_ELAUNCH  (-6)  /* the HIP runtime reported an error at launch */

#define AQ_F16   1
#define AQ_BF16  2

/* Text for a status code (static storage, never NULL). */
const char* aq_status_string(int status);

/* Bytes of the packed device blob of an N x K matrix, 0 if the arguments are invalid.
 * The blob stores exactly the canonical information (bits/8 + 1/16 bytes per weight)
 * re-tiled for the kernels, with N rounded up to 128 and K to 256, plus 256 bytes of
 * per-matrix summary (the largest |d|); its layout is private to this build of the library. */
size_t aq_packed_size(int64_t N, int64_t K, int bits, int block);

/* Eq. 1's stored form -> device blob (re-tiling only, no value changes).
 *   codes   DEVICE uint8  [N][K/32][4*bits]   canonical bitstream (see above)
 *   scales  DEVICE uint16 [N][K/32]           binary16 bit patterns
 *   packed  DEVICE, packed_bytes >= aq_packed_size(N, K, bits, block); written entirely.
 * One-off per matrix (the serialisation step of Appendix D), not on the timed path. */
int aq_pack_weights(const uint8_t* codes, const uint16_t* scales,
                    int64_t N, int64_t K, int bits, int block,
                    void* packed, size_t packed_bytes, void* stream);

/* Decode (batch 1): y[n] = sum_k x[k] * w_hat[n, k], unpack + dequantise fused into the
 * product ("dequantize on the fly inside a hand-written kernel", Appendix D; Eq. 1).
 *   packed  DEVICE blob from aq_pack_weights with the same (N, K, bits, block)
 *   x       DEVICE uint16 [K]  activations, x_dtype = AQ_F16 or AQ_BF16
 *   y       DEVICE float  [N]  overwritten */
int aq_qgemv(const void* packed, int64_t N, int64_t K, int bits, int block,
             const void* x, int x_dtype, float* y, void* stream);

/* A stream of independent decode products in ONE launch: the per-matrix bit-width of
 * Section 4.1 selects the code path per descriptor ("every matmul dispatches to one
 * dense kernel", Section 1); used for a whole backbone pass (7 matrices x L layers).
 * Step 1 (host only): aq_qgemv_batch_plan turns `count` descriptors into a plan image
 *   of aq_qgemv_batch_plan_size(descs, count, block) bytes in HOST memory `plan_host` (0: an invalid descriptor;
 *   the image holds one record per product and one table entry per workgroup of the launch).
 * Step 2: the caller copies that image to 16-byte-aligned DEVICE memory `plan_dev`.
 * Step 3: aq_qgemv_batch(plan_host, plan_dev, stream) launches (one kernel launch); it may be
 *   repeated. */
typedef struct aq_gemv_desc {
    const void* packed;   /* DEVICE blob */
    const void* x;        /* DEVICE uint16 [K] */
    float*      y;        /* DEVICE float [N] */
    int64_t     N, K;
    int32_t     bits;     /* 2, 3 or 4 */
    int32_t     x_dtype;  /* AQ_F16 or AQ_BF16 */
} aq_gemv_desc;

size_t aq_qgemv_batch_plan_size(const aq_gemv_desc* descs /*HOST*/, int count, int block);
int aq_qgemv_batch_plan(const aq_gemv_desc* descs /*HOST*/, int count, int block,
                        void* plan_host, size_t plan_bytes);
int aq_qgemv_batch(const void* plan_host, const void* plan_dev, void* stream);

/* Prefill: Y[m, n] = sum_k X[m, k] * w_hat[n, k] for M rows of activations, on the matrix cores (Eq. 1 fused
 * into the product; Appendix D, "dequantize on the fly").  Two entry points, one per way Eq. 1's scale meets
 * the product; arguments, workspace and errors are the same:
 *   aq_qgemm       code tiles are unpacked to the exact small integers (q - 2^(bits-1)) in LDS and the fp16
 *       block scale d multiplies each block's partial sum in fp32 (Eq. 1 with the factor d taken out of
 *       the block's sum): no weight is ever rounded, only fp32 summation rounds (rel-L2 ~1e-7).  One fp32
 *       multiply-add per 32 matrix-core multiply-adds: the vector ALU bounds the speed.  For M <= 64, where the
 *       weight stream bounds the speed, the same precision is reached another way: d * (q - 2^(bits-1)) goes to the
 *       matrix cores as the exact sum of two binary16 numbers (two multiply-adds per weight) in the streaming
 *       kernel described under aq_qgemm_fast; bf16 activations are converted to binary16 per row as there.
 *   aq_qgemm_fast  w_hat = d * (q - 2^(bits-1)) is formed in binary16 while unpacking and the matrix cores
 *       accumulate over all of K.  The product is exact for bits = 2; for
 *       bits = 3, 4 some codes need up to 14 significant bits and are rounded to binary16's 11
 *       (relative error <= 2^-12 per weight, rel-L2 of Y ~1e-4).  bf16 activations are first converted to
 *       binary16 with one power-of-two factor per row (exact unless an element is 2^38 times smaller than
 *       its row's largest).  A matrix whose largest |d| * 2^(bits-1) would overflow binary16 is computed as
 *       in aq_qgemm (decided on the device from the blob) by the shared-role kernel; the producer /
 *       consumer kernel that serves M = 300-like sizes scales d by a power of two instead, as below.  For M <= 64 the product runs in a kernel
 *       bound by the weight stream (wavefronts keep their packed tiles in registers over all of K; weights
 *       never pass through LDS); there such a matrix has every scale multiplied by one power of two
 *       2^-s first (s <= 4) and the result by 2^s, same error bound unless d < 2^(s-14).
 *   X   DEVICE uint16 [M][ldx], ldx >= K and ldx % 8 == 0, x_dtype = AQ_BF16 or AQ_F16
 *   Y   DEVICE float  [M][ldy], ldy >= N, overwritten for m < M, n < N (a call on a matrix with few rows and a deep K
 *       clears these elements in its first launch and adds two partial sums over halves of K to each with fp32
 *       atomics: the same bits on every call, since two terms sum alike in either order)
 *   workspace DEVICE, 16-byte aligned, workspace_bytes >= aq_qgemm_workspace_size(M, N, K, bits)
 *       (2 bytes per element of X with M rounded up to 16, plus 4 bytes per row).  The call first copies
 *       X into it in the order the matrix cores read their operands, then runs the product from that
 *       copy.  Contents need no initialisation and are scratch: calls that share a workspace must be
 *       ordered on one stream.
 * The list form below (aq_qgemm_batch_plan) takes the choice as `flags`: AQ_GEMM_EXACT = the arithmetic of
 * aq_qgemm, AQ_GEMM_FAST = that of aq_qgemm_fast. */
#define AQ_GEMM_EXACT 0
#define AQ_GEMM_FAST  1
size_t aq_qgemm_workspace_size(int64_t M, int64_t N, int64_t K, int bits);
int aq_qgemm(const void* packed, int64_t N, int64_t K, int bits, int block,
             const void* X, int64_t M, int64_t ldx, int x_dtype,
             float* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);
int aq_qgemm_fast(const void* packed, int64_t N, int64_t K, int bits, int block,
                  const void* X, int64_t M, int64_t ldx, int x_dtype,
                  float* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): aq_qgemm with its workspace taken from a fixed array inside the library
 * (AQ_NOALLOC_SCRATCH_BYTES of device memory per GPU, held until the process ends; the call itself allocates and frees
 * nothing).  Same arithmetic, arguments and errors as aq_qgemm; AQ_ESIZE if aq_qgemm_workspace_size(M, N, K, bits)
 * exceeds AQ_NOALLOC_SCRATCH_BYTES (M = 300 fits up to K = 16384).  Every call on one GPU uses that GPU's one array
 * (its contents are rewritten by each call, nothing has to start at zero): calls that overlap on one GPU, on
 * different streams, race; calls on one stream are ordered. */
#define AQ_NOALLOC_SCRATCH_BYTES (12 * 1024 * 1024)
int aq_qgemm_noalloc(const void* packed, int64_t N, int64_t K, int bits, int block,
                     const void* X, int64_t M, int64_t ldx, int x_dtype,
                     float* Y, int64_t ldy, void* stream);

/* A list of independent prefill products in TWO launches (a whole backbone pass; a lone 4096-row
 * matrix fills only a quarter of the GPU): one that re-orders every distinct activation matrix of
 * the list into the workspace (descriptors with equal X, M, K and ldx share one copy), one for all
 * the products.  Steps: plan on the host (aq_qgemm_batch_plan writes aq_qgemm_batch_plan_size(count)
 * bytes), copy the plan image to 16-byte-aligned DEVICE memory, provide a DEVICE workspace of
 * aq_qgemm_batch_workspace_size(plan_host) bytes, launch; the launch may be repeated.  All
 * descriptors of a plan share x_dtype and the plan's flags (AQ_GEMM_EXACT or AQ_GEMM_FAST). */
typedef struct aq_gemm_desc {
    const void* packed;   /* DEVICE blob */
    const void* X;        /* DEVICE uint16 [M][ldx] */
    float*      Y;        /* DEVICE float [M][ldy] */
    int64_t     N, K, M, ldx, ldy;
    int32_t     bits;     /* 2, 3 or 4 */
    int32_t     x_dtype;  /* AQ_F16 or AQ_BF16 */
} aq_gemm_desc;

size_t aq_qgemm_batch_plan_size(int count);
int aq_qgemm_batch_plan(const aq_gemm_desc* descs /*HOST*/, int count, int block, int flags,
                        void* plan_host, size_t plan_bytes);
size_t aq_qgemm_batch_workspace_size(const void* plan_host);   /* 0 if the plan image is invalid */
int aq_qgemm_batch(const void* plan_host, const void* plan_dev,
                   void* workspace, size_t workspace_bytes, void* stream);

/* Block-level scale optimisation (Section 4.2, Eq. 10-11): the step that produces the codes and scales
 * aq_pack_weights consumes.  For every block of 32 weights along K:
 *   omega_i = F_i * sqrt(sigma_b^2 + w_i^2)       sigma_b^2 = the block's mean squared weight   (Eq. 10, left)
 *   minimise  Phi_b = sum_i omega_i (w_i - s q_i)^2  over the scale s and the codes q_i          (Eq. 10, right)
 *   by alternating  q_i = the codebook entry nearest to w_i / s   and   s = sum(omega w q) / sum(omega q^2)  (Eq. 11)
 * Fixed here where the paper is silent: the codebook is the integers -2^(bits-1) .. 2^(bits-1)-1 (the format's
 * q - z); the start is s = max|w| / 2^(bits-1); `rounds` (0 .. AQ_MAX_ROUNDS) counts scale updates, 0 = plain
 * nearest-code quantisation at the start scale; a block stops early when sum(omega w q) <= 0 or
 * sum(omega q^2) = 0; ties go to the smaller code; the stored scale is d = binary16(s), round to nearest even,
 * capped at 65504, and the stored codes are one more assignment against d; an all-zero block gets d = 0 and
 * the code of zero.  Arithmetic is fp64.
 *   W      DEVICE float  [N][K]   weights
 *   F      DEVICE float  [N][K]   non-negative sensitivities (the diagonal of Eq. 9), or NULL for all ones
 *   codes  DEVICE uint8  [N][K/32][4*bits]   canonical bitstream, written entirely
 *   scales DEVICE uint16 [N][K/32]           binary16 bit patterns, written entirely */
#define AQ_MAX_ROUNDS 64
int aq_optimize_scales(const float* W, const float* F, int64_t N, int64_t K, int bits, int block, int rounds,
                       uint8_t* codes, uint16_t* scales, void* stream);

/* Layer-balanced bit allocation (Section 4.1, Eq. 6 and paragraph "Solver"): HOST-only, no GPU work.
 * Chooses one bit-width per tensor (J tensors in each of L layers) to minimise  sum_l E_l^2,
 * E_l = sum_j S[l][j] * 2^(-2 bits[l][j]),  subject to  sum(bits * size) / sum(size) <= avg_bits_budget,
 * with the paper's greedy procedure: every tensor starts at choices[0]; at each step the single upgrade to the
 * next larger entry of `choices` with the largest (E_l^2 - E~_l^2) / extra_bits is applied.  Fixed here where the
 * paper is silent: an upgrade that would exceed the budget is not a candidate; the loop ends when no candidate is
 * left or no upgrade lowers the objective (S may be negative); ties go to the first tensor in (layer, tensor) order.
 *   S        HOST double  [L][J]   sensitivities (Eq. 5)
 *   sizes    HOST int64   [L][J]   elements per tensor, >= 1
 *   choices  HOST int     [n_choices]  strictly ascending bit-widths in 1..16 (e.g. 2, 3, 4)
 *   bits_out HOST int     [L][J]
 * AQ_EINVAL if choices[0] everywhere already exceeds the budget. */
int aq_allocate_bits(const double* S, const int64_t* sizes, int L, int J, const int* choices, int n_choices,
                     double avg_bits_budget, int* bits_out);

/* Two-level variant of the format: Eq. 1 in its general form, w_hat = s_b (q - z_b) with a stored scale AND a stored
 * real zero point per block of 32, both compressed by the parameters of the super-block (Section 3, "Weight
 * quantization").  The paragraph leaves the compression open; here a super-block is 8 blocks (256 consecutive k of
 * a row) with two binary16 numbers D, M, and a block stores two 4-bit codes a, c:
 *     s_b = D * a,   s_b z_b = M * c,   w_hat = D a q - M c          (bits + 0.375 bits per weight stored)
 * Canonical inputs of aq2_pack_weights (DEVICE, 16-byte aligned):
 *   codes   uint8  [N][K/32][4*bits]     the code bitstream, as for aq_pack_weights
 *   sub     uint8  [N][K/32]             a in the low nibble, c in the high nibble
 *   sup     uint16 [N][ceil(K/256)][2]   binary16 bit patterns of D, M
 * The packed blob (aq2_packed_size bytes) has the base format's tiling with the parameters next to the codes they
 * scale.  aq2_qgemv is aq_qgemv for such a blob: the codes meet x as exact integers on the matrix cores, and a
 * block's sum B = sum (q - 2^(bits-1)) x becomes (D a) B + (2^(bits-1) D a - M c) * (sum of x over the block) in
 * fp32.  aq2_qgemv_batch_plan plans a list of such products (every blob of the list in this format); the plan is
 * launched with aq_qgemv_batch.  aq2_unpack_codes / aq2_dequant_f32 are the parity inverses (the latter returns
 * fp32(D a q - M c), rounded once).
 * aq2_qgemm is aq_qgemm for such a blob (exact products, any M in 1 .. AQ_MAX_M): per block the matrix cores give
 * P = sum_k q x on exact small integers and X_b = sum_k x, and the accumulators take (D a) P - (M c) X_b in fp32 (D a
 * and M c are exact there); no weight is rounded and no magnitude limit applies beyond fp32's.
 * aq2_qgemm_fast is aq_qgemm_fast for such a blob: a weight meets X as the binary16 number
 * fp16(q * fp16(D a) - fp16(M c)), the subtraction fused (three roundings to 11 bits, against one in the base format: relative L2
 * of Y 3e-4 .. 8e-4 on random inputs), X as in aq_qgemm_fast.  LIMIT of this mode only: the caller keeps 15 * (2^bits - 1) * |D| and 15 * |M| inside
 * binary16 (65504); such a matrix is not rescaled, and beyond the limit the result holds infinities or NaNs where
 * aq2_qgemm, aq2_qgemv and aq2_dequant_f32 stay finite.  Workspace of both: aq_qgemm_workspace_size(M, N, K, bits) bytes.
 * aq2_qgemm_batch_plan plans a list of such products in the mode `flags` names (AQ_GEMM_EXACT or AQ_GEMM_FAST; plan of
 * aq_qgemm_batch_plan_size(count) bytes; workspace from
 * aq_qgemm_batch_workspace_size; launched with aq_qgemm_batch).  The decode step through the blocks takes the base
 * format.  Arguments, limits and errors as for the base functions. */
size_t aq2_packed_size(int64_t N, int64_t K, int bits, int block);
int aq2_pack_weights(const uint8_t* codes, const uint8_t* sub, const uint16_t* sup, int64_t N, int64_t K, int bits,
                     int block, void* packed, size_t packed_bytes, void* stream);
int aq2_qgemv(const void* packed, int64_t N, int64_t K, int bits, int block, const void* x, int x_dtype,
              float* y, void* stream);
int aq2_qgemv_batch_plan(const aq_gemv_desc* descs /*HOST*/, int count, int block,
                         void* plan_host, size_t plan_bytes);
int aq2_qgemm(const void* packed, int64_t N, int64_t K, int bits, int block, const void* X, int64_t M, int64_t ldx,
              int x_dtype, float* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);
int aq2_qgemm_fast(const void* packed, int64_t N, int64_t K, int bits, int block, const void* X, int64_t M, int64_t ldx,
                   int x_dtype, float* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);
int aq2_qgemm_batch_plan(const aq_gemm_desc* descs /*HOST*/, int count, int block, int flags,
                         void* plan_host, size_t plan_bytes);
int aq2_unpack_codes(const void* packed, int64_t N, int64_t K, int bits, int block, uint8_t* codes_u8, void* stream);
int aq2_dequant_f32(const void* packed, int64_t N, int64_t K, int bits, int block, float* W, void* stream);

/* Non-uniform codebook variant of the format (Section 3, "Weight quantization": the codes of a format come from a
 * format-specific codebook of representable values, uniform or non-uniform): a block of 32 consecutive weights of a
 * row has one binary16 scale d, and a code q of `bits` bits selects one of 2^bits levels of a table that belongs to
 * the matrix,
 *         w_hat[n][k] = d[n][k/32] * levels[q[n][k]].
 * The base format is the table levels[q] = q - 2^(bits-1).  `levels` is a HOST array of 2^bits finite floats; the
 * caller passes the SAME table to aqc_pack_weights and to every later call on that blob (the blob does not carry it).
 * Canonical inputs of aqc_pack_weights: codes and scales as for aq_pack_weights; the blob has aq_packed_size(N, K,
 * bits, block) bytes and the base format's layout.
 * How a table reaches the matrix cores (aqc_table_info reports it; results do not depend on it beyond fp32 rounding):
 *   AQC_FORM_NATIVE  (bits = 4 and levels = alpha * the sixteen E2M1 numbers 0, 0.5, 1, 1.5, 2, 3, 4, 6 and their
 *               negatives, in any order, each to within float rounding): the codes are re-numbered at packing so that a
 *               stored nibble is the fp4 bit pattern of its level, and the decode kernel multiplies the stored words as
 *               they are;
 *   AQC_FORM_SIGNED  (the levels come in pairs +v, -v, zeros pairing with zeros): the codes are re-numbered to a sign
 *               bit and the index m of the magnitude in ascending order; the magnitude table is written as a multilinear
 *               polynomial of m's bits, mag[m] = sum over subsets S of the bits set in m of coef[S], and the kernel runs
 *               one signed one-bit plane per S (2 / 4 / 8 planes for 2 / 3 / 4 bits);
 *   AQC_FORM_PLANES  (any other table): levels[q] = sum over subsets S of the bits set in q of coef[S], one one-bit
 *               plane per non-empty S (3 / 7 / 15 planes: 4-bit tables of this form are slow).
 * aqc_table_info: form (HOST int, may be NULL), coef (HOST float[16], may be NULL: the coefficients indexed by S,
 *   coef[0] the constant term; for a native table coef[0] = alpha and the rest is 0).
 * aqc_qgemv / aqc_unpack_codes / aqc_dequant_f32 are aq_qgemv / aq_unpack_codes / aq_dequant_f32 for such a blob
 * (aqc_unpack_codes returns the caller's codes, whatever the stored numbering).  A list of products runs in one launch:
 * aqc_qgemv_batch_plan_size / aqc_qgemv_batch_plan (HOST) / copy the image to 16-byte-aligned DEVICE memory /
 * aqc_qgemv_batch, as for aq_qgemv_batch; the tables are read when the plan is made.
 * aqc_qgemm is aq_qgemm_fast for such a blob, at any M in 1 .. AQ_MAX_M: a weight meets X as the binary16 number
 * fp16(d * levels[q]), the product formed in fp32 and rounded once (the caller keeps |d * levels[q]| inside binary16's
 * range, 65504: there is no rescaling), X as in aq_qgemm_fast; there is no exact-product form of it.
 * Workspace: aqc_qgemm_workspace_size(M, N, K, bits) bytes (the re-ordered X and the table).  A list of such products
 * runs like a list of the base format's: aqc_qgemm_batch_plan writes aqc_qgemm_batch_plan_size(count) bytes on the HOST
 * (the base plan image followed by the tables), the caller copies the image to 16-byte-aligned DEVICE memory, provides
 * aq_qgemm_batch_workspace_size(plan_host) bytes of workspace and launches with aq_qgemm_batch.
 * Arguments, ownership and errors otherwise as for the base functions; AQ_EINVAL also for a table with an infinity or
 * a NaN. */
typedef struct aqc_gemv_desc {
    aq_gemv_desc product;  /* packed: a blob from aqc_pack_weights */
    const float* levels;   /* HOST float [2^bits] */
} aqc_gemv_desc;
#define AQC_FORM_PLANES 0
#define AQC_FORM_NATIVE 1
#define AQC_FORM_SIGNED 2
int aqc_table_info(const float* levels /*HOST*/, int bits, int* form /*HOST*/, float* coef /*HOST*/);
int aqc_pack_weights(const uint8_t* codes, const uint16_t* scales, const float* levels /*HOST*/, int64_t N, int64_t K,
                     int bits, int block, void* packed, size_t packed_bytes, void* stream);
int aqc_qgemv(const void* packed, int64_t N, int64_t K, int bits, int block, const float* levels /*HOST*/,
              const void* x, int x_dtype, float* y, void* stream);
size_t aqc_qgemv_batch_plan_size(const aqc_gemv_desc* descs /*HOST*/, int count, int block);
int aqc_qgemv_batch_plan(const aqc_gemv_desc* descs /*HOST*/, int count, int block, void* plan_host, size_t plan_bytes);
int aqc_qgemv_batch(const void* plan_host, const void* plan_dev, void* stream);
typedef struct aqc_gemm_desc {
    aq_gemm_desc product;  /* packed: a blob from aqc_pack_weights */
    const float* levels;   /* HOST float [2^bits] */
} aqc_gemm_desc;
size_t aqc_qgemm_batch_plan_size(int count);
int aqc_qgemm_batch_plan(const aqc_gemm_desc* descs /*HOST*/, int count, int block, void* plan_host, size_t plan_bytes);
size_t aqc_qgemm_workspace_size(int64_t M, int64_t N, int64_t K, int bits);
int aqc_qgemm(const void* packed, int64_t N, int64_t K, int bits, int block, const float* levels /*HOST*/, const void* X,
              int64_t M, int64_t ldx, int x_dtype, float* Y, int64_t ldy, void* workspace, size_t workspace_bytes,
              void* stream);
int aqc_unpack_codes(const void* packed, int64_t N, int64_t K, int bits, int block, const float* levels /*HOST*/,
                     uint8_t* codes_u8, void* stream);
int aqc_dequant_f32(const void* packed, int64_t N, int64_t K, int bits, int block, const float* levels /*HOST*/,
                    float* W, void* stream);

/* One decode step (M = 1) through a stack of transformer blocks, layer by layer, with what sits between the
 * matrices fused into the matrix-vector kernels.  Section 3 ("Vision-Language-Action models") names a block's
 * matrices: the attention projections W_Q, W_K, W_V, W_O and the MLP's W_gate, W_up, W_down; the rest is the
 * published architecture of the backbones the paper quantises (LLaMA-2-7B; a Gemma-2B-sized one):
 *     h = rmsnorm(x; norm_attn)                  rmsnorm(x; g)_i = x_i / sqrt(mean(x^2) + eps) * g_i
 *     q, k, v = W_Q h, W_K h, W_V h              written to qkv[layer] = [q | k | v] (what a key/value cache
 *                                                and a later attention read; no rotary embedding applied)
 *     x += W_O a                                 a = attention over the ONE visible key (the step is the first
 *                                                token of a sequence): query head i gets value head
 *                                                i / (n_heads / n_kv_heads).  Attention over a longer cache
 *                                                is not part of this library.
 *     h2 = rmsnorm(x; norm_mlp);  x += W_down (act(W_gate h2) * W_up h2)
 * A layer is four dependent stages (q/k/v; o; gate/up; down).  Inputs of the products are rounded to binary16
 * times a power of two (11 significant bits); sums are fp32; a stage's partial sums meet in fp32 atomic
 * additions, so the last bits of a result can differ between runs.
 * One launch per stage (4 per layer, each taking its matrices' records as kernel arguments) plus one that clears
 * qkv; consecutive launches on one stream are the barriers between dependent stages.
 *   shape      HOST; d_model, d_ff, n_heads * head_dim multiples of 32 and <= 16384 (this call's own limit), head_dim a multiple of 8,
 *              n_heads a multiple of n_kv_heads, act = AQ_ACT_SILU or AQ_ACT_GELU_TANH, eps >= 0
 *   blocks     HOST array of `layers` records: w[0..6] = DEVICE blobs (aq_pack_weights) of q, k, v, o, gate, up,
 *              down with the shapes the block shape implies and bit-widths bits[0..6]; norm_attn, norm_mlp =
 *              DEVICE float [d_model], 16-byte aligned (the multipliers themselves; a Gemma checkpoint stores g - 1)
 *   x          DEVICE float [d_model], 16-byte aligned: the residual stream, read and overwritten by a step
 *   qkv        DEVICE float [layers][n_heads * head_dim + 2 * n_kv_heads * head_dim], overwritten by a step
 *   workspace  DEVICE, 16-byte aligned, aq_decode_workspace_size(shape) bytes (gate and up of the current layer)
 * aq_decode_plan binds these buffers into a plan image of aq_decode_plan_size(layers) bytes on the HOST (nothing
 * of it is read by the device); aq_decode_step may be repeated (each call advances x by one pass through the
 * stack).  Steps that share buffers must be ordered on one stream. */
#define AQ_ACT_SILU      0
#define AQ_ACT_GELU_TANH 1
typedef struct aq_block_shape {
    int32_t d_model, n_heads, n_kv_heads, head_dim, d_ff;
    int32_t act;
    float   eps;
} aq_block_shape;
typedef struct aq_block_desc {
    const void*  w[7];
    int32_t      bits[7];
    const float* norm_attn;
    const float* norm_mlp;
} aq_block_desc;
size_t aq_decode_plan_size(int layers);
size_t aq_decode_workspace_size(const aq_block_shape* shape);
int aq_decode_plan(const aq_block_shape* shape, const aq_block_desc* blocks /*HOST*/, int layers, int block,
                   float* x, float* qkv, void* workspace, size_t workspace_bytes,
                   void* plan_host, size_t plan_bytes);
int aq_decode_step(const void* plan_host, void* stream);

/* Tensor sensitivity from HSIC (Section 4.1, Eq. 5; the estimator is Eq. 2 of Section 3, "HSIC"):
 *     HSIC(A, B) = (K - 1)^-2 tr(K_A C K_B C),  [K_A]_ij = exp(-gamma_A ||a_i - a_j||^2),  C = I - (1/K) 1 1^T
 *     S = -alpha HSIC(X, Z) + beta HSIC(Z, Y)
 * over K paired calibration samples: X[K][dx] the backbone's input hidden states, Z[K][dz] the output hidden states
 * of the weight matrix being scored, Y[K][dy] the action labels (DEVICE fp32, row strides ldx, ldz, ldy in
 * elements, 16-byte aligned).  The RBF bandwidths are inputs (gamma > 0; the paper does not fix them).
 *   out        DEVICE double [3]: HSIC(X, Z), HSIC(Z, Y), S
 *   workspace  DEVICE, aq_hsic_workspace_size(K) bytes (three K x K fp32 kernel matrices and their row sums)
 * The Gram products run in fp32 on the matrix cores, the sums in fp64.  2 <= K <= 65536.
 * aq_rbf_gram writes one kernel matrix G[K][K] (parity; workspace: K floats). */
size_t aq_hsic_workspace_size(int64_t K);
int aq_rbf_gram(const float* A, int64_t K, int64_t d, int64_t lda, float gamma, float* G, void* workspace,
                size_t workspace_bytes, void* stream);
int aq_hsic_sensitivity(const float* X, int64_t dx, int64_t ldx, float gamma_x, const float* Z, int64_t dz, int64_t ldz,
                        float gamma_z, const float* Y, int64_t dy, int64_t ldy, float gamma_y, int64_t K, double alpha,
                        double beta, double* out, void* workspace, size_t workspace_bytes, void* stream);

/* Parity / debug: the blob decoded back to what Eq. 1 defines.
 *   codes_u8 DEVICE uint8 [N][K]  one code per byte
 *   W        DEVICE float [N][K]  d * (q - 2^(bits-1)); exact in fp32 (11-bit x 4-bit significands) */
int aq_unpack_codes(const void* packed, int64_t N, int64_t K, int bits, int block,
                    uint8_t* codes_u8, void* stream);
int aq_dequant_f32(const void* packed, int64_t N, int64_t K, int bits, int block,
                   float* W, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* AQ_H */
