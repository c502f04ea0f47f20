/*
 * lcd.h -- C ABI of the MI355X (gfx950) library for LCD's smoothed table-lookup linear layer.
 *
 * The operation (paper Sec. 4, "Inference with Table Lookup"; Sec. 3.4 for the smoothing):
 *
 *     Y[m][n] = sum_k ( X[m][k] / s[k] ) * C[n][ idx[n][k] ]        m < M, n < N, k < K
 *
 *   idx[n][k]  2-, 3- or 4-bit index of the centroid that weight (n,k) was clustered to
 *              (Sec. 3.2: a clustered weight W' is its centroid);
 *   C[n][c]    per-output-row codebook of 2^bits fp16 centroids; the centroids already
 *              contain the offline smoothing of the weights (Sec. 3.4: weights are scaled by
 *              the smoothing factor offline, inputs are divided by it at inference);
 *   s[k]       per-input-channel smoothing factor, fp32, > 0;
 *   X, Y       fp16, row-major.  Accumulation is fp32; one rounding to fp16 at the store.
 *
 * Conventions for every entry point
 *   - Pointers marked DEVICE must be device memory of the current HIP device, 16-byte
 *     aligned; pointers marked HOST are ordinary host memory.
 *   - The caller owns every buffer.  The library never allocates, frees or keeps a pointer
 *     after the call has enqueued its work.
 *   - Device work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the default
 *     stream).  No entry point synchronises; results are valid once the stream has reached
 *     the call's work.
 *   - Arguments are validated on the host before anything is launched; a failed call
 *     launches nothing and returns a status != LCD_OK.  lcd_last_error_string() then holds a
 *     message (thread-local).
 *   - Shapes: bits in {2,3,4};  N % 16 == 0;  K % 256 == 0;  N, K >= 1 tile.
 *   - Two calls that share a workspace buffer must be ordered on one stream.
 *   - Every call works on the current HIP device; the little state the launchers keep (the
 *     device's compute-unit count, "dynamic-LDS limit raised" flags) is per device and atomic, and
 *     the error string and the remembered workgroup split of the last grouped decode call are per
 *     thread, so calls from several threads and on several devices of one process do not disturb
 *     each other.  (This build is tested on one GPU.)
 */
#ifndef LCD_H
#define LCD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LCD_OK = 0,
    LCD_ERR_NULL = 1,        /* a required pointer is NULL                          */
    LCD_ERR_BAD_BITS = 2,    /* bits not in {2,3,4}                                 */
    LCD_ERR_BAD_SHAPE = 3,   /* N or K not positive / not a multiple of the tile    */
    LCD_ERR_BAD_M = 4,       /* M out of range for the entry point                  */
    LCD_ERR_SIZE = 5,        /* a buffer-size argument is too small                 */
    LCD_ERR_INDEX_RANGE = 6, /* host packer: an index is >= 2^bits                  */
    LCD_ERR_ALIGN = 7,       /* a device pointer is not 16-byte aligned             */
    LCD_ERR_HIP = 8,         /* the HIP runtime reported an error at launch         */
    LCD_ERR_BAD_SCALE = 9    /* a quantisation scale is not positive and finite     */
} lcd_status;

/* Library version (major*10000 + minor*100 + patch) and the packed-layout revision. */
int lcd_version(void);
int lcd_layout_revision(void);

/* Message of the last failed call on this thread ("" if none), and a fixed name per status. */
const char *lcd_last_error_string(void);
const char *lcd_status_string(lcd_status st);

/* ---- sizes (pure host functions; 0 on invalid arguments) -------------------------------- */

/* Bytes of the packed index matrix: exactly N*K*bits/8 (Sec. 4.2: compact low-bit indices). */
size_t lcd_packed_bytes(int N, int K, int bits);
/* Bytes of the per-layer table lcd_build_lut writes (24*N for 2 bits, 48*N for 3, 32*N for 4). */
size_t lcd_lut_bytes(int N, int bits);
/* Bytes of scratch the product entry points need for this problem (a multiple of 256): the
 * transformed activations (lcd_lut_gemm: smoothed, in matrix-operand order, about 2*K bytes per
 * token with the tokens padded to 128; the decode entry points with M >= 2, or 4 bits: at most
 * M*K fp16 numbers).  One buffer of this size serves every entry point for the problem. */
size_t lcd_workspace_bytes(int M, int N, int K, int bits);

/* ---- index packing (offline, once per layer; Sec. 4.1 "constructed ahead of time") ------- *
 *
 * Input:  idx[N][K], row-major, one index per byte.
 * Output: the packed layout (revision 1), made for 16-byte-per-lane, 1 KiB-per-wavefront
 * contiguous loads.  The matrix is cut into tiles of 16 rows x 256 columns; tile
 * (t = n/16, c = k/256) starts at byte (t*(K/256) + c) * T with T = 1024 (2 bits), 1536
 * (3 bits) or 2048 (4 bits).  Inside a tile, "lane" l = 16*q + i covers row i = n%16 and the 64 columns
 * k%256 in [64q, 64q+64); let w = k%64.
 *   - bytes [16*l, 16*l+16) of the tile are a 128-bit little-endian word whose bits
 *     [2w+1 : 2w] hold idx & 3;
 *   - 3 bits only: bytes [1024 + 8*l, 1024 + 8*l + 8) are two 32-bit little-endian words.
 *     With w = 16*d + 8*a + e (d<4, a<2, e<8), bit (idx >> 2) is stored in word a at bit
 *     8*((e>>2) + 2*(e&1)) + 2*d + ((e&3)>>1).
 *   - 4 bits only (the container for up to 16 centroids, Sec. 4.2): bytes [1024 + 16*l,
 *     1024 + 16*l + 16) are a second 128-bit little-endian word whose bits [2w+1 : 2w] hold
 *     idx >> 2.
 * A codebook with fewer centroids than its container holds (5, 6, 10, ...) simply never uses
 * the upper codes; their codebook entries must be finite (zero is the natural choice).
 * The mapping is a bijection: lcd_unpack_indices(lcd_pack_indices(idx)) == idx, and the
 * device and host packers produce identical bytes.
 *
 * Device packer: idx and packed are DEVICE pointers.  Indices are taken modulo 2^bits (the
 * device cannot report a range error without a sync; use the host twin to validate).
 */
lcd_status lcd_pack_indices(const uint8_t *idx /*DEVICE [N][K]*/, int N, int K, int bits,
                            void *packed /*DEVICE*/, size_t packed_bytes, void *stream);
lcd_status lcd_unpack_indices(const void *packed /*DEVICE*/, int N, int K, int bits,
                              uint8_t *idx /*DEVICE [N][K]*/, void *stream);
/* Host twins (HOST pointers, no GPU needed, no alignment requirement).  The host packer
 * returns LCD_ERR_INDEX_RANGE if any index is >= 2^bits and then leaves `packed` untouched. */
lcd_status lcd_pack_indices_host(const uint8_t *idx /*HOST*/, int N, int K, int bits,
                                 void *packed /*HOST*/, size_t packed_bytes);
lcd_status lcd_unpack_indices_host(const void *packed /*HOST*/, int N, int K, int bits,
                                   uint8_t *idx /*HOST*/);

/* ---- table build (offline, once per layer; Sec. 4.1 / 4.2 "pre-computed values") --------- *
 *
 * codebook: DEVICE, fp16 bit patterns, [N][2^bits] row-major.
 * lut:      DEVICE, lcd_lut_bytes(N,bits) bytes, opaque.  It holds the codebook re-laid out
 *           for the kernels: fp32 per-bucket multipliers in accumulator order for the decode
 *           path (Sec. 4.2: one bucket per weight centroid), and byte-split tables for the
 *           register dequantiser of the batched paths (4 bits: these tables only).
 */
lcd_status lcd_build_lut(const uint16_t *codebook /*DEVICE*/, int N, int bits,
                         void *lut /*DEVICE*/, size_t lut_bytes, void *stream);

/* ---- the product (Sec. 4.2 lookup + accumulation, with Sec. 3.4's division by s) --------- *
 *
 * packed  DEVICE, from lcd_pack_indices;     lut  DEVICE, from lcd_build_lut
 * x       DEVICE fp16 [M][K] row-major;      s    DEVICE fp32 [K], every s[k] > 0 and finite
 *                                                 (not checked); |x/s| must fit fp16
 * y       DEVICE fp16 [M][N] row-major (written, never read)
 * workspace  DEVICE, >= lcd_workspace_bytes(M,N,K,bits) bytes, contents ignored on entry.
 *
 * lcd_lut_gemv: decode path, 1 <= M <= 16, one kernel launch, any K.  M = 1 (and M = 2 with
 *               2 bits): centroid-bucket sums on the sparse matrix core (Sec. 4.2), one sparse
 *               pass per token; otherwise (3 <= M <= 16, M = 2 with 3 bits, every M with 4 bits):
 *               register dequantisation into fp16 MFMA operands with the tokens as the matrix
 *               columns.  The smoothing is fused into the kernel, except on the dequantising
 *               route with K >= 16384, where a small kernel ahead of the product leaves the
 *               smoothed activations in the workspace (same rounding, same result).
 * lcd_lut_gemm: prefill path, any M >= 1 (tuned for M >= 64): a smoothing kernel into the
 *               workspace, then register dequantisation into fp16 MFMA operands.
 * Both give bit-identical results from run to run (fixed reduction order).
 */
lcd_status lcd_lut_gemv(const void *packed, const void *lut, const uint16_t *x, const float *s,
                        uint16_t *y, int M, int N, int K, int bits,
                        void *workspace, size_t workspace_bytes, void *stream);
lcd_status lcd_lut_gemm(const void *packed, const void *lut, const uint16_t *x, const float *s,
                        uint16_t *y, int M, int N, int K, int bits,
                        void *workspace, size_t workspace_bytes, void *stream);

/* ---- decode for callers that cannot allocate -------------------------------------------------- *
 *
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc: the
 * product of lcd_lut_gemv (same arguments, same result bit for bit) with no workspace argument.
 * The scratch the several-token route needs (the smoothed activations, M*K fp16 numbers) lives in a
 * device array inside the library, 1 MiB per GPU, held until the process ends; the call itself
 * allocates and frees nothing, on the host or on the device.
 *   - Limit: 1 <= M <= 16 and M*K <= 16*32768 (so K <= 32768 at 16 tokens); beyond it
 *     LCD_ERR_SIZE and nothing is launched.
 *   - Every call on a GPU uses that GPU's one array: calls that may overlap in time on one GPU
 *     (different streams, different threads) race and must be ordered by the caller.  Nothing in the
 *     array has to start at zero; each call overwrites what it reads.
 *   - The first call on a device looks up the array's device address (once per device, with that
 *     device current); make that call outside stream capture.
 */
lcd_status lcd_lut_gemv_noalloc(const void *packed, const void *lut, const uint16_t *x, const float *s,
                                uint16_t *y, int M, int N, int K, int bits, void *stream);

/* ---- decode with the paper's input transformation in front (Sec. 4.1, Eq. 10-11, b = 8) ---- *
 *
 * The activations are smoothed and quantised to INT8 codes in one step, as the paper's own
 * inference path does,
 *     q[m][k] = clip( round_half_even( X[m][k] / (s[k] * s_q) ), -128, 127 )
 *     Y[m][n] = s_q * sum_k q[m][k] * C[n][ idx[n][k] ]
 * with s_q > 0 the (per-layer) activation quantisation step.  Every step of the quantiser is
 * IEEE binary32 (the product s[k]*s_q, the correctly rounded quotient, the rounding), so the
 * codes are reproducible bit for bit on a CPU; the sum is fp32 (exact on the integer bucket
 * sums), one rounding to fp16 at the store.  Precondition on the data: every s[k]*s_q lies in
 * (2^-64, 2^64) and X is finite (the quotient is computed without range scaling).
 * All other arguments as lcd_lut_gemv (1 <= M <= 16).
 * Routing: as lcd_lut_gemv, except that with 2 bits the codes travel as int8 numbers through the
 * sparse matrix core's int8 instruction (half the matrix instructions per weight, same bits in the
 * result: the bucket sums are integers either way), which then takes up to four tokens (one sparse
 * pass per token) before the dequantising route takes over at M >= 5; with 3 bits and one token the
 * plain pass runs on int8 operands and the sign-flipped pass on fp16 operands.
 */
lcd_status lcd_lut_gemv_q8(const void *packed, const void *lut, const uint16_t *x, const float *s, float s_q,
                           uint16_t *y, int M, int N, int K, int bits,
                           void *workspace, size_t workspace_bytes, void *stream);

/* The prefill path with the same input transformation (Sec. 4.1 applies it to the input of every
 * table-lookup layer, whatever the number of tokens): the smoothing kernel ahead of the matrix kernel
 * quantises instead (same binary32 quantiser, codes bit for bit those of lcd_lut_gemv_q8) and the
 * matrix kernel multiplies the fp32 sums by s_q before the one rounding to fp16.  Any M >= 1;
 * all other arguments, the workspace and the precondition on s*s_q as above. */
lcd_status lcd_lut_gemm_q8(const void *packed, const void *lut, const uint16_t *x, const float *s, float s_q,
                           uint16_t *y, int M, int N, int K, int bits,
                           void *workspace, size_t workspace_bytes, void *stream);

/* ---- grouped decode: several independent layers in ONE launch ---------------------------- *
 *
 * A decoder block applies several table-lookup linear layers per token (Sec. 5 evaluates whole
 * models); each is only a few MB of packed indices, so launching them one by one leaves the
 * GPU mostly idle.  lcd_lut_gemv_grouped runs `count` (1..16) independent products
 *     y_i = (x_i / s_i) . What_i^T            (same M and bits for all, any N_i, K_i)
 * with every argument of problems[i] as in lcd_lut_gemv, in one kernel launch for any M in
 * 1..16: the workgroups are shared out over the layers in proportion to their work.
 * `problems` is a HOST array, read during the call only.  The layers' outputs must not overlap.
 * Workspace: at least lcd_workspace_bytes_grouped(problems, count, M, bits) bytes (DEVICE);
 * for M >= 2 it may receive the layers' transformed activations (at most M*K_i fp16 each).
 * Calls that share a workspace must be ordered on one stream.
 */
typedef struct lcd_gemv_problem {
    const void *packed;   /* DEVICE */
    const void *lut;      /* DEVICE */
    const uint16_t *x;    /* DEVICE fp16 [M][K] */
    const float *s;       /* DEVICE fp32 [K]    */
    uint16_t *y;          /* DEVICE fp16 [M][N] */
    int N, K;
} lcd_gemv_problem;

size_t lcd_workspace_bytes_grouped(const lcd_gemv_problem *problems /*HOST*/, int count, int M, int bits);
lcd_status lcd_lut_gemv_grouped(const lcd_gemv_problem *problems /*HOST*/, int count, int M, int bits,
                                void *workspace, size_t workspace_bytes, void *stream);

/* Layers of different index widths in one call (the paper assigns a centroid count per layer,
 * Sec. 5: 5, 6, 10, ... centroids): bits is a HOST array of `count` widths, each 2, 3 or 4.
 * All layers are validated first; then the layers of each width that occurs go out as one
 * launch, in the order 2, 3, 4, on `stream`.  Workspace as for lcd_lut_gemv_grouped (its size
 * does not depend on the width). */
lcd_status lcd_lut_gemv_grouped_mixed(const lcd_gemv_problem *problems /*HOST*/, const int *bits /*HOST*/, int count,
                                      int M, void *workspace, size_t workspace_bytes, void *stream);

/* The same with the input transformation of lcd_lut_gemv_q8 in front of every layer:
 * s_q is a HOST array of `count` activation quantisation steps, one per layer. */
lcd_status lcd_lut_gemv_q8_grouped(const lcd_gemv_problem *problems /*HOST*/, const float *s_q /*HOST*/, int count,
                                   int M, int bits, void *workspace, size_t workspace_bytes, void *stream);

/* ---- grouped prefill: several independent layers in ONE pair of launches ------------------- *
 *
 * The same product as lcd_lut_gemm for `count` (1..16) layers with one token count M >= 1 and one
 * index width: one smoothing launch for all layers, then one matrix launch whose workgroups take
 * the layers' output tiles one layer after the other (those with the largest K first), so that
 * the compute units the tail of one layer leaves idle start on the next.  Results are bit for
 * bit those of lcd_lut_gemm on every layer.  `problems` is a HOST array, read during the call
 * only; outputs must not overlap.  Workspace: at least
 * lcd_workspace_bytes_gemm_grouped(problems, count, M, bits) bytes (DEVICE; the sum of the
 * layers' lcd_workspace_bytes): every layer's smoothed activations side by side.
 */
size_t lcd_workspace_bytes_gemm_grouped(const lcd_gemv_problem *problems /*HOST*/, int count, int M, int bits);
lcd_status lcd_lut_gemm_grouped(const lcd_gemv_problem *problems /*HOST*/, int count, int M, int bits,
                                void *workspace, size_t workspace_bytes, void *stream);
/* Layers whose x, s and K are the same pointers and size (q/k/v or gate/up of a decoder block read one
 * input) share one smoothed copy: the activations are transformed once per distinct input.
 *
 * The same with the input transformation of lcd_lut_gemm_q8 in front of every layer (Sec. 4.1):
 * s_q is a HOST array of `count` activation quantisation steps, one per layer (layers share a
 * transformed copy only if their steps are equal too). */
lcd_status lcd_lut_gemm_q8_grouped(const lcd_gemv_problem *problems /*HOST*/, const float *s_q /*HOST*/, int count,
                                   int M, int bits, void *workspace, size_t workspace_bytes, void *stream);

/* ---- clustering-side steps that need no calibration data (offline) ------------------------ *
 *
 * Codebooks here are per output row, fp16 [N][2^bits], of which the first `ncent` entries are in
 * use and STRICTLY ASCENDING (the paper sorts the centroids, Sec. 3.2); the rest is ignored.
 *
 * lcd_assign_indices: idx[n][k] = the centroid of row n nearest to w[n][k] (w: DEVICE fp16 [N][K],
 *   e.g. the smoothed weights).  This is the state the reclassification rule of Sec. 3.2 (Eq. 6)
 *   maintains: a weight leaves its cluster once it crosses half the gap to a neighbouring
 *   centroid.  A weight exactly half way stays with the lower centroid; NaN goes to centroid 0.
 *   The decision is exact (no rounding anywhere).  Output as lcd_pack_indices takes it.
 * lcd_cluster_counts: counts[n][i] = number of k with idx[n][k] == i, for i < 2^bits
 *   (DEVICE uint32 [N][2^bits]; the cluster sizes of Sec. 3.3).  idx must be < 16.
 * lcd_merge_closest: Sec. 3.3, Eq. 8, per row: the two closest centroids a, a+1 (smallest gap,
 *   the lowest pair on equal gaps) are replaced by their mean weighted by their cluster sizes --
 *   each centroid by its OWN count, as the text defines it (the printed formula has the counts
 *   crossed), the plain mean if both clusters are empty -- correctly rounded to fp16, ties to even
 *   (the decision between the two neighbouring fp16 numbers is taken in exact integer arithmetic;
 *   centroids must be finite).  codebook_out gets ncent-1 ascending
 *   entries followed by zeros, merged[n] = a (DEVICE uint8 [N]), idx_out the re-numbered indices
 *   (idx - 1 above a; idx_out may be idx itself; codebook_out must not be codebook).
 * Errors: as above; ncent outside 1..2^bits (2..2^bits for the merge) is LCD_ERR_SIZE.
 */
lcd_status lcd_assign_indices(const uint16_t *w /*DEVICE*/, const uint16_t *codebook /*DEVICE*/, int ncent,
                              int N, int K, int bits, uint8_t *idx /*DEVICE [N][K]*/, void *stream);
lcd_status lcd_cluster_counts(const uint8_t *idx /*DEVICE*/, int N, int K, int bits,
                              uint32_t *counts /*DEVICE [N][2^bits]*/, void *stream);
lcd_status lcd_merge_closest(const uint16_t *codebook /*DEVICE*/, const uint32_t *counts /*DEVICE*/,
                             const uint8_t *idx /*DEVICE*/, int ncent, int N, int K, int bits,
                             uint16_t *codebook_out /*DEVICE*/, uint8_t *idx_out /*DEVICE*/,
                             uint8_t *merged /*DEVICE [N]*/, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LCD_H */
