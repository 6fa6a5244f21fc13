/*
 * leanquant.h -- C ABI of the MI355X (gfx950) LeanQuant per-layer quantization pass.
 *
 * The four compute calls are the four parts of Algorithm 1 of the paper
 * (arXiv 2407.10032, "LeanQuant for LLM quantization"):
 *
 *   lq_hessian_accumulate   line 3        H <- 2 X X^T
 *   lq_cholesky_inv         line 4        H^-1 <- Cholesky([H + df avg(diag H) I]^-1)
 *   lq_fit_grid             lines 5-9     loss-error-aware grid per output channel
 *                                         (Eq. 5 with Eq. 6 init, or Eq. 7 with Eq. 8)
 *   lq_quantize_layer       lines 10-21   blocked quantize-and-propagate column loop
 *
 * Around them: lq_hessian_accumulate_host (line 3 with X streamed from host memory),
 * lq_fit_grid_from / lq_kmeanspp_seed (Lloyd iteration from another start, the k-means++
 * seeding of the paper's initialisation table), lq_quantize_exact / lq_hinv_from_factor
 * (Algorithm 2, LeanQuant-Exact), lq_pack_layer / lq_unpack_layer / lq_matvec_packed /
 * lq_matmul_packed (the stored form behind the "Bits" columns of the result tables and the
 * products with it).
 *
 * Conventions shared by all calls
 *   - Every pointer is a DEVICE pointer unless the comment says "host".  The
 *     caller owns every buffer; the library allocates no device memory.  State
 *     kept between calls: a thread-local error string, the side streams mentioned
 *     below, per-device "kernel attributes are set" flags (set once under a mutex),
 *     and the built-in scratch array of lq_fit_grid_static with its per-device address.
 *   - All matrices are row-major fp32 with an explicit leading dimension
 *     counted in elements.  W is r x c with rows = output channels and
 *     columns = input channels, as in the paper (W in R^{r x c}).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; they do not synchronize.  Results are
 *     bit-identical from run to run (no atomics on floating-point data).
 *     lq_cholesky_inv and lq_hessian_accumulate_host also run part of their work on
 *     internal side streams (created once per host thread and device, default
 *     priority), forked from and joined back into `stream` with events, so ordering
 *     with respect to `stream` is unchanged.  The calls of the pass can be recorded
 *     into a HIP graph (kernels and event waits only).
 *   - `ws` is caller-provided scratch of at least lq_workspace_bytes() bytes,
 *     256-byte aligned, whose contents are undefined before and after a call.
 *   - Return value: LQ_OK or an error code; argument errors are found on the
 *     host before anything is launched.  lq_last_error() gives the text.
 */
#ifndef LEANQUANT_H
#define LEANQUANT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LQ_OK = 0,
  LQ_ERR_INVALID_ARG = 1, /* null pointer, bad size, bad leading dimension, bad parameter */
  LQ_ERR_NOT_PD = 2,      /* reserved for synchronous checks; device-side failures use `info` */
  LQ_ERR_UNSUPPORTED = 3, /* valid request outside what the kernels cover (limits below)   */
  LQ_ERR_WORKSPACE = 4,   /* ws is NULL, misaligned or smaller than lq_workspace_bytes()    */
  LQ_ERR_HIP = 5          /* a HIP runtime call or launch failed                            */
} lq_status;

typedef enum { LQ_GRID_NONUNIFORM = 0, LQ_GRID_AFFINE = 1 } lq_grid_mode;

typedef enum {
  LQ_CALL_HESSIAN = 0,
  LQ_CALL_CHOLESKY = 1,
  LQ_CALL_FIT_GRID = 2,
  LQ_CALL_QUANTIZE = 3,
  LQ_CALL_EXACT = 4
} lq_call;

/* Inputs of Algorithm 1 other than W and X, plus the grid-search constants. */
typedef struct lq_params {
  int32_t bits;            /* b: 2, 3 or 4                                                  */
  int32_t mode;            /* lq_grid_mode                                                  */
  int32_t group_size;      /* affine only: columns per (S, Z) group; 0 = whole row.
                              Must divide c.  Must be 0 in non-uniform mode (Section 2.1:
                              one grid per row).                                            */
  int32_t block;           /* B, lazy-update block width: 32, 64 or 128 (paper: 128)          */
  float damp;              /* df, dampening factor (Section 2.2: 0.01)                      */
  float p;                 /* outlier-preservation strength of Eq. 5 / Eq. 7 (paper: 4)     */
  int32_t T;               /* partitions of the weight range in Eq. 7 (paper: 2048)         */
  int32_t t_override;      /* < 0: t = floor(0.2T / 0.3T / 0.4T) for b = 4 / 3 / 2 (Eq. 8);
                              >= 0: use this t (0 = plain min-max grid); at most T/2        */
  int32_t kmeans_max_iter; /* cap on Lloyd updates (the fit stops earlier at a fixed point) */
} lq_params;

/* Fill *P with the paper's settings: b = 4, non-uniform, B = 128, df = 0.01, p = 4,
 * T = 2048, t from Eq. 8, at most 100 Lloyd updates.  P: host pointer. */
void lq_params_default(lq_params* P);

/*
 * Algorithm 1 line 3 / Section 2.2: H <- H + 2 X^T X for a chunk of calibration
 * tokens.  The paper writes X as c x N and H = 2 X X^T; here tokens are rows.
 *   H    [c x c], leading dimension ldh >= c.  Read and written in full (both
 *        triangles are kept equal).  The caller zero-fills it before the first chunk.
 *   X    [n_tokens x c], leading dimension ldx >= c.  Read only.
 *   n_tokens >= 0 (0 is a no-op), c >= 1.
 *   ws   LQ_CALL_HESSIAN scratch (partial sums of the token split).
 * The token range is split over workgroups and the partial sums are added in a
 * fixed order, so the result does not depend on scheduling.
 */
lq_status lq_hessian_accumulate(float* H, int64_t ldh, const float* X, int64_t n_tokens, int64_t c,
                                int64_t ldx, void* ws, size_t ws_bytes, void* stream);

/*
 * The same accumulation (Algorithm 1 line 3) for calibration activations that still sit in
 * HOST memory: X_host is cut into chunks of chunk_tokens rows; chunk k + 1 is copied to the
 * device on an internal copy stream while chunk k is accumulated on `stream` (two staging
 * buffers in ws).  The result is bit-identical to one lq_hessian_accumulate call per chunk.
 *   H         device [c x c] (ldh), as above; zero-filled by the caller before the first call.
 *   X_host    HOST pointer, [n_tokens x c] with leading dimension ldx >= c.  Read only; must
 *             stay valid and unchanged until the work enqueued on `stream` has finished.
 *             Page-locked memory (hipHostMalloc, or a pinned tensor) lets the copies overlap
 *             the kernels; with pageable memory the call is still correct but the copies
 *             block the host.
 *   chunk_tokens >= 1: rows per chunk (8192 - 32768 are sensible).
 *   ws        device scratch of lq_hessian_host_workspace_bytes(c, n_tokens, chunk_tokens)
 *             bytes, 256-byte aligned.
 * The call returns after enqueueing (with page-locked X_host); errors as lq_hessian_accumulate.
 */
lq_status lq_hessian_accumulate_host(float* H, int64_t ldh, const float* X_host, int64_t n_tokens,
                                     int64_t c, int64_t ldx, int64_t chunk_tokens, void* ws,
                                     size_t ws_bytes, void* stream);

/* Scratch size of lq_hessian_accumulate_host (partial sums + two chunk buffers); 0 for
 * invalid arguments.  Host function. */
size_t lq_hessian_host_workspace_bytes(int64_t c, int64_t n_tokens, int64_t chunk_tokens);

/*
 * Algorithm 1 line 4: dampen, invert, factor.
 *   H         [c x c] (ldh), symmetric, read only.
 *   damp      df; lambda = df * mean(diag H) is added to the diagonal.
 *   U         [c x c] (ldu) out: the UPPER Cholesky factor of (H + lambda I)^-1,
 *             i.e. (H + lambda I)^-1 = U^T U; entries below the diagonal are set to 0.
 *             (Rows U[j, j:] are what lines 16-19 of Algorithm 1 read.)
 *   hinv_diag [c] out: diag((H + lambda I)^-1), the inverse-Hessian diagonal of Eq. 5 / Eq. 7.
 *   info      one int32 out: 0 on success; k > 0 if the damped matrix is not positive
 *             definite, where k - 1 is the column at which a non-positive pivot appeared
 *             (U and hinv_diag are then meaningless but finite work still completes).
 *   ws        LQ_CALL_CHOLESKY scratch.
 * Computed as one factorization H_d = R R^T with R upper triangular followed by the
 * triangular inverse U = R^-1, which equals the literal invert-then-factor result.
 */
lq_status lq_cholesky_inv(const float* H, int64_t ldh, int64_t c, float damp, float* U, int64_t ldu,
                          float* hinv_diag, int32_t* info, void* ws, size_t ws_bytes, void* stream);

/*
 * Algorithm 1 lines 5-9: learn the grid of every row from the ORIGINAL weights.
 *   W          [r x c] (ldw), read only.
 *   hinv_diag  [c], from lq_cholesky_inv; importance omega_i is proportional to hinv_diag_i^-p.
 *   P          host pointer.
 *   grid  out  non-uniform: [r x 2^bits] ascending centroids of weighted k-means
 *                           (Eq. 5) started from the evenly spaced grid (Eq. 6);
 *              affine:      [r x (c / group) x 2] = (S, Z) minimizing Eq. 7 over
 *                           t_min, t_max in {0..t}; Z is an integer stored as float.
 * Limits: non-uniform c <= 16384; affine group (or row when group_size = 0) <= 8192.
 * r = 0 is a no-op (pointers are not looked at).
 */
lq_status lq_fit_grid(const float* W, int64_t r, int64_t c, int64_t ldw, const float* hinv_diag,
                      const lq_params* P, float* grid, void* ws, size_t ws_bytes, void* stream);

/*
 * lq_fit_grid with a caller-supplied starting grid for the weighted k-means of Eq. 5 instead of
 * Eq. 6's evenly spaced one (the paper's appendix compares Eq. 6 against k-means++ seeding; any
 * seeding can be computed by the caller and passed here).
 *   init_grid  [r x 2^bits] ascending, or NULL for Eq. 6 (then identical to lq_fit_grid).
 * Non-uniform mode only (an initial grid with an affine P is an argument error).
 */
lq_status lq_fit_grid_from(const float* W, int64_t r, int64_t c, int64_t ldw, const float* hinv_diag,
                           const lq_params* P, const float* init_grid, float* grid, void* ws,
                           size_t ws_bytes, void* stream);

/*
 * lq_fit_grid for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and
 * results as lq_fit_grid (bit-identical: the same kernels run), but the scratch (the importance
 * weights of the c columns, 12 bytes per column, and a row counter) lives in a 192 KiB array inside the library's
 * device image, one copy per GPU for the life of the process.  The call allocates nothing
 * (no hipMalloc / hipFree, no allocating library routine); the first call on a device looks up
 * the array's device address (with that device current) and keeps it.
 *   Limit: c <= 16384 (LQ_ERR_UNSUPPORTED beyond; use lq_fit_grid with a workspace).
 *   The array keeps the previous call's contents; every entry read is written first by the
 *   same call, so nothing is cleared.  All calls on one GPU share the array: two calls whose
 *   work overlaps on that GPU (different streams, or different host threads) race on it --
 *   order them on one stream or with events.
 */
lq_status lq_fit_grid_static(const float* W, int64_t r, int64_t c, int64_t ldw, const float* hinv_diag,
                             const lq_params* P, float* grid, void* stream);

/*
 * Weighted k-means++ seeding of the non-uniform grids: the initialisation that the paper's
 * appendix table on grid point initialisation compares Eq. 6 against.  Per row, centre 0 is
 * drawn with probability proportional to omega_i = (hinv_diag_i)^-p (Eq. 5's weights),
 * centre m with probability proportional to omega_i * min_j (w_i - g_j)^2; a draw takes the
 * first column whose cumulative mass reaches u * total and, if that column has no mass, the
 * next one that has; if no mass is left the first column is taken.  All in float64.
 *   W, r, c, ldw, hinv_diag, P   as lq_fit_grid; P->mode must be LQ_GRID_NONUNIFORM, c <= 16384.
 *   u          device [r x 2^b] float64 in [0, 1): the uniform numbers of the draws, supplied
 *              by the caller so that the result is a function of the arguments.
 *   grid_init  device [r x 2^b] out: the drawn centres (weights of the row) in ascending
 *              order, ready for lq_fit_grid_from.
 *   ws         LQ_CALL_FIT_GRID scratch.
 */
lq_status lq_kmeanspp_seed(const float* W, int64_t r, int64_t c, int64_t ldw, const float* hinv_diag,
                           const lq_params* P, const double* u, float* grid_init, void* ws,
                           size_t ws_bytes, void* stream);

/*
 * Algorithm 1 lines 10-21: for each block of B columns, quantize column by column
 * against the row's grid, scale the error by U_jj, propagate it inside the block,
 * then apply the dense rank-B update to all later columns.
 *   W        [r x c] (ldw) in/out: the working copy; on return it holds W_hat,
 *            the dequantized result Algorithm 1 returns.
 *   U        [c x c] (ldu) from lq_cholesky_inv, read only.
 *   grid     as written by lq_fit_grid for the same P; 16-byte aligned.
 *   codes    [r x c] uint8 out (leading dimension c): index into the ascending grid
 *            (non-uniform) or w_int of Section 2.1 (affine).
 *   row_loss [r] out or NULL: 1/2 sum_j E_kj^2, the loss errors of Eq. 3 summed per row.
 *   ws       LQ_CALL_QUANTIZE scratch (error blocks E of a group of 4 column blocks, packed
 *            diagonal blocks of U).
 * block: 32, 64 or 128.  r = 0 is a no-op (pointers are not looked at).
 */
lq_status lq_quantize_layer(float* W, int64_t r, int64_t c, int64_t ldw, const float* U, int64_t ldu,
                            const float* grid, const lq_params* P, uint8_t* codes, float* row_loss,
                            void* ws, size_t ws_bytes, void* stream);

/*
 * Algorithm 2 of the appendix (LeanQuant-Exact, for small networks): per row, in each of c
 * steps the not yet quantized weight with the smallest loss error (quant(w_i) - w_i)^2 /
 * (2 Hinv_ii) (Eq. 3) is quantized (ties: lowest index), the others move by
 * -Hinv[:, i] / Hinv_ii (w_i - w_hat_i), and row and column i leave the inverse (Eq. 9).
 * O(r c^3) and all in fp64; c <= 2048.
 *   W        [r x c] (ldw) in/out: on return the quantized rows W_hat.
 *   Hinv     [c x c] (ldh) DOUBLE, the symmetric damped inverse Hessian every row starts from,
 *            read only; lq_hinv_from_factor forms it as U^T U from lq_cholesky_inv's factor.
 *   grid     as written by lq_fit_grid for the same P (learned once from the original rows,
 *            lines 3-7 of Algorithm 2); affine mode takes one (S, Z) per row: group_size 0.
 *   codes    [r x c] uint8 out (leading dimension c).
 *   order    [r x c] int32 out or NULL: the index quantized at each step.
 *   row_loss [r] out or NULL: the summed loss errors of the row.
 *   ws       LQ_CALL_EXACT scratch: one c x c double matrix per resident workgroup
 *            (min(r, 512) of them).
 */
lq_status lq_quantize_exact(float* W, int64_t r, int64_t c, int64_t ldw, const double* Hinv,
                            int64_t ldh, const float* grid, const lq_params* P, uint8_t* codes,
                            int32_t* order, float* row_loss, void* ws, size_t ws_bytes, void* stream);

/* Hinv = U^T U in fp64 from the fp32 upper factor U [c x c] (ldu) of lq_cholesky_inv.
 * Hinv [c x c] (ldh) double out.  O(c^3) on the vector units: meant for the small c of
 * lq_quantize_exact. */
lq_status lq_hinv_from_factor(const float* U, int64_t ldu, int64_t c, double* Hinv, int64_t ldh,
                              void* stream);

/*
 * Stored form of a quantized layer.  The "Bits" columns of the paper's result tables count b
 * bits per weight plus sixteen bits per grid point per row (non-uniform grids: one set of 2^b
 * points per row, Section 2.1) or per scale and per zero-point of a group (affine grids):
 * 4.05 / 3.02 / 2.01 and 4.25 at group size 128.  The byte layout is this library's:
 *   packed  [r x packed_ld] bytes, packed_ld >= lq_packed_row_bytes(c, bits): a row's codes
 *           as a little-endian bit stream, code j in bits [j b, (j + 1) b) (bit k of the
 *           stream is bit k % 8 of byte k / 8); unused high bits of the row's last byte are 0;
 *   table   non-uniform: [r x 2^bits] IEEE binary16 bit patterns, the grid rounded to nearest
 *           even; affine: [r x (c / group) x 2] = (binary16 S, int16 Z saturated to 16 bits).
 * lq_pack_layer reads codes [r x c] (leading dimension c) and grid as written by
 * lq_quantize_layer / lq_fit_grid for the same P.  lq_unpack_layer writes the weights the
 * stored form stands for, W_hat[k][j] = table[k][code] or (code - Z) S of the column's group
 * (Section 2.1), into W_hat [r x c] (ldw); they equal lq_quantize_layer's W up to the
 * 16-bit rounding of the table.  codes (may be NULL) receives the unpacked codes [r x c].
 * No workspace.  r = 0 is a no-op.
 */
int64_t lq_packed_row_bytes(int64_t c, int32_t bits);              /* ceil(c bits / 8); -1 if invalid */
double lq_bits_per_weight(int64_t r, int64_t c, const lq_params* P); /* host only; -1 if invalid   */
lq_status lq_pack_layer(const uint8_t* codes, const float* grid, int64_t r, int64_t c,
                        const lq_params* P, uint8_t* packed, int64_t packed_ld, uint16_t* table,
                        void* stream);
lq_status lq_unpack_layer(const uint8_t* packed, int64_t packed_ld, const uint16_t* table, int64_t r,
                          int64_t c, const lq_params* P, float* W_hat, int64_t ldw, uint8_t* codes,
                          void* stream);

/*
 * Product with a stored layer, as a quantized linear layer does when decoding (the paper's
 * appendix on inference efficiency): Y[n][k] = sum_j W_hat[k][j] X[n][j] with W_hat the
 * weights the stored form stands for (see lq_unpack_layer), fp32 accumulation.
 *   packed, table  as written by lq_pack_layer for the same P; packed rows 16 / 4 / 8-byte
 *                  aligned for 4 / 3 / 2 bits (base pointer and packed_ld).
 *   X  [nb x c] fp32, rows contiguous, 16-byte aligned;  Y [nb x r] fp32 out.
 * One pass over the codes serves up to 4 input vectors (2 for c > 8192); larger nb takes
 * ceil(nb / 4) passes.  Limits: c a multiple of 32 and at
 * most 16384; affine groups multiples of 32 columns.  No workspace.
 */
lq_status lq_matvec_packed(const uint8_t* packed, int64_t packed_ld, const uint16_t* table, int64_t r,
                           int64_t c, const lq_params* P, const float* X, int64_t nb, float* Y,
                           void* stream);

/*
 * The same product for a batch (the GEMM form): Y[n][k] = sum_j W_hat[k][j] X[n][j] for nb input
 * vectors, with the stored weights decoded once per 32 or 64 vectors into fp32 tiles in LDS and
 * multiplied on the fp32 matrix cores, fp32 accumulation in a fixed order.  Arguments, layouts
 * and alignment as lq_matvec_packed (X [nb x c], Y [nb x r]); c a multiple of 32 (no upper
 * limit), affine groups multiples of 32 columns.  Meant for nb >= 16: below that
 * lq_matvec_packed's passes over the codes are faster.  No workspace.
 */
lq_status lq_matmul_packed(const uint8_t* packed, int64_t packed_ld, const uint16_t* table, int64_t r,
                           int64_t c, const lq_params* P, const float* X, int64_t nb, float* Y,
                           void* stream);

/* Scratch bytes a call needs (host-only computation).  n_tokens is used by
 * LQ_CALL_HESSIAN only; r by FIT_GRID/QUANTIZE/EXACT; P may be NULL for HESSIAN/CHOLESKY/EXACT.
 * For LQ_CALL_HESSIAN the size depends on how the token range is cut and is NOT monotonic in
 * n_tokens: a workspace shared by calls with different chunk sizes must cover the maximum. */
size_t lq_workspace_bytes(int which_call, int64_t r, int64_t c, int64_t n_tokens, const lq_params* P);

/* Text of the last error on the calling thread ("" if none).  Never NULL.  Host pointer. */
const char* lq_last_error(void);

/* Library version as "major.minor". */
const char* lq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LEANQUANT_H */
