/*
 * vlut.h -- C ABI of the vector-LUT ternary x INT8 mixed-precision GEMM for
 * AMD Instinct MI355X (gfx950).
 *
 * The library computes O = W x A (Vec-LUT paper, Table 2) for ternary weights
 * W in {-1,0,+1}^(M x K) and INT8 activations A in Z^(K x N), N parallel tokens,
 * with the paper's vector-table method (Sec. 3.2, Alg. 1): every g = 4
 * consecutive weights of a row are one base-3 byte, every group of 4 activation
 * rows yields one sub-table of 3^4 = 81 signed partial sums across the N tokens,
 * and each packed byte performs one 1 -> N lookup-accumulate.
 *
 * Conventions for every entry point
 *   - Pointers marked "dev" are device (HBM) pointers of the current HIP device;
 *     pointers marked "host" are ordinary host pointers.  Nothing is copied
 *     between host and device by the library.
 *   - The caller owns every buffer.  The library allocates no device memory.
 *     State it keeps between calls: (i) the per-thread tuning override of
 *     vlut_set_plan (and a per-thread cache of the launch plans chosen for the
 *     last few shapes, emptied by vlut_set_plan); (ii) one 4-byte device flag
 *     per GPU that the pack kernels raise for a non-ternary weight, reset and
 *     read back inside every vlut_pack_weights* call under a host mutex (the
 *     pack calls of one process are therefore serialised); (iii) one bit per
 *     kernel and device that records that the kernel's LDS limit was raised.
 *     None of it influences results.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Runtime entry points only enqueue work on `stream`; they never
 *     synchronise.  vlut_pack_weights is an offline step and may synchronise.
 *   - Return value: VLUT_OK (0) or a negative VLUT_ERR_* code.  Argument checks
 *     (null pointers, shapes, buffer sizes) happen before the first HIP call,
 *     so they behave the same on a machine without a GPU.  No exception crosses
 *     this boundary.
 *   - Shapes: M >= 1, N >= 1, K >= 4 and K % 4 == 0 (the paper's g | K condition,
 *     Sec. 3.3 "Flexible sub-2-bit weight packing"); M, N need not be multiples
 *     of any tile.  Each of M, K, N must be below 2^24.
 */
#ifndef VLUT_H
#define VLUT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VLUT_OK 0
#define VLUT_ERR_NULL (-1)         /* a required pointer is NULL                      */
#define VLUT_ERR_SHAPE (-2)        /* M, K, N, ldx or ldy outside the supported range */
#define VLUT_ERR_SMALL_BUFFER (-3) /* a byte count passed in is below the required one */
#define VLUT_ERR_VALUE (-4)        /* a weight outside {-1,0,+1}                      */
#define VLUT_ERR_DEVICE (-5)       /* a HIP call or kernel launch failed              */
#define VLUT_ERR_UNSUPPORTED (-6)  /* valid request this build cannot serve           */

#define VLUT_GROUP 4     /* g: weights per packed byte (2.00 bits per weight, the paper's I2) */
#define VLUT_ROWS 81     /* 3^g rows per sub-table                                            */

/* Human-readable name of a status code (static storage, never NULL). */
const char* vlut_status_string(int status);

/* Library version, major * 10000 + minor * 100 + patch. */
int vlut_version(void);

/*
 * Bytes of the packed weight blob for an M x K matrix (0 if the shape is
 * invalid).  The blob holds one byte per group of 4 weights (Sec. 3.3
 * "Tile-contiguous packed weight layout"), in tiles of 4 rows x 16 groups;
 * rows are padded to a multiple of 4 and groups to a multiple of 16 with the
 * byte 40 (the all-zero pattern), so the size is
 * ceil(M/4) * ceil(K/64) * 64.  The blob is position independent: it can be
 * saved and reloaded byte for byte.
 */
size_t vlut_packed_weight_bytes(int64_t M, int64_t K);

/*
 * Byte offset, inside the packed blob, of the index of row m and group kg
 * (weights W[m][4kg .. 4kg+3]).  Host-only helper that documents the tile
 * layout; returns (size_t)-1 for an out-of-range argument.
 */
size_t vlut_packed_offset(int64_t M, int64_t K, int64_t m, int64_t kg);

/*
 * Bytes of the quantised activation buffer a_q for K x N activations: ceil(N/8) * K * 8.
 * Layout (token-chunked, the GPU form of Sec. 3.3's token-contiguous activations): tokens are grouped in
 * chunks of 8; a_q[(n/8)][k][n%8], i.e. for every k the 8 tokens of a chunk are 8 consecutive bytes and
 * a chunk's [K][8] block is contiguous.  Tokens past N in the last chunk hold 0.  0 if the shape is invalid.
 */
size_t vlut_act_bytes(int64_t K, int64_t N);

/* Bytes of the full vector table T for K x N activations: (K/4) * 81 * N * 2
 * (Sec. 1 quotes 285.5 MiB for K = 14436, N = 512).  0 if the shape is invalid. */
size_t vlut_lut_bytes(int64_t K, int64_t N);

/*
 * Bytes of scratch vlut_mpgemm / vlut_mpgemm_rows need for this shape (split-K partial sums); may be 0.  One size
 * serves both table variants (lut_or_null NULL or not).  The size depends on the launch plan, hence on the
 * vlut_set_plan override of the CALLING THREAD: query it on the thread that makes the call, after any
 * vlut_set_plan (a size taken under another override may be too small, which vlut_mpgemm reports as
 * VLUT_ERR_SMALL_BUFFER, never by writing out of bounds).  0 also when the override fits the shape with no plan.
 */
size_t vlut_workspace_bytes(int64_t M, int64_t K, int64_t N);

/*
 * Offline weight transformation (Sec. 3.1 stage i, Sec. 3.3): ternary weights
 * to base-3 bytes, idx = sum_j (W[m][4kg+j] + 1) * 3^(3-j), so that the byte's
 * decimal value is the table row (Fig. 5 caption; the digit order follows the
 * worked example of Sec. 3.2: 23 <-> (-1,+1,0,+1)), stored in the tile layout
 * described at vlut_packed_weight_bytes.
 *   w_ternary    dev, int8 [M][K] row-major, every value in {-1,0,+1}
 *   packed       dev, packed_bytes >= vlut_packed_weight_bytes(M, K); fully overwritten
 * Synchronises `stream` to report VLUT_ERR_VALUE when a weight is not ternary
 * (the blob content is then unspecified).
 */
int vlut_pack_weights(const int8_t* w_ternary, int64_t M, int64_t K, uint8_t* packed,
                      size_t packed_bytes, void* stream);

/*
 * Per-token symmetric INT8 quantisation fused with the transposition to the
 * token-contiguous layout (Sec. 3.4 first paragraph; Sec. 3.3 "Fused activation
 * and output transformation").  For every token n, in fp32:
 *   amax = max_k |x[n][k]|;  a_scale[n] = amax / 127;
 *   inv = 127 / amax (0 when amax == 0);
 *   a_q[k][n] = clamp(round_half_even(x[n][k] * inv), -127, 127).
 * -128 is never produced (the INT16 block bound of Sec. 3.4 relies on |q| <= 127).
 *   x        dev, fp32 [N][ldx], feature-contiguous, ldx >= K; finite values
 *   a_q      dev, int8, token-chunked [ceil(N/8)][K][8] (see vlut_act_bytes), 16-byte aligned; the
 *            caller provides vlut_act_bytes(K, N) bytes; fully overwritten, padding tokens included
 *   a_scale  dev, fp32 [N]
 */
int vlut_quantize_act(const float* x, int64_t N, int64_t K, int64_t ldx, int8_t* a_q,
                      float* a_scale, void* stream);

/*
 * Materialises the whole vector table in device memory (Alg. 1 function
 * Precompute, Eq. 1, built with the topological order of Sec. 4):
 *   lut[kg][i][n] = sum_{j<4} (digit_j(i) - 1) * A[4kg+j][n],   A[k][n] = a_q[n/8][k][n%8],
 * digit_0 the most significant base-3 digit of i; int16, layout [K/4][81][N]
 * with N contiguous (Sec. 3.3 "Token-contiguous LUT layout").
 *   lut_bytes >= vlut_lut_bytes(K, N)
 * The hot path does not need this call (it builds table tiles in LDS on the
 * fly, Sec. 3.4 "Streamed precomputing-lookup execution"); it exists for
 * inspection and for the un-streamed variant of vlut_mpgemm.
 */
int vlut_build_lut(const int8_t* a_q, int64_t K, int64_t N, int16_t* lut, size_t lut_bytes,
                   void* stream);

/*
 * Layout ablation (Sec. 5.6 "Vector LUT-centric tensor layout", Sec. 3.3): the same table with the token index
 * outermost, lut[n][kg][i] (one table per token, the scalar-LUT arrangement; vlut_lut_bytes(K, N) bytes), and the
 * mpGeMM on it, where every lookup yields one value for one token.  Same numbers as vlut_mpgemm; arguments as there
 * (no workspace; N <= 262140).  These two calls exist to measure what the token-contiguous layout buys.
 */
int vlut_build_lut_token_outer(const int8_t* a_q, int64_t K, int64_t N, int16_t* lut, size_t lut_bytes,
                               void* stream);
int vlut_mpgemm_token_outer(const uint8_t* packed, float w_scale, const float* a_scale, const int16_t* lut,
                            int64_t M, int64_t K, int64_t N, float* y, int64_t ldy, int32_t* acc_or_null,
                            void* stream);

/*
 * The mpGeMM itself (Alg. 1 main loop, Eq. 2; Sec. 3.4): for every packed byte
 * one lookup of an 81-row sub-table row and a vector add over the tokens,
 * INT16 inside blocks of at most 64 lookups, INT32 across blocks, then the
 * scale step y[n][m] = (float)acc[m][n] * (w_scale * a_scale[n]).
 *   packed        dev, 16-byte aligned (VLUT_ERR_UNSUPPORTED otherwise), blob written by
 *                 vlut_pack_weights for the same M, K
 *   w_scale       per-tensor weight scale
 *   a_q, a_scale  dev, as written by vlut_quantize_act for the same K, N
 *   lut_or_null   dev or NULL.  NULL: sub-tables are built in LDS tile by tile
 *                 (streamed, the default).  Non-NULL: a table written by
 *                 vlut_build_lut for (a_q, K, N) is read instead (un-streamed
 *                 variant kept for the ablation of Sec. 5.6).
 *   y             dev, fp32 [N][ldy], feature-contiguous, ldy >= M; may be NULL
 *                 when acc_or_null is given
 *   acc_or_null   dev or NULL, int32 [M][N] raw accumulators (token-contiguous)
 *   workspace     dev, workspace_bytes >= vlut_workspace_bytes(M, K, N); may be
 *                 NULL when that size is 0
 * For a few tokens (streamed tables, no plan override: always for N <= 2, up to N = 32 while one workgroup per
 * row tile and token pair fits the device at once) a kernel specialised for that case runs instead and needs no
 * workspace; the results are the same numbers.
 */
int vlut_mpgemm(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale,
                const int16_t* lut_or_null, int64_t M, int64_t K, int64_t N, float* y, int64_t ldy,
                int32_t* acc_or_null, void* workspace, size_t workspace_bytes, void* stream);

/*
 * vlut_mpgemm for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same numbers as vlut_mpgemm with
 * lut_or_null == NULL; the split-K partial sums go to a scratch array that is part of the library's device image
 * (VLUT_STATIC_SCRATCH_BYTES per GPU the library runs on, held until the process ends).  The call allocates
 * nothing and frees nothing; the first call on a device looks the array's address up once.
 *   arguments      as in vlut_mpgemm (no lut, no workspace)
 *   returns        VLUT_ERR_UNSUPPORTED when vlut_workspace_bytes(M, K, N) exceeds VLUT_STATIC_SCRATCH_BYTES
 *                  (nothing is launched then); otherwise as vlut_mpgemm
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams or threads)
 * race on it and must be serialised by the caller; calls on one stream are ordered and safe.  Nothing is carried
 * from one call to the next (each call overwrites every slot it later reads).
 */
#define VLUT_STATIC_SCRATCH_BYTES (32u << 20)
size_t vlut_static_scratch_bytes(void);
int vlut_mpgemm_static(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale, int64_t M,
                       int64_t K, int64_t N, float* y, int64_t ldy, int32_t* acc_or_null, void* stream);

/*
 * vlut_mpgemm for several weight matrices that multiply the same activations in one launch (the q/k/v or the
 * gate/up projections of a decoder layer).  The tables depend on the activations only (Eq. 1, Sec. 3.2), so the
 * matrices are stacked along M before vlut_pack_weights and share every table a workgroup builds; each output
 * row carries its own matrix' weight scale:
 *   y[n][m] = (float)acc[m][n] * (w_scale_rows[m] * a_scale[n]).
 *   w_scale_rows  dev, fp32 [M]: the weight scale of the matrix row m belongs to (required)
 * Everything else as in vlut_mpgemm (same workspace size, same error codes).
 */
int vlut_mpgemm_rows(const uint8_t* packed, const float* w_scale_rows, const int8_t* a_q, const float* a_scale,
                     const int16_t* lut_or_null, int64_t M, int64_t K, int64_t N, float* y, int64_t ldy,
                     int32_t* acc_or_null, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Quantisation and mpGeMM in one call, from fp32 activations: the steps of vlut_quantize_act (Sec. 3.4 first
 * paragraph: per-token absmax INT8) and of vlut_mpgemm / vlut_mpgemm_rows (Alg. 1, Eq. 2) with the same readings and
 * the same numbers.  For a few tokens (decoding: always for N <= 2, up to N = 32 where a cost estimate favours it,
 * reported by vlut_query_plan_f32 with J = 0; K <= 35840 for one token, 39936 for more) it is one launch: a
 * workgroup quantises the rows of its one or two tokens itself (absmax over the whole row, codes kept in LDS), so
 * that neither the INT8 activations nor a second kernel are needed.  For more tokens the quantiser runs as a kernel
 * of its own into the workspace, ahead of the lookup kernel (measured to be the faster arrangement); a lookup kernel that quantises the 8 tokens of its tile itself exists as
 * well and is taken when vlut_set_plan forces a plan with J = 16 whose K range per workgroup is at most 8704.
 *   x             dev, fp32 [N][ldx], ldx >= K (16-byte aligned rows are read as float4)
 *   w_scale / w_scale_rows_or_null   per-tensor scale, or (non-NULL) dev fp32 [M] per-row scales as in
 *                 vlut_mpgemm_rows (w_scale is then ignored)
 *   y, ldy, acc_or_null              as in vlut_mpgemm
 *   a_scale_out_or_null              dev or NULL, fp32 [N]: receives the token scales s_n = amax_n / 127
 *   workspace     dev, 16-byte aligned, workspace_bytes >= vlut_workspace_bytes_f32(M, K, N); may be NULL when that
 *                 size is 0
 * vlut_query_plan_f32 tells which form a shape takes:
 *   out5 = {J, R, split_k, workgroups, fused (1) or two launches (0)}  (J, R as in vlut_query_plan)
 * Errors as in vlut_mpgemm; VLUT_ERR_SHAPE also for ldx < K.
 */
size_t vlut_workspace_bytes_f32(int64_t M, int64_t K, int64_t N);            /* 0 if the shape is invalid      */
int vlut_query_plan_f32(int64_t M, int64_t K, int64_t N, int* out5);
int vlut_mpgemm_f32(const uint8_t* packed, float w_scale, const float* w_scale_rows_or_null, const float* x, int64_t ldx,
                    int64_t M, int64_t K, int64_t N, float* y, int64_t ldy, int32_t* acc_or_null,
                    float* a_scale_out_or_null, void* workspace, size_t workspace_bytes, void* stream);

/*
 * 1.60-bit packing (g = 5, the paper's I1; Sec. 3.3 "Flexible sub-2-bit weight packing", Fig. 5): five weights per
 * base-3 byte, idx = sum_j (W[m][5kg+j] + 1) * 3^(4-j) in [0, 243), 243-row sub-tables, INT16 blocks of at most
 * 51 = floor(32767 / (127 * 5)) lookups (Sec. 3.4).  Shapes: K >= 5 and K % 5 == 0 (g | K); together with
 * vlut_quantize_act's K % 4 == 0 the whole path needs K % 20 == 0.  The blob has the tile layout of the 2-bit one
 * with K/5 groups per row: ceil(M/4) * ceil((K/5)/16) * 64 bytes, padded with byte 121 (the all-zero pattern).
 * Results are the same numbers as vlut_mpgemm's: the packing changes the table, not the product.
 */
#define VLUT_GROUP_G5 5
#define VLUT_ROWS_G5 243
size_t vlut_packed_weight_bytes_g5(int64_t M, int64_t K);                    /* 0 if the shape is invalid      */
size_t vlut_packed_offset_g5(int64_t M, int64_t K, int64_t m, int64_t kg);   /* (size_t)-1 if out of range     */
size_t vlut_workspace_bytes_g5(int64_t M, int64_t K, int64_t N);             /* split-K partial sums; may be 0 */
/* As vlut_pack_weights, for the 1.60-bit blob (synchronises `stream` to report VLUT_ERR_VALUE). */
int vlut_pack_weights_g5(const int8_t* w_ternary, int64_t M, int64_t K, uint8_t* packed, size_t packed_bytes,
                         void* stream);
/*
 * As vlut_mpgemm (streamed tables only: there is no materialised-table variant), on a blob written by
 * vlut_pack_weights_g5.  a_q (8-byte aligned) and a_scale as written by vlut_quantize_act for the same K, N.
 */
int vlut_mpgemm_g5(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale, int64_t M, int64_t K,
                   int64_t N, float* y, int64_t ldy, int32_t* acc_or_null, void* workspace, size_t workspace_bytes,
                   void* stream);
/* Tuning hooks of the 1.60-bit kernel: row groups per wave R in {1,2,4,6,9,12,14} and split-K factor (0 = automatic);
 * out3 (host, 3 ints) = { R, split_k, number of workgroup tiles }. */
int vlut_set_plan_g5(int R, int split_k);
int vlut_query_plan_g5(int64_t M, int64_t K, int64_t N, int* out3);

/*
 * Mixed 1.60-bit / 2-bit packing (Sec. 3.3 "Flexible sub-2-bit weight packing": different packings for different
 * groups of weights, so that almost any K is served at close to 1.6 bits per weight).  Here: the first
 * K5 = 20 * floor(K / 20) input features of every row are packed five per byte, the remaining K - K5 < 20 (a multiple
 * of 4, as the quantiser's K % 4 == 0 demands) four per byte; K5 = 0 or K - K5 = 0 leave one part empty.
 *   blob = [vlut_pack_weights_g5 blob of W[:, :K5]] [vlut_pack_weights blob of W[:, K5:]]
 *   vlut_mixed_k5(K)            K5, or -1 if K is not a positive multiple of 4
 * vlut_mpgemm_mixed runs each part through its kernel in partial-sum mode (a_q: the part's range of activation rows)
 * and adds the parts with the split-K parts in one exact INT32 pass before the scale step: the same numbers as
 * vlut_mpgemm.  The workspace (vlut_workspace_bytes_mixed, never 0) is required; other arguments and errors as in
 * vlut_mpgemm (streamed tables only).
 */
int64_t vlut_mixed_k5(int64_t K);
size_t vlut_packed_weight_bytes_mixed(int64_t M, int64_t K);                 /* 0 if the shape is invalid      */
size_t vlut_workspace_bytes_mixed(int64_t M, int64_t K, int64_t N);
int vlut_pack_weights_mixed(const int8_t* w_ternary, int64_t M, int64_t K, uint8_t* packed, size_t packed_bytes,
                            void* stream);
int vlut_mpgemm_mixed(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale, int64_t M,
                      int64_t K, int64_t N, float* y, int64_t ldy, int32_t* acc_or_null, void* workspace,
                      size_t workspace_bytes, void* stream);

/* Bytes of scratch vlut_mpgemm_mfma needs (INT32 partial sums when it splits K over workgroups); may be 0. */
size_t vlut_mfma_workspace_bytes(int64_t M, int64_t K, int64_t N);

/*
 * Same contract and same results as vlut_mpgemm (lut_or_null must be NULL), but
 * computed the multiply-add way the paper contrasts with (Sec. 2.2.1): packed
 * bytes are unpacked to INT8 and multiplied on the INT8 matrix cores, as a tiled
 * GEMM (128 rows x up to 128 tokens per workgroup, operands staged in LDS, K split
 * over workgroups for few tokens).  In-run comparison only.  workspace: 16-byte
 * aligned, workspace_bytes >= vlut_mfma_workspace_bytes(M, K, N); may be NULL when
 * that size is 0.  packed and a_q must be 16-byte aligned.
 */
int vlut_mpgemm_mfma(const uint8_t* packed, float w_scale, const int8_t* a_q, const float* a_scale,
                     const int16_t* lut_or_null, int64_t M, int64_t K, int64_t N, float* y,
                     int64_t ldy, int32_t* acc_or_null, void* workspace, size_t workspace_bytes,
                     void* stream);

/*
 * Tuning hook: forces the launch plan of vlut_mpgemm for subsequent calls from
 * this thread (interleave factor J in {1,2,4,8,16} = sub-tables per 256-byte
 * table row, row groups per wave R in 1..16, `waves` = lookup waves of the 16-wave
 * workgroup: 12 (four waves build the tables) or 14 (two do), split-K factor).
 * Any argument 0 = choose automatically.  Returns VLUT_ERR_UNSUPPORTED for a
 * combination the kernels are not built for.  Whether an accepted override
 * fits a given shape is only known at the call: when it does not (R > 6 where
 * a lane makes more than 64 lookups, a split-K factor above the number of K
 * stages), vlut_mpgemm*, vlut_query_plan* return VLUT_ERR_UNSUPPORTED instead of
 * running another plan.  Results never depend on the plan.
 */
int vlut_set_plan(int J, int R, int waves, int split_k);

/*
 * Reports the launch plan vlut_mpgemm would use for this shape (after any vlut_set_plan override of the
 * calling thread): out4 (host, 4 ints) = { J, R, split_k, number of workgroup tiles }.  (The launch itself has at
 * most one workgroup per compute unit; each walks through its share of the tiles.)
 * With few tokens and no override (N <= 2 always; 3 <= N <= 32 when ceil(N/2) copies of the row tiles are at most
 * 256 workgroups and a cost estimate favours it: few rows per workgroup, or a short K), vlut_mpgemm uses a kernel
 * of its own (two tokens per
 * workgroup, table entries of one dword, every workgroup sweeps all of K, no workspace); it is reported as
 * { 0, rows per workgroup, 1, number of workgroups }.
 */
int vlut_query_plan(int64_t M, int64_t K, int64_t N, int* out4);

/*
 * Lookup waves per workgroup of the plan vlut_query_plan reports (12 or 14: a workgroup tile holds 4 * waves * R output
 * rows); 0 when the few-token kernel runs; a negative VLUT_ERR_* code for an invalid shape or an override that does
 * not fit it.
 */
int vlut_query_lookup_waves(int64_t M, int64_t K, int64_t N);

#ifdef __cplusplus
}
#endif
#endif /* VLUT_H */
