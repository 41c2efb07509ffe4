/* btc.h -- C ABI of the MI355X (gfx950) binary-codebook linear layer.
 *
 * The layer computes  y = W_hat . x  for a weight matrix stored as
 *   - a codebook of K sign patterns of length v (one uint32 bit mask each),
 *   - per weight row, ceil(in/v) indices of ceil(log2 K) bits, one per
 *     length-v chunk of the row, and
 *   - a per-row scale alpha_i and per-row mean mu_i,
 * with  W_hat[i][j*v+t] = alpha_i * (bit t of codebook[idx[i][j]] ? +1 : -1) + mu_i
 * (paper: Algorithm "Binary Transformation and Compression", steps
 * "Reconstruct binary" / "Dequantize"; appendix "Binary Codebook LUT-GEMM",
 * definition of W and of y_r as a sum over blocks; Section "Compression
 * Analysis" for the storage format).
 *
 * Conventions for every entry point
 *   - Every array pointer is a DEVICE pointer owned by the caller unless the
 *     comment says "host".  The library allocates no device memory and keeps
 *     no state between calls; scratch space is the caller's `workspace`.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Compute calls enqueue work and return; only btc_pack and btc_update
 *     wait, to return the result of a range check (see there).
 *   - Array pointers must be 16-byte aligned (BTC_ERR_ALIGN otherwise).
 *   - Errors are returned, never thrown; on an argument error nothing was
 *     enqueued.
 *   - Matrices are row-major.  Activations are X[rows][in], outputs
 *     Y[rows][out] (Y = X W^T, Section "Integration into Transformer
 *     Architecture").  A row of X has exactly `in` elements; positions
 *     in .. nchunks*v-1 of the last chunk are logical zeros and are never read.
 *
 * Besides the layer itself (btc_pack, btc_unpack, btc_gemv, btc_gemm) the
 * library holds the step in front of it at inference, btc_transform (the online
 * activation transform), and one round of the offline codebook clustering that
 * produces the indices, btc_assign and btc_update.
 */
#ifndef BTC_H_
#define BTC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BTC_OK = 0,
  BTC_ERR_NULL = -1,         /* a required pointer is NULL                       */
  BTC_ERR_SHAPE = -2,        /* inconsistent or non-positive sizes               */
  BTC_ERR_UNSUPPORTED = -3,  /* v, K, batch or dtype outside the supported range */
  BTC_ERR_ALIGN = -4,        /* pointer not 16-byte aligned                      */
  BTC_ERR_INDEX_RANGE = -5,  /* btc_pack met an index outside [0, K)             */
  BTC_ERR_HIP = -6,          /* a HIP runtime call failed                        */
  BTC_ERR_WORKSPACE = -7     /* workspace missing or too small                   */
} btc_status;

typedef enum { BTC_F16 = 0, BTC_BF16 = 1, BTC_F32 = 2 } btc_dtype;

/* One packed layer.  Plain data, filled by btc_shape_init. */
typedef struct {
  int32_t out;            /* weight rows    = length of y                          */
  int32_t in;             /* weight columns = length of x                          */
  int32_t v;              /* chunk (sub-vector) length, 1..32                      */
  int32_t K;              /* codebook entries, 2..65536                            */
  int32_t b;              /* index width ceil(log2 K), 1..16                       */
  int32_t nchunks;        /* ceil(in / v) chunks per row                           */
  int32_t words_per_row;  /* ceil(nchunks*b / 32): row stride of `packed`, uint32  */
} btc_shape;

/* Host. Fill *s from (out, in, v, K).  BTC_ERR_SHAPE for non-positive sizes,
 * BTC_ERR_UNSUPPORTED for v > 32 or K outside 2..65536. */
btc_status btc_shape_init(btc_shape* s, int32_t out, int32_t in, int32_t v, int32_t K);

/* Host. Bytes of the packed index stream, out * words_per_row * 4
 * (Compression Analysis: ceil(log2 c) bits per vector, here padded so that
 * every row starts on a 32-bit word). 0 if s is NULL. */
size_t btc_packed_bytes(const btc_shape* s);

/* Host. Bytes of workspace the call would need: rows = batch for btc_gemv
 * (is_gemm = 0), rows = M for btc_gemm (is_gemm != 0).  Always >= 16 so that
 * one buffer serves btc_pack too.
 * The workspace is device memory owned by the caller, 16-byte aligned.  It
 * must be ZERO-FILLED before its first use by btc_gemv; every btc_gemv call
 * leaves it zero again (partial sums travel between workgroups in tagged
 * slots whose empty state is 0; a call with several activation rows parks
 * fp32 partial sums behind them and zeroes them in its second pass), so one
 * buffer serves any number of calls
 * that are ordered on a stream.  Calls that may overlap in time (different
 * streams) need a buffer each: sharing one is a data race.  btc_gemm (and
 * btc_gemm_aq, btc_weight_rowsums) write scratch values there -- partial sums,
 * and for calls with many rows the sign matrix as one byte per weight -- and
 * need no particular contents; give them a buffer of their own, or zero the
 * buffer again before the next btc_gemv: a stale non-zero word in a slot
 * would be read as a valid partial sum, silently.  The table engine waits
 * for a missing partial sum for a bounded number of polls and then stores
 * NaN with status BTC_OK (it cannot happen while every workgroup of the call
 * runs; it would after an aborted earlier call): the outputs are then NaN
 * and the workspace must be zero-filled again. */
size_t btc_workspace_bytes(const btc_shape* s, int32_t rows, int is_gemm);

/* Index matrix -> bit stream (Compression Analysis; storage format of the
 * index matrix I in appendix "Binary Codebook LUT-GEMM").
 *   idx    : int32 [out][nchunks]
 *   packed : uint32 [out][words_per_row]; index j of row i occupies bits
 *            [j*b, (j+1)*b) of row i's stream, bit p of the stream being bit
 *            (p & 31) of word (p >> 5); unused tail bits are written as 0.
 *   workspace : >= 16 bytes, receives a range-check flag.
 * Waits for the stream: returns BTC_ERR_INDEX_RANGE if any index is outside
 * [0, K) (packed is then unspecified). */
btc_status btc_pack(void* stream, const btc_shape* s, const int32_t* idx, uint32_t* packed,
                    void* workspace, size_t workspace_bytes);

/* Bit stream -> index matrix; exact inverse of btc_pack. Enqueues and returns. */
btc_status btc_unpack(void* stream, const btc_shape* s, const uint32_t* packed, int32_t* idx);

/* Decode-time product for a few activation rows (appendix "Binary Codebook
 * LUT-GEMM": y_r = sum_j <x_j, C[I_rj]>; dequantisation alpha * B_hat + mu):
 *   y[m][i] = alpha[i] * sum_j <x[m] chunk j, C[idx[i][j]]> + mu[i] * sum_k x[m][k]
 *   packed   : uint32 [out][words_per_row]    codebook : uint32 [2^b] (entries
 *              K .. 2^b-1 must be readable; bit t of entry k = element t, 1 => +1)
 *   alpha,mu : float [out]
 *   x        : fp16 [batch][in], batch 1..16
 *   y        : [batch][out] of y_dtype (BTC_F16 or BTC_F32, round to nearest even)
 *   workspace: btc_workspace_bytes(s, batch, 0) bytes, see there (zero-filled)
 * Accumulates in fp32.  A stored index >= K reads codebook[index] inside the
 * 2^b-entry table.  Enqueues and returns.  Errors: BTC_ERR_NULL, _SHAPE,
 * _UNSUPPORTED (batch outside 1..16, y_dtype), _ALIGN, _WORKSPACE (missing
 * or too small for the engine chosen), _HIP (launch failed). */
btc_status btc_gemv(void* stream, const btc_shape* s, const uint32_t* packed,
                    const uint32_t* codebook, const float* alpha, const float* mu,
                    const void* x, int32_t batch, void* y, btc_dtype y_dtype,
                    void* workspace, size_t workspace_bytes);

/* btc_gemv for callers that cannot allocate or pass device scratch memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments (without the workspace), same kernels, same
 * results and errors as btc_gemv.  Whatever btc_gemv would park in the caller's workspace goes to a static
 * device array of 8 MiB inside the library (one copy per GPU, held until the process ends; its address is looked
 * up on the first call on a device).  The call allocates nothing, on the host or the device.  A call whose engine
 * needs more than 8 MiB returns BTC_ERR_WORKSPACE and enqueues nothing (use btc_gemv with a workspace of
 * btc_workspace_bytes(s, batch, 0) bytes).  All calls on one GPU share the array: the part a call uses is cleared by
 * a small kernel at its start, calls ordered on one stream are safe, calls that may overlap in time (different
 * streams) race on it. */
btc_status btc_gemv_static(void* stream, const btc_shape* s, const uint32_t* packed,
                           const uint32_t* codebook, const float* alpha, const float* mu,
                           const void* x, int32_t batch, void* y, btc_dtype y_dtype);

/* Test and measurement hook: btc_gemv through ONE chosen engine, so that each engine can be checked against the
 * oracle and timed against the others on any shape (the engines are different ways of carrying out the same
 * blockwise sum of appendix "Binary Codebook LUT-GEMM").  Same arguments, results and errors as btc_gemv;
 * BTC_ENGINE_AUTO is btc_gemv itself; an engine that does not cover the shape or batch size returns
 * BTC_ERR_UNSUPPORTED and enqueues nothing. */
enum {
  BTC_ENGINE_AUTO = 0,
  BTC_ENGINE_EXPAND = 1,    /* codebook expanded to +-1 pairs, activations in registers            */
  BTC_ENGINE_LUT = 2,       /* per-column tables of partial dot products (the paper's scheme)      */
  BTC_ENGINE_MFMA_ONE = 3,  /* fp16 matrix cores, one activation row, one kernel                   */
  BTC_ENGINE_MFMA = 4,      /* fp16 matrix cores, up to 16 activation rows, two kernels            */
  BTC_ENGINE_TILED = 5,     /* the prefill kernel on a few rows                                    */
  BTC_ENGINE_GENERIC = 6,   /* any chunk length and index width                                    */
  BTC_ENGINE_FP4 = 7,       /* 4-bit matrix cores: weights as E2M1, activations as E5M2 pieces     */
  BTC_ENGINE_CODE = 8       /* long vectors, large codebooks: the codebook itself in LDS           */
};
btc_status btc_gemv_engine(void* stream, const btc_shape* s, const uint32_t* packed,
                           const uint32_t* codebook, const float* alpha, const float* mu,
                           const void* x, int32_t batch, void* y, btc_dtype y_dtype,
                           void* workspace, size_t workspace_bytes, int32_t engine);

/* btc_gemv (one activation row) for `count` (1..4) matrices of the SAME shape applied to the SAME activation
 * row, e.g. the q, k, v or the gate, up projections of a decoder layer: y[m] = W_hat[m] . x.  packed, codebook,
 * alpha, mu, y are HOST arrays of `count` device pointers (read before the call returns), each as for btc_gemv;
 * x fp16 [in]; y[m] [out] of y_dtype (BTC_F16 or BTC_F32).  Where the engine on the 4-bit matrix cores covers
 * the setting (v 9 or 10, 7..10 index bits) this is ONE launch whose workgroups are shared out among the
 * matrices -- a decode product of this size is bound by its launch and prologue, not by its bytes -- and every
 * y[m] is bit-identical to that engine's result for matrix m alone; otherwise it is `count` btc_gemv calls
 * sharing the workspace (btc_workspace_bytes(s, 1, 0) bytes, rules as for btc_gemv).  Errors as btc_gemv. */
btc_status btc_gemv_multi(void* stream, const btc_shape* s, int32_t count, const uint32_t* const* packed,
                          const uint32_t* const* codebook, const float* const* alpha,
                          const float* const* mu, const void* x, void* const* y, btc_dtype y_dtype,
                          void* workspace, size_t workspace_bytes);

/* The same for matrices whose NUMBER OF ROWS differs (Section "Integration into Transformer Architecture":
 * the projections that read one activation row; with grouped-query attention q has more rows than k and v):
 * shapes is a HOST array of `count` shapes that agree in `in`, `v` and `K` (else BTC_ERR_SHAPE); y[m] has
 * shapes[m]->out elements.  In the one-launch case the compute units are shared out among the matrices in
 * proportion to their rows; results are bit-identical to btc_gemv_multi / btc_gemv on each matrix.  The
 * workspace must hold the largest btc_workspace_bytes(shapes[m], 1, 0).  Errors as btc_gemv_multi. */
btc_status btc_gemv_multi_shapes(void* stream, const btc_shape* const* shapes, int32_t count,
                                 const uint32_t* const* packed, const uint32_t* const* codebook,
                                 const float* const* alpha, const float* const* mu, const void* x,
                                 void* const* y, btc_dtype y_dtype, void* workspace, size_t workspace_bytes);

/* Prefill product for many activation rows; same definition as btc_gemv with
 *   X : [M][in] of x_dtype (BTC_BF16 or BTC_F16), M >= 1
 *   Y : [M][out] of y_dtype (BTC_F32, BTC_BF16 or BTC_F16)
 * The +-1 patterns are decoded into LDS tiles and contracted on the matrix
 * cores with fp32 accumulation; alpha and mu are applied in fp32 afterwards.
 * Needs btc_workspace_bytes(s, M, 1) bytes of workspace. */
btc_status btc_gemm(void* stream, const btc_shape* s, const uint32_t* packed,
                    const uint32_t* codebook, const float* alpha, const float* mu,
                    const void* X, btc_dtype x_dtype, int32_t M, void* Y, btc_dtype y_dtype,
                    void* workspace, size_t workspace_bytes);

/* Online activation transform in front of the layer (section "Learnable
 * Transformation": transformation pair T = D P, D = diag(sigma) a diagonal sign
 * matrix, P = P1 (x) P2 a Kronecker product; "Integration into Transformer
 * Architecture": X <- X T at inference, the weights hold T^-1):
 *   Y[m][j1*n2 + j2] = sum_{i1,i2} sigma[i] * X[m][i] * P1[i1][j1] * P2[i2][j2],  i = i1*n2 + i2
 *   X         : [M][n1*n2] of x_dtype (BTC_F16 or BTC_BF16), M >= 1
 *   sign_bits : uint32 [ceil(n1*n2 / 32)], bit (i & 31) of word (i >> 5) set => sigma[i] = +1,
 *               clear => -1 (the sign<->bit map of the codebook)
 *   P1, P2    : float [n1][n1], [n2][n2], row-major; n1 <= 128, n2 <= 256
 *   Y         : [M][n1*n2] of y_dtype (BTC_F16, BTC_BF16 or BTC_F32; round to nearest even)
 * All pointers are device memory owned by the caller, 16-byte aligned; X and Y
 * must not overlap.  fp32 accumulation in a fixed order (deterministic).  No
 * workspace.  Enqueues and returns.  Errors: BTC_ERR_NULL, _SHAPE (non-positive
 * sizes), _UNSUPPORTED (n1, n2 or a dtype outside the ranges above, X == Y),
 * _ALIGN, _HIP (launch failed). */
btc_status btc_transform(void* stream, const void* X, btc_dtype x_dtype, int32_t M, int32_t n1,
                         int32_t n2, const uint32_t* sign_bits, const float* P1, const float* P2,
                         void* Y, btc_dtype y_dtype);

/* The decode-time product behind the online activation transform, as one call (sections "Learnable
 * Transformation" and "Integration into Transformer Architecture": every compressed layer sees X T):
 *   y[i] = sum_k W_hat[i][k] * x'[k],   x' = fp16( x T ),  T as in btc_transform, n1 * n2 = in
 * i.e. btc_transform (one fp16 row in, fp16 out) followed by btc_gemv (batch 1), without the second launch
 * where the fused engine covers the setting.
 *
 * btc_transform_prepared_bytes / btc_transform_prepare: once per layer, the factors P1, P2 are split into
 * pairs of fp16 numbers and laid out as matrix-core operands in `prepared` (device memory owned by the
 * caller, 16-byte aligned, at least btc_transform_prepared_bytes(n1, n2) bytes; that size is 0 when nothing
 * uses prepared operands of these sizes: the fused kernel exists for 64 x 64 and 64 x 80, a matrix-core
 * kernel for the transform of one row also for 64 x 128, 86 x 128 and 108 x 128).  Entries of P1 and P2 must be at
 * most 65504 in magnitude.  Enqueues and returns.  Errors: BTC_ERR_NULL, _SHAPE, _UNSUPPORTED (factor
 * sizes), _WORKSPACE (prepared_bytes too small), _ALIGN, _HIP.
 *
 * btc_gemv_transformed: x fp16 [in]; y [out] of y_dtype (BTC_F16 or BTC_F32); sign_bits, P1, P2 as for
 * btc_transform; `prepared` from btc_transform_prepare for the same n1, n2, P1, P2, or NULL; xt_out: fp16
 * [in], receives x' for other consumers of the same transformed row (launched later on the stream), or NULL.
 * With `prepared`, v = 10 and 7..10 index bits the call is one kernel: every workgroup computes x' into LDS on
 * the matrix cores (fp32 accumulation; factors and intermediate carried as two fp16 parts, 2^-22 relative)
 * and needs no workspace.  Otherwise it runs the transform as a launch of its own (on the matrix cores where
 * prepared operands exist, else btc_transform; into xt_out, else into the head of the workspace) and btc_gemv:
 * then `workspace` must hold btc_gemv_transformed_workspace_bytes(s) bytes and follow the rules of btc_gemv's
 * workspace (zero-filled before first use).  x and xt_out must not overlap.  Errors: as btc_gemv and
 * btc_transform, _SHAPE also when n1 * n2 != in.
 *
 * btc_gemv_transformed_multi: the same for `count` (1..4) matrices of one shape that consume the same
 * transformed row (q, k, v; gate, up), pointer arrays as for btc_gemv_multi: one kernel where the fused
 * engine covers the setting, else the transform launch followed by btc_gemv_multi. */
size_t btc_transform_prepared_bytes(int32_t n1, int32_t n2);
btc_status btc_transform_prepare(void* stream, int32_t n1, int32_t n2, const float* P1, const float* P2,
                                 void* prepared, size_t prepared_bytes);
size_t btc_gemv_transformed_workspace_bytes(const btc_shape* s);
btc_status btc_gemv_transformed(void* stream, const btc_shape* s, const uint32_t* packed,
                                const uint32_t* codebook, const float* alpha, const float* mu, const void* x,
                                int32_t n1, int32_t n2, const uint32_t* sign_bits, const float* P1,
                                const float* P2, const void* prepared, void* xt_out, void* y,
                                btc_dtype y_dtype, void* workspace, size_t workspace_bytes);
btc_status btc_gemv_transformed_multi(void* stream, const btc_shape* s, int32_t count,
                                      const uint32_t* const* packed, const uint32_t* const* codebook,
                                      const float* const* alpha, const float* const* mu, const void* x,
                                      int32_t n1, int32_t n2, const uint32_t* sign_bits, const float* P1,
                                      const float* P2, const void* prepared, void* xt_out, void* const* y,
                                      btc_dtype y_dtype, void* workspace, size_t workspace_bytes);

/* E-step of the binary codebook clustering (section "Flash and Accurate Binary
 * Codebook", step "E-step Assignment": z_i = argmin_k ||b_i - c_k||^2, which for
 * +-1 vectors is 4 * POPCNT(b_i xor c_k); a vector identical to a centroid goes to
 * it).  Offline step that produces the index matrix btc_pack stores.
 *   vectors  : uint32 [N], bit t of entry i = element t of vector i (1 => +1), t < v;
 *              bits >= v are ignored
 *   codebook : uint32 [K] centroids in the same form, K 1..65536; v 1..32
 *   z        : int32 [N], index of the nearest centroid; among equally near ones
 *              (duplicates included) the lowest index
 *   dist2    : int32 [N] squared distance to it (4 * Hamming distance), or NULL
 * Device pointers owned by the caller, 16-byte aligned.  Integer arithmetic, exact.
 * Enqueues and returns.  Errors: BTC_ERR_NULL, _SHAPE (N <= 0), _UNSUPPORTED
 * (v or K out of range), _ALIGN, _HIP. */
btc_status btc_assign(void* stream, const uint32_t* vectors, int64_t N, int32_t v,
                      const uint32_t* codebook, int32_t K, int32_t* z, int32_t* dist2);

/* Host. Bytes of workspace btc_update needs: K * (v + 1) 32-bit counters and an
 * error flag.  0 for v or K out of range. */
size_t btc_update_workspace_bytes(int32_t v, int32_t K);

/* M-step of the binary codebook clustering (section "Flash and Accurate Binary
 * Codebook", step "M-step Centroid Update"; algorithm of appendix "Binary Codebook
 * Optimization"): for every cluster k with at least one member,
 *   codebook[k] element t = +1  iff  sum over the members of element t >= 0
 * (the sign of the mean, a zero mean giving +1); bits >= v of a new centroid are 0.
 * A cluster without members keeps its centroid.
 *   vectors  : uint32 [N] sign patterns (bit t = element t, 1 => +1; bits >= v ignored)
 *   z        : int32 [N] cluster of each vector, every entry in [0, K)
 *   codebook : uint32 [K], read and overwritten;  v 1..32, K 1..65536, N < 2^31
 *   workspace: btc_update_workspace_bytes(v, K) bytes, ZERO-FILLED before its first
 *              use; every call leaves it zero again
 * Device pointers owned by the caller, 16-byte aligned.  Integer arithmetic, exact,
 * independent of the order of the atomic additions.  This call WAITS for the stream
 * (like btc_pack): an entry of z outside [0, K) gives BTC_ERR_INDEX_RANGE and leaves
 * the codebook unchanged.  Other errors: BTC_ERR_NULL, _SHAPE (N <= 0),
 * _UNSUPPORTED, _WORKSPACE, _ALIGN, _HIP. */
btc_status btc_update(void* stream, const uint32_t* vectors, const int32_t* z, int64_t N,
                      int32_t v, uint32_t* codebook, int32_t K, void* workspace,
                      size_t workspace_bytes);

/* The layer on quantised activations (section "Activation Quantization on sub-bit LLMs": W0.8A8 and
 * W0.8A4; appendix hyper-parameters: min-max quantisation with a scale per channel, read here as one
 * (offset, step) pair per activation row -- a scale that varied along the contraction index could not be
 * taken out of the integer sum).  Three calls:
 *
 * btc_quantize_rows: for every row m of X,
 *     lo[m] = min_k X[m][k],  step[m] = (max_k X[m][k] - lo[m]) / (2^bits - 1)   (1 for a constant row)
 *     Q[m][k] = round-to-nearest-even((X[m][k] - lo[m]) / step[m]) clamped to [0, 2^bits - 1]
 *   every operation a single IEEE fp32 operation in the order written (X widened exactly), so that the
 *   integer codes are reproducible; X ~ lo + step * Q.
 *     X : [M][n] of x_dtype (BTC_F16 or BTC_BF16), finite values;  bits : 8 or 4;  n <= 65536
 *     Q : uint8 [M][n], one code per byte for both widths;  lo, step : float [M]
 *     qsum : float [M] or NULL: sum_k Q[m][k] (an exact integer)
 * btc_weight_rowsums: wsum[i] = sum_{k < in} W_hat[i][k] = alpha_i * (sum of the row's signs) + mu_i * in,
 *   a per-layer constant of the third call.  wsum : float [out].
 * btc_gemm_aq: Y[m][i] = sum_k W_hat[i][k] * (lo[m] + step[m] * Q[m][k])
 *                     = step[m] * (alpha_i * sum_k B_hat[i][k] Q[m][k] + mu_i * sum_k Q[m][k]) + lo[m] * wsum[i],
 *   any M >= 1 (decode and prefill).  The integer sums are exact (codes and signs are exact in the 16-bit
 *   operand formats, fp32 sums of integers below 2^24); alpha, mu, step, lo are applied in fp32.
 *     Y : [M][out] of y_dtype (BTC_F32, BTC_F16 or BTC_BF16)
 * workspace (second and third call): btc_aq_workspace_bytes(s, M) bytes (M = 1 for btc_weight_rowsums), any
 * contents, clobbered.  Device pointers owned by the caller, 16-byte aligned.  All three enqueue and return.
 * Errors: BTC_ERR_NULL, _SHAPE, _UNSUPPORTED (bits, dtypes, n or in above 65536), _ALIGN, _WORKSPACE, _HIP. */
btc_status btc_quantize_rows(void* stream, const void* X, btc_dtype x_dtype, int32_t M, int32_t n, int32_t bits,
                             uint8_t* Q, float* lo, float* step, float* qsum);
size_t btc_aq_workspace_bytes(const btc_shape* s, int32_t M);
btc_status btc_weight_rowsums(void* stream, const btc_shape* s, const uint32_t* packed, const uint32_t* codebook,
                              const float* alpha, const float* mu, float* wsum, void* workspace,
                              size_t workspace_bytes);
btc_status btc_gemm_aq(void* stream, const btc_shape* s, const uint32_t* packed, const uint32_t* codebook,
                       const float* alpha, const float* mu, const float* wsum, const uint8_t* Q, const float* lo,
                       const float* step, int32_t M, void* Y, btc_dtype y_dtype, void* workspace,
                       size_t workspace_bytes);

/* Decode-time product for the storage variant with several (alpha, mu) pairs per weight row (Table "Study of
 * Number of Split Points"; appendix hyper-parameters: 2 split points by default):
 *   W_hat[i][k] = alpha[i][g] * B_hat[i][k] + mu[i][g],   g = group[i][k] in [0, ngroups),  ngroups 1..4
 *   y[i] = sum_k W_hat[i][k] * x[k]
 *   alpha, mu : float [out][ngroups], row-major
 *   group_map : uint32 [out][ceil(2 in / 32)]: the group of weight k of row i in bits [2k, 2k+2) of row i's
 *               map, bit p of a row's map being bit (p & 31) of its word (p >> 5); values >= ngroups must not occur
 *   x : fp16 [in] (one activation row);  y : [out] of y_dtype (BTC_F16 or BTC_F32);  in <= 32768
 * packed and codebook as for btc_gemv.  fp32 sums in a fixed order.  No workspace.  Enqueues and returns.
 * Errors: BTC_ERR_NULL, _SHAPE, _UNSUPPORTED (ngroups, in, y_dtype), _ALIGN, _HIP. */
btc_status btc_gemv_groups(void* stream, const btc_shape* s, const uint32_t* packed, const uint32_t* codebook,
                           const float* alpha, const float* mu, const uint32_t* group_map, int32_t ngroups,
                           const void* x, void* y, btc_dtype y_dtype);

/* Host. Static string for a status code. */
const char* btc_status_str(btc_status st);

#ifdef __cplusplus
}
#endif
#endif /* BTC_H_ */
