/*
 * llmint8 -- LLM.int8() mixed-precision decomposition matmul for one MI355X
 * (gfx950), arXiv 2208.07339.
 *
 * Problem statement (Section 2.1, above Eq. 6; Section 3): hidden states
 * X_f16 [s x h] (s tokens, h features), weights W_f16 [h x o], threshold alpha;
 * result C_f16 [s x o] approximating X W by Eq. 8:
 *
 *     C = sum_{k in O} X_f16[:,k] W_f16[k,:]  +  S * sum_{k not in O} X_i8[:,k] W_i8[k,:]
 *
 * with O the feature columns of X holding any |x| >= alpha (Section 3.2),
 * X_i8 / W_i8 the absmax codes (Section 2.1) with one constant per row of X
 * and one per column of W (vector-wise quantization, Section 3.1, Eq. 7), and
 * S the outer product of those constants over 127^2.
 *
 * Conventions
 *   - Every matrix/vector pointer is a DEVICE pointer owned by the caller.
 *     fp16 data is IEEE binary16, passed as (const) void*.  X, W, Out are
 *     dense row-major.  Inputs must be finite; with NaN/Inf the results are
 *     unspecified (no fault).
 *   - "Constants" c_x, c_w are stored as the absolute maximum itself (an fp16
 *     value); the paper's multiplier is 127 / absmax.
 *   - Xq and Wq are PRIVATE tiled layouts (see llmint8_xq_bytes /
 *     llmint8_wq_bytes); llmint8_export_rows / llmint8_export_weight turn
 *     them into plain row-major int8 matrices.
 *   - stream is a hipStream_t (NULL = the default stream).  Every call only
 *     enqueues kernels on it: no host synchronisation, no allocation.  The
 *     library may be called from several threads.  Its only process-wide
 *     state: a per-device set-up done once under a lock (kernel attributes of
 *     every kernel variant, the device's compute-unit count, the address of
 *     the static scratch of llmint8_linear_static), by llmint8_init or by the
 *     first call that needs it; and the two test hooks llmint8_debug_* (atomic
 *     integers that every thread's later calls see).  Calls that share a
 *     workspace must be ordered by stream.  A call may be recorded into a HIP
 *     graph by stream capture and replayed; call llmint8_init (or any
 *     llmint8_matmul / llmint8_linear*) on the device once before capturing.
 *   - Return value: LLMINT8_OK or an error code below; nothing is enqueued
 *     when an argument error is returned.  Conditions only visible on the
 *     device (|O| > cap) set bit 0 of the device status word and clamp.
 *   - Speed, not results, depends on a few properties of the arguments: the
 *     fastest kernels of llmint8_matmul / llmint8_linear* need o % 8 == 0,
 *     16-byte aligned Out, c_x, c_w, X_o and W_f16, at most 32 outlier
 *     columns found (whatever cap is) and no accumulator export; anything
 *     else runs a guarded variant of the same kernels.
 */
#ifndef LLMINT8_H
#define LLMINT8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    LLMINT8_OK = 0,
    LLMINT8_INVALID_ARG = 1, /* null pointer, non-positive dimension, cap < 1, unknown granularity */
    LLMINT8_SHAPE = 2,       /* h > LLMINT8_MAX_H, or a size beyond 2^31 elements per row block */
    LLMINT8_WORKSPACE = 3,   /* workspace smaller than llmint8_workspace_bytes() */
    LLMINT8_HIP = 4,         /* a kernel launch failed (hipGetLastError) */
    LLMINT8_STATIC_LIMIT = 5 /* llmint8_linear_static: the sizes need more than LLMINT8_STATIC_SCRATCH_BYTES */
};

/* Largest feature dimension whose int32 accumulator cannot overflow:
 * h * 127^2 <= 2^31 - 1 (Section 2.1: outputs are accumulated as int32). */
#define LLMINT8_MAX_H 133144

typedef void *llmint8_stream_t;

const char *llmint8_status_string(int status);
/* Text of the HIP error behind the calling thread's most recent LLMINT8_HIP return. */
const char *llmint8_last_hip_error(void);

/* Per-device set-up for the CURRENT device (hipSetDevice), done once: kernel attributes of every
 * kernel variant and the address of the static scratch.  Optional (the first call that needs it does the
 * same), thread-safe, cheap when repeated.  Call it outside stream capture. */
int llmint8_init(void);

/* Leading dimension (in fp16 elements) of the gathered-outlier matrix Xo for a
 * given capacity: cap rounded up to a multiple of 16. */
int llmint8_opad(int cap);

/* Bytes of the private int8 buffers.  Wq: ceil(o/32) x ceil(h/128)*4 tiles of
 * 1 KiB; Xq: ceil(s/32) x ceil(h/128)*4 tiles.  A tile holds 32 rows (output
 * columns of W, or tokens of X) by 32 consecutive features; padding is zero. */
size_t llmint8_wq_bytes(int h, int o);
size_t llmint8_xq_bytes(int s, int h);

/* Bytes of scratch any of the calls below may need for these sizes. */
size_t llmint8_workspace_bytes(int s, int h, int o, int cap);

/* Section 3.1 / Section 2.1, done once per weight (the weights are turned into
 * int8 when they are loaded, before any X is seen): c_w[j] = max_k |W[k][j]| over all h rows,
 * W_i8[k][j] = round-half-even(127 W[k][j] / c_w[j]) (0 where c_w[j] = 0).
 *   W_f16  in   [h x o] fp16
 *   Wq     out  llmint8_wq_bytes(h, o) bytes, private layout
 *   cw_f16 out  [o] fp16                                                     */
int llmint8_quantize_weight(const void *W_f16, int h, int o, int8_t *Wq, void *cw_f16, void *ws,
                            size_t ws_bytes, llmint8_stream_t stream);

/* Section 3.2: O = { j : max_i |X[i][j]| >= alpha }, ascending.
 *   idx    out  [cap] int32, first min(|O|, cap) entries valid
 *   count  out  int32 = min(|O|, cap)
 *   status out  int32, bit 0 set iff |O| > cap (may be NULL)                 */
int llmint8_find_outliers(const void *X_f16, int s, int h, float alpha, int32_t *idx, int cap,
                          int32_t *count, int32_t *status, void *ws, size_t ws_bytes,
                          llmint8_stream_t stream);

/* Section 3.1 applied to the non-outlier part of X (Eq. 8 sums the int8 product
 * over k not in O): c_x[i] = max_{j not in O} |X[i][j]|,
 * X_i8[i][j] = round-half-even(127 X[i][j] / c_x[i]) for j not in O and 0 for
 * j in O; Xo[i][t] = X[i][O_t] for t < |O| and 0 for |O| <= t < opad.
 *   idx, count  in   as written by llmint8_find_outliers (device)
 *   Xq     out  llmint8_xq_bytes(s, h) bytes, private layout
 *   cx_f16 out  [s] fp16
 *   Xo_f16 out  [s x llmint8_opad(cap)] fp16                                 */
int llmint8_quantize_rows(const void *X_f16, int s, int h, const int32_t *idx, const int32_t *count,
                          int cap, int8_t *Xq, void *cx_f16, void *Xo_f16, llmint8_stream_t stream);

/* Variant that keeps no 16-bit weights (Section 3.2 counts about 0.1% extra memory for the
 * decomposition): the rows O of W are rebuilt from the codes by inverting the absmax quantization,
 * Wo[t][j] = fp16( W_i8[O_t][j] * c_w[j] / 127 ), rounded once to nearest even; rows t >= |O| are 0.
 *   Wo_f16 out  [llmint8_opad(cap) x o] fp16                                  */
int llmint8_dequantize_rows(const int8_t *Wq, const void *cw_f16, int h, int o, const int32_t *idx,
                            const int32_t *count, int cap, void *Wo_f16, llmint8_stream_t stream);

/* Eq. 7 + Eq. 8: C_i32 = X_i8 W_i8 (int32 accumulation),
 * Out = fp16( C_i32 * c_x (x) c_w / 127^2 + Xo W_f16[O,:] ), the outlier product
 * accumulated in fp32.  Token counts s <= 32 (up to 48 against a wide W) take a weight-streaming
 * kernel unless the shape of W suits the tiled kernel better.  The two kernels add the outlier product
 * up in fp32 in different orders: an output may differ in its last fp16 bit between them (not
 * between the tile shapes or work splits of one kernel).
 *   W_f16       in   the original weights; only rows O are read.  NULL: the rows rebuilt from
 *                    the codes (llmint8_dequantize_rows, done here into ws) take their place
 *   cx_f16      in   [s] fp16.  If the array starts on a 16-byte boundary it is read in aligned
 *                    16-byte pieces, the one that holds c_x[s-1] included: when s is not a multiple
 *                    of 8, up to 14 bytes behind the array (never beyond that aligned piece, so
 *                    never in another page) are read and ignored
 *   Out_f16     out  [s x o] fp16
 *   C_i32_debug out  NULL, or [s x o] int32 receiving the raw accumulators   */
int llmint8_matmul(const int8_t *Xq, const void *cx_f16, const void *Xo_f16, const int32_t *idx,
                   const int32_t *count, int cap, const int8_t *Wq, const void *cw_f16,
                   const void *W_f16, int s, int h, int o, void *Out_f16, int32_t *C_i32_debug,
                   void *ws, size_t ws_bytes, llmint8_stream_t stream);

/* The per-call sequence find_outliers -> quantize_rows -> matmul on one stream (W_f16 may be NULL
 * as for llmint8_matmul): the same outputs as the three calls, bit for bit, from fewer kernels
 * (two for the whole pre-pass when s <= 32, the rebuilt rows of W included).
 * Xq, cx_f16, Xo_f16, idx, count, status are caller-provided scratch/outputs
 * of the sizes given above.                                                   */
int llmint8_linear(const void *X_f16, int s, int h, float alpha, const int8_t *Wq, const void *cw_f16,
                   const void *W_f16, int o, int32_t *idx, int cap, int32_t *count, int32_t *status,
                   int8_t *Xq, void *cx_f16, void *Xo_f16, void *Out_f16, void *ws, size_t ws_bytes,
                   llmint8_stream_t stream);

/* llmint8_linear for callers that cannot allocate and have no workspace to hand over (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the scratch is a static
 * device array inside the library, LLMINT8_STATIC_SCRATCH_BYTES per GPU that uses the library, held
 * until the process ends.  Same arguments as llmint8_linear without ws / ws_bytes, same kernels, same
 * results bit for bit.  Returns LLMINT8_STATIC_LIMIT, with nothing enqueued, when
 * llmint8_workspace_bytes(s, h, o, cap) exceeds LLMINT8_STATIC_SCRATCH_BYTES (every benchmark shape fits).
 * Calls no hipMalloc / hipFree or any allocating routine.  All calls on one GPU share that GPU's array:
 * calls that may overlap on one GPU (different streams, different threads) race on it and must be
 * ordered by the caller; nothing in it needs clearing between calls.  The first call on a device looks
 * the array's address up (hipGetSymbolAddress): make it, or llmint8_init, outside stream capture. */
#define LLMINT8_STATIC_SCRATCH_BYTES (16u << 20)
int llmint8_linear_static(const void *X_f16, int s, int h, float alpha, const int8_t *Wq, const void *cw_f16,
                          const void *W_f16, int o, int32_t *idx, int cap, int32_t *count, int32_t *status,
                          int8_t *Xq, void *cx_f16, void *Xo_f16, void *Out_f16, llmint8_stream_t stream);

/* Baselines of Table 1: the same calls with coarser absmax constants.
 *   LLMINT8_VECTORWISE  one constant per row of X and per column of W (Section 3.1; the calls above)
 *   LLMINT8_ROWWISE     one constant per row of X, ONE for all of W (Section 4.3: row-wise and
 *                       vector-wise treat the hidden states alike and differ on the weight side)
 *   LLMINT8_TENSORWISE  ONE constant for X and one for W (absmax quantization of Section 2.1)
 * A shared constant is written into every entry of cx_f16 / cw_f16, so Eq. 7 and Eq. 8 and therefore
 * llmint8_matmul are unchanged.  With alpha < inf the constants of X are taken over the non-outlier
 * columns only ("row-wise + decomposition" in Table 1); alpha = +inf switches the decomposition off,
 * and llmint8_linear* then skips the scan of X.  The weight side of the granularity is fixed by
 * llmint8_quantize_weight_granular; the per-call functions apply the hidden-state side.          */
enum { LLMINT8_VECTORWISE = 0, LLMINT8_ROWWISE = 1, LLMINT8_TENSORWISE = 2 };
int llmint8_quantize_weight_granular(const void *W_f16, int h, int o, int granularity, int8_t *Wq, void *cw_f16,
                                     void *ws, size_t ws_bytes, llmint8_stream_t stream);
int llmint8_quantize_rows_granular(const void *X_f16, int s, int h, const int32_t *idx, const int32_t *count,
                                   int cap, int granularity, int8_t *Xq, void *cx_f16, void *Xo_f16,
                                   llmint8_stream_t stream);
int llmint8_linear_granular(const void *X_f16, int s, int h, float alpha, int granularity, const int8_t *Wq,
                            const void *cw_f16, const void *W_f16, int o, int32_t *idx, int cap, int32_t *count,
                            int32_t *status, int8_t *Xq, void *cx_f16, void *Xo_f16, void *Out_f16, void *ws,
                            size_t ws_bytes, llmint8_stream_t stream);

/* Measurement support: llmint8_linear_granular that also records two caller-created hipEvent_t on the
 * stream, one between the pre-pass and the matmul kernel and one after it (either may be NULL).  */
int llmint8_linear_events(const void *X_f16, int s, int h, float alpha, int granularity, const int8_t *Wq,
                          const void *cw_f16, const void *W_f16, int o, int32_t *idx, int cap, int32_t *count, int32_t *status,
                          int8_t *Xq, void *cx_f16, void *Xo_f16, void *Out_f16, void *ws, size_t ws_bytes,
                          llmint8_stream_t stream, void *ev_before_matmul, void *ev_after_matmul);

/* Zeropoint variant (Section 2.1, Eq. 1-5; Table 1 "zeropoint vector-wise" and, with alpha < inf,
 * "Zeropoint LLM.int8()"): asymmetric quantization with one set of constants per row of X (over its
 * non-outlier columns) and per column of W, in place of absmax.  For a vector with lo = min, hi = max,
 * D = hi - lo:  nd = 254 / D exactly (Eq. 1);  u(x) = round-half-even(254 x / D) (Eq. 3);
 * zp = u(lo) + 127 (Eq. 2: the printed "X min" read as nd min; the 127 recentres the stored byte
 * into the signed range [-127, 127] the text names);  stored code = u(x) - zp.  A constant vector
 * (D = 0) gets codes 0 and zp 0 and counts as all zero.  Eq. 4: T[i][j] = sum over k not in O of
 * (A[i][k] + zp_x[i]) (B[k][j] + zp_w[j]), computed in the unrolled form of Eq. 5 (int8 MFMA product
 * plus three correction terms, added in double);  Out = fp16(T D_x[i] D_w[j] / 254^2 + Xo W_f16[O,:]).
 *
 * Constants travel as records of four int32 per vector (16-byte aligned arrays zc_x [s][4], zc_w [o][4]):
 *   word 0  fp16 bit patterns of lo (low half) and hi (high half), a zero as +0
 *   word 1  zp
 *   word 2  sum of the vector's codes (row sum of X_i8 / column sum of W_i8 over all h)
 *   word 3  0
 * Xq, Wq, Xo, idx, count, status, ws as in the calls above; W_f16 is required.                  */
int llmint8_zp_quantize_weight(const void *W_f16, int h, int o, int8_t *Wq, int32_t *zc_w, void *ws,
                               size_t ws_bytes, llmint8_stream_t stream);
int llmint8_zp_quantize_rows(const void *X_f16, int s, int h, const int32_t *idx, const int32_t *count, int cap,
                             int8_t *Xq, int32_t *zc_x, void *Xo_f16, llmint8_stream_t stream);
/* C_i32_debug receives the plain int8 product sum_k A[i][k] B[k][j] (the first term of Eq. 5). */
int llmint8_zp_matmul(const int8_t *Xq, const int32_t *zc_x, const void *Xo_f16, const int32_t *idx,
                      const int32_t *count, int cap, const int8_t *Wq, const int32_t *zc_w, const void *W_f16,
                      int s, int h, int o, void *Out_f16, int32_t *C_i32_debug, void *ws, size_t ws_bytes,
                      llmint8_stream_t stream);
/* find_outliers -> zp_quantize_rows -> zp_matmul on one stream; the same outputs as the three calls, bit
 * for bit (for s <= 32 from three kernels in all). */
int llmint8_zp_linear(const void *X_f16, int s, int h, float alpha, const int8_t *Wq, const int32_t *zc_w,
                      const void *W_f16, int o, int32_t *idx, int cap, int32_t *count, int32_t *status,
                      int8_t *Xq, int32_t *zc_x, void *Xo_f16, void *Out_f16, void *ws, size_t ws_bytes,
                      llmint8_stream_t stream);

/* Measurement support: the ceilings the roofline fractions are held against, measured on the box itself.
 * llmint8_probe_mfma: one workgroup per compute unit runs a register-only issue loop of the int8 MFMA
 *   in the shape of the prefill GEMM's main loop (Eq. 7: 4 x 4 accumulator tiles per wave, 64 MFMAs per
 *   iteration), its operands read once from the tiled int8 buffers A_tiles / B_tiles (llmint8_xq_bytes /
 *   llmint8_wq_bytes layouts, or a buffer of zeros; at least one 1 KiB tile each): no memory traffic in
 *   the loop, so its rate is what the matrix cores sustain on operands with those statistics.  *ops (host,
 *   may be NULL) receives the int8 operations the launch performs; time it with events on the stream.
 * llmint8_probe_read: a read-only stream over buf (bytes >= 1024, 16-byte aligned; whole KiB are read).
 * sink: 4 bytes of device memory (written with negligible probability, never read).          */
int llmint8_probe_mfma(const int8_t *A_tiles, size_t a_bytes, const int8_t *B_tiles, size_t b_bytes, int iters,
                       int32_t *sink, double *ops, llmint8_stream_t stream);
int llmint8_probe_read(const void *buf, size_t bytes, int32_t *sink, llmint8_stream_t stream);

/* Test/support: force the workgroup tile of the prefill GEMM (output columns x tokens):
 * 0 = 256 x 256, 1 = 192 x 256, 2 = 128 x 256, 3 = 128 x 128, 4 = 192 x 128, 5 = 192 x 64; -1 = choose
 * from the shape (default).
 * Process-wide; results do not depend on it.                                  */
#define LLMINT8_PREFILL_TILES 6
int llmint8_debug_prefill_tile(int cfg);
/* Test/support: the tile (0 .. LLMINT8_PREFILL_TILES - 1) the library chooses by itself for a product of
 * [s x h] by [h x o]; -1 for a dimension < 1.  Host arithmetic only: needs no GPU.             */
int llmint8_debug_prefill_tile_for(int s, int h, int o);

/* Test/support: force the work split of the decode kernel (column tiles per workgroup, k-tiles per
 * load batch): 1 = 1 x 8, 2 = 2 x 4, 3 = 2 x 8, 4 = 3 x 4, 5 = 1 x 4; 0 = no weight-streaming kernel at all
 * (every token count through the tiled kernel); -1 = not forced (1 x 8; 2 x 4 above 16 tokens when W has
 * enough column tiles to fill the chip that way; the tiled kernel where the shape of W suits it better).
 * Anything else is LLMINT8_INVALID_ARG.  Process-wide; results do not depend on the work split (0 moves
 * short X to the other kernel: see llmint8_matmul).                                */
#define LLMINT8_DECODE_SHAPES 5
int llmint8_debug_decode_shape(int cfg);

/* Test/support: private layouts -> plain row-major int8 ([h x o], [s x h]). */
int llmint8_export_weight(const int8_t *Wq, int h, int o, int8_t *W_i8_rowmajor, llmint8_stream_t stream);
int llmint8_export_rows(const int8_t *Xq, int s, int h, int8_t *X_i8_rowmajor, llmint8_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* LLMINT8_H */
