/*
 * libabft -- checksum-protected GEMM for AMD MI355X (gfx950).
 *
 * For C = A * B the library computes, next to C, the column checksum
 * cc = (e^T A) B (length N) and the row checksum rc = A (B e) (length M),
 * compares them with the sums e^T C and C e of the produced output, flags the
 * rows and columns that disagree and repairs flagged elements by recomputing
 * the tile that holds them.
 *
 * Where the operations are defined in the paper (ALBERTA, arXiv 2310.03841):
 *   checksums of a GEMM layer ............ Sec. III-B.1, paragraph "Checksums"
 *   equality check for fixed point,
 *   tolerance check for floating point ... Sec. III-B.1, item (2) and "Eps Generation"
 *   integer overflow of the sums ......... Sec. III-B.1, item (1)
 *   weight checksum computed offline ..... Sec. III-B.1, "Checksums", remark (2)
 *   output checksum in the GEMM epilogue . Sec. IV-C (memory-overhead paragraph), Sec. V "Optimizations" (2)
 *   correction by replay ................. Sec. III-B.3
 *   single-bit-flip fault model .......... Sec. II-A "Formulation to Quantify Resilience", Sec. III-A
 * The row/column-vector form (instead of the paper's single scalar per sample)
 * is the classic ABFT scheme the paper cites as its origin (Sec. I, Sec. II-B);
 * the paper's scalar is the sum of either vector.
 *
 * Conventions
 *   - All matrix pointers are DEVICE pointers.  Matrices are row-major.
 *   - A is M x K with leading dimension lda (elements).
 *   - B is given as N x K (transB = 1: a Linear layer's weight, or K of Q K^T)
 *     or as K x N (transB = 0: V of attn V); ldb is the leading dimension of
 *     the stored array.
 *   - C is M x N with leading dimension ldc.  ABFT_I8: A, B int8, C int32.
 *     ABFT_BF16 / ABFT_F16: A, B, C in that type, fp32 accumulation, C rounded
 *     to nearest-even from the fp32 accumulator.
 *   - batch > 1: item b uses A + b*strideA etc. (strides in elements); every
 *     item has its own checksums and flags.
 *   - Base pointers, leading dimensions and batch strides must be multiples of
 *     16 bytes (else ABFT_EALIGN).  The buffers must hold rows*ld elements per
 *     item: the library may read (never use) the pad between K and lda.
 *   - The caller owns A, B, C, the flag / count buffers and the stream.  The
 *     context owns its workspace (checksum vectors, tile lists).
 *   - abft_gemm / abft_verify / abft_correct / abft_correct_checksum / abft_inject /
 *     abft_encode_b / abft_discrepancy only enqueue work on `stream` (a hipStream_t
 *     passed as void*): they allocate nothing, copy nothing to the host and never
 *     synchronise.  Results are valid once the stream has reached that point.
 *     They may be captured into a HIP graph (after one eager call of the same kind, which sets
 *     kernel attributes): calls enqueued under capture clear what they accumulate into themselves,
 *     so a replay does not depend on what ran before it; every buffer named at capture is used
 *     by the replays.
 *   - One context must be used from one stream (and one host thread) at a time; different
 *     contexts share nothing and may be used concurrently.
 *   - Return value: ABFT_OK or a negative error code.  A detected fault is NOT
 *     an error: it is reported through the flag vectors and counts.
 */
#ifndef ABFT_H
#define ABFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct abft_ctx abft_ctx;

typedef enum { ABFT_I8 = 0, ABFT_BF16 = 1, ABFT_F16 = 2 } abft_dtype;

/* mode = one base value, optionally OR-ed with flag bits */
enum {
    ABFT_OFF            = 0,    /* plain GEMM: same kernel with every checksum path compiled out */
    ABFT_DETECT         = 1,    /* encode, predicted + observed checksums, compare, flags */
    ABFT_DETECT_CORRECT = 2,    /* DETECT, then the steps of abft_correct */
    ABFT_MODE_MASK      = 0xF,
    ABFT_STORED_SUMS    = 0x20, /* floating point: the GEMM epilogue also sums the values of C as
                                   they are stored (after rounding); abft_verify / abft_correct then
                                   flag, besides |stored sums - prediction| > tau, any row or column
                                   whose re-summed stored C differs from those sums by more than
                                   1e-2 tau (only the order of fp32 summation separates the two, so a
                                   flip in stored C shows far below tau).  Ignored for ABFT_I8, where
                                   the stored values are the accumulators, and not kept with
                                   ABFT_DETECT_CORRECT (a correction replaces summed values). */
    ABFT_B_CHECKSUM_CACHED = 0x10, /* reuse the encoding of B left in the context by abft_encode_b
                                     (or by the previous abft_gemm with the same B and shape):
                                     the paper's offline weight checksum */
    ABFT_A_CHECKSUM_GIVEN = 0x40   /* a = e^T A (and max|A|) come from the caller (abft_supply_a): the
                                      checksum generated while A was produced (Sec. V "Optimizations"
                                      (2)), e.g. the stored-side column sums ABFT_WS_CC_STO of the
                                      protected GEMM whose output this A is.  The call then forms only
                                      the row prediction from A, and a corruption of A between its
                                      producer and this call shows in the column check */
};

enum {
    ABFT_OK         =  0,
    ABFT_EINVAL     = -1,   /* null pointer, unknown dtype/mode, index out of range */
    ABFT_EALIGN     = -2,   /* pointer, leading dimension or stride not a multiple of 16 bytes */
    ABFT_ESHAPE     = -3,   /* non-positive size, ld < row length, or K beyond what the protected
                               GEMM covers (K > 4096; int8 additionally needs K * 2^14 < 2^31) */
    ABFT_EWORKSPACE = -4,   /* shape exceeds what the context was created for */
    ABFT_EHIP       = -5,   /* a HIP runtime call failed (see abft_last_hip_error) */
    ABFT_ESTATE     = -6    /* call needs state that is not there (e.g. cached B encoding) */
};

/* status values written to counts[2] */
enum {
    ABFT_CLEAN            = 0,
    ABFT_LOCALISED        = 1,  /* flags on both sides: candidates = flagged rows x flagged cols */
    ABFT_CHECKSUM_SUSPECT = 2,  /* flags on one side only: not explainable by a corrupted element of C */
    ABFT_TOO_MANY         = 3   /* more flagged tiles than abft_correct repairs; replay the GEMM */
};

typedef struct {
    int64_t M, N, K;
    int64_t batch;                    /* >= 1 */
    int64_t lda, ldb, ldc;            /* elements */
    int64_t strideA, strideB, strideC;/* elements between batch items (ignored if batch == 1) */
    int32_t transB;                   /* 1: B stored N x K;  0: B stored K x N */
    int32_t reserved;
} abft_shape;

typedef struct {
    int64_t max_rows;   /* largest batch*M over all calls */
    int64_t max_cols;   /* largest batch*N */
    int64_t max_depth;  /* largest batch*(K rounded up to 128) */
    int64_t max_batch;
    int32_t device;     /* HIP device ordinal */
    int32_t reserved;
} abft_config;

/* Caller-provided DEVICE buffers that receive the verdict of a call. */
typedef struct {
    uint8_t  *row_flag;   /* [batch*M], 1 = row checksum mismatch */
    uint8_t  *col_flag;   /* [batch*N], 1 = column checksum mismatch */
    uint32_t *counts;     /* [8]: 0 = number of flagged rows, 1 = flagged columns, 2 = status,
                                  3 = tiles recomputed by the last correction,
                                  4 = status before that correction, 5..7 reserved */
    float     tau;        /* floating point only: > 0 overrides the tolerance
                             1e-3 * K * max|A| * max|B| (per batch item); 0 = use that default */
    float     tau_cols;   /* floating point only: > 0 is the tolerance of the column check alone (the
                             row check keeps tau or the default): thresholds calibrated separately
                             for the two checks (Sec. III-B.1 "Eps Generation"); 0 = same as rows */
} abft_result;

/* Workspace vectors that tests and reports may read back (device pointers into the context). */
typedef enum {
    ABFT_WS_A_SUM   = 0,  /* a = e^T A   [batch][K]   int32 / float */
    ABFT_WS_B_SUM   = 1,  /* b = B e     [batch][K] */
    ABFT_WS_CC_PRED = 2,  /* (e^T A) B   [batch][N] */
    ABFT_WS_RC_PRED = 3,  /* A (B e)     [batch][M] */
    ABFT_WS_CC_OBS  = 4,  /* e^T C from the GEMM epilogue (accumulators, before rounding) [batch][N] */
    ABFT_WS_RC_OBS  = 5,  /* C e   from the GEMM epilogue [batch][M] */
    ABFT_WS_CC_VOBS = 6,  /* e^T C re-summed from stored C by abft_verify [batch][N] */
    ABFT_WS_RC_VOBS = 7,  /* C e   re-summed from stored C by abft_verify [batch][M] */
    ABFT_WS_TAU     = 8,  /* tolerance in use [batch] float (floating point only) */
    ABFT_WS_S_PRED  = 9,  /* scalar a.b [batch] (the paper's own scalar check value) */
    ABFT_WS_MAXABS  = 10, /* max|A|, max|B| [batch][2] float (floating point only) */
    ABFT_WS_CC_STO  = 11, /* e^T C of the values as stored, from the GEMM epilogue (ABFT_STORED_SUMS) [batch][N] */
    ABFT_WS_RC_STO  = 12, /* C e   of the values as stored [batch][M] */
    ABFT_WS_C_MAX   = 13  /* max|C as stored| [batch] float, formed with the stored-side sums (what a
                             consumer of this C needs as its max|A|) */
} abft_ws_id;

/* where a flip lands */
enum { ABFT_INJECT_STORED_C = 0, ABFT_INJECT_ACCUMULATOR = 1, ABFT_INJECT_OPERAND_A = 2, ABFT_INJECT_OPERAND_B = 3 };

/* Allocates the context and its device workspace on cfg->device (the only call that allocates). */
int abft_create(abft_ctx **out, const abft_config *cfg);
int abft_destroy(abft_ctx *ctx);

/* Offline weight checksum (Sec. III-B.1 "Checksums", remark (2)): encodes B once; later
 * abft_gemm calls with ABFT_B_CHECKSUM_CACHED and the same shape skip that step. */
int abft_encode_b(abft_ctx *ctx, const void *B, abft_dtype dtype, const abft_shape *s, void *stream);

/* The protected GEMM (Sec. III-B.1 "Checksums"; epilogue fusion of Sec. V "Optimizations" (2)).
 * Enqueues: the pass over B that gives b = B e and max|B| (skipped with
 * ABFT_B_CHECKSUM_CACHED); the GEMM, which besides C produces, from the operand slabs of A it
 * holds on chip, a = e^T A, the row prediction A b and max|A|, and from its accumulators
 * (before rounding) the observed sums e^T C and C e; the finish kernel, which forms the
 * column prediction a B from one read of B, compares both pairs (equality for ABFT_I8,
 * |difference| <= tau otherwise; NaN or Inf always flag) and writes flags, counts and status.
 * A and B must stay unchanged until the finish kernel has run.
 * A batch of at least 64 small problems (per-head attention products: N <= 640, M <= 1024, a row
 * of K at most 640 bytes, operands of one item fitting the local memory of a compute unit; with
 * ABFT_STORED_SUMS only up to N = 256) is one kernel instead: one workgroup per batch item forms b, a, both
 * predictions and both observed sums from on-chip operands and compares them itself.
 * mode ABFT_OFF ignores `r` (may be NULL).  Flags and counts are overwritten. */
int abft_gemm(abft_ctx *ctx, const void *A, const void *B, void *C, abft_dtype dtype, int mode,
              const abft_shape *s, const abft_result *r, void *stream);

/* The protected GEMM of a layer with a bias: C = A B + bias, the bias vector (DEVICE, N entries:
 * float for ABFT_BF16 / ABFT_F16, int32 for ABFT_I8; shared by all batch items) added to every row
 * of the product before rounding.  The checked quantity is adjusted accordingly (Sec. III-B.1
 * "Checksums": the product of the input-side checksums is adjusted by the layer bias): the column
 * prediction gains M bias[j], the row prediction sum_j bias[j], the scalar M sum_j bias[j]; the
 * observed sums are taken from the biased values.  Everything else as abft_gemm (batches of small
 * problems take the tiled kernels here).  abft_verify / abft_correct after this call use the same
 * bias: the vector must stay valid and unchanged until they have run. */
int abft_gemm_bias(abft_ctx *ctx, const void *A, const void *B, const void *bias, void *C,
                   abft_dtype dtype, int mode, const abft_shape *s, const abft_result *r, void *stream);

/* abft_gemm for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments (without a context), same
 * kernels, same results as abft_gemm; the workspace (checksum vectors, partial sums, tickets) is
 * a fixed array of about 3 MB inside the library's device image instead of the pools of a
 * context, so the call allocates nothing, on the device or through any library.  Each GPU holds
 * its own copy of that array from the moment the library is loaded until the process ends; the
 * call uses the copy of the current device.  Limits (ABFT_EWORKSPACE beyond them):
 * batch * M <= ABFT_STATIC_MAX_ROWS, batch * N <= ABFT_STATIC_MAX_COLS,
 * batch * (K rounded up to 128) <= ABFT_STATIC_MAX_DEPTH, batch <= ABFT_STATIC_MAX_BATCH.
 * All calls on one GPU share the array and the state in it (the cached encoding of B, the
 * predictions): calls that overlap in time on one GPU, from different streams or threads, race.
 * Use abft_create contexts where that is needed.  abft_verify / abft_correct have no such
 * variant: use ABFT_DETECT_CORRECT here, or a context. */
#define ABFT_STATIC_MAX_ROWS  65536
#define ABFT_STATIC_MAX_COLS  16384
#define ABFT_STATIC_MAX_DEPTH 16384
#define ABFT_STATIC_MAX_BATCH 64
int abft_gemm_static(const void *A, const void *B, void *C, abft_dtype dtype, int mode,
                     const abft_shape *s, const abft_result *r, void *stream);

/* Producer-side input checksum for the next abft_gemm / abft_gemm_bias on this context called with
 * ABFT_A_CHECKSUM_GIVEN (Sec. V "Optimizations" (2): the checksum is generated while the tensor is
 * produced, so the consumer does not form it again).  a: DEVICE, [batch][K] words (float for
 * ABFT_BF16 / ABFT_F16, int32 in Z/2^32 for ABFT_I8), the column sums of the consumer's A;
 * amax: DEVICE, [batch] float, max|A| (may be NULL: then the call must bring its tolerance in
 * abft_result.tau; ignored for ABFT_I8).  Both must stay valid until that call's kernels have run;
 * the pointers are consumed by that call.  Where A is the stored output of a protected GEMM run
 * with ABFT_STORED_SUMS on the same shape family (consumer M, K = producer M, N), a and amax are
 * that call's ABFT_WS_CC_STO and ABFT_WS_C_MAX.  ABFT_WS_A_SUM is not filled by such a call. */
int abft_supply_a(abft_ctx *ctx, const void *a, const void *amax);

/* Pipelining several independent GEMMs (Sec. IV-C: the check must stay a small fraction of the
 * layer's time).  A protected call is a chain of dependent kernels of which only the GEMM fills
 * the chip; the pass over B and the finish kernel are bound by latency.  Two or three streams,
 * each with a context of its own, hide them: while one stream's GEMM runs, the other streams' small
 * kernels run beside it.  For that the GEMMs must not start together (they would share the chip, end
 * together and leave it idle during both finish kernels, and that state persists).  `event` is a
 * caller-owned hipEvent_t that every following abft_gemm / abft_gemm_bias of this context (any
 * mode, also ABFT_OFF) records on its stream right behind its GEMM kernel, before the finish
 * kernel; the caller lets the other stream wait for it (hipStreamWaitEvent) before that stream's
 * first call, after which the streams stay half a step apart by themselves.  NULL stops the
 * recording.  Nothing is recorded while a call is being captured into a graph, nor by protected
 * calls of a context once one of its calls has been captured.  The event must stay
 * valid until it is replaced or the context destroyed; the library never waits on it. */
int abft_gemm_done_event(abft_ctx *ctx, void *event);

/* Re-sums the stored C and compares with the predictions the last abft_gemm of this shape left
 * in the context (Sec. III-B.1: sum of layer activations vs. checksum product).  Overwrites
 * flags and counts.  Floating point: the stored values are rounded, and the rounding of a row of
 * N (a column of M) of them grows like sqrt(N) (sqrt(M)) while the default tolerance grows with K;
 * where N or M is several times K, clean rows or columns can exceed it (the comparison inside
 * abft_gemm, on the accumulators, is not affected).  A tolerance of the caller's in r->tau
 * (abft_discrepancy gives the statistics to fit it to) or ABFT_STORED_SUMS is the remedy. */
int abft_verify(abft_ctx *ctx, const void *C, abft_dtype dtype, const abft_shape *s,
                const abft_result *r, void *stream);

/* Replay at tile granularity (Sec. III-B.3): recomputes every 32x32 tile of C that holds a
 * (flagged row, flagged column) pair from A and B (same MFMA and k order as abft_gemm, so the
 * repaired elements are bit-identical to an undisturbed run), then checks again and rewrites
 * flags and counts (counts[3] = tiles recomputed, counts[4] = status before).  The second check:
 * when the context holds the sums of this stored C (the last call on it was abft_verify,
 * abft_correct or abft_correct_checksum, and C has not been written since), only the rows and the
 * columns of the recomputed tiles are summed again; otherwise the whole stored C is, as
 * abft_verify does.  At most 256 tiles per call; beyond that status = ABFT_TOO_MANY and the
 * caller replays the GEMM.  A and B must be unchanged since abft_gemm. */
int abft_correct(abft_ctx *ctx, const void *A, const void *B, void *C, abft_dtype dtype,
                 const abft_shape *s, const abft_result *r, void *stream);

/* Checksum-only correction (the inline correction of the classic scheme the paper starts from,
 * Sec. II-B; the paper itself replays, Sec. III-B.3).  ABFT_I8 only (ABFT_EINVAL otherwise: a
 * rounded floating-point sum cannot restore the stored bits).  Uses the flags in `r` and the
 * re-summed stored C of the last abft_verify of this shape (ABFT_ESTATE without one; the flags
 * must be the ones that call wrote).  For every batch item with exactly one flagged row i and
 * one flagged column j whose discrepancies d = re-summed - predicted agree modulo 2^32:
 * C[i][j] -= d, the item's flags are cleared and its re-summed vectors updated.  Every other
 * pattern (several flags, one-sided flags, disagreeing discrepancies) is left untouched for
 * abft_correct.  Reads neither A nor B and does not re-read C.  counts[0..2] = flags and status
 * that remain, counts[3] = elements repaired, counts[4] = status before. */
int abft_correct_checksum(abft_ctx *ctx, void *C, abft_dtype dtype, const abft_shape *s,
                          const abft_result *r, void *stream);

/* Eps generation (Sec. III-B.1 "Eps Generation": the floating-point threshold of a layer is read
 * off the distribution of its checksum discrepancy over fault-free runs, at a chosen
 * confidence).  Writes, for every batch item of the last protected abft_gemm of this shape,
 * statistics of d = observed - predicted: stats[b][0..3] = sum d, sum d^2, max|d|, count over
 * the M rows, stats[b][4..7] the same over the N columns (device floats).  source
 * ABFT_DISC_FUSED: observed = the epilogue's sums of the accumulators; ABFT_DISC_STORED:
 * observed = the re-sum of stored C by the last abft_verify (ABFT_ESTATE without one).  The caller
 * pools these over runs and sets abft_result.tau, e.g. |mean| + z * std.  Floating point only
 * (ABFT_EINVAL for ABFT_I8). */
enum { ABFT_DISC_FUSED = 0, ABFT_DISC_STORED = 1 };
int abft_discrepancy(abft_ctx *ctx, abft_dtype dtype, const abft_shape *s, int source, float *stats,
                     void *stream);

/* Test hook for the single-bit-flip fault model.  ABFT_INJECT_STORED_C inverts bit `bit`
 * (0..31 for int32 C, 0..15 for bf16/f16 C) of C[batch_idx][row][col] on the stream.
 * ABFT_INJECT_ACCUMULATOR arms a one-shot flip of bit 0..31 of the int32/fp32 accumulator of
 * that element, applied inside the next abft_gemm before its epilogue (C may be NULL).
 * ABFT_INJECT_OPERAND_A / _B (the input and weight sites of the same fault model): `C` is the
 * operand's device pointer; (row, col) index the array as stored (A: M x K; B: N x K with
 * transB, else K x N); bit 0..7 for ABFT_I8, 0..15 otherwise.  What the checks see of such a flip
 * depends on when the checksums were taken: a flip before abft_gemm is part of the operands the
 * call encodes (consistent, hence silent); a weight flipped after abft_encode_b and used with
 * ABFT_B_CHECKSUM_CACHED shows as row flags in every row i with A[i,k] != 0. */
int abft_inject(abft_ctx *ctx, void *C, abft_dtype dtype, const abft_shape *s, int64_t batch_idx,
                int64_t row, int64_t col, int bit, int where, void *stream);

/* Device pointer and element count of a workspace vector for the given shape (layout [batch][len]). */
int abft_workspace(abft_ctx *ctx, int which, const abft_shape *s, void **ptr, int64_t *count);

/* Tile the GEMM kernel uses for this problem (rows, cols of C per workgroup; M, N where a
 * workgroup takes a whole batch item). */
int abft_tile_shape(abft_dtype dtype, const abft_shape *s, int *tile_m, int *tile_n);

/* Kernel timing for reports (not a hot call: creates HIP events).  Between begin and end every
 * abft_gemm records events on the caller's stream around its kernels; up to max_calls calls are
 * kept.  abft_profile_end waits for the recorded events and returns average milliseconds per call:
 * ms[0] pass over B (or the clearing kernel that replaces it), ms[1] GEMM kernel, ms[2] finish
 * kernel, ms[3] first event to last.  (Calls that are a single kernel report it as ms[1].) */
int abft_profile_begin(abft_ctx *ctx, int max_calls);
int abft_profile_end(abft_ctx *ctx, double ms[4], int *calls);

/* Report helper (not a hot call: allocates, creates events, waits): runs, on the current device
 * and its default stream, a kernel that issues nothing but the matrix instructions of `dtype` in
 * the GEMM kernel's register shape (one wave per SIMD, sixteen 32 x 32 accumulators) for about
 * `seconds` (at most 2), and returns the rate it sustained in 1e12 operations per second and the
 * shader clock it ran at.  A GEMM kernel's rate divided by this says how well its loop feeds the
 * matrix pipe, apart from the clock the chip grants under that load. */
int abft_mfma_peak(abft_dtype dtype, double seconds, double *tera_ops, double *clock_mhz);

const char *abft_strerror(int code);
/* hipError_t value of the last failing HIP call on this context (0 if none). */
int abft_last_hip_error(const abft_ctx *ctx);
int abft_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ABFT_H */
