// Internal declarations shared by the kernels and the C-ABI shim of libabft.
// Nothing here is part of the public interface (see include/abft.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace abft {

// K is processed in slabs of 128 bytes per operand row.
constexpr int SLAB_BYTES = 128;
// Tiles abft_correct recomputes are CT x CT, aligned.
constexpr int CT = 32;
// Most tiles one abft_correct call repairs.
constexpr int MAX_FIX_TILES = 256;
// Tolerance of the stored-side comparison relative to tau: both sides are fp32 sums of the same
// rounded values, so only the order of summation separates them.
constexpr float STO_TOL_FACTOR = 1e-2f;
// Most flagged rows (columns) per batch item that localisation lists.
constexpr int MAX_LIST = 64;

enum { DT_I8 = 0, DT_BF16 = 1, DT_F16 = 2 };

__host__ __device__ inline int elem_size(int dt) { return dt == DT_I8 ? 1 : 2; }
__host__ __device__ inline int out_size(int dt) { return dt == DT_I8 ? 4 : 2; }

// Device workspace of a context, carved for the shape of the current call.
// All arrays are [batch][len]; checksum values are int32 (ring Z/2^32) for
// DT_I8 and float otherwise, so every element is one 32-bit word.
struct Workspace {
    // B pass: b = B e and max|B| are accumulated with atomics into one of two slots (the
    // context alternates; the finish kernel of a protected GEMM clears the slot not in use)
    uint32_t *b_sum;                // [batch][K]   slot in use
    uint32_t *b_max;                // [batch]      max|B| as float bits, same slot
    float    *maxabs;               // [batch][2]   max|A|, max|B|
    float    *tau;                  // [batch]
    // predicted
    uint32_t *cc_pred;              // [batch][N]   (e^T A) B, written by the finish kernel
    uint32_t *s_pred;               // [batch]
    // one region that must be zero before the protected GEMM, filled by its atomics:
    //   cc_obs [batch][N] | rc_obs [batch][M] | rc_pred [batch][M] | a_sum [batch][K] | a_max [batch]
    //   | cc_sto [batch][N] | rc_sto [batch][M] | c_max [batch]
    uint32_t *cc_obs, *rc_obs;      // observed sums of C (epilogue)
    uint32_t *rc_pred;              // A (B e), from the operand slabs of A in LDS
    uint32_t *a_sum;                // a = e^T A, from the same slabs
    uint32_t *a_max;                // max|A| (float bits)
    uint32_t *cc_sto, *rc_sto;      // sums of C as stored (floating point, on request)
    uint32_t *c_max;                // max|C as stored| (float bits) [batch], formed with them
    size_t zero_words;              // words from cc_obs on
    uint32_t *cc_vobs, *rc_vobs;    // re-summed from stored C
    // correction
    int32_t  *fix_tiles;            // [MAX_FIX_TILES][3] (batch, tile row, tile col)
    uint32_t *fix_count;            // [4]: 0 tiles, 1 overflow flag, 2 ticket, 3 spare
    uint32_t *cmp_ticket;           // [4] ticket and counts, then [64] first-level tickets of the finish kernel
    // not workspace, but travels with it: the layer bias of the current call (device, [N], float or
    // int32 words; null = none).  Added to every row of the product before rounding and sums.
    const uint32_t *bias;
    // likewise: a = e^T A [batch][K] and max|A| [batch] (float bits; may be null) supplied by the
    // caller for this call (null = formed by the GEMM from the slabs of A it holds)
    const uint32_t *a_given, *amax_given;
};

struct Shape {
    int M, N, K, batch, transB;
    long lda, ldb, ldc, sA, sB, sC;
    int Kp;                         // K rounded up to a whole slab (elements)
};

struct InjectArm { int batch, row, col, bit; };   // batch < 0: not armed

struct Verdict {                    // caller buffers
    uint8_t *row_flag, *col_flag;
    uint32_t *counts;
    float tau_override;             // > 0: tolerance of both checks instead of 1e-3 K max|A| max|B|
    float tau_override_cols;        // > 0: tolerance of the column check (the row check keeps the other)
};

// Raises the dynamic-LDS limit of a kernel, once per (kernel, device); contexts may be driven
// from several host threads, so the bookkeeping is behind a mutex.
hipError_t ensure_max_lds(const void *kernel, int bytes);
// Compute units of the current device (cached per device, thread-safe); 0 on error.
int device_cu_count(hipError_t *err);

// ---- launchers (each enqueues on `st`, returns the hipError_t of the launch) ----
hipError_t launch_zero(uint32_t *p, size_t nwords, hipStream_t st);
// zero_ptr / zero_words: a region every block of the pass helps to clear (may be null / 0)
hipError_t launch_encode_b(int dt, const void *B, const Shape &s, const Workspace &w, uint32_t *zero_ptr,
                           size_t zero_words, hipStream_t st);
// Largest K the protected path handles (the column sums of A's slabs are kept in LDS).
int protect_max_k(int dt);
// protect: A-side checksums and observed sums are produced by the kernel (atomics into the
// zeroed region of the workspace); launch_finish turns them into flags.
// stored_sums: also accumulate the row / column sums of the rounded values that are stored
hipError_t launch_gemm(int dt, bool protect, bool stored_sums, const void *A, const void *B, void *C,
                       const Shape &s, const Workspace &w, const InjectArm &arm, hipStream_t st);
// zero_ptr / zero_words: a region every block of the kernel helps to clear (may be null / 0)
hipError_t launch_finish(int dt, const void *B, const Shape &s, const Workspace &w, const Verdict &v,
                         uint32_t *zero_ptr, size_t zero_words, uint32_t *zero2_ptr, size_t zero2_words,
                         hipStream_t st);
// with_sto: a row / column also flags when the re-summed stored C differs from the stored-side
// sums of the GEMM by more than STO_TOL_FACTOR * tau
// zero_ptr / zero_words: a region every block of the kernel helps to clear (may be null / 0)
// gated: the kernel does nothing when the tile list of the correction before it is empty
hipError_t launch_compare(int dt, const Shape &s, const Workspace &w, const Verdict &v, bool after_fix,
                          bool with_sto, uint32_t *zero_ptr, size_t zero_words, hipStream_t st, bool gated = false);
hipError_t launch_verify_sums(int dt, const void *C, const Shape &s, const Workspace &w, hipStream_t st,
                              bool gated = false);
// stale_words: leading words of the re-summing region in use that must be cleared first;
// zero_ptr / zero_words: the other re-summing region, cleared by the final compare
// targeted: the re-summing region in use holds the sums of this C as it was before the call; only
// the rows and columns of the recomputed tiles are summed again, in place (stale_words, zero_ptr unused)
// skip_if_clean: when no tile was listed (the check before found nothing to recompute) the re-sum
// of stored C and the final compare do nothing: flags and counts stay as that check wrote them
// clear_list: the tile list's counters may be non-zero (the final compare of a correction leaves
// them at zero, so only after a call that failed half way)
hipError_t launch_correct(int dt, const void *A, const void *B, void *C, const Shape &s,
                          const Workspace &w, const Verdict &v, bool with_sto, bool clear_list, bool targeted,
                          size_t stale_words, uint32_t *zero_ptr, size_t zero_words, hipStream_t st,
                          bool skip_if_clean = false);
// integers: repairs a single flagged element per batch item from the checksums alone
hipError_t launch_arith_fix(void *C, const Shape &s, const Workspace &w, const Verdict &v, hipStream_t st);
// stored: the sums of the last re-sum of stored C instead of the epilogue's
hipError_t launch_discrepancy(const Shape &s, const Workspace &w, bool stored, float *out, hipStream_t st);
hipError_t launch_flip(void *C, int dt, const Shape &s, long batch_idx, long row, long col, int bit,
                       hipStream_t st);
// inverts one bit of the elem_bytes-wide element at element index idx of `base`
hipError_t launch_flip_at(void *base, long idx, int elem_bytes, int bit, hipStream_t st);
// Batches of small problems (attention heads): one workgroup per batch item, all checksums and
// the comparison inside the GEMM kernel (gemm_item.hip).  v may be null when protect is false.
bool gemm_item_eligible(int dt, const Shape &s, bool stored_sums);
hipError_t launch_gemm_item(int dt, bool protect, bool cached_b, bool stored_sums, const void *A, const void *B, void *C,
                            const Shape &s, const Workspace &w, const Verdict *v, const InjectArm &arm,
                            hipStream_t st);
void gemm_tile_shape(int dt, const Shape &s, int *tm, int *tn);
// report helper: `blocks` workgroups of four waves issue iters x 16 matrix instructions each;
// clk[2 b], clk[2 b + 1] = shader-clock and 100 MHz ticks workgroup b spent in its loop
hipError_t launch_mfma_peak(int dt, int blocks, int iters, unsigned long long *clk, uint32_t *sink, hipStream_t st);

}  // namespace abft
