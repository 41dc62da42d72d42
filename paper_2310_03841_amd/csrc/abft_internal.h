// Internal declarations shared by the kernels and the C-ABI shim of libabft.
// Nothing here is part of the public interface (see include/abft.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace abft {

// Number of rows of the encoded checksum stripe appended to A.
// int8: four signed base-256 digits of the int32 sum; bf16/f16: three terms of
// the fp32 sum (high, middle, low) and one zero row.
constexpr int NTERM = 4;
// K is processed in slabs of 128 bytes per operand row.
constexpr int SLAB_BYTES = 128;
// Tiles abft_correct recomputes are CT x CT, aligned.
constexpr int CT = 32;
// Most tiles one abft_correct call repairs.
constexpr int MAX_FIX_TILES = 256;
// Copies of the encode accumulators (spreads same-cache-line atomics).
constexpr int ENC_ACC_COPIES = 8;
// Most flagged rows (columns) per batch item that localisation lists.
constexpr int MAX_LIST = 64;

enum { DT_I8 = 0, DT_BF16 = 1, DT_F16 = 2 };

__host__ __device__ inline int elem_size(int dt) { return dt == DT_I8 ? 1 : 2; }
__host__ __device__ inline int out_size(int dt) { return dt == DT_I8 ? 4 : 2; }

// Device workspace of a context, carved for the shape of the current call.
// All arrays are [batch][len]; checksum values are int32 (ring Z/2^32) for
// DT_I8 and float otherwise, so every element is one 32-bit word.
struct Workspace {
    // encode
    uint32_t *a_acc, *b_acc;        // [ENC_ACC_COPIES][batch][K] atomic accumulators, self-cleaning
    long acc_stride;                // words between accumulator copies
    uint32_t *a_sum, *b_sum;        // [batch][K]   final a = e^T A, b = B e
    uint32_t *max_acc;              // [batch][2]   atomic max of |A|, |B| (float bits), self-cleaning
    float    *maxabs;               // [batch][2]
    float    *tau;                  // [batch]
    float    *w_a;                  // [batch][NTERM] weights that recombine the stripe terms (fp)
    uint8_t  *stripe_a;             // [batch][NTERM][Kp] terms of a in the operand type
    uint32_t *enc_ticket;           // [batch]
    // predicted
    uint32_t *cc_part;              // [batch][NTERM][N] raw stripe outputs of the GEMM
    uint32_t *cc_pred, *rc_pred;    // [batch][N] recombined, [batch][M] from the A pass
    uint32_t *s_pred;               // [batch]
    // observed
    uint32_t *cc_obs, *rc_obs;      // epilogue sums (atomics)
    uint32_t *row_ticket, *col_ticket, *fin;   // fused compare: per tile row / tile column / launch
    size_t zero_words;              // words from cc_obs on that must be zero before the GEMM
    uint32_t *cc_vobs, *rc_vobs;    // re-summed from stored C
    // correction
    int32_t  *fix_tiles;            // [MAX_FIX_TILES][3] (batch, tile row, tile col)
    uint32_t *fix_count;            // [4]: 0 tiles, 1 overflow flag, 2 ticket, 3 spare
    uint32_t *cmp_ticket;           // [1]
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
    float tau_override;
};

// ---- launchers (each enqueues on `st`, returns the hipError_t of the launch) ----
hipError_t launch_zero(uint32_t *p, size_t nwords, hipStream_t st);
hipError_t launch_encode_b(int dt, const void *B, const Shape &s, const Workspace &w, hipStream_t st);
hipError_t launch_encode_a(int dt, const void *A, const Shape &s, const Workspace &w, float tau_override,
                           uint32_t *zero_ptr, size_t zero_words, hipStream_t st);
int encode_a_max_k(int dt);
// v != nullptr: flags and counts are produced by the last-arriving workgroups of the GEMM itself
hipError_t launch_gemm(int dt, bool protect, const void *A, const void *B, void *C, const Shape &s,
                       const Workspace &w, const InjectArm &arm, const Verdict *v, hipStream_t st);
hipError_t launch_compare(int dt, const Shape &s, const Workspace &w, const Verdict &v, bool after_fix,
                          hipStream_t st);
hipError_t launch_verify_sums(int dt, const void *C, const Shape &s, const Workspace &w, hipStream_t st);
hipError_t launch_correct(int dt, const void *A, const void *B, void *C, const Shape &s,
                          const Workspace &w, const Verdict &v, hipStream_t st);
hipError_t launch_flip(void *C, int dt, const Shape &s, long batch_idx, long row, long col, int bit,
                       hipStream_t st);
void gemm_tile_shape(int dt, const Shape &s, int *tm, int *tn);

}  // namespace abft
