// Kernel arguments shared by the GEMM kernels of libabft.
#pragma once
#include <stdint.h>

namespace abft {

struct GemmArgs {
    const uint8_t *A, *B;
    uint8_t *C;
    const uint8_t *SA;                            // A-side stripe [batch][NTERM][Kp] operand elements
    uint32_t *cc_part;                            // raw stripe outputs: terms of (e^T A) B, [batch][NTERM][N]
    uint32_t *cc_obs, *rc_obs;                    // observed sums (atomics)
    int M, N, K, Kp;
    long lda, ldb, ldc, sA, sB, sC;               // elements
    int tiles_m, tiles_n;
    int n_big, tiles_m_big, tiles_m_small;        // fast path: 256-row tiles first, then 128-row tiles
    int inj_b, inj_row, inj_col, inj_bit;         // armed accumulator flip (inj_b < 0: none)
    // compare fused into the tail of the GEMM (fuse_compare != 0)
    int fuse_compare;
    const uint32_t *rc_pred;                      // [batch][M] from the A pass
    uint32_t *cc_pred;                            // [batch][N] recombined here
    const float *w_a, *tau;
    uint8_t *row_flag, *col_flag;
    uint32_t *counts;
    uint32_t *row_ticket, *col_ticket, *fin;      // zeroed before the launch; fin[3]: ticket, rows, cols
};

// Fast path (gemm_fast.hip): B stored N x K, K a whole number of 128-byte slabs.
bool gemm_fast_eligible(int dt, int M, int N, int K, bool transB, long lda, long ldb);
hipError_t launch_gemm_fast(int dt, bool protect, GemmArgs &g, int batch, hipStream_t st);
void gemm_fast_tile(int *tm, int *tn);

}  // namespace abft
