// Kernel arguments shared by the GEMM kernels of libabft.
#pragma once
#include <stdint.h>

namespace abft {

struct GemmArgs {
    const uint8_t *A, *B;
    uint8_t *C;
    int M, N, K;
    long lda, ldb, ldc, sA, sB, sC;               // elements
    int tiles_m, tiles_n;
    int n_big, tiles_m_big, tiles_m_small;        // fast path: 256-row tiles and 128-row tiles
    int n_small, batch;                           // fast path: 128-row tiles per batch item; batch items
    int inj_b, inj_row, inj_col, inj_bit;         // armed accumulator flip (inj_b < 0: none)
    // protected launches: all of these are accumulated with atomics and start at zero
    uint32_t *cc_obs, *rc_obs;                    // observed sums of C        [batch][N], [batch][M]
    uint32_t *rc_pred;                            // A (B e)                    [batch][M]
    uint32_t *a_sum;                              // e^T A                      [batch][K]
    uint32_t *a_max;                              // max|A| as float bits       [batch]
    uint32_t *cc_sto, *rc_sto;                    // sums of C as stored (after rounding), or null
    uint32_t *c_max;                              // max|C as stored| as float bits [batch] (with cc_sto)
    int a_given;                                  // a = e^T A and max|A| come from the caller: the pass over A's
                                                  // slabs forms the row dots only, nothing is added to a_sum / a_max
    const uint32_t *bias;                         // layer bias [N] (float / int32 words) or null
    const uint32_t *b_sum;                        // B e, complete before the launch [batch][K]
    int mul24_ok;                                 // int8: |b| < 2^23, 24-bit multiplies are exact
};

// Fast path (gemm_fast.hip): B stored N x K, K a whole number of 128-byte slabs.
bool gemm_fast_eligible(int dt, int M, int N, int K, bool transB, long lda, long ldb);
hipError_t launch_gemm_fast(int dt, bool protect, GemmArgs &g, int batch, hipStream_t st);
void gemm_fast_tile(int *tm, int *tn);

}  // namespace abft
