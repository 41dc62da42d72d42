// Epilogue shared by the GEMM kernels: store C, emit the stripe outputs, take the observed
// row / column sums of the M x N block from the accumulators (before rounding) and add them
// to cc_obs / rc_obs.  Paper: output checksum fused with the GEMM epilogue (Sec. IV-C memory
// paragraph, Sec. V "Optimizations" (2)).
//
// Accumulator layout of one 32x32 MFMA block: lane l holds column (l & 31) and, in register i,
// row 8*(i>>2) + 4*(l>>5) + (i&3).  Column sums are therefore in-lane adds plus one exchange
// between the two half-waves; row sums need a reduction over the 32 lanes of a half-wave.
//
// Every loop over accumulator registers is expanded at compile time (static_for): the
// accumulators must be addressed with constant indices to stay in registers.
#pragma once
#include <type_traits>

#include "abft_device.h"
#include "gemm_args.h"

namespace abft {

template <int I, int N, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

template <int DT, int BM, int BN, bool PROT>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &g,
                                              typename Traits<DT>::accv_t (&acc)[BM / 64][BN / 64],
                                              uint8_t *smem, int m0, int n0, int bz)
{
    using T = Traits<DT>;
    typedef typename T::acc_t acc_t;
    constexpr int TM = BM / 2, TN = BN / 2;
    constexpr int MI = TM / 32, NI = TN / 32;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform by construction
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int M = g.M, N = g.N;
    const int Mx = PROT ? M + NTERM : M;
    const int Nx = PROT ? N + NTERM : N;

    acc_t *rs_part = reinterpret_cast<acc_t *>(smem);          // [2][BM] by wave column
    acc_t *cs_part = rs_part + 2 * BM;                         // [2][BN] by wave row
    uint8_t *Cb = g.C + (long)bz * g.sC * T::OS;
    const bool inj_here = g.inj_b == bz && g.inj_row >= m0 && g.inj_row < m0 + BM &&
                          g.inj_col >= n0 && g.inj_col < n0 + BN;

    acc_t colsum[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) colsum[ni] = T::zero();

    static_for<0, MI>([&](auto mi_c) {
        constexpr int mi = decltype(mi_c)::value;
        acc_t rowsum[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) rowsum[i] = T::zero();
        const int br = m0 + wm * TM + mi * 32;                 // first row of this block
        static_for<0, NI>([&](auto ni_c) {
            constexpr int ni = decltype(ni_c)::value;
            const int bc = n0 + wn * TN + ni * 32;             // first column of this block
            const int gc = bc + l32;
            // wave-uniform classification of the 32x32 block
            const bool inside = (br + 32 <= M) && (bc + 32 <= N) && !inj_here;
            if (inside) {
                static_for<0, 16>([&](auto i_c) {
                    constexpr int i = decltype(i_c)::value;
                    const int gr = br + 8 * (i >> 2) + 4 * lh + (i & 3);
                    const acc_t v = acc[mi][ni][i];
                    T::store_c(Cb, (long)gr * g.ldc + gc, v);
                    if (PROT) {
                        colsum[ni] = add_t(colsum[ni], v);
                        rowsum[i] = add_t(rowsum[i], v);
                    }
                });
            } else if (br < Mx && bc < Nx) {
                static_for<0, 16>([&](auto i_c) {
                    constexpr int i = decltype(i_c)::value;
                    const int gr = br + 8 * (i >> 2) + 4 * lh + (i & 3);
                    acc_t v = acc[mi][ni][i];
                    if (inj_here && gr == g.inj_row && gc == g.inj_col)
                        v = from_word<acc_t>(as_word(v) ^ (1u << g.inj_bit));
                    if (gr < M && gc < N) {
                        T::store_c(Cb, (long)gr * g.ldc + gc, v);
                        if (PROT) {
                            colsum[ni] = add_t(colsum[ni], v);
                            rowsum[i] = add_t(rowsum[i], v);
                        }
                    } else if (PROT) {
                        if (gr >= M && gr < Mx) {
                            if (gc < N)
                                g.cc_part[((long)bz * NTERM + (gr - M)) * N + gc] = as_word(v);
                            else if (gc < Nx)
                                g.s_part[(long)bz * NTERM * NTERM + (gr - M) * NTERM + (gc - N)] = as_word(v);
                        } else if (gr < M && gc >= N && gc < Nx) {
                            g.rc_part[((long)bz * NTERM + (gc - N)) * M + gr] = as_word(v);
                        }
                    }
                });
            }
        });
        if (PROT) {
            // row sums: reduce over the 32 lanes that hold one row's columns
            static_for<0, 16>([&](auto i_c) {
                constexpr int i = decltype(i_c)::value;
                acc_t t = half_wave_sum(rowsum[i]);
                if (l32 == 0) rs_part[wn * BM + wm * TM + mi * 32 + 8 * (i >> 2) + 4 * lh + (i & 3)] = t;
            });
        }
    });
    if (PROT) {
        // column sums: the two half-waves hold different rows of the same columns
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            acc_t t = add_t(colsum[ni], __shfl_xor(colsum[ni], 32));
            if (lh == 0) cs_part[wm * BN + wn * TN + ni * 32 + l32] = t;
        }
        __syncthreads();
        for (int t = tid; t < BM + BN; t += 256) {
            if (t < BM) {
                int gr = m0 + t;
                if (gr < M) atomic_add_word(g.rc_obs + (long)bz * M + gr, add_t(rs_part[t], rs_part[BM + t]));
            } else {
                int gc = n0 + (t - BM);
                if (gc < N)
                    atomic_add_word(g.cc_obs + (long)bz * N + gc, add_t(cs_part[t - BM], cs_part[BN + t - BM]));
            }
        }
    }
}

}  // namespace abft
