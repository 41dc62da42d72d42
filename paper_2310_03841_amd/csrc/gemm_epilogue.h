// Epilogue shared by the GEMM kernels: store C, emit the stripe outputs, take the observed
// row / column sums of the M x N block from the accumulators (before rounding) and add them
// to cc_obs / rc_obs.  Paper: output checksum fused with the GEMM epilogue (Sec. IV-C memory
// paragraph, Sec. V "Optimizations" (2)).
//
// The kernels issue their MFMAs with the B fragment as first operand, so one 32x32 block of
// accumulators is laid out "row per lane": lane l holds row (l & 31) of the block and, in
// register i, column 8*(i>>2) + 4*(l>>5) + (i&3) -- four consecutive columns per register
// quad.  Consequences:
//   * C goes out through LDS: each lane packs four converted values into one LDS write, the
//     wave reads the staged rows back 16 bytes per lane and stores whole 256/512-byte row
//     segments to global memory.
//   * row sums are in-lane adds plus one exchange between the half-waves;
//   * column sums need a reduction over the 32 lanes (rows): partial sums are transposed
//     through LDS instead of a 5-step cross-lane butterfly per value.
// Every loop over accumulator registers is expanded at compile time (static_for): the
// accumulators must be addressed with constant indices to stay in registers.
//
// LDS use: each wave owns EPI_WAVE_BYTES at smem + wave * EPI_WAVE_BYTES, then the block-wide
// partial-sum arrays follow.  The caller must have passed a barrier after its last LDS read.
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

// bytes of wave-private LDS the epilogue needs for a wave tile that is TN columns wide
__host__ __device__ constexpr int epi_wave_bytes(int TN) { return 32 * (TN * 4 + 16); }
__host__ __device__ constexpr int epi_total_bytes(int BM, int BN)
{
    return 4 * epi_wave_bytes(BN / 2) + (2 * BM + 2 * BN) * 4 + 16;
}

template <bool IS_INT> __device__ __forceinline__ bool epi_mismatch(uint32_t obs, uint32_t pred, float tol)
{
    if (IS_INT) return obs != pred;                          // equality in Z/2^32
    const float d = fabsf(__uint_as_float(obs) - __uint_as_float(pred));
    return !(d <= tol);                                      // NaN and Inf always flag
}

// Read one accumulator element where it lives (an AGPR) at the point of use.  Without this the
// register allocator moves the whole accumulator set into VGPRs at the top of the epilogue and
// spills part of it.
__device__ __forceinline__ float acc_read(float v)
{
    float r;
    asm("v_accvgpr_read_b32 %0, %1" : "=v"(r) : "a"(v));
    return r;
}
__device__ __forceinline__ int acc_read(int v)
{
    int r;
    asm("v_accvgpr_read_b32 %0, %1" : "=v"(r) : "a"(v));
    return r;
}

// pack converted outputs
// Two fp32 values -> two storage-type values in one word, round to nearest even (the packed
// conversion instructions of gfx950).
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
template <int DT> __device__ __forceinline__ uint32_t pack2(float a, float b);
template <> __device__ __forceinline__ uint32_t pack2<DT_BF16>(float a, float b)
{
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
template <> __device__ __forceinline__ uint32_t pack2<DT_F16>(float a, float b)
{
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
}

template <int DT, int BM, int BN, bool PROT>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &g,
                                              typename Traits<DT>::accv_t (&acc)[BM / 64][BN / 64],
                                              uint8_t *smem, int m0, int n0, int bz, int tile_row_id)
{
    using T = Traits<DT>;
    typedef typename T::acc_t acc_t;
    constexpr int TM = BM / 2, TN = BN / 2;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int OS = T::OS;
    constexpr int WAVE_BYTES = epi_wave_bytes(TN);
    constexpr int CROW = TN * OS + 16;              // staged C row (bytes), padded
    constexpr int SROW = TN * 4 + 16;               // staged 32-bit row (bytes), padded
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform by construction
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int M = g.M, N = g.N;
    const int Mx = PROT ? M + NTERM : M;             // rows M .. Mx-1 are the A-side stripe

    uint8_t *wbuf = smem + wave * WAVE_BYTES;                              // wave-private staging
    acc_t *rs_part = reinterpret_cast<acc_t *>(smem + 4 * WAVE_BYTES);     // [2][BM] by wave column
    acc_t *cs_part = rs_part + 2 * BM;                                     // [2][BN] by wave row
    uint8_t *Cb = g.C + (long)bz * g.sC * OS;
    const bool inj_here = g.inj_b == bz && g.inj_row >= m0 && g.inj_row < m0 + BM &&
                          g.inj_col >= n0 && g.inj_col < n0 + BN;
    const int wr0 = m0 + wm * TM, wc0 = n0 + wn * TN;                      // first row / column of the wave tile
    // staged path: every column of the wave tile is a column of C; rows may run past M
    const bool staged = (wc0 + TN <= N) && !inj_here;

    auto wave_sync = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    static_for<0, MI>([&](auto mi_c) {
        constexpr int mi = decltype(mi_c)::value;
        const int br = wr0 + mi * 32;                                      // first row of this 32-row group
        const int gr = br + l32;                                           // this lane's row
        acc_t rowsum = T::zero();
        if (staged) {
            const int rows_in = M - br < 0 ? 0 : (M - br > 32 ? 32 : M - br);   // rows of C in the group
            if (rows_in > 0) {
                // ---- stage 32 rows of converted C in LDS, four columns per write
                static_for<0, NI>([&](auto ni_c) {
                    constexpr int ni = decltype(ni_c)::value;
                    static_for<0, 4>([&](auto q_c) {
                        constexpr int q = decltype(q_c)::value;
                        const acc_t v0 = acc_read(acc[mi][ni][4 * q]), v1 = acc_read(acc[mi][ni][4 * q + 1]),
                                    v2 = acc_read(acc[mi][ni][4 * q + 2]), v3 = acc_read(acc[mi][ni][4 * q + 3]);
                        if (PROT) rowsum = add_t(rowsum, add_t(add_t(v0, v1), add_t(v2, v3)));
                        uint8_t *d = wbuf + l32 * CROW + (ni * 32 + 8 * q + 4 * lh) * OS;
                        if constexpr (DT == DT_I8) {
                            *reinterpret_cast<i32x4 *>(d) = i32x4{(int)v0, (int)v1, (int)v2, (int)v3};
                        } else {
                            uint2 w;
                            w.x = pack2<DT>((float)v0, (float)v1);
                            w.y = pack2<DT>((float)v2, (float)v3);
                            *reinterpret_cast<uint2 *>(d) = w;
                        }
                    });
                    // keep the scheduler from hoisting every accumulator read to the top: that
                    // would need hundreds of live registers and spill
                    __builtin_amdgcn_sched_barrier(0);
                });
                wave_sync();
                // ---- read rows back, 16 bytes per lane, and store whole row segments
                constexpr int LPR = TN * OS / 16;                          // lanes per row
                constexpr int RPI = 64 / LPR;                              // rows per instruction
                // (all LDS reads first, then the stores: one LDS latency instead of one per row)
                constexpr int NIT = 32 / RPI;
                const int r0 = lane / LPR, cch = lane % LPR;
                i32x4 rowv[NIT];
#pragma unroll
                for (int it = 0; it < NIT; ++it)
                    rowv[it] = *reinterpret_cast<const i32x4 *>(wbuf + (it * RPI + r0) * CROW + cch * 16);
                uint8_t *crow = Cb + ((long)(br + r0) * g.ldc + wc0) * OS + cch * 16;
                const long cstep = (long)RPI * g.ldc * OS;
#pragma unroll
                for (int it = 0; it < NIT; ++it)
                    if (it * RPI + r0 < rows_in) *reinterpret_cast<i32x4 *>(crow + it * cstep) = rowv[it];
                wave_sync();
            }
            if (PROT && br < Mx && br + 32 > M) {
                // ---- the group holds rows of the A-side stripe: their accumulators are the
                // terms of (e^T A) B.  Stage the group as 32-bit words, emit those rows.
                static_for<0, NI>([&](auto ni_c) {
                    constexpr int ni = decltype(ni_c)::value;
                    static_for<0, 4>([&](auto q_c) {
                        constexpr int q = decltype(q_c)::value;
                        uint8_t *d = wbuf + l32 * SROW + (ni * 32 + 8 * q + 4 * lh) * 4;
                        *reinterpret_cast<i32x4 *>(d) =
                            i32x4{(int)as_word(acc_read(acc[mi][ni][4 * q])), (int)as_word(acc_read(acc[mi][ni][4 * q + 1])),
                                  (int)as_word(acc_read(acc[mi][ni][4 * q + 2])), (int)as_word(acc_read(acc[mi][ni][4 * q + 3]))};
                    });
                });
                wave_sync();
#pragma unroll
                for (int t = 0; t < NTERM; ++t) {
                    const int r = M + t - br;
                    if (r >= 0 && r < 32) {
                        for (int c0 = 2 * lane; c0 < TN; c0 += 128) {
                            const uint2 w = *reinterpret_cast<const uint2 *>(wbuf + r * SROW + c0 * 4);
                            uint32_t *dst = g.cc_part + ((long)bz * NTERM + t) * N + wc0 + c0;
                            publish_word(dst, w.x);          // read by the workgroup that compares this column
                            publish_word(dst + 1, w.y);
                        }
                    }
                }
                wave_sync();
            }
        } else if (br < Mx && wc0 < N) {
            // ---- ragged columns or armed flip: element by element
            static_for<0, NI>([&](auto ni_c) {
                constexpr int ni = decltype(ni_c)::value;
                static_for<0, 16>([&](auto i_c) {
                    constexpr int i = decltype(i_c)::value;
                    const int gc = wc0 + ni * 32 + 8 * (i >> 2) + 4 * lh + (i & 3);
                    acc_t v = acc_read(acc[mi][ni][i]);
                    if (inj_here && gr == g.inj_row && gc == g.inj_col)
                        v = from_word<acc_t>(as_word(v) ^ (1u << g.inj_bit));
                    if (gc < N) {
                        if (gr < M) {
                            T::store_c(Cb, (long)gr * g.ldc + gc, v);
                            if (PROT) rowsum = add_t(rowsum, v);
                        } else if (PROT && gr < Mx) {
                            publish_word(g.cc_part + ((long)bz * NTERM + (gr - M)) * N + gc, as_word(v));
                        }
                    }
                });
            });
        }
        if (PROT) {
            // row sums: the two half-waves hold different columns of the same rows
            const acc_t t = add_t(rowsum, __shfl_xor(rowsum, 32));
            if (lh == 0) rs_part[wn * BM + wm * TM + mi * 32 + l32] = t;
        }
    });

    if (PROT) {
        // ---- column sums: a second walk over the accumulators, one block column at a time (16
        // live partial sums instead of 16 * NI), each lane adding up its rows of the MI row
        // groups; the per-lane partials are transposed through LDS: staged as
        // S[l32][column of the wave tile] (fp32 / int32), then every lane adds up the 32 rows
        // of two columns.  Rows past M and the column where a flip is armed are handled here
        // too, so the sums cover exactly what was stored.
        static_for<0, NI>([&](auto ni_c) {
            constexpr int ni = decltype(ni_c)::value;
            acc_t cp[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) cp[i] = T::zero();
            static_for<0, MI>([&](auto mi_c) {
                constexpr int mi = decltype(mi_c)::value;
                const int br = wr0 + mi * 32;
                if (br + 32 <= M && !inj_here) {                 // whole group inside, no flip: plain adds
                    static_for<0, 16>([&](auto i_c) {
                        constexpr int i = decltype(i_c)::value;
                        cp[i] = add_t(cp[i], acc_read(acc[mi][ni][i]));
                    });
                    __builtin_amdgcn_sched_barrier(0);
                } else if (br < M) {
                    const int gr = br + l32;
                    static_for<0, 16>([&](auto i_c) {
                        constexpr int i = decltype(i_c)::value;
                        const int gc = wc0 + ni * 32 + 8 * (i >> 2) + 4 * lh + (i & 3);
                        acc_t v = acc_read(acc[mi][ni][i]);
                        if (inj_here && gr == g.inj_row && gc == g.inj_col)
                            v = from_word<acc_t>(as_word(v) ^ (1u << g.inj_bit));
                        if (gr < M) cp[i] = add_t(cp[i], v);
                    });
                }
            });
            static_for<0, 4>([&](auto q_c) {
                constexpr int q = decltype(q_c)::value;
                uint8_t *d = wbuf + l32 * SROW + (ni * 32 + 8 * q + 4 * lh) * 4;
                *reinterpret_cast<i32x4 *>(d) =
                    i32x4{(int)as_word(cp[4 * q]), (int)as_word(cp[4 * q + 1]),
                          (int)as_word(cp[4 * q + 2]), (int)as_word(cp[4 * q + 3])};
            });
        });
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        for (int c0 = 2 * lane; c0 < TN; c0 += 128) {
            acc_t s0 = T::zero(), s1 = T::zero();
#pragma unroll
            for (int r = 0; r < 32; ++r) {
                const uint2 w = *reinterpret_cast<const uint2 *>(wbuf + r * SROW + c0 * 4);
                s0 = add_t(s0, from_word<acc_t>(w.x));
                s1 = add_t(s1, from_word<acc_t>(w.y));
            }
            cs_part[wm * BN + wn * TN + c0] = s0;
            cs_part[wm * BN + wn * TN + c0 + 1] = s1;
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
        if (g.fuse_compare) {
            // ---- compare and flag without another launch (Sec. III-B.1 item (2)).  The workgroup
            // that completes a tile row compares that row's sums, the one that completes a tile
            // column recombines the stripe terms and compares that column's sums; the last
            // workgroup of the launch publishes counts and status.  Everything the comparing
            // workgroup reads from others was written with device-scope atomics (performed at
            // the coherence point); the barrier waits for this workgroup's outstanding ones
            // before it takes its tickets.
            static_assert(BM <= 256 && BN <= 256, "one row / column per thread in the fused compare");
            int *flag_s = reinterpret_cast<int *>(cs_part + 2 * BN);       // [3] after the partial sums
            __syncthreads();
            if (tid == 0) {
                const unsigned tr = atomicAdd(g.row_ticket + (long)bz * g.tiles_m + tile_row_id, 1u);
                const unsigned tc = atomicAdd(g.col_ticket + (long)bz * g.tiles_n + n0 / BN, 1u);
                flag_s[0] = (tr == (unsigned)g.tiles_n - 1);
                flag_s[1] = (tc == (unsigned)g.tiles_m - 1);
            }
            __syncthreads();
            const bool last_row = flag_s[0], last_col = flag_s[1];
            const float tol = T::IS_INT ? 0.f : g.tau[bz];
            unsigned nr = 0, nc = 0;
            if (last_row) {
                bool f = false;
                for (int t = tid; t < BM; t += 256) {
                    const int gr = m0 + t;
                    if (gr < M) {
                        const uint32_t obs = atomic_read_word(g.rc_obs + (long)bz * M + gr);
                        f = epi_mismatch<T::IS_INT>(obs, g.rc_pred[(long)bz * M + gr], tol);
                        g.row_flag[(long)bz * M + gr] = f ? 1 : 0;
                    }
                }
                nr = __syncthreads_count(f);
            }
            if (last_col) {
                bool f = false;
                for (int t = tid; t < BN; t += 256) {
                    const int gc = n0 + t;
                    if (gc < N) {
                        uint32_t term[NTERM];
#pragma unroll
                        for (int q = 0; q < NTERM; ++q)
                            term[q] = atomic_read_word(g.cc_part + ((long)bz * NTERM + q) * N + gc);
                        uint32_t pred;
                        if (T::IS_INT) {
                            pred = 0;
#pragma unroll
                            for (int q = 0; q < NTERM; ++q) pred += term[q] << (8 * q);
                        } else {
                            float v = 0.f;
#pragma unroll
                            for (int q = NTERM - 1; q >= 0; --q)          // small terms first
                                v += __uint_as_float(term[q]) * g.w_a[(long)bz * NTERM + q];
                            pred = __float_as_uint(v);
                        }
                        g.cc_pred[(long)bz * N + gc] = pred;
                        const uint32_t obs = atomic_read_word(g.cc_obs + (long)bz * N + gc);
                        f = epi_mismatch<T::IS_INT>(obs, pred, tol);
                        g.col_flag[(long)bz * N + gc] = f ? 1 : 0;
                    }
                }
                nc = __syncthreads_count(f);
            }
            if (tid == 0) {
                if (nr) atomicAdd(g.fin + 1, nr);
                if (nc) atomicAdd(g.fin + 2, nc);
            }
            __syncthreads();                         // orders this workgroup's count atomics before its final ticket
            if (tid == 0) {
                const unsigned total = gridDim.x * gridDim.z;
                if (atomicAdd(g.fin, 1u) == total - 1) {
                    const uint32_t r = atomicExch(g.fin + 1, 0u), c = atomicExch(g.fin + 2, 0u);
                    atomicExch(g.fin, 0u);
                    const uint32_t st = (r == 0 && c == 0) ? 0u : ((r == 0 || c == 0) ? 2u : 1u);
                    g.counts[0] = r;
                    g.counts[1] = c;
                    g.counts[2] = st;
                    g.counts[3] = 0u;
                    g.counts[4] = st;
                }
            }
        }
    }
}

}  // namespace abft
