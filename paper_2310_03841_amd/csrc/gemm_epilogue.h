// Epilogue shared by the GEMM kernels: store C, take the observed row / column sums of the
// M x N block from the accumulators (before rounding) and add them to cc_obs / rc_obs, and
// hand over what the pass over A's slabs collected (gemm_apass.h).  Paper: output checksum
// fused with the GEMM epilogue (Sec. IV-C memory paragraph, Sec. V "Optimizations" (2)).
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
// Two paths per group of 32 rows of a wave tile.  The common one (every row and column of the
// group inside C, no flip armed) works from registers as described.  The other one (edges of
// the problem, armed flip) stages the raw 32-bit accumulators in LDS and walks them with an
// ordinary loop, so that it costs little code: straight-line code that is rarely executed still
// has to be fetched past.
//
// LDS use: each wave owns EPI_WAVE_BYTES at smem + wave * EPI_WAVE_BYTES, then the block-wide
// partial-sum arrays follow.  The caller must have passed a barrier after its last LDS read.
#pragma once
#include <type_traits>

#include "abft_device.h"
#include "gemm_args.h"
#include "gemm_apass.h"

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
    return 4 * epi_wave_bytes(BN / 2) + (3 * BM + 2 * BN) * 4 + 16;
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

// The value an accumulator becomes in memory, back as a float (round to nearest even).
template <int DT> __device__ __forceinline__ float stored_value(float v)
{
    const uint32_t w = pack2<DT>(v, 0.f) & 0xFFFFu;
    if constexpr (DT == DT_BF16) return __uint_as_float(w << 16);
    else return f16_bits_to_f32(w);
}

// What a protected tile hands to the epilogue besides its accumulators.
template <int DT> struct EpiProt {
    APassState<DT> st;        // row dots and max|A| of the owned slabs
    const uint32_t *col_lds;  // column sums of the owned slabs, KE words each (LDS)
    int owned;                // number of owned slabs reduced: the j-th is slab slab0 + j * slab_step of K
    int slab0, slab_step;
    int col_copies;           // 1, or 4: one set of column sums per wave, col_stride words apart, to be added up
    int col_stride;
};

template <int DT, int BM, int BN, bool PROT, bool BIAS>
__device__ __forceinline__ void gemm_epilogue_impl(const GemmArgs &g,
                                              typename Traits<DT>::accv_t (&acc)[BM / 64][BN / 64],
                                              uint8_t *smem, int m0, int n0, int bz, const EpiProt<DT> &ep)
{
    using T = Traits<DT>;
    typedef typename T::acc_t acc_t;
    constexpr int TM = BM / 2, TN = BN / 2;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int OS = T::OS;
    constexpr int KE = SLAB_BYTES / T::ES;
    constexpr int CPL = TN / 64;                    // columns per lane when a wave walks a row
    constexpr int WAVE_BYTES = epi_wave_bytes(TN);
    constexpr int CROW = TN * OS + 16;              // staged C row (bytes), padded
    constexpr int SROW = TN * 4 + 16;               // staged 32-bit row (bytes), padded
    const int tid = tile_thread_index(), lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform by construction
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int M = g.M, N = g.N;

    uint8_t *wbuf = smem + wave * WAVE_BYTES;                              // wave-private staging
    acc_t *rs_part = reinterpret_cast<acc_t *>(smem + 4 * WAVE_BYTES);     // [2][BM] by wave column
    acc_t *cs_part = rs_part + 2 * BM;                                     // [2][BN] by wave row
    acc_t *rp = cs_part + 2 * BN;                                          // [BM] row dots of the A pass
    float *amax4 = reinterpret_cast<float *>(rp + BM);                     // [4]
    uint8_t *Cb = g.C + (long)bz * g.sC * OS;
    // layer bias of this tile's columns, staged once (zero beyond N); added to every accumulator
    // value on its way out, before the sums and before rounding
    constexpr bool has_bias = BIAS;
    acc_t *bias_lds = reinterpret_cast<acc_t *>(amax4 + 4);                // [BN]
    if (has_bias) {
        for (int t = tid; t < BN; t += 256) bias_lds[t] = n0 + t < N ? from_word<acc_t>(g.bias[n0 + t]) : T::zero();
        __syncthreads();
    }
    const bool inj_here = g.inj_b == bz && g.inj_row >= m0 && g.inj_row < m0 + BM &&
                          g.inj_col >= n0 && g.inj_col < n0 + BN;
    const int wr0 = m0 + wm * TM, wc0 = n0 + wn * TN;                      // first row / column of the wave tile
    const bool cols_full = (wc0 + TN <= N) && !inj_here;

    auto wave_sync = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    // column partials: of the groups that went the register way (block column ni, register i:
    // this lane's rows) and of the groups that were walked row by row (columns CPL*lane ..)
    acc_t cp[PROT ? NI : 1][16];
    acc_t colacc[CPL];
    // sums of the values as stored (after rounding), on request and for floating point only:
    // edge groups add to these while they walk their rows, register-path groups in a second
    // pass over the accumulators further down
    const bool sto = PROT && !T::IS_INT && g.cc_sto != nullptr;
    float colacc_s[CPL], rowsto[MI];
    float cmax_s = 0.f;                 // max|value as stored| seen by this lane (with the stored-side sums)
#pragma unroll
    for (int j = 0; j < CPL; ++j) colacc_s[j] = 0.f;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) rowsto[mi] = 0.f;
    bool reg_path[MI];
    if (PROT) {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) cp[ni][i] = T::zero();
#pragma unroll
        for (int j = 0; j < CPL; ++j) colacc[j] = T::zero();
    }

    static_for<0, MI>([&](auto mi_c) {
        constexpr int mi = decltype(mi_c)::value;
        const int br = wr0 + mi * 32;                                      // first row of this 32-row group
        reg_path[mi] = cols_full && br + 32 <= M;
        if (cols_full && br + 32 <= M) {
            // ---- register path: one read of every accumulator serves the sums and the store
            acc_t rowsum = T::zero();
            static_for<0, NI>([&](auto ni_c) {
                constexpr int ni = decltype(ni_c)::value;
                static_for<0, 4>([&](auto q_c) {
                    constexpr int q = decltype(q_c)::value;
                    acc_t v0 = acc_read(acc[mi][ni][4 * q]), v1 = acc_read(acc[mi][ni][4 * q + 1]),
                          v2 = acc_read(acc[mi][ni][4 * q + 2]), v3 = acc_read(acc[mi][ni][4 * q + 3]);
                    if (has_bias) {
                        const i32x4 bb = *reinterpret_cast<const i32x4 *>(bias_lds + wn * TN + ni * 32 + 8 * q + 4 * lh);
                        v0 = add_t(v0, from_word<acc_t>((uint32_t)bb[0])); v1 = add_t(v1, from_word<acc_t>((uint32_t)bb[1]));
                        v2 = add_t(v2, from_word<acc_t>((uint32_t)bb[2])); v3 = add_t(v3, from_word<acc_t>((uint32_t)bb[3]));
                    }
                    if (PROT) {
                        cp[PROT ? ni : 0][4 * q] = add_t(cp[PROT ? ni : 0][4 * q], v0);
                        cp[PROT ? ni : 0][4 * q + 1] = add_t(cp[PROT ? ni : 0][4 * q + 1], v1);
                        cp[PROT ? ni : 0][4 * q + 2] = add_t(cp[PROT ? ni : 0][4 * q + 2], v2);
                        cp[PROT ? ni : 0][4 * q + 3] = add_t(cp[PROT ? ni : 0][4 * q + 3], v3);
                        rowsum = add_t(rowsum, add_t(add_t(v0, v1), add_t(v2, v3)));
                    }
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
                __builtin_amdgcn_sched_barrier(0);      // keeps the accumulator reads from all moving to the top
            });
            if (PROT) {
                const acc_t t = add_xor32(rowsum);     // the half-waves hold different columns
                if (lh == 0) rs_part[wn * BM + wm * TM + mi * 32 + l32] = t;
            }
            wave_sync();
            // read rows back, 16 bytes per lane, and store whole row segments
            constexpr int LPR = TN * OS / 16;                              // lanes per row
            constexpr int RPI = 64 / LPR;                                  // rows per instruction
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
                __builtin_nontemporal_store(rowv[it], reinterpret_cast<i32x4 *>(crow + it * cstep));
            wave_sync();
        } else if (br < M && wc0 < N) {
            // ---- edge path: raw accumulators to LDS, then a plain loop over rows
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
            if (inj_here && g.inj_row >= br && g.inj_row < br + 32 && g.inj_col >= wc0 && g.inj_col < wc0 + TN) {
                // the armed flip: one bit of one accumulator, before rounding and before the sums
                if (lane == 0)
                    *reinterpret_cast<uint32_t *>(wbuf + (g.inj_row - br) * SROW + (g.inj_col - wc0) * 4) ^= (1u << g.inj_bit);
                wave_sync();
            }
            const int nrow = M - br < 32 ? M - br : 32;
            // (1) lane <-> CPL consecutive columns, walking the rows: store C, column sums
            for (int r = 0; r < nrow; ++r) {
#pragma unroll
                for (int j = 0; j < CPL; ++j) {
                    const int col = CPL * lane + j, gc = wc0 + col;
                    if (gc < N) {
                        acc_t v = from_word<acc_t>(*reinterpret_cast<const uint32_t *>(wbuf + r * SROW + col * 4));
                        if (has_bias) v = add_t(v, bias_lds[wn * TN + col]);
                        T::store_c(Cb, (long)(br + r) * g.ldc + gc, v);
                        if (PROT) colacc[j] = add_t(colacc[j], v);
                        if constexpr (PROT && !T::IS_INT) {
                            if (sto) {
                                const float sv = stored_value<DT>((float)v);
                                colacc_s[j] += sv;
                                cmax_s = fmaxf(cmax_s, fabsf(sv));
                            }
                        }
                    }
                }
            }
            // (2) lane <-> row, the half-waves split the columns, walking the columns (each lane
            // starts at a different one: no bank conflicts): row sums without cross-lane traffic.
            // Rows of the group past M get a value too; nobody reads it.
            if (PROT) {
                constexpr int HC = TN / 2;
                const int ncol = N - wc0 < TN ? N - wc0 : TN;
                acc_t rs = T::zero();
                float rs_s = 0.f;
                for (int c = 0; c < HC; ++c) {
                    const int col = lh * HC + ((c + l32) & (HC - 1));
                    if (col < ncol) {
                        acc_t v = from_word<acc_t>(*reinterpret_cast<const uint32_t *>(wbuf + l32 * SROW + col * 4));
                        if (has_bias) v = add_t(v, bias_lds[wn * TN + col]);
                        rs = add_t(rs, v);
                        if constexpr (!T::IS_INT) {
                            if (sto) rs_s += stored_value<DT>((float)v);
                        }
                    }
                }
                rs = add_xor32(rs);
                if (lane < 32) rs_part[wn * BM + wm * TM + mi * 32 + lane] = rs;
                if constexpr (!T::IS_INT) {
                    if (sto) {
                        rs_s = add_xor32(rs_s);
                        rowsto[mi] = rs_s;                              // lanes 0..31: row mi * 32 + lane
                    }
                }
            }
            wave_sync();
        } else if (PROT) {
            if (lane < 32) rs_part[wn * BM + wm * TM + mi * 32 + lane] = T::zero();
        }
    });

    if (PROT) {
        // ---- column sums of the register-path groups: transpose the lanes' partials through LDS
        static_for<0, NI>([&](auto ni_c) {
            constexpr int ni = decltype(ni_c)::value;
            static_for<0, 4>([&](auto q_c) {
                constexpr int q = decltype(q_c)::value;
                uint8_t *d = wbuf + l32 * SROW + (ni * 32 + 8 * q + 4 * lh) * 4;
                *reinterpret_cast<i32x4 *>(d) =
                    i32x4{(int)as_word(cp[PROT ? ni : 0][4 * q]), (int)as_word(cp[PROT ? ni : 0][4 * q + 1]),
                          (int)as_word(cp[PROT ? ni : 0][4 * q + 2]), (int)as_word(cp[PROT ? ni : 0][4 * q + 3])};
            });
        });
        wave_sync();
#pragma unroll
        for (int r = 0; r < 32; ++r) {
            if constexpr (CPL == 2) {
                const uint2 w = *reinterpret_cast<const uint2 *>(wbuf + r * SROW + lane * 8);
                colacc[0] = add_t(colacc[0], from_word<acc_t>(w.x));
                colacc[1] = add_t(colacc[1], from_word<acc_t>(w.y));
            } else {
#pragma unroll
                for (int j = 0; j < CPL; ++j)
                    colacc[j] = add_t(colacc[j], from_word<acc_t>(*reinterpret_cast<const uint32_t *>(
                                                     wbuf + r * SROW + (CPL * lane + j) * 4)));
            }
        }
#pragma unroll
        for (int j = 0; j < CPL; ++j) cs_part[wm * BN + wn * TN + CPL * lane + j] = colacc[j];
        if constexpr (!T::IS_INT) {
            if (sto) {
                // ---- stored-side sums of the register-path groups: second pass over the
                // accumulators, each value rounded as the store above rounded it
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int i = 0; i < 16; ++i) cp[PROT ? ni : 0][i] = T::zero();
                static_for<0, MI>([&](auto mi_c) {
                    constexpr int mi = decltype(mi_c)::value;
                    if (reg_path[mi]) {
                        float rsum = 0.f;
                        static_for<0, NI>([&](auto ni_c) {
                            constexpr int ni = decltype(ni_c)::value;
                            static_for<0, 8>([&](auto h_c) {
                                constexpr int h = decltype(h_c)::value;
                                float x0 = (float)acc_read(acc[mi][ni][2 * h]), x1 = (float)acc_read(acc[mi][ni][2 * h + 1]);
                                if (has_bias) {
                                    // register i of a block is column 8 (i >> 2) + 4 lh + (i & 3)
                                    const int cb0 = wn * TN + ni * 32 + 8 * ((2 * h) >> 2) + 4 * lh + ((2 * h) & 3);
                                    x0 += (float)bias_lds[cb0];
                                    x1 += (float)bias_lds[cb0 + 1];
                                }
                                const uint32_t w = pack2<DT>(x0, x1);
                                float s0, s1;
                                if constexpr (DT == DT_BF16) {
                                    s0 = __uint_as_float(w << 16);
                                    s1 = __uint_as_float(w & 0xFFFF0000u);
                                } else {
                                    s0 = f16_bits_to_f32(w & 0xFFFFu);
                                    s1 = f16_bits_to_f32(w >> 16);
                                }
                                cp[PROT ? ni : 0][2 * h] = add_t(cp[PROT ? ni : 0][2 * h], (acc_t)s0);
                                cp[PROT ? ni : 0][2 * h + 1] = add_t(cp[PROT ? ni : 0][2 * h + 1], (acc_t)s1);
                                rsum += s0 + s1;
                                cmax_s = fmaxf(cmax_s, fmaxf(fabsf(s0), fabsf(s1)));
                            });
                            __builtin_amdgcn_sched_barrier(0);
                        });
                        rsum = add_xor32(rsum);
                        rowsto[mi] = rsum;                              // lanes 0..31: row mi * 32 + lane
                    }
                });
                wave_sync();
                static_for<0, NI>([&](auto ni_c) {
                    constexpr int ni = decltype(ni_c)::value;
                    static_for<0, 4>([&](auto q_c) {
                        constexpr int q = decltype(q_c)::value;
                        uint8_t *d = wbuf + l32 * SROW + (ni * 32 + 8 * q + 4 * lh) * 4;
                        *reinterpret_cast<i32x4 *>(d) =
                            i32x4{(int)as_word(cp[PROT ? ni : 0][4 * q]), (int)as_word(cp[PROT ? ni : 0][4 * q + 1]),
                                  (int)as_word(cp[PROT ? ni : 0][4 * q + 2]), (int)as_word(cp[PROT ? ni : 0][4 * q + 3])};
                    });
                });
                wave_sync();
                for (int r = 0; r < 32; ++r)
#pragma unroll
                    for (int j = 0; j < CPL; ++j)
                        colacc_s[j] += __uint_as_float(*reinterpret_cast<const uint32_t *>(wbuf + r * SROW + (CPL * lane + j) * 4));
                // one atomic per row / column of the wave tile (two waves share each)
                if (lane < 32) {
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi) {
                        const int gr = wr0 + mi * 32 + lane;
                        if (gr < M) unsafeAtomicAdd(reinterpret_cast<float *>(g.rc_sto) + (long)bz * M + gr, rowsto[mi]);
                    }
                }
#pragma unroll
                for (int j = 0; j < CPL; ++j) {
                    const int gc = wc0 + CPL * lane + j;
                    if (gc < N) unsafeAtomicAdd(reinterpret_cast<float *>(g.cc_sto) + (long)bz * N + gc, colacc_s[j]);
                }
                // the largest stored magnitude: what a consumer of this C needs as its max|A|
                cmax_s = wave_max(cmax_s);
                if (lane == 0 && cmax_s > 0.f && cmax_s == cmax_s) atomicMax(g.c_max + bz, __float_as_uint(cmax_s));
            }
        }
        // ---- what the pass over A's slabs left in registers (nothing in a tile that reduced no slab:
        // where K has fewer slabs than the tile row has tiles, that is most tiles)
        if (ep.owned > 0) {
            constexpr int P = BM / 32;
            const int c = tid & 7, rg = tid >> 3;
            if (c < P) rp[rg + 32 * c] = ep.st.rdot;
            if (!T::IS_INT) {
                const float m = wave_max(ep.st.amax);
                if (lane == 0) amax4[wave] = m;
            }
        }
        // Barrier over LDS traffic only: the partial sums meet in LDS, and a full barrier would
        // also wait until every store of C issued above has been acknowledged.
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        for (int t = tid; t < BM + BN; t += 256) {
            if (t < BM) {
                const int gr = m0 + t;
                if (gr < M) {
                    atomic_add_word(g.rc_obs + (long)bz * M + gr, add_t(rs_part[t], rs_part[BM + t]));
                    if (ep.owned > 0) atomic_add_word(g.rc_pred + (long)bz * M + gr, rp[t]);
                }
            } else {
                const int gc = n0 + (t - BM);
                if (gc < N)
                    atomic_add_word(g.cc_obs + (long)bz * N + gc, add_t(cs_part[t - BM], cs_part[BN + t - BM]));
            }
        }
        // column sums of A over this tile's rows, for the slabs this workgroup reduced
        for (int t = tid; t < ep.owned * KE && !g.a_given; t += 256) {
            const int k = (ep.slab0 + (t / KE) * ep.slab_step) * KE + (t % KE);
            if (k < g.K) {
                acc_t v = from_word<acc_t>(ep.col_lds[t]);
                for (int w = 1; w < ep.col_copies; ++w) v = add_t(v, from_word<acc_t>(ep.col_lds[w * ep.col_stride + t]));
                atomic_add_word(g.a_sum + (long)bz * g.K + k, v);
            }
        }
        if (!T::IS_INT && tid == 0 && !g.a_given && ep.owned > 0) {
            const float m = fmaxf(fmaxf(amax4[0], amax4[1]), fmaxf(amax4[2], amax4[3]));
            if (m > 0.f) atomicMax(g.a_max + bz, __float_as_uint(m));
        }
    }
}

// With and without a layer bias: two copies of the epilogue behind one uniform branch (a test per
// group of four values inside one copy costs a branch per group).
template <int DT, int BM, int BN, bool PROT>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &g,
                                              typename Traits<DT>::accv_t (&acc)[BM / 64][BN / 64],
                                              uint8_t *smem, int m0, int n0, int bz, const EpiProt<DT> &ep)
{
    if (g.bias != nullptr) gemm_epilogue_impl<DT, BM, BN, PROT, true>(g, acc, smem, m0, n0, bz, ep);
    else gemm_epilogue_impl<DT, BM, BN, PROT, false>(g, acc, smem, m0, n0, bz, ep);
}

}  // namespace abft
