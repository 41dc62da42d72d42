// Input-side checksums of A taken from the operand slabs the GEMM already holds in LDS.
//
// The checksum scheme (Sec. III-B.1 "Checksums") needs two reductions of A: the column sums
// a = e^T A (which give the column checksum prediction (e^T A) B) and the matrix-vector product
// A (B e) (the row checksum prediction).  Both read every element of A exactly once, and every
// element of A passes through LDS on its way to the matrix cores anyway: of the workgroups that
// share a tile row, the one in tile column (s mod tiles_n) reduces slab s while it is resident.
// So A is read from memory once, by the GEMM, and the separate encode pass over A disappears.
//
// LDS slab layout (both GEMM kernels): row r is 128 bytes = eight 16-byte chunks, chunk c stored
// in slot c ^ (r & 7).  Thread t reduces chunk c = t & 7 of rows (t >> 3) + 32 p.
#pragma once
#include "abft_device.h"
#include "gemm_args.h"

namespace abft {

// Sum over each aligned group of 8 lanes; every lane of the group ends with the total.
template <typename T> __device__ __forceinline__ T row8_sum(T v)
{
    v = add_t(v, dpp_get<0xB1>(v));    // lane ^ 1
    v = add_t(v, dpp_get<0x4E>(v));    // lane ^ 2
    v = add_t(v, dpp_get<0x141>(v));   // i <-> 7 - i inside 8 lanes
    return v;
}

// LDS atomic add on a 32-bit checksum word, written as the instruction itself.  Through the
// compiler's atomicAdd every one of these is preceded by a wait for ALL outstanding memory
// operations of the wave: the operand loads of the next slab go straight into LDS
// (global_load_lds) and the compiler, which cannot tell their target from this word, orders the
// atomic behind them -- the pass then stalls for a full load latency in every slab it reduces.
// The words added to here are never a target of those loads.
__device__ __forceinline__ void lds_add_word(uint32_t *p, float v)
{
    const uint32_t a = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint32_t *)p;
    asm volatile("ds_add_f32 %0, %1" :: "v"(a), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_add_word(uint32_t *p, int v)
{
    const uint32_t a = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint32_t *)p;
    asm volatile("ds_add_u32 %0, %1" :: "v"(a), "v"(v) : "memory");
}

// Per-thread state of the A pass that lives across the slabs of one tile.
template <int DT> struct APassState {
    typename Traits<DT>::acc_t rdot;   // dot of row (t >> 3) + 32 (t & 7) with b, over the owned slabs
    float amax;                        // max |A| seen (floating point only)
};

// LDS the pass needs for a tile besides the operand buffers: for every owned slab KE words of
// column sums and KE words of b (staged once, at the start of the tile, zero beyond K).
__host__ __device__ inline int apass_owned_slabs(int nslab, int tiles_n) { return (nslab + tiles_n - 1) / tiles_n; }
__host__ __device__ inline size_t apass_lds_bytes(int dt, int nslab, int tiles_n)
{
    return (size_t)apass_owned_slabs(nslab, tiles_n) * (SLAB_BYTES / elem_size(dt)) * 8;
}
// the same with column sums kept per wave (four waves) instead of added up in place
__host__ __device__ inline size_t apass_lds_bytes_per_wave(int dt, int nslab, int tiles_n)
{
    return (size_t)apass_owned_slabs(nslab, tiles_n) * (SLAB_BYTES / elem_size(dt)) * 20;
}

// Reduce one resident slab of A.  sA: the slab in LDS (BM rows).  b_lds: the KE values of b
// that belong to the slab (LDS).  rows_valid: rows of the tile inside M (rows beyond may hold
// anything, finite or not: they are ignored).  col_lds: KE words of this slab's column sums
// (LDS atomics: the four waves add to the same words).
// GIVEN: the caller supplied a = e^T A and max|A| (a checksum carried over from the kernel that
// produced A): only the row dots are formed.
// SW16: the slab's swizzle is slot = chunk ^ ((row >> 1) & 7) (gemm_fast) instead of chunk ^ (row & 7).
// SPLIT_ONLY: int8 with |b| < 2^23 guaranteed by the caller (mul24_ok is not consulted): the
// element-wise integer form is left out, which is what keeps the fast kernel's registers free of spills.
// PER_WAVE: col_lds is this wave's own KE words for the slab, written with plain stores (the caller
// adds the waves' words up when it hands the sums on).  Measured on the fast kernel: the eight LDS
// atomic adds per wave and slab held the wave's next LDS reads back by some 800 clocks.
template <int DT, int BM, bool GIVEN = false, bool SW16 = false, bool SPLIT_ONLY = false, bool PER_WAVE = false>
__device__ __forceinline__ void a_pass(const uint8_t *sA, const uint32_t *b_lds, int rows_valid,
                                       uint32_t *col_lds, APassState<DT> &st, bool mul24_ok)
{
    using T = Traits<DT>;
    typedef typename T::acc_t acc_t;
    constexpr int CE = 16 / T::ES;
    constexpr int P = BM / 32;
    const int tid = tile_thread_index();
    const int c = tid & 7, rg = tid >> 3;
    const uint8_t *src = sA + rg * SLAB_BYTES + ((c ^ (SW16 ? (rg >> 1) & 7 : rg & 7)) * 16);

    acc_t bv[CE], cs[CE];
#pragma unroll
    for (int q4 = 0; q4 < CE / 4; ++q4) {
        const i32x4 w = *reinterpret_cast<const i32x4 *>(b_lds + c * CE + 4 * q4);
#pragma unroll
        for (int e = 0; e < 4; ++e) bv[4 * q4 + e] = from_word<acc_t>((uint32_t)w[e]);
    }
#pragma unroll
    for (int q = 0; q < CE; ++q) cs[q] = T::zero();
    i32x4 v[P];
#pragma unroll
    for (int p = 0; p < P; ++p) v[p] = *reinterpret_cast<const i32x4 *>(src + p * 32 * SLAB_BYTES);
    acc_t mine = T::zero();
    bool done = false;
    if constexpr (T::IS_INT) {
        if (mul24_ok || SPLIT_ONLY) {
            // |b| <= 128 N < 2^23: b = 256 hi + lo with 0 <= lo < 256 and |hi| < 2^15.  The bytes of a
            // word of A as two pairs of 16-bit integers (bytes 0, 2 and bytes 1, 3): the column sums
            // add pair-wise (at most 8 rows per thread), the row product takes two products per
            // instruction against the pairs of hi and of lo.
            typedef short s16x2 __attribute__((ext_vector_type(2)));
            s16x2 bhi[8], blo[8], csp[8];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int b0 = (int)bv[4 * d], b1 = (int)bv[4 * d + 1], b2 = (int)bv[4 * d + 2], b3 = (int)bv[4 * d + 3];
                bhi[2 * d] = s16x2{(short)(b0 >> 8), (short)(b2 >> 8)};
                bhi[2 * d + 1] = s16x2{(short)(b1 >> 8), (short)(b3 >> 8)};
                blo[2 * d] = s16x2{(short)(b0 & 255), (short)(b2 & 255)};
                blo[2 * d + 1] = s16x2{(short)(b1 & 255), (short)(b3 & 255)};
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) csp[j] = s16x2{0, 0};
#pragma unroll
            for (int p = 0; p < P; ++p) {
                i32x4 x4 = v[p];
                if (rg + 32 * p >= rows_valid) x4 = i32x4{0, 0, 0, 0};
                int dhi = 0, dlo = 0;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const int wd = x4[d];
                    const s16x2 w = s16x2{(short)(wd & 0xFFFF), (short)(wd >> 16)};
                    const s16x2 ev = (w << 8) >> 8, od = w >> 8;       // bytes 0, 2 and 1, 3, sign-extended
                    if (!GIVEN) {
                        csp[2 * d] += ev;
                        csp[2 * d + 1] += od;
                    }
                    dhi = __builtin_amdgcn_sdot2(ev, bhi[2 * d], dhi, false);
                    dhi = __builtin_amdgcn_sdot2(od, bhi[2 * d + 1], dhi, false);
                    dlo = __builtin_amdgcn_sdot2(ev, blo[2 * d], dlo, false);
                    dlo = __builtin_amdgcn_sdot2(od, blo[2 * d + 1], dlo, false);
                }
                acc_t dot = (acc_t)(int)((uint32_t)dhi * 256u + (uint32_t)dlo);
                dot = row8_sum(dot);
                if (c == p) mine = dot;
            }
#pragma unroll
            for (int q = 0; q < CE; ++q) cs[q] = (acc_t)csp[2 * (q >> 2) + (q & 1)][(q >> 1) & 1];
            done = true;
        }
    }
    if (!(T::IS_INT && SPLIT_ONLY) && !done) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            i32x4 x4 = v[p];
            if (rg + 32 * p >= rows_valid) x4 = i32x4{0, 0, 0, 0};
            acc_t dot = T::zero();
#pragma unroll
            for (int q = 0; q < CE; ++q) {
                const acc_t x = T::elem(x4, q);
                if (!GIVEN) cs[q] = add_t(cs[q], x);
                if constexpr (T::IS_INT) {
                    dot = (acc_t)((uint32_t)x * (uint32_t)bv[q] + (uint32_t)dot);
                } else {
                    dot = __builtin_fmaf((float)x, (float)bv[q], (float)dot);
                    if (!GIVEN) st.amax = fmaxf(st.amax, fabsf((float)x));
                }
            }
            dot = row8_sum(dot);
            if (c == p) mine = dot;
        }
    }
    st.rdot = add_t(st.rdot, mine);
    if constexpr (GIVEN) return;
    // Column sums: first over the eight row groups of the wave (lanes with equal c), then one
    // LDS atomic per column and wave.  (LDS atomics in which several lanes of one instruction
    // hit the same word are served one lane at a time.)
#pragma unroll
    for (int q = 0; q < CE; ++q) {
        acc_t t = cs[q];
        t = add_t(t, dpp_get<0x128>(t));      // row_ror:8 inside 16 lanes: lane ^ 8
        t = add_xor16(t);
        t = add_xor32(t);
        cs[q] = t;
    }
    if ((tid & 63) < 8) {
#pragma unroll
        for (int q = 0; q < CE; ++q) {
            if constexpr (PER_WAVE) col_lds[c * CE + q] = as_word(cs[q]);
            else lds_add_word(col_lds + c * CE + q, cs[q]);
        }
    }
}

// The same reduction cut into pieces that the fast GEMM kernel issues one by one behind the MFMAs
// of the slab (the matrix pipe works on an MFMA for 32 clocks; the few vector instructions of a
// piece are issued in its shadow).  begin() requests the thread's chunks of the slab and its values
// of b, piece<k>() takes element (or, int8, half a word) k % 8 of row group k / 8, end() reduces the
// column sums over the wave and writes them to the wave's own words for the slab in LDS.  Same
// arithmetic, in the same order, as a_pass above with SW16, PER_WAVE and (int8) SPLIT_ONLY.
template <int DT, int BM, bool GIVEN> struct APassSteps {
    using T = Traits<DT>;
    typedef typename T::acc_t acc_t;
    typedef short s16x2 __attribute__((ext_vector_type(2)));
    static constexpr int CE = 16 / T::ES;
    static constexpr int P = BM / 32;
    static constexpr int PIECES = P * 8;
    int c, rg, rows_valid;
    i32x4 v[P];
    acc_t bv[T::IS_INT ? 1 : CE], cs[T::IS_INT ? 1 : CE];
    s16x2 bhi[T::IS_INT ? 8 : 1], blo[T::IS_INT ? 8 : 1], csp[T::IS_INT ? 8 : 1], ev, od;
    acc_t dot, mine;
    int dhi, dlo;
    float amax;

    __device__ __forceinline__ void begin(const uint8_t *sA, const uint32_t *b_lds, int rows_valid_)
    {
        const int tid = tile_thread_index();
        c = tid & 7; rg = tid >> 3; rows_valid = rows_valid_;
        const uint8_t *src = sA + rg * SLAB_BYTES + ((c ^ ((rg >> 1) & 7)) * 16);
#pragma unroll
        for (int p = 0; p < P; ++p) v[p] = *reinterpret_cast<const i32x4 *>(src + p * 32 * SLAB_BYTES);
        if constexpr (T::IS_INT) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const i32x4 w = *reinterpret_cast<const i32x4 *>(b_lds + c * CE + 4 * d);
                const int b0 = w[0], b1 = w[1], b2 = w[2], b3 = w[3];
                bhi[2 * d] = s16x2{(short)(b0 >> 8), (short)(b2 >> 8)};
                bhi[2 * d + 1] = s16x2{(short)(b1 >> 8), (short)(b3 >> 8)};
                blo[2 * d] = s16x2{(short)(b0 & 255), (short)(b2 & 255)};
                blo[2 * d + 1] = s16x2{(short)(b1 & 255), (short)(b3 & 255)};
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) csp[j] = s16x2{0, 0};
        } else {
#pragma unroll
            for (int q4 = 0; q4 < CE / 4; ++q4) {
                const i32x4 w = *reinterpret_cast<const i32x4 *>(b_lds + c * CE + 4 * q4);
#pragma unroll
                for (int e = 0; e < 4; ++e) bv[4 * q4 + e] = from_word<acc_t>((uint32_t)w[e]);
            }
#pragma unroll
            for (int q = 0; q < CE; ++q) cs[q] = T::zero();
        }
        mine = T::zero();
        amax = 0.f;
    }

    template <int K> __device__ __forceinline__ void piece()
    {
        if constexpr (K >= 0 && K < PIECES) {
            constexpr int p = K / 8, e = K % 8;
            if constexpr (e == 0) {
                if (rg + 32 * p >= rows_valid) v[p] = i32x4{0, 0, 0, 0};
                dot = T::zero(); dhi = 0; dlo = 0;
            }
            if constexpr (T::IS_INT) {
                constexpr int d = e >> 1;
                if constexpr ((e & 1) == 0) {
                    const int wd = v[p][d];
                    const s16x2 w = s16x2{(short)(wd & 0xFFFF), (short)(wd >> 16)};
                    ev = (w << 8) >> 8; od = w >> 8;                 // bytes 0, 2 and 1, 3, sign-extended
                    if (!GIVEN) { csp[2 * d] += ev; csp[2 * d + 1] += od; }
                } else {
                    dhi = __builtin_amdgcn_sdot2(ev, bhi[2 * d], dhi, false);
                    dhi = __builtin_amdgcn_sdot2(od, bhi[2 * d + 1], dhi, false);
                    dlo = __builtin_amdgcn_sdot2(ev, blo[2 * d], dlo, false);
                    dlo = __builtin_amdgcn_sdot2(od, blo[2 * d + 1], dlo, false);
                }
                if constexpr (e == 7) dot = (acc_t)(int)((uint32_t)dhi * 256u + (uint32_t)dlo);
            } else {
                const acc_t x = T::elem(v[p], e);
                if (!GIVEN) cs[e] = add_t(cs[e], x);
                dot = __builtin_fmaf((float)x, (float)bv[e], (float)dot);
                if (!GIVEN) amax = fmaxf(amax, fabsf((float)x));
            }
            if constexpr (e == 7) {
                dot = row8_sum(dot);
                if (c == p) mine = dot;
            }
        }
    }

    __device__ __forceinline__ void end(uint32_t *col_lds, APassState<DT> &st)
    {
        st.rdot = add_t(st.rdot, mine);
        if constexpr (GIVEN) return;
        if constexpr (!T::IS_INT) st.amax = fmaxf(st.amax, amax);
        acc_t t[CE];
#pragma unroll
        for (int q = 0; q < CE; ++q) {
            if constexpr (T::IS_INT) t[q] = (acc_t)csp[2 * (q >> 2) + (q & 1)][(q >> 1) & 1];
            else t[q] = cs[q];
            t[q] = add_t(t[q], dpp_get<0x128>(t[q]));      // row_ror:8 inside 16 lanes: lane ^ 8
            t[q] = add_xor16(t[q]);
            t[q] = add_xor32(t[q]);
        }
        if ((tile_thread_index() & 63) < 8) {
#pragma unroll
            for (int q = 0; q < CE; ++q) col_lds[c * CE + q] = as_word(t[q]);      // this wave's own words
        }
    }
};

}  // namespace abft
