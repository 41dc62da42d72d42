// Device-side helpers for gfx950 (64-wide wavefronts, MFMA, DPP).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "abft_internal.h"

namespace abft {

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) int i32x16;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

// The thread's index inside its workgroup, as a value the optimiser cannot move or merge.  Code
// that runs once per tile inside a loop over tiles derives dozens of per-lane addresses from
// it; taken from the plain built-in they are all computed once before the loop and held in
// registers across it (40 more vector registers in the fast GEMM kernel).
__device__ __forceinline__ int tile_thread_index()
{
    int t = (int)threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
}

// ---------------------------------------------------------------- conversions
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// fp32 -> bf16, round to nearest even; NaN stays NaN (quiet).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if (f != f) return (u >> 16) | 0x0040u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ float f16_bits_to_f32(uint32_t h)
{
    _Float16 x = __builtin_bit_cast(_Float16, (uint16_t)h);
    return (float)x;
}

// fp32 -> fp16, round to nearest even (the conversion instruction's default mode).
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f)
{
    _Float16 x = (_Float16)f;
    return (uint32_t)__builtin_bit_cast(uint16_t, x);
}

// ---------------------------------------------------------------- per-dtype traits
template <int DT> struct Traits;

template <> struct Traits<DT_I8> {
    typedef int acc_t;
    typedef i32x16 accv_t;
    static constexpr int ES = 1;       // bytes per operand element
    static constexpr int OS = 4;       // bytes per output element
    static constexpr bool IS_INT = true;
    // one 32x32 MFMA step consumes 32 bytes of K per row (16 per half-wave)
    __device__ static __forceinline__ accv_t mfma(i32x4 a, i32x4 b, accv_t c)
    {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    }
    __device__ static __forceinline__ int elem(const i32x4 &v, int e)   // element e of a 16-byte chunk
    {
        return (int)(int8_t)((uint32_t)v[e >> 2] >> (8 * (e & 3)));
    }
    __device__ static __forceinline__ void store_c(void *C, long idx, acc_t v) { ((int *)C)[idx] = v; }
    __device__ static __forceinline__ acc_t load_c(const void *C, long idx) { return ((const int *)C)[idx]; }
    __device__ static __forceinline__ acc_t zero() { return 0; }
};

template <> struct Traits<DT_BF16> {
    typedef float acc_t;
    typedef f32x16 accv_t;
    static constexpr int ES = 2;
    static constexpr int OS = 2;
    static constexpr bool IS_INT = false;
    __device__ static __forceinline__ accv_t mfma(i32x4 a, i32x4 b, accv_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    __device__ static __forceinline__ float elem(const i32x4 &v, int e)
    {
        uint32_t w = (uint32_t)v[e >> 1];
        return __uint_as_float((e & 1) ? (w & 0xFFFF0000u) : (w << 16));
    }
    __device__ static __forceinline__ void store_c(void *C, long idx, acc_t v)
    {
        ((uint16_t *)C)[idx] = (uint16_t)f32_to_bf16_bits(v);
    }
    __device__ static __forceinline__ acc_t load_c(const void *C, long idx)
    {
        return bf16_bits_to_f32(((const uint16_t *)C)[idx]);
    }
    __device__ static __forceinline__ acc_t zero() { return 0.f; }
};

template <> struct Traits<DT_F16> {
    typedef float acc_t;
    typedef f32x16 accv_t;
    static constexpr int ES = 2;
    static constexpr int OS = 2;
    static constexpr bool IS_INT = false;
    __device__ static __forceinline__ accv_t mfma(i32x4 a, i32x4 b, accv_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
    __device__ static __forceinline__ float elem(const i32x4 &v, int e)
    {
        uint32_t w = (uint32_t)v[e >> 1];
        return f16_bits_to_f32((e & 1) ? (w >> 16) : (w & 0xFFFFu));
    }
    __device__ static __forceinline__ void store_c(void *C, long idx, acc_t v)
    {
        ((uint16_t *)C)[idx] = (uint16_t)f32_to_f16_bits(v);
    }
    __device__ static __forceinline__ acc_t load_c(const void *C, long idx)
    {
        return f16_bits_to_f32(((const uint16_t *)C)[idx]);
    }
    __device__ static __forceinline__ acc_t zero() { return 0.f; }
};

// ---------------------------------------------------------------- 32-bit word views of checksum values
__device__ __forceinline__ uint32_t as_word(int v) { return (uint32_t)v; }
__device__ __forceinline__ uint32_t as_word(float v) { return __float_as_uint(v); }
template <typename T> __device__ __forceinline__ T from_word(uint32_t w);
template <> __device__ __forceinline__ int from_word<int>(uint32_t w) { return (int)w; }
template <> __device__ __forceinline__ float from_word<float>(uint32_t w) { return __uint_as_float(w); }

// Device-scope atomic add on a 32-bit checksum word (integer: wraps modulo 2^32).
__device__ __forceinline__ void atomic_add_word(uint32_t *p, int v) { atomicAdd((int *)p, v); }
__device__ __forceinline__ void atomic_add_word(uint32_t *p, float v) { unsafeAtomicAdd((float *)p, v); }

// Reads that must see other workgroups' atomics: go through the atomic unit.
__device__ __forceinline__ uint32_t atomic_read_word(uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Store that other workgroups of the same launch will read: goes to the coherence point.
__device__ __forceinline__ void publish_word(uint32_t *p, uint32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---------------------------------------------------------------- wave-level reductions (DPP)
template <int CTRL> __device__ __forceinline__ int dpp_mov(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
__device__ __forceinline__ int add_t(int a, int b) { return a + b; }
__device__ __forceinline__ float add_t(float a, float b) { return a + b; }
template <int CTRL> __device__ __forceinline__ int dpp_get(int v) { return dpp_mov<CTRL>(v); }
template <int CTRL> __device__ __forceinline__ float dpp_get(float v)
{
    return __int_as_float(dpp_mov<CTRL>(__float_as_int(v)));
}

// Exchange between the rows of 16 lanes and between the halves of a wave with the row-swap
// instructions of gfx950 (v_permlane16_swap, v_permlane32_swap: vector ALU, no trip through the
// LDS crossbar as a lane shuffle takes).  Called with the same value twice, the two results
// hold, lane by lane, the lane's own value and that of lane ^ 16 (lane ^ 32), in either order.
__device__ __forceinline__ int add_xor16(int v)
{
    auto p = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
    return (int)(p[0] + p[1]);
}
__device__ __forceinline__ int add_xor32(int v)
{
    auto p = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
    return (int)(p[0] + p[1]);
}
__device__ __forceinline__ float add_xor16(float v)
{
    auto p = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(p[0]) + __uint_as_float(p[1]);
}
__device__ __forceinline__ float add_xor32(float v)
{
    auto p = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(p[0]) + __uint_as_float(p[1]);
}
__device__ __forceinline__ float max_xor16(float v)
{
    auto p = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(p[0]), __uint_as_float(p[1]));
}
__device__ __forceinline__ float max_xor32(float v)
{
    auto p = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(p[0]), __uint_as_float(p[1]));
}

// Sum over each aligned group of 16 lanes; every lane of the group ends with the total.
template <typename T> __device__ __forceinline__ T row16_sum(T v)
{
    v = add_t(v, dpp_get<0xB1>(v));    // quad_perm [1,0,3,2]: lane ^ 1
    v = add_t(v, dpp_get<0x4E>(v));    // quad_perm [2,3,0,1]: lane ^ 2
    v = add_t(v, dpp_get<0x141>(v));   // row_half_mirror: i <-> 7 - i inside 8 lanes
    v = add_t(v, dpp_get<0x140>(v));   // row_mirror: i <-> 15 - i inside 16 lanes
    return v;
}

// Sum over each half-wave (lanes 0..31 and 32..63); every lane of the half ends with the total.
template <typename T> __device__ __forceinline__ T half_wave_sum(T v)
{
    v = row16_sum(v);
    return add_xor16(v);
}

// Sum over the whole wave; every lane ends with the total.
template <typename T> __device__ __forceinline__ T wave_sum(T v)
{
    v = half_wave_sum(v);
    return add_xor32(v);
}

// Sum over aligned groups of `width` lanes (8, 16, 32 or 64); every lane of a group ends with
// the total.
template <typename V> __device__ __forceinline__ V seg_sum(V v, int width)
{
    v = add_t(v, dpp_get<0xB1>(v));    // lane ^ 1
    v = add_t(v, dpp_get<0x4E>(v));    // lane ^ 2
    v = add_t(v, dpp_get<0x141>(v));   // i <-> 7 - i inside 8 lanes
    if (width >= 16) v = add_t(v, dpp_get<0x140>(v));   // i <-> 15 - i inside 16 lanes
    if (width >= 32) v = add_xor16(v);
    if (width >= 64) v = add_xor32(v);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_get<0xB1>(v));    // lane ^ 1
    v = fmaxf(v, dpp_get<0x4E>(v));    // lane ^ 2
    v = fmaxf(v, dpp_get<0x141>(v));   // i <-> 7 - i inside 8 lanes
    v = fmaxf(v, dpp_get<0x140>(v));   // i <-> 15 - i inside 16 lanes
    v = max_xor16(v);
    v = max_xor32(v);
    return v;
}

// Products of checksum values (integer: in Z/2^32).
__device__ __forceinline__ int mul_t(int x, int y) { return (int)((uint32_t)x * (uint32_t)y); }
__device__ __forceinline__ float mul_t(float x, float y) { return x * y; }

// The check of Sec. III-B.1 item (2): equality for fixed point, tolerance for floating point.
template <bool IS_INT>
__device__ __forceinline__ bool mismatch(uint32_t obs, uint32_t pred, float tol)
{
    if (IS_INT) return obs != pred;                          // equality in Z/2^32
    float d = fabsf(__uint_as_float(obs) - __uint_as_float(pred));
    return !(d <= tol);                                      // NaN and Inf always flag
}

__device__ __forceinline__ uint32_t status_of(uint32_t nr, uint32_t nc)
{
    if (nr == 0 && nc == 0) return 0u;      // clean
    if (nr == 0 || nc == 0) return 2u;      // checksum suspect
    return 1u;                              // localised
}

// Keep the first nbytes (0..16) of a 16-byte chunk, zero the rest.
__device__ __forceinline__ i32x4 mask_chunk(i32x4 v, int nbytes)
{
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        int keep = nbytes - 4 * w;                 // bytes of this word to keep
        uint32_t m = keep >= 4 ? 0xFFFFFFFFu : (keep <= 0 ? 0u : ((1u << (8 * keep)) - 1u));
        v[w] = (int)((uint32_t)v[w] & m);
    }
    return v;
}

}  // namespace abft
