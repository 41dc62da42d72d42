// Kernels around the protected GEMM: encode (input-side checksums and their
// stripe encoding), compare (flags), verify (re-sum stored C), correct
// (localise, recompute tiles, re-check) and the bit-flip test hook.
//
// Paper references: the two input-side vectors and the comparison with the
// output sums are the checksum scheme of Sec. III-B.1 ("Checksums"); equality
// for integers and a tolerance for floating point follow item (2) there; the
// tile recompute is the replay correction of Sec. III-B.3 at tile granularity;
// the flip is the fault model of Sec. II-A / III-A.
#include "abft_device.h"

namespace abft {

// ======================================================================== zero
__global__ void zero_kernel(uint32_t *p, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t step = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += step) p[i] = 0u;
}

hipError_t launch_zero(uint32_t *p, size_t nwords, hipStream_t st)
{
    if (nwords == 0) return hipSuccess;
    size_t blocks = (nwords + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, nwords);
    return hipGetLastError();
}

// ====================================================================== encode
// Input-side checksum vectors (Sec. III-B.1 "Checksums"): a = e^T A (the input summed over its
// rows) and b = B e (the weight reduced over its output dimension), both of length K, plus
// what only a pass over the operands can give: max|A|, max|B| for the tolerance, and the row
// checksum prediction rc_pred = A b.  That last product is a matrix-vector product, bound by
// the read of A, so it rides on the same streaming pass instead of occupying MFMA tiles.
// The pass over B comes first (b must be complete before A b); for a weight it is done once,
// offline (remark (2) of the same paragraph).
constexpr int ENC_UNROLL = 8;     // independent 16-byte loads in flight per thread (B pass)
// Atomics on one cache line are served one after the other (tens of nanoseconds each), so the
// row blocks of a pass spread their column sums over several accumulator copies.
constexpr int ENC_COPIES = ENC_ACC_COPIES;

// Split an int32 sum into four signed base-256 digits: v = d0 + 2^8 d1 + 2^16 d2 + 2^24 d3 (mod 2^32).
__device__ __forceinline__ void split_digits(int v, int8_t d[NTERM])
{
#pragma unroll
    for (int t = 0; t < NTERM; ++t) {
        int8_t lo = (int8_t)(v & 0xFF);
        d[t] = lo;
        v = (int)(((int64_t)v - (int64_t)lo) >> 8);
    }
}

// Sum the accumulator copies of column k, leave them clean for the next call.  The reads go
// through the coherence point (device-scope atomic loads, all in flight at once); the zeros are
// ordinary stores, visible to the next kernel.
template <typename acc_t>
__device__ __forceinline__ acc_t take_copies(uint32_t *acc, long stride, int k)
{
    uint32_t part[ENC_COPIES];
#pragma unroll
    for (int c = 0; c < ENC_COPIES; ++c) part[c] = atomic_read_word(acc + c * stride + k);
    acc_t t = from_word<acc_t>(part[0]);
#pragma unroll
    for (int c = 1; c < ENC_COPIES; ++c) t = add_t(t, from_word<acc_t>(part[c]));
#pragma unroll
    for (int c = 0; c < ENC_COPIES; ++c) acc[c * stride + k] = 0u;
    return t;
}

// ---------------------------------------------------------------- B pass: b = B e, max|B|
// The stored array has `rows` rows of `cols` elements.  reduce_rows = 1 (B stored N x K):
// b[col] = sum over rows.  reduce_rows = 0 (B stored K x N): b[row] = sum over cols.
struct EncBArgs {
    const uint8_t *X;
    long ld, stride;      // elements
    int rows, cols, K;
    int reduce_rows;
    int cw_log2;          // 16-byte chunk columns per block window (power of two <= 64)
    int rpb;              // rows per block
    int nwin, nrb;
    uint32_t *acc;        // [ENC_COPIES][batch][K] atomic accumulators
    long acc_stride;
    uint32_t *sum;        // [batch][K]
    uint32_t *max_acc;    // [batch][2]
    float *maxabs;        // [batch][2]
    uint32_t *ticket;     // [batch]
};

template <int DT>
__global__ __launch_bounds__(256) void encode_b_kernel(EncBArgs e)
{
    using T = Traits<DT>;
    typedef typename T::acc_t acc_t;
    constexpr int ES = T::ES, CE = 16 / ES;
    __shared__ acc_t red[256 * CE];
    __shared__ float fred[4];
    __shared__ int is_last;

    const int tid = threadIdx.x, bz = blockIdx.z;
    const int win = blockIdx.x % e.nwin, rb = blockIdx.x / e.nwin;
    const int CW = 1 << e.cw_log2, RL = 256 >> e.cw_log2;
    const int cx = tid & (CW - 1), ry = tid >> e.cw_log2;
    const int col0 = (win * CW + cx) * CE;
    const bool colok = col0 < e.cols;
    const int nvalid = e.cols - col0;                        // elements of this chunk inside the row
    const uint8_t *Xb = e.X + (long)bz * e.stride * ES;
    const int rbeg = rb * e.rpb;
    const int rend = min(rbeg + e.rpb, e.rows);
    const int iters = (e.rpb + RL * ENC_UNROLL - 1) / (RL * ENC_UNROLL);

    acc_t colacc[CE];
#pragma unroll
    for (int q = 0; q < CE; ++q) colacc[q] = T::zero();
    float mx = 0.f;

    for (int it = 0; it < iters; ++it) {
        // a batch of independent loads first: the pass is bound by memory latency otherwise
        i32x4 v[ENC_UNROLL];
#pragma unroll
        for (int u = 0; u < ENC_UNROLL; ++u) {
            const int r = rbeg + ry + (it * ENC_UNROLL + u) * RL;
            v[u] = i32x4{0, 0, 0, 0};
            if (colok && r < rend) v[u] = *reinterpret_cast<const i32x4 *>(Xb + ((long)r * e.ld + col0) * ES);
        }
#pragma unroll
        for (int u = 0; u < ENC_UNROLL; ++u) {
            const int r = rbeg + ry + (it * ENC_UNROLL + u) * RL;
            i32x4 w = v[u];
            if (nvalid < CE) w = mask_chunk(w, nvalid > 0 ? nvalid * ES : 0);
            acc_t s = T::zero();
#pragma unroll
            for (int q = 0; q < CE; ++q) {
                acc_t x = T::elem(w, q);
                if (!T::IS_INT) mx = fmaxf(mx, fabsf((float)x));
                colacc[q] = add_t(colacc[q], x);
                s = add_t(s, x);
            }
            if (!e.reduce_rows) {
                for (int o = 1; o < CW; o <<= 1) s = add_t(s, __shfl_xor(s, o));
                if (cx == 0 && r < rend) atomic_add_word(e.acc + (long)bz * e.K + r, s);
            }
        }
    }
    if (e.reduce_rows) {
#pragma unroll
        for (int q = 0; q < CE; ++q) red[(ry * CW + cx) * CE + q] = colacc[q];
        __syncthreads();
        // one atomic per column, consecutive lanes on consecutive addresses
        for (int c = tid; c < CW * CE; c += 256) {
            const int col = win * CW * CE + c;
            if (col < e.cols) {
                acc_t t = red[c];
                for (int y = 1; y < RL; ++y) t = add_t(t, red[y * CW * CE + c]);
                atomic_add_word(e.acc + (rb % ENC_COPIES) * e.acc_stride + (long)bz * e.K + col, t);
            }
        }
    }
    if (!T::IS_INT) {
        mx = wave_max(mx);
        __syncthreads();
        if ((tid & 63) == 0) fred[tid >> 6] = mx;
        __syncthreads();
        if (tid == 0)
            atomicMax(e.max_acc + (long)bz * 2 + 1,
                      __float_as_uint(fmaxf(fmaxf(fred[0], fred[1]), fmaxf(fred[2], fred[3]))));
    }
    // Last block of this batch item finalises.  Everything other workgroups must see was
    // written with device-scope atomic read-modify-writes, which are performed at the device's
    // coherence point; the barrier waits for this workgroup's outstanding ones before the
    // ticket is taken.  (A device-wide fence here costs tens of microseconds per launch.)
    __syncthreads();
    if (tid == 0) {
        unsigned t = atomicAdd(e.ticket + bz, 1u);
        is_last = (t == (unsigned)(e.nwin * e.nrb) - 1);
        if (is_last) atomicExch(e.ticket + bz, 0u);
    }
    __syncthreads();
    if (!is_last) return;
    for (int k = tid; k < e.K; k += 256)
        e.sum[(long)bz * e.K + k] = as_word(take_copies<acc_t>(e.acc + (long)bz * e.K, e.acc_stride, k));
    if (!T::IS_INT && tid == 0)
        e.maxabs[(long)bz * 2 + 1] = __uint_as_float(atomicExch(e.max_acc + (long)bz * 2 + 1, 0u));
}

// ---------------------------------------------------------------- A pass: a = e^T A, A b, max|A|, stripe
// A block owns whole rows: CW lanes of 16-byte chunks cover a row in NW windows, 256 / CW rows
// at a time, so the dot product of a row with b completes inside the block (no atomics, no
// zeroing for rc_pred).  Column sums go to the accumulator copies; the last block of a batch
// item turns them into a, its stripe encoding, and the tolerance.
struct EncAArgs {
    const uint8_t *A;
    long lda, sA;
    int M, K, Kp;
    int cw_log2, nwin, rpb, nrb;
    uint32_t *a_acc;
    long acc_stride;
    uint32_t *a_sum;
    const uint32_t *b_sum;
    uint32_t *rc_pred;
    uint8_t *stripe;      // [batch][NTERM][Kp] operand elements
    float *w_a;           // [batch][NTERM]
    uint32_t *max_acc;
    float *maxabs, *tau;
    uint32_t *ticket;
    uint32_t *s_pred;     // [batch] scalar a . b (the paper's own single-number check value)
    float tau_override;
    uint32_t *zero_ptr;
    size_t zero_words;
};

__device__ __forceinline__ int mul_t(int x, int y) { return (int)((uint32_t)x * (uint32_t)y); }
__device__ __forceinline__ float mul_t(float x, float y) { return x * y; }

template <int DT, int NW>
__global__ __launch_bounds__(256) void encode_a_kernel(EncAArgs e)
{
    using T = Traits<DT>;
    typedef typename T::acc_t acc_t;
    constexpr int ES = T::ES, CE = 16 / ES;
    constexpr int UR = NW >= 8 ? 1 : 8 / NW;              // rows in flight per thread
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    __shared__ float fred[4];
    __shared__ int is_last;

    const int tid = threadIdx.x, bz = blockIdx.z, rb = blockIdx.x;
    const int K = e.K, M = e.M;
    // every block takes a share of the words that must start at zero for the GEMM epilogue
    {
        size_t nb = (size_t)gridDim.x * gridDim.z;
        size_t bid = blockIdx.x + (size_t)gridDim.x * blockIdx.z;
        for (size_t i = bid * 256 + tid; i < e.zero_words; i += nb * 256) e.zero_ptr[i] = 0u;
    }
    const int CW = 1 << e.cw_log2, RL = 256 >> e.cw_log2;
    const int cx = tid & (CW - 1), ry = tid >> e.cw_log2;
    const int span = e.nwin * CW * CE;                      // columns covered by the windows (>= K)
    acc_t *bl = reinterpret_cast<acc_t *>(lds);             // b staged, zero beyond K
    acc_t *red = bl + span;                                 // [RL][CW * CE]
    for (int k = tid; k < span; k += 256)
        bl[k] = k < K ? from_word<acc_t>(e.b_sum[(long)bz * K + k]) : T::zero();
    __syncthreads();

    const uint8_t *Ab = e.A + (long)bz * e.sA * ES;
    const int rbeg = rb * e.rpb, rend = min(rbeg + e.rpb, M);
    const int iters = (e.rpb + RL * UR - 1) / (RL * UR);

    acc_t colacc[NW][CE];
#pragma unroll
    for (int w = 0; w < NW; ++w)
#pragma unroll
        for (int q = 0; q < CE; ++q) colacc[w][q] = T::zero();
    float mx = 0.f;

    for (int it = 0; it < iters; ++it) {
        i32x4 v[UR][NW];
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            const int r = rbeg + ry + (it * UR + u) * RL;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const int col0 = (w * CW + cx) * CE;
                v[u][w] = i32x4{0, 0, 0, 0};
                if (w < e.nwin && col0 < K && r < rend)
                    v[u][w] = *reinterpret_cast<const i32x4 *>(Ab + ((long)r * e.lda + col0) * ES);
            }
        }
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            const int r = rbeg + ry + (it * UR + u) * RL;
            acc_t dot = T::zero();
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                if (w < e.nwin) {
                    const int col0 = (w * CW + cx) * CE;
                    i32x4 x4 = v[u][w];
                    if (K - col0 < CE) x4 = mask_chunk(x4, K - col0 > 0 ? (K - col0) * ES : 0);
#pragma unroll
                    for (int q = 0; q < CE; ++q) {
                        const acc_t x = T::elem(x4, q);
                        if (!T::IS_INT) mx = fmaxf(mx, fabsf((float)x));
                        colacc[w][q] = add_t(colacc[w][q], x);
                        dot = add_t(dot, mul_t(x, bl[col0 + q]));
                    }
                }
            }
            for (int o = 1; o < CW; o <<= 1) dot = add_t(dot, __shfl_xor(dot, o));
            if (cx == 0 && r < rend) e.rc_pred[(long)bz * M + r] = as_word(dot);
        }
    }
    // column sums: reduce over the row lanes in LDS, then one coalesced atomic per column
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        if (w < e.nwin) {
            __syncthreads();
#pragma unroll
            for (int q = 0; q < CE; ++q) red[(ry * CW + cx) * CE + q] = colacc[w][q];
            __syncthreads();
            for (int c = tid; c < CW * CE; c += 256) {
                const int col = w * CW * CE + c;
                if (col < K) {
                    acc_t t = red[c];
                    for (int y = 1; y < RL; ++y) t = add_t(t, red[y * CW * CE + c]);
                    atomic_add_word(e.a_acc + (rb % ENC_COPIES) * e.acc_stride + (long)bz * K + col, t);
                }
            }
        }
    }
    if (!T::IS_INT) {
        mx = wave_max(mx);
        __syncthreads();
        if ((tid & 63) == 0) fred[tid >> 6] = mx;
        __syncthreads();
        if (tid == 0)
            atomicMax(e.max_acc + (long)bz * 2, __float_as_uint(fmaxf(fmaxf(fred[0], fred[1]), fmaxf(fred[2], fred[3]))));
    }
    // last block of this batch item finalises (same ordering argument as in the B pass)
    __syncthreads();
    if (tid == 0) {
        unsigned t = atomicAdd(e.ticket + bz, 1u);
        is_last = (t == gridDim.x - 1);
        if (is_last) atomicExch(e.ticket + bz, 0u);
    }
    __syncthreads();
    if (!is_last) return;

    const int Kp = e.Kp;
    uint32_t *sum = e.a_sum + (long)bz * K;
    uint8_t *stripe = e.stripe + (long)bz * NTERM * Kp * ES;
    float amax = 0.f;
    for (int k = tid; k < K; k += 256) {
        const uint32_t w = as_word(take_copies<acc_t>(e.a_acc + (long)bz * K, e.acc_stride, k));
        sum[k] = w;
        if (!T::IS_INT) amax = fmaxf(amax, fabsf(__uint_as_float(w)));
    }
    {
        // scalar a . b, straight from the two sums (b is still staged in LDS)
        acc_t v = T::zero();
        for (int k = tid; k < K; k += 256) v = add_t(v, mul_t(from_word<acc_t>(sum[k]), bl[k]));
        v = wave_sum(v);
        __syncthreads();
        if ((tid & 63) == 0) fred[tid >> 6] = __uint_as_float(as_word(v));
        __syncthreads();
        if (tid == 0) {
            acc_t t = add_t(add_t(from_word<acc_t>(__float_as_uint(fred[0])), from_word<acc_t>(__float_as_uint(fred[1]))),
                            add_t(from_word<acc_t>(__float_as_uint(fred[2])), from_word<acc_t>(__float_as_uint(fred[3]))));
            e.s_pred[bz] = as_word(t);
        }
        __syncthreads();
    }
    float scale = 1.f, inv = 1.f;
    if (DT == DT_F16) {
        // power-of-two pre-scale so the largest |sum| sits in [2^13, 2^14): well inside fp16 range
        amax = wave_max(amax);
        __syncthreads();
        if ((tid & 63) == 0) fred[tid >> 6] = amax;
        __syncthreads();
        amax = fmaxf(fmaxf(fred[0], fred[1]), fmaxf(fred[2], fred[3]));
        int sh = 0;
        if (amax > 0.f && amax <= 3.0e38f) {
            int ex;
            frexpf(amax, &ex);
            sh = 14 - ex;
            sh = sh > 100 ? 100 : (sh < -100 ? -100 : sh);
        }
        scale = ldexpf(1.f, sh);
        inv = ldexpf(1.f, -sh);
    }
    for (int k = tid; k < Kp; k += 256) {
        if (DT == DT_I8) {
            int8_t d[NTERM] = {0, 0, 0, 0};
            if (k < K) split_digits((int)sum[k], d);
#pragma unroll
            for (int t = 0; t < NTERM; ++t) ((int8_t *)stripe)[(long)t * Kp + k] = d[t];
        } else {
            uint16_t h[NTERM] = {0, 0, 0, 0};
            if (k < K) {
                float v = __uint_as_float(sum[k]);
                if (DT == DT_BF16) {
                    // three bf16 terms carry the 24 significant bits of the fp32 sum
                    uint32_t t0 = f32_to_bf16_bits(v);
                    float r1 = v - bf16_bits_to_f32(t0);
                    uint32_t t1 = f32_to_bf16_bits(r1);
                    float r2 = r1 - bf16_bits_to_f32(t1);
                    uint32_t t2 = f32_to_bf16_bits(r2);
                    h[0] = (uint16_t)t0; h[1] = (uint16_t)t1; h[2] = (uint16_t)t2;
                } else {
                    // fp16 terms: each remainder is rescaled by 2^11 to stay in the normal range
                    float x = v * scale;
                    uint32_t t0 = f32_to_f16_bits(x);
                    float r1 = (x - f16_bits_to_f32(t0)) * 2048.f;
                    uint32_t t1 = f32_to_f16_bits(r1);
                    float r2 = (r1 - f16_bits_to_f32(t1)) * 2048.f;
                    uint32_t t2 = f32_to_f16_bits(r2);
                    h[0] = (uint16_t)t0; h[1] = (uint16_t)t1; h[2] = (uint16_t)t2;
                }
            }
#pragma unroll
            for (int t = 0; t < NTERM; ++t) ((uint16_t *)stripe)[(long)t * Kp + k] = h[t];
        }
    }
    if (!T::IS_INT && tid == 0) {
        float *w = e.w_a + (long)bz * NTERM;
        if (DT == DT_BF16) { w[0] = 1.f; w[1] = 1.f; w[2] = 1.f; w[3] = 0.f; }
        else { w[0] = inv; w[1] = inv * (1.f / 2048.f); w[2] = inv * (1.f / 4194304.f); w[3] = 0.f; }
        const float ma = __uint_as_float(atomicExch(e.max_acc + (long)bz * 2, 0u));
        e.maxabs[(long)bz * 2] = ma;
        const float mb = e.maxabs[(long)bz * 2 + 1];
        e.tau[bz] = e.tau_override > 0.f ? e.tau_override : (1e-3f * (float)K) * ma * mb;
    }
}

struct EncPlan { int cw_log2, nwin, rpb, nrb; };

// windowed streaming pass over a rows x cols array (B pass, verify)
static EncPlan plan_window(int rows, int cols, int chunk_elems)
{
    EncPlan p;
    const int chunks = (cols + chunk_elems - 1) / chunk_elems;
    // window width (power of two, 8..64 chunk columns): least padding, then widest
    int best_lg = 3;
    long best_waste = -1;
    for (int lg = 3; lg <= 6; ++lg) {
        const int CW = 1 << lg;
        const long waste = (long)((chunks + CW - 1) / CW) * CW - chunks;
        if (best_waste < 0 || waste <= best_waste) { best_waste = waste; best_lg = lg; }
    }
    p.cw_log2 = best_lg;
    const int CW = 1 << best_lg, RL = 256 / CW;
    p.nwin = (chunks + CW - 1) / CW;
    // rows per block: one batch of ENC_UNROLL loads per thread, more when the matrix is tall:
    // fewer blocks mean fewer atomics on the same cache lines
    int rpb = RL * ENC_UNROLL;
    while ((long)p.nwin * ((rows + rpb - 1) / rpb) > 640) rpb *= 2;
    p.rpb = rpb;
    p.nrb = (rows + rpb - 1) / rpb;
    return p;
}

hipError_t launch_encode_b(int dt, const void *B, const Shape &s, const Workspace &w, hipStream_t st)
{
    EncBArgs e;
    e.X = (const uint8_t *)B; e.ld = s.ldb; e.stride = s.sB; e.K = s.K;
    if (s.transB) { e.rows = s.N; e.cols = s.K; e.reduce_rows = 1; }
    else          { e.rows = s.K; e.cols = s.N; e.reduce_rows = 0; }
    EncPlan p = plan_window(e.rows, e.cols, 16 / elem_size(dt));
    e.cw_log2 = p.cw_log2; e.nwin = p.nwin; e.rpb = p.rpb; e.nrb = p.nrb;
    e.acc = w.b_acc; e.acc_stride = w.acc_stride; e.sum = w.b_sum;
    e.max_acc = w.max_acc; e.maxabs = w.maxabs; e.ticket = w.enc_ticket;
    dim3 grid((unsigned)(e.nwin * e.nrb), 1, (unsigned)s.batch);
    switch (dt) {
    case DT_I8:   hipLaunchKernelGGL(encode_b_kernel<DT_I8>, grid, dim3(256), 0, st, e); break;
    case DT_BF16: hipLaunchKernelGGL(encode_b_kernel<DT_BF16>, grid, dim3(256), 0, st, e); break;
    case DT_F16:  hipLaunchKernelGGL(encode_b_kernel<DT_F16>, grid, dim3(256), 0, st, e); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Largest K the A pass handles (8 windows of 64 chunks of 16 bytes, 4 windows for int8).
int encode_a_max_k(int dt) { return dt == DT_I8 ? 4 * 64 * 16 : 8 * 64 * 8; }

template <int DT>
static hipError_t launch_encode_a_t(EncAArgs &e, int batch, hipStream_t st)
{
    constexpr int CE = 16 / Traits<DT>::ES;
    const int CW = 1 << e.cw_log2;
    const size_t smem = ((size_t)e.nwin * CW * CE + 256 * CE) * 4;
    dim3 grid((unsigned)e.nrb, 1, (unsigned)batch);
    if (e.nwin <= 1)      hipLaunchKernelGGL((encode_a_kernel<DT, 1>), grid, dim3(256), smem, st, e);
    else if (e.nwin <= 2) hipLaunchKernelGGL((encode_a_kernel<DT, 2>), grid, dim3(256), smem, st, e);
    else if (e.nwin <= 4) hipLaunchKernelGGL((encode_a_kernel<DT, 4>), grid, dim3(256), smem, st, e);
    else if (DT != DT_I8 && e.nwin <= 8) hipLaunchKernelGGL((encode_a_kernel<DT, (DT == DT_I8 ? 4 : 8)>), grid, dim3(256), smem, st, e);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_encode_a(int dt, const void *A, const Shape &s, const Workspace &w, float tau_override,
                           uint32_t *zero_ptr, size_t zero_words, hipStream_t st)
{
    EncAArgs e;
    const int ce = 16 / elem_size(dt);
    const int chunks = (s.K + ce - 1) / ce;
    const int nw_max = dt == DT_I8 ? 4 : 8;
    // window width: least padding among (CW, nwin) with nwin <= nw_max, then widest
    int best_lg = -1;
    long best_waste = -1;
    for (int lg = 3; lg <= 6; ++lg) {
        const int CW = 1 << lg, nwin = (chunks + CW - 1) / CW;
        if (nwin > nw_max) continue;
        const long waste = (long)nwin * CW - chunks;
        if (best_waste < 0 || waste <= best_waste) { best_waste = waste; best_lg = lg; }
    }
    if (best_lg < 0) return hipErrorInvalidValue;
    e.cw_log2 = best_lg;
    const int CW = 1 << best_lg, RL = 256 / CW;
    e.nwin = (chunks + CW - 1) / CW;
    int nwt = 1;
    while (nwt < e.nwin) nwt *= 2;
    const int UR = nwt >= 8 ? 1 : 8 / nwt;
    int rpb = RL * UR;
    while ((s.M + rpb - 1) / rpb > 512) rpb *= 2;
    e.rpb = rpb;
    e.nrb = (s.M + rpb - 1) / rpb;
    e.A = (const uint8_t *)A; e.lda = s.lda; e.sA = s.sA; e.M = s.M; e.K = s.K; e.Kp = s.Kp;
    e.a_acc = w.a_acc; e.acc_stride = w.acc_stride; e.a_sum = w.a_sum; e.b_sum = w.b_sum;
    e.rc_pred = w.rc_pred; e.stripe = w.stripe_a; e.w_a = w.w_a;
    e.max_acc = w.max_acc; e.maxabs = w.maxabs; e.tau = w.tau; e.ticket = w.enc_ticket;
    e.tau_override = tau_override; e.zero_ptr = zero_ptr; e.zero_words = zero_words;
    e.s_pred = w.s_pred;
    switch (dt) {
    case DT_I8:   return launch_encode_a_t<DT_I8>(e, s.batch, st);
    case DT_BF16: return launch_encode_a_t<DT_BF16>(e, s.batch, st);
    case DT_F16:  return launch_encode_a_t<DT_F16>(e, s.batch, st);
    }
    return hipErrorInvalidValue;
}

// ===================================================================== compare
// Flags from observed sums against the predictions the last abft_gemm left in the context
// (Sec. III-B.1 item (2): equality for fixed point, tolerance for floating point).  Used by
// abft_verify; abft_gemm does the same comparison in the tail of the GEMM kernel.
struct CmpArgs {
    const uint32_t *cc_pred, *rc_pred;
    const uint32_t *cc_obs, *rc_obs;
    const float *tau;
    uint8_t *row_flag, *col_flag;
    uint32_t *counts;
    uint32_t *ticket;     // [3]: ticket, flagged rows, flagged cols (self-cleaning)
    const uint32_t *fix_count;   // non-null after a correction: [0] tiles listed, [1] overflow
    int M, N, batch;
};

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

template <bool IS_INT>
__global__ __launch_bounds__(256) void compare_kernel(CmpArgs a)
{
    __shared__ int is_last;
    const int bz = blockIdx.z, tid = threadIdx.x;
    const int idx = blockIdx.x * 256 + tid;
    const int M = a.M, N = a.N;
    const float tol = IS_INT ? 0.f : a.tau[bz];
    bool frow = false, fcol = false;
    if (idx < M) {
        frow = mismatch<IS_INT>(a.rc_obs[(long)bz * M + idx], a.rc_pred[(long)bz * M + idx], tol);
        a.row_flag[(long)bz * M + idx] = frow ? 1 : 0;
    } else if (idx < M + N) {
        const int j = idx - M;
        fcol = mismatch<IS_INT>(a.cc_obs[(long)bz * N + j], a.cc_pred[(long)bz * N + j], tol);
        a.col_flag[(long)bz * N + j] = fcol ? 1 : 0;
    }
    const unsigned nr = __syncthreads_count(frow);
    const unsigned nc = __syncthreads_count(fcol);
    if (tid == 0) {
        if (nr) atomicAdd(a.ticket + 1, nr);
        if (nc) atomicAdd(a.ticket + 2, nc);
        unsigned total = gridDim.x * gridDim.z;
        unsigned t = atomicAdd(a.ticket, 1u);
        is_last = (t == total - 1);
    }
    __syncthreads();
    if (is_last && tid == 0) {
        uint32_t r = atomicExch(a.ticket + 1, 0u), c = atomicExch(a.ticket + 2, 0u);
        atomicExch(a.ticket, 0u);
        const uint32_t before = a.counts[2];
        a.counts[0] = r;
        a.counts[1] = c;
        if (a.fix_count) {
            const uint32_t tiles = a.fix_count[0];
            a.counts[2] = a.fix_count[1] ? 3u : status_of(r, c);
            a.counts[3] = tiles > (uint32_t)MAX_FIX_TILES ? (uint32_t)MAX_FIX_TILES : tiles;
            a.counts[4] = before;
        } else {
            a.counts[2] = status_of(r, c);
            a.counts[3] = 0u;
            a.counts[4] = status_of(r, c);
        }
    }
}

hipError_t launch_compare(int dt, const Shape &s, const Workspace &w, const Verdict &v, bool after_fix,
                          hipStream_t st)
{
    CmpArgs a;
    a.fix_count = after_fix ? w.fix_count : nullptr;
    a.cc_pred = w.cc_pred; a.rc_pred = w.rc_pred;
    a.cc_obs = w.cc_vobs; a.rc_obs = w.rc_vobs;
    a.tau = w.tau;
    a.row_flag = v.row_flag; a.col_flag = v.col_flag; a.counts = v.counts;
    a.ticket = w.cmp_ticket;
    a.M = s.M; a.N = s.N; a.batch = s.batch;
    dim3 grid((unsigned)((s.M + s.N + 255) / 256), 1, (unsigned)s.batch);
    if (dt == DT_I8) hipLaunchKernelGGL(compare_kernel<true>, grid, dim3(256), 0, st, a);
    else             hipLaunchKernelGGL(compare_kernel<false>, grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

// ====================================================================== verify
// Column and row sums of the stored C (streaming reduction, HBM-bound).
struct VerArgs {
    const uint8_t *C;
    long ldc, sC;
    int M, N;
    int cw_log2, rpb, nwin, nrb;
    uint32_t *cc_vobs, *rc_vobs;
};

// value q of a 16-byte chunk of stored C
template <int DT> __device__ __forceinline__ typename Traits<DT>::acc_t out_elem(const i32x4 &v, int q)
{
    if (DT == DT_I8) return from_word<typename Traits<DT>::acc_t>((uint32_t)v[q]);
    uint32_t w = (uint32_t)v[q >> 1];
    uint32_t h = (q & 1) ? (w >> 16) : (w & 0xFFFFu);
    if (DT == DT_BF16) return from_word<typename Traits<DT>::acc_t>(h << 16);
    return from_word<typename Traits<DT>::acc_t>(__float_as_uint(f16_bits_to_f32(h)));
}

template <int DT>
__global__ __launch_bounds__(256) void verify_kernel(VerArgs a)
{
    using T = Traits<DT>;
    typedef typename T::acc_t acc_t;
    constexpr int OS = T::OS, CE = 16 / OS;
    __shared__ acc_t red[256 * CE];
    const int tid = threadIdx.x, bz = blockIdx.z;
    const int win = blockIdx.x % a.nwin, rb = blockIdx.x / a.nwin;
    const int CW = 1 << a.cw_log2, RL = 256 >> a.cw_log2;
    const int cx = tid & (CW - 1), ry = tid >> a.cw_log2;
    const int col0 = (win * CW + cx) * CE;
    const bool colok = col0 < a.N;
    const int nvalid = a.N - col0;
    const uint8_t *Cb = a.C + (long)bz * a.sC * OS;
    const int rbeg = rb * a.rpb, rend = min(rbeg + a.rpb, a.M);
    const int iters = (a.rpb + RL * ENC_UNROLL - 1) / (RL * ENC_UNROLL);
    acc_t colacc[CE];
#pragma unroll
    for (int q = 0; q < CE; ++q) colacc[q] = T::zero();
    for (int it = 0; it < iters; ++it) {
        i32x4 v[ENC_UNROLL];
#pragma unroll
        for (int u = 0; u < ENC_UNROLL; ++u) {
            const int r = rbeg + ry + (it * ENC_UNROLL + u) * RL;
            v[u] = i32x4{0, 0, 0, 0};
            if (colok && r < rend) v[u] = *reinterpret_cast<const i32x4 *>(Cb + ((long)r * a.ldc + col0) * OS);
        }
#pragma unroll
        for (int u = 0; u < ENC_UNROLL; ++u) {
            const int r = rbeg + ry + (it * ENC_UNROLL + u) * RL;
            acc_t s = T::zero();
            if (colok && r < rend) {
#pragma unroll
                for (int q = 0; q < CE; ++q) {
                    if (q < nvalid) {
                        acc_t x = out_elem<DT>(v[u], q);
                        colacc[q] = add_t(colacc[q], x);
                        s = add_t(s, x);
                    }
                }
            }
            for (int o = 1; o < CW; o <<= 1) s = add_t(s, __shfl_xor(s, o));
            if (cx == 0 && r < rend) atomic_add_word(a.rc_vobs + (long)bz * a.M + r, s);
        }
    }
#pragma unroll
    for (int q = 0; q < CE; ++q) red[(ry * CW + cx) * CE + q] = colacc[q];
    __syncthreads();
    for (int c = tid; c < CW * CE; c += 256) {
        const int col = win * CW * CE + c;
        if (col < a.N) {
            acc_t t = red[c];
            for (int y = 1; y < RL; ++y) t = add_t(t, red[y * CW * CE + c]);
            atomic_add_word(a.cc_vobs + (long)bz * a.N + col, t);
        }
    }
}

hipError_t launch_verify_sums(int dt, const void *C, const Shape &s, const Workspace &w, hipStream_t st)
{
    VerArgs a;
    a.C = (const uint8_t *)C; a.ldc = s.ldc; a.sC = s.sC; a.M = s.M; a.N = s.N;
    a.cc_vobs = w.cc_vobs; a.rc_vobs = w.rc_vobs;
    EncPlan plan = plan_window(s.M, s.N, 16 / out_size(dt));
    a.cw_log2 = plan.cw_log2; a.nwin = plan.nwin; a.rpb = plan.rpb; a.nrb = plan.nrb;
    dim3 grid((unsigned)(a.nwin * a.nrb), 1, (unsigned)s.batch);
    switch (dt) {
    case DT_I8:   hipLaunchKernelGGL(verify_kernel<DT_I8>, grid, dim3(256), 0, st, a); break;
    case DT_BF16: hipLaunchKernelGGL(verify_kernel<DT_BF16>, grid, dim3(256), 0, st, a); break;
    case DT_F16:  hipLaunchKernelGGL(verify_kernel<DT_F16>, grid, dim3(256), 0, st, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ===================================================================== correct
// Step 1: list flagged rows / columns per batch item, map their cross product to CT x CT tiles.
struct LocArgs {
    const uint8_t *row_flag, *col_flag;
    int M, N;
    int32_t *fix_tiles;
    uint32_t *fix_count;
};

__global__ __launch_bounds__(256) void locate_kernel(LocArgs a)
{
    __shared__ int rows[MAX_LIST], cols[MAX_LIST];
    __shared__ int nr, nc;
    const int bz = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) { nr = 0; nc = 0; }
    __syncthreads();
    for (int i = tid; i < a.M; i += 256)
        if (a.row_flag[(long)bz * a.M + i]) {
            int p = atomicAdd(&nr, 1);
            if (p < MAX_LIST) rows[p] = i / CT;
        }
    for (int j = tid; j < a.N; j += 256)
        if (a.col_flag[(long)bz * a.N + j]) {
            int p = atomicAdd(&nc, 1);
            if (p < MAX_LIST) cols[p] = j / CT;
        }
    __syncthreads();
    if (tid != 0) return;
    if (nr == 0 || nc == 0) return;                     // clean, or one-sided: nothing to recompute
    bool overflow = nr > MAX_LIST || nc > MAX_LIST;
    int r = nr > MAX_LIST ? MAX_LIST : nr, c = nc > MAX_LIST ? MAX_LIST : nc;
    // unique tile rows / tile cols (lists are short under the single-error model)
    int ur = 0, uc = 0;
    for (int i = 0; i < r; ++i) {
        bool dup = false;
        for (int q = 0; q < ur; ++q) dup |= (rows[q] == rows[i]);
        if (!dup) rows[ur++] = rows[i];
    }
    for (int j = 0; j < c; ++j) {
        bool dup = false;
        for (int q = 0; q < uc; ++q) dup |= (cols[q] == cols[j]);
        if (!dup) cols[uc++] = cols[j];
    }
    for (int i = 0; i < ur; ++i)
        for (int j = 0; j < uc; ++j) {
            unsigned p = atomicAdd(a.fix_count, 1u);
            if (p < (unsigned)MAX_FIX_TILES) {
                a.fix_tiles[3 * p + 0] = bz;
                a.fix_tiles[3 * p + 1] = rows[i];
                a.fix_tiles[3 * p + 2] = cols[j];
            } else overflow = true;
        }
    if (overflow) atomicExch(a.fix_count + 1, 1u);
}

// Step 2: one wave recomputes one CT x CT tile of C over the whole K, with the same MFMA
// instruction and the same ascending-k order as the GEMM kernel.
struct FixArgs {
    const uint8_t *A, *B;
    uint8_t *C;
    int M, N, K, transB;
    long lda, ldb, ldc, sA, sB, sC;
    const int32_t *fix_tiles;
    const uint32_t *fix_count;
};

template <int DT>
__global__ __launch_bounds__(64) void recompute_kernel(FixArgs a)
{
    using T = Traits<DT>;
    typedef typename T::accv_t accv_t;
    constexpr int ES = T::ES, CE = 16 / ES;
    unsigned n = a.fix_count[0];
    if (n > (unsigned)MAX_FIX_TILES) n = MAX_FIX_TILES;
    if (blockIdx.x >= n) return;
    const int bz = a.fix_tiles[3 * blockIdx.x], tr = a.fix_tiles[3 * blockIdx.x + 1],
              tc = a.fix_tiles[3 * blockIdx.x + 2];
    const int lane = threadIdx.x, l32 = lane & 31, lh = lane >> 5;
    const int row = tr * CT + l32, col = tc * CT + l32;
    const uint8_t *Ab = a.A + (long)bz * a.sA * ES, *Bb = a.B + (long)bz * a.sB * ES;
    const int K = a.K;
    accv_t acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = T::zero();
    const int steps = (K + 2 * CE - 1) / (2 * CE);
    constexpr int UB = 8;                       // k-steps whose operands are in flight together
    auto load_a = [&](int ks) __attribute__((always_inline)) -> i32x4 {
        const int kb = ks * 2 * CE + lh * CE;
        i32x4 av = {0, 0, 0, 0};
        if (ks < steps && row < a.M && kb < K) {
            av = *reinterpret_cast<const i32x4 *>(Ab + ((long)row * a.lda + kb) * ES);
            if (kb + CE > K) av = mask_chunk(av, (K - kb) * ES);
        }
        return av;
    };
    auto load_b = [&](int ks) __attribute__((always_inline)) -> i32x4 {
        const int kb = ks * 2 * CE + lh * CE;
        i32x4 bv = {0, 0, 0, 0};
        if (ks < steps && col < a.N && kb < K) {
            if (a.transB) {
                bv = *reinterpret_cast<const i32x4 *>(Bb + ((long)col * a.ldb + kb) * ES);
                if (kb + CE > K) bv = mask_chunk(bv, (K - kb) * ES);
            } else {
                // B stored K x N: gather one column element per k
                uint32_t wds[4] = {0, 0, 0, 0};
#pragma unroll
                for (int q = 0; q < CE; ++q) {
                    int k = kb + q;
                    if (k < K) {
                        if (ES == 2) {
                            uint32_t h = *reinterpret_cast<const uint16_t *>(Bb + ((long)k * a.ldb + col) * 2);
                            wds[q >> 1] |= h << (16 * (q & 1));
                        } else {
                            uint32_t h = *(Bb + ((long)k * a.ldb + col));
                            wds[q >> 2] |= h << (8 * (q & 3));
                        }
                    }
                }
                bv[0] = (int)wds[0]; bv[1] = (int)wds[1]; bv[2] = (int)wds[2]; bv[3] = (int)wds[3];
            }
        }
        return bv;
    };
    for (int ks0 = 0; ks0 < steps; ks0 += UB) {
        i32x4 av[UB], bv[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) { av[u] = load_a(ks0 + u); bv[u] = load_b(ks0 + u); }
#pragma unroll
        for (int u = 0; u < UB; ++u)
            if (ks0 + u < steps) acc = T::mfma(bv[u], av[u], acc);   // B first: lane = row of C, registers = columns
    }
    uint8_t *Cb = a.C + (long)bz * a.sC * T::OS;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int gc = tc * CT + 8 * (i >> 2) + 4 * lh + (i & 3);
        if (row < a.M && gc < a.N) T::store_c(Cb, (long)row * a.ldc + gc, acc[i]);
    }
}

hipError_t launch_correct(int dt, const void *A, const void *B, void *C, const Shape &s,
                          const Workspace &w, const Verdict &v, hipStream_t st)
{
    hipError_t e = launch_zero(w.fix_count, 2, st);
    if (e != hipSuccess) return e;
    LocArgs l;
    l.row_flag = v.row_flag; l.col_flag = v.col_flag; l.M = s.M; l.N = s.N;
    l.fix_tiles = w.fix_tiles; l.fix_count = w.fix_count;
    hipLaunchKernelGGL(locate_kernel, dim3((unsigned)s.batch), dim3(256), 0, st, l);
    if ((e = hipGetLastError()) != hipSuccess) return e;

    FixArgs f;
    f.A = (const uint8_t *)A; f.B = (const uint8_t *)B; f.C = (uint8_t *)C;
    f.M = s.M; f.N = s.N; f.K = s.K; f.transB = s.transB;
    f.lda = s.lda; f.ldb = s.ldb; f.ldc = s.ldc; f.sA = s.sA; f.sB = s.sB; f.sC = s.sC;
    f.fix_tiles = w.fix_tiles; f.fix_count = w.fix_count;
    switch (dt) {
    case DT_I8:   hipLaunchKernelGGL(recompute_kernel<DT_I8>, dim3(MAX_FIX_TILES), dim3(64), 0, st, f); break;
    case DT_BF16: hipLaunchKernelGGL(recompute_kernel<DT_BF16>, dim3(MAX_FIX_TILES), dim3(64), 0, st, f); break;
    case DT_F16:  hipLaunchKernelGGL(recompute_kernel<DT_F16>, dim3(MAX_FIX_TILES), dim3(64), 0, st, f); break;
    default: return hipErrorInvalidValue;
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // re-check: the stored C is re-summed as a whole (a streaming pass at HBM speed is cheaper
    // than strided column walks over the touched tiles) and compared with the predictions
    if ((e = launch_zero(w.cc_vobs, (size_t)s.batch * ((size_t)s.M + s.N), st)) != hipSuccess) return e;
    if ((e = launch_verify_sums(dt, C, s, w, st)) != hipSuccess) return e;
    return launch_compare(dt, s, w, v, true, st);
}

// ====================================================================== inject
__global__ void flip_kernel(uint8_t *C, long idx, int os, int bit)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    if (os == 4) {
        uint32_t *p = reinterpret_cast<uint32_t *>(C) + idx;
        *p ^= (1u << bit);
    } else {
        uint16_t *p = reinterpret_cast<uint16_t *>(C) + idx;
        *p = (uint16_t)(*p ^ (uint16_t)(1u << bit));
    }
}

hipError_t launch_flip(void *C, int dt, const Shape &s, long batch_idx, long row, long col, int bit,
                       hipStream_t st)
{
    long idx = batch_idx * s.sC + row * s.ldc + col;
    hipLaunchKernelGGL(flip_kernel, dim3(1), dim3(64), 0, st, (uint8_t *)C, idx, out_size(dt), bit);
    return hipGetLastError();
}

}  // namespace abft
