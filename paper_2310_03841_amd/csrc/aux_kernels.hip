// Kernels around the protected GEMM: the pass over B (its checksum vector), finish (column
// prediction from the sums the GEMM collected, compare, flags), verify (re-sum stored C),
// correct (localise, recompute tiles, re-check) and the bit-flip test hook.
//
// Paper references: the two input-side vectors and the comparison with the
// output sums are the checksum scheme of Sec. III-B.1 ("Checksums"); equality
// for integers and a tolerance for floating point follow item (2) there; the
// tile recompute is the replay correction of Sec. III-B.3 at tile granularity;
// the flip is the fault model of Sec. II-A / III-A.
#include <mutex>

#include "abft_device.h"

namespace abft {

// ======================================================================== per-device launch state
static std::mutex g_launch_lock;

hipError_t ensure_max_lds(const void *kernel, int bytes)
{
    struct Done { const void *kernel; int device; };
    static Done done[512];
    static int n_done = 0;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> hold(g_launch_lock);
    for (int i = 0; i < n_done; ++i)
        if (done[i].kernel == kernel && done[i].device == dev) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    if (n_done < 512) done[n_done++] = Done{kernel, dev};
    return hipSuccess;
}

int device_cu_count(hipError_t *err)
{
    static int cus[64];
    int dev = 0, n = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= 64)) e = hipErrorInvalidDevice;
    if (e == hipSuccess) {
        std::lock_guard<std::mutex> hold(g_launch_lock);
        if (cus[dev] == 0) {
            e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
            if (e == hipSuccess) cus[dev] = n > 0 ? n : 256;
        }
        n = cus[dev];
    }
    if (err) *err = e;
    return e == hipSuccess ? n : 0;
}

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
// max|A|, max|B| for the tolerance and the row checksum prediction rc_pred = A b.  Everything
// that reads A is done by the GEMM kernel on the slabs it holds in LDS (gemm_apass.h); what is
// left here is the pass over B, which must be complete before that (A b needs all of b).  For a
// weight it is done once, offline (remark (2) of the same paragraph).
#ifndef ENC_UNROLL_N
#define ENC_UNROLL_N 8
#endif
constexpr int ENC_UNROLL = ENC_UNROLL_N;     // independent 16-byte loads in flight per thread (B pass)
#ifndef ENC_BATCHES
#define ENC_BATCHES 2
#endif
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
    uint32_t *sum;        // [batch][K]  accumulated with atomics: zero before the launch
    uint32_t *max_acc;    // [batch]     max|B| as float bits, atomic max: zero before the launch
    uint32_t *zero_ptr;   // region every block helps to clear (the next kernel's atomics start at zero)
    size_t zero_words;
};

template <int DT>
__global__ __launch_bounds__(256) void encode_b_kernel(EncBArgs e)
{
    using T = Traits<DT>;
    typedef typename T::acc_t acc_t;
    constexpr int ES = T::ES, CE = 16 / ES;
    __shared__ acc_t red[256 * CE];

    const int tid = threadIdx.x, bz = blockIdx.z;
    {
        const size_t nb = (size_t)gridDim.x * gridDim.z;
        const size_t bid = blockIdx.x + (size_t)gridDim.x * blockIdx.z;
        for (size_t i = bid * 256 + tid; i < e.zero_words; i += nb * 256) e.zero_ptr[i] = 0u;
    }
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
                s = seg_sum(s, CW);
                if (cx == 0 && r < rend) atomic_add_word(e.sum + (long)bz * e.K + r, s);
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
                atomic_add_word(e.sum + (long)bz * e.K + col, t);
            }
        }
    }
    if (!T::IS_INT) {
        mx = wave_max(mx);
        if ((tid & 63) == 0 && mx > 0.f) atomicMax(e.max_acc + bz, __float_as_uint(mx));
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
    // rows per block: ENC_BATCHES batches of ENC_UNROLL loads per thread, more when the matrix is
    // tall: atomics that hit one cache line are served one after the other (tens of nanoseconds
    // each), so fewer row blocks mean less waiting at the end of the pass
    int rpb = RL * ENC_UNROLL * ENC_BATCHES;
    while ((long)p.nwin * ((rows + rpb - 1) / rpb) > 640) rpb *= 2;
    p.rpb = rpb;
    p.nrb = (rows + rpb - 1) / rpb;
    return p;
}

hipError_t launch_encode_b(int dt, const void *B, const Shape &s, const Workspace &w, uint32_t *zero_ptr,
                           size_t zero_words, hipStream_t st)
{
    EncBArgs e;
    e.X = (const uint8_t *)B; e.ld = s.ldb; e.stride = s.sB; e.K = s.K;
    if (s.transB) { e.rows = s.N; e.cols = s.K; e.reduce_rows = 1; }
    else          { e.rows = s.K; e.cols = s.N; e.reduce_rows = 0; }
    EncPlan p = plan_window(e.rows, e.cols, 16 / elem_size(dt));
    e.cw_log2 = p.cw_log2; e.nwin = p.nwin; e.rpb = p.rpb; e.nrb = p.nrb;
    e.sum = w.b_sum; e.max_acc = w.b_max;
    e.zero_ptr = zero_ptr; e.zero_words = zero_ptr ? zero_words : 0;
    dim3 grid((unsigned)(e.nwin * e.nrb), 1, (unsigned)s.batch);
    switch (dt) {
    case DT_I8:   hipLaunchKernelGGL(encode_b_kernel<DT_I8>, grid, dim3(256), 0, st, e); break;
    case DT_BF16: hipLaunchKernelGGL(encode_b_kernel<DT_BF16>, grid, dim3(256), 0, st, e); break;
    case DT_F16:  hipLaunchKernelGGL(encode_b_kernel<DT_F16>, grid, dim3(256), 0, st, e); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Largest K of a protected GEMM: the column sums of A's slabs wait in LDS (4 bytes per column
// of K) next to the operand buffers until the epilogue.
int protect_max_k(int dt) { (void)dt; return 4096; }

// ===================================================================== compare
// Flags from observed sums against the predictions the last abft_gemm left in the context
// (Sec. III-B.1 item (2): equality for fixed point, tolerance for floating point).  Used by
// abft_verify and abft_correct; abft_gemm compares in its finish kernel.
struct CmpArgs {
    const uint32_t *cc_pred, *rc_pred;
    const uint32_t *cc_obs, *rc_obs;
    const float *tau;
    float tau_override;   // > 0: use this tolerance instead of tau[]
    float tau_override_cols;   // > 0: tolerance of the column check
    uint8_t *row_flag, *col_flag;
    uint32_t *counts;
    uint32_t *ticket;     // [3]: ticket, flagged rows, flagged cols (self-cleaning)
    uint32_t *fix_count;  // non-null after a correction: [0] tiles listed, [1] overflow (cleared after use)
    const int32_t *fix_tiles;          // after a correction: the tiles it recomputed
    uint32_t *cc_sto, *rc_sto;         // non-null: stored-side sums of the GEMM (floating point)
    uint32_t *zero_ptr;   // region every block helps to clear: the re-summing region not in use,
    size_t zero_words;    // so that the next re-sum finds it clean
    int M, N, batch;
    const uint32_t *gate; // non-null: if *gate == 0 (no tile was listed for recomputation) the kernel
                          // leaves flags and counts as the check before it wrote them
};

template <bool IS_INT>
__global__ __launch_bounds__(256) void compare_kernel(CmpArgs a)
{
    __shared__ int is_last;
    const int bz = blockIdx.z, tid = threadIdx.x;
    const int idx = blockIdx.x * 256 + tid;
    const int M = a.M, N = a.N;
    {
        const size_t nb = (size_t)gridDim.x * gridDim.z;
        const size_t bid = blockIdx.x + (size_t)gridDim.x * blockIdx.z;
        for (size_t i = bid * 256 + tid; i < a.zero_words; i += nb * 256) a.zero_ptr[i] = 0u;
    }
    if (a.gate && *a.gate == 0u) return;           // uniform over the grid: nobody touches the ticket
    const float tol = IS_INT ? 0.f : (a.tau_override > 0.f ? a.tau_override : a.tau[bz]);
    const float tol_c = (!IS_INT && a.tau_override_cols > 0.f) ? a.tau_override_cols : tol;
    bool frow = false, fcol = false;
    if (!IS_INT && a.fix_count && a.rc_sto && idx < M + N) {
        // After a correction the stored-side sums of the GEMM no longer describe the rows and
        // columns of the recomputed tiles: if the fault was already in the accumulators when the
        // epilogue summed them, those sums contain it, and the repaired values do not.  The fresh
        // re-sum of the repaired rows and columns takes their place.
        unsigned n = a.fix_count[0];
        if (n > (unsigned)MAX_FIX_TILES) n = MAX_FIX_TILES;
        const int mine = (idx < M ? idx : idx - M) / CT, which = idx < M ? 1 : 2;
        bool touched = false;
        for (unsigned t = 0; t < n; ++t)
            touched = touched || (a.fix_tiles[3 * t] == bz && a.fix_tiles[3 * t + which] == mine);
        if (touched) {
            if (idx < M) a.rc_sto[(long)bz * M + idx] = a.rc_obs[(long)bz * M + idx];
            else a.cc_sto[(long)bz * N + idx - M] = a.cc_obs[(long)bz * N + idx - M];
        }
    }
    if (idx < M) {
        frow = mismatch<IS_INT>(a.rc_obs[(long)bz * M + idx], a.rc_pred[(long)bz * M + idx], tol);
        if (!IS_INT && a.rc_sto)
            frow = frow || mismatch<false>(a.rc_obs[(long)bz * M + idx], a.rc_sto[(long)bz * M + idx], STO_TOL_FACTOR * tol);
        a.row_flag[(long)bz * M + idx] = frow ? 1 : 0;
    } else if (idx < M + N) {
        const int j = idx - M;
        fcol = mismatch<IS_INT>(a.cc_obs[(long)bz * N + j], a.cc_pred[(long)bz * N + j], tol_c);
        if (!IS_INT && a.cc_sto)
            fcol = fcol || mismatch<false>(a.cc_obs[(long)bz * N + j], a.cc_sto[(long)bz * N + j], STO_TOL_FACTOR * tol_c);
        a.col_flag[(long)bz * N + j] = fcol ? 1 : 0;
    }
    const unsigned nr = __syncthreads_count(frow);
    const unsigned nc = __syncthreads_count(fcol);
    if (tid == 0) {
        if (nr | nc) {
            // rare: the counts must be at the coherence point before this block's ticket is, so
            // fetch their old values and wait for them
            unsigned o1 = 0, o2 = 0;
            if (nr) o1 = atomicAdd(a.ticket + 1, nr);
            if (nc) o2 = atomicAdd(a.ticket + 2, nc);
            asm volatile("s_waitcnt vmcnt(0)" :: "v"(o1), "v"(o2) : "memory");
        }
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
            // the list is consumed: the next correction starts from an empty one
            const uint32_t tiles = atomicExch(a.fix_count, 0u);
            a.counts[2] = atomicExch(a.fix_count + 1, 0u) ? 3u : status_of(r, c);
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
                          bool with_sto, uint32_t *zero_ptr, size_t zero_words, hipStream_t st, bool gated)
{
    CmpArgs a;
    a.gate = gated ? w.fix_count : nullptr;
    a.zero_ptr = zero_ptr; a.zero_words = zero_ptr ? zero_words : 0;
    a.cc_sto = (with_sto && dt != DT_I8) ? w.cc_sto : nullptr;
    a.rc_sto = a.cc_sto ? w.rc_sto : nullptr;
    a.fix_count = after_fix ? w.fix_count : nullptr;
    a.fix_tiles = w.fix_tiles;
    a.cc_pred = w.cc_pred; a.rc_pred = w.rc_pred;
    a.cc_obs = w.cc_vobs; a.rc_obs = w.rc_vobs;
    a.tau = w.tau; a.tau_override = v.tau_override; a.tau_override_cols = v.tau_override_cols;
    a.row_flag = v.row_flag; a.col_flag = v.col_flag; a.counts = v.counts;
    a.ticket = w.cmp_ticket;
    a.M = s.M; a.N = s.N; a.batch = s.batch;
    dim3 grid((unsigned)((s.M + s.N + 255) / 256), 1, (unsigned)s.batch);
    if (dt == DT_I8) hipLaunchKernelGGL(compare_kernel<true>, grid, dim3(256), 0, st, a);
    else             hipLaunchKernelGGL(compare_kernel<false>, grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

// ====================================================================== finish
// Runs after the protected GEMM, when its atomics have completed a = e^T A, rc_pred = A b,
// max|A| and the observed sums.  Column blocks form the column checksum prediction
// cc_pred = a B (Sec. III-B.1: the product of the input-side checksum with the weight), a
// matrix-vector product bound by one read of B, and compare it with cc_obs; row blocks compare
// rc_pred with rc_obs; the last block to finish writes the counts and the status.
struct FinArgs {
    const uint8_t *B;
    long ldb, sB;
    int transB;
    int M, N, K;
    const uint32_t *a_sum, *b_sum, *cc_obs, *rc_obs, *a_max;
    uint32_t *rc_pred;    // A b from the GEMM; with a bias the finish kernel adds sum(bias) in place
    const uint32_t *bias; // layer bias [N] or null: cc_pred gains M bias[n], rc_pred sum(bias), a.b M sum(bias)
    uint32_t *cc_pred, *s_pred;
    float *maxabs, *tau;
    float tau_override, tau_override_cols;
    uint8_t *row_flag, *col_flag;
    uint32_t *counts;
    uint32_t *ticket;     // [3]: ticket, flagged rows, flagged cols (self-cleaning)
    uint32_t *group_ticket;   // [FIN_MAX_BLOCKS / FIN_GROUP] first-level tickets (self-cleaning)
    int batch;
    int lpr;              // B stored N x K: lanes along one row of B (8, 16, 32 or 64)
    int ksplit;           // 1, or 4 (deep K, lpr = 64): the four waves share four rows of B, a quarter of K each
    int col_blocks;       // units [0, col_blocks) of a batch item take columns, the rest rows
    uint32_t *zero_ptr;   // region every block helps to clear: what the previous protected GEMM of this
    size_t zero_words;    // context accumulated into, so that the next one finds it clean
    const uint32_t *b_max;   // max|B| of the b in use, float bits [batch]
    uint32_t *zero2_ptr;  // second region to clear: the b slot the next pass over B will accumulate into
    size_t zero2_words;
};

// Sum of the layer bias over its N entries, by the whole block (every thread gets the total).
template <typename acc_t>
__device__ __forceinline__ acc_t block_bias_sum(const uint32_t *bias, int N, acc_t *red4)
{
    acc_t v = acc_t(0);
    for (int n = threadIdx.x; n < N; n += 256) v = add_t(v, from_word<acc_t>(bias[n]));
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red4[threadIdx.x >> 6] = v;
    __syncthreads();
    return add_t(add_t(red4[0], red4[1]), add_t(red4[2], red4[3]));
}

constexpr int FIN_KY = 8;          // k lanes of a column block over a B stored K x N
constexpr int FIN_MAX_BLOCKS = 1024;
constexpr int FIN_GROUP = 16;          // blocks per first-level ticket

// Work is cut into units: (batch item, block of columns) and (batch item, block of 256 rows).
// A block takes units blockIdx.x, blockIdx.x + gridDim.x, ...: many small batch items (attention
// heads) then cost few blocks, and few blocks matter because each ends on the same ticket.
template <int DT>
__global__ __launch_bounds__(256) void finish_kernel(FinArgs f)
{
    using T = Traits<DT>;
    typedef typename T::acc_t acc_t;
    constexpr int ES = T::ES, CE = 16 / ES;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    __shared__ acc_t wred[4];
    __shared__ acc_t kpart[4][4];
    __shared__ unsigned wcnt[4][2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int M = f.M, N = f.N, K = f.K;
    {
        const size_t nb = gridDim.x;
        for (size_t i = (size_t)blockIdx.x * 256 + tid; i < f.zero_words; i += nb * 256) f.zero_ptr[i] = 0u;
        for (size_t i = (size_t)blockIdx.x * 256 + tid; i < f.zero2_words; i += nb * 256) f.zero2_ptr[i] = 0u;
    }
    const int row_blocks = (M + 255) / 256;
    const int upi = f.col_blocks + row_blocks;                 // units per batch item
    const int units = upi * f.batch;                           // fits: checked by the launcher
    unsigned nr_w = 0, nc_w = 0;                               // flagged rows / columns seen by this wave
    acc_t sb = T::zero();                                      // sum of the bias
    if (f.bias) sb = block_bias_sum<acc_t>(f.bias, N, wred);

    for (int u = blockIdx.x; u < units; u += gridDim.x) {
        const int bz = u / upi, blk = u - bz * upi;
        const uint8_t *Bb = f.B + (long)bz * f.sB * ES;
        const uint32_t *asum = f.a_sum + (long)bz * K;
        float tol = 0.f;
        if (!T::IS_INT) {
            const float ma = __uint_as_float(f.a_max[bz]), mb = __uint_as_float(f.b_max[bz]);
            tol = f.tau_override > 0.f ? f.tau_override : (1e-3f * (float)K) * ma * mb;
            if (blk == 0 && tid == 0) {
                f.maxabs[(long)bz * 2] = ma;
                f.maxabs[(long)bz * 2 + 1] = mb;
                f.tau[bz] = tol;
            }
        }
        if (blk < f.col_blocks) {
            if (f.transB) {
                // B stored N x K: lpr lanes run along a row of B (K), a wave takes 64 / lpr rows at
                // a time, four times.  The matching values of a come straight from memory, in
                // flight together with B.
                const int nch = (K + CE - 1) / CE;
                const int lpr = f.lpr, rpw = 64 / lpr;
                const int sub = lane / lpr, lc = lane % lpr;
                const bool split = f.ksplit == 4;
                // row of pass 0; pass j: + j * rpw.  Deep K: every wave takes the block's four rows
                // and every fourth run of 64 chunks.
                const int nb = split ? blk * 4 : blk * (16 * rpw) + wave * 4 * rpw + sub;
                acc_t dot[4] = {T::zero(), T::zero(), T::zero(), T::zero()};
                for (int ch = split ? lane + 64 * wave : lc; ch < nch; ch += split ? 256 : lpr) {
                    i32x4 v[4], aw[CE / 4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int n = nb + j * rpw;
                        v[j] = i32x4{0, 0, 0, 0};
                        if (n < N) v[j] = *reinterpret_cast<const i32x4 *>(Bb + ((long)n * f.ldb + ch * CE) * ES);
                    }
                    const int left = K - ch * CE;                       // >= 1
                    if (left >= CE) {
#pragma unroll
                        for (int q4 = 0; q4 < CE / 4; ++q4) {
                            // dword-aligned reads (the batch offset need not be a multiple of four words)
                            const uint32_t *ap = asum + ch * CE + 4 * q4;
                            aw[q4] = i32x4{(int)ap[0], (int)ap[1], (int)ap[2], (int)ap[3]};
                        }
                    } else {
#pragma unroll
                        for (int q4 = 0; q4 < CE / 4; ++q4)
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                aw[q4][e] = (4 * q4 + e < left) ? (int)asum[ch * CE + 4 * q4 + e] : 0;
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        i32x4 w = v[j];
                        if (left < CE) w = mask_chunk(w, left * ES);
#pragma unroll
                        for (int q = 0; q < CE; ++q)
                            dot[j] = add_t(dot[j], mul_t(T::elem(w, q), from_word<acc_t>((uint32_t)aw[q >> 2][q & 3])));
                    }
                }
                if (lpr == 64) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) dot[j] = wave_sum(dot[j]);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) dot[j] = seg_sum(dot[j], lpr);
                }
                if (split) {
                    __syncthreads();                                    // previous unit done with kpart
                    if (lane == 0) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) kpart[wave][j] = dot[j];
                    }
                    __syncthreads();
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        dot[j] = add_t(add_t(kpart[0][j], kpart[1][j]), add_t(kpart[2][j], kpart[3][j]));
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc_t t = dot[j];
                    const int n = nb + j * rpw;
                    bool fl = false;
                    if (lc == 0 && n < N && (!split || wave == 0)) {
                        const long o = (long)bz * N + n;
                        if (f.bias) t = add_t(t, mul_t((acc_t)M, from_word<acc_t>(f.bias[n])));
                        f.cc_pred[o] = as_word(t);
                        fl = mismatch<T::IS_INT>(f.cc_obs[o], as_word(t), f.tau_override_cols > 0.f ? f.tau_override_cols : tol);
                        f.col_flag[o] = fl ? 1 : 0;
                    }
                    nc_w += __popcll(__ballot(fl));
                }
            } else {
                // B stored K x N: a staged in LDS; 32 chunk columns per unit, FIN_KY lanes run along K
                acc_t *al = reinterpret_cast<acc_t *>(lds);
                __syncthreads();                                        // previous unit done with al / red
                for (int k = tid; k < K; k += 256) al[k] = from_word<acc_t>(asum[k]);
                __syncthreads();
                acc_t *red = al + (K + 3) / 4 * 4;                      // [FIN_KY][32 * CE]
                const int cx = tid & 31, ky = tid >> 5;
                const int nst = (blk * 32 + cx) * CE;
                const int left = N - nst;
                acc_t colp[CE];
#pragma unroll
                for (int q = 0; q < CE; ++q) colp[q] = T::zero();
                for (int k0 = ky; k0 < K; k0 += 4 * FIN_KY) {
                    i32x4 v[4];
#pragma unroll
                    for (int uu = 0; uu < 4; ++uu) {
                        const int k = k0 + uu * FIN_KY;
                        v[uu] = i32x4{0, 0, 0, 0};
                        if (k < K && left > 0) v[uu] = *reinterpret_cast<const i32x4 *>(Bb + ((long)k * f.ldb + nst) * ES);
                    }
#pragma unroll
                    for (int uu = 0; uu < 4; ++uu) {
                        const int k = k0 + uu * FIN_KY;
                        if (k < K) {
                            const acc_t ak = al[k];
#pragma unroll
                            for (int q = 0; q < CE; ++q) colp[q] = add_t(colp[q], mul_t(T::elem(v[uu], q), ak));
                        }
                    }
                }
#pragma unroll
                for (int q = 0; q < CE; ++q) red[ky * 32 * CE + cx * CE + q] = colp[q];
                __syncthreads();
                // at most two columns per thread (int8: 512 columns per unit)
                for (int c = tid; c < 32 * CE; c += 256) {
                    const int n = blk * 32 * CE + c;
                    bool fl = false;
                    if (n < N) {
                        acc_t t = red[c];
#pragma unroll
                        for (int y = 1; y < FIN_KY; ++y) t = add_t(t, red[y * 32 * CE + c]);
                        if (f.bias) t = add_t(t, mul_t((acc_t)M, from_word<acc_t>(f.bias[n])));
                        const long o = (long)bz * N + n;
                        f.cc_pred[o] = as_word(t);
                        fl = mismatch<T::IS_INT>(f.cc_obs[o], as_word(t), f.tau_override_cols > 0.f ? f.tau_override_cols : tol);
                        f.col_flag[o] = fl ? 1 : 0;
                    }
                    nc_w += __popcll(__ballot(fl));
                }
            }
        } else {
            const int r = (blk - f.col_blocks) * 256 + tid;
            bool fl = false;
            if (r < M) {
                const long o = (long)bz * M + r;
                uint32_t rpw = f.rc_pred[o];
                if (f.bias) { rpw = as_word(add_t(from_word<acc_t>(rpw), sb)); f.rc_pred[o] = rpw; }
                fl = mismatch<T::IS_INT>(f.rc_obs[o], rpw, tol);
                f.row_flag[o] = fl ? 1 : 0;
            }
            nr_w += __popcll(__ballot(fl));
            if (blk == f.col_blocks) {
                // scalar a . b (the single-number check value of Sec. III-B.1), by the first row unit
                acc_t v = T::zero();
                for (int k = tid; k < K; k += 256)
                    v = add_t(v, mul_t(from_word<acc_t>(asum[k]), from_word<acc_t>(f.b_sum[(long)bz * K + k])));
                v = wave_sum(v);
                __syncthreads();                                        // wred free again
                if (lane == 0) wred[wave] = v;
                __syncthreads();
                if (tid == 0)
                    f.s_pred[bz] = as_word(add_t(add_t(add_t(wred[0], wred[1]), add_t(wred[2], wred[3])), mul_t((acc_t)M, sb)));
            }
        }
    }
    // flagged rows / columns of this block, then its ticket
    if (lane == 0) { wcnt[wave][0] = nr_w; wcnt[wave][1] = nc_w; }
    __syncthreads();
    if (tid == 0) {
        const unsigned nr = wcnt[0][0] + wcnt[1][0] + wcnt[2][0] + wcnt[3][0];
        const unsigned nc = wcnt[0][1] + wcnt[1][1] + wcnt[2][1] + wcnt[3][1];
        if (nr | nc) {
            // rare: the counts must be at the coherence point before this block's ticket is, so
            // fetch their old values and wait for them
            unsigned o1 = 0, o2 = 0;
            if (nr) o1 = atomicAdd(f.ticket + 1, nr);
            if (nc) o2 = atomicAdd(f.ticket + 2, nc);
            asm volatile("s_waitcnt vmcnt(0)" :: "v"(o1), "v"(o2) : "memory");
        }
        // Tickets in two levels (atomics on one word are served one after the other, ~12 ns each):
        // the last block of a group of FIN_GROUP takes a ticket for the group.
        const unsigned grp = blockIdx.x / FIN_GROUP, ngrp = (gridDim.x + FIN_GROUP - 1) / FIN_GROUP;
        const unsigned gsize = min((unsigned)FIN_GROUP, gridDim.x - grp * FIN_GROUP);
        bool last = false;
        if (atomicAdd(f.group_ticket + grp, 1u) == gsize - 1) {
            atomicExch(f.group_ticket + grp, 0u);
            last = atomicAdd(f.ticket, 1u) == ngrp - 1;
        }
        if (last) {
            const uint32_t r = atomicExch(f.ticket + 1, 0u), c = atomicExch(f.ticket + 2, 0u);
            atomicExch(f.ticket, 0u);
            f.counts[0] = r;
            f.counts[1] = c;
            f.counts[2] = status_of(r, c);
            f.counts[3] = 0u;
            f.counts[4] = status_of(r, c);
        }
    }
}

// The same step for a B stored N x K (a Linear layer's weight: the common case), arranged so that
// a block's critical path is one round of loads, one reduction and one ticket: the kernel is bound
// by latency, not by the 2 K N bytes it reads, so everything a block needs is requested before
// anything is used.  A unit is (batch item, block of rows of B): each wave takes FN_RW rows of B
// with its lanes along K (deep K: the four waves share FN_RW rows, a quarter of K each), and the
// unit also compares its share of the M rows.  One ticket per block; the last block writes counts.
constexpr int FN_RW = 8;

template <int DT>
__global__ __launch_bounds__(256) void finish_nk_kernel(FinArgs f)
{
    using T = Traits<DT>;
    typedef typename T::acc_t acc_t;
    constexpr int ES = T::ES, CE = 16 / ES;
    __shared__ acc_t wred[4];
    __shared__ acc_t kpart[4][FN_RW];
    __shared__ unsigned wcnt[4][2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int M = f.M, N = f.N, K = f.K;
    {
        const size_t nb = gridDim.x;
        for (size_t i = (size_t)blockIdx.x * 256 + tid; i < f.zero_words; i += nb * 256) f.zero_ptr[i] = 0u;
        for (size_t i = (size_t)blockIdx.x * 256 + tid; i < f.zero2_words; i += nb * 256) f.zero2_ptr[i] = 0u;
    }
    const int nch = (K + CE - 1) / CE;
    const bool split = f.ksplit == 4;
    const int rpb = split ? FN_RW : 4 * FN_RW;                  // rows of B per unit
    const int units = f.col_blocks * f.batch;
    const int rshare = (M + f.col_blocks - 1) / f.col_blocks;   // rows of C a unit compares
    const bool vec_a = (K & 3) == 0 && ((uintptr_t)f.a_sum & 15u) == 0;     // 16-byte loads of a are aligned
    unsigned nr_w = 0, nc_w = 0;
    acc_t sb = T::zero();                                       // sum of the bias
    if (f.bias) sb = block_bias_sum<acc_t>(f.bias, N, wred);

    for (int u = blockIdx.x; u < units; u += gridDim.x) {
        const int bz = u / f.col_blocks, cb = u - bz * f.col_blocks;
        const uint8_t *Bb = f.B + (long)bz * f.sB * ES;
        const uint32_t *asum = f.a_sum + (long)bz * K;
        // ---- everything the unit will compare against, requested first
        const int nrow0 = cb * rpb + (split ? 0 : wave * FN_RW);
        uint32_t my_obs = 0;
        acc_t my_bias = T::zero();
        if (lane < FN_RW && nrow0 + lane < N) {
            my_obs = f.cc_obs[(long)bz * N + nrow0 + lane];
            if (f.bias) my_bias = mul_t((acc_t)M, from_word<acc_t>(f.bias[nrow0 + lane]));
        }
        const int rbeg = cb * rshare, rend = min(rbeg + rshare, M);
        uint32_t ro = 0, rp = 0;
        if (rbeg + tid < rend) { ro = f.rc_obs[(long)bz * M + rbeg + tid]; rp = f.rc_pred[(long)bz * M + rbeg + tid]; }
        float tol = 0.f;
        if (!T::IS_INT) {
            const float ma = __uint_as_float(f.a_max[bz]), mb = __uint_as_float(f.b_max[bz]);
            tol = f.tau_override > 0.f ? f.tau_override : (1e-3f * (float)K) * ma * mb;
            if (cb == 0 && tid == 0) {
                f.maxabs[(long)bz * 2] = ma;
                f.maxabs[(long)bz * 2 + 1] = mb;
                f.tau[bz] = tol;
            }
        }
        // ---- a B over this wave's rows: two chunks per lane and trip, all loads of a trip in flight
        acc_t dot[FN_RW];
#pragma unroll
        for (int j = 0; j < FN_RW; ++j) dot[j] = T::zero();
        const int cstep = split ? 512 : 128;
        for (int ch0 = split ? wave * 128 : 0; ch0 < nch; ch0 += cstep) {
            i32x4 v[FN_RW][2], aw[2][CE / 4];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int ch = ch0 + 64 * h + lane;
                const bool in = ch < nch && (!split || ch < ch0 + 128);
#pragma unroll
                for (int j = 0; j < FN_RW; ++j) {
                    v[j][h] = i32x4{0, 0, 0, 0};
                    if (in && nrow0 + j < N) v[j][h] = *reinterpret_cast<const i32x4 *>(Bb + ((long)(nrow0 + j) * f.ldb + (long)ch * CE) * ES);
                }
                const int left = K - ch * CE;
#pragma unroll
                for (int q4 = 0; q4 < CE / 4; ++q4) {
                    aw[h][q4] = i32x4{0, 0, 0, 0};
                    if (in) {
                        const uint32_t *ap = asum + ch * CE + 4 * q4;
                        if (vec_a && left >= CE) aw[h][q4] = *reinterpret_cast<const i32x4 *>(ap);
                        else {
#pragma unroll
                            for (int e = 0; e < 4; ++e) aw[h][q4][e] = (4 * q4 + e < left) ? (int)ap[e] : 0;
                        }
                    }
                }
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int left = K - (ch0 + 64 * h + lane) * CE;
#pragma unroll
                for (int j = 0; j < FN_RW; ++j) {
                    i32x4 w = v[j][h];
                    if (left < CE) w = mask_chunk(w, left > 0 ? left * ES : 0);
#pragma unroll
                    for (int q = 0; q < CE; ++q)
                        dot[j] = add_t(dot[j], mul_t(T::elem(w, q), from_word<acc_t>((uint32_t)aw[h][q >> 2][q & 3])));
                }
            }
        }
#pragma unroll
        for (int j = 0; j < FN_RW; ++j) dot[j] = wave_sum(dot[j]);
        if (split) {
            __syncthreads();                                    // previous unit done with kpart
            if (lane == 0) {
#pragma unroll
                for (int j = 0; j < FN_RW; ++j) kpart[wave][j] = dot[j];
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < FN_RW; ++j)
                dot[j] = add_t(add_t(kpart[0][j], kpart[1][j]), add_t(kpart[2][j], kpart[3][j]));
        }
        {
            acc_t mine = dot[0];
#pragma unroll
            for (int j = 1; j < FN_RW; ++j) mine = lane == j ? dot[j] : mine;
            mine = add_t(mine, my_bias);
            bool fl = false;
            if (lane < FN_RW && nrow0 + lane < N && (!split || wave == 0)) {
                const long o = (long)bz * N + nrow0 + lane;
                f.cc_pred[o] = as_word(mine);
                fl = mismatch<T::IS_INT>(my_obs, as_word(mine), f.tau_override_cols > 0.f ? f.tau_override_cols : tol);
                f.col_flag[o] = fl ? 1 : 0;
            }
            nc_w += __popcll(__ballot(fl));
        }
        // ---- this unit's share of the rows
        for (int r = rbeg + tid; r - tid < rend; r += 256) {
            bool fl = false;
            if (r < rend) {
                const long o = (long)bz * M + r;
                if (r != rbeg + tid) { ro = f.rc_obs[o]; rp = f.rc_pred[o]; }
                if (f.bias) { rp = as_word(add_t(from_word<acc_t>(rp), sb)); f.rc_pred[o] = rp; }
                fl = mismatch<T::IS_INT>(ro, rp, tol);
                f.row_flag[o] = fl ? 1 : 0;
            }
            nr_w += __popcll(__ballot(fl));
        }
        if (cb == 0) {
            // scalar a . b (the single-number check value of Sec. III-B.1)
            acc_t sv = T::zero();
            for (int k = tid; k < K; k += 256)
                sv = add_t(sv, mul_t(from_word<acc_t>(asum[k]), from_word<acc_t>(f.b_sum[(long)bz * K + k])));
            sv = wave_sum(sv);
            __syncthreads();                                    // wred free again
            if (lane == 0) wred[wave] = sv;
            __syncthreads();
            if (tid == 0)
                f.s_pred[bz] = as_word(add_t(add_t(add_t(wred[0], wred[1]), add_t(wred[2], wred[3])), mul_t((acc_t)M, sb)));
        }
    }
    if (lane == 0) { wcnt[wave][0] = nr_w; wcnt[wave][1] = nc_w; }
    __syncthreads();
    if (tid == 0) {
        const unsigned nr = wcnt[0][0] + wcnt[1][0] + wcnt[2][0] + wcnt[3][0];
        const unsigned nc = wcnt[0][1] + wcnt[1][1] + wcnt[2][1] + wcnt[3][1];
        if (nr | nc) {
            // rare: the counts must be at the coherence point before this block's ticket is
            unsigned o1 = 0, o2 = 0;
            if (nr) o1 = atomicAdd(f.ticket + 1, nr);
            if (nc) o2 = atomicAdd(f.ticket + 2, nc);
            asm volatile("s_waitcnt vmcnt(0)" :: "v"(o1), "v"(o2) : "memory");
        }
        if (atomicAdd(f.ticket, 1u) == gridDim.x - 1) {
            const uint32_t r = atomicExch(f.ticket + 1, 0u), c = atomicExch(f.ticket + 2, 0u);
            atomicExch(f.ticket, 0u);
            f.counts[0] = r;
            f.counts[1] = c;
            f.counts[2] = status_of(r, c);
            f.counts[3] = 0u;
            f.counts[4] = status_of(r, c);
        }
    }
}

hipError_t launch_finish(int dt, const void *B, const Shape &s, const Workspace &w, const Verdict &v,
                         uint32_t *zero_ptr, size_t zero_words, uint32_t *zero2_ptr, size_t zero2_words,
                         hipStream_t st)
{
    FinArgs f;
    f.b_max = w.b_max; f.zero2_ptr = zero2_ptr; f.zero2_words = zero2_ptr ? zero2_words : 0;
    f.zero_ptr = zero_ptr; f.zero_words = zero_ptr ? zero_words : 0;
    f.B = (const uint8_t *)B; f.ldb = s.ldb; f.sB = s.sB; f.transB = s.transB;
    f.M = s.M; f.N = s.N; f.K = s.K;
    f.a_sum = w.a_given ? w.a_given : w.a_sum;
    f.b_sum = w.b_sum; f.rc_pred = w.rc_pred; f.cc_obs = w.cc_obs; f.rc_obs = w.rc_obs;
    f.bias = w.bias;
    f.a_max = (w.a_given && w.amax_given) ? w.amax_given : w.a_max; f.cc_pred = w.cc_pred; f.s_pred = w.s_pred; f.maxabs = w.maxabs; f.tau = w.tau;
    f.tau_override = v.tau_override; f.tau_override_cols = v.tau_override_cols;
    f.row_flag = v.row_flag; f.col_flag = v.col_flag; f.counts = v.counts; f.ticket = w.cmp_ticket;
    f.group_ticket = w.cmp_ticket + 4;
    const int ce = 16 / elem_size(dt);
    const int nch = (s.K + ce - 1) / ce;
    f.batch = s.batch;
    if (s.transB) {
        // deep K (more than one trip of 128 chunks per row): the waves of a block share its rows
        f.ksplit = nch > 128 ? 4 : 1;
        f.lpr = 64;
        const int rpb = f.ksplit == 4 ? FN_RW : 4 * FN_RW;
        f.col_blocks = (s.N + rpb - 1) / rpb;
        const long units = (long)f.col_blocks * s.batch;
        if (units > 0x7FFFFFFFL) return hipErrorInvalidValue;
        dim3 grid((unsigned)(units < 512 ? units : 512), 1, 1);
        switch (dt) {
        case DT_I8:   hipLaunchKernelGGL(finish_nk_kernel<DT_I8>, grid, dim3(256), 0, st, f); break;
        case DT_BF16: hipLaunchKernelGGL(finish_nk_kernel<DT_BF16>, grid, dim3(256), 0, st, f); break;
        case DT_F16:  hipLaunchKernelGGL(finish_nk_kernel<DT_F16>, grid, dim3(256), 0, st, f); break;
        default: return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
    f.lpr = nch <= 8 ? 8 : (nch <= 16 ? 16 : (nch <= 32 ? 32 : 64));
    f.ksplit = 1;
    f.col_blocks = (s.N + 32 * ce - 1) / (32 * ce);
    const int row_blocks = (s.M + 255) / 256;
    const size_t smem = ((size_t)(s.K + 3) / 4 * 4 + (size_t)FIN_KY * 32 * ce) * 4;
    const long units = (long)(f.col_blocks + row_blocks) * s.batch;
    if (units > 0x7FFFFFFFL) return hipErrorInvalidValue;
    dim3 grid((unsigned)(units < FIN_MAX_BLOCKS ? units : FIN_MAX_BLOCKS), 1, 1);
    switch (dt) {
    case DT_I8:   hipLaunchKernelGGL(finish_kernel<DT_I8>, grid, dim3(256), smem, st, f); break;
    case DT_BF16: hipLaunchKernelGGL(finish_kernel<DT_BF16>, grid, dim3(256), smem, st, f); break;
    case DT_F16:  hipLaunchKernelGGL(finish_kernel<DT_F16>, grid, dim3(256), smem, st, f); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ================================================================= discrepancy
// Statistics of d = observed - predicted over the rows and over the columns of one GEMM: what
// the paper's "Eps Generation" (Sec. III-B.1) fits its thresholds to.  One block per batch
// item; out[bz] = { sum d, sum d^2, max|d|, count } for the rows, then the same for the columns.
struct DiscArgs {
    const uint32_t *cc_pred, *rc_pred, *cc_src, *rc_src;
    int M, N;
    float *out;           // [batch][8]
};

__global__ __launch_bounds__(256) void discrepancy_kernel(DiscArgs a)
{
    __shared__ float red[4][3];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, bz = blockIdx.x;
    for (int side = 0; side < 2; ++side) {
        const int n = side == 0 ? a.M : a.N;
        const uint32_t *src = (side == 0 ? a.rc_src : a.cc_src) + (long)bz * n;
        const uint32_t *pred = (side == 0 ? a.rc_pred : a.cc_pred) + (long)bz * n;
        float s = 0.f, s2 = 0.f, mx = 0.f;
        for (int i = tid; i < n; i += 256) {
            const float dd = __uint_as_float(src[i]) - __uint_as_float(pred[i]);
            s += dd;
            s2 = __builtin_fmaf(dd, dd, s2);
            mx = fmaxf(mx, fabsf(dd));
        }
        s = wave_sum(s);
        s2 = wave_sum(s2);
        mx = wave_max(mx);
        __syncthreads();
        if (lane == 0) { red[wave][0] = s; red[wave][1] = s2; red[wave][2] = mx; }
        __syncthreads();
        if (tid == 0) {
            float *o = a.out + (long)bz * 8 + side * 4;
            o[0] = (red[0][0] + red[1][0]) + (red[2][0] + red[3][0]);
            o[1] = (red[0][1] + red[1][1]) + (red[2][1] + red[3][1]);
            o[2] = fmaxf(fmaxf(red[0][2], red[1][2]), fmaxf(red[2][2], red[3][2]));
            o[3] = (float)n;
        }
    }
}

hipError_t launch_discrepancy(const Shape &s, const Workspace &w, bool stored, float *out, hipStream_t st)
{
    DiscArgs a;
    a.cc_pred = w.cc_pred; a.rc_pred = w.rc_pred;
    a.cc_src = stored ? w.cc_vobs : w.cc_obs;
    a.rc_src = stored ? w.rc_vobs : w.rc_obs;
    a.M = s.M; a.N = s.N; a.out = out;
    hipLaunchKernelGGL(discrepancy_kernel, dim3((unsigned)s.batch), dim3(256), 0, st, a);
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
    const uint32_t *gate; // non-null: nothing to do if *gate == 0 (no tile was recomputed: C is as it was checked)
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
    if (a.gate && *a.gate == 0u) return;
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
            s = seg_sum(s, CW);
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

hipError_t launch_verify_sums(int dt, const void *C, const Shape &s, const Workspace &w, hipStream_t st, bool gated)
{
    VerArgs a;
    a.gate = gated ? w.fix_count : nullptr;
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

constexpr int LOC_THREADS = 1024;

// Appends the CT-tile index of every non-zero byte of flag[0..n) to list (at most MAX_LIST kept;
// *count keeps counting).  Sixteen flags per load where the address allows: flags are almost
// all zero, and the scan is bound by the latency of its loads.
__device__ inline void list_flagged(const uint8_t *flag, int n, int *list, int *count, int tid)
{
    auto note = [&](int i) {
        int p = atomicAdd(count, 1);
        if (p < MAX_LIST) list[p] = i / CT;
    };
    const int head = min(n, (int)((16u - (unsigned)((uintptr_t)flag & 15u)) & 15u));
    const int nchunk = (n - head) / 16;
    const int tail0 = head + nchunk * 16;
    if (tid < head && flag[tid]) note(tid);
    if (tid < n - tail0 && flag[tail0 + tid]) note(tail0 + tid);
    const i32x4 *body = reinterpret_cast<const i32x4 *>(flag + head);
    for (int c0 = 0; c0 < nchunk; c0 += 4 * LOC_THREADS) {
        i32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * LOC_THREADS + tid;
            v[u] = i32x4{0, 0, 0, 0};
            if (c < nchunk) v[u] = body[c];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if ((v[u][0] | v[u][1] | v[u][2] | v[u][3]) == 0) continue;
            const int c = c0 + u * LOC_THREADS + tid;
#pragma unroll
            for (int q = 0; q < 16; ++q)
                if (((unsigned)v[u][q >> 2] >> (8 * (q & 3))) & 0xFFu) note(head + c * 16 + q);
        }
    }
}

__global__ __launch_bounds__(LOC_THREADS) void locate_kernel(LocArgs a)
{
    __shared__ int rows[MAX_LIST], cols[MAX_LIST];
    __shared__ int nr, nc;
    const int bz = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) { nr = 0; nc = 0; }
    __syncthreads();
    list_flagged(a.row_flag + (long)bz * a.M, a.M, rows, &nr, tid);
    list_flagged(a.col_flag + (long)bz * a.N, a.N, cols, &nc, tid);
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

// Step 2: one workgroup recomputes one CT x CT tile of C over the whole K.  Its first wave issues
// every MFMA, the same instruction in the same ascending-k order as the GEMM kernel, so a
// floating-point tile comes back with the bits the GEMM produced.  What bounds the step is the
// latency of the operand loads (a wave keeps 2 * FIX_UB 16-byte loads per lane in flight), so
// FIX_WAVES further waves load, each a different run of FIX_UB k-steps, and hand the operands to
// the first wave through LDS, in the lane layout they are consumed in; while it works through one
// group of runs the loads of the next group are in flight.
constexpr int FIX_WAVES = 8;                    // waves that load (the workgroup has one more)
constexpr int FIX_UB = 8;                       // k-steps a wave loads per group
constexpr size_t FIX_LDS_BYTES = (size_t)FIX_WAVES * FIX_UB * 2 * 64 * 16;

struct FixArgs {
    const uint8_t *A, *B;
    uint8_t *C;
    int M, N, K, transB;
    long lda, ldb, ldc, sA, sB, sC;
    const int32_t *fix_tiles;
    const uint32_t *fix_count;
    uint32_t *cc_vobs;      // non-null: the re-summed column sums of the tile's columns are cleared (they are
                            // accumulated again by resum_touched_kernel)
    const uint32_t *bias;   // layer bias [N] or null
};

template <int DT>
__global__ __launch_bounds__(64 * (FIX_WAVES + 1)) void recompute_kernel(FixArgs a)
{
    using T = Traits<DT>;
    typedef typename T::accv_t accv_t;
    constexpr int ES = T::ES, CE = 16 / ES;
    constexpr int UB = FIX_UB;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    i32x4 *stage = reinterpret_cast<i32x4 *>(lds);          // [FIX_WAVES * UB k-steps][A, B][64 lanes]
    unsigned n = a.fix_count[0];
    if (n > (unsigned)MAX_FIX_TILES) n = MAX_FIX_TILES;
    if (blockIdx.x >= n) return;                            // the whole workgroup leaves
    const int bz = a.fix_tiles[3 * blockIdx.x], tr = a.fix_tiles[3 * blockIdx.x + 1],
              tc = a.fix_tiles[3 * blockIdx.x + 2];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, lh = lane >> 5;
    const int row = tr * CT + l32, col = tc * CT + l32;
    const uint8_t *Ab = a.A + (long)bz * a.sA * ES, *Bb = a.B + (long)bz * a.sB * ES;
    const int K = a.K;
    if (a.cc_vobs && wave == 1 && lane < CT && col < a.N) a.cc_vobs[(long)bz * a.N + col] = 0u;
    accv_t acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = T::zero();
    const int steps = (K + 2 * CE - 1) / (2 * CE);
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
    // every wave takes the same number of trips: the barriers are reached by all
    for (int g0 = 0; g0 < steps; g0 += FIX_WAVES * UB) {
        const int lw = wave - 1;                            // loading wave 0 .. FIX_WAVES - 1
        const int ks0 = g0 + lw * UB;
        i32x4 av[UB], bv[UB];
        if (wave != 0) {
#pragma unroll
            for (int u = 0; u < UB; ++u) { av[u] = load_a(ks0 + u); bv[u] = load_b(ks0 + u); }
        }
        __syncthreads();                                    // the first wave is done with the previous group
        if (wave != 0) {
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                stage[((lw * UB + u) * 2 + 0) * 64 + lane] = av[u];
                stage[((lw * UB + u) * 2 + 1) * 64 + lane] = bv[u];
            }
        }
        __syncthreads();
        if (wave == 0) {
            // whole runs of UB k-steps (a run's k-steps past the end of K hold zeros and add nothing);
            // the operands of the next run are read while the chain of dependent MFMAs of this one runs
            const int nrun = min(FIX_WAVES, (steps - g0 + UB - 1) / UB);
            auto read_run = [&](int r, i32x4 (&x)[UB], i32x4 (&y)[UB]) __attribute__((always_inline)) {
#pragma unroll
                for (int u = 0; u < UB; ++u) {
                    x[u] = stage[((r * UB + u) * 2 + 0) * 64 + lane];
                    y[u] = stage[((r * UB + u) * 2 + 1) * 64 + lane];
                }
            };
            i32x4 x0[UB], y0[UB], x1[UB], y1[UB];
            read_run(0, x0, y0);
            for (int r = 0; r < nrun; r += 2) {
                read_run(min(r + 1, FIX_WAVES - 1), x1, y1);
#pragma unroll
                for (int u = 0; u < UB; ++u) acc = T::mfma(y0[u], x0[u], acc);   // B first: lane = row of C, registers = columns
                if (r + 1 < nrun) {
                    read_run(min(r + 2, FIX_WAVES - 1), x0, y0);
#pragma unroll
                    for (int u = 0; u < UB; ++u) acc = T::mfma(y1[u], x1[u], acc);
                }
            }
        }
    }
    if (wave != 0) return;
    uint8_t *Cb = a.C + (long)bz * a.sC * T::OS;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int gc = tc * CT + 8 * (i >> 2) + 4 * lh + (i & 3);
        if (row < a.M && gc < a.N) {
            typename T::acc_t v = acc[i];
            if (a.bias) v = add_t(v, from_word<typename T::acc_t>(a.bias[gc]));
            T::store_c(Cb, (long)row * a.ldc + gc, v);
        }
    }
}

// Step 3 when the sums of the stored C are at hand (abft_verify ran on this C): only the rows and
// the columns of the recomputed tiles changed, so only their sums are formed again.  Workgroup
// (t, p) serves listed tile t: p < CT sums row p of the tile over all N and stores it; every p sums
// the tile's CT columns over its share of the M rows and adds that to the column sums, which
// recompute_kernel has cleared.  A tile row or tile column listed more than once is summed by
// its first tile only.
constexpr int TOUCH_PARTS = 64;
constexpr int TOUCH_TILES = 8;           // workgroups per part: listed tiles served at a time

struct TouchArgs {
    const uint8_t *C;
    long ldc, sC;
    int M, N;
    const int32_t *fix_tiles;
    const uint32_t *fix_count;
    uint32_t *cc_vobs, *rc_vobs;
};

template <int DT>
__global__ __launch_bounds__(256) void resum_touched_kernel(TouchArgs a)
{
    using T = Traits<DT>;
    typedef typename T::acc_t acc_t;
    constexpr int OS = T::OS, CE = 16 / OS;
    constexpr int CPR = CT / CE;                            // 16-byte chunks across a tile
    constexpr int RL = 256 / CPR;                           // rows a pass of the workgroup covers
    __shared__ acc_t red[256 * CE];
    unsigned n = a.fix_count[0];
    if (n > (unsigned)MAX_FIX_TILES) n = MAX_FIX_TILES;
    const int part = blockIdx.y, tid = threadIdx.x;
    // the grid has TOUCH_TILES workgroups per part; listed tiles beyond that many take further trips
    for (int t = blockIdx.x; t < (int)n; t += gridDim.x) {
        const int bz = a.fix_tiles[3 * t], tr = a.fix_tiles[3 * t + 1], tc = a.fix_tiles[3 * t + 2];
        bool first_row = true, first_col = true;
        for (int q = 0; q < t; ++q)
            if (a.fix_tiles[3 * q] == bz) {
                first_row = first_row && a.fix_tiles[3 * q + 1] != tr;
                first_col = first_col && a.fix_tiles[3 * q + 2] != tc;
            }
        const uint8_t *Cb = a.C + (long)bz * a.sC * OS;
        const int M = a.M, N = a.N;

        const int row = tr * CT + part;
        if (first_row && part < CT && row < M) {
            acc_t s = T::zero();
            const int nch = (N + CE - 1) / CE;
            for (int c = tid; c < nch; c += 256) {
                const i32x4 v = *reinterpret_cast<const i32x4 *>(Cb + ((long)row * a.ldc + (long)c * CE) * OS);
                const int nvalid = N - c * CE;
#pragma unroll
                for (int q = 0; q < CE; ++q)
                    if (q < nvalid) s = add_t(s, out_elem<DT>(v, q));
            }
            s = wave_sum(s);
            if ((tid & 63) == 0) red[tid >> 6] = s;
            __syncthreads();
            if (tid == 0) a.rc_vobs[(long)bz * M + row] = as_word(add_t(add_t(red[0], red[1]), add_t(red[2], red[3])));
            __syncthreads();                                    // red is used again below
        }
        if (!first_col) continue;

        const int mc = (M + TOUCH_PARTS - 1) / TOUCH_PARTS;
        const int rbeg = part * mc, rend = min(rbeg + mc, M);
        const int cx = tid % CPR, ry = tid / CPR;
        const int col0 = tc * CT + cx * CE;
        const int nvalid = N - col0;
        acc_t colacc[CE];
#pragma unroll
        for (int q = 0; q < CE; ++q) colacc[q] = T::zero();
        for (int r0 = rbeg + ry; r0 < rend; r0 += RL * ENC_UNROLL) {
            i32x4 v[ENC_UNROLL];
#pragma unroll
            for (int u = 0; u < ENC_UNROLL; ++u) {
                const int r = r0 + u * RL;
                v[u] = i32x4{0, 0, 0, 0};
                if (nvalid > 0 && r < rend) v[u] = *reinterpret_cast<const i32x4 *>(Cb + ((long)r * a.ldc + col0) * OS);
            }
#pragma unroll
            for (int u = 0; u < ENC_UNROLL; ++u) {
                if (r0 + u * RL < rend) {
#pragma unroll
                    for (int q = 0; q < CE; ++q)
                        if (q < nvalid) colacc[q] = add_t(colacc[q], out_elem<DT>(v[u], q));
                }
            }
        }
#pragma unroll
        for (int q = 0; q < CE; ++q) red[ry * CT + cx * CE + q] = colacc[q];
        __syncthreads();
        if (tid < CT) {
            const int col = tc * CT + tid;
            if (col < N && rbeg < rend) {
                acc_t s = red[tid];
                for (int y = 1; y < RL; ++y) s = add_t(s, red[y * CT + tid]);
                atomic_add_word(a.cc_vobs + (long)bz * N + col, s);
            }
        }
        __syncthreads();                                        // red is free for the next tile
    }
}

template <int DT>
static hipError_t launch_recompute(const FixArgs &f, hipStream_t st)
{
    auto kern = recompute_kernel<DT>;
    hipError_t e = ensure_max_lds(reinterpret_cast<const void *>(kern), (int)FIX_LDS_BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(MAX_FIX_TILES), dim3(64 * (FIX_WAVES + 1)), FIX_LDS_BYTES, st, f);
    return hipGetLastError();
}

hipError_t launch_correct(int dt, const void *A, const void *B, void *C, const Shape &s,
                          const Workspace &w, const Verdict &v, bool with_sto, bool clear_list, bool targeted,
                          size_t stale_words, uint32_t *zero_ptr, size_t zero_words, hipStream_t st, bool skip_if_clean)
{
    hipError_t e = hipSuccess;
    if (clear_list && (e = launch_zero(w.fix_count, 2, st)) != hipSuccess) return e;
    LocArgs l;
    l.row_flag = v.row_flag; l.col_flag = v.col_flag; l.M = s.M; l.N = s.N;
    l.fix_tiles = w.fix_tiles; l.fix_count = w.fix_count;
    hipLaunchKernelGGL(locate_kernel, dim3((unsigned)s.batch), dim3(LOC_THREADS), 0, st, l);
    if ((e = hipGetLastError()) != hipSuccess) return e;

    FixArgs f;
    f.A = (const uint8_t *)A; f.B = (const uint8_t *)B; f.C = (uint8_t *)C;
    f.M = s.M; f.N = s.N; f.K = s.K; f.transB = s.transB;
    f.lda = s.lda; f.ldb = s.ldb; f.ldc = s.ldc; f.sA = s.sA; f.sB = s.sB; f.sC = s.sC;
    f.fix_tiles = w.fix_tiles; f.fix_count = w.fix_count;
    f.cc_vobs = targeted ? w.cc_vobs : nullptr;
    f.bias = w.bias;
    switch (dt) {
    case DT_I8:   e = launch_recompute<DT_I8>(f, st); break;
    case DT_BF16: e = launch_recompute<DT_BF16>(f, st); break;
    case DT_F16:  e = launch_recompute<DT_F16>(f, st); break;
    default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    if (targeted) {
        TouchArgs t;
        t.C = (const uint8_t *)C; t.ldc = s.ldc; t.sC = s.sC; t.M = s.M; t.N = s.N;
        t.fix_tiles = w.fix_tiles; t.fix_count = w.fix_count; t.cc_vobs = w.cc_vobs; t.rc_vobs = w.rc_vobs;
        const dim3 grid(TOUCH_TILES, TOUCH_PARTS);
        switch (dt) {
        case DT_I8:   hipLaunchKernelGGL(resum_touched_kernel<DT_I8>, grid, dim3(256), 0, st, t); break;
        case DT_BF16: hipLaunchKernelGGL(resum_touched_kernel<DT_BF16>, grid, dim3(256), 0, st, t); break;
        default:      hipLaunchKernelGGL(resum_touched_kernel<DT_F16>, grid, dim3(256), 0, st, t); break;
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
        return launch_compare(dt, s, w, v, true, with_sto, nullptr, 0, st);
    }
    // re-check without earlier sums of this C: the stored C is re-summed as a whole (a streaming
    // pass at HBM speed) and compared with the predictions
    if (stale_words && (e = launch_zero(w.cc_vobs, stale_words, st)) != hipSuccess) return e;
    if ((e = launch_verify_sums(dt, C, s, w, st, skip_if_clean)) != hipSuccess) return e;
    return launch_compare(dt, s, w, v, true, with_sto, zero_ptr, zero_words, st, skip_if_clean);
}

// ====================================================================== checksum-only correction
// Integers: one block per batch item.  With exactly one flagged row i and one flagged column j
// whose discrepancies d (re-summed stored C minus prediction, in Z/2^32) agree, the corrupted
// element is C[i][j] and C[i][j] - d its value (the classic scheme of Sec. II-B; no operand is
// read, nothing is recomputed).  The re-summed vectors and the flags of the item are updated
// with it; any other pattern is left as it is.  The last block writes counts and status.
struct ArithArgs {
    uint8_t *row_flag, *col_flag;
    uint32_t *counts;
    uint32_t *ticket;            // [4]: ticket, flagged rows left, flagged cols left, elements fixed (self-cleaning)
    const uint32_t *cc_pred, *rc_pred;
    uint32_t *cc_vobs, *rc_vobs;
    uint32_t *C;
    long ldc, sC;
    int M, N;
};

__global__ __launch_bounds__(256) void arith_fix_kernel(ArithArgs a)
{
    __shared__ int nr, nc, ri, cj;
    const int bz = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) { nr = 0; nc = 0; ri = 0; cj = 0; }
    __syncthreads();
    for (int i = tid; i < a.M; i += 256)
        if (a.row_flag[(long)bz * a.M + i]) { atomicAdd(&nr, 1); atomicMax(&ri, i); }
    for (int j = tid; j < a.N; j += 256)
        if (a.col_flag[(long)bz * a.N + j]) { atomicAdd(&nc, 1); atomicMax(&cj, j); }
    __syncthreads();
    if (tid != 0) return;
    uint32_t r = (uint32_t)nr, c = (uint32_t)nc, fixed = 0;
    if (r == 1 && c == 1) {
        const long ir = (long)bz * a.M + ri, jc = (long)bz * a.N + cj;
        const uint32_t dr = a.rc_vobs[ir] - a.rc_pred[ir], dc = a.cc_vobs[jc] - a.cc_pred[jc];
        if (dr == dc) {
            a.C[(long)bz * a.sC + (long)ri * a.ldc + cj] -= dr;
            a.rc_vobs[ir] -= dr;
            a.cc_vobs[jc] -= dc;
            a.row_flag[ir] = 0;
            a.col_flag[jc] = 0;
            r = 0; c = 0; fixed = 1;
        }
    }
    if (r) atomicAdd(a.ticket + 1, r);
    if (c) atomicAdd(a.ticket + 2, c);
    if (fixed) atomicAdd(a.ticket + 3, fixed);
    __threadfence();
    if (atomicAdd(a.ticket, 1u) == gridDim.x - 1) {
        const uint32_t rr = atomicExch(a.ticket + 1, 0u), cc = atomicExch(a.ticket + 2, 0u),
                       ff = atomicExch(a.ticket + 3, 0u);
        atomicExch(a.ticket, 0u);
        const uint32_t before = a.counts[2];
        a.counts[0] = rr;
        a.counts[1] = cc;
        a.counts[2] = status_of(rr, cc);
        a.counts[3] = ff;
        a.counts[4] = before;
    }
}

hipError_t launch_arith_fix(void *C, const Shape &s, const Workspace &w, const Verdict &v, hipStream_t st)
{
    ArithArgs a;
    a.row_flag = v.row_flag; a.col_flag = v.col_flag; a.counts = v.counts; a.ticket = w.cmp_ticket;
    a.cc_pred = w.cc_pred; a.rc_pred = w.rc_pred; a.cc_vobs = w.cc_vobs; a.rc_vobs = w.rc_vobs;
    a.C = (uint32_t *)C; a.ldc = s.ldc; a.sC = s.sC; a.M = s.M; a.N = s.N;
    hipLaunchKernelGGL(arith_fix_kernel, dim3((unsigned)s.batch), dim3(256), 0, st, a);
    return hipGetLastError();
}

// ====================================================================== inject
__global__ void flip_kernel(uint8_t *C, long idx, int os, int bit)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    if (os == 4) {
        uint32_t *p = reinterpret_cast<uint32_t *>(C) + idx;
        *p ^= (1u << bit);
    } else if (os == 1) {
        C[idx] = (uint8_t)(C[idx] ^ (uint8_t)(1u << bit));
    } else {
        uint16_t *p = reinterpret_cast<uint16_t *>(C) + idx;
        *p = (uint16_t)(*p ^ (uint16_t)(1u << bit));
    }
}

hipError_t launch_flip_at(void *base, long idx, int elem_bytes, int bit, hipStream_t st)
{
    hipLaunchKernelGGL(flip_kernel, dim3(1), dim3(64), 0, st, (uint8_t *)base, idx, elem_bytes, bit);
    return hipGetLastError();
}

hipError_t launch_flip(void *C, int dt, const Shape &s, long batch_idx, long row, long col, int bit,
                       hipStream_t st)
{
    long idx = batch_idx * s.sC + row * s.ldc + col;
    hipLaunchKernelGGL(flip_kernel, dim3(1), dim3(64), 0, st, (uint8_t *)C, idx, out_size(dt), bit);
    return hipGetLastError();
}

// ====================================================================== report: matrix-pipe ceiling
// Nothing but matrix instructions, in the GEMM kernel's own shape: one wave per SIMD, sixteen
// independent 32 x 32 accumulators (all 256 accumulator registers), operands held in registers.
// What it reaches is the ceiling of the matrix pipe at the clock the chip sustains under that
// load; the fraction of it a GEMM kernel reaches says how well its loop feeds the pipe, apart
// from the clock.  Every wave also reads the shader clock counter and the constant 100 MHz
// counter around its loop, which gives the clock it ran at.
template <int DT>
__global__ __launch_bounds__(256) void mfma_peak_kernel(int iters, unsigned long long *clk, uint32_t *sink)
{
    using T = Traits<DT>;
    typedef typename T::accv_t accv_t;
    // Operands with the bit activity of real data: random signs and mantissas, magnitudes in
    // [1/128, 1), four different register sets taken in turn.  (With operands that never change
    // the matrix pipe toggles few bits, draws little power and keeps a clock no GEMM on real data
    // is granted.)
    uint32_t h = (uint32_t)(blockIdx.x * 256 + threadIdx.x) * 2654435761u + 12345u;
    auto next = [&]() __attribute__((always_inline)) -> int {
        h ^= h << 13; h ^= h >> 17; h ^= h << 5;
        uint32_t w = h;
        if (DT == DT_BF16) w = (w & 0x807F807Fu) | 0x3C003C00u | ((w >> 3) & 0x03800380u);
        if (DT == DT_F16) w = (w & 0x83FF83FFu) | 0x20002000u | ((w >> 3) & 0x1C001C00u);
        return (int)w;
    };
    i32x4 a[4], b[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        a[q] = i32x4{next(), next(), next(), next()};
        b[q] = i32x4{next(), next(), next(), next()};
    }
    accv_t acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = T::zero();
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j] = T::mfma(b[j & 3], a[(j >> 2) & 3], acc[j]);
    }
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    // keep the accumulators alive
    typename T::acc_t t = T::zero();
#pragma unroll
    for (int j = 0; j < 16; ++j) t = add_t(t, acc[j][j]);
    if (as_word(t) == 0x7FC12345u) sink[threadIdx.x] = as_word(t);
    if (threadIdx.x == 0) {
        clk[2 * blockIdx.x] = c1 - c0;
        clk[2 * blockIdx.x + 1] = w1 - w0;
    }
}

hipError_t launch_mfma_peak(int dt, int blocks, int iters, unsigned long long *clk, uint32_t *sink, hipStream_t st)
{
    switch (dt) {
    case DT_I8:   hipLaunchKernelGGL(mfma_peak_kernel<DT_I8>, dim3(blocks), dim3(256), 0, st, iters, clk, sink); break;
    case DT_BF16: hipLaunchKernelGGL(mfma_peak_kernel<DT_BF16>, dim3(blocks), dim3(256), 0, st, iters, clk, sink); break;
    case DT_F16:  hipLaunchKernelGGL(mfma_peak_kernel<DT_F16>, dim3(blocks), dim3(256), 0, st, iters, clk, sink); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace abft
