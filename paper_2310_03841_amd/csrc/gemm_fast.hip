// Fast path of the protected GEMM for gfx950: B stored N x K (both operands K-contiguous) and
// K a whole number of 128-byte slabs.  Same mathematics and the same epilogue as gemm_kernel;
// what differs is the data movement:
//   * global -> LDS with direct-to-LDS loads (global_load_lds_dwordx4): no VGPR staging.  One
//     wave instruction fills 8 LDS rows of 128 bytes; the XOR swizzle of the LDS layout is
//     applied by choosing which global 16-byte chunk each lane fetches.
//   * 256 x 256 tiles, 4 waves of 128 x 128 (sixteen 32x32 MFMA blocks per wave), two LDS
//     buffers of 64 KB, one barrier per slab; 128 x 256 tiles fill the last, partial round.
//   * MFMAs take the B fragment first, so a lane owns a row of C (see gemm_epilogue.h).
//   * workgroup -> tile mapping keeps the workgroups that share an XCD (and its L2) on a
//     compact group of tiles.
// Rows of the tile beyond the (stripe-augmented) problem are fetched from a valid row instead
// of being zero-filled: a row of A only influences the same row of C, which is discarded.
#include "abft_device.h"
#include "gemm_args.h"
#include "gemm_epilogue.h"

namespace abft {

typedef const __attribute__((address_space(1))) void *gas_ptr;
typedef __attribute__((address_space(3))) void *las_ptr;

// One BM x BN tile with origin (m0, n0) of batch item bz.
template <int DT, int BM, int BN, bool PROT>
__device__ __forceinline__ void fast_tile(const GemmArgs &g, uint8_t *smem, int m0, int n0, int bz, int tn)
{
    using T = Traits<DT>;
    typedef typename T::accv_t accv_t;
    constexpr int ES = T::ES;
    constexpr int KE = SLAB_BYTES / ES;
    constexpr int TM = BM / 2, TN = BN / 2;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int GA = BM / 32, GB = BN / 32;     // 8-row load groups per wave per slab
    constexpr int BUF = (BM + BN) * SLAB_BYTES;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform by construction
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int M = g.M, N = g.N, K = g.K;

    const uint8_t *Ab = g.A + (long)bz * g.sA * ES;
    const uint8_t *Bb = g.B + (long)bz * g.sB * ES;

    // ---- per-lane global sources.  Load group p of this wave covers tile rows
    // (4 p + wave) * 8 .. + 8; lane l lands in LDS row + (l >> 3), slot (l & 7), and fetches
    // the chunk (l & 7) ^ (l >> 3) so that LDS slot = chunk ^ (row & 7).
    const int lrow = lane >> 3;
    const int lchunk = (lane & 7) ^ lrow;
    // Interior tiles: the rows of consecutive load groups are 32 apart in one matrix, so a lane
    // needs one base pointer and a uniform stride.  Edge tiles (rows past the end) pick the
    // source row by row.
    const bool a_interior = (m0 + BM <= M), b_interior = (n0 + BN <= N);
    const uint8_t *a_lane = Ab + (long)(m0 + wave * 8 + lrow) * g.lda * ES + lchunk * 16;
    const uint8_t *b_lane = Bb + (long)(n0 + wave * 8 + lrow) * g.ldb * ES + lchunk * 16;
    const long a_pstride = 32 * g.lda * ES, b_pstride = 32 * g.ldb * ES;
    auto a_src = [&](int p) __attribute__((always_inline)) -> const uint8_t * {
        const int r = m0 + (4 * p + wave) * 8 + lrow;
        const uint8_t *s = r < M ? Ab + (long)r * g.lda * ES : Ab;
        return s + lchunk * 16;
    };
    auto b_src = [&](int p) __attribute__((always_inline)) -> const uint8_t * {
        const int r = n0 + (4 * p + wave) * 8 + lrow;
        const uint8_t *s = r < N ? Bb + (long)r * g.ldb * ES : Bb;
        return s + lchunk * 16;
    };
    const int a_rows = M - m0, b_rows = N - n0;       // rows of this tile that matter

    // The accumulators are never zero-filled: the first MFMA of every block takes a literal
    // zero as its addend.  Every block is always computed, also where the tile hangs over the
    // edge of the problem: a conditional MFMA would force the accumulators out of the AGPRs.
    accv_t acc[MI][NI];
    accv_t zerov;
#pragma unroll
    for (int i = 0; i < 16; ++i) zerov[i] = T::zero();

    // One loop serves interior and edge tiles (two instances of the MFMA loop that meet in
    // front of the epilogue would push the accumulators through VGPR copies); only the source
    // address of a load depends, wave-uniformly, on where the tile lies.
    auto issue_loads = [&](int s, int buf) __attribute__((always_inline)) {
        const long koff = (long)s * SLAB_BYTES;
        uint8_t *sA = smem + buf * BUF;
        uint8_t *sB = sA + BM * SLAB_BYTES;
#pragma unroll
        for (int p = 0; p < GA; ++p) {
            const int rb = (4 * p + wave) * 8;
            if (a_interior) {
                __builtin_amdgcn_global_load_lds((gas_ptr)(a_lane + p * a_pstride + koff),
                                                 (las_ptr)(sA + rb * SLAB_BYTES), 16, 0, 0);
            } else if (rb < a_rows) {
                __builtin_amdgcn_global_load_lds((gas_ptr)(a_src(p) + koff), (las_ptr)(sA + rb * SLAB_BYTES), 16, 0, 0);
            }
        }
#pragma unroll
        for (int p = 0; p < GB; ++p) {
            const int rb = (4 * p + wave) * 8;
            if (b_interior) {
                __builtin_amdgcn_global_load_lds((gas_ptr)(b_lane + p * b_pstride + koff),
                                                 (las_ptr)(sB + rb * SLAB_BYTES), 16, 0, 0);
            } else if (rb < b_rows) {
                __builtin_amdgcn_global_load_lds((gas_ptr)(b_src(p) + koff), (las_ptr)(sB + rb * SLAB_BYTES), 16, 0, 0);
            }
        }
    };
    // ---- main loop, software-pipelined by hand.  A slab is four MFMA steps of 32 bytes of K.
    // The fragments of step t+1 are read from LDS while the MFMAs of step t run (two register
    // sets); the reads are issued in the first half of a step so that the second half covers
    // their latency.  The barrier sits between steps 2 and 3: by then every wave has read its
    // step-3 fragments, so nobody reads this slab's buffer any more and the loads of slab s+2
    // can be issued into it at once, while step 3 runs and prefetches step 0 of slab s+1.
    i32x4 fa[2][MI], fb[2][NI];
    auto ldfr = [&](int buf, int s4, int set) __attribute__((always_inline)) {
        const uint8_t *sA = smem + buf * BUF;
        const uint8_t *sB = sA + BM * SLAB_BYTES;
        const int sw = ((2 * s4 + lh) ^ (lane & 7)) * 16;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
            fa[set][mi] = *reinterpret_cast<const i32x4 *>(sA + (wm * TM + mi * 32 + l32) * SLAB_BYTES + sw);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
            fb[set][ni] = *reinterpret_cast<const i32x4 *>(sB + (wn * TN + ni * 32 + l32) * SLAB_BYTES + sw);
    };
    auto mfmas = [&](auto first_c, int set) __attribute__((always_inline)) {
        constexpr bool FIRST = decltype(first_c)::value;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                acc[mi][ni] = T::mfma(fb[set][ni], fa[set][mi], FIRST ? zerov : acc[mi][ni]);
    };
    auto interleave = [&]() __attribute__((always_inline)) {
        // scheduling directive: (MFMA, LDS read) x (MI + NI), then the remaining MFMAs
#pragma unroll
        for (int j = 0; j < MI + NI; ++j) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, MI * NI - (MI + NI), 0);
    };
    // Protected tiles reduce the slabs of A they own (slab s belongs to tile column s mod
    // tiles_n) while those are resident: see gemm_apass.h.
    constexpr int AUX_OFF = 2 * (256 + 256) * SLAB_BYTES;           // behind the buffers of the largest tile
    uint32_t *col_lds = reinterpret_cast<uint32_t *>(smem + AUX_OFF);
    EpiProt<DT> ep;
    ep.st.rdot = T::zero(); ep.st.amax = 0.f;
    ep.col_lds = col_lds; ep.tn = tn; ep.tiles_n = g.tiles_n; ep.owned = 0;
    {
        const int nslab = K / KE;
        issue_loads(0, 0);
        if (nslab > 1) issue_loads(1, 1);
        int next_own = tn;
        if (PROT) {
            const int owned = tn < nslab ? (nslab - tn + g.tiles_n - 1) / g.tiles_n : 0;
            for (int t = tid; t < owned * KE; t += 256) col_lds[t] = 0u;
        }
        __syncthreads();
        ldfr(0, 0, 0);
        auto slab = [&](auto first_c, int s) __attribute__((always_inline)) {
            const int buf = s & 1;
            if (PROT && s == next_own) {
                a_pass<DT, BM>(smem + buf * BUF, g.b_sum + (long)bz * K + s * KE, KE, a_rows,
                               col_lds + ep.owned * KE, ep.st, g.mul24_ok != 0);
                next_own += g.tiles_n;
                ep.owned += 1;
            }
            ldfr(buf, 1, 1); mfmas(first_c, 0); interleave();
            ldfr(buf, 2, 0); mfmas(std::false_type{}, 1); interleave();
            ldfr(buf, 3, 1); mfmas(std::false_type{}, 0); interleave();
            __syncthreads();
            if (s + 2 < nslab) issue_loads(s + 2, buf);
            if (s + 1 < nslab) ldfr(buf ^ 1, 0, 0);
            mfmas(std::false_type{}, 1); interleave();
        };
        slab(std::true_type{}, 0);
        for (int s = 1; s < nslab; ++s) slab(std::false_type{}, s);
    }
    __syncthreads();
    gemm_epilogue<DT, BM, BN, PROT>(g, acc, smem, m0, n0, bz, ep);
}

// Workgroup -> tile inside a region of tiles_m x tiles_n tiles: consecutive ids of one XCD
// (workgroups are dealt to the 8 XCDs round-robin) walk GROUP_M tile rows, then the next column,
// so the workgroups that share an L2 work on a compact group of tiles.
__device__ __forceinline__ void map_tile(int bid, int nb, int tiles_m, int tiles_n, int *tm, int *tn)
{
    constexpr int GROUP_M = 8;
    const int q = nb >> 3, r = nb & 7, xcd = bid & 7;
    const int L = xcd * q + (xcd < r ? xcd : r) + (bid >> 3);
    const int per_group = GROUP_M * tiles_n;
    const int grp = L / per_group, in_grp = L % per_group;
    const int first_m = grp * GROUP_M;
    const int gsz = (tiles_m - first_m) < GROUP_M ? (tiles_m - first_m) : GROUP_M;
    *tm = first_m + in_grp % gsz;
    *tn = in_grp / gsz;
}

// The grid mixes two tile shapes against wave quantisation: 256 x 256 tiles cover the first
// big_rows rows in whole rounds of the machine, 128 x 256 tiles cover the rest, are dispatched
// after them and take half as long, so the last round is short.  (600 big tiles on 256 CUs
// would be three rounds for 2.34 rounds of work.)
template <int DT, bool PROT>
__global__ __launch_bounds__(256) void gemm_fast_kernel(GemmArgs g)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int bid = blockIdx.x, bz = blockIdx.z;
    int tm, tn;
    if (bid < g.n_big) {
        map_tile(bid, g.n_big, g.tiles_m_big, g.tiles_n, &tm, &tn);
        fast_tile<DT, 256, 256, PROT>(g, smem, tm * 256, tn * 256, bz, tn);
    } else {
        map_tile(bid - g.n_big, (int)gridDim.x - g.n_big, g.tiles_m_small, g.tiles_n, &tm, &tn);
        fast_tile<DT, 128, 256, PROT>(g, smem, g.tiles_m_big * 256 + tm * 128, tn * 256, bz, tn);
    }
}

// ------------------------------------------------------------------------------------------
static int g_num_cu = 0;

template <int DT, bool PROT>
static hipError_t launch_fast_one(GemmArgs &g, int batch, hipStream_t st)
{
    constexpr int smem_main = 2 * (256 + 256) * SLAB_BYTES;
    constexpr int smem_max = smem_main + (PROT ? 4096 * 4 + 2 * SLAB_BYTES * 4 : 0);
    auto kern = gemm_fast_kernel<DT, PROT>;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem_max);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    if (g_num_cu == 0) {
        int dev = 0, n = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        g_num_cu = n > 0 ? n : 256;
    }
    g.tiles_n = (g.N + 255) / 256;
    const int rows_all_big = (g.M + 255) / 256;
    const long total_big = (long)rows_all_big * g.tiles_n * batch;
    int big_rows = rows_all_big;
    if (total_big % g_num_cu != 0) {
        // whole rounds of big tiles, the remainder of the rows in half-height tiles
        const long rounds = total_big / g_num_cu;
        big_rows = (int)((rounds * g_num_cu) / ((long)g.tiles_n * batch));
        if (big_rows > rows_all_big) big_rows = rows_all_big;
    }
    g.tiles_m_big = big_rows;
    g.n_big = big_rows * g.tiles_n;
    const int rest = g.M - big_rows * 256;
    g.tiles_m_small = rest > 0 ? (rest + 127) / 128 : 0;
    g.tiles_m = g.tiles_m_big + g.tiles_m_small;
    dim3 grid((unsigned)(g.n_big + g.tiles_m_small * g.tiles_n), 1, (unsigned)batch);
    size_t smem = smem_main;
    if (PROT) {
        const int ke = SLAB_BYTES / Traits<DT>::ES;
        smem += (size_t)apass_owned_slabs(g.K / ke, g.tiles_n) * ke * 4;
        if (smem > (size_t)smem_max) return hipErrorInvalidValue;
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, g);
    return hipGetLastError();
}

bool gemm_fast_eligible(int dt, int M, int N, int K, bool transB, long lda, long ldb)
{
    const int ke = SLAB_BYTES / elem_size(dt);
    (void)lda; (void)ldb;
    return transB && (K % ke) == 0 && M >= 512 && N >= 512;
}

void gemm_fast_tile(int *tm, int *tn) { *tm = 256; *tn = 256; }

hipError_t launch_gemm_fast(int dt, bool protect, GemmArgs &g, int batch, hipStream_t st)
{
    switch (dt) {
    case DT_I8:
        return protect ? launch_fast_one<DT_I8, true>(g, batch, st) : launch_fast_one<DT_I8, false>(g, batch, st);
    case DT_BF16:
        return protect ? launch_fast_one<DT_BF16, true>(g, batch, st) : launch_fast_one<DT_BF16, false>(g, batch, st);
    case DT_F16:
        return protect ? launch_fast_one<DT_F16, true>(g, batch, st) : launch_fast_one<DT_F16, false>(g, batch, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace abft
